// Weight packing for the fused group attention kernels: the re-tiling of one layer's four weight
// matrices into the fragment stream the kernel reads, as a device function, so that it can run as
// a kernel of its own (layer_mfma.hip) or as extra workgroups of the first sort kernel (flatten.hip),
// where it costs no launch.
#pragma once
#include "common.h"

namespace ff {

// Stream order: for each 32-wide head-dim unit hp: K rows (2 x KB fragments), V rows, Q rows,
// W_o column slice (NB fragments); then for each 32-wide hidden unit fc: W1 rows (2 x KB), W2
// column slice (NB).  A fragment is 16 output features x 32 inputs; lane (i, q) owns 16 bytes:
// row i, inputs kbase + 16*(s/4) + 4q + (s%4) for slot s = 0..7.
// The six row blocks of a unit (Q a=0,1; K a=0,1; V a=0,1 numbered 0..5) come in this order:
__device__ constexpr int kQkvOrder[6] = {2, 3, 4, 5, 0, 1};
constexpr int kPackBatch = 16;
struct PackBatch {  // up to 16 layers of identical shape packed by one launch
  const uint16_t *w_qkv[kPackBatch], *w_o[kPackBatch], *w1[kPackBatch], *w2[kPackBatch];
  const uint16_t *b_qkv[kPackBatch], *b_o[kPackBatch];
  const uint16_t *ln1_g[kPackBatch], *ln1_b[kPackBatch], *ln2_g[kPackBatch], *ln2_b[kPackBatch], *b1[kPackBatch], *b2[kPackBatch];
  uint4* out[kPackBatch];
};
// What a launch needs to know to pack `layers` layers: `blocks` workgroups of 256 threads per layer.
struct PackJob {
  PackBatch pb;
  int layers, C, F, total_frags, blocks, half;  // half: IEEE half elements instead of bfloat16
  int first;                                    // a launch packs layers first .. first + layers - 1 of the batch
};

inline int pack_frag_count(int C, int F) { return (C / 32) * (6 * (C / 32) + C / 16) + (F / 32) * (2 * (C / 32) + C / 16); }

// Layers w[0..count) (count <= kPackBatch) to packed + l * stride_bytes.
inline void make_pack_job(const ff_layer_weights* w, int count, void* packed, size_t stride_bytes, bool half,
                          PackJob* job) {
  job->first = 0;
  job->layers = count; job->C = w->C; job->F = w->F; job->half = half ? 1 : 0;
  job->total_frags = pack_frag_count(w->C, w->F);
  // one thread per 16 bytes of a fragment, eight per folded bias element, one per other small parameter
  job->blocks = (job->total_frags * 64 + 8 * w->C + 6 * w->C + w->F + 255) / 256;
  for (int l = 0; l < kPackBatch; ++l) {
    const ff_layer_weights* wl = &w[l < count ? l : 0];
    job->pb.w_qkv[l] = (const uint16_t*)wl->w_qkv; job->pb.w_o[l] = (const uint16_t*)wl->w_o;
    job->pb.w1[l] = (const uint16_t*)wl->w1; job->pb.w2[l] = (const uint16_t*)wl->w2;
    job->pb.b_qkv[l] = (const uint16_t*)wl->b_qkv; job->pb.b_o[l] = (const uint16_t*)wl->b_o;
    job->pb.ln1_g[l] = (const uint16_t*)wl->ln1_g; job->pb.ln1_b[l] = (const uint16_t*)wl->ln1_b;
    job->pb.ln2_g[l] = (const uint16_t*)wl->ln2_g; job->pb.ln2_b[l] = (const uint16_t*)wl->ln2_b;
    job->pb.b1[l] = (const uint16_t*)wl->b1; job->pb.b2[l] = (const uint16_t*)wl->b2;
    job->pb.out[l] = (uint4*)((char*)packed + (size_t)(l < count ? l : 0) * stride_bytes);
  }
}

template <bool HALF> __device__ __forceinline__ float pack_el_to_f32(uint16_t h) {
  if constexpr (HALF) return (float)__builtin_bit_cast(_Float16, h);
  else return bf16_to_f32(h);
}
template <bool HALF> __device__ __forceinline__ uint16_t pack_f32_to_el(float f) {
  if constexpr (HALF) return __builtin_bit_cast(uint16_t, (_Float16)f);
  else return f32_to_bf16(f);
}

// After the fragments the packed buffer holds the layer's per-feature vectors as 7C + F floats, in the order
// the kernel keeps them in LDS (pack_param_*): LayerNorm 1 scale and shift, query bias, output-projection
// bias, LayerNorm 2 scale and shift, second and first FFN bias.  The kernel copies that block to LDS as it is.
// The output-projection bias has the value bias folded in.  Every softmax row sums to one, so
// P (V + 1 b_v^T) W_o^T = P V W_o^T + (W_o b_v)^T: the value bias is a constant row added after the
// projection.  (The key bias shifts all scores of a query by the same amount and drops out of the softmax
// altogether.)
__host__ __device__ constexpr int pack_param_count(int C, int F) { return 7 * C + F; }
// bytes of the parameter block, padded to whole 1 KB pieces (the unit of the kernel's copy to LDS)
__host__ __device__ constexpr int pack_param_bytes(int C, int F) { return (pack_param_count(C, F) * 4 + 1023) / 1024 * 1024; }
// Work of workgroup `block` (256 threads) of layer `layer`.
template <bool HALF>
__device__ __forceinline__ void pack_weights_block(const PackBatch& pb, int layer, int block, int C, int F,
                                                   int total_frags) {
  const uint16_t* __restrict__ w_qkv = pb.w_qkv[layer];
  const uint16_t* __restrict__ w_o = pb.w_o[layer];
  const uint16_t* __restrict__ w1 = pb.w1[layer];
  const uint16_t* __restrict__ w2 = pb.w2[layer];
  uint4* __restrict__ out = pb.out[layer];
  const int t = block * 256 + (int)threadIdx.x;
  const int frag = t >> 6, lane = t & 63, i = lane & 15, q = lane >> 4;
  if (frag >= total_frags && t - total_frags * 64 >= 8 * C) {  // the other per-feature vectors, one thread each
    const int pidx = t - total_frags * 64 - 8 * C;             // 0 .. 6C + F - 1; the folded bias sits at [3C, 4C)
    if (pidx >= 6 * C + F) return;
    const int dst = pidx < 3 * C ? pidx : pidx + C;
    const uint16_t* src;
    int o;
    if (dst < C) { src = pb.ln1_g[layer]; o = dst; }
    else if (dst < 2 * C) { src = pb.ln1_b[layer]; o = dst - C; }
    else if (dst < 3 * C) { src = pb.b_qkv[layer]; o = dst - 2 * C; }
    else if (dst < 5 * C) { src = pb.ln2_g[layer]; o = dst - 4 * C; }
    else if (dst < 6 * C) { src = pb.ln2_b[layer]; o = dst - 5 * C; }
    else if (dst < 7 * C) { src = pb.b2[layer]; o = dst - 6 * C; }
    else { src = pb.b1[layer]; o = dst - 7 * C; }
    reinterpret_cast<float*>(out + (size_t)total_frags * 64)[dst] = pack_el_to_f32<HALF>(src[o]);
    return;
  }
  if (frag >= total_frags) {  // folded output bias: eight lanes per output feature
    const int u = t - total_frags * 64, o = u >> 3, seg = u & 7, len = C / 8;
    float acc = 0.f;
    if (o < C) {
      // the lane's C/8 products, sixteen bytes of each operand per load and all loads before the first
      // product (C is a multiple of 64 here): these few workgroups end the launch they ride on
      const uint16_t* __restrict__ bv = pb.b_qkv[layer] + 2 * C;
      const uint4* wv = reinterpret_cast<const uint4*>(w_o + (size_t)o * C + seg * len);
      const uint4* bvv = reinterpret_cast<const uint4*>(bv + seg * len);
      uint4 wq[4], bq[4];
#pragma unroll
      for (int v = 0; v < 4; ++v)
        if (v * 8 < len) { wq[v] = wv[v]; bq[v] = bvv[v]; }
#pragma unroll
      for (int v = 0; v < 4; ++v)
        if (v * 8 < len) {
          const uint32_t wu[4] = {wq[v].x, wq[v].y, wq[v].z, wq[v].w}, bu[4] = {bq[v].x, bq[v].y, bq[v].z, bq[v].w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {  // ascending k, as before
            acc = fmaf(pack_el_to_f32<HALF>((uint16_t)(wu[e] & 0xffffu)), pack_el_to_f32<HALF>((uint16_t)(bu[e] & 0xffffu)), acc);
            acc = fmaf(pack_el_to_f32<HALF>((uint16_t)(wu[e] >> 16)), pack_el_to_f32<HALF>((uint16_t)(bu[e] >> 16)), acc);
          }
        }
    }
    acc += __shfl_xor(acc, 1);
    acc += __shfl_xor(acc, 2);
    acc += __shfl_xor(acc, 4);
    if (o < C && seg == 0)
      reinterpret_cast<float*>(out + (size_t)total_frags * 64)[3 * C + o] = acc + pack_el_to_f32<HALF>(pb.b_o[layer][o]);
    return;
  }
  const int KB = C / 32, NB = C / 16, fr_hp = 6 * KB + NB, fr_fc = 2 * KB + NB, n_hp = C / 32;
  const uint16_t* src;
  int kbase;
  bool halve = false;  // W2 carries the 0.5 of the GELU (the kernel computes twice the GELU)
  if (frag < n_hp * fr_hp) {
    const int hp = frag / fr_hp, r = frag % fr_hp;
    if (r < 6 * KB) {
      const int lc = kQkvOrder[r / KB], which = lc / 2, a = lc % 2, kb = r % KB;
      src = w_qkv + (size_t)(which * C + 32 * hp + 16 * a + i) * C;
      kbase = 32 * kb;
    } else {
      const int nb = r - 6 * KB;
      src = w_o + (size_t)(16 * nb + i) * C;
      kbase = 32 * hp;
    }
  } else {
    const int f2 = frag - n_hp * fr_hp, fc = f2 / fr_fc, r = f2 % fr_fc;
    if (r < 2 * KB) {
      const int a = r / KB, kb = r % KB;
      src = w1 + (size_t)(32 * fc + 16 * a + i) * C;
      kbase = 32 * kb;
    } else {
      const int nb = r - 2 * KB;
      src = w2 + (size_t)(16 * nb + i) * F;
      kbase = 32 * fc;
      halve = true;
    }
  }
  // slots 0..3 are inputs kbase + 4q .. + 3, slots 4..7 the same plus 16: two 8-byte loads
  uint32_t u[4];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint2 v = *reinterpret_cast<const uint2*>(src + kbase + 16 * h + 4 * q);
    u[2 * h] = v.x;
    u[2 * h + 1] = v.y;
  }
  if (halve) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const uint32_t lo = pack_f32_to_el<HALF>(0.5f * pack_el_to_f32<HALF>((uint16_t)(u[s] & 0xffffu)));
      const uint32_t hi = pack_f32_to_el<HALF>(0.5f * pack_el_to_f32<HALF>((uint16_t)(u[s] >> 16)));
      u[s] = lo | (hi << 16);
    }
  }
  out[(size_t)frag * 64 + lane] = make_uint4(u[0], u[1], u[2], u[3]);
}

}  // namespace ff
