// Group attention layer (paper Sec. 4.2.2, Eq. (2)), plain fp32-arithmetic kernels.
//
//   F'  = F  + MHSA(LN1(F)),   F'' = F' + FFN(LN2(F'))
//
// This is the exact-arithmetic path: storage type T (float or bf16), every product, sum,
// exponential and erf in fp32 on the vector ALUs.  It serves dtype FF_F32 and any shape the
// MFMA kernels do not cover.  Three kernels, intermediates in the caller's workspace:
//   k_ln_qkv    rows of the sorted order: gather, LN1, packed QKV projection   -> qkv [n, 3C] f32
//               (weights staged through LDS from 8192 rows on)
//   k_attention one workgroup per (group, head): softmax(Q K^T / sqrt(d)) V     -> o   [n, C]  f32
//   k_out_ffn   rows: out-proj + residual, LN2, Linear+GELU, Linear + residual, scatter
#include "common.h"

namespace ff {
namespace {

constexpr int RB = 4;            // sorted rows per workgroup in the row kernels ...
constexpr int kRowsWide = 16;    // ... or sixteen, from kRowsWideMin rows on (512 workgroups)
constexpr int64_t kRowsWideMin = 8192;
constexpr size_t kRowLdsMax = 64 * 1024;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

// LayerNorm of RB rows of width C held in LDS (src -> dst), one wavefront per row.
__device__ __forceinline__ void ln_rows(const float* src, float* dst, int C, int rows,
                                        const float* g_s, const float* b_s, float eps) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  for (int r = w; r < rows; r += (int)(blockDim.x >> 6)) {
    float s = 0.f;
    for (int k = lane; k < C; k += 64) s += src[r * C + k];
    const float mu = wave_sum(s) / (float)C;
    float q = 0.f;
    for (int k = lane; k < C; k += 64) { float t = src[r * C + k] - mu; q += t * t; }
    const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)C + eps);
    for (int k = lane; k < C; k += 64) dst[r * C + k] = (src[r * C + k] - mu) * rstd * g_s[k] + b_s[k];
  }
}

// acc[r] = sum over k of in[r * ld + k] * W[j * K + k] for the workgroup's RBT rows (in LDS) and every
// output feature j < N, thread t owning features t, t + 256, ...; the sum runs over k in ascending
// order whatever the staging.  TILED: the weights pass through LDS in tiles of 256 features x KT
// inputs, read from memory along k by neighbouring threads (a thread streaming its own weight row
// touches a cache line of its own per load, 64 lines per wavefront instruction).  `in(j)` names the
// LDS rows feature j multiplies, `ep(j, acc)` takes the sums.  Every thread of the workgroup must call.
constexpr int KT = 16;
template <typename T, int RBT, bool TILED, typename In, typename Ep>
__device__ __forceinline__ void rows_by_weights(const T* __restrict__ W, int N, int K, int ld, float* wt, In in, Ep ep) {
  for (int j0 = 0; j0 < N; j0 += 256) {
    const int j = j0 + (int)threadIdx.x;
    float acc[RBT];
#pragma unroll
    for (int r = 0; r < RBT; ++r) acc[r] = 0.f;
    if (TILED) {
      const float* src = in(j < N ? j : N - 1);
      const float* mine = wt + threadIdx.x * (KT + 1);
      for (int k0 = 0; k0 < K; k0 += KT) {
        __syncthreads();  // the previous tile has been used
        for (int t = threadIdx.x; t < 256 * KT; t += 256) {
          const int jj = t / KT, kk = t - jj * KT;
          wt[jj * (KT + 1) + kk] =
              j0 + jj < N && k0 + kk < K ? Elem<T>::load(W + (int64_t)(j0 + jj) * K + k0 + kk) : 0.f;
        }
        __syncthreads();
        if (j >= N) continue;
        if (k0 + KT <= K) {
#pragma unroll
          for (int kk = 0; kk < KT; ++kk) {
            const float wv = mine[kk];
#pragma unroll
            for (int r = 0; r < RBT; ++r) acc[r] = fmaf(src[r * ld + k0 + kk], wv, acc[r]);
          }
        } else {
          for (int kk = 0; k0 + kk < K; ++kk) {
            const float wv = mine[kk];
#pragma unroll
            for (int r = 0; r < RBT; ++r) acc[r] = fmaf(src[r * ld + k0 + kk], wv, acc[r]);
          }
        }
      }
    } else if (j < N) {
      const float* src = in(j);
      const T* wrow = W + (int64_t)j * K;
#pragma unroll 8
      for (int k = 0; k < K; ++k) {  // eight weight loads in flight
        const float wv = Elem<T>::load(wrow + k);
#pragma unroll
        for (int r = 0; r < RBT; ++r) acc[r] = fmaf(src[r * ld + k], wv, acc[r]);
      }
    }
    if (j < N) ep(j, acc);
  }
}

template <typename T, int RBT, bool TILED>
__global__ __launch_bounds__(256) void k_ln_qkv(const T* __restrict__ feats, const int32_t* __restrict__ perm,
                                                 int64_t n, int C, const T* __restrict__ ln_g,
                                                 const T* __restrict__ ln_b, float eps,
                                                 const T* __restrict__ w_qkv, const T* __restrict__ b_qkv,
                                                 const T* __restrict__ pos_embed, float* __restrict__ qkv) {
  extern __shared__ float lds[];
  float* X = lds;              // [RBT][C]
  float* U = X + RBT * C;      // [RBT][C]
  float* gs = U + RBT * C;     // [C]
  float* bs = gs + C;          // [C]
  float* wt = bs + C;          // TILED: [256][KT + 1]
  const int64_t p0 = (int64_t)blockIdx.x * RBT;
  const int rows = (int)((n - p0) < RBT ? (n - p0) : RBT);
  for (int i = threadIdx.x; i < C; i += blockDim.x) { gs[i] = Elem<T>::load(ln_g + i); bs[i] = Elem<T>::load(ln_b + i); }
  for (int i = threadIdx.x; i < RBT * C; i += blockDim.x) {
    const int r = i / C, k = i - r * C;
    X[i] = r < rows ? Elem<T>::load(feats + (int64_t)perm[p0 + r] * C + k) : 0.f;
  }
  __syncthreads();
  ln_rows(X, U, C, rows, gs, bs, eps);
  for (int i = threadIdx.x + rows * C; i < RBT * C; i += blockDim.x) U[i] = 0.f;  // rows beyond n
  __syncthreads();
  if (pos_embed) {  // queries and keys are projected from LN(F) + PE (kept in X), values from LN(F)
    for (int i = threadIdx.x; i < RBT * C; i += blockDim.x) {
      const int r = i / C, k = i - r * C;
      X[i] = r < rows ? U[i] + Elem<T>::load(pos_embed + (int64_t)perm[p0 + r] * C + k) : 0.f;
    }
    __syncthreads();
  }
  rows_by_weights<T, RBT, TILED>(
      w_qkv, 3 * C, C, C, wt, [&](int j) { return pos_embed && j < 2 * C ? X : U; },
      [&](int j, const float* acc) {
        const float bj = Elem<T>::load(b_qkv + j);
        for (int r = 0; r < rows; ++r) qkv[(p0 + r) * 3 * (int64_t)C + j] = acc[r] + bj;
      });
}

// One workgroup per (group, head); one thread per query row (looping when the group is larger
// than the workgroup).  Plain two-pass softmax over the group's real members.
// EXACT: d == DMAX, so the loops over the head dimension carry no bound test (with one, every element
// became a branch and a load of its own).
template <int DMAX, bool STAGED, bool EXACT>
__global__ __launch_bounds__(256) void k_attention(const float* __restrict__ qkv, const int32_t* __restrict__ group_offsets,
                                                    const int32_t* __restrict__ num_groups, int C, int d, int G,
                                                    float* __restrict__ o) {
  extern __shared__ float kv_s[];  // STAGED: the group's K and V slices of this head, [m][d] each
  const int g = blockIdx.x, h = blockIdx.y;
  if (g >= *num_groups) return;
  const int64_t start = group_offsets[g];
  int m = group_offsets[g + 1] - group_offsets[g];
  m = m < G ? m : G;  // a list of full groups only: the next start may lie beyond this group's end
  const float scale = 1.0f / sqrtf((float)d);
  const int64_t ld = 3 * (int64_t)C;
  // Every query of the group walks over the same keys and values: from LDS when they fit (one trip
  // to memory for the whole workgroup), else straight from memory.
  const float* kbase = qkv + start * ld + C + h * d;
  int64_t kld = ld, voff = C;
  if (STAGED) {
    for (int t = threadIdx.x; t < m * d; t += blockDim.x) {
      const int j = t / d, c = t - j * d;
      kv_s[t] = kbase[j * ld + c];
      kv_s[G * d + t] = kbase[j * ld + C + c];
    }
    __syncthreads();
    kbase = kv_s; kld = d; voff = (int64_t)G * d;
  }
  for (int i = threadIdx.x; i < m; i += blockDim.x) {
    float q[DMAX], acc[DMAX];
    const float* qrow = qkv + (start + i) * ld + h * d;
#pragma unroll
    for (int c = 0; c < DMAX; ++c) { q[c] = EXACT || c < d ? qrow[c] : 0.f; acc[c] = 0.f; }
    float mx = -INFINITY;
    for (int j = 0; j < m; ++j) {
      const float* krow = kbase + j * kld;
      float s = 0.f;
#pragma unroll
      for (int c = 0; c < DMAX; ++c) if (EXACT || c < d) s = fmaf(q[c], krow[c], s);
      mx = fmaxf(mx, s * scale);
    }
    float sum = 0.f;
    for (int j = 0; j < m; ++j) {
      const float* krow = kbase + j * kld;
      const float* vrow = krow + voff;
      float s = 0.f;
#pragma unroll
      for (int c = 0; c < DMAX; ++c) if (EXACT || c < d) s = fmaf(q[c], krow[c], s);
      const float e = expf(s * scale - mx);
      sum += e;
#pragma unroll
      for (int c = 0; c < DMAX; ++c) if (EXACT || c < d) acc[c] = fmaf(e, vrow[c], acc[c]);
    }
    const float inv = 1.0f / sum;
    float* orow = o + (start + i) * (int64_t)C + h * d;
#pragma unroll
    for (int c = 0; c < DMAX; ++c) if (EXACT || c < d) orow[c] = acc[c] * inv;
  }
}

template <typename T, typename TO, int RBT, bool TILED>
__global__ __launch_bounds__(256) void k_out_ffn(const T* __restrict__ feats, const int32_t* __restrict__ perm,
                                                  int64_t n, int C, int F, const float* __restrict__ o,
                                                  const T* __restrict__ w_o, const T* __restrict__ b_o,
                                                  const T* __restrict__ ln_g, const T* __restrict__ ln_b, float eps,
                                                  const T* __restrict__ w1, const T* __restrict__ b1,
                                                  const T* __restrict__ w2, const T* __restrict__ b2,
                                                  TO* __restrict__ out) {
  extern __shared__ float lds[];
  float* O = lds;               // [RBT][C]
  float* X1 = O + RBT * C;      // [RBT][C]
  float* U = X1 + RBT * C;      // [RBT][C]
  float* H = U + RBT * C;       // [RBT][F]
  float* gs = H + RBT * F;      // [C]
  float* bs = gs + C;           // [C]
  float* wt = bs + C;           // TILED: [256][KT + 1]
  const int64_t p0 = (int64_t)blockIdx.x * RBT;
  const int rows = (int)((n - p0) < RBT ? (n - p0) : RBT);
  for (int i = threadIdx.x; i < C; i += blockDim.x) { gs[i] = Elem<T>::load(ln_g + i); bs[i] = Elem<T>::load(ln_b + i); }
  for (int i = threadIdx.x; i < RBT * C; i += blockDim.x) O[i] = i < rows * C ? o[p0 * C + i] : 0.f;
  __syncthreads();
  rows_by_weights<T, RBT, TILED>(
      w_o, C, C, C, wt, [&](int) { return O; },
      [&](int j, const float* acc) {
        const float bj = Elem<T>::load(b_o + j);
#pragma unroll
        for (int r = 0; r < RBT; ++r) {
          const float x = r < rows ? Elem<T>::load(feats + (int64_t)perm[p0 + r] * C + j) : 0.f;
          X1[r * C + j] = x + (acc[r] + bj);
        }
      });
  __syncthreads();
  ln_rows(X1, U, C, RBT, gs, bs, eps);
  __syncthreads();
  rows_by_weights<T, RBT, TILED>(
      w1, F, C, C, wt, [&](int) { return U; },
      [&](int f, const float* acc) {
        const float bf = Elem<T>::load(b1 + f);
#pragma unroll
        for (int r = 0; r < RBT; ++r) {
          const float v = acc[r] + bf;
          H[r * F + f] = 0.5f * v * (1.0f + erff(v * 0.70710678118654752440f));
        }
      });
  __syncthreads();
  rows_by_weights<T, RBT, TILED>(
      w2, C, F, F, wt, [&](int) { return H; },
      [&](int j, const float* acc) {
        const float bj = Elem<T>::load(b2 + j);
        for (int r = 0; r < rows; ++r)
          Elem<TO>::store(out + (int64_t)perm[p0 + r] * C + j, X1[r * C + j] + (acc[r] + bj));
      });
}

// The QKV kernel takes sixteen rows per workgroup with staged weights when there are enough rows to
// fill the chip that way and its LDS fits (measured at 30k rows, C = 128: 1102 -> 181 us); four rows
// with weights straight from memory otherwise (faster below a few thousand rows).  The out-proj / FFN
// kernel never stages: its three narrower products (half the threads idle when a product has 128
// outputs, two workgroups per compute unit) were slower that way, 445 against 309 us; it takes
// sixteen rows where its LDS fits (225 us) and four otherwise.
struct RowPlan { int rb; bool tiled; size_t lds; };
RowPlan qkv_plan(int64_t n, int C) {
  const size_t wide = ((size_t)2 * kRowsWide * C + 2 * C + 256 * (KT + 1)) * 4;
  if (n >= kRowsWideMin && wide <= kRowLdsMax) return {kRowsWide, true, wide};
  return {RB, false, ((size_t)2 * RB * C + 2 * C) * 4};
}

template <typename T, typename TO>
int launch_typed(const void* feats, void* out, int64_t n, const int32_t* perm, const int32_t* group_offsets,
                 const int32_t* num_groups, int32_t max_groups, const ff_layer_weights* w, int d, int G,
                 float* qkv, float* o, hipStream_t stream) {
  const int C = w->C, F = w->F;
  const RowPlan pa = qkv_plan(n, C);
  auto run_qkv = [&](auto kern) {
    hipLaunchKernelGGL(kern, dim3((unsigned)ceil_div(n, pa.rb)), dim3(256), pa.lds, stream, (const T*)feats, perm, n, C,
                       (const T*)w->ln1_g, (const T*)w->ln1_b, w->ln_eps, (const T*)w->w_qkv, (const T*)w->b_qkv,
                       (const T*)w->pos_embed, qkv);
  };
  if (pa.tiled) run_qkv(k_ln_qkv<T, kRowsWide, true>);
  else run_qkv(k_ln_qkv<T, RB, false>);
  dim3 ga((unsigned)max_groups, (unsigned)w->heads);
  const size_t lds_kv = (size_t)2 * G * d * 4;  // G can be far larger than any group: then no staging
  const bool staged = (int64_t)G * d * 8 <= 48 * 1024;
#define FF_ATT(D)                                                                                                     \
  do {                                                                                                                \
    if (staged && d == D)                                                                                             \
      hipLaunchKernelGGL((k_attention<D, true, true>), ga, dim3(256), lds_kv, stream, qkv, group_offsets, num_groups, \
                         C, d, G, o);                                                                                 \
    else if (staged)                                                                                                  \
      hipLaunchKernelGGL((k_attention<D, true, false>), ga, dim3(256), lds_kv, stream, qkv, group_offsets,            \
                         num_groups, C, d, G, o);                                                                     \
    else                                                                                                              \
      hipLaunchKernelGGL((k_attention<D, false, false>), ga, dim3(256), 0, stream, qkv, group_offsets, num_groups, C, \
                         d, G, o);                                                                                    \
  } while (0)
  if (d <= 16) FF_ATT(16);
  else if (d <= 32) FF_ATT(32);
  else if (d <= 64) FF_ATT(64);
  else FF_ATT(128);
#undef FF_ATT
  const size_t ffn_wide = ((size_t)3 * kRowsWide * C + (size_t)kRowsWide * F + 2 * C) * 4;
  auto run_ffn = [&](auto kern, int rb) {
    hipLaunchKernelGGL(kern, dim3((unsigned)ceil_div(n, rb)), dim3(256),
                       ((size_t)3 * rb * C + (size_t)rb * F + 2 * C) * 4, stream, (const T*)feats, perm, n, C, F, o,
                       (const T*)w->w_o, (const T*)w->b_o, (const T*)w->ln2_g, (const T*)w->ln2_b, w->ln_eps,
                       (const T*)w->w1, (const T*)w->b1, (const T*)w->w2, (const T*)w->b2, (TO*)out);
  };
  if (n >= kRowsWideMin && ffn_wide <= kRowLdsMax) run_ffn(k_out_ffn<T, TO, kRowsWide, false>, kRowsWide);
  else run_ffn(k_out_ffn<T, TO, RB, false>, RB);
  return launch_status();
}

}  // namespace

size_t layer_generic_workspace_bytes(int64_t n, const ff_layer_weights* w) {
  return align_up((size_t)n * 3 * w->C * 4, 256) + align_up((size_t)n * w->C * 4, 256);
}

int layer_generic_launch(const void* feats, void* out, int64_t n, const int32_t* perm,
                         const int32_t* group_offsets, const int32_t* num_groups, int32_t max_groups,
                         const ff_layer_weights* w, int G, int dtype, bool out_f32,
                         void* workspace, size_t workspace_bytes, hipStream_t stream) {
  const int C = w->C, F = w->F, d = C / w->heads;
  if (d > 128) return FF_ERR_UNSUPPORTED;
  if ((size_t)(3 * RB * C + RB * F + 2 * C) * 4 > 64 * 1024) return FF_ERR_UNSUPPORTED;
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < layer_generic_workspace_bytes(n, w))
    return FF_ERR_WORKSPACE;
  if (n == 0 || max_groups == 0) return FF_OK;
  float* qkv = (float*)workspace;
  float* o = (float*)((char*)workspace + align_up((size_t)n * 3 * C * 4, 256));
  if (dtype == FF_F32)
    return launch_typed<float, float>(feats, out, n, perm, group_offsets, num_groups, max_groups, w, d, G, qkv, o, stream);
  if (dtype == FF_F16) {
    if (out_f32)
      return launch_typed<f16_t, float>(feats, out, n, perm, group_offsets, num_groups, max_groups, w, d, G, qkv, o, stream);
    return launch_typed<f16_t, f16_t>(feats, out, n, perm, group_offsets, num_groups, max_groups, w, d, G, qkv, o, stream);
  }
  if (out_f32)
    return launch_typed<bf16_t, float>(feats, out, n, perm, group_offsets, num_groups, max_groups, w, d, G, qkv, o, stream);
  return launch_typed<bf16_t, bf16_t>(feats, out, n, perm, group_offsets, num_groups, max_groups, w, d, G, qkv, o, stream);
}

}  // namespace ff
