// Group attention layer (paper Sec. 4.2.2, Eq. (2); Sec. 4.3 'Efficient MHSA' / 'Efficient FFN')
// as ONE fused kernel on the bf16 matrix cores of gfx950:
//
//   gather -> LN1 -> packed QKV projection -> per-head softmax(Q K^T / sqrt(d)) V -> out-proj
//   + residual -> LN2 -> Linear + GELU -> Linear + residual -> scatter
//
// Scores, probabilities, Q/K/V and the FFN hidden activations never leave the chip.
//
// Mapping.  A wavefront owns NVB blocks of 16 pillars of one group ("its" pillars); WPG wavefronts
// share a group, NW wavefronts form a workgroup.  Everything is computed transposed, features x
// pillars, with v_mfma_f32_16x16x32_bf16: the weight tile is the A operand (16 output features x
// 32 inputs), the activations of 16 pillars are the B operand, and the accumulator holds
// D[feature 4q+j][pillar i] in lane (i = lane & 15, q = lane >> 4).  That accumulator layout is,
// after conversion to bf16, directly a B operand of the next product whose 8 k-slots in lane q
// are inputs {4q..4q+3} of two consecutive 16-blocks; weights are pre-permuted along k to match
// (pack kernel below), so activations chain from product to product in registers without any
// LDS round trip.  V is produced with the operand roles swapped (pillars x features), which is
// exactly the A operand P*V needs.  LayerNorm statistics and the softmax need only a reduction
// over the four lanes that share a pillar.
//
// Weights reach the matrix cores through LDS.  The packed stream is cut into 16 KB chunks that the
// workgroup copies asynchronously (global memory -> LDS, no registers) into a ring of as many slots
// as the LDS holds; slots are refilled only at workgroup barriers (one per head-dim unit, where the
// group's K and V are exchanged anyway, and a few in the FFN).  Every wavefront reads the fragments
// in stream order through a window of 8 fragments in registers, requested 8 products ahead of
// their use, so that LDS latency is hidden behind the matrix cores.
#include "common.h"
#include "pack_weights.h"
#include <atomic>

namespace ff {
namespace {

// ---- number format of the 16-bit storage and of the matrix-core operands --------------------------------
// This source builds the bfloat16 kernels; layer_mfma_f16.hip defines FF_LAYER_F16 and includes it
// to build the IEEE half kernels (the precision the paper runs in, Sec. 5.1) from the same code.
#ifdef FF_LAYER_F16
typedef _Float16 el8 __attribute__((ext_vector_type(8)));
typedef _Float16 el4 __attribute__((ext_vector_type(4)));
typedef _Float16 el2 __attribute__((ext_vector_type(2)));
constexpr uint32_t kOnePair = 0x3c003c00u;  // two ones
__device__ __forceinline__ float el_to_f32(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }
__device__ __forceinline__ float el_lo(uint32_t u) { return el_to_f32((uint16_t)(u & 0xffffu)); }
__device__ __forceinline__ float el_hi(uint32_t u) { return el_to_f32((uint16_t)(u >> 16)); }
#define FF_LAYER_SYM(name) name##_f16
#else
typedef __bf16 el8 __attribute__((ext_vector_type(8)));
typedef short el4 __attribute__((ext_vector_type(4)));
typedef __bf16 el2 __attribute__((ext_vector_type(2)));
constexpr uint32_t kOnePair = 0x3f803f80u;  // two ones
__device__ __forceinline__ float el_to_f32(uint16_t h) { return bf16_to_f32(h); }
__device__ __forceinline__ float el_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float el_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
#define FF_LAYER_SYM(name) name
#endif
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

union Frag8 {  // eight 16-bit elements = one operand of the k=32 product
  el8 v;
  uint32_t u[4];
  u32x4 q;
};
union Frag4 {  // four 16-bit elements = one operand of the k=16 product
  el4 v;
  uint32_t u[2];
  u32x2 d;
};

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  f32x2 f = {lo, hi};
  el2 r = __builtin_convertvector(f, el2);  // round to nearest even
  return *reinterpret_cast<uint32_t*>(&r);
}
__device__ __forceinline__ void load4(const uint16_t* p, float* o) {  // 4 consecutive elements -> fp32
  const uint2 u = *reinterpret_cast<const uint2*>(p);
  o[0] = el_lo(u.x);
  o[1] = el_hi(u.x);
  o[2] = el_lo(u.y);
  o[3] = el_hi(u.y);
}
// Reductions over the 4 lanes that share a pillar (lane, lane^16, lane^32, lane^48), on the
// vector ALU: v_permlane16_swap / v_permlane32_swap with both operands equal to v return the
// pair (v from the even half, v from the odd half) in every lane.
__device__ __forceinline__ float quad_sum(float v) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}
__device__ __forceinline__ float quad_max(float v) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ f32x4 mfma32(const Frag8& a, const Frag8& b, f32x4 c) {
#ifdef FF_LAYER_F16
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a.v, b.v, c, 0, 0, 0);
#else
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, c, 0, 0, 0);
#endif
}
// The k = 16 product takes no accumulator: it can only START a chain, from zero.  A k = 16 product issued right
// behind a k = 32 product that writes the accumulator it reads has been seen to read the old value on this chip,
// so every product that continues a chain goes through mfma32 (an odd 16-wide block multiplies zeros in its
// upper half), and this signature keeps a chained k = 16 call from compiling.
__device__ __forceinline__ f32x4 mfma16_from_zero(const Frag4& a, const Frag4& b) {
  const f32x4 z = {0.f, 0.f, 0.f, 0.f};
#ifdef FF_LAYER_F16
  return __builtin_amdgcn_mfma_f32_16x16x16f16(a.v, b.v, z, 0, 0, 0);
#else
  return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a.v, b.v, z, 0, 0, 0);
#endif
}
// GELU(v) = v * Phi(v) with the upper tail 1 - Phi(t) ~ 0.5 * exp(-(a t + b t^2 + c t^3)), t = |v|
// (coefficients fitted to the erf form; all positive, so the exponent is monotone for any t):
//   GELU(v) = max(v, 0) - 0.5 t e = 0.5 (v + t (1 - e)),   e = exp(-(a t + b t^2 + c t^3)),
// max abs error 8.6e-5.  This returns 2 GELU(v); the factor 0.5 is folded into the packed W2
// (exact in bf16).  Five vector operations and one transcendental per element.
__device__ __forceinline__ float gelu2_fast(float v) {
  constexpr float L2E = 1.44269504088896340736f;
  const float t = fabsf(v);
  float p = fmaf(t, -0.01916250660946074f * L2E, -0.33840941696965965f * L2E);
  p = fmaf(t, p, -0.7908370960657618f * L2E);
  const float e = __builtin_amdgcn_exp2f(p * t);
  return v + fmaf(-t, e, t);
}

// Number of 1 KB fragments of the packed weight stream of one layer.
__host__ __device__ constexpr int frags_per_hp(int C) { return 6 * (C / 32) + C / 16; }
__host__ __device__ constexpr int frags_per_fc(int C) { return 2 * (C / 32) + C / 16; }

// ---- weight packing (pack_weights.h) as a kernel of its own: grid (blocks per layer, layers) -----------
#ifdef FF_LAYER_F16
constexpr bool kHalf = true;
#else
constexpr bool kHalf = false;
#endif
__global__ __launch_bounds__(256) void k_pack_weights(PackBatch pb, int C, int F, int total_frags) {
  pack_weights_block<kHalf>(pb, blockIdx.y, blockIdx.x, C, F, total_frags);
}

// ---- the fused layer ------------------------------------------------------------------------------
// LDS map (bytes): [weight ring RING x 16 KB][small parameters as fp32: (7C + F) x 4][K/V exchange, 2 buffers].
template <int C, int F>
struct ParamOff {  // float offsets inside the small-parameter area
  static constexpr int LN1G = 0, LN1B = C, BQ = 2 * C, BO = 3 * C, LN2G = 4 * C, LN2B = 5 * C, B2 = 6 * C,
                       B1 = 7 * C, TOTAL = 7 * C + F;
};

// Fragments per staged chunk: 16 (16 KB), or 8 for the narrow layer, whose hidden unit is 8 fragments (units are
// whole chunks).
__host__ __device__ constexpr int chunk_frags(int C) { return C >= 128 ? 16 : 8; }
constexpr int kLdsBytes = 160 * 1024;  // LDS of one compute unit
constexpr int kComputeUnits = 256;      // of an MI355X
constexpr int kWindow = 8;             // weight fragments a wavefront keeps in flight (LDS -> registers)

template <int C, int F, int NVB, int WPG, int NW, int MINW>
struct LdsPlan {
  static constexpr int NKB = NVB * WPG, GPW = NW / WPG;
  static constexpr int WGS = (MINW * 4 / NW) > 1 ? (MINW * 4 / NW) : 1;  // workgroups meant to share a compute unit
  static constexpr int PARAMS = pack_param_bytes(C, F);   // padded to whole 1 KB pieces
  static constexpr int KVX_ONE = 2 * 2 * NKB * 64 * 8;                     // K and V of one group, one unit
  static constexpr int KVX = WPG > 1 ? 2 * GPW * KVX_ONE : 0;              // double buffered
  static constexpr int NCHUNK = ((C / 32) * (6 * (C / 32) + C / 16) + (F / 32) * (2 * (C / 32) + C / 16)) / chunk_frags(C);
  static constexpr int FIT = (kLdsBytes / WGS - PARAMS - KVX) / (chunk_frags(C) * 1024);
  static constexpr int RING0 = FIT < NCHUNK ? FIT : NCHUNK;
  // Mappings with rolled loops (more than two wavefronts per SIMD at C = 128) compute ring slots at run time: a
  // power of two keeps that to a mask.
  static constexpr bool ROLLED_128 = C == 128 && NW > 8;
  static constexpr int RING = ROLLED_128 && RING0 >= 4 && RING0 < 8 ? 4 : RING0;
  static constexpr int TOTAL = RING * chunk_frags(C) * 1024 + PARAMS + KVX;
  static_assert(RING >= 2, "weight ring");
};

template <int C, int DH, int F, int NVB, int WPG, int NW, int MINW, bool OUT_F32, bool PE>
__global__ __launch_bounds__(NW * 64, MINW) void k_layer_mfma(const uint16_t* __restrict__ feats, void* __restrict__ out,
                                                               const uint16_t* __restrict__ pos_embed,
                                                               const int32_t* __restrict__ perm,
                                                               const int32_t* __restrict__ goff,
                                                               const int32_t* __restrict__ num_groups, int max_groups,
                                                               const u32x4* __restrict__ packed, float eps,
                                                               int n, int G, int drop,
                                                               const int32_t* __restrict__ out_index, int in_sorted) {
  constexpr int KB = C / 32;          // 32-wide blocks of the input features
  constexpr int NB = C / 16;          // 16-wide blocks of the output features
  constexpr int HP = C / 32;          // 32-wide head-dim units
  constexpr int FC = F / 32;          // 32-wide hidden units
  constexpr int NKB = NVB * WPG;      // key blocks of a group
  constexpr int NT = NW * 64;
  constexpr int GPW = NW / WPG;       // groups per workgroup
  constexpr int CF = chunk_frags(C);
  constexpr int FH = 6 * KB + NB;     // fragments of one head-dim unit: Q, K, V rows, W_o slice
  constexpr int FF = 2 * KB + NB;     // fragments of one hidden unit: W1 rows, W2 slice
  constexpr int CPH = FH / CF, CPF = FF / CF;
  // C = 128: the unit loops are unrolled completely, which turns the ring bookkeeping into constants
  // (about 30 KB of code).  Wider layers keep rolled loops.
  constexpr int FULL_UNROLL = C <= 128 && NW <= 8 ? 16 : 1;  // more waves per SIMD leave too few registers for it:
  // with three or four, the hidden units are still unrolled completely (their chunk numbers and ring slots become
  // constants) and the head-dim units in pairs (the ring of four slots repeats every two units)
  constexpr int FFN_UNROLL = C <= 128 && MINW >= 3 ? 16 : FULL_UNROLL;
  constexpr int ATT_UNROLL = C <= 128 && MINW >= 3 ? 2 : FULL_UNROLL;
  constexpr bool LEAN = ((NW + 3) / 4 >= 3 && MINW <= 2 && C >= 256) || MINW >= 4;  // C = 256 with three wavefronts on a SIMD
                                                                              // (168 registers each), C = 128 with four (128)
  constexpr int PF = LEAN ? 4 : kWindow;
  using LP = LdsPlan<C, F, NVB, WPG, NW, MINW>;
  constexpr int NCHUNK = LP::NCHUNK, RING = LP::RING;
  using PO = ParamOff<C, F>;
  static_assert(DH == 16 || DH == 32, "head dim");
  static_assert(FH % CF == 0 && FF % CF == 0 && CF % PF == 0, "units are whole chunks");

  extern __shared__ u32x4 lds[];
  u32x4* ring = lds;                                            // [RING][CF * 64]
  // These areas lie beyond the 64 KB an LDS instruction reaches from a base register: their offset
  // is hidden from constant folding so that each gets a base register of its own.
  uint32_t par_units = RING * CF * 64;
  asm volatile("" : "+v"(par_units));
  float* par = reinterpret_cast<float*>(lds + par_units);       // [PO::TOTAL]
  u32x2* kvx = reinterpret_cast<u32x2*>(reinterpret_cast<char*>(par) + LP::PARAMS);  // K/V exchange, only when WPG > 1

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, i = lane & 15, q = lane >> 4;
  const int wu = __builtin_amdgcn_readfirstlane(w);
  const int gl = wu / WPG, part = wu % WPG;
  const int g = blockIdx.x * GPW + gl;
  // group_offsets has at least max_groups + 1 entries: read this group's bounds without waiting
  // for num_groups, so that the loads travel together.
  const int gc = g < max_groups ? g : max_groups - 1;
  const int off0 = goff[gc], off1 = goff[gc + 1];
  const int ngroups = *num_groups;
  // Groups of the first (or only) frame start at g * G: fetch the pillar indices from there
  // without waiting for the offsets, and use them if the guess turns out right.
  int32_t guess[NVB];
#pragma unroll
  for (int vb = 0; vb < NVB; ++vb) {
    // (unsigned 32-bit: g * G stays below n + num_frames * G, and one minimum clamps it)
    const uint32_t at = (uint32_t)g * (uint32_t)G + (uint32_t)((part * NVB + vb) * 16 + i);
    guess[vb] = perm[at < (uint32_t)n ? at : (uint32_t)n - 1u];
  }
  // in_sorted: row p of feats is the pillar at sorted position p (the previous layer of a block wrote
  // its result in this layer's order), so the rows of a group are contiguous and need no index.
  // in_sorted == 2 (one frame): they are fetched from the guessed start without waiting for anything.
  // Rows are fetched whole when the wavefront has LDS to turn them around in (STAGE): lane (q, i) takes
  // the i-th 16 bytes of row 4k + q in its k-th load, so that an instruction reads four complete rows.
  // With 8 bytes per lane in the accumulator layout (16 rows x 32 bytes per instruction) every row was
  // touched by eight instructions, and the burst of all wavefronts at kernel start took 2.1 us instead
  // of 0.8 to drain.  The rows then go through the wavefront's share of the K/V exchange buffer (not in
  // use yet), 16-byte pieces swizzled by row so that neither the writes nor the reads conflict.
  // C = 256: a row is 32 pieces, a load instruction reads two rows, and the 4 KB share turns the rows
  // around in two phases of sixteen pieces each (a lane's piece belongs to phase `ph`).
  constexpr bool STAGE = (C == 128 || C == 256) && WPG > 1 && !(LEAN && OUT_F32);  // (the lean mapping with fp32
                                                                                    // output has no registers for it)
  constexpr int LPR = C / 8, RPI = 64 / LPR, PH = C / 128;  // lanes per row, rows per instruction, phases
  constexpr int NRL = STAGE ? 16 * NVB / RPI : 1;            // 16-byte loads per lane
  const int lr = lane / LPR, piece32 = lane % LPR, ph = piece32 >> 4;  // my row within an instruction, my piece
  constexpr int NBX = STAGE ? 1 : NB;       // raw rows of the early fetch without staging: 8 bytes per 16-feature block
  uint2 early[NVB][NBX];
  u32x4 rowv[NRL];
  if (in_sorted == 2) {
    if constexpr (STAGE) {
#pragma unroll
      for (int k = 0; k < NRL; ++k) {
        const uint32_t at = (uint32_t)g * (uint32_t)G + (uint32_t)(part * NVB * 16 + RPI * k + lr);
        // (non-temporal: a row is read once per layer, and what arrives was written by another XCD)
        rowv[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(
            feats + (size_t)(at < (uint32_t)n ? at : (uint32_t)n - 1u) * C + 8 * piece32));
      }
    } else {
#pragma unroll
      for (int vb = 0; vb < NVB; ++vb) {
        const uint32_t at = (uint32_t)g * (uint32_t)G + (uint32_t)((part * NVB + vb) * 16 + i);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          early[vb][nb] = *reinterpret_cast<const uint2*>(feats + (size_t)(at < (uint32_t)n ? at : (uint32_t)n - 1u) * C + 16 * nb + 4 * q);
      }
    }
  }
  int start = 0, m = 0;
  // A list of full groups only ('Drop Residual') has the next start beyond this group's end.
  if (g < ngroups) { start = off0; m = off1 - off0 < G ? off1 - off0 : G; }

  // ---- weight stream: global memory -> LDS ring -> registers -----------------------------------------
  // Chunk c of the packed stream lives in ring slot c % RING.  `issued` chunks have been requested,
  // chunks below `visible` are known to have landed for every wavefront.  Both advance only at
  // workgroup barriers that every wavefront reaches with the same values.
  int issued = 0, visible = 0;
  auto issue = [&](int chunk) {  // asynchronous copy, 1 KB per instruction, no registers in between
#pragma unroll
    for (int t = 0; t < (CF + NW - 1) / NW; ++t) {
      const int f = wu + t * NW;
      if ((t + 1) * NW <= CF || f < CF) {  // wave-uniform
        if constexpr (LEAN) {  // per-lane address form of the copy below: at 168 registers the scalar operands
                               // of the other form cost three spilled registers
          const u32x4* srcv = packed + ((size_t)chunk * CF + f) * 64 + lane;
          const uint32_t dst = (uint32_t)reinterpret_cast<uintptr_t>(
              (__attribute__((address_space(3))) void*)(ring + ((chunk % RING) * CF + f) * 64));
          asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                       :
                       : "s"(dst), "v"(srcv)
                       : "memory", "m0");
        } else {
          // The copy is written in assembly so that the compiler does not know of it: while it sees an
          // LDS-writing load in flight it waits for every counter to drain at each use of an LDS value
          // (lgkmcnt(0) after every refill of the register window, one exposed LDS latency each time).
          // The protocol above already orders these copies against the reads of the ring (vmcnt(0) and a
          // barrier before a chunk is read), and a vmcnt the compiler computes for its own loads only
          // waits longer with copies in flight that it does not count.
          const uint64_t src = reinterpret_cast<uint64_t>(packed + ((size_t)chunk * CF + f) * 64);  // wave-uniform
          const uint32_t dst = (uint32_t)reinterpret_cast<uintptr_t>(
              (__attribute__((address_space(3))) void*)(ring + ((chunk % RING) * CF + f) * 64));     // LDS byte address
          asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                       :
                       : "s"(dst), "v"(lane * 16), "s"(src)
                       : "memory", "m0");
        }
      }
    }
  };
  // Barrier.  Every wavefront has finished with all chunks below `consumed` when it arrives.
  auto sync = [&](int consumed) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // my share of every issued chunk has landed
    __syncthreads();
    visible = issued;
    const int lim = consumed + RING < NCHUNK ? consumed + RING : NCHUNK;
    while (issued < lim) { issue(issued); ++issued; }
  };
  // Before the first read of chunk cn.  voluntary: also stop when free slots could be refilled: two of
  // them, or all that is left of the stream (a barrier for a single slot is one barrier more in the
  // FFN, where nothing else needs one).
  auto boundary = [&](int cn, int consumed, bool voluntary) {
    if (cn >= NCHUNK) return;
    const int lim = consumed + RING < NCHUNK ? consumed + RING : NCHUNK;
    if (voluntary && lim > issued && (lim - issued >= 2 || lim == NCHUNK)) sync(consumed);
    while (cn >= visible) sync(consumed);
  };
  // An LDS read reaches 64 KB beyond its base register through the immediate offset; the ring can be
  // larger, so there are two bases, the second one hidden from constant folding.
  uint32_t hi_units = 4 * CF * 64;  // slots 4.. start here (u32x4 units)
  asm volatile("" : "+v"(hi_units));
  const u32x4* ring_lo = ring + lane;
  const u32x4* ring_hi = ring + hi_units + lane;
  auto slot_ptr = [&](int chunk) -> const u32x4* {
    const int slot = chunk % RING;
    return slot < 4 ? ring_lo + slot * CF * 64 : ring_hi + (slot - 4) * CF * 64;
  };

  issue(0);
  issue(1);
  issued = 2;

  // The per-feature vectors (LayerNorm scales and shifts, biases) follow the fragments in the packed buffer as
  // fp32 in the order of ParamOff: they go to LDS the way the weights do, 1 KB per instruction, spread over the
  // wavefronts, and are there for everyone after the first barrier.
  {
    constexpr int PIECES = LP::PARAMS / 1024;
#pragma unroll
    for (int t = 0; t < (PIECES + NW - 1) / NW; ++t) {
      const int piece = wu + t * NW;
      if ((t + 1) * NW <= PIECES || piece < PIECES) {  // wave-uniform
        const u32x4* srcp = packed + ((size_t)NCHUNK * CF + piece) * 64;
        // (LDS byte address from the ring's base: the pointer `par` sits in a vector register)
        const uint32_t dst = (uint32_t)reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) void*)ring) +
                             (uint32_t)(RING * CF + piece) * 1024u;
        if constexpr (LEAN) {
          const u32x4* srcv = srcp + lane;
          asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(dst), "v"(srcv) : "memory", "m0");
        } else {
          const uint64_t src = reinterpret_cast<uint64_t>(srcp);  // wave-uniform
          asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                       :
                       : "s"(dst), "v"(lane * 16), "s"(src)
                       : "memory", "m0");
        }
      }
    }
  }

  // ---- gather + LN1 ---------------------------------------------------------------------------------
  f32x4 x1[NVB][NB];  // residual stream of my pillars, accumulator layout
  int32_t row[NVB];   // pillar index, -1 for padding slots
  int32_t orow[NVB];  // row of `out` the result goes to
  const bool guessed = (int64_t)g * G == start;  // wave-uniform
#pragma unroll
  for (int vb = 0; vb < NVB; ++vb) {
    const int s = (part * NVB + vb) * 16 + i;
    if (guessed) row[vb] = s < m ? guess[vb] : -1;
    else row[vb] = s < m ? perm[start + s] : -1;
  }
  // rowv (whole rows, 16 bytes per lane) -> raw (accumulator layout) through the wavefront's LDS share
  auto turn_rows = [&](uint2 (&raw)[NVB][NB]) {
    u32x4* stg = reinterpret_cast<u32x4*>(kvx) + wu * (NVB * 256);  // [row][16-byte piece ^ (row & 15)]
#pragma unroll
    for (int p = 0; p < PH; ++p) {
#pragma unroll
      for (int k = 0; k < NRL; ++k) {
        const int r = RPI * k + lr;
        if (PH == 1 || ph == p) stg[r * 16 + (i ^ (r & 15))] = rowv[k];
      }
      // No barrier: the pieces are this wavefront's own, and its LDS instructions execute in order.  The
      // compiler must keep that order too (it sees stores and loads of different types).
      asm volatile("" ::: "memory");
#pragma unroll
      for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
        for (int nb = 8 * p; nb < 8 * p + 8; ++nb) {
          const int piece = 2 * (nb - 8 * p) + (q >> 1);
          raw[vb][nb] = *reinterpret_cast<const uint2*>(
              reinterpret_cast<const char*>(stg + (vb * 16 + i) * 16 + (piece ^ i)) + (q & 1) * 8);
        }
      asm volatile("" ::: "memory");
    }
  };
  if (in_sorted == 2 && guessed) {  // the early fetch hit
    uint2 raw[NVB][NB];
    if constexpr (STAGE) {
      turn_rows(raw);
    } else {
#pragma unroll
      for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) raw[vb][nb] = early[vb][nb];
    }
#pragma unroll
    for (int vb = 0; vb < NVB; ++vb) {
      const bool live = (part * NVB + vb) * 16 + i < m;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const uint2 u = raw[vb][nb];
        // (padding slots: the bits are cleared before the conversion, two instructions per block instead of a
        // branch around each block)
        const uint32_t keep = live ? 0xffffffffu : 0u;
        x1[vb][nb] = f32x4{el_lo(u.x & keep), el_hi(u.x & keep), el_lo(u.y & keep), el_hi(u.y & keep)};
      }
    }
  } else {
    // every lane loads (padding slots read a valid row and drop it): loads under a condition of their
    // own are waited for one by one
    uint2 raw[NVB][NB];
    int32_t srcv[NVB];  // row of feats for my pillar of block vb
#pragma unroll
    for (int vb = 0; vb < NVB; ++vb) {
      const int s = (part * NVB + vb) * 16 + i;
      srcv[vb] = row[vb] >= 0 ? (in_sorted ? start + s : row[vb]) : 0;
    }
    if constexpr (STAGE) {
#pragma unroll
      for (int k = 0; k < NRL; ++k) {  // row RPI k + lr of the wavefront: its index is held by the lane of that number
        const int32_t sr = __shfl(srcv[RPI * k / 16], (RPI * k) % 16 + lr, 64);
        rowv[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(feats + (int64_t)sr * C + 8 * piece32));
      }
        turn_rows(raw);
    } else {
#pragma unroll
      for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          raw[vb][nb] = *reinterpret_cast<const uint2*>(feats + (int64_t)srcv[vb] * C + 16 * nb + 4 * q);
      }
#pragma unroll
    for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const uint2 u = raw[vb][nb];
        const uint32_t keep = row[vb] >= 0 ? 0xffffffffu : 0u;
        x1[vb][nb] = f32x4{el_lo(u.x & keep), el_hi(u.x & keep), el_lo(u.y & keep), el_hi(u.y & keep)};
      }
  }
  // Positional embedding of my pillars, still bf16, in the layout of `act` (Eq. (2), second argument
  // of the attention): it is added to the LayerNorm output on the way to the query and key products.
  Frag8 pef[PE ? NVB : 1][PE ? KB : 1];
  if constexpr (PE) {
    uint2 praw[NVB][NB];
    if constexpr (STAGE && C == 128 && MINW <= 2) {  // whole rows through the LDS turn-around, like the features
                                                      // (where the registers allow it)
      int32_t prow[NVB];
#pragma unroll
      for (int vb = 0; vb < NVB; ++vb) prow[vb] = row[vb] >= 0 ? row[vb] : 0;
#pragma unroll
      for (int k = 0; k < NRL; ++k) {
        const int32_t sr = __shfl(prow[RPI * k / 16], (RPI * k) % 16 + lr, 64);
        rowv[k] = *reinterpret_cast<const u32x4*>(pos_embed + (int64_t)sr * C + 8 * piece32);
      }
      turn_rows(praw);
    } else {
#pragma unroll
      for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          praw[vb][nb] = *reinterpret_cast<const uint2*>(pos_embed + (int64_t)(row[vb] >= 0 ? row[vb] : 0) * C + 16 * nb + 4 * q);
    }
#pragma unroll
    for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        pef[vb][nb / 2].u[(nb & 1) * 2 + 0] = row[vb] >= 0 ? praw[vb][nb].x : 0u;
        pef[vb][nb / 2].u[(nb & 1) * 2 + 1] = row[vb] >= 0 ? praw[vb][nb].y : 0u;
      }
  }
  if (drop) {
    // Pillars of no group skip the layer: their rows are copied.  The wavefronts of group g take the
    // sorted positions between its end and the next group's start, those of group index 0 also the
    // positions before the first start (every position when the list is empty).
    auto copy_rows = [&](int lo, int hi) {
      constexpr int LPR = C / 8, RPW = 64 / LPR;  // 16 bytes per lane, several rows per wavefront
      const int sub = lane / LPR, col = (lane % LPR) * 8;
      hi = hi < n ? hi : n;
      for (int p = lo + part * RPW + sub; p < hi; p += WPG * RPW) {
        const int32_t pillar = perm[p];
        const u32x4 v = *reinterpret_cast<const u32x4*>(feats + (int64_t)(in_sorted ? p : pillar) * C + col);
        const int64_t at = (int64_t)(out_index ? out_index[pillar] : pillar) * C + col;
        if constexpr (OUT_F32) {
          float* dst = reinterpret_cast<float*>(out) + at;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            dst[2 * e] = el_lo(v[e]);
            dst[2 * e + 1] = el_hi(v[e]);
          }
        } else {
          *reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(out) + at) = v;
        }
      }
    };
    if (g == 0) copy_rows(0, ngroups > 0 ? off0 : n);
    if (g < ngroups) copy_rows(start + m, off1);
  }
  sync(0);  // chunks 0 and 1 and the small parameters are in LDS; the rest of the ring is requested
  // out_index: the next layer of a block wants its input in its own sorted order.  Fetched only now:
  // the barrier above waits for every load in flight, and this one hangs on the pillar index.
#pragma unroll
  for (int vb = 0; vb < NVB; ++vb) orow[vb] = out_index && row[vb] >= 0 ? out_index[row[vb]] : row[vb];

  // The window: fragments j .. j + PF - 1 of the stream are in registers (or on their way) while
  // fragment j is being used.
  Frag8 win[PF];
  auto fill_window = [&]() {
    const u32x4* p0 = slot_ptr(0);
#pragma unroll
    for (int f = 0; f < PF; ++f) win[f].q = p0[f * 64];
  };
  if (!LEAN) fill_window();  // early, so that the reads overlap the LayerNorm arithmetic
  __builtin_amdgcn_sched_barrier(0);

  Frag8 act[NVB][KB];  // normalised activations as B operands (LN1 output, later LN2 output)
  Frag8 actqk[PE ? NVB : 1][PE ? KB : 1];  // LN1 output plus the positional embedding: input of Q and K
  auto layer_norm = [&](int goff_f, int boff_f, bool first) {
    float sc[NVB], sh[NVB];  // y = x * sc + sh  with sc = rstd, sh = -mean * rstd
#pragma unroll
    for (int vb = 0; vb < NVB; ++vb) {
      float s = 0.f, ss = 0.f;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
        for (int j = 0; j < 4; ++j) { s += x1[vb][nb][j]; ss = fmaf(x1[vb][nb][j], x1[vb][nb][j], ss); }
      }
      const float mu = quad_sum(s) * (1.0f / C);
      const float var = fmaxf(quad_sum(ss) * (1.0f / C) - mu * mu, 0.f);
      sc[vb] = rsqrtf(var + eps);
      sh[vb] = -mu * sc[vb];
    }
    // the affine parameters come from LDS four feature blocks at a time, all eight reads of a batch
    // issued before the first is used (read, wait, use per block exposed the LDS latency every time)
    constexpr int NBG = LEAN ? 1 : 4;  // the lean mapping has no registers for a batch
    static_assert(NB % NBG == 0, "feature blocks per parameter batch");
#pragma unroll
    for (int nb0 = 0; nb0 < NB; nb0 += NBG) {
      f32x4 gmv[NBG], btv[NBG];
#pragma unroll
      for (int u = 0; u < NBG; ++u) {
        gmv[u] = *reinterpret_cast<const f32x4*>(par + goff_f + 16 * (nb0 + u) + 4 * q);
        btv[u] = *reinterpret_cast<const f32x4*>(par + boff_f + 16 * (nb0 + u) + 4 * q);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < NBG; ++u) {
      const int nb = nb0 + u;
      const f32x4 gm = gmv[u], bt = btv[u];
#pragma unroll
      for (int vb = 0; vb < NVB; ++vb) {
        float y[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) y[j] = fmaf(fmaf(x1[vb][nb][j], sc[vb], sh[vb]), gm[j], bt[j]);
        act[vb][nb / 2].u[(nb & 1) * 2 + 0] = pack2(y[0], y[1]);
        act[vb][nb / 2].u[(nb & 1) * 2 + 1] = pack2(y[2], y[3]);
        if constexpr (PE) {
          if (first) {
            const uint32_t p01 = pef[vb][nb / 2].u[(nb & 1) * 2 + 0], p23 = pef[vb][nb / 2].u[(nb & 1) * 2 + 1];
            actqk[vb][nb / 2].u[(nb & 1) * 2 + 0] =
                pack2(y[0] + el_lo(p01), y[1] + el_hi(p01));
            actqk[vb][nb / 2].u[(nb & 1) * 2 + 1] =
                pack2(y[2] + el_lo(p23), y[3] + el_hi(p23));
          }
        }
      }
      }
    }
  };
  auto add_bias_rows = [&](int off_f) {  // x1 += per-feature vector
    constexpr int NBG = LEAN ? 1 : 8;  // reads of a batch issued together, as in layer_norm
#pragma unroll
    for (int nb0 = 0; nb0 < NB; nb0 += NBG) {
      f32x4 b[NBG];
#pragma unroll
      for (int u = 0; u < NBG; ++u) b[u] = *reinterpret_cast<const f32x4*>(par + off_f + 16 * (nb0 + u) + 4 * q);
#pragma unroll
      for (int u = 0; u < NBG; ++u)
#pragma unroll
        for (int vb = 0; vb < NVB; ++vb) x1[vb][nb0 + u] += b[u];
    }
  };
  // Bias of the Q rows of a unit (accumulator layout).  K and V start from zero: the key bias has no
  // effect on the softmax and the value bias is part of the folded output bias.
  f32x4 bqk[2];
  auto load_unit_bias = [&](int hp) {
#pragma unroll
    for (int c = 0; c < 2; ++c) bqk[c] = *reinterpret_cast<const f32x4*>(par + PO::BQ + 32 * hp + 16 * c + 4 * q);
  };
  if (!LEAN) load_unit_bias(0);
  layer_norm(PO::LN1G, PO::LN1B, true);
  add_bias_rows(PO::BO);  // residual + output-projection bias
  if (LEAN) { __builtin_amdgcn_sched_barrier(0); fill_window(); }
  const float qscale = rsqrtf((float)DH) * 1.44269504088896340736f;  // 1/sqrt(d) * log2(e)
  // wave-uniform: some key slots are padding.  A wavefront past the last group (m == 0) keeps all its
  // (zero) keys instead, so that it computes finite numbers it never stores rather than -inf - -inf.
  const bool short_group = m > 0 && m < NKB * 16;

  // ---- attention: one 32-wide head-dim unit per iteration (two heads of 16 or one head of 32) --------
#pragma unroll ATT_UNROLL
  for (int hp = 0; hp < HP; ++hp) {
    const int c0 = hp * CPH;
    const u32x4* pb[CPH + 1];
#pragma unroll
    for (int k = 0; k <= CPH; ++k) pb[k] = slot_ptr(c0 + k);
    // fragment j of this unit has been used: refill its window slot with fragment j + PF
    auto refill = [&](int j) {
      const int jj = j + PF, k = jj / CF;
      __builtin_amdgcn_sched_barrier(0);
      if (jj % CF == 0) boundary(c0 + k, c0 + (j + 1) / CF, WPG == 1);
      win[j % PF].q = pb[k][(jj % CF) * 64];  // a hidden unit always follows: the chunk exists
      __builtin_amdgcn_sched_barrier(0);
    };
    if (LEAN) load_unit_bias(hp);
    Frag4 Qf[2][NVB], Kf[2][NVB], Vf[2][NVB];  // bf16 fragments of my pillars, index [16-block a][vb]
    u32x2* kv = kvx + (size_t)((hp & 1) * GPW + gl) * (2 * 2 * NKB * 64) + lane;  // this unit's exchange buffer

    // Six accumulation chains: Q a=0,1 and K a=0,1 as D[feature][pillar], V a=0,1 with the operand
    // roles swapped as D[pillar][feature].  The conversion of a finished chain is issued after the
    // first product of the next one.
    {
      f32x4 acc[2][NVB];
      auto finish = [&](int ch) {
        const int a = ch & 1;
#pragma unroll
        for (int vb = 0; vb < NVB; ++vb) {
          Frag4& dst = ch < 2 ? Qf[a][vb] : ch < 4 ? Kf[a][vb] : Vf[a][vb];
          dst.u[0] = pack2(acc[ch & 1][vb][0], acc[ch & 1][vb][1]);
          dst.u[1] = pack2(acc[ch & 1][vb][2], acc[ch & 1][vb][3]);
          // K/V of the whole group go through LDS: [K|V][16-block a][key block][lane]
          if (WPG > 1 && ch >= 2) kv[(((ch >= 4 ? 1 : 0) * 2 + a) * NKB + part * NVB + vb) * 64] = dst.d;
        }
      };
      // Stream order (kQkvOrder): K and V first, so that their way to LDS overlaps the Q products
      // instead of standing between the last product and the barrier.
#pragma unroll
      for (int p = 0; p < 6; ++p) {
        const int ch = kQkvOrder[p];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
          const int j = p * KB + kb;
          const Frag8 wf = win[j % PF];
          if (kb == 0) {  // the accumulator starts from the bias
#pragma unroll
            for (int vb = 0; vb < NVB; ++vb)
              acc[ch & 1][vb] = ch < 2 ? bqk[ch] : f32x4{0.f, 0.f, 0.f, 0.f};
          }
#pragma unroll
          for (int vb = 0; vb < NVB; ++vb)
            acc[ch & 1][vb] = ch < 4 ? mfma32(wf, PE ? actqk[PE ? vb : 0][PE ? kb : 0] : act[vb][kb], acc[ch & 1][vb])
                                     : mfma32(act[vb][kb], wf, acc[ch & 1][vb]);
          if (kb == 0 && p > 0) finish(kQkvOrder[p - 1]);
          refill(j);
        }
      }
      finish(kQkvOrder[5]);
    }
    if (WPG > 1) sync(c0 + (6 * KB) / CF);  // K/V of the group are in LDS
    if (!LEAN) load_unit_bias(hp + 1 < HP ? hp + 1 : hp);
    auto Kget = [&](int a, int jb) -> Frag4 {
      if (WPG == 1) return Kf[a][jb];
      Frag4 f; f.d = kv[((0 * 2 + a) * NKB + jb) * 64]; return f;
    };
    auto Vget = [&](int a, int jb) -> Frag4 {
      if (WPG == 1) return Vf[a][jb];
      Frag4 f; f.d = kv[((1 * 2 + a) * NKB + jb) * 64]; return f;
    };
    Frag8 Of[NVB];  // attention output of this unit as B operand of the output projection
    constexpr int NH = 32 / DH;   // heads in this unit
    constexpr int NA = DH / 16;   // 16-blocks of head dims per head
    // The (head, pillar-block) instances are independent; they go through the softmax in
    // lockstep stages so that the long per-instance dependency chains interleave.  HJ heads are
    // staged jointly, limited by the registers the score tiles take.
    constexpr int VJ = NVB * NKB <= 16 ? NVB : (16 / NKB >= 1 ? 16 / NKB : 1);
    constexpr int HJ = (NH * VJ * NKB <= 16 && MINW < 4) ? NH : 1;
    static_assert(NVB % VJ == 0, "pillar blocks per stage");
#pragma unroll
    for (int v0 = 0; v0 < NVB; v0 += VJ)
#pragma unroll
    for (int h0 = 0; h0 < NH; h0 += HJ) {
      f32x4 S[HJ][VJ][NKB];  // scores, transposed: S[key 16*jb + 4q + j][query i]
#pragma unroll
      for (int hh = 0; hh < HJ; ++hh) {
        const int h = h0 + hh;
#pragma unroll
        for (int vb = 0; vb < VJ; ++vb) {
#pragma unroll
          for (int jb = 0; jb < NKB; ++jb) {
            const f32x4 z = f32x4{0.f, 0.f, 0.f, 0.f};
            if (DH == 16) {
              // the only k=16 products left: their accumulator input is zero, so they depend on no
              // earlier product (see the note at the odd key block below)
              S[hh][vb][jb] = mfma16_from_zero(Kget(h, jb), Qf[h][v0 + vb]);
            } else {
              Frag8 k8, q8;
              const Frag4 k0 = Kget(0, jb), k1 = Kget(1, jb);
              k8.u[0] = k0.u[0]; k8.u[1] = k0.u[1]; k8.u[2] = k1.u[0]; k8.u[3] = k1.u[1];
              q8.u[0] = Qf[0][v0 + vb].u[0]; q8.u[1] = Qf[0][v0 + vb].u[1]; q8.u[2] = Qf[1][v0 + vb].u[0]; q8.u[3] = Qf[1][v0 + vb].u[1];
              S[hh][vb][jb] = mfma32(k8, q8, z);
            }
          }
        }
      }
      if (short_group) {  // keys beyond the group's real members
#pragma unroll
        for (int hh = 0; hh < HJ; ++hh)
#pragma unroll
          for (int vb = 0; vb < VJ; ++vb)
#pragma unroll
            for (int jb = 0; jb < NKB; ++jb)
#pragma unroll
              for (int j = 0; j < 4; ++j)
                if (16 * jb + 4 * q + j >= m) S[hh][vb][jb][j] = -INFINITY;
      }
      float mxs[HJ][VJ];
#pragma unroll
      for (int hh = 0; hh < HJ; ++hh) {
#pragma unroll
        for (int vb = 0; vb < VJ; ++vb) {
          float mx = S[hh][vb][0][0];
#pragma unroll
          for (int jb = 0; jb < NKB; ++jb)
#pragma unroll
            for (int j = 0; j < 4; ++j) mx = fmaxf(mx, S[hh][vb][jb][j]);
          mxs[hh][vb] = mx;
        }
      }
#pragma unroll
      for (int hh = 0; hh < HJ; ++hh)
#pragma unroll
        for (int vb = 0; vb < VJ; ++vb) mxs[hh][vb] = -quad_max(mxs[hh][vb]) * qscale;
      // p = 2^((s - max) * log2(e) / sqrt(d)): the score scale lives in the exponent argument
#pragma unroll
      for (int hh = 0; hh < HJ; ++hh)
#pragma unroll
        for (int vb = 0; vb < VJ; ++vb)
#pragma unroll
          for (int jb = 0; jb < NKB; ++jb)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              S[hh][vb][jb][j] = __builtin_amdgcn_exp2f(fmaf(S[hh][vb][jb][j], qscale, mxs[hh][vb]));
            }
      // O^T[d][query] = sum over keys V^T[d][key] P^T[key][query], two key blocks per product.
      // The row sums of P come from the matrix cores as well: an all-ones A operand makes every
      // accumulator row the sum over keys of the (bf16-rounded) probabilities.
      f32x4 O[HJ][VJ][NA], rowsum[HJ][VJ];
#pragma unroll
      for (int hh = 0; hh < HJ; ++hh) {
        const int h = h0 + hh;
#pragma unroll
        for (int vb = 0; vb < VJ; ++vb) {
          rowsum[hh][vb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int a = 0; a < NA; ++a) O[hh][vb][a] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int jb = 0; jb + 1 < NKB; jb += 2) {
            Frag8 p8;
            p8.u[0] = pack2(S[hh][vb][jb][0], S[hh][vb][jb][1]); p8.u[1] = pack2(S[hh][vb][jb][2], S[hh][vb][jb][3]);
            p8.u[2] = pack2(S[hh][vb][jb + 1][0], S[hh][vb][jb + 1][1]);
            p8.u[3] = pack2(S[hh][vb][jb + 1][2], S[hh][vb][jb + 1][3]);
#pragma unroll
            for (int a = 0; a < NA; ++a) {
              const int ab = DH == 16 ? h : a;
              const Frag4 v0 = Vget(ab, jb), v1 = Vget(ab, jb + 1);
              Frag8 v8;
              v8.u[0] = v0.u[0]; v8.u[1] = v0.u[1]; v8.u[2] = v1.u[0]; v8.u[3] = v1.u[1];
              O[hh][vb][a] = mfma32(v8, p8, O[hh][vb][a]);
            }
            Frag8 ones;
            ones.u[0] = ones.u[1] = ones.u[2] = ones.u[3] = kOnePair;
            rowsum[hh][vb] = mfma32(ones, p8, rowsum[hh][vb]);
          }
          if (NKB & 1) {
            // The odd last key block: a k=32 product whose upper half multiplies zeros.  A k=16
            // product here was wrong on this chip: issued right behind a k=32 product into the same
            // accumulator it read the accumulator before that product had written it (row sums of 48
            // instead of 80, whenever the scheduler put the two back to back), so every product of an
            // accumulation chain is of one kind.  The k=16 product takes the same 16 cycles anyway.
            constexpr int jb = NKB - 1;
            Frag8 p8;
            p8.u[0] = pack2(S[hh][vb][jb][0], S[hh][vb][jb][1]); p8.u[1] = pack2(S[hh][vb][jb][2], S[hh][vb][jb][3]);
            p8.u[2] = p8.u[3] = 0u;
#pragma unroll
            for (int a = 0; a < NA; ++a) {
              const Frag4 v0 = Vget(DH == 16 ? h : a, jb);
              Frag8 v8;
              v8.u[0] = v0.u[0]; v8.u[1] = v0.u[1]; v8.u[2] = v8.u[3] = 0u;
              O[hh][vb][a] = mfma32(v8, p8, O[hh][vb][a]);
            }
            Frag8 ones;
            ones.u[0] = ones.u[1] = ones.u[2] = ones.u[3] = kOnePair;
            rowsum[hh][vb] = mfma32(ones, p8, rowsum[hh][vb]);
          }
        }
      }
#pragma unroll
      for (int hh = 0; hh < HJ; ++hh) {
        const int h = h0 + hh;
#pragma unroll
        for (int vb = 0; vb < VJ; ++vb) {
          const float inv = __builtin_amdgcn_rcpf(rowsum[hh][vb][0]);
#pragma unroll
          for (int a = 0; a < NA; ++a) {
            const int slot = DH == 16 ? h : a;
            Of[v0 + vb].u[slot * 2 + 0] = pack2(O[hh][vb][a][0] * inv, O[hh][vb][a][1] * inv);
            Of[v0 + vb].u[slot * 2 + 1] = pack2(O[hh][vb][a][2] * inv, O[hh][vb][a][3] * inv);
          }
        }
      }
    }
    // output projection of this unit, accumulated into the residual stream
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int j = 6 * KB + nb;
      const Frag8 wf = win[j % PF];
#pragma unroll
      for (int vb = 0; vb < NVB; ++vb) x1[vb][nb] = mfma32(wf, Of[vb], x1[vb][nb]);
      refill(j);
    }
  }

  // ---- FFN ------------------------------------------------------------------------------------------
  f32x4 b1r[2];
  auto load_b1 = [&](int fc) {
#pragma unroll
    for (int a = 0; a < 2; ++a) b1r[a] = *reinterpret_cast<const f32x4*>(par + PO::B1 + 32 * fc + 16 * a + 4 * q);
  };
  if (!LEAN) load_b1(0);
  layer_norm(PO::LN2G, PO::LN2B, false);
  add_bias_rows(PO::B2);
#pragma unroll FFN_UNROLL
  for (int fc = 0; fc < FC; ++fc) {
    const int c0 = HP * CPH + fc * CPF;
    const u32x4* pb[CPF + 1];
#pragma unroll
    for (int k = 0; k <= CPF; ++k) pb[k] = slot_ptr(c0 + k);
    auto refill = [&](int j) {
      const int jj = j + PF, k = jj / CF;
      __builtin_amdgcn_sched_barrier(0);
      if (jj % CF == 0) boundary(c0 + k, c0 + (j + 1) / CF, true);
      if (k < CPF || fc + 1 < FC) win[j % PF].q = pb[k][(jj % CF) * 64];
      __builtin_amdgcn_sched_barrier(0);
    };
    Frag8 Hf[NVB];
    if (LEAN) load_b1(fc);
    {
      f32x4 acc[2][NVB];
      auto finish = [&](int a) {
#pragma unroll
        for (int vb = 0; vb < NVB; ++vb) {
          Hf[vb].u[a * 2 + 0] = pack2(gelu2_fast(acc[a][vb][0]), gelu2_fast(acc[a][vb][1]));
          Hf[vb].u[a * 2 + 1] = pack2(gelu2_fast(acc[a][vb][2]), gelu2_fast(acc[a][vb][3]));
        }
      };
#pragma unroll
      for (int a = 0; a < 2; ++a) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
          const int j = a * KB + kb;
          const Frag8 wf = win[j % PF];
          if (kb == 0) {
#pragma unroll
            for (int vb = 0; vb < NVB; ++vb) acc[a][vb] = b1r[a];
          }
#pragma unroll
          for (int vb = 0; vb < NVB; ++vb) acc[a][vb] = mfma32(wf, act[vb][kb], acc[a][vb]);
          if (kb == 0 && a == 1) finish(0);
          refill(j);
        }
      }
      finish(1);
    }
    if (!LEAN) load_b1(fc + 1 < FC ? fc + 1 : fc);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int j = 2 * KB + nb;
      const Frag8 wf = win[j % PF];
#pragma unroll
      for (int vb = 0; vb < NVB; ++vb) x1[vb][nb] = mfma32(wf, Hf[vb], x1[vb][nb]);
      refill(j);
    }
  }

  // ---- scatter -------------------------------------------------------------------------------------
  if constexpr (STAGE && !OUT_F32) {
    // The way the rows came in: through the wavefront's LDS share (free again since the attention
    // ended), so that a store instruction writes four complete rows instead of 32 bytes of sixteen.
    u32x4* stg = reinterpret_cast<u32x4*>(kvx) + wu * (NVB * 256);
#pragma unroll
    for (int p = 0; p < PH; ++p) {
#pragma unroll
      for (int vb = 0; vb < NVB; ++vb)
#pragma unroll
        for (int nb = 8 * p; nb < 8 * p + 8; ++nb) {
          const int piece = 2 * (nb - 8 * p) + (q >> 1);
          *reinterpret_cast<uint2*>(reinterpret_cast<char*>(stg + (vb * 16 + i) * 16 + (piece ^ i)) + (q & 1) * 8) =
              make_uint2(pack2(x1[vb][nb][0], x1[vb][nb][1]), pack2(x1[vb][nb][2], x1[vb][nb][3]));
        }
      asm volatile("" ::: "memory");  // keeps the order of the LDS stores above and the loads below
#pragma unroll
      for (int k = 0; k < NRL; ++k) {
        const int r = RPI * k + lr;
        const int32_t orw = __shfl(orow[RPI * k / 16], (RPI * k) % 16 + lr, 64);  // output row of row r
        if (PH == 1 || ph == p) {
          const u32x4 v = stg[r * 16 + (i ^ (r & 15))];
          if (orw >= 0)  // non-temporal: the next reader is another XCD, and the kernel's end has less to write back
            __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(out) + (size_t)orw * C + 8 * piece32));
        }
      }
      asm volatile("" ::: "memory");
    }
  } else {
#pragma unroll
    for (int vb = 0; vb < NVB; ++vb) {
      if (row[vb] < 0) continue;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const size_t o = (size_t)orow[vb] * C + 16 * nb + 4 * q;
        if (OUT_F32) {
          *reinterpret_cast<float4*>(reinterpret_cast<float*>(out) + o) =
              make_float4(x1[vb][nb][0], x1[vb][nb][1], x1[vb][nb][2], x1[vb][nb][3]);
        } else {
          *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(out) + o) =
              make_uint2(pack2(x1[vb][nb][0], x1[vb][nb][1]), pack2(x1[vb][nb][2], x1[vb][nb][3]));
        }
      }
    }
  }
}

template <int C, int DH, int F, int NVB, int WPG, int NW, int MINW>
int launch_cfg(const void* feats, void* out, const void* pos_embed, const int32_t* perm, const int32_t* goff,
               const int32_t* num_groups,
               int32_t max_groups, const u32x4* packed, float eps, bool out_f32, int n, int G,
               int drop, const int32_t* out_index, int in_sorted, hipStream_t stream) {
  constexpr int GPW = NW / WPG;
  const size_t lds_bytes = LdsPlan<C, F, NVB, WPG, NW, MINW>::TOTAL;
  const unsigned blocks = (unsigned)((max_groups + GPW - 1) / GPW);
  // The dynamic LDS size has to be allowed once per kernel and device (output type and positional
  // embedding make four kernels of a mapping).
  static std::atomic<uint64_t> allowed[4] = {{0}, {0}, {0}, {0}};  // bit d: done on device d
  auto go = [&](auto kern, int which) -> int {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return FF_ERR_LAUNCH;
    const uint64_t bit = 1ull << (dev & 63);
    if (!(allowed[which].load(std::memory_order_acquire) & bit)) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)lds_bytes) != hipSuccess)
        return FF_ERR_LAUNCH;
      allowed[which].fetch_or(bit, std::memory_order_release);
    }
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(NW * 64), lds_bytes, stream, (const uint16_t*)feats, out,
                       (const uint16_t*)pos_embed, perm, goff,
                       num_groups, (int)max_groups, packed, eps, n, G, drop, out_index, in_sorted);
    return launch_status();
  };
  if (pos_embed) {
    // Three mappings have no registers left for the second operand set (they would spill, which no
    // shipped mapping may): they are not built with a positional embedding.
    constexpr bool kFits = !(C == 128 && NVB == 2 && WPG == 1) && !(C == 256 && NW == 10) && !(C == 128 && NW == 12);
    if constexpr (kFits) {
      if (out_f32) return go(k_layer_mfma<C, DH, F, NVB, WPG, NW, MINW, true, true>, 3);
      return go(k_layer_mfma<C, DH, F, NVB, WPG, NW, MINW, false, true>, 2);
    } else {
      return FF_ERR_UNSUPPORTED;
    }
  }
  if (out_f32) return go(k_layer_mfma<C, DH, F, NVB, WPG, NW, MINW, true, false>, 1);
  return go(k_layer_mfma<C, DH, F, NVB, WPG, NW, MINW, false, false>, 0);
}

}  // namespace

// Shapes with a fused kernel: (C, head dim, F) = (128, 16, 256), (256, 32, 512) and (64, 16, 128), G <= 128.
static int shape_id(const ff_layer_weights* w) {
  const int C = w->C, F = w->F, d = C / w->heads;
  if (C == 128 && d == 16 && F == 256) return 1;
  if (C == 256 && d == 32 && F == 512) return 2;
  if (C == 64 && d == 16 && F == 128) return 3;
  return 0;
}

#ifndef FF_LAYER_F16  // the same for both formats
bool layer_mfma_supported(const ff_layer_weights* w, int G) { return shape_id(w) != 0 && G <= 128; }
#endif

static size_t layer_mfma_frag_count(const ff_layer_weights* w) {
  const int C = w->C, F = w->F;
  return (size_t)((C / 32) * frags_per_hp(C) + (F / 32) * frags_per_fc(C));
}

#ifndef FF_LAYER_F16
size_t layer_mfma_packed_bytes(const ff_layer_weights* w) {
  return layer_mfma_frag_count(w) * (size_t)1024 + (size_t)pack_param_bytes(w->C, w->F);
}
#endif

// Packs `count` layers of identical shape; layer l goes to packed + l * stride_bytes.
int FF_LAYER_SYM(layer_mfma_pack)(const ff_layer_weights* w, int count, void* packed, size_t stride_bytes,
                                  hipStream_t stream) {
  for (int l0 = 0; l0 < count; l0 += kPackBatch) {
    const int nl = count - l0 < kPackBatch ? count - l0 : kPackBatch;
    PackJob job;
    make_pack_job(w + l0, nl, (char*)packed + (size_t)l0 * stride_bytes, stride_bytes, kHalf, &job);
    hipLaunchKernelGGL(k_pack_weights, dim3((unsigned)job.blocks, (unsigned)nl), dim3(256), 0, stream, job.pb, job.C,
                       job.F, job.total_frags);
  }
  return launch_status();
}

// variant: 0 = chosen from the shape; 1.. = a specific wave/group mapping (tuning and tests).
int FF_LAYER_SYM(layer_mfma_launch)(const void* feats, void* out, int64_t n, const int32_t* perm, const int32_t* group_offsets,
                      const int32_t* num_groups, int32_t max_groups, const ff_layer_weights* w, int G,
                      bool out_f32, bool drop, const void* packed, int variant, const int32_t* out_index,
                      int in_sorted, hipStream_t stream) {
  if (max_groups == 0 || n == 0) return FF_OK;
  const u32x4* pk = (const u32x4*)packed;
#define FF_GO(C, DH, F, NVB, WPG, NW, MINW) \
  return launch_cfg<C, DH, F, NVB, WPG, NW, MINW>(feats, out, w->pos_embed, perm, group_offsets, num_groups, max_groups, pk, \
                                                  w->ln_eps, out_f32, (int)n, G, drop ? 1 : 0, out_index, in_sorted, stream)
  const int shape = shape_id(w);
  // (pillar blocks per wave, waves per group, waves per workgroup, min waves per SIMD)
  if (shape == 1) {
    if (variant == 0) {
      // G <= 64: two, three or four groups per workgroup (8, 12, 16 wavefronts; one workgroup per compute unit).
      // More wavefronts on a SIMD hide more of each other's stalls, but a round (one workgroup per compute
      // unit) takes longer and the attention loop is no longer unrolled completely: 16.4, 23.2 and 28.8 us a
      // round at this shape.  Many rounds: four groups lead (60,000 groups: 1.76, 1.61, 1.56 ms); few: the
      // number of rounds decides (measured, in us: 938 groups 33 / 44 / 30, 1407: 49 / 48 / 56, 1875: 65 / 69 /
      // 60, 2344: 81 / 89 / 81, 3750: 128 / 120 / 115, 7500: 256 / 228 / 219, 15,000: 477 / 419 / 390).
      auto rounds = [&](int per_wg) { return ceil_div(ceil_div((int64_t)max_groups, per_wg), kComputeUnits); };
      const int64_t c2 = rounds(2) * 164, c4 = rounds(4) * 288;
      // (the three-group mapping has no registers for a positional embedding)
      const int64_t c3 = w->pos_embed ? INT64_MAX : rounds(3) * 232;
      variant = G <= 32 ? 10 : G > 64 ? 9 : (c2 <= c3 && c2 <= c4) ? 7 : c3 <= c4 ? 11 : 12;
    }
    switch (variant) {
      case 1: if (G <= 32) FF_GO(128, 16, 256, 2, 1, 4, 2); break;
      case 2: if (G <= 64) FF_GO(128, 16, 256, 2, 2, 4, 1); break;  // 512 registers
      case 4: if (G <= 128) FF_GO(128, 16, 256, 2, 4, 4, 1); break;
      case 6: if (G <= 64) FF_GO(128, 16, 256, 1, 4, 4, 2); break;
      case 7: if (G <= 64) FF_GO(128, 16, 256, 1, 4, 8, 2); break;
      case 9: if (G <= 128) FF_GO(128, 16, 256, 1, 8, 8, 2); break;
      case 10: if (G <= 32) FF_GO(128, 16, 256, 1, 2, 8, 2); break;
      case 11: if (G <= 64) FF_GO(128, 16, 256, 1, 4, 12, 3); break;  // three groups, three waves per SIMD
      case 12: if (G <= 64) FF_GO(128, 16, 256, 1, 4, 16, 4); break;  // four groups, four waves per SIMD
      default: break;
    }
  } else if (shape == 2) {
    // with a positional embedding the ten-wave mapping has no registers to spare: one group per workgroup instead
    if (variant == 0) variant = G <= 32 ? 1 : G <= 64 ? 2 : G <= 80 ? (w->pos_embed ? 6 : 3) : 4;
    switch (variant) {
      case 1: if (G <= 32) FF_GO(256, 32, 512, 1, 2, 8, 2); break;
      case 2: if (G <= 64) FF_GO(256, 32, 512, 1, 4, 8, 2); break;
      case 3: if (G <= 80) FF_GO(256, 32, 512, 1, 5, 10, 2); break;  // lean: 168 registers, no scratch
      case 4: if (G <= 128) FF_GO(256, 32, 512, 1, 8, 8, 2); break;
      case 5: if (G <= 64) FF_GO(256, 32, 512, 2, 2, 4, 1); break;
      case 6: if (G <= 80) FF_GO(256, 32, 512, 1, 5, 5, 1); break;
      default: break;
    }
  } else if (shape == 3) {  // the narrow layer (64 features, 4 heads): the whole 64 KB weight stream stays in the ring
    if (variant == 0) variant = G <= 32 ? 1 : G <= 64 ? 2 : 4;
    switch (variant) {
      case 1: if (G <= 32) FF_GO(64, 16, 128, 1, 2, 8, 2); break;
      case 2: if (G <= 64) FF_GO(64, 16, 128, 1, 4, 8, 2); break;
      case 4: if (G <= 128) FF_GO(64, 16, 128, 1, 8, 8, 2); break;
      default: break;
    }
  }
#undef FF_GO
  return FF_ERR_UNSUPPORTED;
}

}  // namespace ff
