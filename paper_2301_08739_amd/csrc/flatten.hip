// Window-based sorting and equal-size grouping (paper Sec. 4.2.1, Eq. (1); Sec. 4.2.2 'Window
// Shift'; Sec. 4.3 'Reuse Sorting' is the caller keeping the result).
//
// Each pillar becomes ONE 64-bit word  (compact_key << idx_bits) | original_index, where the
// compact key packs the tuple fields (b, W_major, W_minor, L_major, L_minor) using only as many
// bits as the geometry needs.  An LSD radix sort over the compact-key bits, 8 bits per pass, is
// stable, so equal tuples keep ascending original index.  The word carries the index, so a pass
// moves 8 bytes per pillar each way.
//
// Pass structure: per-tile digit histogram -> exclusive scan over (digit, tile) -> stable
// rank-and-scatter.  Ranking inside a tile is done per wavefront with ballot-based digit matching
// and LDS counters; keys are staged through LDS so global writes come out in runs.
#include "common.h"

namespace ff {

namespace {

struct KeyParams {
  int32_t B, grid_x, grid_y, win_x, win_y;
  int32_t sx, sy;                       // shift added to x / y
  int32_t axis;
  int32_t bits_b, bits_w1, bits_w2, bits_l1, bits_l2;
  int32_t key_bits, idx_bits;
};

__device__ __forceinline__ uint32_t field_mask(int bits) { return bits >= 32 ? 0xffffffffu : ((1u << bits) - 1u); }

// ---- A1: coords -> sortable word ----------------------------------------------------------------
__global__ __launch_bounds__(256) void k_keygen(const int32_t* __restrict__ coords, int64_t n,
                                                 KeyParams kp, uint64_t* __restrict__ words) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  uint32_t b = (uint32_t)coords[3 * i + 0];
  uint32_t X = (uint32_t)(coords[3 * i + 1] + kp.sx);
  uint32_t Y = (uint32_t)(coords[3 * i + 2] + kp.sy);
  uint32_t Wx = X / (uint32_t)kp.win_x, Lx = X - Wx * (uint32_t)kp.win_x;
  uint32_t Wy = Y / (uint32_t)kp.win_y, Ly = Y - Wy * (uint32_t)kp.win_y;
  uint32_t w1 = kp.axis == 0 ? Wx : Wy, w2 = kp.axis == 0 ? Wy : Wx;
  uint32_t l1 = kp.axis == 0 ? Lx : Ly, l2 = kp.axis == 0 ? Ly : Lx;
  // Fields are masked to their widths so that a coordinate outside the geometry can only
  // disturb the order, never another field's bits or any index computed from them.
  uint64_t k = b & field_mask(kp.bits_b);
  k = (k << kp.bits_w1) | (w1 & field_mask(kp.bits_w1));
  k = (k << kp.bits_w2) | (w2 & field_mask(kp.bits_w2));
  k = (k << kp.bits_l1) | (l1 & field_mask(kp.bits_l1));
  k = (k << kp.bits_l2) | (l2 & field_mask(kp.bits_l2));
  words[i] = (kp.idx_bits >= 64 ? 0ull : (k << kp.idx_bits)) | (uint64_t)i;
}

// ---- block-wide exclusive scan of one uint32 per thread (256 threads) -------------------------
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    uint32_t t = __shfl_up(v, d, 64);
    if (lane >= d) v += t;
  }
  return v;
}

template <int THREADS>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* wave_totals /*[THREADS/64]*/,
                                                         uint32_t* block_total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  uint32_t inc = wave_inclusive_scan(v);
  if (lane == 63) wave_totals[w] = inc;
  __syncthreads();
  uint32_t base = 0, total = 0;
#pragma unroll
  for (int i = 0; i < THREADS / 64; ++i) {
    uint32_t t = wave_totals[i];
    if (i < w) base += t;
    total += t;
  }
  if (block_total) *block_total = total;
  __syncthreads();
  return base + inc - v;
}

// ---- A2, step 1: digit histogram of one tile ---------------------------------------------------
__global__ __launch_bounds__(kSortThreads) void k_radix_hist(const uint64_t* __restrict__ in, int64_t n,
                                                              int shift, uint32_t mask, int64_t tiles,
                                                              uint32_t* __restrict__ tile_hist) {
  __shared__ uint32_t h[kBins];
  const int tid = threadIdx.x;
  h[tid] = 0;
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * kTile;
#pragma unroll
  for (int r = 0; r < kKeysPerThread; ++r) {
    int64_t e = base + r * kSortThreads + tid;
    if (e < n) atomicAdd(&h[(uint32_t)(in[e] >> shift) & mask], 1u);
  }
  __syncthreads();
  tile_hist[(int64_t)tid * tiles + blockIdx.x] = h[tid];
}

// ---- A2, step 2: exclusive scan over the (digit-major, tile-minor) table -------------------------
__global__ __launch_bounds__(1024) void k_scan_table(uint32_t* __restrict__ table, int64_t len) {
  __shared__ uint32_t wave_totals[16];
  __shared__ uint32_t carry_s;
  if (threadIdx.x == 0) carry_s = 0;
  __syncthreads();
  for (int64_t base = 0; base < len; base += 1024) {
    int64_t i = base + threadIdx.x;
    uint32_t v = i < len ? table[i] : 0u;
    uint32_t total;
    uint32_t ex = block_exclusive_scan<1024>(v, wave_totals, &total);
    uint32_t carry = carry_s;
    if (i < len) table[i] = carry + ex;
    __syncthreads();
    if (threadIdx.x == 0) carry_s = carry + total;
    __syncthreads();
  }
}

// ---- A2, step 3: stable rank inside the tile, then scatter ----------------------------------
__global__ __launch_bounds__(kSortThreads) void k_radix_scatter(const uint64_t* __restrict__ in,
                                                                 uint64_t* __restrict__ out, int64_t n,
                                                                 int shift, uint32_t mask, int64_t tiles,
                                                                 const uint32_t* __restrict__ tile_base) {
  constexpr int KPT = kKeysPerThread;
  constexpr int WAVES = kSortThreads / 64;
  __shared__ uint32_t wave_cnt[WAVES][kBins];
  __shared__ uint32_t digit_start[kBins];
  __shared__ uint32_t gbase[kBins];
  __shared__ uint32_t wave_totals[WAVES];
  __shared__ uint64_t stage[kTile];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int64_t tile_start = (int64_t)blockIdx.x * kTile;
  const int tile_count = (int)((n - tile_start) < (int64_t)kTile ? (n - tile_start) : (int64_t)kTile);

#pragma unroll
  for (int i = 0; i < WAVES; ++i) wave_cnt[i][tid] = 0;
  gbase[tid] = tile_base[(int64_t)tid * tiles + blockIdx.x];
  __syncthreads();

  // Element order inside the tile: wave-major, then round, then lane.  Each wave owns a
  // contiguous run of 64*KPT words, so stability only needs (wave, round, lane) order.
  uint64_t key[KPT];
  uint32_t rank[KPT];
  const uint64_t lanes_below = (1ull << lane) - 1ull;
#pragma unroll
  for (int r = 0; r < KPT; ++r) {
    const int e = w * 64 * KPT + r * 64 + lane;
    const bool valid = e < tile_count;
    key[r] = valid ? in[tile_start + e] : ~0ull;
    const uint32_t d = (uint32_t)(key[r] >> shift) & mask;
    uint64_t same = __ballot(valid);
#pragma unroll
    for (int b = 0; b < kRadixBits; ++b) {
      const bool bit = (d >> b) & 1u;
      const uint64_t bal = __ballot(bit);
      same &= bit ? bal : ~bal;
    }
    const uint32_t below = __popcll(same & lanes_below);
    const uint32_t cnt = __popcll(same);
    uint32_t prev = 0;
    if (valid) prev = wave_cnt[w][d];
    if (valid && below == 0) wave_cnt[w][d] = prev + cnt;
    rank[r] = prev + below;
  }
  __syncthreads();

  // Thread d: per-wave exclusive prefix of digit d, and the tile's exclusive scan over digits.
  uint32_t total = 0;
#pragma unroll
  for (int i = 0; i < WAVES; ++i) {
    uint32_t c = wave_cnt[i][tid];
    wave_cnt[i][tid] = total;
    total += c;
  }
  digit_start[tid] = block_exclusive_scan<kSortThreads>(total, wave_totals, nullptr);
  __syncthreads();

#pragma unroll
  for (int r = 0; r < KPT; ++r) {
    const int e = w * 64 * KPT + r * 64 + lane;
    if (e < tile_count) {
      const uint32_t d = (uint32_t)(key[r] >> shift) & mask;
      stage[digit_start[d] + wave_cnt[w][d] + rank[r]] = key[r];
    }
  }
  __syncthreads();

#pragma unroll
  for (int r = 0; r < KPT; ++r) {
    const int j = r * kSortThreads + tid;
    if (j < tile_count) {
      const uint64_t k = stage[j];
      const uint32_t d = (uint32_t)(k >> shift) & mask;
      out[(int64_t)gbase[d] + (uint32_t)(j - digit_start[d])] = k;
    }
  }
}

// ---- A3: frame boundaries and group bases (only launched when num_frames > 1) -----------------
__global__ __launch_bounds__(256) void k_frames(const uint64_t* __restrict__ sorted, int64_t n, int B, int G,
                                                 int frame_shift /* bit position of the frame field */,
                                                 int32_t* __restrict__ frame_start /*[B+1]*/,
                                                 int32_t* __restrict__ group_base /*[B+1]*/,
                                                 int32_t* __restrict__ group_offsets,
                                                 int32_t* __restrict__ num_groups) {
  __shared__ uint32_t wave_totals[4];
  __shared__ uint32_t carry_s;
  const int tid = threadIdx.x;
  for (int b = tid; b <= B; b += 256) {
    int64_t lo = 0, hi = n;  // first position whose frame field is >= b
    if (b == B) lo = n;
    while (lo < hi) {
      int64_t mid = (lo + hi) >> 1;
      uint32_t f = (uint32_t)(sorted[mid] >> frame_shift);
      if (f < (uint32_t)b) lo = mid + 1; else hi = mid;
    }
    frame_start[b] = (int32_t)lo;
  }
  if (tid == 0) carry_s = 0;
  __syncthreads();
  for (int base = 0; base < B; base += 256) {
    int b = base + tid;
    uint32_t g = 0;
    if (b < B) g = (uint32_t)((frame_start[b + 1] - frame_start[b] + G - 1) / G);
    uint32_t total;
    uint32_t ex = block_exclusive_scan<256>(g, wave_totals, &total);
    uint32_t carry = carry_s;
    if (b < B) group_base[b] = (int32_t)(carry + ex);
    __syncthreads();
    if (tid == 0) carry_s = carry + total;
    __syncthreads();
  }
  if (tid == 0) {
    group_base[B] = (int32_t)carry_s;
    *num_groups = (int32_t)carry_s;
    group_offsets[carry_s] = (int32_t)n;
  }
}

// ---- outputs: perm, exported keys, group offsets ----------------------------------------------
__global__ __launch_bounds__(256) void k_finalize(const uint64_t* __restrict__ sorted, int64_t n, KeyParams kp, int G,
                                                   const int32_t* __restrict__ frame_start,
                                                   const int32_t* __restrict__ group_base,
                                                   int32_t* __restrict__ perm, uint64_t* __restrict__ keys_sorted,
                                                   int32_t* __restrict__ group_offsets,
                                                   int32_t* __restrict__ num_groups) {
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (kp.B == 1 && p == 0) {
    const int32_t ng = (int32_t)((n + G - 1) / G);
    *num_groups = ng;
    group_offsets[ng] = (int32_t)n;
  }
  if (p >= n) return;
  const uint64_t word = sorted[p];
  const uint64_t idx_mask = kp.idx_bits >= 64 ? ~0ull : ((1ull << kp.idx_bits) - 1ull);
  perm[p] = (int32_t)(word & idx_mask);
  uint64_t k = kp.idx_bits >= 64 ? 0ull : (word >> kp.idx_bits);
  const uint64_t l2 = k & field_mask(kp.bits_l2); k >>= kp.bits_l2;
  const uint64_t l1 = k & field_mask(kp.bits_l1); k >>= kp.bits_l1;
  const uint64_t w2 = k & field_mask(kp.bits_w2); k >>= kp.bits_w2;
  const uint64_t w1 = k & field_mask(kp.bits_w1); k >>= kp.bits_w1;
  const uint64_t b = k & field_mask(kp.bits_b);
  if (keys_sorted) keys_sorted[p] = (b << 48) | (w1 << 32) | (w2 << 16) | (l1 << 8) | l2;
  int32_t fs = 0, gb = 0;
  if (kp.B > 1) {
    const int fb = b < (uint64_t)kp.B ? (int)b : kp.B - 1;
    fs = frame_start[fb];
    gb = group_base[fb];
  }
  const int32_t rel = (int32_t)p - fs;
  if (rel % G == 0) group_offsets[gb + rel / G] = (int32_t)p;
}

}  // namespace

int make_flatten_plan(int64_t n, const ff_geom* g, int axis, int shift, FlattenPlan* plan) {
  if (!g || n < 0 || n > 0x7fffffffLL) return FF_ERR_ARG;
  if (g->num_frames < 1 || g->grid_x < 1 || g->grid_y < 1) return FF_ERR_ARG;
  if (g->win_x < 1 || g->win_x > 256 || g->win_y < 1 || g->win_y > 256) return FF_ERR_ARG;
  if (axis != 0 && axis != 1) return FF_ERR_ARG;
  if (g->num_frames > 65535) return FF_ERR_UNSUPPORTED;
  const int64_t sx = shift ? g->win_x / 2 : 0, sy = shift ? g->win_y / 2 : 0;
  const int64_t nwx = ceil_div((int64_t)g->grid_x + sx, g->win_x);
  const int64_t nwy = ceil_div((int64_t)g->grid_y + sy, g->win_y);
  if (nwx > 65535 || nwy > 65535) return FF_ERR_UNSUPPORTED;
  const int bwx = bit_width_u64((uint64_t)nwx - 1), bwy = bit_width_u64((uint64_t)nwy - 1);
  const int blx = bit_width_u64((uint64_t)g->win_x - 1), bly = bit_width_u64((uint64_t)g->win_y - 1);
  plan->bits_b = bit_width_u64((uint64_t)g->num_frames - 1);
  plan->bits_w1 = axis == 0 ? bwx : bwy;
  plan->bits_w2 = axis == 0 ? bwy : bwx;
  plan->bits_l1 = axis == 0 ? blx : bly;
  plan->bits_l2 = axis == 0 ? bly : blx;
  plan->key_bits = plan->bits_b + plan->bits_w1 + plan->bits_w2 + plan->bits_l1 + plan->bits_l2;
  plan->idx_bits = n > 0 ? bit_width_u64((uint64_t)n - 1) : 0;
  if (plan->key_bits + plan->idx_bits > 64) return FF_ERR_UNSUPPORTED;
  plan->passes = (plan->key_bits + kRadixBits - 1) / kRadixBits;
  plan->tiles = ceil_div(n, kTile);
  size_t off = 0;
  plan->off_buf0 = off; off += align_up((size_t)n * 8, 256);
  plan->off_buf1 = off; off += align_up((size_t)n * 8, 256);
  plan->off_hist = off; off += align_up((size_t)kBins * (size_t)(plan->tiles > 0 ? plan->tiles : 1) * 4, 256);
  plan->off_frames = off; off += align_up(((size_t)g->num_frames + 1) * 2 * 4, 256);
  plan->total = off;
  return FF_OK;
}

size_t flatten_workspace_bytes(int64_t n, const ff_geom* g) {
  // Independent of axis and shift: the shifted plan is never smaller.
  FlattenPlan p;
  if (make_flatten_plan(n, g, 0, 1, &p) != FF_OK) return 0;
  return p.total;
}

int flatten_launch(const int32_t* coords, int64_t n, const ff_geom* g, int axis, int shift, int G,
                   int32_t* perm, int32_t* group_offsets, int32_t* num_groups, uint64_t* keys_sorted,
                   void* workspace, size_t workspace_bytes, hipStream_t stream) {
  FlattenPlan plan;
  int st = make_flatten_plan(n, g, axis, shift, &plan);
  if (st != FF_OK) return st;
  if (G < 1 || !group_offsets || !num_groups) return FF_ERR_ARG;
  if (n > 0 && (!coords || !perm)) return FF_ERR_ARG;
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < plan.total) return FF_ERR_WORKSPACE;

  char* ws = (char*)workspace;
  uint64_t* buf[2] = {(uint64_t*)(ws + plan.off_buf0), (uint64_t*)(ws + plan.off_buf1)};
  uint32_t* hist = (uint32_t*)(ws + plan.off_hist);
  int32_t* frame_start = (int32_t*)(ws + plan.off_frames);
  int32_t* group_base = frame_start + (g->num_frames + 1);

  KeyParams kp;
  kp.B = g->num_frames; kp.grid_x = g->grid_x; kp.grid_y = g->grid_y;
  kp.win_x = g->win_x; kp.win_y = g->win_y;
  kp.sx = shift ? g->win_x / 2 : 0; kp.sy = shift ? g->win_y / 2 : 0;
  kp.axis = axis;
  kp.bits_b = plan.bits_b; kp.bits_w1 = plan.bits_w1; kp.bits_w2 = plan.bits_w2;
  kp.bits_l1 = plan.bits_l1; kp.bits_l2 = plan.bits_l2;
  kp.key_bits = plan.key_bits; kp.idx_bits = plan.idx_bits;

  const unsigned eblocks = (unsigned)(n > 0 ? ceil_div(n, 256) : 1);
  int cur = 0;
  if (n > 0) {
    hipLaunchKernelGGL(k_keygen, dim3(eblocks), dim3(256), 0, stream, coords, n, kp, buf[0]);
    for (int pass = 0; pass < plan.passes; ++pass) {
      const int lo = pass * kRadixBits;
      const int nb = plan.key_bits - lo < kRadixBits ? plan.key_bits - lo : kRadixBits;
      const int sh = plan.idx_bits + lo;
      const uint32_t mask = (1u << nb) - 1u;
      hipLaunchKernelGGL(k_radix_hist, dim3((unsigned)plan.tiles), dim3(kSortThreads), 0, stream,
                         buf[cur], n, sh, mask, plan.tiles, hist);
      hipLaunchKernelGGL(k_scan_table, dim3(1), dim3(1024), 0, stream, hist, (int64_t)kBins * plan.tiles);
      hipLaunchKernelGGL(k_radix_scatter, dim3((unsigned)plan.tiles), dim3(kSortThreads), 0, stream,
                         buf[cur], buf[cur ^ 1], n, sh, mask, plan.tiles, hist);
      cur ^= 1;
    }
  }
  if (g->num_frames > 1) {
    hipLaunchKernelGGL(k_frames, dim3(1), dim3(256), 0, stream, buf[cur], n, g->num_frames, G,
                       plan.idx_bits + plan.key_bits - plan.bits_b, frame_start, group_base,
                       group_offsets, num_groups);
  }
  hipLaunchKernelGGL(k_finalize, dim3(eblocks), dim3(256), 0, stream, buf[cur], n, kp, G,
                     frame_start, group_base, perm, keys_sorted, group_offsets, num_groups);
  return launch_status();
}

}  // namespace ff
