// Window-based sorting and equal-size grouping (paper Sec. 4.2.1, Eq. (1); Sec. 4.2.2 'Window
// Shift'; Sec. 4.3 'Reuse Sorting' is the caller keeping the result).
//
// Each pillar becomes ONE 64-bit word  (compact_key << idx_bits) | original_index, where the
// compact key packs the tuple fields (b, W_major, W_minor, L_major, L_minor) using only as many
// bits as the geometry needs.  An LSD radix sort over the compact-key bits is stable, so equal
// tuples keep ascending original index.  The word carries the index, so a pass moves 8 bytes per
// pillar each way.
//
// S sort configurations of the same cloud are sorted together, one grid row each.  Workgroups on
// different XCDs of this chip talk through memory (two microseconds and more per flag round trip),
// so no kernel waits for another workgroup: everything a pass needs is in memory when it starts.
//   * A table counts[pass][tile][digit] says how many words with that digit of that pass the tile
//     holds in the order the pass reads them.  Key generation writes the rows of the first pass
//     (plain stores) and zeroes the others; each pass adds, for every word it places, one to the
//     row of the tile the word lands in for the next pass.  Nothing has to be cleared beforehand.
//   * Small clouds (at most 128 tiles of 1024 words: launch and latency bound): digits of up to 10
//     bits, and a pass reads the whole table of its pass itself (column sums = global digit
//     starts, rows of earlier tiles = its own offsets): key generation + one launch per pass.
//   * Larger clouds (bandwidth bound): per-word atomics would dominate, so passes after the first
//     count their tiles in a kernel of their own, and a small scan kernel turns the table of a pass
//     into exclusive prefixes over the tiles plus per-digit totals.  Tiles of 1024, 2048 or 4096
//     words by cloud size, so that clouds of a few hundred thousand words still fill the chip.
//   * A tile ranks its words with per-wavefront ballot matching and LDS counters and scatters
//     through an LDS stage so that global writes come out in runs.
//   * The last pass writes perm, exported keys and group offsets itself when its digit contains
//     the whole frame field; otherwise two small output kernels run.
#include "common.h"
#include "pack_weights.h"

namespace ff {

namespace {

constexpr int kMaxSorts = 4;
constexpr int kSmallKpt = 4, kSmallMaxTiles = 128;  // small clouds: tiles of 1024 words
constexpr int kLargeKpt = 16;                       // larger clouds: tiles of 4096 words
// In between, the tables are scanned by their own kernel as for larger clouds, but tiles of 4096 words
// would leave most compute units without a workgroup.  Tiles of 1024 words up to 256 K words, of 2048
// words up to 1.5 M (measured: 140 K words 63 -> 52 us, 400 K 68 -> 58, 1 M 73 -> 67, 1.5 M 80 -> 75;
// from 2 M words on the large tiles are ahead).
constexpr int kMidKptA = 4, kMidMaxTilesA = 256;
constexpr int kMidKptB = 8, kMidMaxTilesB = 768;
constexpr int kScanThreads = 1024;
constexpr int kScanStrip = 64;  // digits per workgroup of the column scan (narrower strips were no faster)
// Above 1024 tiles (4 M words) a thread of the 64-digit strip would own more rows than it keeps in
// registers; strips of 16 digits give four times the workgroups and keep every thread within 64 rows
// up to 4096 tiles.
constexpr int kScanNarrow = 16;
constexpr int kScanWideTiles = 1024;

struct KeyParams {
  int32_t B, win_x, win_y, win_z;       // win_z = 1 and stride = 3 for bird's-eye-view pillars
  int32_t sx, sy, sz;                   // shift added to x / y / z
  int32_t axis, stride;                 // stride: int32 per row of coords (3: b,x,y; 4: b,x,y,z)
  int32_t bits_b, bits_w1, bits_w2, bits_w3, bits_l1, bits_l2, bits_l3;  // w3 / l3: the z fields (0 bits in 2-D)
  int32_t key_bits, idx_bits;
};

struct Batch {
  KeyParams kp[kMaxSorts];
  int32_t* perm[kMaxSorts];
  int32_t* inv_perm[kMaxSorts];  // nullptr, or sorted position of every pillar (inverse of perm)
  int32_t* group_offsets[kMaxSorts];
  int32_t* num_groups[kMaxSorts];
  uint64_t* keys_sorted[kMaxSorts];
};

// Groups a frame of `count` pillars is cut into: ceil(count / G), or floor when short groups are dropped.
// (count + G - 1 would overflow for a G near the top of the int range.)
__device__ __forceinline__ uint32_t groups_of(uint32_t count, int G, int drop) {
  const uint32_t full = count / (uint32_t)G;
  return drop || full * (uint32_t)G == count ? full : full + 1u;
}

__device__ __forceinline__ uint32_t field_mask(int bits) { return bits >= 32 ? 0xffffffffu : ((1u << bits) - 1u); }

// ---- block-wide exclusive scan of one uint32 per thread ---------------------------------------
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

__device__ __forceinline__ uint32_t digit_rb(uint64_t word, int idx_bits, int key_bits, int pass, int rb) {
  const int lo = pass * rb;
  const int nb = key_bits - lo < rb ? key_bits - lo : rb;
  if (nb <= 0) return 0u;
  return (uint32_t)(word >> (idx_bits + lo)) & ((1u << nb) - 1u);
}

// Cell of point i (see PointCells).  Comparisons with NaN fail, so such a point is dropped.
__device__ __forceinline__ void point_cell(const PointCells& pt, int64_t i, int32_t* c) {
  const float cx = floorf((pt.xy[2 * i] - pt.x_min) / pt.voxel_x), cy = floorf((pt.xy[2 * i + 1] - pt.y_min) / pt.voxel_y);
  const int b = pt.frame ? pt.frame[i] : 0;
  const bool keep = cx >= 0.f && cx < (float)pt.grid_x && cy >= 0.f && cy < (float)pt.grid_y && b >= 0 && b < pt.B;
  c[0] = keep ? b : pt.B;
  c[1] = keep ? (int)cx : 0;
  c[2] = keep ? (int)cy : 0;
  c[3] = 0;
}

__device__ __forceinline__ uint64_t make_word_at(const int32_t* __restrict__ c, int64_t i, const KeyParams& kp);
__device__ __forceinline__ uint64_t make_word(const int32_t* __restrict__ coords, int64_t i, const KeyParams& kp) {
  return make_word_at(coords + (int64_t)kp.stride * i, i, kp);
}
__device__ __forceinline__ uint64_t make_word_at(const int32_t* __restrict__ c, int64_t i, const KeyParams& kp) {
  const uint32_t b = (uint32_t)c[0];
  const uint32_t X = (uint32_t)(c[1] + kp.sx);
  const uint32_t Y = (uint32_t)(c[2] + kp.sy);
  const uint32_t Wx = X / (uint32_t)kp.win_x, Lx = X - Wx * (uint32_t)kp.win_x;
  const uint32_t Wy = Y / (uint32_t)kp.win_y, Ly = Y - Wy * (uint32_t)kp.win_y;
  uint32_t Wz = 0u, Lz = 0u;
  if (kp.stride > 3) {  // uniform: pillars pay for no third division
    const uint32_t Z = (uint32_t)(c[3] + kp.sz);
    Wz = Z / (uint32_t)kp.win_z;
    Lz = Z - Wz * (uint32_t)kp.win_z;
  }
  const uint32_t w1 = kp.axis == 0 ? Wx : Wy, w2 = kp.axis == 0 ? Wy : Wx;
  const uint32_t l1 = kp.axis == 0 ? Lx : Ly, l2 = kp.axis == 0 ? Ly : Lx;
  // Fields are masked to their widths so that a coordinate outside the geometry can only
  // disturb the order, never another field's bits or any index computed from them.
  uint64_t k = b & field_mask(kp.bits_b);
  k = (k << kp.bits_w1) | (w1 & field_mask(kp.bits_w1));
  k = (k << kp.bits_w2) | (w2 & field_mask(kp.bits_w2));
  k = (k << kp.bits_w3) | (Wz & field_mask(kp.bits_w3));  // 3-D windows: z is the last window and the last local field
  k = (k << kp.bits_l1) | (l1 & field_mask(kp.bits_l1));
  k = (k << kp.bits_l2) | (l2 & field_mask(kp.bits_l2));
  k = (k << kp.bits_l3) | (Lz & field_mask(kp.bits_l3));
  return (k << kp.idx_bits) | (uint64_t)i;
}

__device__ __forceinline__ uint64_t exported_key(uint64_t k, const KeyParams& kp, uint32_t* frame) {
  k >>= kp.bits_l3;  // the exported format has no z fields (it is only produced for 2-D keys)
  const uint64_t l2 = k & field_mask(kp.bits_l2); k >>= kp.bits_l2;
  const uint64_t l1 = k & field_mask(kp.bits_l1); k >>= kp.bits_l1;
  k >>= kp.bits_w3;
  const uint64_t w2 = k & field_mask(kp.bits_w2); k >>= kp.bits_w2;
  const uint64_t w1 = k & field_mask(kp.bits_w1); k >>= kp.bits_w1;
  const uint64_t b = k & field_mask(kp.bits_b);
  *frame = (uint32_t)b;
  return (b << 48) | (w1 << 32) | (w2 << 16) | (l1 << 8) | l2;
}

// ---- A1: coords -> sortable words, plus the digit counts of the first pass ---------------------------
// counts [S][P][tiles][BINS]
// A sort kernel can take workgroups along that do not sort: they re-tile layer weights for the fused
// attention kernels (pack_weights.h), work that does not depend on the sort and would otherwise cost
// a launch of its own in front of the first layer.  Such a launch has a wider grid; the workgroups
// are numbered in dispatch order, the first tiles * sorts of them sort, the rest pack.
__device__ __forceinline__ void pack_tail(const PackJob& pack, int id) {
  int layer = id / pack.blocks;
  const int blk = id - layer * pack.blocks;
  if (layer >= pack.layers) return;
  layer += pack.first;
  if (pack.half) pack_weights_block<true>(pack.pb, layer, blk, pack.C, pack.F, pack.total_frags);
  else pack_weights_block<false>(pack.pb, layer, blk, pack.C, pack.F, pack.total_frags);
}

template <int RB, int KPT>
__global__ __launch_bounds__(kSortThreads) void k_keygen(const int32_t* __restrict__ coords, int64_t n, Batch bt, int P,
                                                          int64_t tiles, uint64_t* __restrict__ words,
                                                          uint32_t* __restrict__ counts, PackJob pack, PointCells pts) {
  constexpr int BINS = 1 << RB, TILE = kSortThreads * KPT;
  static_assert(kSortThreads == 256, "pack_weights_block works in workgroups of 256 threads");
  const int64_t wg = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;  // dispatch order
  if (wg >= tiles * gridDim.y) {  // the same for the whole workgroup
    pack_tail(pack, (int)(wg - tiles * gridDim.y));
    return;
  }
  __shared__ uint32_t h[BINS];
  const int s = (int)(wg / tiles), tid = threadIdx.x;
  const int64_t tile = wg % tiles;
  const KeyParams kp = bt.kp[s];
  for (int t = tid; t < BINS; t += kSortThreads) h[t] = 0u;
  __syncthreads();
#pragma unroll 4
  for (int r = 0; r < KPT; ++r) {
    const int64_t i = tile * TILE + r * kSortThreads + tid;
    if (i < n) {
      uint64_t word;
      if (pts.xy) {  // the same for every thread
        int32_t cell[4];
        point_cell(pts, i, cell);
        word = make_word_at(cell, i, kp);
      } else {
        word = make_word(coords, i, kp);
      }
      words[(int64_t)s * n + i] = word;
      atomicAdd(&h[digit_rb(word, kp.idx_bits, kp.key_bits, 0, RB)], 1u);
    }
  }
  __syncthreads();
  for (int p = 0; p < P; ++p) {
    const size_t base = (((size_t)s * P + p) * tiles + tile) * BINS;
    for (int t = tid; t < BINS; t += kSortThreads) counts[base + t] = p == 0 ? h[t] : 0u;
  }
}

// ---- digit counts of one pass, one table row per tile (larger clouds, passes after the first) ---------
template <int RB, int KPT>
__global__ __launch_bounds__(kSortThreads) void k_tile_counts(const uint64_t* __restrict__ in_all, int64_t n, Batch bt, int pass,
                                                               int P, int64_t tiles, uint32_t* __restrict__ counts) {
  constexpr int BINS = 1 << RB, TILE = kSortThreads * KPT;
  __shared__ uint32_t h[BINS];
  const int s = blockIdx.y, tid = threadIdx.x;
  const int64_t tile = blockIdx.x;
  const int idx_bits = bt.kp[s].idx_bits, key_bits = bt.kp[s].key_bits;
  const uint64_t* in = in_all + (int64_t)s * n;
  for (int t = tid; t < BINS; t += kSortThreads) h[t] = 0u;
  __syncthreads();
  uint64_t key[KPT];
#pragma unroll
  for (int r = 0; r < KPT; ++r) {
    const int64_t i = tile * TILE + r * kSortThreads + tid;
    key[r] = i < n ? in[i] : ~0ull;
  }
#pragma unroll
  for (int r = 0; r < KPT; ++r) {
    const int64_t i = tile * TILE + r * kSortThreads + tid;
    if (i < n) atomicAdd(&h[digit_rb(key[r], idx_bits, key_bits, pass, RB)], 1u);
  }
  __syncthreads();
  const size_t base = (((size_t)s * P + pass) * tiles + tile) * BINS;
  for (int t = tid; t < BINS; t += kSortThreads) counts[base + t] = h[t];
}

// ---- exclusive prefixes of a pass's table over the tiles, and the per-digit totals ------------------
// One workgroup per W digits (a strip of the table, W * 4 bytes of every row).  The rows are cut into
// 1024 / W runs, W lanes take one run.  Up to 64 rows per run are loaded at once and stay in registers
// between the two sweeps.
template <int RB, int W>
__global__ __launch_bounds__(kScanThreads) void k_scan_cols(uint32_t* __restrict__ counts, uint32_t* __restrict__ totals,
                                                             int pass, int P, int64_t tiles) {
  constexpr int BINS = 1 << RB, RUNS = kScanThreads / W, ROWS = 64;
  __shared__ uint32_t part[RUNS][W];
  const int s = blockIdx.y, dl = threadIdx.x % W, c = threadIdx.x / W;
  const int d = blockIdx.x * W + dl;
  uint32_t* tab = counts + ((size_t)s * P + pass) * tiles * BINS + d;
  const int64_t per = (tiles + RUNS - 1) / RUNS;
  const int64_t r0 = c * per, r1 = r0 + per < tiles ? r0 + per : tiles;
  const bool fits = per <= ROWS;  // the same for every thread
  uint32_t v[ROWS];
  uint32_t sum = 0;
  if (fits) {
#pragma unroll
    for (int u = 0; u < ROWS; ++u) v[u] = r0 + u < r1 ? tab[(size_t)(r0 + u) * BINS] : 0u;
#pragma unroll
    for (int u = 0; u < ROWS; ++u) sum += v[u];
  } else {
    for (int64_t r = r0; r < r1; r += 8) {
      uint32_t t[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) t[u] = r + u < r1 ? tab[(size_t)(r + u) * BINS] : 0u;
#pragma unroll
      for (int u = 0; u < 8; ++u) sum += t[u];
    }
  }
  part[c][dl] = sum;
  __syncthreads();
  uint32_t run = 0, total = 0;
#pragma unroll 8
  for (int i = 0; i < RUNS; ++i) {
    const uint32_t t = part[i][dl];
    if (i < c) run += t;
    total += t;
  }
  if (c == 0) totals[((size_t)s * P + pass) * BINS + d] = total;
  if (fits) {
#pragma unroll
    for (int u = 0; u < ROWS; ++u) {
      if (r0 + u < r1) tab[(size_t)(r0 + u) * BINS] = run;
      run += v[u];
    }
  } else {
    for (int64_t r = r0; r < r1; r += 8) {
      uint32_t t[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) t[u] = r + u < r1 ? tab[(size_t)(r + u) * BINS] : 0u;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (r + u < r1) tab[(size_t)(r + u) * BINS] = run;
        run += t[u];
      }
    }
  }
}

// ---- A2: one radix pass ----------------------------------------------------------------------------
// SCANNED: the table row of this tile already holds the counts of earlier tiles and `totals` the
// per-digit totals (k_scan_cols ran); otherwise the workgroup adds the table up itself.
template <int RB, int KPT, bool FUSE, bool SCANNED>
__global__ __launch_bounds__(kSortThreads) void k_pass(const uint64_t* __restrict__ in_all, uint64_t* __restrict__ out_all,
                                                        int64_t n, Batch bt, int pass, int P, int64_t tiles, int G,
                                                        int drop, uint32_t* __restrict__ counts,
                                                        const uint32_t* __restrict__ totals, PackJob pack) {
  constexpr int BINS = 1 << RB, BPT = BINS / kSortThreads, WAVES = kSortThreads / 64, TILE = kSortThreads * KPT;
  static_assert(BPT == 1 || BPT == 2 || BPT == 4, "digits of 8, 9 or 10 bits");
  // LDS is what limits the workgroups per compute unit (4 with 9-bit digits and 4096 words: 40 KB), so
  // the two arrays are reused: wave_cnt holds the per-wavefront digit counters until the words are
  // staged, then the output tables (row 0: gbase, output position of a word = gbase[digit] + its stage
  // slot; row 1: gdig, first output position of a digit over the whole array; rows 2 and 3: the frame
  // table of the last pass).  stage holds the per-wavefront match tables (one 64-bit lane mask per
  // digit), then the scratch of the block scans, then the words in output order.
  __shared__ uint32_t wave_cnt[WAVES][BINS];
  __shared__ uint64_t stage[TILE > WAVES * BINS ? TILE : WAVES * BINS];
  static_assert(WAVES >= 4, "rows of wave_cnt are reused for four tables");
  uint32_t* wave_totals = reinterpret_cast<uint32_t*>(stage);
  uint32_t* gbase = &wave_cnt[0][0];
  uint32_t* gdig = &wave_cnt[1][0];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int64_t wg = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;  // dispatch order
  if (wg >= tiles * gridDim.y) {  // the same for the whole workgroup
    pack_tail(pack, (int)(wg - tiles * gridDim.y));
    return;
  }
  const int s = (int)(wg / tiles);
  const int64_t tile = wg % tiles;
  const KeyParams kp = bt.kp[s];
  const int idx_bits = kp.idx_bits, key_bits = kp.key_bits;
  const uint64_t* in = in_all + (int64_t)s * n;
  uint64_t* out = out_all + (int64_t)s * n;
  const uint32_t* cnt_tab = counts + ((size_t)s * P + pass) * tiles * BINS;
  uint32_t* next_tab = counts + ((size_t)s * P + pass + 1) * tiles * BINS;
  const int64_t tile_start = tile * TILE;
  const int tile_count = (int)((n - tile_start) < (int64_t)TILE ? (n - tile_start) : (int64_t)TILE);
  // Element order inside the tile: wave-major, then round, then lane.  Each wave owns a contiguous
  // run of 64 * KPT words, so stability only needs (wave, round, lane) order.
  uint64_t key[KPT];
  uint32_t rank[KPT];
  const uint64_t lanes_below = (1ull << lane) - 1ull;
#pragma unroll
  for (int r = 0; r < KPT; ++r) {
    const int e = w * 64 * KPT + r * 64 + lane;
    key[r] = e < tile_count ? in[tile_start + e] : ~0ull;
  }

  // Thread t owns digits t * BPT ..: their counts over the whole array and over earlier tiles.
  uint32_t gtot[BPT], before[BPT];
  if (SCANNED) {
#pragma unroll
    for (int k = 0; k < BPT; ++k) {
      gtot[k] = totals[((size_t)s * P + pass) * BINS + tid * BPT + k];
      before[k] = cnt_tab[(size_t)tile * BINS + tid * BPT + k];
    }
  } else {  // column sums, 32 rows per memory round trip
#pragma unroll
    for (int k = 0; k < BPT; ++k) { gtot[k] = 0; before[k] = 0; }
    for (int t0 = 0; t0 < tiles; t0 += 32) {
      uint32_t v[32][BPT];
#pragma unroll
      for (int u = 0; u < 32; ++u) {
        const int64_t t = t0 + u < tiles ? t0 + u : tiles - 1;
        if (BPT == 4) {
          const uint4 q = *reinterpret_cast<const uint4*>(cnt_tab + (size_t)t * BINS + tid * 4);
          v[u][0] = q.x; v[u][1 % BPT] = q.y; v[u][2 % BPT] = q.z; v[u][3 % BPT] = q.w;
        } else if (BPT == 2) {
          const uint2 q = *reinterpret_cast<const uint2*>(cnt_tab + (size_t)t * BINS + tid * 2);
          v[u][0] = q.x; v[u][1 % BPT] = q.y;
        } else {
          v[u][0] = cnt_tab[(size_t)t * BINS + tid];
        }
      }
#pragma unroll
      for (int u = 0; u < 32; ++u)
#pragma unroll
        for (int k = 0; k < BPT; ++k) {
          if (t0 + u < tiles) gtot[k] += v[u][k];
          if (t0 + u < tile) before[k] += v[u][k];
        }
    }
  }
#pragma unroll
  for (int i = 0; i < WAVES; ++i)
#pragma unroll
    for (int k = 0; k < BPT; ++k) { wave_cnt[i][tid + k * kSortThreads] = 0; stage[i * BINS + tid + k * kSortThreads] = 0ull; }
  __syncthreads();
  // Rank inside the wavefront's run: lanes with the same digit find each other through the match
  // table (every lane ORs its bit into the digit's entry; LDS instructions of a wavefront execute in
  // order, so the read that follows sees all of them), the first of them adds the count to the
  // wavefront's running digit counter and clears the entry for the next round.
  unsigned long long* match = reinterpret_cast<unsigned long long*>(stage) + w * BINS;
#pragma unroll
  for (int r = 0; r < KPT; ++r) {
    const int e = w * 64 * KPT + r * 64 + lane;
    const bool valid = e < tile_count;
    const uint32_t d = digit_rb(key[r], idx_bits, key_bits, pass, RB);
    unsigned long long same = 0ull;
    uint32_t prev = 0;
    if (valid) atomicOr(&match[d], 1ull << lane);
    if (valid) { same = match[d]; prev = wave_cnt[w][d]; }
    const uint32_t below = __popcll(same & lanes_below);
    const uint32_t cnt = __popcll(same);
    if (valid && below == 0) { wave_cnt[w][d] = prev + cnt; match[d] = 0ull; }
    rank[r] = prev + below;
  }
  __syncthreads();

  uint32_t total[BPT];
  uint32_t tsum = 0, gsum = 0;
#pragma unroll
  for (int k = 0; k < BPT; ++k) {
    const int d = tid * BPT + k;
    uint32_t run = 0;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) {
      const uint32_t c = wave_cnt[i][d];
      wave_cnt[i][d] = run;  // exclusive prefix over the tile's waves
      run += c;
    }
    total[k] = run;
    tsum += run;
    gsum += gtot[k];
  }
  const uint32_t gex = block_exclusive_scan<kSortThreads>(gsum, wave_totals, nullptr);
  const uint32_t tex = block_exclusive_scan<kSortThreads>(tsum, wave_totals, nullptr);
  uint32_t gb[BPT], gd[BPT];
  {
    uint32_t grun = gex, trun = tex;
#pragma unroll
    for (int k = 0; k < BPT; ++k) {
      const int d = tid * BPT + k;
      gb[k] = grun + before[k] - trun;
      gd[k] = grun;
#pragma unroll
      for (int i = 0; i < WAVES; ++i) wave_cnt[i][d] += trun;  // first stage slot of (wave, digit)
      trun += total[k];
      grun += gtot[k];
    }
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < KPT; ++r) {
    const int e = w * 64 * KPT + r * 64 + lane;
    if (e < tile_count) {
      const uint32_t d = digit_rb(key[r], idx_bits, key_bits, pass, RB);
      stage[wave_cnt[w][d] + rank[r]] = key[r];
    }
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < BPT; ++k) {
    gbase[tid * BPT + k] = gb[k];
    if (FUSE) gdig[tid * BPT + k] = gd[k];
  }
  __syncthreads();

  if (!FUSE) {
#pragma unroll
    for (int r = 0; r < KPT; ++r) {
      const int j = r * kSortThreads + tid;
      uint32_t slot = 0xffffffffu;  // table entry of the next pass this word counts for (none: no word here)
      if (j < tile_count) {
        const uint64_t k = stage[j];
        const uint32_t d = digit_rb(k, idx_bits, key_bits, pass, RB);
        const int64_t pos = (int64_t)(gbase[d] + (uint32_t)j);
        if (pos < n) {
          out[pos] = k;
          if (!SCANNED && pass + 1 < P)  // small clouds: the next pass finds this word in tile pos / TILE
            slot = (uint32_t)(pos / TILE) * BINS + digit_rb(k, idx_bits, key_bits, pass + 1, RB);
        }
      }
      if (!SCANNED && pass + 1 < P) {
        // One atomic per run of neighbouring lanes that count the same table entry.  Words next to each other in
        // the stage share this pass's digit and land side by side; when the cloud arrives in an order that
        // follows the grid (a voxeliser's row-major output) they mostly share the next digit as well, and
        // one atomic per word then queues up on a few addresses.
        const uint32_t prev = __shfl_up(slot, 1, 64);
        const bool head = lane == 0 || prev != slot;
        const uint64_t heads = __ballot(head);
        if (head && slot != 0xffffffffu) {
          const uint64_t later = lane == 63 ? 0ull : (heads >> (lane + 1));
          const uint32_t run = later ? (uint32_t)__builtin_ctzll(later) + 1u : 64u - (uint32_t)lane;
          atomicAdd(&next_tab[slot], run);
        }
      }
    }
    return;
  }

  // ---- last pass: the output position is final -------------------------------------------------------
  int32_t* __restrict__ const perm_s = bt.perm[s];  // read once: the stores below must not wait for them
  int32_t* __restrict__ const inv_s = bt.inv_perm[s];
  uint64_t* __restrict__ const keys_s = bt.keys_sorted[s];
  int32_t* __restrict__ const goff_s = bt.group_offsets[s];
  const uint32_t idx_mask = idx_bits >= 32 ? ~0u : (1u << idx_bits) - 1u;  // n < 2^31
  uint32_t pos_r[KPT], idx_r[KPT];
#pragma unroll
  for (int r = 0; r < KPT; ++r) {
    const int j = r * kSortThreads + tid;
    const uint64_t word = stage[j < tile_count ? j : 0];
    const uint32_t d = digit_rb(word, idx_bits, key_bits, pass, RB);
    pos_r[r] = j < tile_count ? gbase[d] + (uint32_t)j : 0xffffffffu;
    idx_r[r] = (uint32_t)word & idx_mask;
  }
#pragma unroll
  for (int r = 0; r < KPT; ++r)
    if ((int64_t)pos_r[r] < n) perm_s[pos_r[r]] = (int32_t)idx_r[r];
  if (inv_s) {  // the same for the whole workgroup
#pragma unroll
    for (int r = 0; r < KPT; ++r)
      if ((int64_t)pos_r[r] < n) inv_s[idx_r[r]] = (int32_t)pos_r[r];
  }
  if (keys_s) {  // the same for the whole workgroup
#pragma unroll
    for (int r = 0; r < KPT; ++r) {
      if ((int64_t)pos_r[r] < n) {
        uint32_t b;
        keys_s[pos_r[r]] = exported_key(stage[r * kSortThreads + tid] >> idx_bits, kp, &b);
      }
    }
  }
  // Frame b starts where the first last-pass digit of frame b starts; group bases are the running
  // sum of the frames' group counts, ceil(frame size / G), or floor when short groups are dropped.
  // The group list follows from that table alone: every workgroup builds the table and writes its
  // share of the list.
  __syncthreads();  // the stage has been read: its memory serves the block scan again
  uint32_t* fstart = &wave_cnt[2][0];
  uint32_t* fgroup = &wave_cnt[3][0];
  const int B = kp.B;
  const int nb_last = key_bits - pass * RB;       // bits of this digit (>= bits_b, checked by the host)
  const int fshift = nb_last - kp.bits_b;
  uint32_t gcount[BPT], fs[BPT], gs = 0;
#pragma unroll
  for (int k = 0; k < BPT; ++k) {
    const int b = tid * BPT + k;
    uint32_t c = 0, lo = 0;
    if (b < B) {
      lo = gdig[(uint32_t)b << fshift];
      const uint32_t hi = b + 1 < B ? gdig[(uint32_t)(b + 1) << fshift] : (uint32_t)n;
      c = groups_of(hi - lo, G, drop);
    }
    gcount[k] = c;
    fs[k] = lo;
    gs += c;
  }
  uint32_t ng_total = 0;
  uint32_t gexcl = block_exclusive_scan<kSortThreads>(gs, wave_totals, &ng_total);
#pragma unroll
  for (int k = 0; k < BPT; ++k) {
    const int b = tid * BPT + k;
    if (b < B) { fstart[b] = fs[k]; fgroup[b] = gexcl; }
    gexcl += gcount[k];
  }
  __syncthreads();
  for (int64_t gi = tile * kSortThreads + tid; gi < (int64_t)ng_total; gi += tiles * kSortThreads) {
    int lo = 0, hi = B;  // the last frame whose group base is at or below gi (empty frames share a base)
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (fgroup[mid] <= (uint32_t)gi) lo = mid; else hi = mid;
    }
    goff_s[gi] = (int32_t)(fstart[lo] + ((uint32_t)gi - fgroup[lo]) * (uint32_t)G);
  }
  if (tile == 0 && tid == 0) {
    *bt.num_groups[s] = (int32_t)ng_total;
    goff_s[ng_total] = (int32_t)n;
  }
}

// ---- A3: frame boundaries and group bases for many frames (num_frames > 256) ---------------------
__global__ __launch_bounds__(256) void k_frames(const uint64_t* __restrict__ sorted_all, int64_t n, Batch bt, int G,
                                                 int drop, int32_t* __restrict__ frame_tab /*[S][2][B+1]*/) {
  __shared__ uint32_t wave_totals[4];
  __shared__ uint32_t carry_s;
  const int s = blockIdx.x;
  const KeyParams kp = bt.kp[s];
  const int B = kp.B;
  const uint64_t* sorted = sorted_all + (int64_t)s * n;
  int32_t* frame_start = frame_tab + (int64_t)s * 2 * (B + 1);
  int32_t* group_base = frame_start + (B + 1);
  const int frame_shift = kp.idx_bits + kp.key_bits - kp.bits_b;
  const int tid = threadIdx.x;
  for (int b = tid; b <= B; b += 256) {
    int64_t lo = 0, hi = n;  // first position whose frame field is >= b
    if (b == B) lo = n;
    while (lo < hi) {
      const int64_t mid = (lo + hi) >> 1;
      const uint32_t f = (uint32_t)(sorted[mid] >> frame_shift);
      if (f < (uint32_t)b) lo = mid + 1; else hi = mid;
    }
    frame_start[b] = (int32_t)lo;
  }
  if (tid == 0) carry_s = 0;
  __syncthreads();
  for (int base = 0; base < B; base += 256) {
    const int b = base + tid;
    uint32_t g = 0;
    if (b < B) g = groups_of((uint32_t)(frame_start[b + 1] - frame_start[b]), G, drop);
    uint32_t total;
    const uint32_t ex = block_exclusive_scan<256>(g, wave_totals, &total);
    const uint32_t carry = carry_s;
    if (b < B) group_base[b] = (int32_t)(carry + ex);
    __syncthreads();
    if (tid == 0) carry_s = carry + total;
    __syncthreads();
  }
  if (tid == 0) group_base[B] = (int32_t)carry_s;
}

// ---- outputs: perm, exported keys, group offsets, num_groups ----------------------------------------
// For a small cloud with at most 256 frames every block recomputes the frame table itself (B binary
// searches and one block scan); otherwise it reads the table k_frames wrote.
__global__ __launch_bounds__(256) void k_finalize(const uint64_t* __restrict__ sorted_all, int64_t n, Batch bt, int G,
                                                   int drop, const int32_t* __restrict__ frame_tab) {
  __shared__ int32_t fstart_s[257], gbase_s[257];
  __shared__ uint32_t wave_totals[4];
  const int s = blockIdx.y;
  const KeyParams kp = bt.kp[s];
  const int B = kp.B, tid = threadIdx.x;
  const uint64_t* sorted = sorted_all + (int64_t)s * n;
  const int frame_shift = kp.idx_bits + kp.key_bits - kp.bits_b;
  const int32_t* fstart = fstart_s;
  const int32_t* gbase = gbase_s;
  if (B == 1) {
    if (tid == 0) { fstart_s[0] = 0; fstart_s[1] = (int32_t)n; gbase_s[0] = 0; gbase_s[1] = (int32_t)groups_of((uint32_t)n, G, drop); }
    __syncthreads();
  } else if (B <= 256 && n <= 65536) {
    if (tid == 0) fstart_s[B] = (int32_t)n;
    if (tid < B) {
      int64_t lo = 0, hi = n;
      while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        const uint32_t f = (uint32_t)(sorted[mid] >> frame_shift);
        if (f < (uint32_t)tid) lo = mid + 1; else hi = mid;
      }
      fstart_s[tid] = (int32_t)lo;
    }
    __syncthreads();
    uint32_t g = 0;
    if (tid < B) g = groups_of((uint32_t)(fstart_s[tid + 1] - fstart_s[tid]), G, drop);
    uint32_t total;
    const uint32_t ex = block_exclusive_scan<256>(g, wave_totals, &total);
    if (tid < B) gbase_s[tid] = (int32_t)ex;
    if (tid == 0) gbase_s[B] = (int32_t)total;
    __syncthreads();
  } else {
    fstart = frame_tab + (int64_t)s * 2 * (B + 1);
    gbase = fstart + (B + 1);
  }
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + tid;
  if (p == 0) {
    const int32_t ng = gbase[B];
    *bt.num_groups[s] = ng;
    bt.group_offsets[s][ng] = (int32_t)n;
  }
  if (p >= n) return;
  const uint64_t word = sorted[p];
  const uint64_t idx_mask = (1ull << kp.idx_bits) - 1ull;
  bt.perm[s][p] = (int32_t)(word & idx_mask);
  if (bt.inv_perm[s]) bt.inv_perm[s][word & idx_mask] = (int32_t)p;
  uint64_t k = word >> kp.idx_bits;
  k >>= kp.bits_l3;
  const uint64_t l2 = k & field_mask(kp.bits_l2); k >>= kp.bits_l2;
  const uint64_t l1 = k & field_mask(kp.bits_l1); k >>= kp.bits_l1;
  k >>= kp.bits_w3;
  const uint64_t w2 = k & field_mask(kp.bits_w2); k >>= kp.bits_w2;
  const uint64_t w1 = k & field_mask(kp.bits_w1); k >>= kp.bits_w1;
  const uint64_t b = k & field_mask(kp.bits_b);
  if (bt.keys_sorted[s]) bt.keys_sorted[s][p] = (b << 48) | (w1 << 32) | (w2 << 16) | (l1 << 8) | l2;
  const int fb = b < (uint64_t)B ? (int)b : B - 1;
  const int32_t rel = (int32_t)p - fstart[fb], gi = rel / G;
  if (rel == gi * G && gi < gbase[fb + 1] - gbase[fb]) bt.group_offsets[s][gbase[fb] + gi] = (int32_t)p;
}

// Pass plan for keys of `key_bits` bits: digit width and number of passes.
struct PassPlan { bool small; int kpt, rb, passes; int64_t tiles; };
inline PassPlan pass_plan(int64_t n, int key_bits) {
  PassPlan pp;
  pp.small = ceil_div(n > 0 ? n : 1, (int64_t)kSortThreads * kSmallKpt) <= kSmallMaxTiles;
  pp.kpt = pp.small ? kSmallKpt
         : ceil_div(n, (int64_t)kSortThreads * kMidKptA) <= kMidMaxTilesA ? kMidKptA
         : ceil_div(n, (int64_t)kSortThreads * kMidKptB) <= kMidMaxTilesB ? kMidKptB : kLargeKpt;
  pp.passes = (key_bits + 9) / 10;
  // the narrowest digit that still needs no extra pass: smaller tables, longer runs per digit
  pp.rb = 8 * pp.passes >= key_bits ? 8 : 9 * pp.passes >= key_bits ? 9 : 10;
  pp.tiles = ceil_div(n > 0 ? n : 1, (int64_t)kSortThreads * pp.kpt);
  return pp;
}

struct Layout {
  size_t off_words0, off_words1, off_counts, off_totals, off_frames, total;
};

// Workspace for S sorts of n words whose keys have at most max_key_bits bits (a call may sort
// narrower keys than the workspace query assumed, and a narrower key can pick a wider digit).
void make_layout(int64_t n, int S, int num_frames, int max_key_bits, Layout* L) {
  size_t count_words = 0, total_words = 0;
  for (int kb = 0; kb <= max_key_bits; ++kb) {
    const PassPlan pp = pass_plan(n, kb);
    const size_t pc = pp.passes > 0 ? pp.passes : 1;  // key generation always fills one table
    const size_t cw = (size_t)S * pc * (size_t)pp.tiles * ((size_t)1 << pp.rb);
    const size_t tw = (size_t)S * pc * ((size_t)1 << pp.rb);
    if (cw > count_words) count_words = cw;
    if (tw > total_words) total_words = tw;
  }
  size_t off = 0;
  L->off_words0 = off; off += align_up((size_t)S * n * 8, 256);
  L->off_words1 = off; off += align_up((size_t)S * n * 8, 256);
  L->off_counts = off; off += align_up(count_words * 4 + 256, 256);
  L->off_totals = off; off += align_up(total_words * 4 + 256, 256);
  L->off_frames = off; off += align_up((size_t)S * 2 * ((size_t)num_frames + 1) * 4, 256);
  L->total = off;
}

}  // namespace

int make_flatten_plan(int64_t n, const ff_geom* g, int axis, int shift, FlattenPlan* plan) {
  return make_flatten_plan_z(n, g, nullptr, axis, shift, plan);
}

int make_flatten_plan_z(int64_t n, const ff_geom* g, const FlattenZ* z, int axis, int shift, FlattenPlan* plan) {
  if (!g || n < 0 || n > 0x7fffffffLL) return FF_ERR_ARG;
  if (z && (z->grid_z < 1 || z->win_z < 1 || z->win_z > 256)) return FF_ERR_ARG;
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
  plan->bits_w3 = plan->bits_l3 = 0;
  if (z) {
    const int64_t nwz = ceil_div((int64_t)z->grid_z + (shift ? z->win_z / 2 : 0), z->win_z);
    if (nwz > 65535) return FF_ERR_UNSUPPORTED;
    plan->bits_w3 = bit_width_u64((uint64_t)nwz - 1);
    plan->bits_l3 = bit_width_u64((uint64_t)z->win_z - 1);
  }
  plan->key_bits = plan->bits_b + plan->bits_w1 + plan->bits_w2 + plan->bits_w3 + plan->bits_l1 + plan->bits_l2 +
                   plan->bits_l3;
  plan->idx_bits = n > 0 ? bit_width_u64((uint64_t)n - 1) : 0;
  if (plan->key_bits + plan->idx_bits > 64) return FF_ERR_UNSUPPORTED;
  plan->passes = (plan->key_bits + kRadixBits - 1) / kRadixBits;
  return FF_OK;
}

size_t flatten_workspace_bytes(int64_t n, const ff_geom* g, int num_sorts) {
  return flatten_workspace_bytes_z(n, g, nullptr, num_sorts);
}

size_t flatten_workspace_bytes_z(int64_t n, const ff_geom* g, const FlattenZ* z, int num_sorts) {
  // Independent of axis and shift: the shifted plan never has fewer key bits.
  FlattenPlan p;
  if (num_sorts < 1 || num_sorts > kMaxSorts) return 0;
  if (make_flatten_plan_z(n, g, z, 0, 1, &p) != FF_OK) return 0;
  Layout L;
  make_layout(n, num_sorts, g->num_frames, p.key_bits, &L);
  return L.total;
}

int flatten_launch(const int32_t* coords, int64_t n, const ff_geom* g, int num_sorts, const int* axis,
                   const int* shift, int G, int drop, int32_t* const* perm, int32_t* const* inv_perm,
                   int32_t* const* group_offsets, int32_t* const* num_groups, uint64_t* const* keys_sorted,
                   void* workspace, size_t workspace_bytes, const PackJob* pack, hipStream_t stream) {
  return flatten_launch_z(coords, n, g, nullptr, num_sorts, axis, shift, G, drop, perm, inv_perm, group_offsets,
                          num_groups, keys_sorted, workspace, workspace_bytes, pack, stream);
}

static int flatten_launch_impl(const int32_t* coords, const PointCells* pts, int64_t n, const ff_geom* g,
                               const FlattenZ* z, int num_sorts, const int* axis, const int* shift, int G, int drop,
                               int32_t* const* perm, int32_t* const* inv_perm, int32_t* const* group_offsets,
                               int32_t* const* num_groups, uint64_t* const* keys_sorted, void* workspace,
                               size_t workspace_bytes, const PackJob* pack, hipStream_t stream);

int flatten_launch_z(const int32_t* coords, int64_t n, const ff_geom* g, const FlattenZ* z, int num_sorts,
                     const int* axis, const int* shift, int G, int drop, int32_t* const* perm,
                     int32_t* const* inv_perm, int32_t* const* group_offsets, int32_t* const* num_groups,
                     uint64_t* const* keys_sorted, void* workspace, size_t workspace_bytes, const PackJob* pack,
                     hipStream_t stream) {
  return flatten_launch_impl(coords, nullptr, n, g, z, num_sorts, axis, shift, G, drop, perm, inv_perm, group_offsets,
                             num_groups, keys_sorted, workspace, workspace_bytes, pack, stream);
}

int flatten_launch_points(const PointCells* pts, int64_t n, const ff_geom* g, int32_t* perm, int32_t* group_offsets,
                          int32_t* num_groups, uint64_t* keys_sorted, void* workspace, size_t workspace_bytes,
                          hipStream_t stream) {
  if (!pts || (n > 0 && !pts->xy)) return FF_ERR_ARG;
  const int axis = 0, shift = 0;
  return flatten_launch_impl(nullptr, pts, n, g, nullptr, 1, &axis, &shift, 0x40000000, 0, &perm, nullptr,
                             &group_offsets, &num_groups, &keys_sorted, workspace, workspace_bytes, nullptr, stream);
}

static int flatten_launch_impl(const int32_t* coords, const PointCells* pts, int64_t n, const ff_geom* g,
                               const FlattenZ* z, int num_sorts, const int* axis, const int* shift, int G, int drop,
                               int32_t* const* perm, int32_t* const* inv_perm, int32_t* const* group_offsets,
                               int32_t* const* num_groups, uint64_t* const* keys_sorted, void* workspace,
                               size_t workspace_bytes, const PackJob* pack, hipStream_t stream) {
  if (num_sorts < 1 || num_sorts > kMaxSorts || G < 1) return FF_ERR_ARG;
  if (z && keys_sorted) return FF_ERR_ARG;  // the exported key format has no room for the z fields
  Batch bt;
  int max_key_bits = 0;
  for (int s = 0; s < num_sorts; ++s) {
    FlattenPlan plan;
    const int st = make_flatten_plan_z(n, g, z, axis[s], shift[s], &plan);
    if (st != FF_OK) return st;
    if (!group_offsets[s] || !num_groups[s] || (n > 0 && !perm[s])) return FF_ERR_ARG;
    KeyParams& kp = bt.kp[s];
    kp.B = g->num_frames; kp.win_x = g->win_x; kp.win_y = g->win_y; kp.win_z = z ? z->win_z : 1;
    kp.sx = shift[s] ? g->win_x / 2 : 0; kp.sy = shift[s] ? g->win_y / 2 : 0;
    kp.sz = z && shift[s] ? z->win_z / 2 : 0;
    kp.axis = axis[s]; kp.stride = z ? 4 : 3;
    kp.bits_b = plan.bits_b; kp.bits_w1 = plan.bits_w1; kp.bits_w2 = plan.bits_w2; kp.bits_w3 = plan.bits_w3;
    kp.bits_l1 = plan.bits_l1; kp.bits_l2 = plan.bits_l2; kp.bits_l3 = plan.bits_l3;
    kp.key_bits = plan.key_bits; kp.idx_bits = plan.idx_bits;
    bt.perm[s] = perm[s]; bt.group_offsets[s] = group_offsets[s]; bt.num_groups[s] = num_groups[s];
    bt.keys_sorted[s] = keys_sorted ? keys_sorted[s] : nullptr;
    bt.inv_perm[s] = inv_perm ? inv_perm[s] : nullptr;
    if (plan.key_bits > max_key_bits) max_key_bits = plan.key_bits;
  }
  for (int s = num_sorts; s < kMaxSorts; ++s) {
    bt.kp[s] = bt.kp[0]; bt.perm[s] = nullptr; bt.group_offsets[s] = nullptr; bt.num_groups[s] = nullptr;
    bt.keys_sorted[s] = nullptr;
    bt.inv_perm[s] = nullptr;
  }
  if (n > 0 && !coords && !pts) return FF_ERR_ARG;
  const PointCells point_src = pts ? *pts : PointCells();  // xy == nullptr: integer coordinates
  Layout L;
  make_layout(n, num_sorts, g->num_frames, max_key_bits, &L);
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < L.total) return FF_ERR_WORKSPACE;

  char* ws = (char*)workspace;
  uint64_t* buf[2] = {(uint64_t*)(ws + L.off_words0), (uint64_t*)(ws + L.off_words1)};
  uint32_t* counts = (uint32_t*)(ws + L.off_counts);
  uint32_t* totals = (uint32_t*)(ws + L.off_totals);
  int32_t* frame_tab = (int32_t*)(ws + L.off_frames);

  int cur = 0;
  bool outputs_done = false;
  if (n > 0) {
    const PassPlan pp = pass_plan(n, max_key_bits);
    const int P = pp.passes > 0 ? pp.passes : 1;  // zero key bits: the words are generated in order
    // The last pass can write the outputs itself when its digit contains the whole frame field.
    bool fuse = pp.passes > 0;
    for (int s = 0; s < num_sorts; ++s)
      fuse = fuse && bt.kp[s].key_bits - (pp.passes - 1) * pp.rb >= bt.kp[s].bits_b;
    const dim3 grid((unsigned)pp.tiles, (unsigned)num_sorts), block(kSortThreads);
    // The first radix pass takes the weight-packing workgroups along (key generation when there is no
    // pass): that launch is bound by the latency of a few sort workgroups and leaves most of the chip idle.
    PackJob no_job = PackJob();
    no_job.layers = 0; no_job.blocks = 1;
    const PackJob job = pack ? *pack : no_job;
    // With radix passes to run, the layers are shared out between key generation and the first pass (both
    // launches are short and leave most compute units idle; one of them alone would be stretched by the packing).
    PackJob job_a = job, job_b = no_job;   // job_a: key generation (everything when there is no pass), job_b: first pass
    if (pp.passes > 0 && job.layers > 0) {
      job_a.layers = job.layers / 2;
      job_b = job;
      job_b.first = job_a.layers;
      job_b.layers = job.layers - job_a.layers;
      if (job_a.layers == 0) job_a = no_job;
    }
    const dim3 grid_a((unsigned)(pp.tiles + ceil_div((int64_t)job_a.layers * job_a.blocks, num_sorts)), (unsigned)num_sorts);
    const dim3 grid_pack((unsigned)(pp.tiles + ceil_div((int64_t)job_b.layers * job_b.blocks, num_sorts)), (unsigned)num_sorts);
#define FF_PASSES(RB, KPT, SCANNED)                                                                                  \
    do {                                                                                                             \
      hipLaunchKernelGGL((k_keygen<RB, KPT>), grid_a, block, 0, stream, coords, n, bt, P, pp.tiles, buf[0], counts,  \
                         job_a, point_src);                                                                          \
      for (int pass = 0; pass < pp.passes; ++pass) {                                                                 \
        if (SCANNED) {                                                                                               \
          if (pass > 0)                                                                                              \
            hipLaunchKernelGGL((k_tile_counts<RB, KPT>), grid, block, 0, stream, buf[cur], n, bt, pass, P, pp.tiles, \
                               counts);                                                                              \
          if (pp.tiles > kScanWideTiles)                                                                             \
            hipLaunchKernelGGL((k_scan_cols<RB, kScanNarrow>), dim3((1u << RB) / kScanNarrow, (unsigned)num_sorts),  \
                               dim3(kScanThreads), 0, stream, counts, totals, pass, P, pp.tiles);                   \
          else                                                                                                       \
            hipLaunchKernelGGL((k_scan_cols<RB, kScanStrip>), dim3((1u << RB) / kScanStrip, (unsigned)num_sorts),    \
                               dim3(kScanThreads), 0, stream, counts, totals, pass, P, pp.tiles);                   \
        }                                                                                                            \
        if (fuse && pass == pp.passes - 1)                                                                           \
          hipLaunchKernelGGL((k_pass<RB, KPT, true, SCANNED>), pass == 0 ? grid_pack : grid, block, 0, stream,      \
                             buf[cur], buf[cur ^ 1], n, bt, pass, P, pp.tiles, G, drop, counts, totals,              \
                             pass == 0 ? job_b : no_job);                                                              \
        else                                                                                                         \
          hipLaunchKernelGGL((k_pass<RB, KPT, false, SCANNED>), pass == 0 ? grid_pack : grid, block, 0, stream,     \
                             buf[cur], buf[cur ^ 1], n, bt, pass, P, pp.tiles, G, drop, counts, totals,              \
                             pass == 0 ? job_b : no_job);                                                              \
        cur ^= 1;                                                                                                    \
      }                                                                                                              \
    } while (0)
    if (!pp.small && pp.kpt == kMidKptA && pp.rb == 8) FF_PASSES(8, kMidKptA, true);
    else if (!pp.small && pp.kpt == kMidKptA && pp.rb == 9) FF_PASSES(9, kMidKptA, true);
    else if (!pp.small && pp.kpt == kMidKptA) FF_PASSES(10, kMidKptA, true);
    else if (pp.kpt == kMidKptB && pp.rb == 8) FF_PASSES(8, kMidKptB, true);
    else if (pp.kpt == kMidKptB && pp.rb == 9) FF_PASSES(9, kMidKptB, true);
    else if (pp.kpt == kMidKptB) FF_PASSES(10, kMidKptB, true);
    else if (!pp.small && pp.rb == 8) FF_PASSES(8, kLargeKpt, true);
    else if (!pp.small && pp.rb == 9) FF_PASSES(9, kLargeKpt, true);
    else if (!pp.small) FF_PASSES(10, kLargeKpt, true);
    else if (pp.rb == 8) FF_PASSES(8, kSmallKpt, false);
    else if (pp.rb == 9) FF_PASSES(9, kSmallKpt, false);
    else FF_PASSES(10, kSmallKpt, false);
#undef FF_PASSES
    outputs_done = fuse;
  }
  if (!outputs_done) {
    if (g->num_frames > 256 || (g->num_frames > 1 && n > 65536))  // else every output block derives it itself
      hipLaunchKernelGGL(k_frames, dim3((unsigned)num_sorts), dim3(256), 0, stream, buf[cur], n, bt, G, drop, frame_tab);
    hipLaunchKernelGGL(k_finalize, dim3((unsigned)(n > 0 ? ceil_div(n, 256) : 1), (unsigned)num_sorts), dim3(256), 0,
                       stream, buf[cur], n, bt, G, drop, frame_tab);
  }
  return launch_status();
}

}  // namespace ff
