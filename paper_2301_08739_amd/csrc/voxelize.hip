// Pillar voxelisation, the step in front of the FWA blocks (paper Sec. 5.1 'Model': the point cloud
// is voxelised into sparse bird's-eye-view pillars of 0.32 m x 0.32 m).  Here in its plain form: a
// pillar is a non-empty cell, its feature vector the mean of its points' feature vectors, pillars
// come out in ascending (frame, x, y) order; the learned per-point network of PointPillars is not
// part of it.  HBM/latency bound integer work that reuses the window sort:
//   flatten         the radix argsort of flatten.hip with 1 x 1 windows, its key generation fed by the points:
//                   cell of every point (float32: floor((x - x_min) / voxel)), dropped points -> frame B,
//                   points ordered by (frame, x, y)
//   k_seg_count     per 1024 sorted points: how many cells start there
//   k_seg_scan      exclusive prefix over those counts, total = number of pillars (above 262,144 points only)
//   k_seg_starts    numbers the cell starts: start position and cell of every pillar
//   k_seg_mean      sixteen lanes per pillar: mean of its points' features, point -> pillar
#include "common.h"

namespace ff {
namespace {

constexpr int kSegBlock = 1024;
constexpr int kPointsInFlight = 8;  // per lane of k_seg_mean
constexpr int kSegDirectBlocks = 256;  // up to 262,144 points the blocks' prefixes need no launch of their own

// exported key of the sort: frame << 48 | x << 32 | y << 16 (window 1 x 1: no local fields)
// The key at sorted position p and the one before it, loaded without conditions (positions clamped
// into the array) so that a thread's loads travel together; starts_cell then tells whether p is the
// first point of a cell inside the grid.
struct KeyPair { uint64_t k, before; };
__device__ __forceinline__ KeyPair load_pair(const uint64_t* __restrict__ keys, int64_t p, int64_t m) {
  const int64_t pc = p < m ? p : m - 1;
  return {keys[pc], keys[pc > 0 ? pc - 1 : 0]};
}
__device__ __forceinline__ bool starts_cell(const KeyPair& kp, int64_t p, int64_t m, int B) {
  return p < m && (int)(kp.k >> 48) < B && (p == 0 || kp.before != kp.k);
}

__global__ __launch_bounds__(256) void k_seg_count(const uint64_t* __restrict__ keys, int64_t m, int B,
                                                    uint32_t* __restrict__ block_counts, int32_t* __restrict__ kept) {
  __shared__ uint32_t wave_sums[4];
  if (blockIdx.x == 0 && threadIdx.x == 0) *kept = (int32_t)m;  // lowered by k_seg_starts
  const int64_t p0 = (int64_t)blockIdx.x * kSegBlock;
  uint32_t c = 0;
  if (m > 0) {  // the same for every thread
    KeyPair kp[kSegBlock / 256];
#pragma unroll
    for (int r = 0; r < kSegBlock / 256; ++r) kp[r] = load_pair(keys, p0 + r * 256 + threadIdx.x, m);
#pragma unroll
    for (int r = 0; r < kSegBlock / 256; ++r)
      if (starts_cell(kp[r], p0 + r * 256 + threadIdx.x, m, B)) ++c;
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) c += __shfl_xor(c, d, 64);
  if ((threadIdx.x & 63) == 0) wave_sums[threadIdx.x >> 6] = c;
  __syncthreads();
  if (threadIdx.x == 0) block_counts[blockIdx.x] = wave_sums[0] + wave_sums[1] + wave_sums[2] + wave_sums[3];
}

// One workgroup: block_counts -> exclusive prefixes in place, total -> *num_pillars.  Only for more
// blocks than k_seg_starts adds up by itself.
__global__ __launch_bounds__(1024) void k_seg_scan(uint32_t* __restrict__ block_counts, int64_t nb,
                                                    int32_t* __restrict__ num_pillars) {
  __shared__ uint32_t wave_sums[16];
  __shared__ uint32_t carry_s;
  if (threadIdx.x == 0) carry_s = 0;
  __syncthreads();
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  for (int64_t base = 0; base < nb; base += 1024) {
    const int64_t i = base + threadIdx.x;
    const uint32_t v = i < nb ? block_counts[i] : 0u;
    uint32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const uint32_t t = __shfl_up(inc, d, 64);
      if (lane >= d) inc += t;
    }
    if (lane == 63) wave_sums[w] = inc;
    __syncthreads();
    uint32_t before = carry_s, total = 0;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const uint32_t t = wave_sums[k];
      if (k < w) before += t;
      total += t;
    }
    if (i < nb) block_counts[i] = before + inc - v;
    __syncthreads();
    if (threadIdx.x == 0) carry_s += total;
    __syncthreads();
  }
  if (threadIdx.x == 0) *num_pillars = (int32_t)carry_s;
}

// Cell starts get their pillar numbers (block-local scan on top of the block's prefix): writes where
// each pillar's run of sorted points starts, its cell, and -1 for the points that were dropped.
// SCANNED: block_base holds exclusive prefixes (k_seg_scan ran).  Otherwise it holds the blocks'
// counts and every workgroup adds up the ones before it (a few KB from L2: cheaper than a dependent
// launch); workgroup 0 also writes the total.
template <bool SCANNED>
__global__ __launch_bounds__(256) void k_seg_starts(const uint64_t* __restrict__ keys, const int32_t* __restrict__ perm,
                                                     int64_t m, int B, const uint32_t* __restrict__ block_base, int nb,
                                                     int32_t* __restrict__ num_pillars,
                                                     int32_t* __restrict__ starts, int32_t* __restrict__ kept,
                                                     int32_t* __restrict__ coords, int32_t* __restrict__ point_to_pillar) {
  __shared__ uint32_t wave_sums[4];
  __shared__ uint32_t base_sums[4][2];
  uint32_t base = 0;
  if (SCANNED) {
    base = block_base[blockIdx.x];
  } else {
    uint32_t before = 0, all = 0;
    for (int i = threadIdx.x; i < nb; i += 256) {
      const uint32_t c = block_base[i];
      all += c;
      if (i < (int)blockIdx.x) before += c;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) { before += __shfl_xor(before, d, 64); all += __shfl_xor(all, d, 64); }
    if ((threadIdx.x & 63) == 0) { base_sums[threadIdx.x >> 6][0] = before; base_sums[threadIdx.x >> 6][1] = all; }
    __syncthreads();
    base = base_sums[0][0] + base_sums[1][0] + base_sums[2][0] + base_sums[3][0];
    if (blockIdx.x == 0 && threadIdx.x == 0)
      *num_pillars = (int32_t)(base_sums[0][1] + base_sums[1][1] + base_sums[2][1] + base_sums[3][1]);
  }
  const int64_t p0 = (int64_t)blockIdx.x * kSegBlock;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  // thread t owns positions p0 + 4t .. p0 + 4t + 3, so that cell starts are numbered in sorted order
  bool head[4];
  KeyPair kp[4];
  uint32_t mine = 0;
#pragma unroll
  for (int r = 0; r < 4; ++r) kp[r] = m > 0 ? load_pair(keys, p0 + 4 * threadIdx.x + r, m) : KeyPair{0, 0};
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    head[r] = starts_cell(kp[r], p0 + 4 * threadIdx.x + r, m, B);
    mine += head[r] ? 1u : 0u;
  }
  uint32_t inc = mine;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t t = __shfl_up(inc, d, 64);
    if (lane >= d) inc += t;
  }
  if (lane == 63) wave_sums[w] = inc;
  __syncthreads();
  uint32_t pid = base + inc - mine;
  for (int k = 0; k < w; ++k) pid += wave_sums[k];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int64_t p = p0 + 4 * threadIdx.x + r;
    if (p >= m) continue;
    const uint64_t k = kp[r].k;
    if ((int)(k >> 48) >= B) {  // dropped points sort behind all pillars
      if (point_to_pillar) point_to_pillar[perm[p]] = -1;
      if (p == 0 || (int)(kp[r].before >> 48) < B) *kept = (int32_t)p;
    }
    if (!head[r]) continue;
    starts[pid] = (int32_t)p;
    coords[3 * (int64_t)pid + 0] = (int32_t)(k >> 48);
    coords[3 * (int64_t)pid + 1] = (int32_t)((k >> 32) & 0xffffu);
    coords[3 * (int64_t)pid + 2] = (int32_t)((k >> 16) & 0xffffu);
    ++pid;
  }
}

// Sixteen lanes per pillar: lane l adds the points l, l + 16, ... of the pillar's run in float32, the
// sixteen partial sums are combined in a fixed tree, so the result does not depend on timing.
__global__ __launch_bounds__(256) void k_seg_mean(const int32_t* __restrict__ perm, const float* __restrict__ pfeats,
                                                   int Cp, const int32_t* __restrict__ num_pillars,
                                                   const int32_t* __restrict__ starts, const int32_t* __restrict__ kept,
                                                   float* __restrict__ feats, int32_t* __restrict__ point_to_pillar) {
  const int np = *num_pillars, sub = threadIdx.x & 15;
  const bool vec4 = Cp % 4 == 0 && (reinterpret_cast<uintptr_t>(pfeats) & 15) == 0;
  const int64_t stride = (int64_t)gridDim.x * (blockDim.x / 16);
  for (int64_t pid = (int64_t)blockIdx.x * (blockDim.x / 16) + (threadIdx.x >> 4); pid < np; pid += stride) {
    const int lo = starts[pid], hi = pid + 1 < np ? starts[pid + 1] : *kept;
    const float inv = 1.0f / (float)(hi - lo);
    for (int c0 = 0; c0 < Cp; c0 += 4) {  // four features at a time
      float acc[4] = {0.f, 0.f, 0.f, 0.f};
      // eight points per lane and round, their loads in flight together: a pillar of several hundred
      // points (a dense object, the cell under the sensor) is a chain of dependent round trips otherwise
      for (int q = lo + sub; q < hi; q += 16 * kPointsInFlight) {
        int32_t src[kPointsInFlight];
#pragma unroll
        for (int u = 0; u < kPointsInFlight; ++u) src[u] = q + 16 * u < hi ? perm[q + 16 * u] : -1;
        if (point_to_pillar && c0 == 0) {  // the point indices are at hand here (Cp >= 1: this round always runs)
#pragma unroll
          for (int u = 0; u < kPointsInFlight; ++u)
            if (src[u] >= 0) point_to_pillar[src[u]] = (int32_t)pid;
        }
        float v[kPointsInFlight][4];
        if (vec4) {  // four features of a point in one 16-byte load (the same for every thread)
#pragma unroll
          for (int u = 0; u < kPointsInFlight; ++u) {
            const float4 t = *reinterpret_cast<const float4*>(pfeats + (int64_t)(src[u] >= 0 ? src[u] : 0) * Cp + c0);
            v[u][0] = src[u] >= 0 ? t.x : 0.f; v[u][1] = src[u] >= 0 ? t.y : 0.f;
            v[u][2] = src[u] >= 0 ? t.z : 0.f; v[u][3] = src[u] >= 0 ? t.w : 0.f;
          }
        } else {
#pragma unroll
          for (int u = 0; u < kPointsInFlight; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j)
              v[u][j] = src[u] >= 0 && c0 + j < Cp ? pfeats[(int64_t)src[u] * Cp + c0 + j] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kPointsInFlight; ++u)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[j] += v[u][j];
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int d = 8; d >= 1; d >>= 1) acc[j] += __shfl_xor(acc[j], d, 16);
        if (sub == 0 && c0 + j < Cp) feats[pid * Cp + c0 + j] = acc[j] * inv;
      }
    }
  }
}

struct VoxLayout {
  ff_geom geom;  // the geometry the sort sees: one extra frame, 1 x 1 windows
  size_t off_perm, off_keys, off_goff, off_ng, off_blocks, off_starts, off_flat, flat_bytes, total;
  int64_t nb;
};

int make_vox_layout(int64_t m, const ff_geom* g, VoxLayout* L) {
  if (!g || m < 0 || m > 0x7fffffffLL) return FF_ERR_ARG;
  if (g->num_frames < 1 || g->num_frames > 65534 || g->grid_x < 1 || g->grid_x > 65535 || g->grid_y < 1 ||
      g->grid_y > 65535)
    return FF_ERR_ARG;
  L->geom = *g;
  L->geom.num_frames = g->num_frames + 1;
  L->geom.win_x = L->geom.win_y = 1;
  L->flat_bytes = flatten_workspace_bytes(m, &L->geom, 1);
  if (L->flat_bytes == 0) return FF_ERR_UNSUPPORTED;
  L->nb = ceil_div(m > 0 ? m : 1, kSegBlock);
  size_t off = 0;
  L->off_perm = off;   off += align_up((size_t)m * 4, 256);
  L->off_keys = off;   off += align_up((size_t)m * 8, 256);
  L->off_goff = off;   off += align_up((size_t)(L->geom.num_frames + 2) * 4, 256);  // one group per frame
  L->off_ng = off;     off += 256;
  L->off_blocks = off; off += align_up((size_t)L->nb * 4, 256);
  L->off_starts = off; off += align_up((size_t)(m + 1) * 4, 256);
  L->off_flat = off;   off += align_up(L->flat_bytes, 256);
  L->total = off;
  return FF_OK;
}

}  // namespace

size_t voxelize_workspace_bytes(int64_t m, const ff_geom* g) {
  VoxLayout L;
  return make_vox_layout(m, g, &L) == FF_OK ? L.total : 0;
}

int voxelize_launch(const float* xy, const int32_t* frame, const float* pfeats, int64_t m, int Cp, const ff_geom* g,
                    const ff_voxel_grid* v, int32_t* coords, float* feats, int32_t* num_pillars,
                    int32_t* point_to_pillar, void* workspace, size_t workspace_bytes, hipStream_t stream) {
  VoxLayout L;
  int st = make_vox_layout(m, g, &L);
  if (st != FF_OK) return st;
  if (!v || !(v->voxel_x > 0.f) || !(v->voxel_y > 0.f) || Cp < 1 || !num_pillars) return FF_ERR_ARG;
  if (m > 0 && (!xy || !pfeats || !coords || !feats)) return FF_ERR_ARG;
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < L.total) return FF_ERR_WORKSPACE;
  char* ws = (char*)workspace;
  int32_t* perm = (int32_t*)(ws + L.off_perm);
  uint64_t* keys = (uint64_t*)(ws + L.off_keys);
  int32_t* goff = (int32_t*)(ws + L.off_goff);
  int32_t* ng = (int32_t*)(ws + L.off_ng);
  uint32_t* blocks = (uint32_t*)(ws + L.off_blocks);
  // key generation computes the cells itself: no array of cells, no launch for it
  const PointCells pts{xy, frame, g->num_frames, g->grid_x, g->grid_y, v->x_min, v->y_min, v->voxel_x, v->voxel_y};
  st = flatten_launch_points(&pts, m, &L.geom, perm, goff, ng, keys, ws + L.off_flat, L.flat_bytes, stream);
  if (st != FF_OK) return st;
  int32_t* starts = (int32_t*)(ws + L.off_starts);
  int32_t* kept = ng + 1;  // number of points inside the grid (a spare word beside the sort's group count)
  hipLaunchKernelGGL(k_seg_count, dim3((unsigned)L.nb), dim3(256), 0, stream, keys, m, g->num_frames, blocks, kept);
  if (L.nb <= kSegDirectBlocks) {
    hipLaunchKernelGGL(k_seg_starts<false>, dim3((unsigned)L.nb), dim3(256), 0, stream, keys, perm, m, g->num_frames,
                       blocks, (int)L.nb, num_pillars, starts, kept, coords, point_to_pillar);
  } else {
    hipLaunchKernelGGL(k_seg_scan, dim3(1), dim3(1024), 0, stream, blocks, L.nb, num_pillars);
    hipLaunchKernelGGL(k_seg_starts<true>, dim3((unsigned)L.nb), dim3(256), 0, stream, keys, perm, m, g->num_frames,
                       blocks, (int)L.nb, num_pillars, starts, kept, coords, point_to_pillar);
  }
  int64_t mean_blocks = ceil_div(m > 0 ? m : 1, 16);  // a pillar per sixteen lanes; there are at most m pillars
  if (mean_blocks > 256 * 32) mean_blocks = 256 * 32;
  hipLaunchKernelGGL(k_seg_mean, dim3((unsigned)mean_blocks), dim3(256), 0, stream, perm, pfeats, Cp, num_pillars, starts,
                     kept, feats, point_to_pillar);
  return launch_status();
}

}  // namespace ff
