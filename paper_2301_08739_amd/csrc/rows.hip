// Row gather / scatter between pillar order and the flattened (sorted) order: the explicit form
// of the reshape [N, C] -> [N/G, G, C] of paper Sec. 4.2.1.  Pure data movement, HBM-bound:
// every thread moves one 16-byte piece, consecutive threads move consecutive pieces of a row.
#include "common.h"

namespace ff {
namespace {

template <bool SCATTER>
__global__ __launch_bounds__(256) void k_rows(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                               const int32_t* __restrict__ perm, int64_t n, int vec_per_row) {
  const int64_t total = n * vec_per_row;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t p = i / vec_per_row;
    const int v = (int)(i - p * vec_per_row);
    const int64_t r = perm[p];
    if (SCATTER) dst[r * vec_per_row + v] = src[i];
    else         dst[i] = src[r * vec_per_row + v];
  }
}

// Rows of sorted positions outside every group skip the layer ('Drop Residual', Sec. 4.3): for a
// residual layer that means out = feats.  A workgroup looks at 64 consecutive sorted positions; a
// position p is grouped when the last group start at or before p lies less than G before it.
template <typename T, typename TO>
__global__ __launch_bounds__(256) void k_copy_ungrouped(const T* __restrict__ feats, TO* __restrict__ out,
                                                         const int32_t* __restrict__ perm,
                                                         const int32_t* __restrict__ group_offsets,
                                                         const int32_t* __restrict__ num_groups, int max_groups,
                                                         int64_t n, int C, int G) {
  __shared__ int32_t row_of[64];
  const int64_t p0 = (int64_t)blockIdx.x * 64;
  if (threadIdx.x < 64) {
    const int64_t p = p0 + threadIdx.x;
    int32_t row = -1;
    if (p < n) {
      int ng = max_groups > 0 ? *num_groups : 0;
      ng = ng < 0 ? 0 : (ng > max_groups ? max_groups : ng);
      int lo = 0, hi = ng;  // first group start beyond p
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (group_offsets[mid] <= p) lo = mid + 1; else hi = mid;
      }
      if (lo == 0 || p >= (int64_t)group_offsets[lo - 1] + G) row = perm[p];
    }
    row_of[threadIdx.x] = row;
  }
  __syncthreads();
  for (int r = 0; r < 64; ++r) {
    const int32_t row = row_of[r];
    if (row < 0) continue;
    for (int k = threadIdx.x; k < C; k += blockDim.x)
      Elem<TO>::store(out + (int64_t)row * C + k, Elem<T>::load(feats + (int64_t)row * C + k));
  }
}

// ---- sparse pillars -> dense bird's-eye-view map (the step after the FWA blocks, Sec. 5.1 'Model') -----
// bev[b][y][x][:] = feats[i][:] for pillar i = (b, x, y), zero elsewhere; channels last, so that a
// pillar's features stay one contiguous row.  Two launches: zero fill (the map is mostly empty:
// 30k of 219k cells at the paper's resolution), then one 16-byte piece per thread.
__global__ __launch_bounds__(256) void k_fill_zero(uint4* __restrict__ dst, int64_t pieces) {
  const uint4 z = make_uint4(0u, 0u, 0u, 0u);
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < pieces; i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = z;
}

__global__ __launch_bounds__(256) void k_bev_scatter(const uint4* __restrict__ feats, const int32_t* __restrict__ coords,
                                                      int64_t n, int vec_per_row, int B, int gx, int gy,
                                                      uint4* __restrict__ bev) {
  const int64_t total = n * vec_per_row;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t p = i / vec_per_row;
    const int v = (int)(i - p * vec_per_row);
    const int32_t b = coords[3 * p], x = coords[3 * p + 1], y = coords[3 * p + 2];
    if ((uint32_t)b >= (uint32_t)B || (uint32_t)x >= (uint32_t)gx || (uint32_t)y >= (uint32_t)gy) continue;  // outside the map
    bev[(((int64_t)b * gy + y) * gx + x) * vec_per_row + v] = feats[i];
  }
}

}  // namespace

int bev_scatter_launch(const void* feats, const int32_t* coords, int64_t n, const ff_geom* g, int C, int dtype,
                       void* bev, hipStream_t stream) {
  if (!g || n < 0 || C < 1 || (dtype != FF_F32 && dtype != FF_BF16 && dtype != FF_F16)) return FF_ERR_ARG;
  if (g->num_frames < 1 || g->grid_x < 1 || g->grid_y < 1 || !bev) return FF_ERR_ARG;
  const size_t row_bytes = (size_t)C * (dtype == FF_F32 ? 4 : 2);
  if (row_bytes % 16) return FF_ERR_UNSUPPORTED;
  if (((uintptr_t)bev & 15) || ((uintptr_t)feats & 15)) return FF_ERR_ARG;
  if (n > 0 && (!feats || !coords)) return FF_ERR_ARG;
  const int vec = (int)(row_bytes / 16);
  const int64_t pieces = (int64_t)g->num_frames * g->grid_x * g->grid_y * vec;
  int64_t fb = ceil_div(pieces, 256 * 8);
  if (fb > 256 * 64) fb = 256 * 64;
  hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)fb), dim3(256), 0, stream, (uint4*)bev, pieces);
  if (n > 0) {
    int64_t blocks = ceil_div(n * vec, 256);
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(k_bev_scatter, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint4*)feats, coords, n, vec,
                       g->num_frames, g->grid_x, g->grid_y, (uint4*)bev);
  }
  return launch_status();
}

// ---- coordinate check: how many rows of coords lie outside the geometry -------------------------------------
// result[0] = rows with a frame, x or y outside [0, num_frames) x [0, grid_x) x [0, grid_y), result[1] = index of
// the first such row (n if there is none).  Two launches: the two words are set, then every workgroup adds its
// count (and lowers the index) with one atomic each.
__global__ void k_check_init(int32_t* __restrict__ result, int32_t n) { result[0] = 0; result[1] = n; }

__global__ __launch_bounds__(256) void k_check_coords(const int32_t* __restrict__ coords, int64_t n, int B, int gx, int gy,
                                                       int32_t* __restrict__ result) {
  __shared__ uint32_t bad_s;
  __shared__ int32_t first_s;
  if (threadIdx.x == 0) { bad_s = 0u; first_s = 0x7fffffff; }
  __syncthreads();
  uint32_t bad = 0;
  int32_t first = 0x7fffffff;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    const int32_t b = coords[3 * i], x = coords[3 * i + 1], y = coords[3 * i + 2];
    if ((uint32_t)b >= (uint32_t)B || (uint32_t)x >= (uint32_t)gx || (uint32_t)y >= (uint32_t)gy) {
      ++bad;
      if ((int32_t)i < first) first = (int32_t)i;
    }
  }
  if (bad) { atomicAdd(&bad_s, bad); atomicMin(&first_s, first); }
  __syncthreads();
  if (threadIdx.x == 0 && bad_s) { atomicAdd(&result[0], (int32_t)bad_s); atomicMin(&result[1], first_s); }
}

int check_coords_launch(const int32_t* coords, int64_t n, const ff_geom* g, int32_t* result, hipStream_t stream) {
  if (!g || n < 0 || n > 0x7fffffffLL || !result || (n > 0 && !coords)) return FF_ERR_ARG;
  if (g->num_frames < 1 || g->grid_x < 1 || g->grid_y < 1) return FF_ERR_ARG;
  hipLaunchKernelGGL(k_check_init, dim3(1), dim3(1), 0, stream, result, (int32_t)n);
  if (n > 0) {
    int64_t blocks = ceil_div(n, 256 * 4);
    if (blocks > 256 * 8) blocks = 256 * 8;
    hipLaunchKernelGGL(k_check_coords, dim3((unsigned)blocks), dim3(256), 0, stream, coords, n, g->num_frames, g->grid_x,
                       g->grid_y, result);
  }
  return launch_status();
}

int rows_copy_ungrouped_launch(const void* feats, void* out, int64_t n, const int32_t* perm,
                               const int32_t* group_offsets, const int32_t* num_groups, int32_t max_groups, int C,
                               int G, int dtype, bool out_f32, hipStream_t stream) {
  if (n < 0 || C < 1 || G < 1 || max_groups < 0 || (dtype != FF_F32 && dtype != FF_BF16 && dtype != FF_F16)) return FF_ERR_ARG;
  if (n == 0) return FF_OK;
  if (!feats || !out || !perm || (max_groups > 0 && (!group_offsets || !num_groups))) return FF_ERR_ARG;
  const dim3 grid((unsigned)ceil_div(n, 64)), block(256);
  if (dtype == FF_F32)
    hipLaunchKernelGGL((k_copy_ungrouped<float, float>), grid, block, 0, stream, (const float*)feats, (float*)out,
                       perm, group_offsets, num_groups, (int)max_groups, n, C, G);
  else if (out_f32 && dtype == FF_F16)
    hipLaunchKernelGGL((k_copy_ungrouped<f16_t, float>), grid, block, 0, stream, (const f16_t*)feats, (float*)out,
                       perm, group_offsets, num_groups, (int)max_groups, n, C, G);
  else if (out_f32)
    hipLaunchKernelGGL((k_copy_ungrouped<bf16_t, float>), grid, block, 0, stream, (const bf16_t*)feats, (float*)out,
                       perm, group_offsets, num_groups, (int)max_groups, n, C, G);
  else  // 16 bits to the same 16 bits: a bit copy for either format
    hipLaunchKernelGGL((k_copy_ungrouped<bf16_t, bf16_t>), grid, block, 0, stream, (const bf16_t*)feats,
                       (bf16_t*)out, perm, group_offsets, num_groups, (int)max_groups, n, C, G);
  return launch_status();
}

int rows_launch(bool scatter, const void* src, void* dst, const int32_t* perm, int64_t n, int C,
                int dtype, hipStream_t stream) {
  if (n < 0 || C < 1 || (dtype != FF_F32 && dtype != FF_BF16 && dtype != FF_F16)) return FF_ERR_ARG;
  const size_t row_bytes = (size_t)C * (dtype == FF_F32 ? 4 : 2);
  if (row_bytes % 16) return FF_ERR_UNSUPPORTED;
  if (n == 0) return FF_OK;
  if (!src || !dst || !perm || src == dst) return FF_ERR_ARG;
  if (((uintptr_t)src | (uintptr_t)dst) & 15) return FF_ERR_ARG;
  const int vec = (int)(row_bytes / 16);
  int64_t blocks = ceil_div(n * vec, 256);
  if (blocks > 256 * 32) blocks = 256 * 32;
  if (scatter)
    hipLaunchKernelGGL(k_rows<true>, dim3((unsigned)blocks), dim3(256), 0, stream,
                       (const uint4*)src, (uint4*)dst, perm, n, vec);
  else
    hipLaunchKernelGGL(k_rows<false>, dim3((unsigned)blocks), dim3(256), 0, stream,
                       (const uint4*)src, (uint4*)dst, perm, n, vec);
  return launch_status();
}

}  // namespace ff
