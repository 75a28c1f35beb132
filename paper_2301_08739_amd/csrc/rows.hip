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

}  // namespace

int rows_launch(bool scatter, const void* src, void* dst, const int32_t* perm, int64_t n, int C,
                int dtype, hipStream_t stream) {
  if (n < 0 || C < 1 || (dtype != FF_F32 && dtype != FF_BF16)) return FF_ERR_ARG;
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
