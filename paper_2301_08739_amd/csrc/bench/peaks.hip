// Two micro-benchmarks that bench.py times beside the library's kernels, so that every roofline fraction
// can be read against what THIS box reaches as well as against the data-sheet peaks: a plain streaming
// copy (HBM bandwidth) and a loop of independent bf16 matrix-core products (dense MFMA rate).  Built into
// libffpeaks.so, a bench-only library; nothing in libflatformer.so depends on it.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// dst[i] = src[i], 16 bytes per lane, four pieces in flight per lane, grid-stride.
__global__ __launch_bounds__(256) void k_stream_copy(u32x4* __restrict__ dst, const u32x4* __restrict__ src, size_t pieces) {
  const size_t stride = (size_t)gridDim.x * 256 * 4;
  for (size_t base = ((size_t)blockIdx.x * 4) * 256 + threadIdx.x; base < pieces; base += stride) {
    u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (base + u * 256 < pieces) v[u] = __builtin_nontemporal_load(src + base + u * 256);
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (base + u * 256 < pieces) __builtin_nontemporal_store(v[u], dst + base + u * 256);
  }
}

// Every wavefront issues iters x 8 independent matrix-core products.  SHAPE 0: v_mfma_f32_16x16x32_bf16
// (16,384 flop), SHAPE 1: v_mfma_f32_32x32x16_bf16 (32,768 flop).  Thread 0 of workgroup 0 also reports how many
// shader-clock cycles and how many ticks of the constant 100 MHz counter its loop took: their ratio is the clock
// the chip really ran the loop at.
template <int SHAPE>
__global__ __launch_bounds__(256) void k_mfma_loop(float* __restrict__ sink, int iters, long long* __restrict__ ticks) {
  typedef float f32x16 __attribute__((ext_vector_type(16)));
  bf16x8 a, b;
#pragma unroll
  for (int j = 0; j < 8; ++j) { a[j] = (__bf16)(float)((threadIdx.x + j) & 3); b[j] = (__bf16)(float)(j & 1); }
  float s = 0.f;
  long long c0 = 0, w0 = 0, c1 = 0, w1 = 0;
  if constexpr (SHAPE == 0) {
    f32x4 acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = f32x4{0.f, 0.f, 0.f, 0.f};
    c0 = clock64(); w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int k = 0; k < 8; ++k)  // (written as assembly: the accumulators stay in place, the loop is the eight products)
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc[k]) : "v"(a), "v"(b));
    }
    c1 = clock64(); w1 = wall_clock64();
#pragma unroll
    for (int k = 0; k < 8; ++k) s += acc[k][0] + acc[k][1] + acc[k][2] + acc[k][3];
  } else {
    f32x16 acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[k][e] = 0.f;
    c0 = clock64(); w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int k = 0; k < 8; ++k)
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[k]) : "v"(a), "v"(b));
    }
    c1 = clock64(); w1 = wall_clock64();
#pragma unroll
    for (int k = 0; k < 8; ++k) s += acc[k][0] + acc[k][5] + acc[k][10] + acc[k][15];
  }
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
  if (ticks && blockIdx.x == 0 && threadIdx.x == 0) { ticks[0] = c1 - c0; ticks[1] = w1 - w0; }
}

}  // namespace

extern "C" {

// Copies `bytes` (a multiple of 16; both pointers 16-byte aligned, device memory) on `stream`.
// Returns 0, or -1 for bad arguments, -4 if the launch failed.
int ffpeak_stream_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || bytes % 16 || ((uintptr_t)dst | (uintptr_t)src) % 16) return -1;
  if (bytes == 0) return 0;
  const size_t pieces = bytes / 16;
  size_t blocks = (pieces + 1023) / 1024;
  if (blocks > 256 * 32) blocks = 256 * 32;
  hipLaunchKernelGGL(k_stream_copy, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (u32x4*)dst,
                     (const u32x4*)src, pieces);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

// Launches `blocks` workgroups of four wavefronts, each wavefront issuing iters x 8 products of `shape`
// (0: 16x16x32, 1: 32x32x16, both bf16 with fp32 accumulation).  sink: device floats, blocks x 256 of them.
// ticks: NULL, or two device int64: shader-clock cycles and 100 MHz ticks of one wavefront's loop.
// *flops receives the number of floating-point operations the launch performs.
int ffpeak_mfma_bf16(float* sink, int blocks, int iters, int shape, long long* ticks, double* flops, void* stream) {
  if (!sink || blocks < 1 || iters < 1 || shape < 0 || shape > 1) return -1;
  if (shape == 0)
    hipLaunchKernelGGL(k_mfma_loop<0>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, sink, iters, ticks);
  else
    hipLaunchKernelGGL(k_mfma_loop<1>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, sink, iters, ticks);
  if (flops) *flops = (double)blocks * 4.0 * (double)iters * 8.0 * (2.0 * 16 * 16 * 32) * (shape == 1 ? 2.0 : 1.0);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // extern "C"
