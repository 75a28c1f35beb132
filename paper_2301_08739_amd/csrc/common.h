// Internal helpers shared by the HIP translation units of libflatformer.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/flatformer.h"

namespace ff {

constexpr int kWave = 64;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
// number of bits needed to represent values 0..v (0 for v == 0)
inline int bit_width_u64(uint64_t v) { int b = 0; while (v) { ++b; v >>= 1; } return b; }

inline int launch_status() { return hipGetLastError() == hipSuccess ? FF_OK : FF_ERR_LAUNCH; }

// ---- bf16 <-> f32 on the device (round to nearest even) -------------------------------------
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;  // NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Storage-type traits: T is float, bf16_t or f16_t (16-bit wrappers).
struct bf16_t { uint16_t bits; };
struct f16_t { uint16_t bits; };
template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(p->bits); }
  static __device__ __forceinline__ void store(bf16_t* p, float v) { p->bits = f32_to_bf16(v); }
};
template <> struct Elem<f16_t> {  // IEEE half, round to nearest even
  static __device__ __forceinline__ float load(const f16_t* p) { return (float)__builtin_bit_cast(_Float16, p->bits); }
  static __device__ __forceinline__ void store(f16_t* p, float v) { p->bits = __builtin_bit_cast(uint16_t, (_Float16)v); }
};

// ---- flatten plan (host) -------------------------------------------------------------------------
struct FlattenPlan {
  int bits_b, bits_w1, bits_w2, bits_l1, bits_l2;  // live bits of each tuple field, in sort priority
  int bits_w3, bits_l3;                            // the z fields of 3-D windows (0 for pillars)
  int key_bits;                                    // sum of the above
  int idx_bits;                                    // bits of n-1
  int passes;                                      // radix passes of 8 bits over the key bits
};

constexpr int kRadixBits = 8;
constexpr int kBins = 1 << kRadixBits;
constexpr int kSortThreads = 256;

int make_flatten_plan(int64_t n, const ff_geom* g, int axis, int shift, FlattenPlan* plan);
size_t flatten_workspace_bytes(int64_t n, const ff_geom* g, int num_sorts);
// The same with a third voxel coordinate (z == nullptr: pillars).  coords then has four columns
// (b, x, y, z); z is the last of the window fields and the last of the local fields of the key.
struct FlattenZ { int32_t grid_z, win_z; };
int make_flatten_plan_z(int64_t n, const ff_geom* g, const FlattenZ* z, int axis, int shift, FlattenPlan* plan);
size_t flatten_workspace_bytes_z(int64_t n, const ff_geom* g, const FlattenZ* z, int num_sorts);

// num_sorts (1..4) sort configurations of the same cloud, sorted together.  pack: nullptr, or layer
// weights to re-tile in extra workgroups of the first kernel (n > 0 only; see pack_weights.h).
struct PackJob;
int flatten_launch(const int32_t* coords, int64_t n, const ff_geom* g, int num_sorts, const int* axis,
                   const int* shift, int G, int drop, int32_t* const* perm, int32_t* const* inv_perm /* or nullptr */,
                   int32_t* const* group_offsets, int32_t* const* num_groups, uint64_t* const* keys_sorted,
                   void* workspace, size_t workspace_bytes, const PackJob* pack, hipStream_t stream);

int flatten_launch_z(const int32_t* coords, int64_t n, const ff_geom* g, const FlattenZ* z, int num_sorts,
                     const int* axis, const int* shift, int G, int drop, int32_t* const* perm,
                     int32_t* const* inv_perm, int32_t* const* group_offsets, int32_t* const* num_groups,
                     uint64_t* const* keys_sorted, void* workspace, size_t workspace_bytes, const PackJob* pack,
                     hipStream_t stream);

// The same sort fed by raw points instead of integer coordinates: key generation computes the cell of
// point i itself, (frame, floor((x - x_min) / voxel_x), floor((y - y_min) / voxel_y)) in float32, and puts a
// point outside the grid or the frame range into frame B at cell (0, 0) (g->num_frames counts that frame).
struct PointCells {
  const float* xy;        // [n, 2]
  const int32_t* frame;   // [n] or nullptr (all points in frame 0)
  int32_t B, grid_x, grid_y;
  float x_min, y_min, voxel_x, voxel_y;
};
int flatten_launch_points(const PointCells* pts, int64_t n, const ff_geom* g, int32_t* perm, int32_t* group_offsets,
                          int32_t* num_groups, uint64_t* keys_sorted, void* workspace, size_t workspace_bytes,
                          hipStream_t stream);

int rows_launch(bool scatter, const void* src, void* dst, const int32_t* perm, int64_t n, int C,
                int dtype, hipStream_t stream);
// out[perm[p], :] = feats[perm[p], :] for every sorted position p outside all groups, a group being
// G positions from its start.  max_groups == 0: no group exists, every row is copied.
int rows_copy_ungrouped_launch(const void* feats, void* out, int64_t n, const int32_t* perm,
                               const int32_t* group_offsets, const int32_t* num_groups, int32_t max_groups, int C,
                               int G, int dtype, bool out_f32, hipStream_t stream);

// result[0] = rows of coords outside the geometry, result[1] = index of the first one (n: none)
int check_coords_launch(const int32_t* coords, int64_t n, const ff_geom* g, int32_t* result, hipStream_t stream);

// bev [num_frames][grid_y][grid_x][C] = rows of feats at their pillars' cells, zero elsewhere
int bev_scatter_launch(const void* feats, const int32_t* coords, int64_t n, const ff_geom* g, int C, int dtype,
                       void* bev, hipStream_t stream);

size_t voxelize_workspace_bytes(int64_t m, const ff_geom* g);
int voxelize_launch(const float* xy, const int32_t* frame, const float* pfeats, int64_t m, int Cp, const ff_geom* g,
                    const ff_voxel_grid* v, int32_t* coords, float* feats, int32_t* num_pillars,
                    int32_t* point_to_pillar, void* workspace, size_t workspace_bytes, hipStream_t stream);

size_t layer_generic_workspace_bytes(int64_t n, const ff_layer_weights* w);
int layer_generic_launch(const void* feats, void* out, int64_t n, const int32_t* perm,
                         const int32_t* group_offsets, const int32_t* num_groups, int32_t max_groups,
                         const ff_layer_weights* w, int G, int dtype, bool out_f32,
                         void* workspace, size_t workspace_bytes, hipStream_t stream);

// Fused bf16 matrix-core layer (layer_mfma.hip)
bool layer_mfma_supported(const ff_layer_weights* w, int G);
size_t layer_mfma_packed_bytes(const ff_layer_weights* w);
int layer_mfma_pack(const ff_layer_weights* w, int count, void* packed, size_t stride_bytes, hipStream_t stream);
// out_index: nullptr, or for every pillar the row of `out` its result goes to (instead of its own
// index).  in_sorted: 0 = feats is in pillar order; 1 = row p of feats is the pillar at sorted
// position p; 2 = the same, and groups start at multiples of G (one frame), which lets the kernel
// fetch its rows before it has read the group list.
int layer_mfma_launch(const void* feats, void* out, int64_t n, const int32_t* perm, const int32_t* group_offsets,
                      const int32_t* num_groups, int32_t max_groups, const ff_layer_weights* w, int G,
                      bool out_f32, bool drop, const void* packed, int variant, const int32_t* out_index,
                      int in_sorted, hipStream_t stream);
// the same two for IEEE half storage (layer_mfma_f16.hip); shapes and packed size do not differ
int layer_mfma_pack_f16(const ff_layer_weights* w, int count, void* packed, size_t stride_bytes, hipStream_t stream);
int layer_mfma_launch_f16(const void* feats, void* out, int64_t n, const int32_t* perm, const int32_t* group_offsets,
                          const int32_t* num_groups, int32_t max_groups, const ff_layer_weights* w, int G,
                          bool out_f32, bool drop, const void* packed, int variant, const int32_t* out_index,
                          int in_sorted, hipStream_t stream);

}  // namespace ff
