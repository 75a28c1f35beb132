// extern "C" entry points: argument checks, workspace carving and launch order.  No kernel lives
// here; see flatten.hip, rows.hip, layer_generic.hip, layer_mfma.hip.
#include "common.h"
#include "pack_weights.h"
#include <atomic>

using namespace ff;

namespace {

int check_weights(const ff_layer_weights* w, int dtype) {
  if (!w) return FF_ERR_ARG;
  if (dtype != FF_F32 && dtype != FF_BF16 && dtype != FF_F16) return FF_ERR_ARG;
  if (w->C < 1 || w->F < 1 || w->heads < 1) return FF_ERR_ARG;
  if (!w->ln1_g || !w->ln1_b || !w->w_qkv || !w->b_qkv || !w->w_o || !w->b_o || !w->ln2_g || !w->ln2_b ||
      !w->w1 || !w->b1 || !w->w2 || !w->b2)
    return FF_ERR_ARG;
  if (w->C % w->heads) return FF_ERR_UNSUPPORTED;
  if (((size_t)w->C * (dtype == FF_F32 ? 4 : 2)) % 16) return FF_ERR_UNSUPPORTED;
  return FF_OK;
}

size_t elem_size(int dtype) { return dtype == FF_F32 ? 4 : 2; }
// Do the byte ranges [a, a + an) and [b, b + bn) share a byte?  (Empty ranges and null pointers never do.)
bool overlaps(const void* a, size_t an, const void* b, size_t bn) {
  if (!a || !b || an == 0 || bn == 0) return false;
  const uintptr_t x = (uintptr_t)a, y = (uintptr_t)b;
  return x < y + bn && y < x + an;
}
bool is_16bit(int dtype) { return dtype == FF_BF16 || dtype == FF_F16; }  // the types with a fused matrix-core kernel

}  // namespace

extern "C" {

size_t ff_flatten_workspace_bytes(int64_t n, const ff_geom* g) { return flatten_workspace_bytes(n, g, 1); }

int ff_flatten(const int32_t* coords, int64_t n, const ff_geom* g, int axis, int shift, int G, int tail,
               int32_t* perm, int32_t* group_offsets, int32_t* num_groups, uint64_t* keys_sorted,
               void* workspace, size_t workspace_bytes, void* stream) {
  if (tail != FF_TAIL_MASK && tail != FF_TAIL_DROP) return FF_ERR_ARG;
  if (shift != 0 && shift != 1) return FF_ERR_ARG;
  return flatten_launch(coords, n, g, 1, &axis, &shift, G, tail == FF_TAIL_DROP, &perm, nullptr, &group_offsets, &num_groups, &keys_sorted,
                        workspace, workspace_bytes, nullptr, (hipStream_t)stream);
}

int ff_check_coords(const int32_t* coords, int64_t n, const ff_geom* g, int32_t* result, void* stream) {
  return check_coords_launch(coords, n, g, result, (hipStream_t)stream);
}

size_t ff_flatten_batch_workspace_bytes(int64_t n, const ff_geom* g, int num_sorts) {
  return flatten_workspace_bytes(n, g, num_sorts);
}

int ff_flatten_batch(const int32_t* coords, int64_t n, const ff_geom* g, int num_sorts, const int* axis,
                     const int* shift, int G, int tail, int32_t* const* perm, int32_t* const* group_offsets,
                     int32_t* const* num_groups, void* workspace, size_t workspace_bytes, void* stream) {
  if (tail != FF_TAIL_MASK && tail != FF_TAIL_DROP) return FF_ERR_ARG;
  if (num_sorts < 1 || num_sorts > 4 || !axis || !shift || !perm || !group_offsets || !num_groups) return FF_ERR_ARG;
  for (int s = 0; s < num_sorts; ++s)
    if (shift[s] != 0 && shift[s] != 1) return FF_ERR_ARG;
  return flatten_launch(coords, n, g, num_sorts, axis, shift, G, tail == FF_TAIL_DROP, perm, nullptr, group_offsets,
                        num_groups, nullptr, workspace, workspace_bytes, nullptr, (hipStream_t)stream);
}

// ---- ff_flatten for callers that cannot allocate ----------------------------------------------------------
// The sort's scratch (two word buffers, digit tables, frame table) lives in this array instead of a caller's
// workspace.  Every device the library runs on holds its own copy, at its own address, until the process
// ends; host code never uses the array's name as an address, only what hipGetSymbolAddress returned for the
// current device.
static __device__ __align__(256) unsigned char scratch[FF_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
static std::atomic<void*> scratch_ptr[kMaxDevices];  // per device: address of `scratch` there (nullptr: not asked yet)

static int scratch_on_current_device(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return FF_ERR_LAUNCH;
  void* p = scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return FF_ERR_LAUNCH;
    scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return FF_OK;
}
}  // namespace

int ff_flatten_noalloc(const int32_t* coords, int64_t n, const ff_geom* g, int axis, int shift, int G, int tail,
                       int32_t* perm, int32_t* group_offsets, int32_t* num_groups, uint64_t* keys_sorted,
                       void* stream) {
  const size_t need = flatten_workspace_bytes(n, g, 1);
  if (need == 0) {  // the geometry or n is invalid: report it the way ff_flatten does
    FlattenPlan fp;
    const int st = make_flatten_plan(n, g, axis == 1 ? 1 : 0, 1, &fp);
    return st != FF_OK ? st : FF_ERR_ARG;
  }
  if (need > (size_t)FF_NOALLOC_SCRATCH_BYTES) return FF_ERR_UNSUPPORTED;  // the cloud is too large for the array
  void* ws = nullptr;
  const int st = scratch_on_current_device(&ws);
  if (st != FF_OK) return st;
  return ff_flatten(coords, n, g, axis, shift, G, tail, perm, group_offsets, num_groups, keys_sorted, ws,
                    (size_t)FF_NOALLOC_SCRATCH_BYTES, stream);
}

namespace {
static int split_geom3(const ff_geom3* g, ff_geom* g2, FlattenZ* z) {
  if (!g) return FF_ERR_ARG;
  g2->num_frames = g->num_frames; g2->grid_x = g->grid_x; g2->grid_y = g->grid_y;
  g2->win_x = g->win_x; g2->win_y = g->win_y;
  z->grid_z = g->grid_z; z->win_z = g->win_z;
  return FF_OK;
}
}  // namespace

size_t ff_flatten3d_workspace_bytes(int64_t n, const ff_geom3* g) {
  ff_geom g2;
  FlattenZ z;
  if (split_geom3(g, &g2, &z) != FF_OK) return 0;
  return flatten_workspace_bytes_z(n, &g2, &z, 1);
}

int ff_flatten3d(const int32_t* coords, int64_t n, const ff_geom3* g, int axis, int shift, int G, int tail,
                 int32_t* perm, int32_t* group_offsets, int32_t* num_groups, void* workspace, size_t workspace_bytes,
                 void* stream) {
  ff_geom g2;
  FlattenZ z;
  if (split_geom3(g, &g2, &z) != FF_OK) return FF_ERR_ARG;
  if (tail != FF_TAIL_MASK && tail != FF_TAIL_DROP) return FF_ERR_ARG;
  if (shift != 0 && shift != 1) return FF_ERR_ARG;
  return flatten_launch_z(coords, n, &g2, &z, 1, &axis, &shift, G, tail == FF_TAIL_DROP, &perm, nullptr, &group_offsets,
                          &num_groups, nullptr, workspace, workspace_bytes, nullptr, (hipStream_t)stream);
}

size_t ff_pack_weights_bytes(const ff_layer_weights* w, int dtype) {
  if (check_weights(w, dtype) != FF_OK || !is_16bit(dtype)) return 0;
  if (!layer_mfma_supported(w, 1)) return 0;
  return layer_mfma_packed_bytes(w);
}

int ff_pack_weights(const ff_layer_weights* w, int dtype, void* packed, void* stream) {
  int st = check_weights(w, dtype);
  if (st != FF_OK) return st;
  if (!is_16bit(dtype) || !layer_mfma_supported(w, 1)) return FF_ERR_UNSUPPORTED;
  if (!packed || ((uintptr_t)packed & 255)) return FF_ERR_ARG;
  return dtype == FF_F16 ? layer_mfma_pack_f16(w, 1, packed, 0, (hipStream_t)stream)
                         : layer_mfma_pack(w, 1, packed, 0, (hipStream_t)stream);
}

size_t ff_group_attention_workspace_bytes(int64_t n, int G, const ff_layer_weights* w, int dtype) {
  if (n < 0 || check_weights(w, dtype) != FF_OK) return 0;
  // Sized for either path so that a flag can switch kernels without a new query.
  size_t b = layer_generic_workspace_bytes(n, w);
  if (is_16bit(dtype) && layer_mfma_supported(w, G)) {
    const size_t p = align_up(layer_mfma_packed_bytes(w), 256);
    if (p > b) b = p;
  }
  return b;
}

}  // extern "C"

namespace {
// Does this call run on the fused matrix-core kernel?
bool takes_fused_path(const ff_layer_weights* w, int G, int dtype, uint32_t flags) {
  return is_16bit(dtype) && !(flags & FF_FLAG_FORCE_GENERIC) && layer_mfma_supported(w, G);
}

// ff_group_attention plus the two internal options of the fused kernel that ff_fwa_block uses to hand
// features from layer to layer in sorted order (see layer_mfma_launch); they need the fused path.
int group_attention(const void* feats, void* out, int64_t n, const int32_t* perm,
                    const int32_t* group_offsets, const int32_t* num_groups, int32_t max_groups,
                    const ff_layer_weights* w, int G, int dtype, uint32_t flags, void* workspace,
                    size_t workspace_bytes, const int32_t* out_index, int in_sorted, void* stream) {
  int st = check_weights(w, dtype);
  if (st != FF_OK) return st;
  if (n < 0 || n > 0x7fffffffLL || max_groups < 0 || G < 1) return FF_ERR_ARG;
  if (G > 1024) return FF_ERR_UNSUPPORTED;
  if (n > 0 && (!feats || !out || !perm || !group_offsets || !num_groups)) return FF_ERR_ARG;
  if ((uintptr_t)w->pos_embed & 15) return FF_ERR_ARG;
  if (n > 0) {  // the two [n, C] buffers must not share a byte, nor may either reach into the workspace
    const size_t in_bytes = (size_t)n * w->C * elem_size(dtype);
    const size_t out_bytes = (size_t)n * w->C * ((flags & FF_FLAG_OUT_F32) ? 4 : elem_size(dtype));
    if (overlaps(feats, in_bytes, out, out_bytes)) return FF_ERR_ARG;
    if (overlaps(workspace, workspace_bytes, feats, in_bytes) || overlaps(workspace, workspace_bytes, out, out_bytes))
      return FF_ERR_ARG;
  }
  const bool out_f32 = (flags & FF_FLAG_OUT_F32) != 0;
  const bool drop = (flags & FF_FLAG_TAIL_DROP) != 0;
  if (drop && n > 0 && max_groups == 0)  // no group can exist: every row skips the layer
    return rows_copy_ungrouped_launch(feats, out, n, perm, group_offsets, num_groups, 0, w->C, G, dtype, out_f32,
                                      (hipStream_t)stream);
  if (takes_fused_path(w, G, dtype, flags)) {
    if (n == 0 || max_groups == 0) return FF_OK;
    const void* packed = w->packed;
    if (!packed) {
      if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < layer_mfma_packed_bytes(w))
        return FF_ERR_WORKSPACE;
      st = dtype == FF_F16 ? layer_mfma_pack_f16(w, 1, workspace, 0, (hipStream_t)stream)
                           : layer_mfma_pack(w, 1, workspace, 0, (hipStream_t)stream);
      if (st != FF_OK) return st;
      packed = workspace;
    }
    const int variant = (int)((flags >> 8) & 0xf);
    if (dtype == FF_F16)
      return layer_mfma_launch_f16(feats, out, n, perm, group_offsets, num_groups, max_groups, w, G, out_f32, drop,
                                   packed, variant, out_index, in_sorted, (hipStream_t)stream);
    return layer_mfma_launch(feats, out, n, perm, group_offsets, num_groups, max_groups, w, G, out_f32, drop,
                             packed, variant, out_index, in_sorted, (hipStream_t)stream);
  }
  if (out_index || in_sorted) return FF_ERR_UNSUPPORTED;  // only the fused kernel has these
  st = layer_generic_launch(feats, out, n, perm, group_offsets, num_groups, max_groups, w, G, dtype, out_f32,
                            workspace, workspace_bytes, (hipStream_t)stream);
  if (st != FF_OK || !drop || n == 0) return st;
  // The row kernels above wrote every row; the rows of no group get the input back.
  return rows_copy_ungrouped_launch(feats, out, n, perm, group_offsets, num_groups, max_groups, w->C, G, dtype,
                                    out_f32, (hipStream_t)stream);
}
}  // namespace

extern "C" {

int ff_group_attention(const void* feats, void* out, int64_t n, const int32_t* perm,
                       const int32_t* group_offsets, const int32_t* num_groups, int32_t max_groups,
                       const ff_layer_weights* w, int G, int dtype, uint32_t flags,
                       void* workspace, size_t workspace_bytes, void* stream) {
  return group_attention(feats, out, n, perm, group_offsets, num_groups, max_groups, w, G, dtype, flags, workspace,
                         workspace_bytes, nullptr, 0, stream);
}

int ff_group_attention_path(const ff_layer_weights* w, int G, int dtype, uint32_t flags) {
  const int st = check_weights(w, dtype);
  if (st != FF_OK) return st;
  if (G < 1) return FF_ERR_ARG;
  if (G > 1024) return FF_ERR_UNSUPPORTED;
  return takes_fused_path(w, G, dtype, flags) ? FF_PATH_FUSED : FF_PATH_PLAIN;
}

int ff_gather(const void* src, void* dst, const int32_t* perm, int64_t n, int C, int dtype, void* stream) {
  return rows_launch(false, src, dst, perm, n, C, dtype, (hipStream_t)stream);
}

int ff_scatter(const void* src, void* dst, const int32_t* perm, int64_t n, int C, int dtype, void* stream) {
  return rows_launch(true, src, dst, perm, n, C, dtype, (hipStream_t)stream);
}

size_t ff_voxelize_workspace_bytes(int64_t m, const ff_geom* g) { return voxelize_workspace_bytes(m, g); }

int ff_voxelize(const float* xy, const int32_t* frame, const float* point_feats, int64_t m, int Cp, const ff_geom* g,
                const ff_voxel_grid* v, int32_t* coords, float* feats, int32_t* num_pillars, int32_t* point_to_pillar,
                void* workspace, size_t workspace_bytes, void* stream) {
  return voxelize_launch(xy, frame, point_feats, m, Cp, g, v, coords, feats, num_pillars, point_to_pillar, workspace,
                         workspace_bytes, (hipStream_t)stream);
}

int ff_bev_scatter(const void* feats, const int32_t* coords, int64_t n, const ff_geom* g, int C, int dtype, void* bev,
                   void* stream) {
  return bev_scatter_launch(feats, coords, n, g, C, dtype, bev, (hipStream_t)stream);
}

// Workspace layout of ff_fwa_block:
//   [flatten scratch][perm x S][inverse perm x S][group_offsets x S][num_groups x S][feature buffer A]
//   [feature buffer B][layer scratch][packed weights]
// with S = number of distinct (axis, shift) pairs the schedule uses (at most 4).
// When every layer runs on the fused kernel the features travel from layer to layer in sorted order:
// layer l writes row inverse_perm_{l+1}[pillar], which is where layer l+1 finds the members of its
// groups side by side, so only the first layer gathers through an index and only the last one
// writes pillar order.
namespace {
struct BlockPlan {
  int sorts;  // distinct sort configurations used by layers 0..L-1 (schedule order x, y, sx, sy)
  int64_t max_groups;
  size_t off_flat, off_perm, off_inv, off_goff, off_ng, off_a, off_b, off_layer, off_packed, total;
  bool chain;  // features are handed on in sorted order
  size_t flat_bytes, layer_bytes, packed_stride;  // packed_stride == 0: nothing to pre-pack
};

static int make_block_plan(int64_t n, const ff_geom* g, const FlattenZ* z, int G, const ff_layer_weights* layers,
                    int num_layers, int dtype, BlockPlan* p) {
  if (n < 0 || n > 0x7fffffffLL || !g || G < 1 || num_layers < 1 || !layers) return FF_ERR_ARG;
  for (int l = 0; l < num_layers; ++l) {
    int st = check_weights(&layers[l], dtype);
    if (st != FF_OK) return st;
    if (layers[l].C != layers[0].C) return FF_ERR_ARG;
  }
  p->sorts = num_layers < 4 ? num_layers : 4;
  p->flat_bytes = flatten_workspace_bytes_z(n, g, z, p->sorts);
  if (p->flat_bytes == 0) { FlattenPlan fp; int st = make_flatten_plan_z(n, g, z, 0, 1, &fp); if (st != FF_OK) return st; }
  p->max_groups = ceil_div(n, G) + g->num_frames;
  p->layer_bytes = 0;
  for (int l = 0; l < num_layers; ++l) {
    size_t b = ff_group_attention_workspace_bytes(n, G, &layers[l], dtype);
    if (b > p->layer_bytes) p->layer_bytes = b;
  }
  const size_t feat_bytes = align_up((size_t)n * layers[0].C * elem_size(dtype), 256);
  size_t off = 0;
  p->off_flat = off;  off += align_up(p->flat_bytes, 256);
  p->off_perm = off;  off += p->sorts * align_up((size_t)n * 4, 256);
  p->chain = num_layers > 1;
  for (int l = 0; l < num_layers; ++l) p->chain = p->chain && takes_fused_path(&layers[l], G, dtype, 0);
  p->off_inv = off;   off += (p->chain ? p->sorts : 0) * align_up((size_t)n * 4, 256);
  p->off_goff = off;  off += p->sorts * align_up((size_t)(p->max_groups + 1) * 4, 256);
  p->off_ng = off;    off += 256;
  p->off_a = off;     off += feat_bytes;
  p->off_b = off;     off += feat_bytes;
  p->off_layer = off; off += align_up(p->layer_bytes, 256);
  // One batched packing launch for the whole stack when every layer has the same packable shape
  // and the caller did not pre-pack.
  p->packed_stride = 0;
  if (is_16bit(dtype) && layer_mfma_supported(&layers[0], G)) {
    bool same = true;
    for (int l = 0; l < num_layers; ++l)
      same = same && layers[l].F == layers[0].F && layers[l].heads == layers[0].heads && !layers[l].packed;
    if (same) p->packed_stride = align_up(layer_mfma_packed_bytes(&layers[0]), 256);
  }
  p->off_packed = off; off += p->packed_stride * num_layers;
  p->total = off;
  return FF_OK;
}
}  // namespace

namespace {
static int fwa_block(const int32_t* coords, int64_t n, const ff_geom* g, const FlattenZ* z, int G, int tail,
              const ff_layer_weights* layers, int num_layers, int dtype, const void* feats_in, void* feats_out,
              void* workspace, size_t workspace_bytes, void* stream) {
  if (tail != FF_TAIL_MASK && tail != FF_TAIL_DROP) return FF_ERR_ARG;
  const bool drop = tail == FF_TAIL_DROP;
  BlockPlan p;
  int st = make_block_plan(n, g, z, G, layers, num_layers, dtype, &p);
  if (st != FF_OK) return st;
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < p.total) return FF_ERR_WORKSPACE;
  if (n > 0 && (!coords || !feats_in || !feats_out)) return FF_ERR_ARG;
  {  // input, output and workspace must be three disjoint byte ranges
    const size_t fb = (size_t)n * layers[0].C * elem_size(dtype);
    if (overlaps(feats_in, fb, feats_out, fb) || overlaps(workspace, p.total, feats_in, fb) ||
        overlaps(workspace, p.total, feats_out, fb))
      return FF_ERR_ARG;
  }
  char* ws = (char*)workspace;
  const size_t perm_stride = align_up((size_t)n * 4, 256);
  const size_t goff_stride = align_up((size_t)(p.max_groups + 1) * 4, 256);
  {  // all sort configurations of the schedule in one batched flatten
    int axis[4], shift[4];
    int32_t *perm[4], *inv[4], *goff[4], *ng[4];
    for (int s = 0; s < p.sorts; ++s) {
      axis[s] = s % 2; shift[s] = (s / 2) % 2;
      perm[s] = (int32_t*)(ws + p.off_perm + s * perm_stride);
      inv[s] = (int32_t*)(ws + p.off_inv + s * perm_stride);
      goff[s] = (int32_t*)(ws + p.off_goff + s * goff_stride);
      ng[s] = (int32_t*)(ws + p.off_ng) + s;
    }
    // The layers' weights are re-tiled by extra workgroups of the first sort kernel when one launch can
    // take them all; otherwise by a launch of their own.
    PackJob job;
    const bool ride = p.packed_stride && n > 0 && num_layers <= kPackBatch;
    if (ride) make_pack_job(layers, num_layers, ws + p.off_packed, p.packed_stride, dtype == FF_F16, &job);
    st = flatten_launch_z(coords, n, g, z, p.sorts, axis, shift, G, drop, perm, p.chain ? inv : nullptr, goff, ng, nullptr,
                          ws + p.off_flat, p.flat_bytes, ride ? &job : nullptr, (hipStream_t)stream);
    if (st != FF_OK) return st;
    if (p.packed_stride && n > 0 && !ride) {
      st = dtype == FF_F16
               ? layer_mfma_pack_f16(layers, num_layers, ws + p.off_packed, p.packed_stride, (hipStream_t)stream)
               : layer_mfma_pack(layers, num_layers, ws + p.off_packed, p.packed_stride, (hipStream_t)stream);
      if (st != FF_OK) return st;
    }
  }
  const void* cur = feats_in;
  void* bufs[2] = {ws + p.off_a, ws + p.off_b};
  for (int l = 0; l < num_layers; ++l) {
    const int s = l % 4;
    void* dst = (l == num_layers - 1) ? feats_out : bufs[l & 1];
    ff_layer_weights wl = layers[l];
    if (p.packed_stride) wl.packed = ws + p.off_packed + (size_t)l * p.packed_stride;
    const bool last = l == num_layers - 1;
    const int32_t* next_inv = p.chain && !last ? (const int32_t*)(ws + p.off_inv + ((l + 1) % 4) * perm_stride) : nullptr;
    const int in_sorted = p.chain && l > 0 ? (g->num_frames == 1 ? 2 : 1) : 0;
    st = group_attention(cur, dst, n, (const int32_t*)(ws + p.off_perm + s * perm_stride),
                         (const int32_t*)(ws + p.off_goff + s * goff_stride), (const int32_t*)(ws + p.off_ng) + s,
                         (int32_t)p.max_groups, &wl, G, dtype, drop ? FF_FLAG_TAIL_DROP : 0u, ws + p.off_layer,
                         p.layer_bytes, next_inv, in_sorted, stream);
    if (st != FF_OK) return st;
    cur = dst;
  }
  return FF_OK;
}
}  // namespace

size_t ff_fwa_block_workspace_bytes(int64_t n, const ff_geom* g, int G, const ff_layer_weights* layers,
                                    int num_layers, int dtype) {
  BlockPlan p;
  if (make_block_plan(n, g, nullptr, G, layers, num_layers, dtype, &p) != FF_OK) return 0;
  return p.total;
}

int ff_fwa_block(const int32_t* coords, int64_t n, const ff_geom* g, int G, int tail,
                 const ff_layer_weights* layers, int num_layers, int dtype, const void* feats_in, void* feats_out,
                 void* workspace, size_t workspace_bytes, void* stream) {
  return fwa_block(coords, n, g, nullptr, G, tail, layers, num_layers, dtype, feats_in, feats_out, workspace,
                   workspace_bytes, stream);
}

size_t ff_fwa_block3d_workspace_bytes(int64_t n, const ff_geom3* g, int G, const ff_layer_weights* layers,
                                      int num_layers, int dtype) {
  ff_geom g2;
  FlattenZ z;
  BlockPlan p;
  if (split_geom3(g, &g2, &z) != FF_OK) return 0;
  if (make_block_plan(n, &g2, &z, G, layers, num_layers, dtype, &p) != FF_OK) return 0;
  return p.total;
}

int ff_fwa_block3d(const int32_t* coords, int64_t n, const ff_geom3* g, int G, int tail,
                   const ff_layer_weights* layers, int num_layers, int dtype, const void* feats_in, void* feats_out,
                   void* workspace, size_t workspace_bytes, void* stream) {
  ff_geom g2;
  FlattenZ z;
  if (split_geom3(g, &g2, &z) != FF_OK) return FF_ERR_ARG;
  return fwa_block(coords, n, &g2, &z, G, tail, layers, num_layers, dtype, feats_in, feats_out, workspace,
                   workspace_bytes, stream);
}

const char* ff_status_string(int status) {
  switch (status) {
    case FF_OK: return "ok";
    case FF_ERR_ARG: return "invalid argument";
    case FF_ERR_UNSUPPORTED: return "unsupported configuration";
    case FF_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case FF_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

int ff_version(void) { return 100; }

}  // extern "C"
