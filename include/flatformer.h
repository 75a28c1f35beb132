/*
 * flatformer.h -- C ABI of the MI355X (gfx950) Flattened Window Attention library.
 *
 * The library implements the hot path of FlatFormer's Flattened Window Attention
 * (paper Sec. 4.2): window-based sorting of sparse BEV pillars, equal-size
 * grouping of the sorted order, and a pre-LayerNorm transformer layer applied
 * independently inside every group.
 *
 * Conventions shared by every entry point
 *  - Pointers are DEVICE pointers unless the parameter is a struct passed by the
 *    host (ff_geom, ff_layer_weights: host structs whose pointer members are
 *    device pointers).  `stream` is a hipStream_t passed as void* (NULL = the
 *    default stream).
 *  - Ownership: the caller allocates and owns every buffer, including the
 *    workspace.  The library never allocates or frees device memory and never
 *    synchronises the stream; outputs are valid once the stream reaches the
 *    point after the call.  Every entry point can therefore be captured into a
 *    HIP graph; call it once outside a capture first (the first launch of a
 *    fused layer kernel on a device sets a function attribute).
 *  - Errors: every function returns an ff_status (0 = success, negative =
 *    failure).  Preconditions that can be checked on the host are checked before
 *    anything is launched; on FF_ERR_ARG / FF_ERR_UNSUPPORTED / FF_ERR_WORKSPACE
 *    nothing has been written.  The library never throws and never aborts.
 *  - Row-major everywhere.  Linear layers follow y = x * W^T + b with W stored
 *    [out_features, in_features].
 */
#ifndef FLATFORMER_H
#define FLATFORMER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FF_OK = 0,
  FF_ERR_ARG = -1,         /* null pointer, negative size, inconsistent shape   */
  FF_ERR_UNSUPPORTED = -2, /* valid request outside the built kernels' limits   */
  FF_ERR_WORKSPACE = -3,   /* workspace missing, misaligned or too small        */
  FF_ERR_LAUNCH = -4       /* the HIP runtime refused a launch                  */
} ff_status;

typedef enum { FF_F32 = 0, FF_BF16 = 1, FF_F16 = 2 /* IEEE half, the paper's inference precision */ } ff_dtype;

typedef enum {
  FF_TAIL_MASK = 0, /* a frame's last group may be short; it attends over its real members only */
  FF_TAIL_DROP = 1  /* short groups are left out of the list ('Drop Residual', Sec. 4.3): every   */
                    /* listed group has exactly G members, the others' pillars skip the layer    */
} ff_tail;

/* Geometry of the BEV grid.  coords[:,0] in [0,num_frames), coords[:,1] in
 * [0,grid_x), coords[:,2] in [0,grid_y).  Window sizes 1..256.  Limits:
 * num_frames <= 65535 and at most 65535 windows per axis (the exported key has
 * 16-bit frame and window fields and 8-bit in-window fields). */
typedef struct {
  int32_t num_frames;
  int32_t grid_x, grid_y;
  int32_t win_x, win_y;
} ff_geom;

/* ---- window-based sorting + equal-size grouping (Sec. 4.2.1, Eq. (1)) -------------------
 *
 * For pillar i with (b, x, y):  X = x + sx, Y = y + sy, where (sx, sy) = (win_x/2, win_y/2)
 * rounded down when `shift` is set (Sec. 4.2.2 'Window Shift') and (0,0) otherwise;
 * (Wx, Lx) = divmod(X, win_x), (Wy, Ly) = divmod(Y, win_y).  The sort tuple is
 * (b, Wx, Wy, Lx, Ly) for axis 0 and (b, Wy, Wx, Ly, Lx) for axis 1 ('Alternate Sorting
 * Axis'); equal tuples keep ascending original index.  The exported key packs the tuple as
 * b<<48 | t1<<32 | t2<<16 | t3<<8 | t4.
 *
 *   perm[p]          original index of the pillar at sorted position p            [n]
 *   group_offsets    start of every group in the sorted order, then n             [>= ceil(n/G)+num_frames+1]
 *                    (only the first *num_groups + 1 entries are written)
 *   num_groups       number of groups = sum over frames of ceil(n_b / G)          [1]
 *                    (FF_TAIL_DROP: of floor(n_b / G))
 *   keys_sorted      exported key of every sorted position, or NULL               [n]
 *
 * Groups never cross frames; within a frame they are consecutive runs of G sorted pillars,
 * the last one possibly shorter ('Equal-Size Grouping').  With FF_TAIL_DROP that shorter group
 * is not listed: group_offsets holds the starts of the full groups only, then n, so that group g
 * is positions group_offsets[g] .. group_offsets[g]+G-1 and group_offsets[g+1] may lie beyond its
 * end.  n == 0 is legal (num_groups = 0, group_offsets[0] = 0).  Duplicate coordinates are legal.  Coordinates outside the geometry
 * give an unspecified (but still bijective) perm; no memory outside the buffers is touched.
 *
 * Limit: bits(key fields actually used) + bits(n-1) must not exceed 64 (FF_ERR_UNSUPPORTED
 * otherwise); every configuration with n < 2^24 and fewer than 2^40 cells satisfies it.
 * workspace: ff_flatten_workspace_bytes(n, g) bytes, 256-byte aligned.
 */
size_t ff_flatten_workspace_bytes(int64_t n, const ff_geom* g);

int ff_flatten(const int32_t* coords /* [n,3] (b,x,y) */, int64_t n, const ff_geom* g,
               int axis /* 0: x-major, 1: y-major */, int shift /* 0 | 1 */,
               int G, int tail /* ff_tail */,
               int32_t* perm, int32_t* group_offsets, int32_t* num_groups,
               uint64_t* keys_sorted, void* workspace, size_t workspace_bytes, void* stream);

/* ---- coordinate check (a debugging aid; the sorts never need it) ---------------------------------------------
 * ff_flatten and the blocks stay memory-safe with coordinates outside the geometry, but the order they then
 * produce is unspecified.  This call counts such rows on the device: result[0] = number of rows of coords
 * with a frame, x or y outside [0, num_frames) x [0, grid_x) x [0, grid_y), result[1] = index of the first
 * such row, n if there is none.  result: device int32 [2].  Asynchronous like every other call; the caller
 * reads the two words after synchronising the stream. */
int ff_check_coords(const int32_t* coords /* [n,3] (b,x,y) */, int64_t n, const ff_geom* g,
                    int32_t* result /* device [2] */, void* stream);

/* ---- several sort configurations of one cloud in one call ('Reuse Sorting', Sec. 4.3: the coordinates do
 * not change inside a stage, so each (axis, shift) pair is sorted once and reused by every layer and block
 * that needs it).  num_sorts (1..4) configurations axis[s], shift[s] are sorted together, one launch set for
 * all of them; perm / group_offsets / num_groups are HOST arrays of num_sorts device pointers, each as in
 * ff_flatten.  This is what ff_fwa_block runs in front of its layers; a caller that keeps the results can
 * run later blocks on the same cloud through ff_group_attention without sorting again.
 * workspace: ff_flatten_batch_workspace_bytes(n, g, num_sorts) bytes, 256-byte aligned. */
size_t ff_flatten_batch_workspace_bytes(int64_t n, const ff_geom* g, int num_sorts);

int ff_flatten_batch(const int32_t* coords /* [n,3] (b,x,y) */, int64_t n, const ff_geom* g, int num_sorts,
                     const int* axis /* host [num_sorts] */, const int* shift /* host [num_sorts] */,
                     int G, int tail /* ff_tail */,
                     int32_t* const* perm, int32_t* const* group_offsets, int32_t* const* num_groups,
                     void* workspace, size_t workspace_bytes, void* stream);

/* ---- ff_flatten without a workspace, for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops that must not call hipMalloc, harnesses that forbid it.  Arguments, outputs
 * and errors are ff_flatten's; the scratch memory of the sort is a static device array of
 * FF_NOALLOC_SCRATCH_BYTES inside the library (each GPU the library runs on holds its own copy until the
 * process ends).  The call allocates and frees nothing and does not synchronise.
 *  - Limit: ff_flatten_workspace_bytes(n, g) must not exceed FF_NOALLOC_SCRATCH_BYTES, else
 *    FF_ERR_UNSUPPORTED and nothing is written (a 468 x 468 grid with 13 x 13 windows fits up to
 *    about 400,000 pillars).
 *  - Every call on a GPU uses that GPU's one array: calls that overlap in time on the same GPU (two
 *    streams, two threads) race with each other; serialise them.  Nothing in the array has to be cleared
 *    between calls, and nothing of a call is kept in it afterwards.
 *  - The first call on a device looks up the array's address there (hipGetSymbolAddress); make that call
 *    outside a graph capture. */
#define FF_NOALLOC_SCRATCH_BYTES (8u << 20)

int ff_flatten_noalloc(const int32_t* coords /* [n,3] (b,x,y) */, int64_t n, const ff_geom* g,
                       int axis, int shift, int G, int tail /* ff_tail */,
                       int32_t* perm, int32_t* group_offsets, int32_t* num_groups,
                       uint64_t* keys_sorted /* or NULL */, void* stream);

/* ---- the same for three-dimensional windows (footnote of Sec. 4.2.1: the method applies to 3-D point
 * clouds; no configuration of the paper uses it) -----------------------------------------------------
 * coords [n,4] = (b, x, y, z) voxel indices.  The shift is half a window on all three axes.  The
 * sort tuple keeps the two-axis alternation of the pillar case and appends z to both halves:
 * (b, Wx, Wy, Wz, Lx, Ly, Lz) for axis 0 and (b, Wy, Wx, Wz, Ly, Lx, Lz) for axis 1.  Outputs, tail
 * modes, limits (the seven fields' live bits plus bits(n-1) must fit 64 bits; windows 1..256; at
 * most 65535 windows per axis) and workspace rules are those of ff_flatten; there is no exported
 * key (seven fields do not fit its format). */
typedef struct {
  int32_t num_frames;
  int32_t grid_x, grid_y, grid_z;
  int32_t win_x, win_y, win_z;
} ff_geom3;

size_t ff_flatten3d_workspace_bytes(int64_t n, const ff_geom3* g);

int ff_flatten3d(const int32_t* coords /* [n,4] (b,x,y,z) */, int64_t n, const ff_geom3* g,
                 int axis /* 0 | 1 */, int shift /* 0 | 1 */, int G, int tail /* ff_tail */,
                 int32_t* perm, int32_t* group_offsets, int32_t* num_groups,
                 void* workspace, size_t workspace_bytes, void* stream);

/* ---- group attention layer (Sec. 4.2.2, Eq. (2)) --------------------------------------------
 *
 *   F'  = F  + MHSA(LN1(F))      softmax(Q K^T / sqrt(d)) V per head, inside each group
 *   F'' = F' + FFN(LN2(F'))      FFN = Linear(C->F) -> GELU(erf form) -> Linear(F->C)
 *
 * All parameter arrays have the element type `dtype` of the call.  LayerNorm uses the
 * biased variance and ln_eps.  w_qkv rows [0,C) are the query projection, [C,2C) key,
 * [2C,3C) value; head h owns rows h*d..(h+1)*d-1 of each third, d = C / heads.
 *
 * PE(C), the second argument of MHSA in Eq. (2), is a global absolute positional embedding the
 * paper gives no formula for.  It enters as pos_embed: NULL, or a device array [n, C] of the
 * call's dtype in pillar order (row i belongs to pillar i, like feats), computed by the caller.
 * When given, queries and keys are projected from LN(F) + PE and values from LN(F).
 */
typedef struct {
  const void *ln1_g, *ln1_b; /* [C]            */
  const void *w_qkv, *b_qkv; /* [3C, C], [3C]  */
  const void *w_o, *b_o;     /* [C, C],  [C]   */
  const void *ln2_g, *ln2_b; /* [C]            */
  const void *w1, *b1;       /* [F, C],  [F]   */
  const void *w2, *b2;       /* [C, F],  [C]   */
  int32_t C, F, heads;
  float ln_eps;
  const void* packed;        /* NULL, or the buffer written by ff_pack_weights for THESE weights */
  const void* pos_embed;     /* NULL, or [n, C] per-call input (see above); not a weight, never packed */
} ff_layer_weights;

/* Weight pre-packing for the matrix-core kernels (optional).  The fused bf16 kernel reads the
 * four weight matrices in a tile order of its own.  With packed == NULL, ff_group_attention and
 * ff_fwa_block re-pack the weights into their workspace on every call (one small extra launch
 * per layer).  Weights that stay fixed across calls can be packed once: allocate
 * ff_pack_weights_bytes(w, dtype) bytes (256-byte aligned), call ff_pack_weights, and store the
 * pointer in w->packed.  ff_pack_weights_bytes returns 0 when the configuration has no packed
 * form (fp32, or a shape only the plain kernels cover); `packed` is then ignored.  A packed
 * buffer is specific to the dtype it was packed for. */
size_t ff_pack_weights_bytes(const ff_layer_weights* w, int dtype);
int ff_pack_weights(const ff_layer_weights* w, int dtype, void* packed, void* stream);

/* Flags of ff_group_attention. */
#define FF_FLAG_OUT_F32 1u      /* store `out` as float32 even when dtype is a 16-bit type */
#define FF_FLAG_FORCE_GENERIC 2u /* use the plain fp32-arithmetic kernels for any dtype */
#define FF_FLAG_TAIL_DROP 4u     /* the group list was made with FF_TAIL_DROP: rows of no group are copied through */
/* Tuning knob: bits 8..11 select one wave-to-group mapping of the fused bf16 kernel (1..15; 0 =
 * chosen from the shape).  A mapping that cannot hold G returns FF_ERR_UNSUPPORTED. */
#define FF_FLAG_VARIANT(v) (((uint32_t)(v) & 0xfu) << 8)

size_t ff_group_attention_workspace_bytes(int64_t n, int G, const ff_layer_weights* w, int dtype);

/* feats [n,C] and out [n,C] are in pillar order and must not overlap: a group reads rows that
 * other groups write.  Row perm[p] of feats is member p of the sorted order; group g owns
 * sorted positions group_offsets[g] .. min(group_offsets[g+1], group_offsets[g]+G)-1 (1..G of
 * them; the clamp only matters for a list made with FF_TAIL_DROP).  num_groups is the
 * device scalar written by ff_flatten; max_groups is a host upper bound used to size the launch
 * (e.g. ceil(n/G) + num_frames - 1) and group_offsets must hold at least max_groups + 1 readable
 * entries (ff_flatten's buffer does for that bound).  num_groups < 0 (a failed flatten) computes
 * nothing.  Every row that belongs to a group is written exactly once.  Rows of sorted positions
 * that no group covers are left untouched in `out`, unless FF_FLAG_TAIL_DROP is set: then each
 * such row of `out` receives the row of `feats` (converted when the storage types differ), which
 * is what skipping the layer means for a residual layer; max_groups may then be as small as
 * floor(n/G), and 0 copies everything.
 * dtype FF_F32: fp32 arithmetic throughout.  FF_BF16 / FF_F16: 16-bit storage, matrix-core operands
 * of that type, fp32 accumulation, statistics, softmax and GELU.
 * Limits (FF_ERR_UNSUPPORTED otherwise): C % heads == 0, C*sizeof(dtype) % 16 == 0, 1 <= G <= 1024. */
int ff_group_attention(const void* feats, void* out, int64_t n,
                       const int32_t* perm, const int32_t* group_offsets,
                       const int32_t* num_groups, int32_t max_groups,
                       const ff_layer_weights* w, int G, int dtype, uint32_t flags,
                       void* workspace, size_t workspace_bytes, void* stream);

/* Which kernels a call of ff_group_attention with these weights, group size, dtype and flags would run
 * (host-side, launches nothing): FF_PATH_FUSED, the single matrix-core kernel (16-bit dtypes; shapes
 * (C, head dim, F) = (128, 16, 256), (256, 32, 512) and (64, 16, 128) with G <= 128), or FF_PATH_PLAIN, the
 * three fp32-arithmetic kernels that serve every other shape, FF_F32 and FF_FLAG_FORCE_GENERIC, at a
 * fraction of the speed.  A negative value is the ff_status the call itself would return for these arguments. */
#define FF_PATH_PLAIN 0
#define FF_PATH_FUSED 1
int ff_group_attention_path(const ff_layer_weights* w, int G, int dtype, uint32_t flags);

/* ---- row gather / scatter (the 'reshape' of Sec. 4.2.1 made explicit) ---------------------------
 * gather:  dst[p, :] = src[perm[p], :]     scatter:  dst[perm[p], :] = src[p, :]
 * C * sizeof(dtype) must be a multiple of 16; src and dst must not overlap. */
int ff_gather(const void* src, void* dst, const int32_t* perm, int64_t n, int C, int dtype, void* stream);
int ff_scatter(const void* src, void* dst, const int32_t* perm, int64_t n, int C, int dtype, void* stream);

/* ---- pillar voxelisation (the step in front of the FWA blocks: Sec. 5.1 'Model' voxelises the point
 * cloud into sparse bird's-eye-view pillars of 0.32 m x 0.32 m, following PointPillars) -------------
 * Point i lies in cell ( floor((x_i - x_min) / voxel_x), floor((y_i - y_min) / voxel_y) ) of frame
 * frame[i] (float32 arithmetic); points outside the grid or with a frame id outside [0, num_frames)
 * are dropped.  A pillar is a non-empty cell.  Outputs, pillars in ascending (frame, x, y) order:
 *   coords           (b, x, y) of every pillar                                  [capacity m][3]
 *   feats            mean of the pillar's points' feature vectors, float32      [capacity m][Cp]
 *                    (float32 sums in a fixed order: the result does not depend on timing)
 *   num_pillars      device scalar                                              [1]
 *   point_to_pillar  NULL, or for every point its pillar, -1 if dropped         [m]
 * Only the first *num_pillars rows of coords and feats are written.  The learned per-point network
 * that PointPillars applies before pooling is not part of this entry point.  The window sizes of g
 * are ignored; num_frames <= 65534, grid_x, grid_y <= 65535.
 * workspace: ff_voxelize_workspace_bytes(m, g) bytes, 256-byte aligned. */
typedef struct {
  float x_min, y_min;     /* lower corner of cell (0, 0), metres   */
  float voxel_x, voxel_y; /* cell size, metres (> 0)                */
} ff_voxel_grid;

size_t ff_voxelize_workspace_bytes(int64_t m, const ff_geom* g);

int ff_voxelize(const float* xy /* [m,2] */, const int32_t* frame /* [m], or NULL: all frame 0 */,
                const float* point_feats /* [m,Cp] */, int64_t m, int Cp,
                const ff_geom* g, const ff_voxel_grid* v,
                int32_t* coords, float* feats, int32_t* num_pillars, int32_t* point_to_pillar,
                void* workspace, size_t workspace_bytes, void* stream);

/* ---- sparse pillars -> dense bird's-eye-view map (the step after the FWA blocks: Sec. 5.1 'Model'
 * hands the pillar features to a regular BEV encoder, which wants a dense map) ---------------------
 * bev[b][y][x][c] = feats[i][c] for pillar i with coords (b, x, y), zero in every other cell.
 * bev: device array [num_frames][grid_y][grid_x][C] of `dtype`, channels last (a pillar's C features
 * stay contiguous; 16-byte aligned), written completely.  C * sizeof(dtype) must be a multiple of 16.
 * Coordinates must be unique (what pillar voxelisation produces); with duplicates one of the rows wins,
 * which one is unspecified.  Pillars outside the geometry are skipped. */
int ff_bev_scatter(const void* feats /* [n,C] */, const int32_t* coords /* [n,3] (b,x,y) */, int64_t n,
                   const ff_geom* g, int C, int dtype, void* bev, void* stream);

/* ---- the whole block: sorts computed once and reused, then the layer stack ------------------
 * Layer l sorts along axis l % 2 with the shift on when (l / 2) % 2 == 1 (x, y, shifted x,
 * shifted y, x, ...); each distinct (axis, shift) pair is flattened once and reused by every
 * layer that needs it ('Reuse Sorting', Sec. 4.3).  layers: host array of num_layers structs.
 * tail (ff_tail) is handed to the sorts; with FF_TAIL_DROP the pillars of a layer's short groups
 * skip that layer (they can still be grouped by another layer's sort).
 * feats_in / feats_out: [n, C] in pillar order, must not overlap. */
size_t ff_fwa_block_workspace_bytes(int64_t n, const ff_geom* g, int G,
                                    const ff_layer_weights* layers, int num_layers, int dtype);

int ff_fwa_block(const int32_t* coords, int64_t n, const ff_geom* g, int G, int tail,
                 const ff_layer_weights* layers, int num_layers, int dtype,
                 const void* feats_in, void* feats_out,
                 void* workspace, size_t workspace_bytes, void* stream);

/* The block over voxels with a third coordinate (footnote of Sec. 4.2.1): ff_fwa_block with the sorts
 * of ff_flatten3d.  coords [n,4] = (b, x, y, z); everything else as above. */
size_t ff_fwa_block3d_workspace_bytes(int64_t n, const ff_geom3* g, int G,
                                      const ff_layer_weights* layers, int num_layers, int dtype);

int ff_fwa_block3d(const int32_t* coords, int64_t n, const ff_geom3* g, int G, int tail,
                   const ff_layer_weights* layers, int num_layers, int dtype,
                   const void* feats_in, void* feats_out,
                   void* workspace, size_t workspace_bytes, void* stream);

const char* ff_status_string(int status);
int ff_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FLATFORMER_H */
