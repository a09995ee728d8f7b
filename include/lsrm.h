/*
 * lsrm.h -- C boundary of the MI355X (gfx950) native-sparse-attention layer with
 * 3D-aware block routing.
 *
 * One layer call works on a joint sequence of N = n_obj + n_views * grid^2 tokens:
 * first the object (volume) tokens, then the image-patch tokens of view 0, 1, ...
 * Tokens are grouped in blocks of 64 consecutive tokens (block id = token / 64):
 * object blocks are spatially coherent runs (the caller orders object tokens, e.g.
 * along a Morton curve), image blocks are 8x8 patch tiles, tile-major inside a view
 * (tile grid row-major, patches row-major inside a tile).  [Sec. 3.2, "Block
 * Partitioning and Compression": 8x8 image blocks, spatial volume blocks.]
 *
 * Conventions for every entry point
 *   - pointers named d_* are DEVICE pointers owned by the caller; everything else
 *     (params, seg_offsets) is HOST memory read during the call;
 *   - tensors are dense row-major with the shapes given; bf16 is the 16-bit
 *     brain-float bit pattern (uint16_t here);
 *   - work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default
 *     stream) and the call returns without synchronising; a call enqueues kernel launches only (no memset or
 *     copy nodes, and event records only where the caller passes events), so calls may be recorded into a HIP
 *     graph (lsrm_route_blocks_static: after its first call on the device);
 *   - no global state apart from lsrm_route_blocks_static's address lookup; calls may come from any
 *     thread and any device may be current;
 *   - the library allocates no device memory: scratch comes from the caller
 *     (d_ws / ws_bytes, size from lsrm_workspace_bytes, 256-byte aligned), except in
 *     lsrm_route_blocks_static, which uses a fixed array inside the library;
 *   - nothing throws or aborts: the return value is LSRM_OK or a negative code,
 *     and on error no kernel has been launched.
 */
#ifndef LSRM_H
#define LSRM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t lsrm_status;
enum {
    LSRM_OK = 0,
    LSRM_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, misaligned segment, ... */
    LSRM_ERR_UNSUPPORTED = -2, /* block != 64, d not in {32,64,128}, topk > 128, ..         */
    LSRM_ERR_WORKSPACE = -3,   /* d_ws null / too small / misaligned                        */
    LSRM_ERR_HIP = -4,         /* a HIP runtime call or kernel launch failed                */
    LSRM_ERR_TOO_LARGE = -5    /* lsrm_route_blocks_static: the problem needs more than the
                                  library's fixed scratch                                   */
};

/* Human-readable text for a status code (static storage). */
const char *lsrm_strerror(lsrm_status s);

/*
 * Pinhole camera, world -> camera: x_cam = R * p + t (R row-major).  Intrinsics are
 * in PATCH units: (u, v) = (fx * x/z + cx, fy * y/z + cy) and the centre of patch
 * (row r, column c) is (c + 0.5, r + 0.5); the centre of tile (ti, tj) is
 * (8 tj + 4, 8 ti + 4).  16 floats, same order as the struct.
 */
typedef struct lsrm_camera {
    float R[9];
    float t[3];
    float fx, fy, cx, cy;
} lsrm_camera;

/*
 * Problem statement shared by all calls.  [App. A: q in R^{N x h_q x d_h},
 * k, v in R^{N x h_kv x d_h}; Sec. 3.3: routing from token coordinates + cameras.]
 */
typedef struct lsrm_nsa_params {
    int32_t n_obj;    /* object tokens, multiple of 64 (may be 0)                          */
    int32_t n_views;  /* M, number of views (may be 0)                                     */
    int32_t grid;     /* S, patches per image side, multiple of 8                          */
    int32_t block;    /* tokens per block; must be 64                                      */
    int32_t h_q;      /* query heads                                                       */
    int32_t h_kv;     /* key/value heads, a divisor of h_q: query head i reads key/value
                         head i / (h_q / h_kv) (grouped-query heads, App. A)               */
    int32_t d;        /* head dimension: 32, 64 or 128                                     */
    int32_t topk;     /* K routed key blocks per query block (<= 128)                      */
    int32_t window;   /* W, even: query i sees keys j with -W/2 <= j - i < W/2             */
    int32_t n_seg;    /* number of window segments                                         */
    const int32_t *seg_offsets; /* HOST, n_seg + 1 ascending token offsets, multiples of 64,
                                   first 0, last N; the window never crosses a boundary.
                                   NULL means the default: [objects], [view 0], [view 1]...
                                   At most 63 segments (explicit or default: 62 views with object
                                   tokens); more returns LSRM_ERR_UNSUPPORTED from the attention calls. */
    float scale;      /* softmax scale; 0 selects 1/sqrt(d)                                */
    int32_t gate_channels; /* 0: d_gates is [N, h_q, 3], one weight per head and branch;
                              1: d_gates is [N, 3, h_q, d], one weight per output channel
                              and branch (App. A: gating weights of the token's dimension) */
    int32_t window_mode;   /* 0: sliding window (`window`, `seg_offsets`); 1: the window branch of a
                              query sees the tokens of its own block (App. A, "Window"); `window`
                              and the segments are then unused                                  */
    const int32_t *d_block_count; /* DEVICE, nullable, [N/64]: block b holds d_block_count[b] active
                              tokens (1..64) in its first slots (Sec. 3.2: blocks hold a variable
                              number of active tokens); the other slots are padding: never a key
                              in any branch, excluded from the block average, and their own
                              output rows are unspecified.  NULL: every block is full.
                              Read by lsrm_nsa_compress, lsrm_nsa_forward and lsrm_nsa_backward
                              (pass the same counts to all three).                            */
    int32_t kv_packed;     /* lsrm_nsa_forward only.  0: the call repacks d_k, d_v into its workspace
                              itself.  1: d_ws already holds their repacked form, written by
                              lsrm_nsa_compress_pack with the same params, d_k, d_v and d_ws (and not
                              touched since by anything but lsrm_nsa_forward): the repacking pass is
                              skipped.  Other calls ignore the field.                          */
    const int32_t *d_group_offsets; /* DEVICE, nullable, [n_groups + 1]: spatial blocks larger than 64 tokens
                              (Sec. 3.2: 8 x 8 x 8 volume blocks hold up to 512 active tokens).  Spatial block g
                              is the run of 64-slot blocks d_group_offsets[g] .. d_group_offsets[g+1] - 1
                              (ascending, first 0, last N / 64; the caller lays a spatial block's tokens out in
                              consecutive 64-slot blocks, the last one padded, with d_block_count giving the
                              fill).  Then: d_kc, d_vc are [n_groups, h_kv, d], one compressed pair per spatial
                              block, the average of all its active tokens (lsrm_nsa_compress*); the compressed
                              branch attends those n_groups pairs; with window_mode 1 the window of a query is
                              its whole spatial block; lsrm_nsa_backward differentiates accordingly.  Routing
                              tables keep listing 64-slot blocks (a caller that selects a spatial block lists
                              its 64-slot blocks; rows hold up to 128).  NULL: every 64-slot block is its own
                              spatial block.                                                    */
    int32_t n_groups;      /* number of spatial blocks when d_group_offsets is given (1 .. N / 64), else 0   */
} lsrm_nsa_params;

enum { LSRM_WS_ROUTE = 0, LSRM_WS_FORWARD = 1, LSRM_WS_BACKWARD = 2, LSRM_WS_ROUTE_3D = 3 };

/* Bytes of scratch the given call needs for these params (0 on invalid params). */
size_t lsrm_workspace_bytes(const lsrm_nsa_params *p, int which_call);

/*
 * 3D-aware block routing.  [Sec. 3.3 "3D-Aware Block Routing": blocks are selected by
 * geometry -- project the query's 3D position into each view with the known camera
 * parameters and rank image blocks by distance of their 2D centres to the projection;
 * rank volume blocks by distance to the query.  Block-level reading: an object block
 * is represented by the centroid of its 64 token positions; the same projected
 * distance serves both directions.]
 *
 *   d_pos   [n_obj, 3] fp32   object token positions in sequence order
 *   d_cams  [n_views] lsrm_camera
 *   d_idx   [NB, topk] int32  OUT.  Row b < n_obj/64: the topk image tiles nearest to
 *           the projection of object block b's centroid, over all views, as global
 *           block ids n_obj/64 + tile.  Row n_obj/64 + t: the topk object blocks whose
 *           projected centroid is nearest to the centre of tile t.  Ascending by
 *           (squared distance, block id); ties go to the lowest id; missing
 *           candidates are -1.
 *   d_dist2 [NB, topk] fp32   OUT, nullable: the squared distances (+inf for -1).
 * Distances are evaluated in fp32 in a fixed operation order without fused
 * multiply-add, so indices and distances are reproducible bit for bit:
 *   centroid c = (((p0 + p1) + p2) + ... + p63) * (1/64) per component;
 *   x = ((R0 c.x + R1 c.y) + R2 c.z) + t0 (likewise y, z);  z <= 1e-6 -> +inf;
 *   u = fx (x / z) + cx;  v = fy (y / z) + cy;  d2 = (u - ut)^2 + (v - vt)^2.
 */
lsrm_status lsrm_route_blocks(const lsrm_nsa_params *p, const float *d_pos, const lsrm_camera *d_cams,
                              int32_t *d_idx, float *d_dist2, void *d_ws, size_t ws_bytes, void *stream);

/*
 * lsrm_route_blocks for callers that cannot allocate device memory or own no workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels
 * and results as lsrm_route_blocks, without d_ws: the projections pass through a fixed array of
 * LSRM_STATIC_ROUTE_SCRATCH_BYTES that the library's code object holds on every GPU it runs on until
 * the process ends.  The call itself allocates nothing (no hipMalloc / hipFree, no allocating
 * library routine); on its first use on a device it looks the array's address up and keeps it
 * (the one piece of state this library holds, guarded by a mutex).
 * LSRM_ERR_TOO_LARGE when (n_obj / 64) * n_views * 8 bytes exceed the array (131072 block-view pairs;
 * the largest benchmark configuration needs 73728).
 * All calls on one GPU share the array: calls that overlap in time on the same GPU (different
 * streams, or threads) race on it and must be serialised by the caller; calls on one stream are
 * ordered.  Nothing in it needs to start at zero: every element read is written earlier in the same call.
 */
#define LSRM_STATIC_ROUTE_SCRATCH_BYTES (1u << 20)
lsrm_status lsrm_route_blocks_static(const lsrm_nsa_params *p, const float *d_pos, const lsrm_camera *d_cams,
                                     int32_t *d_idx, float *d_dist2, void *stream);

/*
 * Budgets of the four geometric selection rules.  [Sec. 3.3, paragraphs "Image/Volume to Image
 * Blocks" and "Image/Volume to Volume Blocks"; App. hyper-parameter table: volume budgets
 * B^i2v = B^v2v in {8, 16}, image budgets B^v2i = B^i2i in {2M, 4M}.  The paper gives no value
 * for the per-view candidate count B^i.]
 */
typedef struct lsrm_route3d_params {
    int32_t prefilter; /* B^i >= 1: tiles kept per view by 2-D centre distance (clipped to the
                          number of tiles of a view)                                          */
    int32_t k_v2v;     /* volume blocks selected by a volume (object) query block, >= 0       */
    int32_t k_v2i;     /* image blocks selected by a volume query block                       */
    int32_t k_i2v;     /* volume blocks selected by an image query block                      */
    int32_t k_i2i;     /* image blocks selected by an image query block                       */
    int32_t per_token; /* 0: one query per block, its point the centroid of the block (the table the
                          attention calls take); 1: one query per token, its point the token's own
                          coordinate, as Sec. 3.3 words the rules: d_idx, d_dist2 are [N, topk]  */
} lsrm_route3d_params;

/*
 * Routing by the four geometric selection rules, per query block.  [Sec. 3.3: a query with 3-D
 * point p selects (a) the volume blocks whose spatial centres are nearest to p and (b) image
 * blocks in two steps: per view, the B^i blocks whose 2-D centres lie nearest to the projection
 * of p are candidates; candidates are ranked by the smallest 3-D distance between p and the
 * points of the block.  Block-level reading: p is the centroid of the query block's 64 token
 * points; a volume block's centre is the centroid of its 64 positions.]
 *
 *   r          HOST budgets; max(k_v2v + k_v2i, k_i2v + k_i2i) must not exceed p->topk
 *   d_pos      [n_obj, 3] fp32            object token positions (voxel centres), sequence order
 *   d_pos_img  [n_views * grid^2, 3] fp32 the 3-D point of every image token (the surface point
 *              seen by its patch), sequence order: 64 consecutive points = one tile
 *   d_cams     [n_views] lsrm_camera
 *   d_idx      [NB, topk] int32  OUT.  Row of query block b: first the selected volume blocks
 *              (ids in [0, n_obj/64)), ascending by (squared centre distance, id) and including b
 *              itself when b is a volume block; then the selected image blocks (ids n_obj/64 +
 *              tile), ascending by (squared minimum point distance, id); then -1.  Fewer entries
 *              than the budget appear when there are fewer candidates (a view that has p at or
 *              behind its image plane, z <= 1e-6, contributes none).
 *   d_dist2    [NB, topk] fp32  OUT, nullable: the squared 3-D distances (+inf for -1).
 * With r->per_token the rows are query tokens in sequence order (token i < n_obj is a volume query with
 * point d_pos[i], the others image queries with point d_pos_img[i - n_obj]) and the outputs have N rows;
 * the attention calls, which share one list per query block, do not take that table.
 * The per-block table is a valid d_idx for lsrm_nsa_forward / lsrm_nsa_backward.  Arithmetic is fp32 in a
 * fixed order without fused multiply-add (bit-reproducible): centroids and projection as in
 * lsrm_route_blocks; d2 = ((dx dx + dy dy) + dz dz).  Positions must be finite.
 * LSRM_ERR_UNSUPPORTED if n_views * min(prefilter, tiles per view) exceeds 4096.
 */
lsrm_status lsrm_route_blocks_3d(const lsrm_nsa_params *p, const lsrm_route3d_params *r, const float *d_pos,
                                 const float *d_pos_img, const lsrm_camera *d_cams, int32_t *d_idx,
                                 float *d_dist2, void *d_ws, size_t ws_bytes, void *stream);

/*
 * Block compression.  [Sec. 3.2, k_cmp = AvgPool(.), v_cmp = AvgPool(.); App. A
 * "Compressed".  The learned residual module applied before the average in the paper
 * is upstream of this call.]
 *   d_k, d_v   [N, h_kv, d] bf16
 *   d_kc, d_vc [N/64, h_kv, d] bf16  OUT: mean over the 64 tokens of each block (over its
 *              d_block_count[b] active tokens when counts are given), accumulated in fp32 in
 *              token order, rounded to nearest-even bf16.  With d_group_offsets: [n_groups, h_kv, d],
 *              the mean over all active tokens of each spatial block.
 */
lsrm_status lsrm_nsa_compress(const lsrm_nsa_params *p, const uint16_t *d_k, const uint16_t *d_v,
                              uint16_t *d_kc, uint16_t *d_vc, void *stream);

/*
 * Block compression and the forward's repacking of K and V in one pass over K and V.  [Sec. 3.2,
 * App. A "Compressed", as lsrm_nsa_compress.]  The layer needs K and V twice before attention starts:
 * averaged per block, and rearranged into the order the matrix units read them; both are bound by
 * the same HBM reads, so a caller that runs compress and forward back to back saves one pass.
 *   d_k, d_v, d_kc, d_vc   as in lsrm_nsa_compress.  The averages are the same means; the fp32
 *              partial sums are added in a different (fixed) order, so single values may differ
 *              from lsrm_nsa_compress by one rounding of the bf16 result.
 *   d_ws, ws_bytes   the workspace of the lsrm_nsa_forward call that follows
 *              (lsrm_workspace_bytes(p, LSRM_WS_FORWARD)); that call must set params.kv_packed = 1.
 */
lsrm_status lsrm_nsa_compress_pack(const lsrm_nsa_params *p, const uint16_t *d_k, const uint16_t *d_v,
                                   uint16_t *d_kc, uint16_t *d_vc, void *d_ws, size_t ws_bytes, void *stream);

/*
 * NSA forward.  [App. A, Eq. (nsa_1): o_i = w_cmp CmpAttn(q_i, k_cmp, v_cmp)
 * + w_sel SelAttn(q_i, k_sel, v_sel) + w_win WinAttn(q_i, k_win, v_win); three
 * separate softmaxes, no causal mask.]
 *   d_q [N, h_q, d], d_k, d_v [N, h_kv, d], d_kc, d_vc [N/64, h_kv, d]   bf16
 *   d_idx   [NB, topk] int32  any routing table: block ids in [0, NB) or -1 (skipped);
 *           all queries of block b attend every token of the listed blocks.  A row
 *           of -1 gives a zero selected branch.  A block listed twice in a row enters
 *           that row's softmax twice (its tokens weigh double against the others).
 *   d_gates [N, h_q, 3] fp32  gate weights (cmp, sel, win), already passed through
 *           the sigmoid of Eq. (nsa_2), hence in [0, 1] (the forward is linear in them whatever their
 *           sign; lsrm_nsa_backward treats a negative per-head gate as zero); [N, 3, h_q, d] fp32, 16-byte aligned, when
 *           params.gate_channels is 1 (the sum of Eq. (nsa_1) is then taken per channel)
 *   d_out   [N, h_q, d] bf16  OUT
 *   d_lse   [3, N, h_q] fp32  OUT, nullable: natural-log sum-exp of the scaled scores
 *           of each branch (-inf for an empty key set)
 *   d_out_branch [3, N, h_q, d] bf16  OUT, nullable: the un-gated branch outputs
 *   ev_attn_start, ev_attn_stop  nullable hipEvent_t (as void*), created by the caller:
 *           recorded on `stream` immediately before and after the fused attention
 *           kernel alone (the call also runs a short repacking of V before it), so a
 *           caller can time that kernel with hipEventElapsedTime.
 * bf16 MFMA contractions with fp32 accumulation; softmax in fp32.
 */
lsrm_status lsrm_nsa_forward(const lsrm_nsa_params *p, const uint16_t *d_q, const uint16_t *d_k,
                             const uint16_t *d_v, const uint16_t *d_kc, const uint16_t *d_vc,
                             const int32_t *d_idx, const float *d_gates, uint16_t *d_out, float *d_lse,
                             uint16_t *d_out_branch, void *d_ws, size_t ws_bytes, void *stream,
                             void *ev_attn_start, void *ev_attn_stop);

/*
 * NSA backward: gradients of the forward above with respect to q, k and v, for a given
 * gradient of the output.  [App. A, Eq. (nsa_1): the layer is trained end to end (Sec. 4,
 * implementation details); the paper gives no backward algorithm.  Reading: analytic gradients
 * of the three softmax branches with the routing table and the gate weights held constant, and
 * the average pooling differentiated: dk[t] += dk_cmp[t / 64] / 64, likewise dv.]
 *   d_q, d_k, d_v, d_kc, d_vc, d_idx, d_gates   as passed to lsrm_nsa_forward (per-head gates must be >= 0)
 *   d_lse        [3, N, h_q] fp32          as written by lsrm_nsa_forward (required)
 *   d_out_branch [3, N, h_q, d] bf16       as written by lsrm_nsa_forward (required)
 *   d_dout       [N, h_q, d] bf16          gradient of the loss with respect to d_out
 *   d_dq [N, h_q, d], d_dk, d_dv [N, h_kv, d] bf16   OUT (a key/value head collects the gradients of
 *           every query head that reads it)
 *   ev_start, ev_stop  nullable hipEvent_t (as void*): recorded on `stream` before the first and
 *           after the last kernel of the call.
 * With P = softmax probabilities recomputed from d_lse, D_i = dout_i . out_branch_i and
 * dP = dout V^T:  dV = g P^T dout,  dS = g P (dP - D),  dQ = scale dS K,  dK = scale dS^T Q
 * per branch (g the branch's gate; with per-channel gates g P is P and dout is replaced by the
 * channel-wise product gate * dout, rounded to bf16), bf16 MFMA contractions with fp32 accumulation,
 * P and dS rounded to bf16 as MFMA operands.  No atomics on floating-point data: every gradient element
 * is summed in a fixed order (dK/dV go through reverse lists of the routing table, sorted by
 * query block), so results are reproducible bit for bit.
 * Every head dimension, head grouping, gate layout, window mode and block-count setting of the
 * forward is supported.  With d_block_count, padding slots are neither queries nor keys: their rows
 * of d_dout (and of d_k, d_v) are never looked at, and their rows of d_dq, d_dk, d_dv are zero.
 */
lsrm_status lsrm_nsa_backward(const lsrm_nsa_params *p, const uint16_t *d_q, const uint16_t *d_k,
                              const uint16_t *d_v, const uint16_t *d_kc, const uint16_t *d_vc,
                              const int32_t *d_idx, const float *d_gates, const float *d_lse,
                              const uint16_t *d_out_branch, const uint16_t *d_dout, uint16_t *d_dq,
                              uint16_t *d_dk, uint16_t *d_dv, void *d_ws, size_t ws_bytes, void *stream,
                              void *ev_start, void *ev_stop);

#ifdef __cplusplus
}
#endif
#endif /* LSRM_H */
