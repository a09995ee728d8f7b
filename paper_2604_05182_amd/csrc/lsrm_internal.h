// Internal declarations shared by the HIP translation units of liblsrm (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/lsrm.h"

namespace lsrm {

constexpr int kBlock = 64;

struct Shape {
    int n_obj, n_views, grid, h, d, topk, window;
    int h_kv;           // key/value heads, divides h
    int gate_channels;  // 0: gates [N, H, 3]; 1: gates [N, 3, H, d]
    int own_block;      // window branch = the query's own block; `window` is then 128 (every slot of the block
                        // within reach) and the kernels treat the block as its own segment
    int kv_packed;      // the forward workspace already holds the tile images of k and v (lsrm_nsa_compress_pack)
    const int32_t *goff;   // device, nullable [ng + 1]: spatial blocks as runs of 64-slot blocks
    int ng;                // number of spatial blocks (0 without goff)
    int nbc;               // compressed pairs: ng with groups, else nb
    int group_window;      // window branch = the query's spatial block (groups with window_mode 1): the kernels take the
                           // window segment of a block from the blk_seg table and `window` is 2^30
    const int32_t *count;  // device, nullable [nb]: active tokens per block
    int nb_obj, tiles_per_view, n_tiles, nb;
    int64_t n;
    float scale;
};

// Validates params; fills `s`.  Returns LSRM_OK or an error code.
lsrm_status make_shape(const lsrm_nsa_params *p, Shape *s);

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

#define LSRM_HIP_CHECK(expr)                         \
    do {                                             \
        hipError_t e_ = (expr);                      \
        if (e_ != hipSuccess) return LSRM_ERR_HIP;   \
    } while (0)

// launchers (each validates nothing: callers in api.hip have done so)
lsrm_status launch_route(const Shape &s, const float *d_pos, const lsrm_camera *d_cams, int32_t *d_idx,
                         float *d_dist2, void *d_ws, hipStream_t st);
size_t route_ws_bytes(const Shape &s);
// Same kernels, the projections going through the library's fixed per-GPU scratch; calls nothing that allocates.
lsrm_status launch_route_static(const Shape &s, const float *d_pos, const lsrm_camera *d_cams, int32_t *d_idx,
                                float *d_dist2, hipStream_t st);

lsrm_status launch_route_3d(const Shape &s, const lsrm_route3d_params &r, const float *d_pos, const float *d_pos_img,
                            const lsrm_camera *d_cams, int32_t *d_idx, float *d_dist2, void *d_ws, hipStream_t st);
size_t route3d_ws_bytes(const Shape &s);

// Tables derived from the group offsets, for the attention kernels (tab: 3 nb + ng int32 of workspace):
//   blk_grp [nb]     spatial block of every 64-slot block
//   blk_seg [nb][2]  first token and end token of that spatial block
//   grp_tok [ng]     active tokens of every spatial block
struct GroupTables {
    const int32_t *blk_grp, *blk_seg, *grp_tok;
};
inline size_t group_tables_bytes(const Shape &s) { return s.ng > 0 ? align_up(((size_t)3 * s.nb + s.ng) * 4, 256) : 0; }
lsrm_status launch_group_tables(const Shape &s, int32_t *tab, GroupTables *out, hipStream_t st);

lsrm_status launch_compress(const Shape &s, const uint16_t *d_k, const uint16_t *d_v, uint16_t *d_kc,
                            uint16_t *d_vc, hipStream_t st);  // honours s.count

lsrm_status launch_forward(const Shape &s, const int32_t *seg_host, int n_seg, const uint16_t *d_q,
                           const uint16_t *d_k, const uint16_t *d_v, const uint16_t *d_kc,
                           const uint16_t *d_vc, const int32_t *d_idx, const float *d_gates, uint16_t *d_out,
                           float *d_lse, uint16_t *d_out_branch, void *d_ws, hipStream_t st, hipEvent_t ev_start,
                           hipEvent_t ev_stop);
size_t forward_ws_bytes(const Shape &s);
// Pooling and packing in one pass over k and v: kc, vc as launch_compress writes them (same mean, fp32 partial sums
// added in a different order) and the tile images of (k, v) in the forward workspace d_ws.
lsrm_status launch_compress_pack(const Shape &s, const uint16_t *d_k, const uint16_t *d_v, uint16_t *d_kc,
                                 uint16_t *d_vc, void *d_ws, hipStream_t st);
// Step schedule of the selected branch (schedule.hip): the rows of d_idx reordered so that the four query blocks of
// an attention workgroup meet a block they share at the same step; d_sched [ceil(nb / 4) * 4, topk] int32, an entry
// is block id | owner << 28.
size_t sel_schedule_bytes(const Shape &s);
lsrm_status launch_sel_schedule(const Shape &s, const int32_t *d_idx, int32_t *d_sched, hipStream_t st);
// Tile images (see forward.hip): one image per (tile, head) = row-order fragments of `rows_src`, then transposed
// fragments of `t_src`, both [n_rows, H, d] bf16; n_tiles tiles of 32 rows.  rows_only: the backward's
// flavour -- row-order fragments only (t_src unused), slots swizzled as backward.hip expects.
// count (device, nullable, one entry per 64 rows): rows at or beyond their block's count read as zeros.
lsrm_status launch_pack_tiles(int d, const uint16_t *rows_src, const uint16_t *t_src, char *img, int64_t n_rows, int h,
                              int n_tiles, hipStream_t st, bool rows_only, const int32_t *count);

lsrm_status launch_backward(const Shape &s, const int32_t *seg_host, int n_seg, const uint16_t *d_q,
                            const uint16_t *d_k, const uint16_t *d_v, const uint16_t *d_kc, const uint16_t *d_vc,
                            const int32_t *d_idx, const float *d_gates, const float *d_lse,
                            const uint16_t *d_out_branch, const uint16_t *d_dout, uint16_t *d_dq, uint16_t *d_dk,
                            uint16_t *d_dv, void *d_ws, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop);
size_t backward_ws_bytes(const Shape &s);

}  // namespace lsrm
