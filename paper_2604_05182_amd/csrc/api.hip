// C boundary of liblsrm: argument validation and dispatch.  See include/lsrm.h for the
// meaning, layout and ownership of every argument.
#include <vector>

#include "lsrm_internal.h"

namespace lsrm {

lsrm_status make_shape(const lsrm_nsa_params *p, Shape *s) {
    if (p == nullptr || s == nullptr) return LSRM_ERR_INVALID_ARG;
    if (p->n_obj < 0 || p->n_views < 0 || p->grid < 0 || p->h_q <= 0 || p->h_kv <= 0 || p->d <= 0 || p->topk < 0 ||
        p->window < 0 || p->n_seg < 0)
        return LSRM_ERR_INVALID_ARG;
    if (p->n_obj % kBlock != 0 || p->grid % 8 != 0 || (p->window & 1) != 0) return LSRM_ERR_INVALID_ARG;
    if (!(p->scale >= 0.0f) || __builtin_isinf(p->scale)) return LSRM_ERR_INVALID_ARG;
    if (p->h_q % p->h_kv != 0 || (p->gate_channels != 0 && p->gate_channels != 1)) return LSRM_ERR_INVALID_ARG;
    if (p->window_mode != 0 && p->window_mode != 1) return LSRM_ERR_INVALID_ARG;
    if (p->kv_packed != 0 && p->kv_packed != 1) return LSRM_ERR_INVALID_ARG;
    if (p->block != kBlock || (p->d != 32 && p->d != 64 && p->d != 128) || p->topk > 128) return LSRM_ERR_UNSUPPORTED;
    int64_t n_img = (int64_t)p->n_views * p->grid * p->grid;
    int64_t n = (int64_t)p->n_obj + n_img;
    if (n > (int64_t)1 << 30) return LSRM_ERR_UNSUPPORTED;
    s->n_obj = p->n_obj;
    s->n_views = p->n_views;
    s->grid = p->grid;
    s->h = p->h_q;
    s->h_kv = p->h_kv;
    s->gate_channels = p->gate_channels;
    s->d = p->d;
    s->topk = p->topk;
    s->own_block = p->window_mode == 1;
    s->window = s->own_block ? 128 : p->window;
    s->count = p->d_block_count;
    s->kv_packed = p->kv_packed;
    s->goff = p->d_group_offsets;
    s->ng = p->d_group_offsets != nullptr ? p->n_groups : 0;
    s->group_window = 0;
    if (s->ng > 0 && p->window_mode == 1) {
        // the window is the query's spatial block: a sliding window without reach limit inside per-block segments
        s->own_block = 0;
        s->group_window = 1;
        s->window = 1 << 30;
    }
    s->nb_obj = p->n_obj / kBlock;
    s->tiles_per_view = (p->grid / 8) * (p->grid / 8);
    s->n_tiles = p->n_views * s->tiles_per_view;
    s->nb = s->nb_obj + s->n_tiles;
    if (p->d_group_offsets != nullptr ? (p->n_groups < 1 || p->n_groups > s->nb) : p->n_groups != 0) return LSRM_ERR_INVALID_ARG;
    s->nbc = s->ng > 0 ? s->ng : s->nb;
    s->n = n;
    s->scale = p->scale > 0.0f ? p->scale : 1.0f / __builtin_sqrtf((float)p->d);
    return LSRM_OK;
}

// Segment offsets for the window: the caller's, validated, or the default split into
// [objects], [view 0], [view 1], ...
static lsrm_status make_segments(const lsrm_nsa_params *p, const Shape &s, std::vector<int32_t> *seg) {
    seg->clear();
    if (p->seg_offsets == nullptr) {
        seg->push_back(0);
        if (s.n_obj > 0) seg->push_back(s.n_obj);
        for (int m = 0; m < s.n_views; ++m)
            if (s.grid > 0) seg->push_back(s.n_obj + (m + 1) * s.grid * s.grid);
        return LSRM_OK;
    }
    if (p->n_seg < 1) return s.n == 0 ? LSRM_OK : LSRM_ERR_INVALID_ARG;
    for (int i = 0; i <= p->n_seg; ++i) {
        int32_t o = p->seg_offsets[i];
        if (o % kBlock != 0) return LSRM_ERR_INVALID_ARG;
        if (i == 0 ? o != 0 : o < seg->back()) return LSRM_ERR_INVALID_ARG;
        seg->push_back(o);
    }
    if (seg->back() != s.n) return LSRM_ERR_INVALID_ARG;
    return LSRM_OK;
}

static bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

}  // namespace lsrm

using namespace lsrm;

extern "C" {

const char *lsrm_strerror(lsrm_status s) {
    switch (s) {
        case LSRM_OK: return "ok";
        case LSRM_ERR_INVALID_ARG: return "invalid argument";
        case LSRM_ERR_UNSUPPORTED: return "unsupported configuration";
        case LSRM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case LSRM_ERR_HIP: return "HIP runtime error";
        case LSRM_ERR_TOO_LARGE: return "problem exceeds the fixed scratch of the allocation-free entry point";
        default: return "unknown status";
    }
}

size_t lsrm_workspace_bytes(const lsrm_nsa_params *p, int which_call) {
    Shape s;
    if (make_shape(p, &s) != LSRM_OK) return 0;
    switch (which_call) {
        case LSRM_WS_ROUTE: return route_ws_bytes(s);
        case LSRM_WS_FORWARD: return forward_ws_bytes(s);
        case LSRM_WS_BACKWARD: return backward_ws_bytes(s);
        case LSRM_WS_ROUTE_3D: return route3d_ws_bytes(s);
        default: return 0;
    }
}

lsrm_status lsrm_route_blocks(const lsrm_nsa_params *p, const float *d_pos, const lsrm_camera *d_cams, int32_t *d_idx,
                              float *d_dist2, void *d_ws, size_t ws_bytes, void *stream) {
    Shape s;
    lsrm_status rc = make_shape(p, &s);
    if (rc != LSRM_OK) return rc;
    if (s.nb == 0 || s.topk == 0) return LSRM_OK;
    if (d_idx == nullptr) return LSRM_ERR_INVALID_ARG;
    if (s.n_obj > 0 && d_pos == nullptr) return LSRM_ERR_INVALID_ARG;
    if (s.n_views > 0 && d_cams == nullptr) return LSRM_ERR_INVALID_ARG;
    if (d_ws == nullptr || !aligned(d_ws, 256) || ws_bytes < route_ws_bytes(s)) return LSRM_ERR_WORKSPACE;
    return launch_route(s, d_pos, d_cams, d_idx, d_dist2, d_ws, static_cast<hipStream_t>(stream));
}

lsrm_status lsrm_route_blocks_static(const lsrm_nsa_params *p, const float *d_pos, const lsrm_camera *d_cams,
                                     int32_t *d_idx, float *d_dist2, void *stream) {
    Shape s;
    lsrm_status rc = make_shape(p, &s);
    if (rc != LSRM_OK) return rc;
    if (s.nb == 0 || s.topk == 0) return LSRM_OK;
    if (d_idx == nullptr) return LSRM_ERR_INVALID_ARG;
    if (s.n_obj > 0 && d_pos == nullptr) return LSRM_ERR_INVALID_ARG;
    if (s.n_views > 0 && d_cams == nullptr) return LSRM_ERR_INVALID_ARG;
    return launch_route_static(s, d_pos, d_cams, d_idx, d_dist2, static_cast<hipStream_t>(stream));
}

lsrm_status lsrm_route_blocks_3d(const lsrm_nsa_params *p, const lsrm_route3d_params *r, const float *d_pos,
                                 const float *d_pos_img, const lsrm_camera *d_cams, int32_t *d_idx, float *d_dist2,
                                 void *d_ws, size_t ws_bytes, void *stream) {
    Shape s;
    lsrm_status rc = make_shape(p, &s);
    if (rc != LSRM_OK) return rc;
    if (r == nullptr || r->prefilter < 1 || r->k_v2v < 0 || r->k_v2i < 0 || r->k_i2v < 0 || r->k_i2i < 0 ||
        (r->per_token != 0 && r->per_token != 1))
        return LSRM_ERR_INVALID_ARG;
    if ((int64_t)r->k_v2v + r->k_v2i > s.topk || (int64_t)r->k_i2v + r->k_i2i > s.topk) return LSRM_ERR_INVALID_ARG;
    if (s.nb == 0 || s.topk == 0) return LSRM_OK;
    if (d_idx == nullptr) return LSRM_ERR_INVALID_ARG;
    if (s.n_obj > 0 && d_pos == nullptr) return LSRM_ERR_INVALID_ARG;
    if (s.n_tiles > 0 && (d_cams == nullptr || d_pos_img == nullptr)) return LSRM_ERR_INVALID_ARG;
    const int pre = r->prefilter < s.tiles_per_view ? r->prefilter : s.tiles_per_view;
    if ((int64_t)s.n_views * pre > 4096) return LSRM_ERR_UNSUPPORTED;
    if (d_ws == nullptr || !aligned(d_ws, 256) || ws_bytes < route3d_ws_bytes(s)) return LSRM_ERR_WORKSPACE;
    return launch_route_3d(s, *r, d_pos, d_pos_img, d_cams, d_idx, d_dist2, d_ws, static_cast<hipStream_t>(stream));
}

lsrm_status lsrm_nsa_compress(const lsrm_nsa_params *p, const uint16_t *d_k, const uint16_t *d_v, uint16_t *d_kc,
                              uint16_t *d_vc, void *stream) {
    Shape s;
    lsrm_status rc = make_shape(p, &s);
    if (rc != LSRM_OK) return rc;
    if (s.nb == 0) return LSRM_OK;
    if (d_k == nullptr || d_v == nullptr || d_kc == nullptr || d_vc == nullptr) return LSRM_ERR_INVALID_ARG;
    if (!aligned(d_k, 16) || !aligned(d_v, 16) || !aligned(d_kc, 16) || !aligned(d_vc, 16)) return LSRM_ERR_INVALID_ARG;
    return launch_compress(s, d_k, d_v, d_kc, d_vc, static_cast<hipStream_t>(stream));
}

lsrm_status lsrm_nsa_compress_pack(const lsrm_nsa_params *p, const uint16_t *d_k, const uint16_t *d_v, uint16_t *d_kc,
                                   uint16_t *d_vc, void *d_ws, size_t ws_bytes, void *stream) {
    Shape s;
    lsrm_status rc = make_shape(p, &s);
    if (rc != LSRM_OK) return rc;
    if (s.nb == 0) return LSRM_OK;
    if (d_k == nullptr || d_v == nullptr || d_kc == nullptr || d_vc == nullptr) return LSRM_ERR_INVALID_ARG;
    if (!aligned(d_k, 16) || !aligned(d_v, 16) || !aligned(d_kc, 16) || !aligned(d_vc, 16)) return LSRM_ERR_INVALID_ARG;
    if (d_ws == nullptr || !aligned(d_ws, 256) || ws_bytes < forward_ws_bytes(s)) return LSRM_ERR_WORKSPACE;
    return launch_compress_pack(s, d_k, d_v, d_kc, d_vc, d_ws, static_cast<hipStream_t>(stream));
}

lsrm_status lsrm_nsa_forward(const lsrm_nsa_params *p, const uint16_t *d_q, const uint16_t *d_k, const uint16_t *d_v,
                             const uint16_t *d_kc, const uint16_t *d_vc, const int32_t *d_idx, const float *d_gates,
                             uint16_t *d_out, float *d_lse, uint16_t *d_out_branch, void *d_ws, size_t ws_bytes,
                             void *stream, void *ev_attn_start, void *ev_attn_stop) {
    Shape s;
    lsrm_status rc = make_shape(p, &s);
    if (rc != LSRM_OK) return rc;
    std::vector<int32_t> seg;
    rc = make_segments(p, s, &seg);
    if (rc != LSRM_OK) return rc;
    if (s.nb == 0) return LSRM_OK;
    if (d_q == nullptr || d_k == nullptr || d_v == nullptr || d_kc == nullptr || d_vc == nullptr ||
        d_gates == nullptr || d_out == nullptr)
        return LSRM_ERR_INVALID_ARG;
    if (s.topk > 0 && d_idx == nullptr) return LSRM_ERR_INVALID_ARG;
    if (!aligned(d_q, 16) || !aligned(d_k, 16) || !aligned(d_v, 16) || !aligned(d_kc, 16) || !aligned(d_vc, 16) ||
        !aligned(d_out, 16) || (d_out_branch != nullptr && !aligned(d_out_branch, 16)))
        return LSRM_ERR_INVALID_ARG;
    if (s.gate_channels && !aligned(d_gates, 16)) return LSRM_ERR_INVALID_ARG;
    if (d_ws == nullptr || !aligned(d_ws, 256) || ws_bytes < forward_ws_bytes(s)) return LSRM_ERR_WORKSPACE;
    return launch_forward(s, seg.data(), (int)seg.size() - 1, d_q, d_k, d_v, d_kc, d_vc, d_idx, d_gates, d_out, d_lse,
                          d_out_branch, d_ws, static_cast<hipStream_t>(stream), static_cast<hipEvent_t>(ev_attn_start),
                          static_cast<hipEvent_t>(ev_attn_stop));
}

lsrm_status lsrm_nsa_backward(const lsrm_nsa_params *p, const uint16_t *d_q, const uint16_t *d_k, const uint16_t *d_v,
                              const uint16_t *d_kc, const uint16_t *d_vc, const int32_t *d_idx, const float *d_gates,
                              const float *d_lse, const uint16_t *d_out_branch, const uint16_t *d_dout, uint16_t *d_dq,
                              uint16_t *d_dk, uint16_t *d_dv, void *d_ws, size_t ws_bytes, void *stream, void *ev_start,
                              void *ev_stop) {
    Shape s;
    lsrm_status rc = make_shape(p, &s);
    if (rc != LSRM_OK) return rc;
    std::vector<int32_t> seg;
    rc = make_segments(p, s, &seg);
    if (rc != LSRM_OK) return rc;
    if (s.nb == 0) return LSRM_OK;
    const void *in[] = {d_q, d_k, d_v, d_kc, d_vc, d_out_branch, d_dout, d_dq, d_dk, d_dv};
    for (const void *ptr : in)
        if (ptr == nullptr || !aligned(ptr, 16)) return LSRM_ERR_INVALID_ARG;
    if (d_gates == nullptr || d_lse == nullptr) return LSRM_ERR_INVALID_ARG;
    if (s.gate_channels && !aligned(d_gates, 16)) return LSRM_ERR_INVALID_ARG;
    if (s.topk > 0 && d_idx == nullptr) return LSRM_ERR_INVALID_ARG;
    if (d_ws == nullptr || !aligned(d_ws, 256) || ws_bytes < backward_ws_bytes(s)) return LSRM_ERR_WORKSPACE;
    return launch_backward(s, seg.data(), (int)seg.size() - 1, d_q, d_k, d_v, d_kc, d_vc, d_idx, d_gates, d_lse,
                           d_out_branch, d_dout, d_dq, d_dk, d_dv, d_ws, static_cast<hipStream_t>(stream),
                           static_cast<hipEvent_t>(ev_start), static_cast<hipEvent_t>(ev_stop));
}

}  // extern "C"
