/*
 * CPU oracle for the NSA layer with 3D-aware block routing.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU
 * library is compared against.  Only the tests, the smoke check and the
 * benchmark's cpu-baseline leg may call it; the product path never does, and this
 * file shares no code, header, table or helper with the HIP sources.
 *
 * What is computed (section / equation of the paper in brackets):
 *   - routing        [Sec. 3.3 "3D-Aware Block Routing"]: key blocks are chosen from
 *                    geometry alone.  In the block-level reading used here an object
 *                    block is represented by the centroid of its 64 token positions,
 *                    the centroid is projected into every view with the known
 *                    pinhole parameters, and blocks are ranked by the squared 2-D
 *                    distance between that projection and the centres of the 8x8
 *                    image-patch tiles.  Object query blocks keep the K nearest
 *                    tiles (over all views); image query tiles keep the K object
 *                    blocks whose projection falls nearest to them.  The result is
 *                    defined as an exhaustive sort by (distance, block id).
 *   - compression    [Sec. 3.2 "Block Partitioning and Compression"; App. A
 *                    "Compressed"]: one key/value pair per block, the in-block
 *                    average (the learned residual module is upstream of this layer).
 *   - three branches [App. A, Eq. (nsa_1)]: CmpAttn over all compressed pairs,
 *                    SelAttn over every token of the routed blocks, WinAttn over a
 *                    local window, each its own softmax, combined by a gated sum.
 *                    The window is either token level (keys j with
 *                    -W/2 <= j - i < W/2, clipped to the query's segment: object
 *                    tokens / each view) or the query's own block (App. A).  Blocks
 *                    may hold fewer than 64 active tokens.  No causal mask anywhere.
 *   - backward       analytic gradients of the above with routing and gates fixed.
 *
 * Precision: inputs are fp32 (bf16 values widened).  Routing distances are
 * evaluated in fp32 with a fixed operation order and no fused multiply-add (build
 * with -ffp-contract=off) because the routed indices are compared bit for bit.
 * Everything else accumulates in double.
 *
 * Parity with the authors' own implementation is unpinned: the paper prints no
 * worked numeric example.  The functions here are pinned by the CPU tests against
 * brute-force dense-mask attention, closed forms and hand-built routing cases.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define BLK 64

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ routing */

/* Centroid of each object block: left-to-right fp32 sum of its 64 positions, times 1/64. */
void oracle_centroids(int n_obj, const float *pos, float *cent) {
    int nb = n_obj / BLK;
    for (int b = 0; b < nb; ++b) {
        for (int c = 0; c < 3; ++c) {
            float s = pos[(size_t)(BLK * b) * 3 + c];
            for (int t = 1; t < BLK; ++t) s = s + pos[(size_t)(BLK * b + t) * 3 + c];
            cent[b * 3 + c] = s * (1.0f / 64.0f);
        }
    }
}

/*
 * Squared 2-D distance (patch units) between the projection of centroid c into the
 * camera cam = {R[9] row-major, t[3], fx, fy, cx, cy} and the centre of tile (ti, tj).
 * Every product and sum is rounded to fp32, in exactly this order.  A centroid at or
 * behind the image plane (z <= 1e-6) is infinitely far from every tile of that view.
 */
static float tile_dist2(const float *c, const float *cam, int ti, int tj) {
    float x = ((cam[0] * c[0] + cam[1] * c[1]) + cam[2] * c[2]) + cam[9];
    float y = ((cam[3] * c[0] + cam[4] * c[1]) + cam[5] * c[2]) + cam[10];
    float z = ((cam[6] * c[0] + cam[7] * c[1]) + cam[8] * c[2]) + cam[11];
    if (!(z > 1e-6f)) return INFINITY;
    float u = cam[12] * (x / z) + cam[14];
    float v = cam[13] * (y / z) + cam[15];
    float ut = (float)(8 * tj + 4);
    float vt = (float)(8 * ti + 4);
    float du = u - ut;
    float dv = v - vt;
    float d2 = du * du + dv * dv;
    if (d2 != d2) d2 = INFINITY;
    return d2;
}

typedef struct { float d2; int32_t id; } cand_t;

static int cand_cmp(const void *a, const void *b) {
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (x->d2 < y->d2) return -1;
    if (x->d2 > y->d2) return 1;
    return (x->id > y->id) - (x->id < y->id);
}

/*
 * idx [NB, K] int32, dist2 [NB, K] fp32 (dist2 may be NULL), NB = n_obj/64 + M*(S/8)^2.
 * Row b < NB_obj: the K image tiles nearest to block b, as global block ids
 * NB_obj + tile, ascending by (d2, id).  Row NB_obj + t: the K object blocks nearest
 * to tile t.  If fewer than K candidates exist the tail is -1 / +inf.
 */
void oracle_route(int n_obj, int n_views, int grid, int topk, const float *pos, const float *cams,
                  int32_t *idx, float *dist2) {
    int nbo = n_obj / BLK;
    int tg = grid / 8;
    int tpv = tg * tg;
    int nt = n_views * tpv;
    float *cent = (float *)malloc(sizeof(float) * 3 * (size_t)(nbo > 0 ? nbo : 1));
    float *dm = (float *)malloc(sizeof(float) * (size_t)(nbo > 0 ? nbo : 1) * (size_t)(nt > 0 ? nt : 1));
    oracle_centroids(n_obj, pos, cent);
    for (int b = 0; b < nbo; ++b)
        for (int m = 0; m < n_views; ++m)
            for (int ti = 0; ti < tg; ++ti)
                for (int tj = 0; tj < tg; ++tj)
                    dm[(size_t)b * nt + m * tpv + ti * tg + tj] = tile_dist2(cent + 3 * b, cams + 16 * m, ti, tj);
    int maxc = nbo > nt ? nbo : nt;
    cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (size_t)(maxc > 0 ? maxc : 1));
    for (int b = 0; b < nbo; ++b) {
        for (int t = 0; t < nt; ++t) { cand[t].d2 = dm[(size_t)b * nt + t]; cand[t].id = nbo + t; }
        qsort(cand, nt, sizeof(cand_t), cand_cmp);
        for (int k = 0; k < topk; ++k) {
            idx[(size_t)b * topk + k] = k < nt ? cand[k].id : -1;
            if (dist2) dist2[(size_t)b * topk + k] = k < nt ? cand[k].d2 : INFINITY;
        }
    }
    for (int t = 0; t < nt; ++t) {
        for (int b = 0; b < nbo; ++b) { cand[b].d2 = dm[(size_t)b * nt + t]; cand[b].id = b; }
        qsort(cand, nbo, sizeof(cand_t), cand_cmp);
        for (int k = 0; k < topk; ++k) {
            idx[(size_t)(nbo + t) * topk + k] = k < nbo ? cand[k].id : -1;
            if (dist2) dist2[(size_t)(nbo + t) * topk + k] = k < nbo ? cand[k].d2 : INFINITY;
        }
    }
    free(cand); free(dm); free(cent);
}

/*
 * The four geometric selection rules of Sec. 3.3 ("Image/Volume to Image Blocks",
 * "Image/Volume to Volume Blocks") at block granularity: the query is a block, represented by
 * the centroid p of the 3-D coordinates of its 64 tokens (object tokens: voxel centres; image
 * tokens: the surface point assigned to each patch, an input here).
 *   to volume blocks : squared 3-D distance from p to the centre (centroid) of every object
 *                      block; the k_v2v (object query) or k_i2v (image query) smallest.
 *   to image blocks  : p is projected into every view; per view the `prefilter` tiles whose 2-D
 *                      centres are nearest to the projection are candidates (a view that has p
 *                      behind its image plane contributes none); a candidate's distance is the
 *                      smallest squared 3-D distance from p to the 64 points of the tile; the
 *                      k_v2i (object query) or k_i2i (image query) smallest over all views.
 * Row layout: [volume ids ascending by (d2, id)] [image ids (nb_obj + tile) ascending by (d2, id)]
 * then -1 / +inf up to `width`.  All arithmetic fp32 in the order written, no fused multiply-add.
 *   pos [n_obj, 3], pos_img [n_views * grid^2, 3] (sequence order: 64 consecutive tokens = one
 *   tile), cams [n_views, 16];  idx, dist2 [NB, width].
 */
static float sqdist3(const float *a, const float *b) {
    float dx = a[0] - b[0], dy = a[1] - b[1], dz = a[2] - b[2];
    return (dx * dx + dy * dy) + dz * dz;
}

/*
 * per_token == 0: the queries are blocks (query id = block id, point = centroid of the block), the
 * reading used for the attention kernels.  per_token == 1: the queries are tokens, as the paper words
 * the rules (query id = token index in sequence order, point = the token's own coordinate; a token
 * below n_obj is a volume query).  queries (nullable) lists the nq query ids to evaluate, in output
 * row order; NULL = all of them (nq ignored).  idx, dist2: [number of queries, width].
 */
void oracle_route_3d(int n_obj, int n_views, int grid, int width, int prefilter, int k_v2v, int k_v2i, int k_i2v,
                     int k_i2i, int per_token, const int32_t *queries, int nq, const float *pos,
                     const float *pos_img, const float *cams, int32_t *idx, float *dist2) {
    int nbo = n_obj / BLK;
    int tg = grid / 8;
    int tpv = tg * tg;
    int nt = n_views * tpv;
    int nb = nbo + nt;
    float *cent = (float *)malloc(sizeof(float) * 3 * (size_t)(nb > 0 ? nb : 1));
    oracle_centroids(n_obj, pos, cent);
    oracle_centroids(nt * BLK, pos_img, cent + 3 * (size_t)nbo);
    int maxc = nbo > n_views * prefilter ? nbo : n_views * prefilter;
    if (tpv > maxc) maxc = tpv;
    cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (size_t)(maxc > 0 ? maxc : 1));
    cand_t *view = (cand_t *)malloc(sizeof(cand_t) * (size_t)(tpv > 0 ? tpv : 1));
    int n_all = per_token ? n_obj + nt * BLK : nb;
    int n_rows = queries ? nq : n_all;
    for (int row = 0; row < n_rows; ++row) {
        int b = queries ? queries[row] : row;
        const float *p;
        int volume_query;
        if (per_token) {
            volume_query = b < n_obj;
            p = volume_query ? pos + 3 * (size_t)b : pos_img + 3 * (size_t)(b - n_obj);
        } else {
            volume_query = b < nbo;
            p = cent + 3 * (size_t)b;
        }
        int kv = volume_query ? k_v2v : k_i2v, ki = volume_query ? k_v2i : k_i2i;
        int at = 0;
        /* volume blocks */
        for (int j = 0; j < nbo; ++j) { cand[j].d2 = sqdist3(p, cent + 3 * (size_t)j); cand[j].id = j; }
        qsort(cand, nbo, sizeof(cand_t), cand_cmp);
        for (int k = 0; k < kv && k < nbo && at < width; ++k, ++at) {
            idx[(size_t)row * width + at] = cand[k].id;
            if (dist2) dist2[(size_t)row * width + at] = cand[k].d2;
        }
        /* image blocks */
        int nc = 0;
        for (int m = 0; m < n_views; ++m) {
            if (tile_dist2(p, cams + 16 * m, 0, 0) == INFINITY) continue; /* behind the image plane */
            for (int ti = 0; ti < tg; ++ti)
                for (int tj = 0; tj < tg; ++tj) {
                    view[ti * tg + tj].d2 = tile_dist2(p, cams + 16 * m, ti, tj);
                    view[ti * tg + tj].id = m * tpv + ti * tg + tj;
                }
            qsort(view, tpv, sizeof(cand_t), cand_cmp);
            for (int c = 0; c < prefilter && c < tpv; ++c) {
                int tile = view[c].id;
                const float *pts = pos_img + 3 * (size_t)tile * BLK;
                float best = sqdist3(p, pts);
                for (int t = 1; t < BLK; ++t) {
                    float d = sqdist3(p, pts + 3 * t);
                    if (d < best) best = d;
                }
                cand[nc].d2 = best;
                cand[nc].id = nbo + tile;
                ++nc;
            }
        }
        qsort(cand, nc, sizeof(cand_t), cand_cmp);
        for (int k = 0; k < ki && k < nc && at < width; ++k, ++at) {
            idx[(size_t)row * width + at] = cand[k].id;
            if (dist2) dist2[(size_t)row * width + at] = cand[k].d2;
        }
        for (; at < width; ++at) {
            idx[(size_t)row * width + at] = -1;
            if (dist2) dist2[(size_t)row * width + at] = INFINITY;
        }
    }
    free(view); free(cand); free(cent);
}

/* ------------------------------------------------------------------ pooling */

/*
 * Spatial blocks larger than 64 tokens (Sec. 3.2: 8 x 8 x 8 volume blocks with a variable number of active
 * tokens, up to 512): a spatial block is a run of consecutive 64-slot blocks, group g = 64-slot blocks
 * off[g] .. off[g+1]-1 (off ascending, off[0] = 0, off[ng] = N / 64).  With groups the compressed pair is one
 * per spatial block (the average of all its active tokens) and the own-block window (App. A) is the whole
 * spatial block; routing tables keep listing 64-slot blocks.  NULL / ng = 0: every 64-slot block is its own
 * spatial block.
 */
typedef struct { int ng; const int32_t *off; } groups_t;

static int group_of(const groups_t *g, int64_t blk) {
    for (int a = 0; a < g->ng; ++a)
        if (blk >= g->off[a] && blk < g->off[a + 1]) return a;
    return -1;
}

static int max_group_blocks(const groups_t *g) {
    int m = 1;
    for (int a = 0; g && a < g->ng; ++a)
        if (g->off[a + 1] - g->off[a] > m) m = g->off[a + 1] - g->off[a];
    return m;
}

/*
 * out[b, h, :] = mean over the active tokens t of block b of x[64 b + t, h, :];  x is [N, H, d],
 * out is [N/64, H, d].  count (nullable) [N/64]: block b has count[b] active tokens (1..64), held in
 * its first slots (Sec. 3.2: blocks hold a variable number of active tokens); NULL = all 64.
 * With groups (ng > 0): out is [ng, H, d], row g the mean over the active tokens of all 64-slot blocks of group g.
 */
void oracle_pool(int64_t n, int h, int d, const float *x, const int32_t *count, int ng, const int32_t *goff,
                 float *out) {
    int64_t nb = n / BLK;
    size_t row = (size_t)h * d;
    if (ng > 0) {
#pragma omp parallel for schedule(static)
        for (int g = 0; g < ng; ++g) {
            for (size_t c = 0; c < row; ++c) {
                double s = 0.0;
                int64_t tot = 0;
                for (int64_t b = goff[g]; b < goff[g + 1]; ++b) {
                    int cnt = count ? count[b] : BLK;
                    for (int t = 0; t < cnt; ++t) s += (double)x[((size_t)(BLK * b + t)) * row + c];
                    tot += cnt;
                }
                out[(size_t)g * row + c] = (float)(s / (double)tot);
            }
        }
        return;
    }
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < nb; ++b) {
        int cnt = count ? count[b] : BLK;
        for (size_t c = 0; c < row; ++c) {
            double s = 0.0;
            for (int t = 0; t < cnt; ++t) s += (double)x[((size_t)(BLK * b + t)) * row + c];
            out[(size_t)b * row + c] = (float)(s / (double)cnt);
        }
    }
}

/* ------------------------------------------------------------------ forward */

/*
 * One softmax attention of a single query vector over an explicit list of key rows.
 * s_j = scale * <q, K[rows[j]]>,  p = softmax(s),  o = sum_j p_j V[rows[j]].
 * Returns log-sum-exp; an empty list gives o = 0 and lse = -inf.  p (optional, length
 * n) receives the probabilities.
 */
static double attend(const float *qv, int d, double scale, const float *kbase, const float *vbase,
                     size_t stride, const int64_t *rows, int n, double *s, double *o) {
    for (int c = 0; c < d; ++c) o[c] = 0.0;
    if (n == 0) return -INFINITY;
    double m = -INFINITY;
    for (int j = 0; j < n; ++j) {
        const float *kr = kbase + (size_t)rows[j] * stride;
        double acc = 0.0;
        for (int c = 0; c < d; ++c) acc += (double)qv[c] * (double)kr[c];
        s[j] = acc * scale;
        if (s[j] > m) m = s[j];
    }
    double l = 0.0;
    for (int j = 0; j < n; ++j) { s[j] = exp(s[j] - m); l += s[j]; }
    for (int j = 0; j < n; ++j) {
        const float *vr = vbase + (size_t)rows[j] * stride;
        double p = s[j] / l;
        s[j] = p;
        for (int c = 0; c < d; ++c) o[c] += p * (double)vr[c];
    }
    return m + log(l);
}

static int segment_of(const int32_t *seg, int n_seg, int64_t i) {
    for (int s = 0; s < n_seg; ++s)
        if (i >= seg[s] && i < seg[s + 1]) return s;
    return -1;
}

/*
 * Key rows of the three branches for query token i (block qb = i / 64). Returns counts.
 *   window_mode 0: keys j with -W/2 <= j - i < W/2 inside the query's segment (the configs' sliding window);
 *   window_mode 1: the tokens of the query's own block (App. A, "Window").
 *   count (nullable): active tokens per block (its first count[b] slots); inactive slots are nobody's key.
 *   grp (nullable): spatial blocks as groups of 64-slot blocks: the compressed keys are the groups' pairs and
 *   the own-block window is the query's whole group.
 */
static void key_sets(int64_t i, int64_t nb, int topk, int window, int window_mode, const int32_t *count,
                     const groups_t *grp, int n_seg, const int32_t *seg, const int32_t *idx, int64_t *rc, int *nc,
                     int64_t *rs, int *ns, int64_t *rw, int *nw) {
    int64_t qb = i / BLK;
    *nc = 0;
    if (grp)
        for (int g = 0; g < grp->ng; ++g) rc[(*nc)++] = g;
    else
        for (int64_t b = 0; b < nb; ++b) rc[(*nc)++] = b;
    *ns = 0;
    for (int k = 0; k < topk; ++k) {
        int32_t kb = idx[qb * topk + k];
        if (kb < 0) continue;
        int cnt = count ? count[kb] : BLK;
        for (int t = 0; t < cnt; ++t) rs[(*ns)++] = (int64_t)kb * BLK + t;
    }
    *nw = 0;
    if (window_mode == 1) {
        int64_t b0 = qb, b1 = qb + 1;
        if (grp) {
            int g = group_of(grp, qb);
            b0 = grp->off[g];
            b1 = grp->off[g + 1];
        }
        for (int64_t b = b0; b < b1; ++b) {
            int cnt = count ? count[b] : BLK;
            for (int t = 0; t < cnt; ++t) rw[(*nw)++] = b * BLK + t;
        }
        return;
    }
    int sg = segment_of(seg, n_seg, i);
    if (sg >= 0) {
        int64_t lo = i - window / 2, hi = i + window / 2;
        if (lo < seg[sg]) lo = seg[sg];
        if (hi > seg[sg + 1]) hi = seg[sg + 1];
        for (int64_t j = lo; j < hi; ++j)
            if (!count || (j % BLK) < count[j / BLK]) rw[(*nw)++] = j;
    }
}

/*
 * NSA forward for the listed query blocks (App. A, Eq. nsa_1 and nsa_2), with grouped-query
 * heads: h query heads, h_kv key/value heads, query head hh reads key/value head hh / (h / h_kv)
 * (App. A: q in R^{N x h_q x d_h}, k, v in R^{N x h_kv x d_h}; LSRM uses h_q = 32, h_kv = 2).
 *   q [N, H, d];  k, v [N, h_kv, d];  kc, vc [NB, h_kv, d] (pooled), all fp32;  idx [NB, K];
 *   gates: gate_channels == 0: [N, H, 3], one weight per head and branch;
 *          gate_channels == 1: [N, 3, H, d], one weight per output channel and branch (App. A:
 *          the gating weights have the dimension of the token, h_q * d_h);
 *   seg [n_seg + 1] token offsets;  qblocks [nq] block ids;
 *   window_mode, count: see key_sets (kc, vc must have been pooled with the same count); rows of
 *   inactive slots are computed like any other query row (their outputs mean nothing).
 * Outputs are compact over the listed blocks (row r = 64 * position-in-list + t):
 *   out [nq*64, H, d];  lse [3, nq*64, H] (nullable);  ob [3, nq*64, H, d] (nullable).
 */
void oracle_nsa_forward(int64_t n, int h, int h_kv, int d, int topk, int window, int window_mode,
                        const int32_t *count, float scale, int n_seg, const int32_t *seg, const float *q, const float *k, const float *v,
                        const float *kc, const float *vc, const int32_t *idx, const float *gates,
                        int gate_channels, const int32_t *qblocks, int nq, int ng, const int32_t *goff, float *out,
                        float *lse, float *ob) {
    int64_t nb = n / BLK;
    groups_t gst = {ng, goff};
    const groups_t *grp = ng > 0 ? &gst : NULL;
    size_t stride = (size_t)h * d;        /* row stride of q and the outputs */
    size_t stride_kv = (size_t)h_kv * d;  /* row stride of k, v, kc, vc */
    int group = h / h_kv;
    double sc = scale > 0.0f ? (double)scale : 1.0 / sqrt((double)d);
    size_t maxkeys = (size_t)nb;
    if ((size_t)topk * BLK > maxkeys) maxkeys = (size_t)topk * BLK;
    if ((size_t)window + BLK > maxkeys) maxkeys = (size_t)window + BLK;
    int64_t rows_out = (int64_t)nq * BLK;
    size_t maxwin = (size_t)window + (size_t)BLK * max_group_blocks(grp);
    if (maxwin > maxkeys) maxkeys = maxwin;
#pragma omp parallel
    {
        int64_t *rc = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nb > 0 ? nb : 1));
        int64_t *rs = (int64_t *)malloc(sizeof(int64_t) * (size_t)(topk > 0 ? topk : 1) * BLK);
        int64_t *rw = (int64_t *)malloc(sizeof(int64_t) * maxwin);
        double *s = (double *)malloc(sizeof(double) * maxkeys);
        double *o = (double *)malloc(sizeof(double) * (size_t)d * 3);
#pragma omp for schedule(dynamic, 1) collapse(2)
        for (int iq = 0; iq < nq; ++iq) {
            for (int hh = 0; hh < h; ++hh) {
                size_t kvo = (size_t)(hh / group) * d; /* offset of this query head's key/value head */
                for (int t = 0; t < BLK; ++t) {
                    int64_t i = (int64_t)qblocks[iq] * BLK + t;
                    int64_t r = (int64_t)iq * BLK + t;
                    int nc, ns, nw;
                    key_sets(i, nb, topk, window, window_mode, count, grp, n_seg, seg, idx, rc, &nc, rs, &ns, rw, &nw);
                    const float *qv = q + (size_t)i * stride + (size_t)hh * d;
                    double l0 = attend(qv, d, sc, kc + kvo, vc + kvo, stride_kv, rc, nc, s, o);
                    double l1 = attend(qv, d, sc, k + kvo, v + kvo, stride_kv, rs, ns, s, o + d);
                    double l2 = attend(qv, d, sc, k + kvo, v + kvo, stride_kv, rw, nw, s, o + 2 * d);
                    for (int c = 0; c < d; ++c) {
                        double acc = 0.0;
                        for (int br = 0; br < 3; ++br) {
                            double g = gate_channels ? (double)gates[(((size_t)i * 3 + br) * h + hh) * d + c]
                                                     : (double)gates[((size_t)i * h + hh) * 3 + br];
                            acc += g * o[br * d + c];
                        }
                        out[((size_t)r * h + hh) * d + c] = (float)acc;
                    }
                    if (lse) {
                        lse[((size_t)0 * rows_out + r) * h + hh] = (float)l0;
                        lse[((size_t)1 * rows_out + r) * h + hh] = (float)l1;
                        lse[((size_t)2 * rows_out + r) * h + hh] = (float)l2;
                    }
                    if (ob)
                        for (int br = 0; br < 3; ++br)
                            for (int c = 0; c < d; ++c)
                                ob[(((size_t)br * rows_out + r) * h + hh) * d + c] = (float)o[br * d + c];
                }
            }
        }
        free(rc); free(rs); free(rw); free(s); free(o);
    }
}

/* ------------------------------------------------------------------ backward */

/*
 * Gradients of  L = sum_i <dout_i, out_i>  with respect to q, k, v (all [N, H, d]),
 * routing indices and gates held fixed, through the three branches and the pooling.
 * For one softmax attention with probabilities p_j and output o:
 *   dp_j = <do, v_j>,  ds_j = p_j (dp_j - <do, o>),
 *   dq += scale * sum_j ds_j k_j,  dk_j += scale * ds_j q,  dv_j += p_j do,
 * where do = gate * dout for that branch.  Pooled keys/values pass their gradient
 * to the 64 tokens of their block, divided by 64.  Gradients are accumulated in
 * double, single-threaded over queries (this is a definition, not a fast path).
 * With grouped-query heads (h_kv < h) a key/value head collects the gradients of all the
 * query heads that read it; with per-channel gates `gate * dout` is a product per channel.
 * With per-block counts (oracle_nsa_backward only) the padding slots of a block are neither
 * queries nor keys: their gradients are zero, and a pooled pair passes its gradient to the
 * count[b] active tokens of its block, divided by count[b].
 * dq is fp32 [N, H, d]; dk, dv are fp32 [N, h_kv, d].
 */
void oracle_nsa_backward(int64_t n, int h, int h_kv, int d, int topk, int window, int window_mode,
                         const int32_t *count, float scale, int n_seg, const int32_t *seg, const float *q, const float *k, const float *v,
                         const float *kc, const float *vc, const int32_t *idx, const float *gates,
                         int gate_channels, const float *dout, int ng, const int32_t *goff, float *dq, float *dk,
                         float *dv) {
    int64_t nb = n / BLK;
    groups_t gst = {ng, goff};
    const groups_t *grp = ng > 0 ? &gst : NULL;
    size_t stride = (size_t)h * d;        /* rows of q, dout, dq */
    size_t stride_kv = (size_t)h_kv * d;  /* rows of k, v, kc, vc, dk, dv */
    int group = h / h_kv;
    size_t total = (size_t)n * stride, total_kv = (size_t)n * stride_kv;
    size_t totalc = (size_t)(grp ? ng : nb) * stride_kv;  /* pooled pairs: one per spatial block */
    double sc = scale > 0.0f ? (double)scale : 1.0 / sqrt((double)d);
    size_t maxkeys = (size_t)nb;
    if ((size_t)topk * BLK > maxkeys) maxkeys = (size_t)topk * BLK;
    if ((size_t)window + BLK > maxkeys) maxkeys = (size_t)window + BLK;
    double *gq = (double *)calloc(total, sizeof(double));
    double *gk = (double *)calloc(total_kv, sizeof(double));
    double *gv = (double *)calloc(total_kv, sizeof(double));
    double *gkc = (double *)calloc(totalc > 0 ? totalc : 1, sizeof(double));
    double *gvc = (double *)calloc(totalc > 0 ? totalc : 1, sizeof(double));
    int64_t *rc = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nb > 0 ? nb : 1));
    int64_t *rs = (int64_t *)malloc(sizeof(int64_t) * (size_t)(topk > 0 ? topk : 1) * BLK);
    size_t maxwin = (size_t)window + (size_t)BLK * max_group_blocks(grp);
    if (maxwin > maxkeys) maxkeys = maxwin;
    int64_t *rw = (int64_t *)malloc(sizeof(int64_t) * maxwin);
    double *p = (double *)malloc(sizeof(double) * maxkeys);
    double *o = (double *)malloc(sizeof(double) * (size_t)d);
    double *gd = (double *)malloc(sizeof(double) * (size_t)d); /* gate times dout: the gradient reaching one branch */
    for (int64_t i = 0; i < n; ++i) {
        int nc, ns, nw;
        if (count && (i % BLK) >= count[i / BLK]) continue; /* padding slot: no query lives here */
        key_sets(i, nb, topk, window, window_mode, count, grp, n_seg, seg, idx, rc, &nc, rs, &ns, rw, &nw);
        for (int hh = 0; hh < h; ++hh) {
            size_t kvo = (size_t)(hh / group) * d; /* this query head's key/value head */
            const float *qv = q + (size_t)i * stride + (size_t)hh * d;
            const float *dor = dout + (size_t)i * stride + (size_t)hh * d;
            double *gqr = gq + (size_t)i * stride + (size_t)hh * d;
            for (int br = 0; br < 3; ++br) {
                const float *kb = (br == 0 ? kc : k) + kvo;
                const float *vb = (br == 0 ? vc : v) + kvo;
                double *gkb = (br == 0 ? gkc : gk) + kvo;
                double *gvb = (br == 0 ? gvc : gv) + kvo;
                const int64_t *rows = br == 0 ? rc : (br == 1 ? rs : rw);
                int cnt = br == 0 ? nc : (br == 1 ? ns : nw);
                if (cnt == 0) continue;
                for (int c = 0; c < d; ++c) {
                    double g = gate_channels ? (double)gates[(((size_t)i * 3 + br) * h + hh) * d + c]
                                             : (double)gates[((size_t)i * h + hh) * 3 + br];
                    gd[c] = g * (double)dor[c];
                }
                attend(qv, d, sc, kb, vb, stride_kv, rows, cnt, p, o);
                double delta = 0.0;
                for (int c = 0; c < d; ++c) delta += gd[c] * o[c];
                for (int j = 0; j < cnt; ++j) {
                    const float *kr = kb + (size_t)rows[j] * stride_kv;
                    const float *vr = vb + (size_t)rows[j] * stride_kv;
                    double *gkr = gkb + (size_t)rows[j] * stride_kv;
                    double *gvr = gvb + (size_t)rows[j] * stride_kv;
                    double dp = 0.0;
                    for (int c = 0; c < d; ++c) dp += gd[c] * (double)vr[c];
                    double ds = p[j] * (dp - delta) * sc;
                    for (int c = 0; c < d; ++c) {
                        gqr[c] += ds * (double)kr[c];
                        gkr[c] += ds * (double)qv[c];
                        gvr[c] += p[j] * gd[c];
                    }
                }
            }
        }
    }
    for (int64_t j = 0; j < n; ++j) {
        int cnt = count ? count[j / BLK] : BLK;
        if ((j % BLK) >= cnt) continue; /* the mean was taken over the active tokens only */
        int64_t pair = j / BLK; /* the pooled pair this token went into, and how many tokens it averaged */
        double tokens = (double)cnt;
        if (grp) {
            pair = group_of(grp, j / BLK);
            tokens = 0.0;
            for (int64_t b = grp->off[pair]; b < grp->off[pair + 1]; ++b) tokens += count ? count[b] : BLK;
        }
        for (size_t c = 0; c < stride_kv; ++c) {
            gk[(size_t)j * stride_kv + c] += gkc[(size_t)pair * stride_kv + c] / tokens;
            gv[(size_t)j * stride_kv + c] += gvc[(size_t)pair * stride_kv + c] / tokens;
        }
    }
    for (size_t e = 0; e < total; ++e) dq[e] = (float)gq[e];
    for (size_t e = 0; e < total_kv; ++e) { dk[e] = (float)gk[e]; dv[e] = (float)gv[e]; }
    free(gq); free(gk); free(gv); free(gkc); free(gvc);
    free(rc); free(rs); free(rw); free(p); free(o); free(gd);
}

/*
 * Gradients of the same layer for a sample of blocks and heads (full-size parity checks).
 * The arithmetic per (query, head, branch) is that of oracle_nsa_backward (grouped-query heads
 * and per-channel gates included); only what is accumulated differs:
 *   dq  [n_qb*64, n_hs, d]  rows of the listed query blocks, listed query heads `heads`;
 *   dk, dv [n_kb*64, n_kvs, d]  rows of the listed key blocks, listed key/value heads `kvheads`
 *           -- every query of the sequence that attends them contributes, through every query
 *           head of the key/value head's group (pooled keys of the listed blocks included,
 *           spread back over their 64 tokens as in the full function).
 * A (query, branch, head) that feeds neither a wanted dq row nor a listed key block and
 * key/value head is skipped.  OpenMP over queries with per-thread accumulators.
 * Full blocks only (no per-block counts).
 */
void oracle_nsa_backward_sampled(int64_t n, int h, int h_kv, int d, int topk, int window, int window_mode,
                                 float scale, int n_seg, const int32_t *seg, const float *q, const float *k,
                                 const float *v, const float *kc, const float *vc, const int32_t *idx,
                                 const float *gates, int gate_channels, const float *dout,
                                 const int32_t *qblocks, int n_qb, const int32_t *kblocks, int n_kb,
                                 const int32_t *heads, int n_hs, const int32_t *kvheads, int n_kvs, float *dq,
                                 float *dk, float *dv) {
    int64_t nb = n / BLK;
    size_t stride = (size_t)h * d;        /* rows of q, dout */
    size_t stride_kv = (size_t)h_kv * d;  /* rows of k, v, kc, vc */
    int group = h / h_kv;
    double sc = scale > 0.0f ? (double)scale : 1.0 / sqrt((double)d);
    size_t maxkeys = (size_t)nb;
    if ((size_t)topk * BLK > maxkeys) maxkeys = (size_t)topk * BLK;
    if ((size_t)window + BLK > maxkeys) maxkeys = (size_t)window + BLK;
    /* position of a block / head in the sample lists, or -1 */
    int32_t *qpos = (int32_t *)malloc(sizeof(int32_t) * (size_t)(nb > 0 ? nb : 1));
    int32_t *kpos = (int32_t *)malloc(sizeof(int32_t) * (size_t)(nb > 0 ? nb : 1));
    int32_t *hpos = (int32_t *)malloc(sizeof(int32_t) * (size_t)h);
    int32_t *kvpos = (int32_t *)malloc(sizeof(int32_t) * (size_t)h_kv);
    for (int64_t b = 0; b < nb; ++b) qpos[b] = kpos[b] = -1;
    for (int a = 0; a < h; ++a) hpos[a] = -1;
    for (int a = 0; a < h_kv; ++a) kvpos[a] = -1;
    for (int a = 0; a < n_qb; ++a) qpos[qblocks[a]] = a;
    for (int a = 0; a < n_kb; ++a) kpos[kblocks[a]] = a;
    for (int a = 0; a < n_hs; ++a) hpos[heads[a]] = a;
    for (int a = 0; a < n_kvs; ++a) kvpos[kvheads[a]] = a;
    size_t qstride = (size_t)n_hs * d, kstride = (size_t)n_kvs * d;
    size_t tot_q = (size_t)n_qb * BLK * qstride, tot_k = (size_t)n_kb * BLK * kstride, tot_c = (size_t)n_kb * kstride;
    double *gq = (double *)calloc(tot_q > 0 ? tot_q : 1, sizeof(double));
    double *gk = (double *)calloc(tot_k > 0 ? tot_k : 1, sizeof(double));
    double *gv = (double *)calloc(tot_k > 0 ? tot_k : 1, sizeof(double));
    double *gkc = (double *)calloc(tot_c > 0 ? tot_c : 1, sizeof(double));
    double *gvc = (double *)calloc(tot_c > 0 ? tot_c : 1, sizeof(double));
#pragma omp parallel
    {
        double *tk = (double *)calloc(tot_k > 0 ? tot_k : 1, sizeof(double));
        double *tv = (double *)calloc(tot_k > 0 ? tot_k : 1, sizeof(double));
        double *tkc = (double *)calloc(tot_c > 0 ? tot_c : 1, sizeof(double));
        double *tvc = (double *)calloc(tot_c > 0 ? tot_c : 1, sizeof(double));
        int64_t *rc = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nb > 0 ? nb : 1));
        int64_t *rs = (int64_t *)malloc(sizeof(int64_t) * (size_t)(topk > 0 ? topk : 1) * BLK);
        int64_t *rw = (int64_t *)malloc(sizeof(int64_t) * ((size_t)window + BLK));
        double *p = (double *)malloc(sizeof(double) * maxkeys);
        double *o = (double *)malloc(sizeof(double) * (size_t)d);
        double *gd = (double *)malloc(sizeof(double) * (size_t)d); /* gate times dout for one branch */
#pragma omp for schedule(dynamic, 16)
        for (int64_t i = 0; i < n; ++i) {
            int nc, ns, nw;
            key_sets(i, nb, topk, window, window_mode, NULL, NULL, n_seg, seg, idx, rc, &nc, rs, &ns, rw, &nw);
            int qa = qpos[i / BLK];
            for (int br = 0; br < 3; ++br) {
                const int64_t *rows = br == 0 ? rc : (br == 1 ? rs : rw);
                int cnt = br == 0 ? nc : (br == 1 ? ns : nw);
                if (cnt == 0) continue;
                int touches = 0; /* does the key set meet a listed key block? */
                for (int j = 0; j < cnt && !touches; ++j) {
                    int64_t blk = br == 0 ? rows[j] : rows[j] / BLK;
                    if (kpos[blk] >= 0) touches = 1;
                }
                for (int hh = 0; hh < h; ++hh) {
                    int ha = qa >= 0 ? hpos[hh] : -1;               /* column of dq fed by this head, or -1 */
                    int kva = touches ? kvpos[hh / group] : -1;      /* column of dk, dv fed by this head, or -1 */
                    if (ha < 0 && kva < 0) continue;
                    size_t kvo = (size_t)(hh / group) * d;
                    const float *qv = q + (size_t)i * stride + (size_t)hh * d;
                    const float *dor = dout + (size_t)i * stride + (size_t)hh * d;
                    for (int c = 0; c < d; ++c) {
                        double g = gate_channels ? (double)gates[(((size_t)i * 3 + br) * h + hh) * d + c]
                                                 : (double)gates[((size_t)i * h + hh) * 3 + br];
                        gd[c] = g * (double)dor[c];
                    }
                    const float *kb = (br == 0 ? kc : k) + kvo;
                    const float *vb = (br == 0 ? vc : v) + kvo;
                    attend(qv, d, sc, kb, vb, stride_kv, rows, cnt, p, o);
                    double delta = 0.0;
                    for (int c = 0; c < d; ++c) delta += gd[c] * o[c];
                    for (int j = 0; j < cnt; ++j) {
                        int64_t blk = br == 0 ? rows[j] : rows[j] / BLK;
                        int ka = kva >= 0 ? kpos[blk] : -1;
                        if (ka < 0 && ha < 0) continue;
                        const float *kr = kb + (size_t)rows[j] * stride_kv;
                        const float *vr = vb + (size_t)rows[j] * stride_kv;
                        double dp = 0.0;
                        for (int c = 0; c < d; ++c) dp += gd[c] * (double)vr[c];
                        double ds = p[j] * (dp - delta) * sc;
                        if (ha >= 0) {
                            double *gqr = gq + ((size_t)qa * BLK + (size_t)(i % BLK)) * qstride + (size_t)ha * d;
                            for (int c = 0; c < d; ++c) gqr[c] += ds * (double)kr[c];
                        }
                        if (ka >= 0) {
                            double *gkr, *gvr;
                            if (br == 0) {
                                gkr = tkc + (size_t)ka * kstride + (size_t)kva * d;
                                gvr = tvc + (size_t)ka * kstride + (size_t)kva * d;
                            } else {
                                size_t row = (size_t)ka * BLK + (size_t)(rows[j] % BLK);
                                gkr = tk + row * kstride + (size_t)kva * d;
                                gvr = tv + row * kstride + (size_t)kva * d;
                            }
                            for (int c = 0; c < d; ++c) {
                                gkr[c] += ds * (double)qv[c];
                                gvr[c] += p[j] * gd[c];
                            }
                        }
                    }
                }
            }
        }
#pragma omp critical
        {
            for (size_t e = 0; e < tot_k; ++e) { gk[e] += tk[e]; gv[e] += tv[e]; }
            for (size_t e = 0; e < tot_c; ++e) { gkc[e] += tkc[e]; gvc[e] += tvc[e]; }
        }
        free(tk); free(tv); free(tkc); free(tvc);
        free(rc); free(rs); free(rw); free(p); free(o); free(gd);
    }
    for (size_t e = 0; e < tot_q; ++e) dq[e] = (float)gq[e];
    for (int a = 0; a < n_kb; ++a)
        for (int t = 0; t < BLK; ++t)
            for (size_t c = 0; c < kstride; ++c) {
                size_t e = ((size_t)a * BLK + (size_t)t) * kstride + c;
                dk[e] = (float)(gk[e] + gkc[(size_t)a * kstride + c] / 64.0);
                dv[e] = (float)(gv[e] + gvc[(size_t)a * kstride + c] / 64.0);
            }
    free(gq); free(gk); free(gv); free(gkc); free(gvc); free(qpos); free(kpos); free(hpos); free(kvpos);
}
