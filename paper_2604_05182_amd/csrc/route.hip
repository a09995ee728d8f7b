// 3D-aware block routing on gfx950 (Sec. 3.3 of the paper, block-level reading).
//
// Two kernels:
//   project_blocks  one thread per object block: centroid of its 64 positions, then its
//                   pinhole projection (u, v) into every view.
//   select_topk     one 256-thread workgroup per query block (object block or image
//                   tile): evaluates the squared 2-D distance to every candidate once
//                   (keys parked in LDS) and extracts the K smallest (distance, id)
//                   keys by K rounds of a workgroup-wide minimum.
// and, for the four selection rules (volume/image query -> volume/image blocks):
//   block_points    one thread per block of either modality: centroid of its 64 points.
//   select_3d       one 256-thread workgroup per query block: a wave per view projects the
//                   query point, keeps the B^i tiles with the nearest 2-D centres and
//                   measures each one's point set (64 lanes = 64 points, minimum squared 3-D
//                   distance); the workgroup then extracts the nearest volume blocks by
//                   centre distance and the nearest of the surviving tiles.
// The whole file is built with floating-point contraction off: every product and sum
// below is rounded to fp32 exactly as written, which is what makes the indices
// reproducible bit for bit.  Plain ALU work, latency bound and tiny next to attention.
#include "lsrm_internal.h"

namespace lsrm {

namespace {

// Pinhole projection of (cx, cy, cz) in patch units; x = +inf marks a point at or behind the
// image plane (infinitely far from every tile of that view).
__device__ __forceinline__ float2 project(const lsrm_camera &c, float cx, float cy, float cz) {
    float x = ((c.R[0] * cx + c.R[1] * cy) + c.R[2] * cz) + c.t[0];
    float y = ((c.R[3] * cx + c.R[4] * cy) + c.R[5] * cz) + c.t[1];
    float z = ((c.R[6] * cx + c.R[7] * cy) + c.R[8] * cz) + c.t[2];
    float2 r;
    if (!(z > 1e-6f)) {
        r.x = __builtin_inff();
        r.y = 0.0f;
    } else {
        r.x = c.fx * (x / z) + c.cx;
        r.y = c.fy * (y / z) + c.cy;
    }
    return r;
}

__global__ __launch_bounds__(256) void project_blocks(int nb_obj, int n_views, const float *__restrict__ pos,
                                                      const lsrm_camera *__restrict__ cams,
                                                      float2 *__restrict__ uv /* [nb_obj, n_views] */) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= nb_obj) return;
    const float *p = pos + (size_t)b * kBlock * 3;
    float sx = p[0], sy = p[1], sz = p[2];
    for (int t = 1; t < kBlock; ++t) {
        sx = sx + p[3 * t + 0];
        sy = sy + p[3 * t + 1];
        sz = sz + p[3 * t + 2];
    }
    const float inv = 1.0f / 64.0f;
    float cx = sx * inv, cy = sy * inv, cz = sz * inv;
    for (int m = 0; m < n_views; ++m) uv[(size_t)b * n_views + m] = project(cams[m], cx, cy, cz);
}

__device__ __forceinline__ float dist2(float2 p, int ti, int tj) {
    if (__builtin_isinf(p.x) && p.x > 0.0f) return __builtin_inff();
    float ut = (float)(8 * tj + 4);
    float vt = (float)(8 * ti + 4);
    float du = p.x - ut;
    float dv = p.y - vt;
    float d2 = du * du + dv * dv;
    if (d2 != d2) d2 = __builtin_inff();
    return d2;
}

// 64-bit selection key: non-negative fp32 bit patterns order like unsigned integers, so
// (distance bits, candidate id) compares lexicographically as one integer.
__device__ __forceinline__ unsigned long long make_key(float d2, unsigned id) {
    return ((unsigned long long)__float_as_uint(d2) << 32) | id;
}

__device__ __forceinline__ unsigned long long wave_min_u64(unsigned long long v) {
    for (int off = 32; off >= 1; off >>= 1) {
        unsigned long long o = __shfl_xor(v, off, 64);
        v = o < v ? o : v;
    }
    return v;
}

// Keys of all candidates of one query block are computed once into LDS; every thread
// remembers the smallest key of its own strided slice that is still unselected, a round
// is one workgroup-wide minimum over those, and only the winning thread rescans its slice.
// `cache_keys` is false when the candidate keys do not fit in LDS: keys are then
// recomputed on every scan (same results, slower).
__global__ __launch_bounds__(256) void select_topk(int nb_obj, int n_views, int tg, int topk, int cache_keys,
                                                   const float2 *__restrict__ uv, int32_t *__restrict__ idx,
                                                   float *__restrict__ dist2_out) {
    extern __shared__ unsigned long long key_cache[];
    const int row = blockIdx.x;  // query block
    const int tpv = tg * tg;
    const int n_tiles = n_views * tpv;
    const bool obj_row = row < nb_obj;
    const int n_cand = obj_row ? n_tiles : nb_obj;
    const int id_base = obj_row ? nb_obj : 0;
    int qm = 0, qi = 0, qj = 0;
    if (!obj_row) {
        int t = row - nb_obj;
        qm = t / tpv;
        int r = t % tpv;
        qi = r / tg;
        qj = r % tg;
    }
    auto key_of = [&](int c) {
        float d2;
        if (obj_row) {
            int m = c / tpv, r = c % tpv;
            d2 = dist2(uv[(size_t)row * n_views + m], r / tg, r % tg);
        } else {
            d2 = dist2(uv[(size_t)c * n_views + qm], qi, qj);
        }
        return make_key(d2, (unsigned)c);
    };
    __shared__ unsigned long long wmin[4];
    const unsigned long long kNone = ~0ull;
    // smallest key of this thread's slice strictly above `floor_key` (any key if !have_floor)
    auto scan = [&](bool have_floor, unsigned long long floor_key) {
        unsigned long long best = kNone;
        for (int c = threadIdx.x; c < n_cand; c += blockDim.x) {
            unsigned long long key = cache_keys ? key_cache[c] : key_of(c);
            if ((!have_floor || key > floor_key) && key < best) best = key;
        }
        return best;
    };
    if (cache_keys) {
        for (int c = threadIdx.x; c < n_cand; c += blockDim.x) key_cache[c] = key_of(c);
        // each thread only ever reads back the entries it wrote itself: no barrier needed
    }
    unsigned long long mine = scan(false, 0);
    for (int k = 0; k < topk; ++k) {
        unsigned long long best = wave_min_u64(mine);
        if ((threadIdx.x & 63) == 0) wmin[threadIdx.x >> 6] = best;
        __syncthreads();
        unsigned long long b0 = wmin[0], b1 = wmin[1], b2 = wmin[2], b3 = wmin[3];
        __syncthreads();
        unsigned long long m01 = b0 < b1 ? b0 : b1, m23 = b2 < b3 ? b2 : b3;
        best = m01 < m23 ? m01 : m23;
        if (threadIdx.x == 0) {
            if (best == kNone) {
                idx[(size_t)row * topk + k] = -1;
                if (dist2_out) dist2_out[(size_t)row * topk + k] = __builtin_inff();
            } else {
                idx[(size_t)row * topk + k] = id_base + (int)(unsigned)(best & 0xffffffffu);
                if (dist2_out) dist2_out[(size_t)row * topk + k] = __uint_as_float((unsigned)(best >> 32));
            }
        }
        if (best == kNone) {
            // no candidates left: the remaining entries are all empty
            for (int kk = k + 1 + threadIdx.x; kk < topk; kk += blockDim.x) {
                idx[(size_t)row * topk + kk] = -1;
                if (dist2_out) dist2_out[(size_t)row * topk + kk] = __builtin_inff();
            }
            return;
        }
        if (mine == best) mine = scan(true, best);  // keys are distinct: exactly one thread owns the winner
    }
}

// ---------------------------------------------------------------- four selection rules (Sec. 3.3)

// Centroid of each block's 64 points, summed left to right.  Blocks [0, nb_obj) read `pos`,
// the others `pos_img`; the result is padded to float4.
__global__ __launch_bounds__(256) void block_points(int nb_obj, int nb, const float *__restrict__ pos,
                                                    const float *__restrict__ pos_img, float4 *__restrict__ cent) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= nb) return;
    const float *p = b < nb_obj ? pos + (size_t)b * kBlock * 3 : pos_img + (size_t)(b - nb_obj) * kBlock * 3;
    float sx = p[0], sy = p[1], sz = p[2];
    for (int t = 1; t < kBlock; ++t) {
        sx = sx + p[3 * t + 0];
        sy = sy + p[3 * t + 1];
        sz = sz + p[3 * t + 2];
    }
    const float inv = 1.0f / 64.0f;
    cent[b] = make_float4(sx * inv, sy * inv, sz * inv, 0.0f);
}

__device__ __forceinline__ float sqdist3(float ax, float ay, float az, float bx, float by, float bz) {
    float dx = ax - bx, dy = ay - by, dz = az - bz;
    return (dx * dx + dy * dy) + dz * dz;
}

__device__ __forceinline__ float wave_min_f32(float v) {
    for (int off = 32; off >= 1; off >>= 1) v = fminf(v, __shfl_xor(v, off, 64));
    return v;
}

// Emits the k smallest of n_cand distinct keys (key_at(c), c < n_cand) in ascending order, as
// (id = low word, distance = high word), by rounds of a workgroup-wide minimum; keys equal to
// all-ones do not exist.  Every thread of the 256-thread workgroup must call it; returns the
// number emitted (the same in every thread).
template <class KeyAt>
__device__ __forceinline__ int wg_extract(int n_cand, KeyAt key_at, int k, int32_t *idx_out, float *d2_out,
                                          unsigned long long *wmin /* LDS, 4 entries */) {
    const unsigned long long kNone = ~0ull;
    auto scan = [&](bool have_floor, unsigned long long floor_key) {
        unsigned long long best = kNone;
        for (int c = threadIdx.x; c < n_cand; c += blockDim.x) {
            unsigned long long key = key_at(c);
            if ((!have_floor || key > floor_key) && key < best) best = key;
        }
        return best;
    };
    unsigned long long mine = scan(false, 0);
    int n = 0;
    for (; n < k; ++n) {
        unsigned long long best = wave_min_u64(mine);
        if ((threadIdx.x & 63) == 0) wmin[threadIdx.x >> 6] = best;
        __syncthreads();
        unsigned long long b0 = wmin[0], b1 = wmin[1], b2 = wmin[2], b3 = wmin[3];
        __syncthreads();
        unsigned long long m01 = b0 < b1 ? b0 : b1, m23 = b2 < b3 ? b2 : b3;
        best = m01 < m23 ? m01 : m23;
        if (best == kNone) break;
        if (threadIdx.x == 0) {
            idx_out[n] = (int)(unsigned)(best & 0xffffffffu);
            if (d2_out) d2_out[n] = __uint_as_float((unsigned)(best >> 32));
        }
        if (mine == best) mine = scan(true, best);
    }
    return n;
}

struct Route3d {
    int nb_obj, n_views, tg, width, prefilter, k_v2v, k_v2i, k_i2v, k_i2i, cache_keys;
};

// Dynamic LDS: [nb_obj keys if cache_keys][n_views * prefilter candidate keys].
__global__ __launch_bounds__(256) void select_3d(Route3d a, const float4 *__restrict__ cent,
                                                 const float *__restrict__ pos_img,
                                                 const lsrm_camera *__restrict__ cams, int32_t *__restrict__ idx,
                                                 float *__restrict__ dist2_out) {
    extern __shared__ unsigned long long key_cache[];
    __shared__ unsigned long long wmin[4];
    const unsigned long long kNone = ~0ull;
    unsigned long long *vol_keys = key_cache;
    unsigned long long *img_keys = key_cache + (a.cache_keys ? a.nb_obj : 0);
    const int row = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int tpv = a.tg * a.tg;
    const bool obj_row = row < a.nb_obj;
    const int kv = obj_row ? a.k_v2v : a.k_i2v;
    const int ki = obj_row ? a.k_v2i : a.k_i2i;
    const float4 p = cent[row];

    // image rule, first two steps: a wave per view
    if (ki > 0) {
        for (int m = wave; m < a.n_views; m += 4) {
            const float2 uv = project(cams[m], p.x, p.y, p.z);
            unsigned long long *out = img_keys + (size_t)m * a.prefilter;
            if (dist2(uv, 0, 0) == __builtin_inff()) {  // no tile of this view is a candidate
                for (int c = lane; c < a.prefilter; c += 64) out[c] = kNone;
                continue;
            }
            unsigned long long floor_key = 0;
            for (int c = 0; c < a.prefilter; ++c) {
                unsigned long long best = kNone;
                for (int t = lane; t < tpv; t += 64) {
                    unsigned long long key = make_key(dist2(uv, t / a.tg, t % a.tg), (unsigned)t);
                    if ((c == 0 || key > floor_key) && key < best) best = key;
                }
                best = wave_min_u64(best);
                floor_key = best;
                const int tile = m * tpv + (int)(unsigned)(best & 0xffffffffu);
                const float *q = pos_img + ((size_t)tile * kBlock + lane) * 3;
                float d = wave_min_f32(sqdist3(p.x, p.y, p.z, q[0], q[1], q[2]));
                if (lane == 0) out[c] = make_key(d, (unsigned)(a.nb_obj + tile));
            }
        }
    }

    // volume rule
    int32_t *idx_row = idx + (size_t)row * a.width;
    float *d2_row = dist2_out ? dist2_out + (size_t)row * a.width : nullptr;
    auto vol_key = [&](int j) {
        float4 c = cent[j];
        return make_key(sqdist3(p.x, p.y, p.z, c.x, c.y, c.z), (unsigned)j);
    };
    int at = 0;
    if (kv > 0) {
        if (a.cache_keys) {
            // every thread reads back only the entries it wrote itself
            for (int j = threadIdx.x; j < a.nb_obj; j += blockDim.x) vol_keys[j] = vol_key(j);
            at = wg_extract(a.nb_obj, [&](int j) { return vol_keys[j]; }, kv, idx_row, d2_row, wmin);
        } else {
            at = wg_extract(a.nb_obj, vol_key, kv, idx_row, d2_row, wmin);
        }
    }
    __syncthreads();  // candidate keys of all views are in LDS
    if (ki > 0)
        at += wg_extract(a.n_views * a.prefilter, [&](int c) { return img_keys[c]; }, ki, idx_row + at,
                         d2_row ? d2_row + at : nullptr, wmin);
    for (int k = at + threadIdx.x; k < a.width; k += blockDim.x) {
        idx_row[k] = -1;
        if (d2_row) d2_row[k] = __builtin_inff();
    }
}

}  // namespace

size_t route3d_ws_bytes(const Shape &s) {
    size_t n = (size_t)s.nb * sizeof(float4);
    return align_up(n > 0 ? n : 256, 256);
}

lsrm_status launch_route_3d(const Shape &s, const lsrm_route3d_params &r, const float *d_pos, const float *d_pos_img,
                            const lsrm_camera *d_cams, int32_t *d_idx, float *d_dist2, void *d_ws, hipStream_t st) {
    if (s.nb == 0 || s.topk == 0) return LSRM_OK;
    float4 *cent = reinterpret_cast<float4 *>(d_ws);
    hipLaunchKernelGGL(block_points, dim3((s.nb + 255) / 256), dim3(256), 0, st, s.nb_obj, s.nb, d_pos, d_pos_img,
                       cent);
    LSRM_HIP_CHECK(hipGetLastError());
    Route3d a;
    a.nb_obj = s.nb_obj;
    a.n_views = s.n_views;
    a.tg = s.grid / 8;
    a.width = s.topk;
    a.prefilter = r.prefilter < s.tiles_per_view ? r.prefilter : s.tiles_per_view;
    a.k_v2v = r.k_v2v;
    a.k_v2i = r.k_v2i;
    a.k_i2v = r.k_i2v;
    a.k_i2i = r.k_i2i;
    if (a.prefilter < 1) a.k_v2i = a.k_i2i = 0;  // no tiles at all
    const size_t cand_bytes = (size_t)s.n_views * (a.prefilter > 0 ? a.prefilter : 0) * sizeof(unsigned long long);
    const size_t vol_bytes = (size_t)s.nb_obj * sizeof(unsigned long long);
    if (cand_bytes > 32 * 1024) return LSRM_ERR_UNSUPPORTED;
    a.cache_keys = vol_bytes + cand_bytes <= 60 * 1024 ? 1 : 0;
    const size_t lds = cand_bytes + (a.cache_keys ? vol_bytes : 0);
    hipLaunchKernelGGL(select_3d, dim3(s.nb), dim3(256), lds, st, a, cent, d_pos_img, d_cams, d_idx, d_dist2);
    LSRM_HIP_CHECK(hipGetLastError());
    return LSRM_OK;
}

size_t route_ws_bytes(const Shape &s) {
    size_t n = (size_t)s.nb_obj * (size_t)s.n_views * sizeof(float2);
    return align_up(n > 0 ? n : 256, 256);
}

lsrm_status launch_route(const Shape &s, const float *d_pos, const lsrm_camera *d_cams, int32_t *d_idx,
                         float *d_dist2, void *d_ws, hipStream_t st) {
    float2 *uv = reinterpret_cast<float2 *>(d_ws);
    if (s.nb_obj > 0 && s.n_views > 0) {
        int grid = (s.nb_obj + 255) / 256;
        hipLaunchKernelGGL(project_blocks, dim3(grid), dim3(256), 0, st, s.nb_obj, s.n_views, d_pos, d_cams, uv);
        LSRM_HIP_CHECK(hipGetLastError());
    }
    if (s.nb > 0 && s.topk > 0) {
        const int max_cand = s.nb_obj > s.n_tiles ? s.nb_obj : s.n_tiles;
        const size_t lds = (size_t)max_cand * sizeof(unsigned long long);
        const int cache_keys = lds <= 60 * 1024 ? 1 : 0;  // default dynamic-LDS limit; beyond it keys are recomputed
        hipLaunchKernelGGL(select_topk, dim3(s.nb), dim3(256), cache_keys ? lds : 0, st, s.nb_obj, s.n_views,
                           s.grid / 8, s.topk, cache_keys, uv, d_idx, d_dist2);
        LSRM_HIP_CHECK(hipGetLastError());
    }
    return LSRM_OK;
}

}  // namespace lsrm
