// 3D-aware block routing on gfx950 (Sec. 3.3 of the paper, block-level reading).
//
// Two kernels:
//   project_blocks  one thread per object block: centroid of its 64 positions, then its
//                   pinhole projection (u, v) into every view.
//   select_topk     one 256-thread workgroup per query block (object block or image
//                   tile): evaluates the squared 2-D distance to every candidate once
//                   (keys parked in LDS) and extracts the K smallest (distance, id)
//                   keys by K rounds of a workgroup-wide minimum.
// The whole file is built with floating-point contraction off: every product and sum
// below is rounded to fp32 exactly as written, which is what makes the indices
// reproducible bit for bit.  Plain ALU work, latency bound and tiny next to attention.
#include "lsrm_internal.h"

namespace lsrm {

namespace {

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
    for (int m = 0; m < n_views; ++m) {
        const lsrm_camera c = cams[m];
        float x = ((c.R[0] * cx + c.R[1] * cy) + c.R[2] * cz) + c.t[0];
        float y = ((c.R[3] * cx + c.R[4] * cy) + c.R[5] * cz) + c.t[1];
        float z = ((c.R[6] * cx + c.R[7] * cy) + c.R[8] * cz) + c.t[2];
        float2 r;
        if (!(z > 1e-6f)) {
            r.x = __builtin_inff();  // marks "behind the camera": infinitely far from every tile
            r.y = 0.0f;
        } else {
            r.x = c.fx * (x / z) + c.cx;
            r.y = c.fy * (y / z) + c.cy;
        }
        uv[(size_t)b * n_views + m] = r;
    }
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

}  // namespace

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
