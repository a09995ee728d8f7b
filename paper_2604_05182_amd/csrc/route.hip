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

#include <mutex>

// Fixed scratch of lsrm_route_blocks_static, the entry point for callers that cannot allocate: the
// projections project_blocks hands to select_topk ([n_obj/64, n_views] float2).  One copy per GPU, held
// until the process ends.  In host code this name is only a handle for hipGetSymbolAddress -- never a
// device address; kernels receive the address looked up in static_scratch() below.
static __device__ __align__(256) unsigned char scratch[LSRM_STATIC_ROUTE_SCRATCH_BYTES];

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

// Wave-wide minima without the LDS crossbar: four data-parallel-primitive steps fold each row of
// 16 lanes (lane xor 1, xor 2, mirror within 8, mirror within 16), then the four row results are
// read as scalars.  All 64 lanes must be active.  The result is wave-uniform.
template <class Op>
__device__ __forceinline__ unsigned row_fold(unsigned v, Op op) {
    v = op(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
    v = op(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
    v = op(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, false));  // row_half_mirror
    v = op(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, false));  // row_mirror
    return v;
}

__device__ __forceinline__ unsigned wave_min_u32(unsigned v) {
    v = row_fold(v, [](unsigned a, unsigned b) { return a < b ? a : b; });
    unsigned r0 = __builtin_amdgcn_readlane(v, 0), r1 = __builtin_amdgcn_readlane(v, 16);
    unsigned r2 = __builtin_amdgcn_readlane(v, 32), r3 = __builtin_amdgcn_readlane(v, 48);
    unsigned a = r0 < r1 ? r0 : r1, b = r2 < r3 ? r2 : r3;
    return a < b ? a : b;
}

// Non-negative floats order like their bit patterns.
__device__ __forceinline__ float wave_min_nonneg_f32(float v) { return __uint_as_float(wave_min_u32(__float_as_uint(v))); }

__device__ __forceinline__ unsigned long long wave_min_u64(unsigned long long v) {
    const unsigned hi = (unsigned)(v >> 32), lo = (unsigned)v;
    const unsigned hi_min = wave_min_u32(hi);
    const unsigned lo_min = wave_min_u32(hi == hi_min ? lo : 0xffffffffu);
    return ((unsigned long long)hi_min << 32) | lo_min;
}

constexpr unsigned long long kNoKey = ~0ull;

// The k smallest of a set of distinct keys (none equal to all-ones), in ascending order, found by
// one wave: lane l looks at candidates first + l', first + l' + step, ... below n_cand, where l' is
// `me` (the lane id for a wave working alone, the thread id when the four waves of a workgroup
// each take a quarter).  A round is one wave-wide minimum; only the lane that owned the winner
// rescans its candidates.  emit(r, key) is called by every lane for r = 0 .. count-1; returns count.
template <class KeyAt, class Emit>
__device__ __forceinline__ int wave_extract(int me, int step, int n_cand, KeyAt key_at, int k, Emit emit) {
    auto scan = [&](bool have_floor, unsigned long long floor_key) {
        unsigned long long best = kNoKey;
        for (int c = me; c < n_cand; c += step) {
            unsigned long long key = key_at(c);
            if ((!have_floor || key > floor_key) && key < best) best = key;
        }
        return best;
    };
    unsigned long long mine = scan(false, 0);
    int n = 0;
    for (; n < k; ++n) {
        const unsigned long long best = wave_min_u64(mine);
        if (best == kNoKey) break;
        emit(n, best);
        if (mine == best) mine = scan(true, best);
    }
    return n;
}

// Top-k over the whole workgroup (256 threads): every wave extracts the k smallest keys of its
// quarter into `stage` (LDS, 4 * k entries), then wave 0 merges them.  Returns, in wave 0 only,
// the number of keys emitted; the other waves get -1 and have nothing left to do for this list.
template <class KeyAt, class Emit>
__device__ __forceinline__ int wg_topk(int n_cand, KeyAt key_at, int k, unsigned long long *stage, Emit emit) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned long long *mine = stage + (size_t)wave * k;
    int n = wave_extract(threadIdx.x, 256, n_cand, key_at, k, [&](int r, unsigned long long key) {
        if (lane == 0) mine[r] = key;
    });
    for (int r = n + lane; r < k; r += 64) mine[r] = kNoKey;
    __syncthreads();
    if (wave != 0) return -1;
    return wave_extract(lane, 64, 4 * k, [&](int c) { return stage[c]; }, k, emit);
}

// One workgroup per query block.  The squared distances of all candidates are computed once into
// LDS (the candidate id is the array index), then extracted with wg_topk.  `cache_keys` is false
// when they do not fit: distances are then recomputed on every scan (same results, slower).
// Dynamic LDS: [n_cand floats if cache_keys, padded to 8 bytes][4 * topk keys].
__global__ __launch_bounds__(256) void select_topk(int nb_obj, int n_views, int tg, int topk, int cache_keys,
                                                   const float2 *__restrict__ uv, int32_t *__restrict__ idx,
                                                   float *__restrict__ dist2_out) {
    extern __shared__ unsigned long long lds_base[];
    const int row = blockIdx.x;  // query block
    const int tpv = tg * tg;
    const int n_tiles = n_views * tpv;
    const bool obj_row = row < nb_obj;
    const int n_cand = obj_row ? n_tiles : nb_obj;
    const int id_base = obj_row ? nb_obj : 0;
    const int max_cand = nb_obj > n_tiles ? nb_obj : n_tiles;
    float *d2_cache = reinterpret_cast<float *>(lds_base);
    unsigned long long *stage = lds_base + (cache_keys ? (max_cand + 1) / 2 : 0);
    int qm = 0, qi = 0, qj = 0;
    if (!obj_row) {
        int t = row - nb_obj;
        qm = t / tpv;
        int r = t % tpv;
        qi = r / tg;
        qj = r % tg;
    }
    auto d2_of = [&](int c) {
        if (obj_row) {
            int m = c / tpv, r = c % tpv;
            return dist2(uv[(size_t)row * n_views + m], r / tg, r % tg);
        }
        return dist2(uv[(size_t)c * n_views + qm], qi, qj);
    };
    int32_t *idx_row = idx + (size_t)row * topk;
    float *d2_row = dist2_out ? dist2_out + (size_t)row * topk : nullptr;
    auto emit = [&](int r, unsigned long long key) {
        if ((threadIdx.x & 63) == 0) {
            idx_row[r] = id_base + (int)(unsigned)(key & 0xffffffffu);
            if (d2_row) d2_row[r] = __uint_as_float((unsigned)(key >> 32));
        }
    };
    int n;
    if (cache_keys) {
        // every thread reads back only the entries it wrote itself: no barrier needed
        for (int c = threadIdx.x; c < n_cand; c += blockDim.x) d2_cache[c] = d2_of(c);
        n = wg_topk(n_cand, [&](int c) { return make_key(d2_cache[c], (unsigned)c); }, topk, stage, emit);
    } else {
        n = wg_topk(n_cand, [&](int c) { return make_key(d2_of(c), (unsigned)c); }, topk, stage, emit);
    }
    if (n < 0) return;
    for (int k = n + (threadIdx.x & 63); k < topk; k += 64) {  // fewer candidates than topk
        idx_row[k] = -1;
        if (d2_row) d2_row[k] = __builtin_inff();
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

struct Route3d {
    int nb_obj, n_views, tg, width, prefilter, k_v2v, k_v2i, k_i2v, k_i2i, cache_keys;
    int per_token, n_obj;  // queries are tokens (point = own coordinate) instead of blocks (point = centroid)
};

// Dynamic LDS: [n_views * prefilter candidate keys][4 * max(k_v2v, k_i2v) staged keys]
// [nb_obj floats if cache_keys].
__global__ __launch_bounds__(256) void select_3d(Route3d a, const float4 *__restrict__ cent,
                                                 const float *__restrict__ pos, const float *__restrict__ pos_img,
                                                 const lsrm_camera *__restrict__ cams, int32_t *__restrict__ idx,
                                                 float *__restrict__ dist2_out) {
    extern __shared__ unsigned long long lds_base[];
    unsigned long long *img_keys = lds_base;
    unsigned long long *stage = img_keys + (size_t)a.n_views * a.prefilter;
    float *vol_d2 = reinterpret_cast<float *>(stage + 4 * (size_t)(a.k_v2v > a.k_i2v ? a.k_v2v : a.k_i2v));
    const int row = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int tpv = a.tg * a.tg;
    const bool obj_row = row < (a.per_token ? a.n_obj : a.nb_obj);
    const int kv = obj_row ? a.k_v2v : a.k_i2v;
    const int ki = obj_row ? a.k_v2i : a.k_i2i;
    float4 p;
    if (a.per_token) {
        const float *q = obj_row ? pos + (size_t)row * 3 : pos_img + (size_t)(row - a.n_obj) * 3;
        p = make_float4(q[0], q[1], q[2], 0.0f);
    } else {
        p = cent[row];
    }

    // image rule, first two steps: a wave per view
    if (ki > 0) {
        for (int m = wave; m < a.n_views; m += 4) {
            const float2 uv = project(cams[m], p.x, p.y, p.z);
            unsigned long long *out = img_keys + (size_t)m * a.prefilter;
            if (dist2(uv, 0, 0) == __builtin_inff()) {  // no tile of this view is a candidate
                for (int c = lane; c < a.prefilter; c += 64) out[c] = kNoKey;
                continue;
            }
            // candidates in groups of four: pick four tiles, then fetch and measure their point sets
            // together so that the memory latency is paid once per group
            unsigned long long floor_key = 0;
            for (int c0 = 0; c0 < a.prefilter; c0 += 4) {
                int tile[4];
                float d[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    tile[u] = -1;
                    if (c0 + u < a.prefilter) {
                        unsigned long long best = kNoKey;
                        for (int t = lane; t < tpv; t += 64) {
                            unsigned long long key = make_key(dist2(uv, t / a.tg, t % a.tg), (unsigned)t);
                            if ((c0 + u == 0 || key > floor_key) && key < best) best = key;
                        }
                        best = wave_min_u64(best);
                        floor_key = best;
                        tile[u] = m * tpv + (int)(unsigned)(best & 0xffffffffu);
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    d[u] = 0.0f;
                    if (tile[u] >= 0) {
                        const float *q = pos_img + ((size_t)tile[u] * kBlock + lane) * 3;
                        d[u] = sqdist3(p.x, p.y, p.z, q[0], q[1], q[2]);
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (tile[u] >= 0) {
                        float dmin = wave_min_nonneg_f32(d[u]);
                        if (lane == 0) out[c0 + u] = make_key(dmin, (unsigned)(a.nb_obj + tile[u]));
                    }
                }
            }
        }
    }

    // volume rule: per-wave extraction, merged by wave 0 (the barrier inside also publishes img_keys)
    int32_t *idx_row = idx + (size_t)row * a.width;
    float *d2_row = dist2_out ? dist2_out + (size_t)row * a.width : nullptr;
    auto vol_d2_of = [&](int j) {
        float4 c = cent[j];
        return sqdist3(p.x, p.y, p.z, c.x, c.y, c.z);
    };
    int at = 0;
    auto emit = [&](int r, unsigned long long key) {
        if (lane == 0) {
            idx_row[at + r] = (int)(unsigned)(key & 0xffffffffu);
            if (d2_row) d2_row[at + r] = __uint_as_float((unsigned)(key >> 32));
        }
    };
    if (kv > 0) {
        int n;
        if (a.cache_keys) {
            // every thread reads back only the entries it wrote itself
            for (int j = threadIdx.x; j < a.nb_obj; j += blockDim.x) vol_d2[j] = vol_d2_of(j);
            n = wg_topk(a.nb_obj, [&](int j) { return make_key(vol_d2[j], (unsigned)j); }, kv, stage, emit);
        } else {
            n = wg_topk(a.nb_obj, [&](int j) { return make_key(vol_d2_of(j), (unsigned)j); }, kv, stage, emit);
        }
        if (n < 0) return;
        at = n;
    } else {
        __syncthreads();
        if (wave != 0) return;
    }
    // wave 0 alone: the image budget out of the surviving candidates, then the padding
    if (ki > 0)
        at += wave_extract(lane, 64, a.n_views * a.prefilter, [&](int c) { return img_keys[c]; }, ki, emit);
    for (int k = at + lane; k < a.width; k += 64) {
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
    a.per_token = r.per_token;
    a.n_obj = s.n_obj;
    if (a.prefilter < 1) a.k_v2i = a.k_i2i = 0;  // no tiles at all
    const int k_vol = a.k_v2v > a.k_i2v ? a.k_v2v : a.k_i2v;
    const size_t cand_bytes = ((size_t)s.n_views * (a.prefilter > 0 ? a.prefilter : 0) + 4 * (size_t)k_vol) *
                              sizeof(unsigned long long);
    const size_t vol_bytes = (size_t)s.nb_obj * sizeof(float);
    if (cand_bytes > 36 * 1024) return LSRM_ERR_UNSUPPORTED;  // api.hip has bounded both terms below this
    a.cache_keys = vol_bytes + cand_bytes <= 60 * 1024 ? 1 : 0;
    const size_t lds = cand_bytes + (a.cache_keys ? vol_bytes : 0);
    const unsigned n_queries = r.per_token ? (unsigned)s.n : (unsigned)s.nb;
    hipLaunchKernelGGL(select_3d, dim3(n_queries), dim3(256), lds, st, a, cent, d_pos, d_pos_img, d_cams, d_idx,
                       d_dist2);
    LSRM_HIP_CHECK(hipGetLastError());
    return LSRM_OK;
}

// Device address of `scratch` on the current device, looked up once per device (every GPU holds its
// own copy of the array at its own address).
static lsrm_status static_scratch(void **out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void *addr[kMaxDevices] = {};
    int dev = -1;
    LSRM_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return LSRM_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(mu);
    if (addr[dev] == nullptr) {
        void *ptr = nullptr;
        LSRM_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (ptr == nullptr) return LSRM_ERR_HIP;
        addr[dev] = ptr;
    }
    *out = addr[dev];
    return LSRM_OK;
}

lsrm_status launch_route_static(const Shape &s, const float *d_pos, const lsrm_camera *d_cams, int32_t *d_idx,
                                float *d_dist2, hipStream_t st) {
    if (route_ws_bytes(s) > (size_t)LSRM_STATIC_ROUTE_SCRATCH_BYTES) return LSRM_ERR_TOO_LARGE;
    void *ws = nullptr;
    lsrm_status rc = static_scratch(&ws);
    if (rc != LSRM_OK) return rc;
    // project_blocks writes every projection select_topk reads, so nothing of the previous call's
    // contents needs clearing.
    return launch_route(s, d_pos, d_cams, d_idx, d_dist2, ws, st);
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
        const size_t stage_bytes = 4 * (size_t)s.topk * sizeof(unsigned long long);
        const size_t cache_bytes = (size_t)((max_cand + 1) / 2) * sizeof(unsigned long long);
        // default dynamic-LDS limit; beyond it distances are recomputed
        const int cache_keys = cache_bytes + stage_bytes <= 60 * 1024 ? 1 : 0;
        const size_t lds = stage_bytes + (cache_keys ? cache_bytes : 0);
        hipLaunchKernelGGL(select_topk, dim3(s.nb), dim3(256), lds, st, s.nb_obj, s.n_views,
                           s.grid / 8, s.topk, cache_keys, uv, d_idx, d_dist2);
        LSRM_HIP_CHECK(hipGetLastError());
    }
    return LSRM_OK;
}

}  // namespace lsrm
