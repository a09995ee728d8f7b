// NSA forward on gfx950 (App. A, Eq. nsa_1): compressed, selected and window attention,
// each its own softmax, combined by the gated sum, in one kernel.
//
// Work decomposition
//   One workgroup owns one (query block of 64 tokens, head) and carries it through all
//   three branches.  A wavefront holds QT tiles of 32 query rows: QT = 1 means two
//   wavefronts per workgroup that share every K/V tile through LDS (d = 128: the state
//   of 32 rows fits 256 registers, so two wavefronts run per SIMD and one's softmax
//   overlaps the other's MFMAs); QT = 2 means a single self-contained wavefront per
//   workgroup with no barriers at all (d = 64).  Workgroups are numbered so that each
//   of the 8 XCDs walks a contiguous range of (head, query block) units: the L2 of an
//   XCD then holds one head's pooled keys/values and the neighbouring windows / routed
//   blocks.
//
// Per 32-key step, per wavefront and query tile
//   S^T = K Q^T        v_mfma_f32_32x32x16_bf16, A = 32 keys x 16 channels, B = Q^T.
//                      With S transposed, each lane owns one query column, so the row
//                      max / row sum of the softmax are in-lane reductions plus one
//                      exchange between the two lane halves (v_permlane32_swap).
//   P^T -> bf16        the accumulator layout of S^T is already the B-operand layout of
//                      the next contraction once the key rows of the A operand are
//                      loaded in a fixed permutation (bits 2 and 3 of the row swapped),
//                      so P never leaves registers.
//   O^T += V^T P^T     A = 32 channels x 16 keys from a pre-transposed copy of V.
//
// Data movement
//   K rows come straight from the caller's [N, H, d] tensor, V from a packed transposed
//   copy made once per call ([block][head][half][d][32 keys], 16-byte chunks XOR-swizzled
//   so that LDS reads are bank-conflict free).  Both are copied global -> LDS with
//   global_load_lds_dwordx4 (no VGPR staging; scalar base + per-lane 32-bit offset),
//   double buffered per workgroup, and read back as ds_read_b128 MFMA fragments.
//   The gated sum of the branches is carried between branches in an fp32 scratch tile in
//   MFMA-fragment order (fully coalesced) instead of in registers; the final tile goes
//   through LDS so that the bf16 output rows are written as whole 16-byte chunks.
#include "lsrm_internal.h"

namespace lsrm {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kMaxSeg = 63;
constexpr float kMinusHuge = -1.0e30f;  // initial running maximum: finite, so no inf - inf

#define LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

struct FwdArgs {
    const uint16_t *q, *k, *v_t, *kc, *vc_t;  // v_t / vc_t: packed transposed copies
    const int32_t *idx;
    const float *gates;
    int32_t seg[kMaxSeg + 1];  // window segment offsets (tokens)
    uint16_t *out;
    float *lse;
    uint16_t *out_branch;
    float *gsum;  // scratch: running gated sum, fragment order
    int64_t n;
    int nb, h, topk, window, n_seg;
    int units, units_per_xcd;
    float scale_log2e, scale;
};

template <int D, int QT>
struct Geo {
    static constexpr int NS = D / 16;           // 16-channel slabs of the QK^T contraction
    static constexpr int ND = D / 32;           // 32-channel tiles of the PV output
    static constexpr int K_BYTES = 32 * D * 2;  // 32 key rows
    static constexpr int V_BYTES = D * 64;      // D channel rows x 32 keys
    static constexpr int STAGE = K_BYTES + V_BYTES;
    static constexpr int NW = 2 / QT;           // wavefronts per workgroup
    static constexpr int THREADS = 64 * NW;
    static constexpr int K_INST = K_BYTES / 1024 / NW;  // copy instructions per wavefront and tile
    static constexpr int V_INST = V_BYTES / 1024 / NW;
    static constexpr int OUT_ROW = 2 * D + 8;   // padded bf16 row of the output transpose (bytes)
    static constexpr int LDS_BYTES = 2 * STAGE > NW * 32 * OUT_ROW ? 2 * STAGE : NW * 32 * OUT_ROW;
};

// swizzle of the 16-byte chunk index inside a K row held in LDS
template <int D>
__device__ __forceinline__ int k_swz(int row) {
    return D == 128 ? (row & 15) : ((row >> 1) & 7);
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    bf16x2 p;
    p[0] = (__bf16)a;
    p[1] = (__bf16)b;
    return *reinterpret_cast<uint32_t *>(&p);
}

// max / sum across the two lane halves (lanes i and i + 32 hold the same query)
__device__ __forceinline__ float half_max(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

struct TileSrc {
    const uint16_t *k_rows;  // row 0 of the 32-key sub-tile, this head
    int rows_valid;          // rows >= rows_valid are clamped (their scores get masked)
    const uint16_t *v_t;     // packed transposed V sub-tile, contiguous V_BYTES
    int j0;                  // index of key 0 of the sub-tile in mask coordinates
    bool need_mask;
};

template <int D, int QT>
struct WaveCtx {
    using G = Geo<D, QT>;
    bf16x8 qf[QT][G::NS];
    f32x16 o[QT][G::ND];
    float m[QT], l[QT];
    int lo[QT], hi[QT];
    uint32_t koff[G::K_INST];  // per-lane byte offsets of this wavefront's K copy instructions
    int krow[G::K_INST];       // and the tile row / 16-byte chunk each of them fetches
    int kchunk[G::K_INST];
};

// Issues this wavefront's share of the global -> LDS copies of one 32-key sub-tile.
template <int D, int QT>
__device__ __forceinline__ void issue_tile(const WaveCtx<D, QT> &c, const TileSrc &t, uint32_t row_stride_bytes,
                                           char *lds_stage, int wave, int lane) {
    using G = Geo<D, QT>;
    const char *kbase = reinterpret_cast<const char *>(t.k_rows);
    if (__builtin_expect(t.rows_valid >= 32, 1)) {
#pragma unroll
        for (int j = 0; j < G::K_INST; ++j) {
            const int i = wave + G::NW * j;
            __builtin_amdgcn_global_load_lds(GLB_PTR(kbase + c.koff[j]), LDS_PTR(lds_stage + i * 1024), 16, 0, 0);
        }
    } else {
#pragma unroll
        for (int j = 0; j < G::K_INST; ++j) {
            const int i = wave + G::NW * j;
            const int srow = c.krow[j] < t.rows_valid ? c.krow[j] : t.rows_valid - 1;
            const uint32_t off = (uint32_t)srow * row_stride_bytes + (uint32_t)c.kchunk[j] * 16u;
            __builtin_amdgcn_global_load_lds(GLB_PTR(kbase + off), LDS_PTR(lds_stage + i * 1024), 16, 0, 0);
        }
    }
    const char *vbase = reinterpret_cast<const char *>(t.v_t);
#pragma unroll
    for (int j = 0; j < G::V_INST; ++j) {
        const int i = wave + G::NW * j;
        __builtin_amdgcn_global_load_lds(GLB_PTR(vbase + i * 1024 + (uint32_t)lane * 16u),
                                         LDS_PTR(lds_stage + G::K_BYTES + i * 1024), 16, 0, 0);
    }
}

template <int D, int QT>
__device__ __forceinline__ void reset_branch(WaveCtx<D, QT> &c) {
    using G = Geo<D, QT>;
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        c.m[qt] = kMinusHuge;
        c.l[qt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < G::ND; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) c.o[qt][dt][i] = 0.f;
    }
}

// One 32-key step: fragments are already in registers.
//
// The running maximum m is allowed to lag: it is raised (and O, l rescaled) only when a
// new score exceeds it by more than kLag in the log2 domain, so probabilities stay
// below 2^kLag -- harmless in fp32 and bf16, whose exponent ranges are the same -- and
// the rescale of the O accumulators becomes a rare, wave-uniform branch.
constexpr float kLag = 8.0f;

template <int D, int QT>
__device__ __forceinline__ void step_compute(WaveCtx<D, QT> &c, const bf16x8 (&kf)[Geo<D, QT>::NS],
                                             const bf16x8 (&vf)[Geo<D, QT>::ND][2], int j0, bool need_mask, int hh,
                                             float sl2) {
    using G = Geo<D, QT>;
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        f32x16 s;
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < G::NS; ++ks) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], c.qf[qt][ks], s, 0, 0, 0);
        if (need_mask) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                int j = j0 + 16 * (i / 8) + 8 * hh + (i % 8);
                if (j < c.lo[qt] || j >= c.hi[qt]) s[i] = -__builtin_inff();
            }
        }
        float mx = fmaxf(s[0], s[1]);
#pragma unroll
        for (int i = 2; i < 16; i += 2) mx = fmaxf(mx, fmaxf(s[i], s[i + 1]));
        mx = half_max(mx);
        // m starts at kMinusHuge (finite), so the first real score always raises it and no
        // inf - inf ever appears; a fully masked step (mx = -inf) never does.
        const bool raise = (mx - c.m[qt]) * sl2 > kLag;
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(raise) != 0, 0)) {
            float m_new = raise ? mx : c.m[qt];
            float alpha = raise ? __builtin_amdgcn_exp2f((c.m[qt] - m_new) * sl2) : 1.0f;
            c.m[qt] = m_new;
            c.l[qt] *= alpha;
#pragma unroll
            for (int dt = 0; dt < G::ND; ++dt)
#pragma unroll
                for (int i = 0; i < 16; ++i) c.o[qt][dt][i] *= alpha;
        }
        const float mc = c.m[qt] * sl2;
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            s[i] = __builtin_amdgcn_exp2f(s[i] * sl2 - mc);
            psum += s[i];
        }
        c.l[qt] += psum;
        union {
            bf16x8 v;
            uint32_t u[4];
        } pb[2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int j = 0; j < 4; ++j) pb[ks].u[j] = pack_bf16(s[8 * ks + 2 * j], s[8 * ks + 2 * j + 1]);
#pragma unroll
        for (int dt = 0; dt < G::ND; ++dt)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
                c.o[qt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt][ks], pb[ks].v, c.o[qt][dt], 0, 0, 0);
    }
}

template <int D, int QT>
__device__ __forceinline__ void read_frags(const char *lds_stage, int r_perm, int r, int hh,
                                           bf16x8 (&kf)[Geo<D, QT>::NS], bf16x8 (&vf)[Geo<D, QT>::ND][2]) {
    using G = Geo<D, QT>;
    const int ksw = k_swz<D>(r_perm);
#pragma unroll
    for (int ks = 0; ks < G::NS; ++ks) {
        int slot = (2 * ks + hh) ^ ksw;
        kf[ks] = *reinterpret_cast<const bf16x8 *>(lds_stage + r_perm * (2 * D) + slot * 16);
    }
#pragma unroll
    for (int dt = 0; dt < G::ND; ++dt) {
        int row = 32 * dt + r;
        int vsw = (row >> 2) & 3;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            int slot = (2 * ks + hh) ^ vsw;
            vf[dt][ks] = *reinterpret_cast<const bf16x8 *>(lds_stage + G::K_BYTES + row * 64 + slot * 16);
        }
    }
}

// Streams n_steps sub-tiles produced by src(t) through the two LDS stages of the workgroup.
// n_steps and src are uniform over the workgroup, so every wavefront meets every barrier.
template <int D, int QT, typename SrcFn>
__device__ __forceinline__ void run_steps(WaveCtx<D, QT> &c, int n_steps, SrcFn src, uint32_t row_stride_bytes,
                                          char *lds, int wave, int lane, float sl2) {
    using G = Geo<D, QT>;
    const int r = lane & 31, hh = lane >> 5;
    const int r_perm = (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1);
    if (n_steps <= 0) return;
    TileSrc cur = src(0);
    if (G::NW > 1) __syncthreads();  // every wavefront is done with both stages (previous branch)
    issue_tile<D, QT>(c, cur, row_stride_bytes, lds, wave, lane);
    for (int t = 0; t < n_steps; ++t) {
        char *stage = lds + (t & 1) * G::STAGE;
        bf16x8 kf[G::NS];
        bf16x8 vf[G::ND][2];
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's copies of step t have landed
        if (G::NW > 1) __syncthreads();      // ... and the partner's; also: everyone finished reading step t-1
        read_frags<D, QT>(stage, r_perm, r, hh, kf, vf);
        TileSrc nxt = cur;
        if (t + 1 < n_steps) {
            nxt = src(t + 1);
            issue_tile<D, QT>(c, nxt, row_stride_bytes, lds + ((t + 1) & 1) * G::STAGE, wave, lane);
        }
        step_compute<D, QT>(c, kf, vf, cur.j0, cur.need_mask, hh, sl2);
        cur = nxt;
    }
}

// Ends a branch: normalises, applies the gate and folds the result into the running
// gated sum kept in the fp32 scratch tile (written by branch 0, updated by branch 1,
// consumed by branch 2, which converts to bf16 and stores the output rows through LDS).
// Optionally stores the un-gated branch output and its log-sum-exp.
template <int D, int QT>
__device__ __forceinline__ void finish_branch(WaveCtx<D, QT> &c, const FwdArgs &a, int branch, int qb, int head,
                                              int wave, int lane, char *lds) {
    using G = Geo<D, QT>;
    const int r = lane & 31, hh = lane >> 5;
    if (branch == 2 && G::NW > 1) __syncthreads();  // the copy stages are about to be reused for the output
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int64_t row0 = (int64_t)qb * 64 + 32 * (wave * QT + qt);
        const int64_t row = row0 + r;
        const float l_tot = half_sum(c.l[qt]);
        const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
        const float w = a.gates[(row * a.h + head) * 3 + branch] * inv;
        if (a.lse != nullptr && hh == 0) {
            float v = l_tot > 0.f ? c.m[qt] * a.scale + __logf(l_tot) : -__builtin_inff();
            a.lse[((int64_t)branch * a.n + row) * a.h + head] = v;
        }
        if (a.out_branch != nullptr) {
#pragma unroll
            for (int dt = 0; dt < G::ND; ++dt) {
                uint16_t *dst = a.out_branch + (((int64_t)branch * a.n + row) * a.h + head) * D + 32 * dt + 4 * hh;
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    uint2 w2;
                    w2.x = pack_bf16(c.o[qt][dt][4 * gq + 0] * inv, c.o[qt][dt][4 * gq + 1] * inv);
                    w2.y = pack_bf16(c.o[qt][dt][4 * gq + 2] * inv, c.o[qt][dt][4 * gq + 3] * inv);
                    *reinterpret_cast<uint2 *>(dst + 8 * gq) = w2;
                }
            }
        }
        // scratch tile of this (32-row tile, head): [ND][4][64 lanes] float4
        f32x4 *gs = reinterpret_cast<f32x4 *>(a.gsum) + (((row0 >> 5) * a.h + head) * (G::ND * 4)) * 64 + lane;
        char *tr = lds + wave * 32 * G::OUT_ROW;  // output transpose region of this wavefront
#pragma unroll
        for (int dt = 0; dt < G::ND; ++dt) {
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                f32x4 v;
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = w * c.o[qt][dt][4 * gq + j];
                if (branch > 0) {
                    f32x4 prev = gs[(dt * 4 + gq) * 64];
                    v += prev;
                }
                if (branch < 2) {
                    gs[(dt * 4 + gq) * 64] = v;
                } else {
                    uint2 w2;
                    w2.x = pack_bf16(v[0], v[1]);
                    w2.y = pack_bf16(v[2], v[3]);
                    *reinterpret_cast<uint2 *>(tr + r * G::OUT_ROW + (32 * dt + 8 * gq + 4 * hh) * 2) = w2;
                }
            }
        }
        if (branch == 2) {
            // rows of this tile back from LDS as whole 16-byte chunks: 4 (d=128) or 8 (d=64) rows per pass
            constexpr int CH = D / 8;
            constexpr int ROWS = 64 / CH;
#pragma unroll
            for (int it = 0; it < 32 / ROWS; ++it) {
                const int rr = it * ROWS + lane / CH, ch = lane % CH;
                uint4 val = *reinterpret_cast<const uint4 *>(tr + rr * G::OUT_ROW + ch * 16);
                *reinterpret_cast<uint4 *>(a.out + ((row0 + rr) * a.h + head) * D + ch * 8) = val;
            }
        }
    }
}

template <int D, int QT>
__global__ __launch_bounds__((Geo<D, QT>::THREADS), 2) void nsa_forward_kernel(FwdArgs a) {
    using G = Geo<D, QT>;
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    // XCD-aware numbering: hardware deals consecutive workgroups round-robin to the 8 XCDs
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    if (slot >= a.units_per_xcd) return;
    const int unit = xcd * a.units_per_xcd + slot;
    if (unit >= a.units) return;
    const int head = unit / a.nb;
    const int qb = unit % a.nb;
    const int lane = threadIdx.x & 63;
    const int wave = G::NW > 1 ? __builtin_amdgcn_readfirstlane(threadIdx.x >> 6) : 0;
    const int r = lane & 31, hh = lane >> 5;
    const uint32_t row_stride_bytes = (uint32_t)a.h * D * 2;
    const float sl2 = a.scale_log2e;

    WaveCtx<D, QT> c;
    {
        constexpr int ROWS_PER_INST = 1024 / (D * 2);
        constexpr int CHUNKS = D / 8;
#pragma unroll
        for (int j = 0; j < G::K_INST; ++j) {
            const int i = wave + G::NW * j;
            const int row = i * ROWS_PER_INST + lane / CHUNKS;
            const int chunk = (lane % CHUNKS) ^ k_swz<D>(row);
            c.krow[j] = row;
            c.kchunk[j] = chunk;
            c.koff[j] = (uint32_t)row * row_stride_bytes + (uint32_t)chunk * 16u;
        }
    }
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const uint16_t *qrow = a.q + (((int64_t)qb * 64 + 32 * (wave * QT + qt) + r) * a.h + head) * D + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < G::NS; ++ks) c.qf[qt][ks] = *reinterpret_cast<const bf16x8 *>(qrow + 16 * ks);
    }

    // ---------------- compressed branch: all NB pooled pairs
    {
        reset_branch<D, QT>(c);
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            c.lo[qt] = 0;
            c.hi[qt] = a.nb;
        }
        const int n_steps = (a.nb + 31) / 32;
        auto src = [&](int t) {
            TileSrc s;
            s.k_rows = a.kc + ((int64_t)(32 * t) * a.h + head) * D;
            s.rows_valid = a.nb - 32 * t;
            s.v_t = a.vc_t + (((int64_t)(t >> 1) * a.h + head) * 2 + (t & 1)) * (D * 32);
            s.j0 = 32 * t;
            s.need_mask = 32 * t + 32 > a.nb;
            return s;
        };
        run_steps<D, QT>(c, n_steps, src, row_stride_bytes, lds, wave, lane, sl2);
        finish_branch<D, QT>(c, a, 0, qb, head, wave, lane, lds);
    }

    // ---------------- selected branch: every token of the routed blocks
    {
        reset_branch<D, QT>(c);
        int my = lane < a.topk ? a.idx[(int64_t)qb * a.topk + lane] : -1;
        if (my >= a.nb) my = -1;
        const unsigned long long valid = __ballot(my >= 0);
        const int n_valid = __popcll(valid);
        const int rank = __popcll(valid & ((1ull << lane) - 1ull));
        // compact the valid entries to lanes 0..n_valid-1
        int packed = __builtin_amdgcn_ds_permute((my >= 0 ? rank : 63) * 4, my);
        if (n_valid == 64) packed = my;
        auto src = [&](int t) {
            int kb = __builtin_amdgcn_readlane(packed, t >> 1);
            TileSrc s;
            s.k_rows = a.k + (((int64_t)kb * 64 + 32 * (t & 1)) * a.h + head) * D;
            s.rows_valid = 32;
            s.v_t = a.v_t + (((int64_t)kb * a.h + head) * 2 + (t & 1)) * (D * 32);
            s.j0 = 0;
            s.need_mask = false;
            return s;
        };
        run_steps<D, QT>(c, 2 * n_valid, src, row_stride_bytes, lds, wave, lane, sl2);
        finish_branch<D, QT>(c, a, 1, qb, head, wave, lane, lds);
    }

    // ---------------- window branch: keys j with -W/2 <= j - i < W/2 inside the segment
    {
        reset_branch<D, QT>(c);
        const int q0 = qb * 64;
        int seg_lo = 0, seg_hi = 0;
        for (int s = 0; s < a.n_seg; ++s) {
            int lo = a.seg[s], hi = a.seg[s + 1];
            if (q0 >= lo && q0 < hi) {
                seg_lo = lo;
                seg_hi = hi;
            }
        }
        const int half = a.window / 2;
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            int i = q0 + 32 * (wave * QT + qt) + r;
            c.lo[qt] = max(seg_lo, i - half);
            c.hi[qt] = min(seg_hi, i + half);
        }
        // tile range of the whole query block (uniform over the workgroup)
        const int k_start = max(seg_lo, q0 - half);
        const int k_end = min(seg_hi, q0 + 63 + half);  // exclusive
        const int full_lo = max(seg_lo, q0 + 63 - half);
        const int full_hi = min(seg_hi, q0 + half);
        const int st0 = k_start / 32;
        const int n_steps = k_end > k_start ? (k_end - 1) / 32 - st0 + 1 : 0;
        auto src = [&](int t) {
            int st = st0 + t;
            TileSrc s;
            s.k_rows = a.k + ((int64_t)(32 * st) * a.h + head) * D;
            s.rows_valid = 32;
            s.v_t = a.v_t + (((int64_t)(st >> 1) * a.h + head) * 2 + (st & 1)) * (D * 32);
            s.j0 = 32 * st;
            s.need_mask = (32 * st < full_lo) || (32 * st + 32 > full_hi);
            return s;
        };
        run_steps<D, QT>(c, n_steps, src, row_stride_bytes, lds, wave, lane, sl2);
        finish_branch<D, QT>(c, a, 2, qb, head, wave, lane, lds);
    }
}

// Packs a [n_rows, H, D] bf16 tensor into per-block transposed sub-tiles:
//   dst[block][head][half][channel][slot][8]  with key t = 32 half + 8 (slot ^ ((channel >> 2) & 3)) + j
// Rows at or beyond n_rows read as zero.  One workgroup per (block, head).
template <int D>
__global__ __launch_bounds__(256) void pack_transposed(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst,
                                                       int64_t n_rows, int h) {
    __shared__ uint16_t tile[64][D + 2];
    const int64_t blk = blockIdx.x;
    const int head = blockIdx.y;
    constexpr int CH = D / 8;
    for (int e = threadIdx.x; e < 64 * CH; e += 256) {
        int t = e / CH, cc = e % CH;
        int64_t row = blk * 64 + t;
        uint4 val = make_uint4(0, 0, 0, 0);
        if (row < n_rows) val = *reinterpret_cast<const uint4 *>(src + (row * h + head) * D + cc * 8);
        uint32_t w[4] = {val.x, val.y, val.z, val.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            tile[t][cc * 8 + 2 * j] = (uint16_t)(w[j] & 0xffffu);
            tile[t][cc * 8 + 2 * j + 1] = (uint16_t)(w[j] >> 16);
        }
    }
    __syncthreads();
    uint16_t *out = dst + ((blk * h + head) * 2) * (int64_t)(D * 32);
    for (int e = threadIdx.x; e < 2 * D * 4; e += 256) {
        int half = e / (D * 4);
        int ch = (e / 4) % D;
        int slot = e % 4;
        int cidx = slot ^ ((ch >> 2) & 3);
        int t0 = 32 * half + 8 * cidx;
        uint32_t w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) w[j] = (uint32_t)tile[t0 + 2 * j][ch] | ((uint32_t)tile[t0 + 2 * j + 1][ch] << 16);
        *reinterpret_cast<uint4 *>(out + (int64_t)e * 8) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

struct WsLayout {
    size_t v_t, vc_t, gsum, total;
};

WsLayout ws_layout(const Shape &s) {
    WsLayout w;
    size_t off = 0;
    w.v_t = off;
    off += align_up((size_t)s.nb * 64 * s.h * s.d * 2, 256);
    w.vc_t = off;
    off += align_up((size_t)((s.nb + 63) / 64) * 64 * s.h * s.d * 2, 256);
    w.gsum = off;
    off += align_up((size_t)s.nb * 64 * s.h * s.d * 4, 256);
    w.total = off > 0 ? off : 256;
    return w;
}

template <int D, int QT>
lsrm_status launch_forward_d(const Shape &s, const int32_t *seg_host, int n_seg, FwdArgs a, const uint16_t *d_v,
                             const uint16_t *d_vc, char *ws, const WsLayout &w, hipStream_t st, hipEvent_t ev_start,
                             hipEvent_t ev_stop) {
    using G = Geo<D, QT>;
    for (int i = 0; i <= n_seg; ++i) a.seg[i] = seg_host[i];
    hipLaunchKernelGGL(pack_transposed<D>, dim3(s.nb, s.h), dim3(256), 0, st, d_v, (uint16_t *)(ws + w.v_t), s.n, s.h);
    LSRM_HIP_CHECK(hipGetLastError());
    hipLaunchKernelGGL(pack_transposed<D>, dim3((s.nb + 63) / 64, s.h), dim3(256), 0, st, d_vc,
                       (uint16_t *)(ws + w.vc_t), (int64_t)s.nb, s.h);
    LSRM_HIP_CHECK(hipGetLastError());
    a.v_t = (const uint16_t *)(ws + w.v_t);
    a.vc_t = (const uint16_t *)(ws + w.vc_t);
    a.gsum = (float *)(ws + w.gsum);
    a.units = s.nb * s.h;
    a.units_per_xcd = (a.units + 7) / 8;
    if (ev_start != nullptr) LSRM_HIP_CHECK(hipEventRecord(ev_start, st));
    hipLaunchKernelGGL((nsa_forward_kernel<D, QT>), dim3(a.units_per_xcd * 8), dim3(G::THREADS), G::LDS_BYTES, st, a);
    LSRM_HIP_CHECK(hipGetLastError());
    if (ev_stop != nullptr) LSRM_HIP_CHECK(hipEventRecord(ev_stop, st));
    return LSRM_OK;
}

}  // namespace

size_t forward_ws_bytes(const Shape &s) { return ws_layout(s).total; }

lsrm_status launch_forward(const Shape &s, const int32_t *seg_host, int n_seg, const uint16_t *d_q,
                           const uint16_t *d_k, const uint16_t *d_v, const uint16_t *d_kc, const uint16_t *d_vc,
                           const int32_t *d_idx, const float *d_gates, uint16_t *d_out, float *d_lse,
                           uint16_t *d_out_branch, void *d_ws, hipStream_t st, hipEvent_t ev_start,
                           hipEvent_t ev_stop) {
    if (s.nb == 0) return LSRM_OK;
    if (n_seg > kMaxSeg) return LSRM_ERR_UNSUPPORTED;
    FwdArgs a{};
    a.q = d_q;
    a.k = d_k;
    a.kc = d_kc;
    a.idx = d_idx;
    a.gates = d_gates;
    a.out = d_out;
    a.lse = d_lse;
    a.out_branch = d_out_branch;
    a.n = s.n;
    a.nb = s.nb;
    a.h = s.h;
    a.topk = s.topk;
    a.window = s.window;
    a.n_seg = n_seg;
    a.scale = s.scale;
    a.scale_log2e = s.scale * 1.4426950408889634f;
    WsLayout w = ws_layout(s);
    char *ws = reinterpret_cast<char *>(d_ws);
    if (s.d == 64) return launch_forward_d<64, 2>(s, seg_host, n_seg, a, d_v, d_vc, ws, w, st, ev_start, ev_stop);
    return launch_forward_d<128, 1>(s, seg_host, n_seg, a, d_v, d_vc, ws, w, st, ev_start, ev_stop);
}

}  // namespace lsrm
