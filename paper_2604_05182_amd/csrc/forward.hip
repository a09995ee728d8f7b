// NSA forward on gfx950 (App. A, Eq. nsa_1): compressed, selected and window attention,
// each its own softmax, combined by the gated sum, in one kernel.
//
// Work decomposition
//   One 512-thread workgroup owns NP = 4 consecutive query blocks of one head and carries
//   them through all three branches.  A wavefront holds 32 query rows (two wavefronts per
//   query block); its state fits 256 registers, so two wavefronts run per SIMD.  In the
//   compressed and window branches every K/V tile is copied to LDS once and used by all
//   four query blocks (a ring of 2 NP tile slots, refilled as soon as a slot is free); in
//   the selected branch each query block streams its own routed blocks (two stages of NP
//   slots).  Workgroups are numbered so that each of the 8 XCDs walks a contiguous range
//   of (head, query block) units: the L2 of an XCD then holds one head's pooled
//   keys/values and the neighbouring windows / routed blocks.
//
// Per 32-key step, per wavefront
//   S^T = K Q^T        v_mfma_f32_32x32x16_bf16, A = 32 keys x 16 channels, B = Q^T.
//                      With S transposed, each lane owns one query column, so the row
//                      max / row sum of the softmax are in-lane reductions plus one
//                      exchange between the two lane halves (v_permlane32_swap).
//   P^T -> bf16        the accumulator layout of S^T is already the B-operand layout of
//                      the next contraction once the key rows of the A operand are
//                      loaded in a fixed permutation (bits 2 and 3 of the row swapped),
//                      so P never leaves registers.
//   O^T += V^T P^T     A = 32 channels x 16 keys from a pre-transposed copy of V.
//   A wavefront issues in order and the matrix pipe takes one MFMA at a time, so MFMA and
//   VALU work only overlap if they alternate in program order.  The shared phases are
//   therefore software pipelined by hand over three tiles: the QK^T MFMAs of tile t+1 and
//   the PV MFMAs of tile t-1 are issued alternately, each followed by its share of the
//   exponentials of tile t (scheduling barriers keep the compiler from regrouping them).
//
// Data movement
//   K rows come straight from the caller's [N, H, d] tensor, V from a packed transposed
//   copy made once per call ([block][head][half][d][32 keys], 16-byte chunks XOR-swizzled
//   so that LDS reads are bank-conflict free).  Both are copied global -> LDS with
//   global_load_lds_dwordx4 (no VGPR staging; scalar base + per-lane 32-bit offset),
//   the copy instructions of a tile split over the wavefronts that share it, s_waitcnt
//   vmcnt placed by hand, and read back as ds_read_b128 MFMA fragments.
//   The gated sum of the branches is carried between branches in an fp32 scratch tile in
//   MFMA-fragment order (fully coalesced) instead of in registers; the final tile goes
//   through LDS so that the bf16 output rows are written as whole 16-byte chunks.
#include "lsrm_internal.h"

#include <type_traits>

#ifndef LSRM_QT64
#define LSRM_QT64 1
#endif
#ifndef LSRM_QT128
#define LSRM_QT128 1
#endif
#ifndef LSRM_PAR64
#define LSRM_PAR64 1
#endif
#ifndef LSRM_PAR128
#define LSRM_PAR128 0
#endif

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
    int units, units_per_xcd, groups_per_head;
    float scale_log2e, scale;
};

// NP = query blocks per workgroup, QT = 32-row query tiles per wavefront (1 or 2), so a query
// block is held by NW = 2 / QT wavefronts.
// LDS is a ring of 2 NP tile slots of 32 keys each (K rows, then the V^T slab).  The shared
// phases use it as one ring; the selected phase as two stages of NP slots.
template <int D_, int NP_, int QT_>
struct Geo {
    static constexpr int D = D_, NP = NP_, QT = QT_;
    static constexpr int NW = 2 / QT;           // wavefronts per query block
    static constexpr int ROWS = 32 * QT;        // query rows per wavefront
    static constexpr int NS = D / 16;           // 16-channel slabs of the QK^T contraction
    static constexpr int ND = D / 32;           // 32-channel tiles of the PV output
    static constexpr int K_BYTES = 32 * D * 2;  // 32 key rows
    static constexpr int V_BYTES = D * 64;      // D channel rows x 32 keys
    static constexpr int TILE = K_BYTES + V_BYTES;
    static constexpr int WAVES = NW * NP;
    static constexpr int THREADS = 64 * WAVES;
    static constexpr int WAVES_PER_SIMD = WAVES / 4;
    static constexpr int NSLOT = 2 * NP;        // tile slots in LDS
    static constexpr int K_INST = K_BYTES / 1024;  // 1 KB copy instructions per tile
    static constexpr int V_INST = V_BYTES / 1024;
    static constexpr int SH_IPT = (K_INST + V_INST) / WAVES;  // shared phases: copy instructions per wavefront and tile
    static constexpr int SH_K = K_INST % WAVES == 0 ? K_INST / WAVES : 1;  // of which key instructions (at most)
    static constexpr int PR_K = K_INST / NW;    // selected phase: a wavefront copies its share of its block's tile
    static constexpr int PR_V = V_INST / NW;
    static constexpr int KQ = NS < 4 ? NS : 4;  // operand fragments kept in registers (rolling queues)
    static constexpr int VQ = 2 * ND < 4 ? 2 * ND : 4;
    static constexpr int OUT_ROW = 2 * D + 8;   // padded bf16 row of the output staging (bytes)
    static constexpr int LDS_BYTES = NSLOT * TILE;
    static_assert(QT == 1 || QT == 2, "");
    static_assert(WAVES % 4 == 0 && WAVES * ROWS * OUT_ROW <= LDS_BYTES, "output staging must fit in the tile slots");
    static_assert(SH_IPT >= 1 && (K_INST + V_INST) % WAVES == 0 && NSLOT >= 6, "");
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

// s_waitcnt immediates (vmcnt is split over bits [3:0] and [15:14], expcnt is bits [6:4],
// lgkmcnt bits [11:8]; counters that are not waited for are left at their maxima)
constexpr int vmcnt_imm(int n) { return (n & 0xF) | ((n >> 4) << 14) | 0x0F70; }            // vmcnt <= n
constexpr int vm_lgkm_imm(int n) { return (n & 0xF) | ((n >> 4) << 14) | 0x0070; }          // vmcnt <= n, lgkmcnt == 0

// Workgroup barrier without the memory fence that __syncthreads() implies: the fence
// would wait for every outstanding copy (vmcnt(0)) and defeat the prefetch ring.  What
// must be visible is ordered by hand: a wavefront waits for its own copies (s_waitcnt
// vmcnt) and its own LDS reads (lgkmcnt) before the barrier and reads LDS only after it.
__device__ __forceinline__ void wg_barrier() { asm volatile("s_barrier" ::: "memory"); }

// Results of an MFMA become readable by VALU instructions only a fixed number of cycles
// after issue, and the hardware does not interlock that dependency: the compiler pads
// with s_nop, but it has been seen to misplace the padding when a branch separates the
// MFMA from its first VALU reader.  Every such (rare) path starts with this explicit
// settle instead; 24 wait states cover the 8-pass MFMA used here.
__device__ __forceinline__ void mfma_settle() { asm volatile("s_nop 15\n\ts_nop 7" ::: "memory"); }

struct TileSrc {
    const uint16_t *k_rows;  // row 0 of the 32-key tile, this head
    int rows_valid;          // rows >= rows_valid are clamped (their scores get masked)
    const uint16_t *v_t;     // packed transposed V tile, contiguous V_BYTES
};

template <class G>
struct WaveCtx {
    bf16x8 qf[G::QT][G::NS];
    f32x16 o[G::QT][G::ND];
    float m[G::QT], l[G::QT];
    int lo[G::QT], hi[G::QT];   // valid key range of this lane's queries in mask coordinates
    uint32_t kf_off[G::NS];     // per-lane LDS byte offsets (inside a tile slot) of the K and V^T fragments
    uint32_t vf_off[G::ND][2];
};

template <int D>
__device__ __forceinline__ void k_copy_geometry(int inst, int lane, uint32_t row_stride_bytes, int *row, int *chunk,
                                                uint32_t *off) {
    constexpr int ROWS_PER_INST = 1024 / (D * 2);
    constexpr int CHUNKS = D / 8;
    *row = inst * ROWS_PER_INST + lane / CHUNKS;
    *chunk = (lane % CHUNKS) ^ k_swz<D>(*row);
    *off = (uint32_t)(*row) * row_stride_bytes + (uint32_t)(*chunk) * 16u;
}

// Shared phases: the wavefronts of the workgroup split the K_INST + V_INST copy instructions
// of one tile evenly (SH_IPT each).
// Per-lane source geometry of a wavefront's K copy instructions in the shared phases.
template <class G>
struct SharedCopy {
    uint32_t koff[G::SH_K];
    int krow[G::SH_K], kchunk[G::SH_K];
    __device__ __forceinline__ void init(int wave, int lane, uint32_t row_stride_bytes) {
#pragma unroll
        for (int j = 0; j < G::SH_K; ++j)
            k_copy_geometry<G::D>((wave + G::WAVES * j) % G::K_INST, lane, row_stride_bytes, &krow[j], &kchunk[j],
                                  &koff[j]);
    }
};

template <class G>
__device__ __forceinline__ void issue_shared(const SharedCopy<G> &c, const TileSrc &t, uint32_t row_stride_bytes,
                                             char *slot, int wave, int lane) {
    const char *kbase = reinterpret_cast<const char *>(t.k_rows);
    const char *vbase = reinterpret_cast<const char *>(t.v_t);
    auto copy_k = [&](int j, int inst) {
        uint32_t off = c.koff[j];
        if (__builtin_expect(t.rows_valid < 32, 0)) {
            const int srow = c.krow[j] < t.rows_valid ? c.krow[j] : t.rows_valid - 1;
            off = (uint32_t)srow * row_stride_bytes + (uint32_t)c.kchunk[j] * 16u;
        }
        __builtin_amdgcn_global_load_lds(GLB_PTR(kbase + off), LDS_PTR(slot + inst * 1024), 16, 0, 0);
    };
    auto copy_v = [&](int inst) {
        __builtin_amdgcn_global_load_lds(GLB_PTR(vbase + inst * 1024 + (uint32_t)lane * 16u),
                                         LDS_PTR(slot + G::K_BYTES + inst * 1024), 16, 0, 0);
    };
    if constexpr (G::K_INST % G::WAVES == 0) {
        // every wavefront copies K_INST / WAVES key instructions and as many value instructions
#pragma unroll
        for (int j = 0; j < G::SH_K; ++j) copy_k(j, wave + G::WAVES * j);
#pragma unroll
        for (int j = 0; j < G::V_INST / G::WAVES; ++j) copy_v(wave + G::WAVES * j);
    } else {
        // fewer key instructions than wavefronts: the first K_INST wavefronts copy keys, the rest values
        static_assert(G::K_INST % G::WAVES == 0 || (G::SH_IPT == 1 && G::K_INST + G::V_INST == G::WAVES), "");
        if (wave < G::K_INST)
            copy_k(0, wave);
        else
            copy_v(wave - G::K_INST);
    }
}

// Selected phase: the NW wavefronts of a query block split the copies of their own tile.
template <class G>
__device__ __forceinline__ void issue_own(const uint32_t (&koff)[G::PR_K], const TileSrc &t, char *slot, int sub,
                                          int lane) {
    const char *kbase = reinterpret_cast<const char *>(t.k_rows);
    const char *vbase = reinterpret_cast<const char *>(t.v_t);
#pragma unroll
    for (int j = 0; j < G::PR_K; ++j) {
        const int i = sub + G::NW * j;
        __builtin_amdgcn_global_load_lds(GLB_PTR(kbase + koff[j]), LDS_PTR(slot + i * 1024), 16, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < G::PR_V; ++j) {
        const int i = sub + G::NW * j;
        __builtin_amdgcn_global_load_lds(GLB_PTR(vbase + i * 1024 + (uint32_t)lane * 16u),
                                         LDS_PTR(slot + G::K_BYTES + i * 1024), 16, 0, 0);
    }
}

template <class G>
__device__ __forceinline__ void reset_branch(WaveCtx<G> &c) {
#pragma unroll
    for (int qt = 0; qt < G::QT; ++qt) {
        c.m[qt] = kMinusHuge;
        c.l[qt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < G::ND; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) c.o[qt][dt][i] = 0.f;
    }
}

// ---- pieces of one 32-key step of one wavefront ------------------------------------------
template <class G>
__device__ __forceinline__ void read_k(const WaveCtx<G> &c, const char *slot, bf16x8 (&kf)[G::NS]) {
#pragma unroll
    for (int ks = 0; ks < G::NS; ++ks) kf[ks] = *reinterpret_cast<const bf16x8 *>(slot + c.kf_off[ks]);
}
template <class G>
__device__ __forceinline__ void read_v(const WaveCtx<G> &c, const char *slot, bf16x8 (&vf)[G::ND][2]) {
#pragma unroll
    for (int dt = 0; dt < G::ND; ++dt)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) vf[dt][ks] = *reinterpret_cast<const bf16x8 *>(slot + c.vf_off[dt][ks]);
}

// S^T = K Q^T for 32 keys x the 32 queries of row tile qt
template <class G>
__device__ __forceinline__ void qk_scores(const WaveCtx<G> &c, const bf16x8 (&kf)[G::NS], f32x16 (&s)[G::QT]) {
#pragma unroll
    for (int qt = 0; qt < G::QT; ++qt)
#pragma unroll
        for (int i = 0; i < 16; ++i) s[qt][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < G::NS; ++ks)
#pragma unroll
        for (int qt = 0; qt < G::QT; ++qt)
            s[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], c.qf[qt][ks], s[qt], 0, 0, 0);
}

// Keys outside [lo, hi) of this lane's query get a score of -inf.
__device__ __forceinline__ void mask_scores(int lo, int hi, f32x16 &s, int j0, int lane) {
    const int hh = lane >> 5;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        int j = j0 + 16 * (i / 8) + 8 * hh + (i % 8);
        if (j < lo || j >= hi) s[i] = -__builtin_inff();
    }
}

__device__ __forceinline__ float lane_max(const f32x16 &s) {
    float mx = fmaxf(s[0], s[1]);
#pragma unroll
    for (int i = 2; i < 16; i += 2) mx = fmaxf(mx, fmaxf(s[i], s[i + 1]));
    return mx;
}

// Folds the maximum of a new score tile into the running maximum of row tile qt.
//
// The running maximum m is allowed to lag: it is raised (and O, l rescaled) only when a
// new score exceeds it by more than kLag in the log2 domain, so probabilities stay
// below 2^kLag -- harmless in fp32 and bf16, whose exponent ranges are the same -- and
// the rescale of the O accumulators becomes a rare, wave-uniform branch.  m starts at
// kMinusHuge (finite), so the first real score always raises it and no inf - inf ever
// appears; a fully masked tile (maximum -inf) never does.
constexpr float kLag = 8.0f;

// `pending` (nullable) are probabilities that were computed against the old maximum but not
// yet accumulated into O (the software pipeline keeps one tile of them): they are rescaled
// together with O and l.
template <class G>
__device__ __forceinline__ void update_max(WaveCtx<G> &c, int qt, float mx_lane, float sl2, uint32_t *pending) {
    const float mx = half_max(mx_lane);
    const bool raise = (mx - c.m[qt]) * sl2 > kLag;
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(raise) != 0, 0)) {
        mfma_settle();  // the O accumulators may still be in flight
        float m_new = raise ? mx : c.m[qt];
        float alpha = raise ? __builtin_amdgcn_exp2f((c.m[qt] - m_new) * sl2) : 1.0f;
        c.m[qt] = m_new;
        c.l[qt] *= alpha;
#pragma unroll
        for (int dt = 0; dt < G::ND; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) c.o[qt][dt][i] *= alpha;
        if (pending != nullptr) {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                float lo = __uint_as_float(pending[k] << 16), hi = __uint_as_float(pending[k] & 0xffff0000u);
                pending[k] = pack_bf16(lo * alpha, hi * alpha);
            }
        }
    }
}

union BFrag {
    bf16x8 v;
    uint32_t u[4];
};

// The MFMA block of one step.  Up to three tiles are in flight in a wavefront:
//   QK   the QK^T MFMAs of the tile whose scores are produced now        (-> s_next)
//   exp  the exponentials of the tile whose scores `s` are complete, already masked and
//        folded into the running maximum                                  (-> pu, c.l)
//   PV   the V^T P^T MFMAs of the tile before that (probabilities pu_prev)
// A wavefront issues in order and the matrix pipe runs one MFMA at a time, so MFMA and VALU
// work only overlap when they alternate in program order: the QK and PV MFMAs are issued
// alternately and every MFMA is followed by its share of the exponentials (one v_exp, its
// fma and sum, half a bf16 pack at d = 128) -- about as many VALU cycles as the MFMA takes.
// The empty asm statements pin each result to its place in the program (the compiler
// otherwise sinks the arithmetic to its first use) and the scheduling barriers keep the
// machine scheduler from regrouping; neither emits an instruction.
// pu[qt][k] = bf16 pair (p[2k], p[2k+1]) of row tile qt: pu[qt][0..3] / [4..7] are the B
// operands of the two 16-key slabs of the PV contraction.
// The A operands come from two rolling queues of LDS fragments (kq: K rows, vq: V^T rows):
// the MFMA that consumes fragment i is followed by the ds_read of fragment i + queue depth
// of the same stream, which continues into the next tile (k_nxt / v_nxt), so the queues
// enter the next block already primed.  LDS reads are thereby spread under the MFMAs, and
// only a few fragments are live at a time.
template <class G, bool QK, bool PV>
__device__ __forceinline__ void mfma_block(WaveCtx<G> &c, const f32x16 (&s)[G::QT], bf16x8 (&kq)[G::KQ],
                                           f32x16 (&s_next)[G::QT], bf16x8 (&vq)[G::VQ],
                                           const uint32_t (&pu_prev)[G::QT][8], uint32_t (&pu)[G::QT][8], float sl2,
                                           const char *k_cur, const char *k_nxt, const char *v_cur,
                                           const char *v_nxt) {
    constexpr int QT = G::QT;
    constexpr int NQ = QK ? G::NS * QT : 0, NPV = PV ? 2 * G::ND * QT : 0, NG = NQ + NPV;
    constexpr int NE = 16 * QT;
    float mc[QT], psum[QT], p[NE];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        mc[qt] = c.m[qt] * sl2;
        psum[qt] = 0.f;
    }
    if constexpr (NG == 0) {
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            p[e] = __builtin_amdgcn_exp2f(s[e / 16][e % 16] * sl2 - mc[e / 16]);
            psum[e / 16] += p[e];
        }
#pragma unroll
        for (int k = 0; k < NE / 2; ++k) pu[k / 8][k % 8] = pack_bf16(p[2 * k], p[2 * k + 1]);
    } else {
        constexpr int E = NE / NG;  // exponentials per MFMA
        static_assert(E >= 1 && E * NG == NE, "");
        BFrag pb[QT][2];
        if (PV) {
#pragma unroll
            for (int qt = 0; qt < QT; ++qt)
#pragma unroll
                for (int k = 0; k < 8; ++k) pb[qt][k / 4].u[k % 4] = pu_prev[qt][k];
        }
        if (QK) {
#pragma unroll
            for (int qt = 0; qt < QT; ++qt)
#pragma unroll
                for (int i = 0; i < 16; ++i) s_next[qt][i] = 0.f;
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const bool do_qk = QK && (!PV || (g % 2) == 0);
            if (do_qk) {
                const int i = PV ? g / 2 : g;
                const int ks = i / QT, qt = i % QT;
                s_next[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kq[ks % G::KQ], c.qf[qt][ks], s_next[qt], 0, 0, 0);
                asm volatile("" : "+v"(s_next[qt]));
                if (qt == QT - 1) {
                    const int nf = ks + G::KQ;
                    kq[ks % G::KQ] =
                        *reinterpret_cast<const bf16x8 *>((nf < G::NS ? k_cur : k_nxt) + c.kf_off[nf % G::NS]);
                }
            } else {
                const int i = QK ? g / 2 : g;
                const int f = i / QT, qt = i % QT;
                const int ks = f / G::ND, dt = f % G::ND;
                c.o[qt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vq[f % G::VQ], pb[qt][ks].v, c.o[qt][dt], 0, 0, 0);
                asm volatile("" : "+v"(c.o[qt][dt]));
                if (qt == QT - 1) {
                    const int nf = (f + G::VQ) % (2 * G::ND);
                    vq[f % G::VQ] = *reinterpret_cast<const bf16x8 *>((f + G::VQ < 2 * G::ND ? v_cur : v_nxt) +
                                                                      c.vf_off[nf % G::ND][nf / G::ND]);
                }
            }
#pragma unroll
            for (int e = g * E; e < (g + 1) * E; ++e) {
                p[e] = __builtin_amdgcn_exp2f(s[e / 16][e % 16] * sl2 - mc[e / 16]);
                psum[e / 16] += p[e];
                if (e & 1) {
                    pu[e / 16][(e % 16) / 2] = pack_bf16(p[e - 1], p[e]);
                    asm volatile("" : "+v"(pu[e / 16][(e % 16) / 2]));
                } else {
                    asm volatile("" : "+v"(p[e]));
                }
            }
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) asm volatile("" : "+v"(psum[qt]));
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) c.l[qt] += psum[qt];
}

// O^T += V^T P^T of the last tile (pipeline drain): the queue holds its first fragments.
template <class G>
__device__ __forceinline__ void pv_drain(WaveCtx<G> &c, bf16x8 (&vq)[G::VQ], const uint32_t (&pu)[G::QT][8],
                                         const char *v_cur) {
    BFrag pb[G::QT][2];
#pragma unroll
    for (int qt = 0; qt < G::QT; ++qt)
#pragma unroll
        for (int k = 0; k < 8; ++k) pb[qt][k / 4].u[k % 4] = pu[qt][k];
#pragma unroll
    for (int f = 0; f < 2 * G::ND; ++f) {
        const int ks = f / G::ND, dt = f % G::ND;
#pragma unroll
        for (int qt = 0; qt < G::QT; ++qt)
            c.o[qt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vq[f % G::VQ], pb[qt][ks].v, c.o[qt][dt], 0, 0, 0);
        if (f + G::VQ < 2 * G::ND) {
            const int nf = f + G::VQ;
            vq[f % G::VQ] = *reinterpret_cast<const bf16x8 *>(v_cur + c.vf_off[nf % G::ND][nf / G::ND]);
        }
    }
}

// Exponentials of the scores of one row tile against its running maximum -> bf16 pairs.
template <class G>
__device__ __forceinline__ void exp_tile(WaveCtx<G> &c, int qt, const f32x16 &s, uint32_t (&pu)[8], float sl2) {
    const float mc = c.m[qt] * sl2;
    float psum = 0.f, p[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        p[e] = __builtin_amdgcn_exp2f(s[e] * sl2 - mc);
        psum += p[e];
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) pu[k] = pack_bf16(p[2 * k], p[2 * k + 1]);
    c.l[qt] += psum;
}

// PV of row tile 0 (probabilities pu0) with the exponentials of row tile 1 in its shadow.
template <class G>
__device__ __forceinline__ void pv0_exp1(WaveCtx<G> &c, const bf16x8 (&vf)[G::ND][2], const uint32_t (&pu0)[8],
                                         const f32x16 &s1, uint32_t (&pu1)[8], float sl2) {
    constexpr int NG = 2 * G::ND, E = 16 / NG;
    BFrag pb[2];
#pragma unroll
    for (int k = 0; k < 8; ++k) pb[k / 4].u[k % 4] = pu0[k];
    const float mc = c.m[1] * sl2;
    float psum = 0.f, p[16];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const int ks = g / G::ND, dt = g % G::ND;
        c.o[0][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt][ks], pb[ks].v, c.o[0][dt], 0, 0, 0);
#pragma unroll
        for (int e = g * E; e < (g + 1) * E; ++e) {
            p[e] = __builtin_amdgcn_exp2f(s1[e] * sl2 - mc);
            psum += p[e];
            if (e & 1) {
                pu1[e / 2] = pack_bf16(p[e - 1], p[e]);
                asm volatile("" : "+v"(pu1[e / 2]));
            } else {
                asm volatile("" : "+v"(p[e]));
            }
        }
        asm volatile("" : "+v"(psum));
        __builtin_amdgcn_sched_barrier(0);
    }
    c.l[1] += psum;
}

template <class G>
__device__ __forceinline__ void pv_tile(WaveCtx<G> &c, int qt, const bf16x8 (&vf)[G::ND][2], const uint32_t (&pu)[8]) {
    BFrag pb[2];
#pragma unroll
    for (int k = 0; k < 8; ++k) pb[k / 4].u[k % 4] = pu[k];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int dt = 0; dt < G::ND; ++dt)
            c.o[qt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt][ks], pb[ks].v, c.o[qt][dt], 0, 0, 0);
}

// Non-pipelined step (selected phase): fragments, scores, softmax and PV of one tile in
// sequence; with two row tiles the exponentials of the second run under the PV of the first.
template <class G>
__device__ __forceinline__ void step_compute(WaveCtx<G> &c, const char *slot, int lane, float sl2) {
    bf16x8 kf[G::NS];
    bf16x8 vf[G::ND][2];
    read_k<G>(c, slot, kf);
    read_v<G>(c, slot, vf);
    f32x16 s[G::QT];
    qk_scores<G>(c, kf, s);
#pragma unroll
    for (int qt = 0; qt < G::QT; ++qt) update_max<G>(c, qt, lane_max(s[qt]), sl2, nullptr);
    uint32_t pu[G::QT][8];
    exp_tile<G>(c, 0, s[0], pu[0], sl2);
    if constexpr (G::QT == 2) {
        pv0_exp1<G>(c, vf, pu[0], s[1], pu[1], sl2);
        pv_tile<G>(c, 1, vf, pu[1]);
    } else {
        pv_tile<G>(c, 0, vf, pu[0]);
    }
}

// Shared phase (compressed and window branches): every tile is used by all query blocks of
// the workgroup.  Tiles go through the ring of NSLOT slots; a slot is refilled as soon as
// every wavefront is done with it.
//   src(t)  -> TileSrc of tile t (uniform over the workgroup)
//   msk(t)  -> (j0, need_mask) of tile t for this wavefront
// Step t runs mfma_block with QK of tile t+1, the exponentials of tile t and PV of tile t-1,
// reloading its operand registers on the fly with the K fragments of tile t+2 and the V
// fragments of tile t.  After the block (one barrier per step) the slot of tile t-1 is
// refilled with tile t-1+NSLOT and the maximum of tile t+1 is folded into the running
// maximum.  Every wavefront runs every step: a tile outside a wavefront's own key range is
// simply fully masked (the step body is kept unconditional on purpose -- a conditional
// update of the accumulator tuples makes the compiler shuffle them through copies).
// Scores and probabilities alternate between two register sets (index = tile parity), so
// nothing is copied from step to step.
template <class G, typename SrcFn, typename MaskFn>
__device__ __forceinline__ void run_shared(WaveCtx<G> &c, int n_steps, SrcFn src, MaskFn msk,
                                           uint32_t row_stride_bytes, char *lds, int wave, int lane, float sl2) {
    constexpr int R = G::NSLOT, QT = G::QT;
    constexpr bool PAR = G::D == 64 ? LSRM_PAR64 : LSRM_PAR128;
    if (n_steps <= 0) return;
    auto slot = [&](int t) { return lds + (t % R) * G::TILE; };
    SharedCopy<G> cp;
    cp.init(wave, lane, row_stride_bytes);
    __builtin_amdgcn_s_waitcnt(vm_lgkm_imm(0));
    wg_barrier();  // every wavefront is done with the slots (previous phase)
    for (int t = 0; t < R && t < n_steps; ++t) issue_shared<G>(cp, src(t), row_stride_bytes, slot(t), wave, lane);
    // tiles 0, 1 and 2 must have landed before the first block reads them
    if (n_steps >= R)
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((R - 3) * G::SH_IPT));
    else
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    wg_barrier();
    bf16x8 kq[G::KQ], vq[G::VQ];
    f32x16 S[2][QT];         // scores
    uint32_t P[2][QT][8];    // probabilities
    int j0;
    bool need_mask;
    {
        bf16x8 kf[G::NS];
        read_k<G>(c, slot(0), kf);
        qk_scores<G>(c, kf, S[0]);
    }
    // prime the queues: first K fragments of tile 1 (stale but finite data if there is none), first V fragments of tile 0
#pragma unroll
    for (int i = 0; i < G::KQ; ++i) kq[i] = *reinterpret_cast<const bf16x8 *>(slot(1) + c.kf_off[i]);
#pragma unroll
    for (int f = 0; f < G::VQ; ++f) vq[f] = *reinterpret_cast<const bf16x8 *>(slot(0) + c.vf_off[f % G::ND][f / G::ND]);
    msk(0, &j0, &need_mask);
    mfma_settle();  // a branch follows the MFMAs that produced the scores
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        if (need_mask) mask_scores(c.lo[qt], c.hi[qt], S[0][qt], j0, lane);
        update_max<G>(c, qt, lane_max(S[0][qt]), sl2, nullptr);
    }

    // What follows every MFMA block but the last: sync, refill a slot, fold the maximum of
    // the scores just produced (s_next); pu are the probabilities still to be accumulated.
    auto after_block = [&](int t, f32x16 (&s_next)[QT], uint32_t (&pu)[QT][8]) {
        // Before the barrier this wavefront's LDS reads have returned and its share of tile
        // t+3 (read during the next block) has landed; later tiles may stay in flight.
        // Copies issued so far: tiles 0 .. t-2+R.  Near the end fewer are outstanding: wait for all.
        if (t - 2 + R < n_steps && t >= 1)
            __builtin_amdgcn_s_waitcnt(vm_lgkm_imm((R - 5) * G::SH_IPT));
        else if (t == 0 && n_steps >= R)
            __builtin_amdgcn_s_waitcnt(vm_lgkm_imm((R - 4) * G::SH_IPT));
        else
            __builtin_amdgcn_s_waitcnt(vm_lgkm_imm(0));
        wg_barrier();  // tile t+3 has landed for everyone; everyone has fetched the fragments of tile t-1
        if (t >= 1 && t - 1 + R < n_steps)
            issue_shared<G>(cp, src(t - 1 + R), row_stride_bytes, slot(t - 1), wave, lane);
        msk(t + 1, &j0, &need_mask);
        mfma_settle();  // s_next and O come from the MFMAs just issued; branches follow
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            if (__builtin_expect(need_mask, 0)) mask_scores(c.lo[qt], c.hi[qt], s_next[qt], j0, lane);
            update_max<G>(c, qt, lane_max(s_next[qt]), sl2, pu[qt]);
        }
    };
    // Scores and probabilities of tile t live in S[A], P[A]: with PAR, A is the parity of t and
    // nothing is copied from step to step; without, A = 0 and the sets are copied after a step.
    auto rotate = [&]() {
        if (!PAR) {
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) {
                S[0][qt] = S[1][qt];
#pragma unroll
                for (int k = 0; k < 8; ++k) P[1][qt][k] = P[0][qt][k];
            }
        }
    };
    // QK(t+1) || exp(t) || PV(t-1); the queues move on to K(t+2) and V(t)  (stale slots past the end: unused)
    auto full_step = [&](auto par, int t) {
        constexpr int A = PAR ? decltype(par)::value : 0;
        mfma_block<G, true, true>(c, S[A], kq, S[A ^ 1], vq, P[A ^ 1], P[A], sl2, slot(t + 1), slot(t + 2),
                                  slot(t - 1), slot(t));
        after_block(t, S[A ^ 1], P[A]);
        rotate();
    };
    // exp(n-1) || PV(n-2); then the drain: PV of the last tile
    auto last_step = [&](auto par, int t) {
        constexpr int A = PAR ? decltype(par)::value : 0;
        mfma_block<G, false, true>(c, S[A], kq, S[A ^ 1], vq, P[A ^ 1], P[A], sl2, nullptr, nullptr, slot(t - 1),
                                   slot(t));
        pv_drain<G>(c, vq, P[A], slot(t));
    };
    using Even = std::integral_constant<int, 0>;
    using Odd = std::integral_constant<int, 1>;

    if (n_steps >= 2) {
        // QK(1) || exp(0)
        mfma_block<G, true, false>(c, S[0], kq, S[1], vq, P[1], P[0], sl2, slot(1), slot(2), nullptr, nullptr);
        after_block(0, S[1], P[0]);
        rotate();
        if constexpr (PAR) {
            int t = 1;
            for (; t + 2 < n_steps; t += 2) {
                full_step(Odd{}, t);
                full_step(Even{}, t + 1);
            }
            if (t + 1 < n_steps) {
                full_step(Odd{}, t);
                last_step(Even{}, t + 1);
            } else {
                last_step(Odd{}, t);
            }
        } else {
            for (int t = 1; t + 1 < n_steps; ++t) full_step(Even{}, t);
            last_step(Even{}, n_steps - 1);
        }
    } else {
        mfma_block<G, false, false>(c, S[0], kq, S[1], vq, P[1], P[0], sl2, nullptr, nullptr, nullptr, nullptr);
        pv_drain<G>(c, vq, P[0], slot(0));
    }
}

// Selected phase: each query block streams its own routed blocks in 32-key steps through
// two stages of NP slots, copied ahead.
//   One wavefront per query block: nothing is shared, so the wavefronts run free of each
//   other between the barrier that opens the phase and the one that opens the next.
//   Two wavefronts per query block: they split the copies and meet at a workgroup barrier
//   every step; a block whose list is shorter than the longest of the workgroup keeps
//   meeting the barriers (second loop) without computing.
template <class G, typename SrcFn>
__device__ __forceinline__ void run_own(WaveCtx<G> &c, int n_steps, int my_steps, SrcFn src,
                                        uint32_t row_stride_bytes, char *lds, int qbi, int sub, int lane, float sl2) {
    constexpr int NP = G::NP;
    if (n_steps <= 0) return;
    uint32_t koff[G::PR_K];  // per-lane source offsets of this wavefront's K copy instructions
#pragma unroll
    for (int j = 0; j < G::PR_K; ++j) {
        int row, chunk;
        k_copy_geometry<G::D>(sub + G::NW * j, lane, row_stride_bytes, &row, &chunk, &koff[j]);
    }
    __builtin_amdgcn_s_waitcnt(vm_lgkm_imm(0));
    wg_barrier();
    if constexpr (G::NW == 1) {
        constexpr int IPT = G::PR_K + G::PR_V;
        char *stage[2] = {lds + qbi * G::TILE, lds + (NP + qbi) * G::TILE};
        if (my_steps > 0) issue_own<G>(koff, src(0), stage[0], 0, lane);
        if (my_steps > 1) issue_own<G>(koff, src(1), stage[1], 0, lane);
        for (int t = 0; t < my_steps; ++t) {
            // tile t has landed (the copies of tile t+1 may stay in flight)
            if (t + 1 < my_steps)
                __builtin_amdgcn_s_waitcnt(vmcnt_imm(IPT));
            else
                __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            bf16x8 kf[G::NS];
            bf16x8 vf[G::ND][2];
            read_k<G>(c, stage[t & 1], kf);
            read_v<G>(c, stage[t & 1], vf);
            f32x16 s[G::QT];
            qk_scores<G>(c, kf, s);
            // the fragments are in registers: the slot can take the tile after next
            __builtin_amdgcn_s_waitcnt(vm_lgkm_imm(63));
            if (t + 2 < my_steps) issue_own<G>(koff, src(t + 2), stage[t & 1], 0, lane);
            mfma_settle();
#pragma unroll
            for (int qt = 0; qt < G::QT; ++qt) update_max<G>(c, qt, lane_max(s[qt]), sl2, nullptr);
            uint32_t pu[G::QT][8];
            exp_tile<G>(c, 0, s[0], pu[0], sl2);
            if constexpr (G::QT == 2) {
                pv0_exp1<G>(c, vf, pu[0], s[1], pu[1], sl2);
                pv_tile<G>(c, 1, vf, pu[1]);
            } else {
                pv_tile<G>(c, 0, vf, pu[0]);
            }
        }
    } else {
        if (my_steps > 0) issue_own<G>(koff, src(0), lds + qbi * G::TILE, sub, lane);
        for (int t = 0; t < my_steps; ++t) {
            __builtin_amdgcn_s_waitcnt(vm_lgkm_imm(0));
            wg_barrier();
            if (t + 1 < my_steps)
                issue_own<G>(koff, src(t + 1), lds + (((t + 1) & 1) * NP + qbi) * G::TILE, sub, lane);
            step_compute<G>(c, lds + ((t & 1) * NP + qbi) * G::TILE, lane, sl2);
        }
        for (int t = my_steps; t < n_steps; ++t) {
            __builtin_amdgcn_s_waitcnt(vm_lgkm_imm(0));
            wg_barrier();
        }
    }
}

// Ends a branch: normalises, applies the gate and folds the result into the running
// gated sum kept in the fp32 scratch tile (written by branch 0, updated by branch 1,
// consumed by branch 2, which converts to bf16 and stores the output rows through LDS).
// Optionally stores the un-gated branch output and its log-sum-exp.
template <class G>
__device__ __forceinline__ void finish_branch(WaveCtx<G> &c, const FwdArgs &a, int branch, int64_t row0, int head,
                                              int wave, int lane, char *lds) {
    constexpr int D = G::D;
    const int r = lane & 31, hh = lane >> 5;
    char *tr = lds + wave * G::ROWS * G::OUT_ROW;  // output staging region of this wavefront
#pragma unroll
    for (int qt = 0; qt < G::QT; ++qt) {
        const int64_t row = row0 + 32 * qt + r;
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
        f32x4 *gs = reinterpret_cast<f32x4 *>(a.gsum) + ((((row0 >> 5) + qt) * a.h + head) * (G::ND * 4)) * 64 + lane;
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
                    *reinterpret_cast<uint2 *>(tr + (32 * qt + r) * G::OUT_ROW + (32 * dt + 8 * gq + 4 * hh) * 2) = w2;
                }
            }
        }
    }
    if (branch == 2) {
        // rows of this wavefront back from LDS as whole 16-byte chunks: 4 (d=128) or 8 (d=64) rows per pass
        constexpr int CH = D / 8;
        constexpr int RPP = 64 / CH;
#pragma unroll
        for (int it = 0; it < G::ROWS / RPP; ++it) {
            const int rr = it * RPP + lane / CH, ch = lane % CH;
            uint4 val = *reinterpret_cast<const uint4 *>(tr + rr * G::OUT_ROW + ch * 16);
            *reinterpret_cast<uint4 *>(a.out + ((row0 + rr) * a.h + head) * D + ch * 8) = val;
        }
    }
}

// Window geometry of one query block (all values uniform over its wavefronts).
struct WinRange {
    int seg_lo, seg_hi;    // segment of the block
    int full_lo, full_hi;  // keys inside [full_lo, full_hi) are visible to all 64 queries of the block
    int st0, st1;          // 32-key tiles [st0, st1) intersect the block's window
};

__device__ __forceinline__ WinRange window_range(const FwdArgs &a, int qb) {
    WinRange w;
    const int q0 = qb * 64;
    w.seg_lo = 0;
    w.seg_hi = 0;
    for (int s = 0; s < a.n_seg; ++s) {
        int lo = a.seg[s], hi = a.seg[s + 1];
        if (q0 >= lo && q0 < hi) {
            w.seg_lo = lo;
            w.seg_hi = hi;
        }
    }
    const int half = a.window / 2;
    const int k_start = max(w.seg_lo, q0 - half);
    const int k_end = min(w.seg_hi, q0 + 63 + half);  // exclusive
    w.full_lo = max(w.seg_lo, q0 + 63 - half);
    w.full_hi = min(w.seg_hi, q0 + half);
    w.st0 = k_start / 32;
    w.st1 = k_end > k_start ? (k_end - 1) / 32 + 1 : w.st0;
    return w;
}

template <class G>
__global__ __launch_bounds__((G::THREADS), (G::WAVES_PER_SIMD)) void nsa_forward_kernel(FwdArgs a) {
    constexpr int D = G::D, NP = G::NP;
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    // XCD-aware numbering: hardware deals consecutive workgroups round-robin to the 8 XCDs
    const int xcd = blockIdx.x & 7, slot_id = blockIdx.x >> 3;
    if (slot_id >= a.units_per_xcd) return;
    const int unit = xcd * a.units_per_xcd + slot_id;
    if (unit >= a.units) return;
    const int head = unit / a.groups_per_head;
    const int group = unit % a.groups_per_head;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int qbi = wave / G::NW, sub = wave % G::NW;  // query block inside the group, wavefront inside the block
    const int r = lane & 31, hh = lane >> 5;
    const int qb = group * NP + qbi;
    const bool active = qb < a.nb;  // a trailing group may have fewer than NP query blocks
    const int64_t row0 = (int64_t)(active ? qb : 0) * 64 + G::ROWS * sub;
    const uint32_t row_stride_bytes = (uint32_t)a.h * D * 2;
    const float sl2 = a.scale_log2e;

    WaveCtx<G> c;
    {
        const int r_perm = (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1);
        const int ksw = k_swz<D>(r_perm);
#pragma unroll
        for (int ks = 0; ks < G::NS; ++ks) c.kf_off[ks] = r_perm * (2 * D) + (((2 * ks + hh) ^ ksw) * 16);
#pragma unroll
        for (int dt = 0; dt < G::ND; ++dt) {
            const int row = 32 * dt + r;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
                c.vf_off[dt][ks] = G::K_BYTES + row * 64 + (((2 * ks + hh) ^ ((row >> 2) & 3)) * 16);
        }
    }
    // A fully masked step may read a slot that no copy has filled yet: make sure it holds
    // finite values (0 * NaN would poison the accumulators).
    for (int off = threadIdx.x * 16; off < G::LDS_BYTES; off += G::THREADS * 16)
        *reinterpret_cast<uint4 *>(lds + off) = make_uint4(0, 0, 0, 0);
    {
        // (an inactive wavefront reads the rows of block 0: finite values, results discarded)
#pragma unroll
        for (int qt = 0; qt < G::QT; ++qt) {
            const uint16_t *qrow = a.q + ((row0 + 32 * qt + r) * a.h + head) * D + 8 * hh;
#pragma unroll
            for (int ks = 0; ks < G::NS; ++ks) c.qf[qt][ks] = *reinterpret_cast<const bf16x8 *>(qrow + 16 * ks);
        }
    }

    // ---------------- compressed branch: all NB pooled pairs
    {
        reset_branch<G>(c);
#pragma unroll
        for (int qt = 0; qt < G::QT; ++qt) {
            c.lo[qt] = 0;
            c.hi[qt] = a.nb;
        }
        const int n_steps = (a.nb + 31) / 32;
        auto src = [&](int t) {
            TileSrc s;
            s.k_rows = a.kc + ((int64_t)(32 * t) * a.h + head) * D;
            s.rows_valid = a.nb - 32 * t;
            s.v_t = a.vc_t + (((int64_t)(t >> 1) * a.h + head) * 2 + (t & 1)) * (D * 32);
            return s;
        };
        auto msk = [&](int t, int *j0, bool *need) {
            *j0 = 32 * t;
            *need = 32 * t + 32 > a.nb;
        };
        run_shared<G>(c, n_steps, src, msk, row_stride_bytes, lds, wave, lane, sl2);
        if (active) finish_branch<G>(c, a, 0, row0, head, wave, lane, lds);
    }

    // ---------------- selected branch: every token of the routed blocks
    {
        reset_branch<G>(c);
        int packed = -1, my_valid = 0, max_valid = 0;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int qbp = group * NP + p;
            int v = (qbp < a.nb && lane < a.topk) ? a.idx[(int64_t)qbp * a.topk + lane] : -1;
            if (v >= a.nb) v = -1;
            const unsigned long long valid = __ballot(v >= 0);
            const int n_valid = __popcll(valid);
            max_valid = max(max_valid, n_valid);
            if (p == qbi) {
                // compact the valid entries of this block's row to lanes 0..n_valid-1
                const int rank = __popcll(valid & ((1ull << lane) - 1ull));
                packed = __builtin_amdgcn_ds_permute((v >= 0 ? rank : 63) * 4, v);
                if (n_valid == 64) packed = v;
                my_valid = n_valid;
            }
        }
        auto src = [&](int t) {
            int kb = __builtin_amdgcn_readlane(packed, t >> 1);
            TileSrc s;
            s.k_rows = a.k + (((int64_t)kb * 64 + 32 * (t & 1)) * a.h + head) * D;
            s.rows_valid = 32;
            s.v_t = a.v_t + (((int64_t)kb * a.h + head) * 2 + (t & 1)) * (D * 32);
            return s;
        };
        run_own<G>(c, 2 * max_valid, 2 * my_valid, src, row_stride_bytes, lds, qbi, sub, lane, sl2);
        if (active) finish_branch<G>(c, a, 1, row0, head, wave, lane, lds);
    }

    // ---------------- window branch: keys j with -W/2 <= j - i < W/2 inside the segment
    {
        reset_branch<G>(c);
        WinRange mine = window_range(a, active ? qb : 0);
        int st_min = 0x7fffffff, st_max = 0;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int qbp = group * NP + p;
            if (qbp < a.nb) {
                WinRange w = window_range(a, qbp);
                if (w.st1 > w.st0) {
                    st_min = min(st_min, w.st0);
                    st_max = max(st_max, w.st1);
                }
            }
        }
        {
            const int half_w = a.window / 2;
#pragma unroll
            for (int qt = 0; qt < G::QT; ++qt) {
                const int i = (int)row0 + 32 * qt + r;
                c.lo[qt] = max(mine.seg_lo, i - half_w);
                c.hi[qt] = min(mine.seg_hi, i + half_w);
            }
        }
        const int n_steps = st_max > st_min ? st_max - st_min : 0;
        auto src = [&](int t) {
            int st = st_min + t;
            TileSrc s;
            s.k_rows = a.k + ((int64_t)(32 * st) * a.h + head) * D;
            s.rows_valid = 32;
            s.v_t = a.v_t + (((int64_t)(st >> 1) * a.h + head) * 2 + (st & 1)) * (D * 32);
            return s;
        };
        auto msk = [&](int t, int *j0, bool *need) {
            int st = st_min + t;
            *j0 = 32 * st;
            *need = (32 * st < mine.full_lo) || (32 * st + 32 > mine.full_hi);  // also true outside [st0, st1)
        };
        run_shared<G>(c, n_steps, src, msk, row_stride_bytes, lds, wave, lane, sl2);
        __builtin_amdgcn_s_waitcnt(vm_lgkm_imm(0));
        wg_barrier();  // the tile slots are about to be reused for the output rows
        if (active) finish_branch<G>(c, a, 2, row0, head, wave, lane, lds);
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

template <class G>
lsrm_status launch_forward_d(const Shape &s, const int32_t *seg_host, int n_seg, FwdArgs a, const uint16_t *d_v,
                             const uint16_t *d_vc, char *ws, const WsLayout &w, hipStream_t st, hipEvent_t ev_start,
                             hipEvent_t ev_stop) {
    constexpr int D = G::D, NP = G::NP;
    for (int i = 0; i <= n_seg; ++i) a.seg[i] = seg_host[i];
    hipLaunchKernelGGL(pack_transposed<D>, dim3(s.nb, s.h), dim3(256), 0, st, d_v, (uint16_t *)(ws + w.v_t), s.n, s.h);
    LSRM_HIP_CHECK(hipGetLastError());
    hipLaunchKernelGGL(pack_transposed<D>, dim3((s.nb + 63) / 64, s.h), dim3(256), 0, st, d_vc,
                       (uint16_t *)(ws + w.vc_t), (int64_t)s.nb, s.h);
    LSRM_HIP_CHECK(hipGetLastError());
    a.v_t = (const uint16_t *)(ws + w.v_t);
    a.vc_t = (const uint16_t *)(ws + w.vc_t);
    a.gsum = (float *)(ws + w.gsum);
    a.groups_per_head = (s.nb + NP - 1) / NP;
    a.units = a.groups_per_head * s.h;
    a.units_per_xcd = (a.units + 7) / 8;
    static bool attr_set = false;
    if (!attr_set) {
        LSRM_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(&nsa_forward_kernel<G>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_BYTES));
        attr_set = true;
    }
    if (ev_start != nullptr) LSRM_HIP_CHECK(hipEventRecord(ev_start, st));
    hipLaunchKernelGGL((nsa_forward_kernel<G>), dim3(a.units_per_xcd * 8), dim3(G::THREADS), G::LDS_BYTES, st, a);
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
    if (s.d == 64) return launch_forward_d<Geo<64, 4, LSRM_QT64>>(s, seg_host, n_seg, a, d_v, d_vc, ws, w, st, ev_start, ev_stop);
    return launch_forward_d<Geo<128, 4, LSRM_QT128>>(s, seg_host, n_seg, a, d_v, d_vc, ws, w, st, ev_start, ev_stop);
}

}  // namespace lsrm
