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
//   keys/values and the neighbouring windows / routed blocks.  With grouped-query heads the
//   query heads that share a key/value head are consecutive, hence run back to back on the
//   same tile images.
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
//   VALU work only overlap if they alternate in program order.  All phases are
//   therefore software pipelined by hand over three tiles: the QK^T MFMAs of tile t+1 and
//   the PV MFMAs of tile t-1 are issued alternately, each followed by its share of the
//   exponentials of tile t (scheduling barriers keep the compiler from regrouping them).
//
// Data movement
//   K and V are repacked once per call into tile images: per (head, 32-key tile) the exact
//   bytes of an LDS slot, K fragments then V^T fragments in MFMA operand order (see
//   issue_shared), head-major so that one head's keys and values are one contiguous range.
//   Tiles are copied global -> LDS with global_load_lds_dwordx4 (no VGPR staging), 1 KB
//   contiguous on both sides per instruction, the copy instructions of a tile split over
//   the wavefronts that share it, s_waitcnt vmcnt placed by hand, and read back as
//   conflict-free ds_read_b128 MFMA fragments.
//   The gated sum of the branches is carried between branches in registers at d <= 64 and, at d = 128,
//   where they do not suffice, in a bf16 scratch tile in MFMA-fragment order (fully coalesced); the
//   final tile goes through LDS so that the bf16 output rows are written as whole 16-byte chunks.
#include "lsrm_internal.h"

#include <type_traits>

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
    const uint16_t *q;
    const char *kv, *kvc;  // packed tile images of (k, v) and of the pooled (kc, vc)
    const int32_t *idx;    // routing table [NB, topk]
    const int32_t *sched;  // d = 128: the routing rows in step order, block id | owner << 28 (schedule.hip)
    const float *gates;
    int32_t seg[kMaxSeg + 1];  // window segment offsets (tokens)
    uint16_t *out;
    float *lse;
    uint16_t *out_branch;
    uint16_t *gsum;  // d = 128: scratch for the running gated sum, bf16 in accumulator-fragment order
    int64_t n;
    int nb, h, topk, window, n_seg;
    int nbc;                 // compressed pairs (spatial blocks): nb unless blocks are grouped
    const int32_t *blk_seg;  // nullable [nb][2]: window segment (first and end token) of every block, instead of `seg`
    int h_kv, group;    // key/value heads; query heads per key/value head (query head i reads head i / group)
    int gate_channels;  // gates are [N, 3, H, d] (one per output channel) instead of [N, H, 3]
    int own_block;      // the window branch sees the query's own block (App. A) instead of a sliding window
    const int32_t *count;  // nullable [NB]: active tokens per block (its first count[b] slots)
    int groups_per_head, groups_per_xcd;  // query-block groups of one head, and the share of one XCD
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
    // tile slots in LDS: NST per query block; the selected phase copies NST - 1 steps ahead.  The 16 KB tiles of
    // d = 128 fill the LDS with two stages; four stages for the smaller tiles of d <= 64 were measured: 0.7 %
    // faster at d = 64 with 180 K tokens, 1 % slower with 57 K, 6 % slower at d = 32 -- hence two everywhere.
    static constexpr int NST = 2;
    static constexpr int NSLOT = NST * NP;
    static constexpr int T_INST = TILE / 1024;  // 1 KB copy instructions per tile
    // shared phases: copy instructions per wavefront and tile (a small tile, d = 32, has fewer
    // instructions than the workgroup has wavefronts: the first T_INST wavefronts issue one each
    // and the others none, whose waits for SH_IPT copies per tile are then trivially met)
    static constexpr int SH_IPT = T_INST >= WAVES ? T_INST / WAVES : 1;
    static constexpr int KQ = 2, VQ = 2;        // operand fragments kept in registers (rolling queues)
    static constexpr int OUT_ROW = 2 * D + 8;   // padded bf16 row of the output staging (bytes)
    static constexpr bool GSUM_REGS = D_ <= 64; // the running gated sum fits the registers beside the accumulators
    // d = 128: the running gated sum of the first GSUM_LDS_WAVES wavefronts stays in the LDS the ring leaves free
    // (8 KB each in bf16: 32 of the CU's 160 KB), the others' goes through the scratch buffer in memory
    static constexpr int GSUM_LDS_WAVES = GSUM_REGS ? 0 : 4;
    static constexpr int GSUM_LDS_BYTES = 32 * D_ * 2;  // per wavefront
    static constexpr int LDS_BYTES = NSLOT * TILE;
    static_assert(QT == 1 || QT == 2, "");
    static_assert(WAVES % 4 == 0 && WAVES * ROWS * OUT_ROW <= LDS_BYTES, "output staging must fit in the tile slots");
    static_assert((T_INST % WAVES == 0 || WAVES % T_INST == 0) && T_INST % NW == 0 && NSLOT >= 7, "");
};

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
constexpr int kLgkmOnly = 0xC07F;                                                            // lgkmcnt == 0, vmcnt left alone

// Bare workgroup barrier.  No barrier, fenced or not, waits for global -> LDS copies in flight
// (they are counted by vmcnt, which a workgroup-scope fence leaves alone), so what must be
// visible is ordered by hand: a wavefront waits for its own copies (s_waitcnt vmcnt, counted so
// that later tiles stay in flight) and its own LDS reads (lgkmcnt) before the barrier, and reads
// what others copied only after it.
__device__ __forceinline__ void wg_barrier() { asm volatile("s_barrier" ::: "memory"); }

// Results of an MFMA become readable by VALU instructions only a fixed number of cycles
// after issue, and the hardware does not interlock that dependency: the compiler pads
// with s_nop, but it has been seen to misplace the padding when a branch separates the
// MFMA from its first VALU reader.  Every such (rare) path starts with this explicit
// settle instead; 24 wait states cover the 8-pass MFMA used here.
__device__ __forceinline__ void mfma_settle() { asm volatile("s_nop 15\n\ts_nop 7" ::: "memory"); }

template <class G>
struct WaveCtx {
    bf16x8 qf[G::QT][G::NS];
    f32x16 o[G::QT][G::ND];
    float m[G::QT], l[G::QT];
    // running gated sum of the branches, kept in registers where they suffice (d <= 64); at d = 128 it goes
    // through a bf16 scratch tile in global memory instead (fp32 there cost 1.8 % of the kernel for 7 % less
    // rounding error in `out`, whose own bf16 rounding and that of the probabilities dominate either way)
    f32x16 g[G::QT][G::GSUM_REGS ? G::ND : 1];
    int lo[G::QT], hi[G::QT];   // valid key range of this lane's queries in mask coordinates
    uint32_t lane16;            // lane * 16: byte offset of this lane inside any 1 KB fragment or copy instruction
};

// A tile (32 keys of one head) is stored in global memory as the exact image of its LDS slot:
// K_BYTES of K fragments, then V_BYTES of V^T fragments, each fragment 64 lanes x 16 bytes in
// the order the MFMA A operand wants them.  A copy instruction therefore moves 1 KB that is
// contiguous on both sides, and a fragment read is one ds_read_b128 at (slot + lane * 16) plus
// an immediate offset: conflict free, no per-fragment address registers or arithmetic.
//   K fragment ks (hh = lane bit 5, r = lane & 31): key perm(r), channels 16 ks + 8 hh + 0..7,
//     perm = bits 2 and 3 of r swapped (makes the S^T accumulator the B operand of the PV MFMA);
//   V^T fragment f = ks2 * ND + dt: channel 32 dt + r, keys 16 ks2 + 8 hh + 0..7.
// (Gathering the K fragments straight from the caller's [N, H, d] tensor instead -- every copy
// instruction touching 32 rows -- was measured: the attention kernel lost more than the packing
// pass costs.)

// Shared phases: the wavefronts of the workgroup split the T_INST copy instructions of a tile.
template <class G>
__device__ __forceinline__ void issue_shared(const WaveCtx<G> &c, const char *tile, char *slot, int wave) {
    if (G::T_INST < G::WAVES && wave >= G::T_INST) return;
#pragma unroll
    for (int j = 0; j < G::SH_IPT; ++j) {
        const int i = wave + G::WAVES * j;
        __builtin_amdgcn_global_load_lds(GLB_PTR(tile + i * 1024 + c.lane16), LDS_PTR(slot + i * 1024), 16, 0, 0);
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
    for (int ks = 0; ks < G::NS; ++ks) kf[ks] = *reinterpret_cast<const bf16x8 *>(slot + c.lane16 + ks * 1024);
}
template <class G>
__device__ __forceinline__ void read_v(const WaveCtx<G> &c, const char *slot, bf16x8 (&vf)[G::ND][2]) {
#pragma unroll
    for (int dt = 0; dt < G::ND; ++dt)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
            vf[dt][ks] = *reinterpret_cast<const bf16x8 *>(slot + c.lane16 + G::K_BYTES + (ks * G::ND + dt) * 1024);
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

// The running maximum m of a row is kept optimistically: the exponentials of a tile are taken
// against the current m without looking at the tile's own maximum first, and only their row sum
// (which the softmax needs anyway) is examined afterwards.  If it exceeds kSumLimit -- some
// probability would be above 2^10, or infinite: m starts at kMinusHuge, so the first real tile of
// a branch always lands here -- the tile is redone: m is raised to the tile's maximum, O and l are
// rescaled, the probabilities recomputed.  Otherwise every probability is at most 2^10, harmless in
// fp32 and in bf16 (same exponent range), and the step has spent nothing on the maximum: no
// in-lane reduction, no exchange between lane halves, no wait for the score MFMAs to retire.
// A fully masked tile gives zeros and never redoes; a row whose keys are all masked so far keeps
// m = kMinusHuge.
constexpr float kSumLimit = 1024.0f;

// Wave-uniform: does any lane need its tile redone?  (psum is a sum of exponentials of finite or -inf arguments: never NaN)
__device__ __forceinline__ bool sum_overflow(float psum) {
    return __builtin_amdgcn_ballot_w64(!(psum <= kSumLimit)) != 0;
}

// Redoes the exponentials of one tile (scores s, already masked) of row tile qt after raising m to
// the tile's maximum; O and l (which do not yet contain this tile) are rescaled.  Rare path.
template <class G>
__device__ __forceinline__ void redo_tile(WaveCtx<G> &c, int qt, const f32x16 &s, uint32_t (&pu)[8], float &psum,
                                          float sl2) {
    mfma_settle();  // the O accumulators (and, at the start of a phase, s itself) may still be in flight
    const float mx = half_max(lane_max(s));
    const float m_new = fmaxf(c.m[qt], mx);
    const float alpha = __builtin_amdgcn_exp2f((c.m[qt] - m_new) * sl2);
    c.m[qt] = m_new;
    c.l[qt] *= alpha;
#pragma unroll
    for (int dt = 0; dt < G::ND; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) c.o[qt][dt][i] *= alpha;
    const float mc = m_new * sl2;
    float p[16];
    psum = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        p[e] = __builtin_amdgcn_exp2f(s[e] * sl2 - mc);
        psum += p[e];
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) pu[k] = pack_bf16(p[2 * k], p[2 * k + 1]);
}

// After the exponentials of a tile: redo where needed, then add the row sums to l.
template <class G>
__device__ __forceinline__ void close_tile(WaveCtx<G> &c, const f32x16 (&s)[G::QT], uint32_t (&pu)[G::QT][8],
                                           float (&psum)[G::QT], float sl2) {
#pragma unroll
    for (int qt = 0; qt < G::QT; ++qt) {
        if (__builtin_expect(sum_overflow(psum[qt]), 0)) redo_tile<G>(c, qt, s[qt], pu[qt], psum[qt], sl2);
        c.l[qt] += psum[qt];
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
// The row sums of the tile come back in psum (not yet added to l: see close_tile).
// The empty asm statements pin each result to its place in the program (the compiler
// otherwise sinks the arithmetic to its first use) and the scheduling barriers keep the
// machine scheduler from regrouping; neither emits an instruction.
// pu[qt][k] = bf16 pair (p[2k], p[2k+1]) of row tile qt: pu[qt][0..3] / [4..7] are the B
// operands of the two 16-key slabs of the PV contraction.
// The A operands come from two rolling queues of LDS fragments (kq: K rows, vq: V^T rows):
// the MFMA that consumes fragment i is followed by the ds_read of fragment i + queue depth
// of the same stream, which continues into the next tile (k_nxt / v_nxt), so the queues
// enter the next block already primed.  k_cur .. v_nxt are per-lane addresses: slot + lane * 16.  LDS reads are thereby spread under the MFMAs, and
// only a few fragments are live at a time.
template <class G, bool QK, bool PV>
__device__ __forceinline__ void mfma_block(WaveCtx<G> &c, const f32x16 (&s)[G::QT], bf16x8 (&kq)[G::KQ],
                                           f32x16 (&s_next)[G::QT], bf16x8 (&vq)[G::VQ],
                                           const uint32_t (&pu_prev)[G::QT][8], uint32_t (&pu)[G::QT][8],
                                           float (&psum)[G::QT], float sl2, const char *k_cur, const char *k_nxt,
                                           const char *v_cur, const char *v_nxt) {
    constexpr int QT = G::QT;
    constexpr int NQ = QK ? G::NS * QT : 0, NPV = PV ? 2 * G::ND * QT : 0, NG = NQ + NPV;
    constexpr int NE = 16 * QT;
    float mc[QT], p[NE];
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
                        *reinterpret_cast<const bf16x8 *>((nf < G::NS ? k_cur : k_nxt) + (nf % G::NS) * 1024);
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
                                                                      G::K_BYTES + nf * 1024);
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
            vq[f % G::VQ] = *reinterpret_cast<const bf16x8 *>(v_cur + G::K_BYTES + nf * 1024);
        }
    }
}

// Shared phase (compressed and window branches): every tile is used by all query blocks of
// the workgroup.  Tiles go through the ring of NSLOT slots; a slot is refilled as soon as
// every wavefront is done with it.
//   src(t)  -> global address of the image of tile t (uniform over the workgroup)
//   msk(t)  -> (j0, need_mask, cap) of tile t for this wavefront: keys outside the lane's [lo, hi) or at and
//              beyond cap are masked; tiles in [mf_lo, mf_hi) need none
// Step t runs mfma_block with QK of tile t+1, the exponentials of tile t and PV of tile t-1,
// reloading its operand registers on the fly with the K fragments of tile t+2 and the V
// fragments of tile t.  Once per step (one barrier) the slot of tile t-2 is refilled with
// tile t-2+NSLOT, and after the block the row sums of tile t decide whether it must be redone
// against a higher running maximum (close_tile).  Every wavefront runs every step: a tile outside a wavefront's own key range is
// simply fully masked (the step body is kept unconditional on purpose -- a conditional
// update of the accumulator tuples makes the compiler shuffle them through copies).
// Scores and probabilities alternate between two register sets (index = tile parity), so
// nothing is copied from step to step.
// [w_lo, w_hi): the steps whose tiles this wavefront's queries can see at all.  Outside it the wavefront only keeps
// the ring going (waits, barriers, its share of the copies): in the window branch the four query blocks of a
// workgroup see 34 of the 40 tiles the workgroup streams.  w_lo is rounded down to an even step (the register set
// of a tile is its parity).
template <class G, typename SrcFn, typename MaskFn>
__device__ __forceinline__ void run_shared(WaveCtx<G> &c, int n_steps, int w_lo, int w_hi, SrcFn src, MaskFn msk,
                                           int mf_lo, int mf_hi, char *lds, int wave, int lane, float sl2) {
    constexpr int R = G::NSLOT, QT = G::QT;
    constexpr bool PAR = true;  // scores and probabilities alternate between two register sets by tile parity
    if (n_steps <= 0) return;
    w_hi = min(w_hi, n_steps);
    w_lo = max(w_lo, 0) & ~1;
    if (w_hi <= w_lo) w_lo = w_hi = 0;
    auto slot = [&](int t) { return lds + (t % R) * G::TILE; };
    auto lslot = [&](int t) { return lds + (t % R) * G::TILE + c.lane16; };  // this lane's fragment base
    // The two wavefronts that share a SIMD (w and w + 4 of an 8-wavefront workgroup) run half a
    // step apart: one meets the step's barrier before its MFMA block, the other after it, so
    // one's latency-bound work between blocks coincides with the other's MFMA block.
    const bool lag = G::WAVES == 8 && wave >= 4;
    // (LDS reads only: no copy is in flight at the end of a phase, and the stores the previous branch's epilogue has
    // just issued -- outputs, the gated-sum scratch -- need not have been acknowledged before the first copies of this
    // phase go out; they are older than those copies, so the counted waits below cover them)
    __builtin_amdgcn_s_waitcnt(kLgkmOnly);
    wg_barrier();  // every wavefront is done with the slots (previous phase)
    for (int t = 0; t < R && t < n_steps; ++t) issue_shared<G>(c, src(t), slot(t), wave);
    // tiles 0, 1 and 2 must have landed before the first block reads them
    if (n_steps >= R)
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((R - 3) * G::SH_IPT));
    else
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    wg_barrier();
    bf16x8 kq[G::KQ], vq[G::VQ];
    f32x16 S[2][QT];         // scores
    uint32_t P[2][QT][8];    // probabilities
    int j0, cap;  // first key of the tile; keys at or beyond `cap` are inactive slots
    bool need_mask;
    float psum[QT];

    // One workgroup barrier per step keeps the ring consistent.  Before barrier t a wavefront has
    // finished (at least) MFMA block t-1 and waited for its own copies of tiles <= t+3; after it,
    // tile t+3 is complete for everyone and nobody reads tile t-2 any more, whose slot is refilled.
    // Copies issued before the wait: tiles 0 .. t-3+R; tiles t+4 and later may stay in flight
    // (near the end of the phase fewer are outstanding: wait for all).
    auto sync = [&](int t) {
        if (t >= 2 && t - 3 + R < n_steps)
            __builtin_amdgcn_s_waitcnt(vmcnt_imm((R - 6) * G::SH_IPT));
        else if (t == 1 && n_steps >= R)
            __builtin_amdgcn_s_waitcnt(vmcnt_imm((R - 5) * G::SH_IPT));
        else if (t == 0 && n_steps >= R)
            __builtin_amdgcn_s_waitcnt(vmcnt_imm((R - 4) * G::SH_IPT));
        else
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        wg_barrier();
        if (t >= 2 && t - 2 + R < n_steps) issue_shared<G>(c, src(t - 2 + R), slot(t - 2), wave);
    };
    // After an MFMA block: mask the scores just produced (s_next, tile t+1) where the tile needs it,
    // and close tile t (scores s, probabilities pu: redone if their row sums say so).
    auto post = [&](int t, const f32x16 (&s)[QT], f32x16 (&s_next)[QT], uint32_t (&pu)[QT][8]) {
        msk(t + 1, &j0, &need_mask, &cap);
        if (__builtin_expect(need_mask, 0)) {
            mfma_settle();  // s_next comes from the MFMAs just issued
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) mask_scores(c.lo[qt], min(c.hi[qt], cap), s_next[qt], j0, lane);
        }
        close_tile<G>(c, s, pu, psum, sl2);
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
    // The same two pieces for the steps in the middle of a phase, where nothing is conditional:
    // every copy exists and the tile needs no mask.
    auto sync_fast = [&](int t) {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((R - 6) * G::SH_IPT));
        wg_barrier();
        issue_shared<G>(c, src(t - 2 + R), slot(t - 2), wave);
    };
    auto post_fast = [&](const f32x16 (&s)[QT], uint32_t (&pu)[QT][8]) { close_tile<G>(c, s, pu, psum, sl2); };
    // QK(t+1) || exp(t) || PV(t-1); the queues move on to K(t+2) and V(t)  (stale slots past the end: unused)
    auto full_step = [&](auto par, auto fast, int t) {
        constexpr int A = PAR ? decltype(par)::value : 0;
        constexpr bool FAST = decltype(fast)::value;
        if (lag) {
            if constexpr (FAST) sync_fast(t); else sync(t);
        }
        mfma_block<G, true, true>(c, S[A], kq, S[A ^ 1], vq, P[A ^ 1], P[A], psum, sl2, lslot(t + 1), lslot(t + 2),
                                  lslot(t - 1), lslot(t));
        if (!lag) {
            if constexpr (FAST) sync_fast(t); else sync(t);
        }
        if constexpr (FAST) post_fast(S[A], P[A]); else post(t, S[A], S[A ^ 1], P[A]);
        rotate();
    };
    // exp(n-1) || PV(n-2); then the drain: PV of the last tile
    auto last_step = [&](auto par, int t) {
        constexpr int A = PAR ? decltype(par)::value : 0;
        mfma_block<G, false, true>(c, S[A], kq, S[A ^ 1], vq, P[A ^ 1], P[A], psum, sl2, nullptr, nullptr,
                                   lslot(t - 1), lslot(t));
        close_tile<G>(c, S[A], P[A], psum, sl2);
        pv_drain<G>(c, vq, P[A], lslot(t));
    };
    using Even = std::integral_constant<int, 0>;
    using Odd = std::integral_constant<int, 1>;
    // full steps t0 .. t1-1
    auto run_range = [&](int t0, int t1, auto fast) {
        int t = t0;
        if constexpr (PAR) {
            if (t < t1 && (t & 1) == 0) {
                full_step(Even{}, fast, t);
                ++t;
            }
            for (; t + 1 < t1; t += 2) {
                full_step(Odd{}, fast, t);
                full_step(Even{}, fast, t + 1);
            }
            if (t < t1) full_step(Odd{}, fast, t);
        } else {
            for (; t < t1; ++t) full_step(Even{}, fast, t);
        }
    };

    // barriers 0 .. n_steps - 2 in all, whatever the wavefront's own range is
    int ts = 0;  // the next barrier
    auto idle_to = [&](int upto) {
        for (; ts < upto; ++ts) sync(ts);
    };
    if (w_hi <= w_lo) {
        idle_to(n_steps - 1);
        return;
    }
    idle_to(w_lo);  // (behind barrier w_lo - 1 tiles up to w_lo + 2 are complete for everyone)
    {
        bf16x8 kf[G::NS];
        read_k<G>(c, slot(w_lo), kf);
        qk_scores<G>(c, kf, S[0]);
    }
    // prime the queues: first K fragments of the second tile (stale but finite data if there is none), first V
    // fragments of the first
#pragma unroll
    for (int i = 0; i < G::KQ; ++i) kq[i] = *reinterpret_cast<const bf16x8 *>(lslot(w_lo + 1) + i * 1024);
#pragma unroll
    for (int f = 0; f < G::VQ; ++f) vq[f] = *reinterpret_cast<const bf16x8 *>(lslot(w_lo) + G::K_BYTES + f * 1024);
    msk(w_lo, &j0, &need_mask, &cap);
    if (need_mask) {
        mfma_settle();  // the mask reads the scores the MFMAs above produce
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) mask_scores(c.lo[qt], min(c.hi[qt], cap), S[0][qt], j0, lane);
    }
    if (w_hi - w_lo >= 2) {
        // QK(w_lo + 1) || exp(w_lo)
        if (lag) sync(w_lo);
        mfma_block<G, true, false>(c, S[0], kq, S[1], vq, P[1], P[0], psum, sl2, lslot(w_lo + 1), lslot(w_lo + 2), nullptr,
                                   nullptr);
        if (!lag) sync(w_lo);
        post(w_lo, S[0], S[1], P[0]);
        rotate();
        // full steps w_lo + 1 .. w_hi - 2; those in [t_lo, t_hi) take the unconditional path
        const int t_end = w_hi - 1;
        int t_lo = max(max(2, w_lo + 1), mf_lo - 1), t_hi = min(n_steps - R + 2, mf_hi - 1);
        t_lo = min(t_lo, t_end);
        t_hi = max(min(t_hi, t_end), t_lo);
        run_range(w_lo + 1, t_lo, std::false_type{});
        run_range(t_lo, t_hi, std::true_type{});
        run_range(t_hi, t_end, std::false_type{});
        if (PAR && (t_end & 1))
            last_step(Odd{}, t_end);
        else
            last_step(Even{}, t_end);
        ts = w_hi - 1;
    } else {
        mfma_block<G, false, false>(c, S[0], kq, S[1], vq, P[1], P[0], psum, sl2, nullptr, nullptr, nullptr, nullptr);
        close_tile<G>(c, S[0], P[0], psum, sl2);
        pv_drain<G>(c, vq, P[0], lslot(w_lo));
        ts = w_lo;
    }
    idle_to(n_steps - 1);
}

// Selected phase: each query block streams its own routed blocks in 32-key tiles through its NST
// slots; its two wavefronts split the copies, and all wavefronts meet at a workgroup barrier every step.
// CNT: blocks may hold fewer than 64 active tokens; valid(t) is the number of active keys of tile t
// (0..32) and the scores of the others are masked.
// Three tiles are in flight like in the shared phases: step t of a query block runs
// mfma_block with QK of its tile t+1, the exponentials of tile t and PV of tile t-1, so every MFMA
// has its share of the exponentials behind it.  Tile tau lives in stage tau mod NST of the block's NST
// slots, K and V parts copied separately.  Barrier t comes before step t; behind it K(t) and
// V(t-2) are dead, and K(t+NST) and V(t+NST-2) are copied over them, NST-1 steps ahead of their use.
// The operand queues are primed from LDS at the start of every step (the next tile's fragments are
// still in flight while a step runs, so the queues cannot roll across tiles).
// Steps 0 .. n (the last one is the PV of tile n-1); every wavefront meets barriers 0 .. n_steps.
template <class G, bool CNT, typename SrcFn, typename OwnFn, typename ValidFn>
__device__ __forceinline__ void run_own(WaveCtx<G> &c, int n_steps, int my_steps, SrcFn src, OwnFn own, ValidFn valid,
                                         char *lds, int qbi, int sub, int lane, float sl2) {
    constexpr int NP = G::NP;
    if (n_steps <= 0) return;
    static_assert(G::NW == 2 && G::QT == 1, "two wavefronts per query block");
    constexpr int KI = G::K_BYTES / 1024 / G::NW, VI = G::V_BYTES / 1024 / G::NW;
    const int n = my_steps;
    constexpr int NST = G::NST;
    static_assert((NST & (NST - 1)) == 0 && NST >= 2, "");
    // tile tau of this query block lives in the slot of its owner: the query block of the group that copies it (this
    // one, unless the step schedule lets a lower-numbered query block of the group meet the same key block at the
    // same step: the tile is then copied once and read by all of them)
    auto stage = [&](int tau) { return lds + ((tau & (NST - 1)) * NP + own(tau)) * G::TILE; };
    auto lstage = [&](int tau) { return stage(tau) + c.lane16; };
    auto issue_part = [&](const char *tile, char *slot, int n_inst) {
#pragma unroll 8
        for (int j = 0; j < n_inst; ++j) {
            const int i = sub + G::NW * j;
            __builtin_amdgcn_global_load_lds(GLB_PTR(tile + i * 1024 + c.lane16), LDS_PTR(slot + i * 1024), 16, 0, 0);
        }
    };
    auto issue_k = [&](int tau) {
        if (own(tau) == qbi) issue_part(src(tau), stage(tau), KI);
    };
    auto issue_v = [&](int tau) {
        if (own(tau) == qbi) issue_part(src(tau) + G::K_BYTES, stage(tau) + G::K_BYTES, VI);
    };
    // barrier t: K(t+1) and V(t-1) have landed (both were issued behind barrier t+1-NST; what the NST-2
    // barriers since then issued may stay in flight) and every LDS read of this wavefront is done.  Every
    // wavefront waits for its own copies before the barrier, so behind it the tiles are there for all
    // wavefronts, whoever copied them; all wavefronts are at the same step, so the slots overwritten behind
    // barrier t (K of step t, V of step t-2) are dead for all of them.
    auto sync = [&](int t) {
        if (NST > 2 && t + NST - 1 < n)
            __builtin_amdgcn_s_waitcnt(vm_lgkm_imm((NST - 2) * (KI + VI)));
        else
            __builtin_amdgcn_s_waitcnt(vm_lgkm_imm(0));
        wg_barrier();
        if (t + NST < n) issue_k(t + NST);
        if (t + NST - 2 < n) issue_v(t + NST - 2);
    };
    bf16x8 kq[G::KQ], vq[G::VQ];
    f32x16 S[2][1];
    uint32_t P[2][1][8];
    float psum[1];
    auto prime_k = [&](const char *ls) {
#pragma unroll
        for (int i = 0; i < G::KQ; ++i) kq[i] = *reinterpret_cast<const bf16x8 *>(ls + i * 1024);
    };
    auto prime_v = [&](const char *ls) {
#pragma unroll
        for (int f = 0; f < G::VQ; ++f) vq[f] = *reinterpret_cast<const bf16x8 *>(ls + G::K_BYTES + f * 1024);
    };
    auto mask_next = [&](int t, f32x16 &s_next) {
        if constexpr (CNT) {
            if (t + 1 < n) {
                const int vld = valid(t + 1);
                if (vld < 32) {
                    mfma_settle();
                    mask_scores(0, vld, s_next, 0, lane);
                }
            }
        }
    };
    // (LDS reads only: no copy is in flight at the end of a phase, and the stores the previous branch's epilogue has
    // just issued -- outputs, the gated-sum scratch -- need not have been acknowledged before the first copies of this
    // phase go out; they are older than those copies, so the counted waits below cover them)
    __builtin_amdgcn_s_waitcnt(kLgkmOnly);
    wg_barrier();  // every wavefront is done with the slots (previous phase)
#pragma unroll
    for (int tau = 0; tau < NST; ++tau)
        if (tau < n) issue_k(tau);
#pragma unroll
    for (int tau = 0; tau < NST - 2; ++tau)
        if (tau < n) issue_v(tau);
    __builtin_amdgcn_s_waitcnt(vm_lgkm_imm(0));
    wg_barrier();
    if (n > 0) {
        bf16x8 kf[G::NS];
        read_k<G>(c, stage(0), kf);
        qk_scores<G>(c, kf, S[0]);
        mask_next(-1, S[0][0]);
    }
    auto full_step = [&](auto par, int t) {
        constexpr int A = decltype(par)::value;
        sync(t);
        const char *k_nx = lstage(t + 1), *v_pv = lstage(t - 1);
        prime_k(k_nx);
        prime_v(v_pv);
        mfma_block<G, true, true>(c, S[A], kq, S[A ^ 1], vq, P[A ^ 1], P[A], psum, sl2, k_nx, k_nx, v_pv, v_pv);
        mask_next(t, S[A ^ 1][0]);
        close_tile<G>(c, S[A], P[A], psum, sl2);
    };
    auto last_steps = [&](auto par, int t) {  // t = n - 1 >= 1: exp(t) || PV(t-1), then the PV of tile t
        constexpr int A = decltype(par)::value;
        sync(t);
        const char *v_pv = lstage(t - 1);
        prime_v(v_pv);
        mfma_block<G, false, true>(c, S[A], kq, S[A ^ 1], vq, P[A ^ 1], P[A], psum, sl2, nullptr, nullptr, v_pv, v_pv);
        close_tile<G>(c, S[A], P[A], psum, sl2);
        sync(t + 1);
        const char *v_last = lstage(t);
        prime_v(v_last);
        pv_drain<G>(c, vq, P[A], v_last);
    };
    using Even = std::integral_constant<int, 0>;
    using Odd = std::integral_constant<int, 1>;
    int done = 0;  // barriers 0 .. done-1 are behind us
    if (n >= 2) {
        sync(0);
        const char *k1 = lstage(1);
        prime_k(k1);
        mfma_block<G, true, false>(c, S[0], kq, S[1], vq, P[1], P[0], psum, sl2, k1, k1, nullptr, nullptr);
        mask_next(0, S[1][0]);
        close_tile<G>(c, S[0], P[0], psum, sl2);
        int t = 1;
        for (; t + 2 < n; t += 2) {
            full_step(Odd{}, t);
            full_step(Even{}, t + 1);
        }
        if (t + 1 < n) {
            full_step(Odd{}, t);
            ++t;
        }
        if (t & 1)
            last_steps(Odd{}, t);
        else
            last_steps(Even{}, t);
        done = n + 1;
    } else if (n == 1) {
        sync(0);
        mfma_block<G, false, false>(c, S[0], kq, S[1], vq, P[1], P[0], psum, sl2, nullptr, nullptr, nullptr, nullptr);
        close_tile<G>(c, S[0], P[0], psum, sl2);
        sync(1);
        const char *v_last = lstage(0);
        prime_v(v_last);
        pv_drain<G>(c, vq, P[0], v_last);
        done = 2;
    }
    for (int t = done; t <= n_steps; ++t) {
        __builtin_amdgcn_s_waitcnt(vm_lgkm_imm(0));
        wg_barrier();
    }
}

// Ends a branch: normalises, applies the gate and folds the result into the running
// gated sum (registers, or the scratch tile: written by branch 0, updated by branch 1,
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
        const float w = a.gate_channels ? inv : a.gates[(row * a.h + head) * 3 + branch] * inv;
        // per-channel gates of this row, branch and head: D floats
        const f32x4 *gch = reinterpret_cast<const f32x4 *>(a.gates + ((row * 3 + branch) * a.h + head) * D) + hh;
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
#pragma unroll
        for (int dt = 0; dt < G::ND; ++dt) {
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                f32x4 v;
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = w * c.o[qt][dt][4 * gq + j];
                if (a.gate_channels) v *= gch[8 * dt + 2 * gq];  // channels 32 dt + 8 gq + 4 hh + 0..3
                if constexpr (G::GSUM_REGS) {
                    if (branch > 0) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) v[j] += c.g[qt][dt][4 * gq + j];
                    }
                    if (branch < 2) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) c.g[qt][dt][4 * gq + j] = v[j];
                    }
                } else {
                    // bf16 pairs in accumulator order: 8 bytes per lane and fragment, fully coalesced; in LDS for the
                    // first wavefronts of the workgroup (behind the ring), in the scratch buffer for the others
                    static_assert(G::QT == 1, "");
                    // (the scratch buffer holds the query tiles of wavefronts GSUM_LDS_WAVES .. WAVES - 1 only)
                    const int64_t gtile = (row0 / (32 * G::WAVES)) * (G::WAVES - G::GSUM_LDS_WAVES) + (wave - G::GSUM_LDS_WAVES);
                    uint2 *slot = reinterpret_cast<uint2 *>(a.gsum) +
                                  ((gtile * a.h + head) * (G::ND * 4) + dt * 4 + gq) * 64 + lane;
                    uint2 *slot_lds =
                        reinterpret_cast<uint2 *>(lds + G::LDS_BYTES + wave * G::GSUM_LDS_BYTES) + (dt * 4 + gq) * 64 + lane;
                    const bool in_lds = wave < G::GSUM_LDS_WAVES;
                    if (branch > 0) {
                        // (address spaces spelled out: one pointer that may be either would become a flat load)
                        unsigned long long raw;
                        if (in_lds)
                            raw = *(const __attribute__((address_space(3))) unsigned long long *)slot_lds;
                        else
                            raw = *(const __attribute__((address_space(1))) unsigned long long *)slot;
                        const uint2 pv = make_uint2((uint32_t)raw, (uint32_t)(raw >> 32));
                        v[0] += __uint_as_float(pv.x << 16);
                        v[1] += __uint_as_float(pv.x & 0xffff0000u);
                        v[2] += __uint_as_float(pv.y << 16);
                        v[3] += __uint_as_float(pv.y & 0xffff0000u);
                    }
                    if (branch < 2) {
                        uint2 w2;
                        w2.x = pack_bf16(v[0], v[1]);
                        w2.y = pack_bf16(v[2], v[3]);
                        if (in_lds)
                            *slot_lds = w2;
                        else
                            *slot = w2;
                    }
                }
                if (branch == 2) {
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
    if (a.blk_seg != nullptr) {  // segments per block (the query's spatial block), looked up instead of scanned
        w.seg_lo = a.blk_seg[2 * qb];
        w.seg_hi = a.blk_seg[2 * qb + 1];
    } else {
        for (int s = 0; s < a.n_seg; ++s) {
            int lo = a.seg[s], hi = a.seg[s + 1];
            if (q0 >= lo && q0 < hi) {
                w.seg_lo = lo;
                w.seg_hi = hi;
            }
        }
    }
    if (a.own_block) {
        // the block is its own segment (a.window is 128 in this mode: every query reaches every slot);
        // with counts, the segment ends at the last active token
        w.seg_lo = q0;
        w.seg_hi = q0 + (a.count != nullptr ? a.count[qb] : 64);
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

// CNT: a.count is given (variable number of active tokens per block).
// WIDE: routing rows of 65..128 entries (two per lane of the list holder instead of one).
template <class G, bool CNT, bool WIDE>
__global__ __launch_bounds__((G::THREADS), (G::WAVES_PER_SIMD)) void nsa_forward_kernel(FwdArgs a) {
    constexpr int D = G::D, NP = G::NP;
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    // XCD-aware numbering: hardware deals consecutive workgroups round-robin to the 8 XCDs
    // and runs them roughly in launch order.  All XCDs work on the same head at the same time (so the
    // K/V working set of the moment is one head: it fits the last-level cache and the pooled
    // keys/values fit every L2), each XCD on its own contiguous eighth of the head's query blocks
    // (so neighbouring windows and routed blocks meet in its L2).
    const int xcd = blockIdx.x & 7, slot_id = blockIdx.x >> 3;
    const int head = slot_id / a.groups_per_xcd;
    const int group = xcd * a.groups_per_xcd + slot_id % a.groups_per_xcd;
    if (group >= a.groups_per_head) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int qbi = wave / G::NW, sub = wave % G::NW;  // query block inside the group, wavefront inside the block
    const int r = lane & 31, hh = lane >> 5;
    const int qb = group * NP + qbi;
    const bool active = qb < a.nb;  // a trailing group may have fewer than NP query blocks
    const int64_t row0 = (int64_t)(active ? qb : 0) * 64 + G::ROWS * sub;
    const int kvh = head / a.group;                         // key/value head of this query head
    // images are stored head-major: the tiles of one head are contiguous
    const int64_t tile_stride = G::TILE;
    const int64_t head_kv = (int64_t)kvh * (2 * a.nb) * G::TILE, head_kvc = (int64_t)kvh * ((a.nbc + 31) / 32) * G::TILE;
    const float sl2 = a.scale_log2e;

    WaveCtx<G> c;
    c.lane16 = (uint32_t)lane * 16u;
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
            c.hi[qt] = a.nbc;
        }
        const int n_steps = (a.nbc + 31) / 32;
        const char *base = a.kvc + head_kvc;
        auto src = [&](int t) { return base + t * tile_stride; };
        auto msk = [&](int t, int *j0, bool *need, int *cap) {
            *j0 = 32 * t;
            *need = 32 * t + 32 > a.nbc;
            *cap = 0x7fffffff;
        };
        run_shared<G>(c, n_steps, 0, n_steps, src, msk, 0, a.nbc / 32, lds, wave, lane, sl2);
        if (active) finish_branch<G>(c, a, 0, row0, head, wave, lane, lds);
    }

    // ---------------- selected branch: every token of the routed blocks
    {
        reset_branch<G>(c);
        // this query block's routing row, valid entries first: entry u sits in lane u % 64 of register u / 64
        constexpr int NR = WIDE ? 2 : 1;
        int packed[NR], pcount[NR], my_valid = 0, max_valid = 0;
#pragma unroll
        for (int j = 0; j < NR; ++j) packed[j] = -1, pcount[j] = 0;
        if constexpr (D == 128) {
            // rows of the step schedule (schedule.hip): already compact, block id | owner << 28
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                int n_valid = 0;
#pragma unroll
                for (int j = 0; j < NR; ++j) {
                    const int col = lane + 64 * j;
                    const int v = col < a.topk ? a.sched[((int64_t)group * NP + p) * a.topk + col] : -1;
                    n_valid += __popcll(__ballot(v >= 0));
                    if (p == qbi) packed[j] = v;
                }
                max_valid = max(max_valid, n_valid);
                if (p == qbi) my_valid = n_valid;
            }
        } else {
            // rows of the routing table: compacted through this wavefront's 512 bytes behind the tile slots
            int *scratch = reinterpret_cast<int *>(lds + G::LDS_BYTES) + wave * 128;
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                const int qbp = group * NP + p;
                int v[NR], n_valid = 0;
                unsigned long long bal[NR];
#pragma unroll
                for (int j = 0; j < NR; ++j) {
                    const int col = lane + 64 * j;
                    v[j] = (qbp < a.nb && col < a.topk) ? a.idx[(int64_t)qbp * a.topk + col] : -1;
                    if (v[j] >= a.nb) v[j] = -1;
                    bal[j] = __ballot(v[j] >= 0);
                    n_valid += __popcll(bal[j]);
                }
                max_valid = max(max_valid, n_valid);
                if (p == qbi) {
                    int before = 0;
#pragma unroll
                    for (int j = 0; j < NR; ++j) {
                        if (v[j] >= 0) scratch[before + __popcll(bal[j] & ((1ull << lane) - 1ull))] = v[j];
                        before += __popcll(bal[j]);
                    }
                    // (LDS operations of a wavefront complete in order: the reads below see the writes above)
#pragma unroll
                    for (int j = 0; j < NR; ++j) packed[j] = lane + 64 * j < n_valid ? scratch[lane + 64 * j] : -1;
                    my_valid = n_valid;
                }
            }
        }
        if constexpr (CNT) {
#pragma unroll
            for (int j = 0; j < NR; ++j) pcount[j] = lane + 64 * j < my_valid ? a.count[packed[j] & 0xFFFFFF] : 0;
        }
        // entry u of the row / of the counts (wave-uniform u)
        auto entry = [&](int u) {
            if constexpr (WIDE) {
                const int e0 = __builtin_amdgcn_readlane(packed[0], u & 63), e1 = __builtin_amdgcn_readlane(packed[NR - 1], u & 63);
                return u < 64 ? e0 : e1;
            } else {
                return __builtin_amdgcn_readlane(packed[0], u);
            }
        };
        const char *base = a.kv + head_kv;
        auto src = [&](int t) { return base + (2 * (entry(t >> 1) & 0xFFFFFF) + (t & 1)) * tile_stride; };
        // the query block whose wavefronts copy this query block's tile of step t (always itself without a schedule)
        auto own = [&](int t) { return D == 128 ? (entry(t >> 1) >> 28) & 3 : qbi; };
        auto valid = [&](int t) {  // active keys of tile t of this query block's list
            const int u = t >> 1;
            int cnt;
            if constexpr (WIDE) {
                const int c0 = __builtin_amdgcn_readlane(pcount[0], u & 63), c1 = __builtin_amdgcn_readlane(pcount[NR - 1], u & 63);
                cnt = u < 64 ? c0 : c1;
            } else {
                cnt = __builtin_amdgcn_readlane(pcount[0], u);
            }
            return min(32, max(0, cnt - 32 * (t & 1)));
        };
        run_own<G, CNT>(c, 2 * max_valid, 2 * my_valid, src, own, valid, lds, qbi, sub, lane, sl2);
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
        const char *base = a.kv + head_kv;
        auto src = [&](int t) { return base + (st_min + t) * tile_stride; };
        auto msk = [&](int t, int *j0, bool *need, int *cap) {
            int st = st_min + t;
            *j0 = 32 * st;
            *need = (32 * st < mine.full_lo) || (32 * st + 32 > mine.full_hi);  // also true outside [st0, st1)
            *cap = 0x7fffffff;
            if constexpr (CNT) {
                // slots of the tile's block beyond its active tokens (in own-block mode the segment already ends there)
                if (!a.own_block && st < 2 * a.nb) {
                    const int vld = min(32, max(0, a.count[st >> 1] - 32 * (st & 1)));
                    if (vld < 32) {
                        *need = true;
                        *cap = 32 * st + vld;
                    }
                }
            }
        };
        // tiles wholly inside the range that every query of the block sees (none is known to be, with counts)
        const int mf_lo = CNT ? 0 : max(0, (mine.full_lo - 32 * st_min + 31) >> 5);
        const int mf_hi = CNT ? 0 : (mine.full_hi - 32 * st_min) >> 5;
        // The steps of this wavefront's own query block (a query block past the end of the sequence sees nothing).
        // Measured: attention kernel 0.5 % faster at config 4, 1.6 % at config 3, 2.5 % at config 2; 0.6 % slower at
        // config 6 (d = 32), where the restructured loop costs more than the skipped tiles save.
        const int w_lo = active ? mine.st0 - st_min : 0, w_hi = active ? mine.st1 - st_min : 0;
        run_shared<G>(c, n_steps, w_lo, w_hi, src, msk, mf_lo, mf_hi, lds, wave, lane, sl2);
        __builtin_amdgcn_s_waitcnt(vm_lgkm_imm(0));
        wg_barrier();  // the tile slots are about to be reused for the output rows
        if (active) finish_branch<G>(c, a, 2, row0, head, wave, lane, lds);
    }
}

// Builds the tile images (see issue_shared) of a K and a V tensor, both [n_rows, H, D] bf16:
// img[head][tile] = K fragments (K_BYTES) then V^T fragments (V_BYTES).
// Rows at or beyond n_rows read as zero (their scores are masked in the attention kernel).
// One workgroup per (64-row block, head) = two tiles.
// count (nullable, one entry per 64-row block): rows of a block at or beyond its count read as zero too.
// ROWS_ONLY (the backward's images): only the row-order fragments of k are written, img[tile][head] is
// K_BYTES long, and inside a fragment the 16-byte slot of (row position r, channel half hh) is
// hh * 32 + (r ^ 4 hh) instead of hh * 32 + r (keeps the backward's transposing LDS loads off shared banks).
// Position of the image of (tile, head), in images.  The attention kernel's images are head-major
// (img[head][tile]): all workgroups in flight work on one head, whose keys and values are then one
// contiguous range instead of 16 KB pieces spread over the whole buffer -- measured 3 % faster at the
// largest shape.  The backward's row-only images are img[tile][head] (the other order changed nothing there).
template <bool ROWS_ONLY>
__device__ __forceinline__ int64_t image_index(int64_t tile, int head, int h, int n_tiles) {
    return ROWS_ONLY ? tile * h + head : (int64_t)head * n_tiles + tile;
}

// POOL (with the full images only): the block averages of k and v are written as well (kc, vc [n_rows / 64, H, D]
// bf16: Sec. 3.2, the compressed pair of the block), so that one pass over K and V serves both the pooling and
// the packing.  A thread sums its rows in fp32 in token order (rows t, t + 2048 / D, ...); the partial sums of
// the 2048 / D threads that share a channel group are added in thread order; one rounding to bf16.
template <int D, bool ROWS_ONLY, bool POOL = false>
__global__ __launch_bounds__(256) void pack_tiles(const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
                                                  char *__restrict__ img, int64_t n_rows, int h, int n_tiles,
                                                  const int32_t *__restrict__ count, uint16_t *__restrict__ kc = nullptr,
                                                  uint16_t *__restrict__ vc = nullptr) {
    static_assert(!(POOL && ROWS_ONLY), "");
    constexpr int K_BYTES = 32 * D * 2, TILE = ROWS_ONLY ? K_BYTES : K_BYTES + D * 64;
    constexpr int CH = D / 8;  // 16-byte chunks per row
    // Both tensors' rows of the block are staged in LDS, so that the images are written in image order (a wavefront
    // writes 1 KB contiguous per instruction; written straight from the loaded registers, K chunks would go out as
    // 16-byte pieces 512 bytes apart).  Row pitch D + 16 elements: 16-byte aligned, and the 4 rows x 4 column
    // groups that 16 lanes address in one transposing load fall in distinct banks.
    constexpr int PITCH = D + 16;
    __shared__ __attribute__((aligned(16))) uint16_t kt[64][PITCH];
    __shared__ __attribute__((aligned(16))) uint16_t vt[ROWS_ONLY ? 1 : 64][PITCH];
    __shared__ float psum[POOL ? 2 : 1][POOL ? 256 / CH : 1][POOL ? D + 1 : 1];  // [k, v][thread group][channel]
    const int64_t blk = blockIdx.x;
    const int head = blockIdx.y;
    const int n_act = count != nullptr ? count[blk] : 64;
    float ak[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, av[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // all loads of the thread first (64 CH / 256 chunks of k and as many of v), so that they are in flight together
    constexpr int NIT = 64 * CH / 256;
    uint4 kin[NIT], vin[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int e = threadIdx.x + 256 * it;
        const int t = e / CH, cc = e % CH;
        const int64_t row = blk * 64 + t;
        kin[it] = make_uint4(0, 0, 0, 0);
        vin[it] = make_uint4(0, 0, 0, 0);
        if (row < n_rows && t < n_act) {
            kin[it] = *reinterpret_cast<const uint4 *>(k + (row * h + head) * D + cc * 8);
            if (!ROWS_ONLY) vin[it] = *reinterpret_cast<const uint4 *>(v + (row * h + head) * D + cc * 8);
        }
    }
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int e = threadIdx.x + 256 * it;
        const int t = e / CH, cc = e % CH;
        const uint4 kval = kin[it], vval = vin[it];
        *reinterpret_cast<uint4 *>(&kt[t][cc * 8]) = kval;
        if (ROWS_ONLY) continue;
        *reinterpret_cast<uint4 *>(&vt[t][cc * 8]) = vval;
        if (POOL) {
            const uint32_t kw[4] = {kval.x, kval.y, kval.z, kval.w}, w[4] = {vval.x, vval.y, vval.z, vval.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                ak[2 * j] += __uint_as_float(kw[j] << 16);
                ak[2 * j + 1] += __uint_as_float(kw[j] & 0xffff0000u);
                av[2 * j] += __uint_as_float(w[j] << 16);
                av[2 * j + 1] += __uint_as_float(w[j] & 0xffff0000u);
            }
        }
    }
    if (POOL) {
        // (every thread keeps one chunk column cc = threadIdx.x % CH: 256 is a multiple of CH)
        const int grp = threadIdx.x / CH, cc = threadIdx.x % CH;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            psum[0][grp][cc * 8 + j] = ak[j];
            psum[1][grp][cc * 8 + j] = av[j];
        }
    }
    __syncthreads();
    // K: a permutation of 16-byte chunks.  Chunk q of a tile's K part = fragment ks = cc / 2, lane (hh = cc % 2,
    // r = q % 32) with cc = q / 32: source row perm(r) of the tile, source chunk cc.
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int e = threadIdx.x + 256 * it;
        const int half = e / (32 * CH), q = e % (32 * CH);
        const int cc = q / 32, rr = q % 32;
        const int r = ROWS_ONLY ? rr ^ ((cc & 1) << 2) : rr;
        const int tt = (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1);
        const uint4 kval = *reinterpret_cast<const uint4 *>(&kt[32 * half + tt][cc * 8]);
        const int64_t tile = blk * 2 + half;
        if (tile < n_tiles)
            *reinterpret_cast<uint4 *>(img + image_index<ROWS_ONLY>(tile, head, h, n_tiles) * TILE + q * 16) = kval;
    }
    if (ROWS_ONLY) return;
    if (POOL) {
        if (threadIdx.x < 2 * D) {
            const int which = threadIdx.x / D, c = threadIdx.x % D;
            float sum = 0.f;
            for (int g = 0; g < 256 / CH; ++g) sum += psum[which][g][c];
            const float mean = sum / (float)n_act;
            uint32_t u = __float_as_uint(mean);
            u += 0x7fffu + ((u >> 16) & 1u);  // round to nearest even
            (which == 0 ? kc : vc)[(blk * h + head) * D + c] = (uint16_t)(u >> 16);
        }
    }
    // V^T: chunk e of a tile = fragment f = e / 64 (ks2 = f / ND, dt = f % ND), lane = e % 64
    // (hh = lane / 32, r = lane % 32): channel 32 dt + r, keys 16 ks2 + 8 hh + 0..7.  Read with the transposing LDS
    // load (ds_read_b64_tr_b16: within a group of 16 lanes, lane j receives as element e the 16-bit element j % 4 of
    // what lane 4 e + j / 4 addressed): lane j of a group addresses row k0 + j / 4, channels c0 + 4 (j % 4) .. + 3, and
    // receives channel c0 + j of rows k0 .. k0 + 3; two loads give the 8 keys of the chunk.
    constexpr int ND = D / 32;
    const uint32_t vt_base = (uint32_t)(uintptr_t)&vt[0][0];  // (the low 32 bits of a generic LDS pointer are the LDS address)
    for (int e = threadIdx.x; e < 2 * 2 * ND * 64; e += 256) {
        const int half = e / (2 * ND * 64);
        const int f = (e / 64) % (2 * ND), ln = e % 64;
        const int ks2 = f / ND, dt = f % ND, hh = ln / 32, r = ln % 32;
        const int j = ln & 15, c0 = 32 * dt + (r & 16), t0 = 32 * half + 16 * ks2 + 8 * hh;
        const int64_t tile = blk * 2 + half;
        const uint32_t addr = vt_base + (uint32_t)(((t0 + (j >> 2)) * PITCH + c0 + 4 * (j & 3)) * 2);
        uint2 lo, hi;
        asm volatile("ds_read_b64_tr_b16 %0, %2\n\tds_read_b64_tr_b16 %1, %2 offset:%3\n\ts_waitcnt lgkmcnt(0)"
                     : "=&v"(lo), "=&v"(hi)
                     : "v"(addr), "n"(4 * PITCH * 2)
                     : "memory");
        if (tile >= n_tiles) continue;
        *reinterpret_cast<uint4 *>(img + image_index<ROWS_ONLY>(tile, head, h, n_tiles) * TILE + K_BYTES + (f * 64 + ln) * 16) =
            make_uint4(lo.x, lo.y, hi.x, hi.y);
    }
}

struct WsLayout {
    size_t kv, kvc, gsum, sched, gtab, total;
};

WsLayout ws_layout(const Shape &s) {
    WsLayout w;
    const size_t tile = (size_t)32 * s.d * 2 * 2;  // K and V^T parts of one (tile, head)
    size_t off = 0;
    w.kv = off;
    off += align_up((size_t)s.nb * 2 * s.h_kv * tile, 256);
    w.kvc = off;
    off += align_up((size_t)((s.nbc + 31) / 32) * s.h_kv * tile, 256);
    w.gsum = off;
    // (d = 128: bf16, the query tiles of four of a workgroup's eight wavefronts; the others' stay in LDS; in registers at d <= 64)
    off += s.d == 128 ? align_up((size_t)((s.nb + 3) / 4) * 4 * 32 * s.h * s.d * 2, 256) : 0;
    w.sched = off;
    off += s.d == 128 ? sel_schedule_bytes(s) : 0;
    w.gtab = off;
    off += group_tables_bytes(s);
    w.total = off > 0 ? off : 256;
    return w;
}

template <class G>
lsrm_status launch_forward_d(const Shape &s, const int32_t *seg_host, int n_seg, FwdArgs a, const uint16_t *d_k,
                             const uint16_t *d_v, const uint16_t *d_kc, const uint16_t *d_vc, char *ws,
                             const WsLayout &w, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
    constexpr int D = G::D, NP = G::NP;
    for (int i = 0; i <= n_seg; ++i) a.seg[i] = seg_host[i];
    const int tiles_c = (s.nbc + 31) / 32;
    if (s.group_window) {
        GroupTables gt;
        lsrm_status rc = launch_group_tables(s, reinterpret_cast<int32_t *>(ws + w.gtab), &gt, st);
        if (rc != LSRM_OK) return rc;
        a.blk_seg = gt.blk_seg;
    }
    if (!s.kv_packed) {
        hipLaunchKernelGGL((pack_tiles<D, false>), dim3(s.nb, s.h_kv), dim3(256), 0, st, d_k, d_v, ws + w.kv, s.n, s.h_kv,
                           2 * s.nb, a.count);
        LSRM_HIP_CHECK(hipGetLastError());
    }
    hipLaunchKernelGGL((pack_tiles<D, false>), dim3((s.nbc + 63) / 64, s.h_kv), dim3(256), 0, st, d_kc, d_vc, ws + w.kvc,
                       (int64_t)s.nbc, s.h_kv, tiles_c, (const int32_t *)nullptr);
    LSRM_HIP_CHECK(hipGetLastError());
    if (D == 128) {
        lsrm_status rc = launch_sel_schedule(s, a.idx, reinterpret_cast<int32_t *>(ws + w.sched), st);
        if (rc != LSRM_OK) return rc;
    }
    a.sched = reinterpret_cast<const int32_t *>(ws + w.sched);
    a.kv = ws + w.kv;
    a.kvc = ws + w.kvc;
    a.gsum = reinterpret_cast<uint16_t *>(ws + w.gsum);
    a.groups_per_head = (s.nb + NP - 1) / NP;
    a.groups_per_xcd = (a.groups_per_head + 7) / 8;
    // dynamic LDS: the tile slots, then 512 bytes per wavefront for compacting a routing row
    // behind the ring: the routing-row scratch of the selected phase (d <= 64) or the LDS part of the running gated sum
    constexpr int kLds = G::LDS_BYTES + (G::GSUM_LDS_WAVES > 0 ? G::GSUM_LDS_WAVES * G::GSUM_LDS_BYTES : G::WAVES * 512);
    const bool cnt = a.count != nullptr, wide = s.topk > 64;
    const void *kern = cnt ? (wide ? reinterpret_cast<const void *>(&nsa_forward_kernel<G, true, true>)
                                   : reinterpret_cast<const void *>(&nsa_forward_kernel<G, true, false>))
                           : (wide ? reinterpret_cast<const void *>(&nsa_forward_kernel<G, false, true>)
                                   : reinterpret_cast<const void *>(&nsa_forward_kernel<G, false, false>));
    // (set on every launch: cheap, and right whichever device is current and whichever thread calls)
    LSRM_HIP_CHECK(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, kLds));
    if (ev_start != nullptr) LSRM_HIP_CHECK(hipEventRecord(ev_start, st));
    const dim3 grid(8 * a.groups_per_xcd * s.h);
    void *kargs[] = {&a};
    LSRM_HIP_CHECK(hipLaunchKernel(kern, grid, dim3(G::THREADS), kargs, kLds, st));
    LSRM_HIP_CHECK(hipGetLastError());
    if (ev_stop != nullptr) LSRM_HIP_CHECK(hipEventRecord(ev_stop, st));
    return LSRM_OK;
}

}  // namespace

size_t forward_ws_bytes(const Shape &s) { return ws_layout(s).total; }

lsrm_status launch_compress_pack(const Shape &s, const uint16_t *d_k, const uint16_t *d_v, uint16_t *d_kc,
                                 uint16_t *d_vc, void *d_ws, hipStream_t st) {
    if (s.nb == 0) return LSRM_OK;
    char *img = reinterpret_cast<char *>(d_ws) + ws_layout(s).kv;
    const dim3 grid(s.nb, s.h_kv);
    if (s.ng > 0) {
        // a spatial block's average spans several 64-slot blocks, i.e. several workgroups of the packing pass: the
        // two are separate passes here
        lsrm_status rc = launch_pack_tiles(s.d, d_k, d_v, img, s.n, s.h_kv, 2 * s.nb, st, false, s.count);
        if (rc != LSRM_OK) return rc;
        return launch_compress(s, d_k, d_v, d_kc, d_vc, st);
    }
#define LSRM_POOL_PACK(DD) \
    hipLaunchKernelGGL((pack_tiles<DD, false, true>), grid, dim3(256), 0, st, d_k, d_v, img, s.n, s.h_kv, 2 * s.nb, s.count, \
                       d_kc, d_vc)
    if (s.d == 32)
        LSRM_POOL_PACK(32);
    else if (s.d == 64)
        LSRM_POOL_PACK(64);
    else
        LSRM_POOL_PACK(128);
#undef LSRM_POOL_PACK
    LSRM_HIP_CHECK(hipGetLastError());
    return LSRM_OK;
}

lsrm_status launch_pack_tiles(int d, const uint16_t *rows_src, const uint16_t *t_src, char *img, int64_t n_rows, int h,
                              int n_tiles, hipStream_t st, bool rows_only, const int32_t *count) {
    if (n_tiles <= 0) return LSRM_OK;
    const dim3 grid((n_tiles + 1) / 2, h);
#define LSRM_PACK(DD, RO) \
    hipLaunchKernelGGL((pack_tiles<DD, RO>), grid, dim3(256), 0, st, rows_src, t_src, img, n_rows, h, n_tiles, count)
    if (d == 32) {
        if (rows_only) LSRM_PACK(32, true); else LSRM_PACK(32, false);
    } else if (d == 64) {
        if (rows_only) LSRM_PACK(64, true); else LSRM_PACK(64, false);
    } else {
        if (rows_only) LSRM_PACK(128, true); else LSRM_PACK(128, false);
    }
#undef LSRM_PACK
    LSRM_HIP_CHECK(hipGetLastError());
    return LSRM_OK;
}

lsrm_status launch_forward(const Shape &s, const int32_t *seg_host, int n_seg, const uint16_t *d_q,
                           const uint16_t *d_k, const uint16_t *d_v, const uint16_t *d_kc, const uint16_t *d_vc,
                           const int32_t *d_idx, const float *d_gates, uint16_t *d_out, float *d_lse,
                           uint16_t *d_out_branch, void *d_ws, hipStream_t st, hipEvent_t ev_start,
                           hipEvent_t ev_stop) {
    if (s.nb == 0) return LSRM_OK;
    if (n_seg > kMaxSeg) return LSRM_ERR_UNSUPPORTED;
    FwdArgs a{};
    a.q = d_q;
    a.idx = d_idx;
    a.gates = d_gates;
    a.out = d_out;
    a.lse = d_lse;
    a.out_branch = d_out_branch;
    a.n = s.n;
    a.nb = s.nb;
    a.nbc = s.nbc;
    a.blk_seg = nullptr;
    a.h = s.h;
    a.h_kv = s.h_kv;
    a.group = s.h / s.h_kv;
    a.gate_channels = s.gate_channels;
    a.own_block = s.own_block;
    a.count = s.count;
    a.topk = s.topk;
    a.window = s.window;
    a.n_seg = n_seg;
    a.scale = s.scale;
    a.scale_log2e = s.scale * 1.4426950408889634f;
    WsLayout w = ws_layout(s);
    char *ws = reinterpret_cast<char *>(d_ws);
    if (s.d == 32) return launch_forward_d<Geo<32, 4, 1>>(s, seg_host, n_seg, a, d_k, d_v, d_kc, d_vc, ws, w, st, ev_start, ev_stop);
    if (s.d == 64) return launch_forward_d<Geo<64, 4, 1>>(s, seg_host, n_seg, a, d_k, d_v, d_kc, d_vc, ws, w, st, ev_start, ev_stop);
    return launch_forward_d<Geo<128, 4, 1>>(s, seg_host, n_seg, a, d_k, d_v, d_kc, d_vc, ws, w, st, ev_start, ev_stop);
}

}  // namespace lsrm
