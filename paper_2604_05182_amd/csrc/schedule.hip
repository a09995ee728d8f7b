// Step schedule of the selected branch (App. A, "Selected"; Sec. 3.3: geometric routing makes
// neighbouring queries select the same blocks).
//
// The attention kernel carries four consecutive query blocks per workgroup through the selected
// branch in lockstep: at step s every query block works on one of its routed key blocks.  Query
// blocks that are neighbours in the sequence are neighbours in space, so their routing rows overlap
// heavily (about half of the blocks a group of four lists are distinct).  This kernel orders each
// row so that a block listed by several rows of a group is met by all of them at the same step;
// the workgroup then copies that block's tiles to LDS once and the query blocks read the same slot.
// The order inside a row does not change the result: the selected branch is one softmax over the
// union of the listed blocks' tokens.
//
// Output: sched[groups * 4, topk] int32.  Row r holds the valid entries of idx row r, reordered,
// as  block id | owner << 28  (owner = lowest-numbered query block of the group that meets the
// block at this step; it is the one whose wavefronts issue the copy), then -1.
//
// Greedy order (one wavefront per group): at every step, while some row of the group still has
// no block for this step, pick the unscheduled block that serves the most of those rows, preferring
// one whose remaining rows are all served now, then the lowest block id; give it to those rows.
// A block that a row lists twice is attended twice: its second occurrence is scheduled on its own.
// On the benchmark tables the list is within 1 % of the number of distinct blocks of the group.
#include "lsrm_internal.h"

namespace lsrm {

namespace {

constexpr int NP = 4;  // query blocks per group: the attention kernel's workgroup

// Wave-wide maximum without the LDS crossbar: four data-parallel-primitive steps fold each row of 16 lanes, then
// the four row results are read as scalars.  All 64 lanes must be active; the result is wave-uniform.
__device__ __forceinline__ unsigned wave_max_u32(unsigned v) {
    auto mx = [](unsigned a, unsigned b) { return a > b ? a : b; };
    v = mx(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
    v = mx(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
    v = mx(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, false));  // row_half_mirror
    v = mx(v, (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, false));  // row_mirror
    const unsigned r0 = __builtin_amdgcn_readlane(v, 0), r1 = __builtin_amdgcn_readlane(v, 16);
    const unsigned r2 = __builtin_amdgcn_readlane(v, 32), r3 = __builtin_amdgcn_readlane(v, 48);
    return mx(mx(r0, r1), mx(r2, r3));
}

// EPL: routing-row entries per lane (topk <= 64 * EPL).
template <int EPL>
__global__ __launch_bounds__(64) void build_sel_schedule(const int32_t *__restrict__ idx, int32_t *__restrict__ sched,
                                                         int nb, int topk) {
    constexpr int NE = NP * EPL;
    const int group = blockIdx.x, lane = threadIdx.x;
    int e[NE];        // entry (row p = i / EPL, column lane + 64 (i % EPL)): block id, or -1
    unsigned m[NE];   // rows that list this block and have not met it yet (bit p; own row included); 0: scheduled or no entry
    unsigned pos[NE]; // byte p': column of this block in row p' (valid where bit p' of m was set at the start)
    bool dup[NE];
    int cnt[NP];
#pragma unroll
    for (int i = 0; i < NE; ++i) {
        const int p = i / EPL, col = lane + 64 * (i % EPL);
        const int qb = group * NP + p;
        int v = (qb < nb && col < topk) ? idx[(int64_t)qb * topk + col] : -1;
        if (v < 0 || v >= nb) v = -1;
        e[i] = v;
        m[i] = v >= 0 ? 1u << p : 0u;
        pos[i] = 0;
        dup[i] = false;
    }
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        cnt[p] = 0;
#pragma unroll
        for (int j = 0; j < EPL; ++j) cnt[p] += __popcll(__ballot(e[p * EPL + j] >= 0));
    }
    // partners: for every entry, the first column of every other row that holds the same block; an entry with an
    // earlier occurrence of its block in its own row is a repeat and stays alone
#pragma unroll
    for (int pp = 0; pp < NP; ++pp) {
        for (int k = 0; k < topk; ++k) {
            int v;
            if (EPL == 1 || k < 64)
                v = __builtin_amdgcn_readlane(e[pp * EPL], k & 63);
            else
                v = __builtin_amdgcn_readlane(e[pp * EPL + (EPL - 1)], k & 63);
            if (v < 0) continue;
#pragma unroll
            for (int i = 0; i < NE; ++i) {
                const int p = i / EPL, col = lane + 64 * (i % EPL);
                if (e[i] != v) continue;
                if (p == pp) {
                    if (k < col) dup[i] = true;
                } else if (((m[i] >> pp) & 1u) == 0u) {
                    m[i] |= 1u << pp;
                    pos[i] |= (unsigned)k << (8 * pp);
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < NE; ++i)
        if (dup[i]) m[i] = 1u << (i / EPL);

    int32_t *out = sched + (int64_t)group * NP * topk;
    int done[NP] = {0, 0, 0, 0};  // blocks scheduled so far per row
    for (int s = 0; s < topk; ++s) {
        unsigned free_rows = 0;
#pragma unroll
        for (int p = 0; p < NP; ++p)
            if (done[p] < cnt[p]) free_rows |= 1u << p;
        if (free_rows == 0) break;
        // every row in free_rows has met exactly s blocks
        for (int pick = 0; pick < NP && free_rows != 0; ++pick) {
            unsigned bk = 0, bm = 0, bpos = 0;
            int be = 0, bi = 0;
#pragma unroll
            for (int i = 0; i < NE; ++i) {
                const int p = i / EPL;
                if (m[i] == 0 || ((free_rows >> p) & 1u) == 0u) continue;
                const unsigned a = m[i] & free_rows;
                const unsigned key = ((unsigned)__popc(a) << 28) | ((m[i] & ~free_rows) == 0 ? 1u << 27 : 0u) |
                                     (0x7FFFFFFu - (unsigned)e[i]);
                if (key > bk) {
                    bk = key;
                    bm = m[i];
                    bpos = pos[i];
                    be = e[i];
                    bi = i;
                }
            }
            const unsigned kmax = wave_max_u32(bk);
            if (kmax == 0) {  // cannot happen (a free row has an unscheduled entry); never spin
                free_rows = 0;
                break;
            }
            const int winner = __ffsll((unsigned long long)__ballot(bk == kmax)) - 1;
            const unsigned wm = (unsigned)__builtin_amdgcn_readlane((int)bm, winner);
            const unsigned wpos = (unsigned)__builtin_amdgcn_readlane((int)bpos, winner);
            const int wb = __builtin_amdgcn_readlane(be, winner);
            const int wi = __builtin_amdgcn_readlane(bi, winner);
            const int wp = wi / EPL, wcol = winner + 64 * (wi % EPL);
            const unsigned a = wm & free_rows;  // rows that meet the block at this step
            const int val = wb | ((__ffs(a) - 1) << 28);  // owner: the lowest row served
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                if (((wm >> p) & 1u) == 0u) continue;
                const int col = p == wp ? wcol : (int)((wpos >> (8 * p)) & 0xFFu);
                const bool mine = lane == (col & 63);
                const bool now = ((a >> p) & 1u) != 0u;
#pragma unroll
                for (int j = 0; j < EPL; ++j) {
                    if (mine && j == (col >> 6)) m[p * EPL + j] = now ? 0u : (m[p * EPL + j] & ~a);
                }
                if (now) {
                    if (lane == 0) out[p * topk + s] = val;
                    ++done[p];
                }
            }
            free_rows &= ~a;
        }
    }
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int j = 0; j < EPL; ++j) {
            const int col = lane + 64 * j;
            if (col < topk && col >= done[p]) out[p * topk + col] = -1;
        }
}

}  // namespace

size_t sel_schedule_bytes(const Shape &s) {
    const size_t groups = ((size_t)s.nb + NP - 1) / NP;
    return align_up(groups * NP * (size_t)(s.topk > 0 ? s.topk : 1) * sizeof(int32_t), 256);
}

lsrm_status launch_sel_schedule(const Shape &s, const int32_t *d_idx, int32_t *d_sched, hipStream_t st) {
    if (s.nb == 0 || s.topk == 0) return LSRM_OK;
    const int groups = (s.nb + NP - 1) / NP;
    if (s.topk <= 64)
        hipLaunchKernelGGL((build_sel_schedule<1>), dim3(groups), dim3(64), 0, st, d_idx, d_sched, s.nb, s.topk);
    else
        hipLaunchKernelGGL((build_sel_schedule<2>), dim3(groups), dim3(64), 0, st, d_idx, d_sched, s.nb, s.topk);
    LSRM_HIP_CHECK(hipGetLastError());
    return LSRM_OK;
}

}  // namespace lsrm
