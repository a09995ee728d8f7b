// NSA backward on gfx950 (App. A, Eq. nsa_1 differentiated): gradients with respect to q, k, v
// of the gated sum of the compressed, selected and window branches, routing table and gate
// weights held constant, average pooling differentiated.
//
// Per branch, with P the softmax probabilities (recomputed from the saved log-sum-exp), g the
// gate, D_i = dout_i . o_branch_i and dP = dout V^T:
//     dV = (g P)^T dout        dS = (g P) o (dP - D)        dQ = scale dS K        dK = scale dS^T Q
// A per-head gate is folded into the exponent: g P = exp2(S scale log2e - (lse log2e - log2 g)); with
// per-channel gates the incoming gradient of each branch is gate o dout instead (three images of it).
// With grouped-query heads a key/value head walks the query tiles of every query head that reads it.
//
// No floating-point atomics: the work is split into passes that each own their output rows.
//   bwd_dq_kernel    one workgroup per (query block, head): walks the same key tiles as the forward
//                    (pooled, routed, window) and accumulates dQ^T in registers.
//   bwd_dkv_kernel   one workgroup per (key block, key/value head): walks the query tiles that attend it --
//                    MODE 1: pooled keys, every query tile of the sequence (split into ranges whose
//                    partial sums are added in order by MODE 0); MODE 0: token keys, the query tiles
//                    of the window and of the reverse routing list (query blocks in ascending order),
//                    key blocks taken longest list first -- accumulates dK^T and dV^T in registers, adds
//                    the pooled gradients / 64.  With grouped-query heads the heads of a group are dealt to
//                    several workgroups, whose sums MODE 2 adds in order before finishing the rows.
// Every operand tile is a "tile image" (see forward.hip): MFMA A-operand fragments in row order
// (rows permuted so that an accumulator is directly the B operand of the next contraction); the
// fragments of the transposed tile are read out of the same bytes in LDS (see mfma_tr).  The
// transposed S^T = K Q^T form of the forward is
// used in the dQ pass (one query per lane: lse and D are per-lane scalars); the dK/dV pass uses
// S = Q K^T (one key per lane; lse and D of the 32 queries of the tile come from a small
// per-tile table copied to LDS with the tile).
// Steps are not software pipelined: the copy of tile t+1 (global -> LDS) overlaps the arithmetic of tile t, and
// nothing inside a loop may make the compiler wait for all memory operations (see tr_issue, run_segment).
#include "lsrm_internal.h"

#include <type_traits>
#include <utility>

constexpr int kBwdNbuf = 2;         // tile buffers of the dQ kernel
constexpr int kBwdDkvNbuf = 2;      // tile buffers of the dK/dV kernels (three, copies two steps ahead: slower, 51 -> 65 ms on the pooled keys at d = 128)
constexpr int kBwdSplitTarget = 2048;  // pooled-key workgroups aimed at when the query range is split

namespace lsrm {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kMaxSeg = 63;
constexpr float kLog2e = 1.4426950408889634f;

#define LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

struct BwdArgs {
    const uint16_t *q, *k, *v, *kc, *vc, *dout, *out_branch;
    const int32_t *idx;
    const float *gates, *lse;
    const char *img_q, *img_k, *img_v, *img_kc, *img_vc;  // tile images
    const char *img_do[3];    // images of the gradient that reaches each branch: one shared image of dout with
                              // per-head gates (the gate is folded into the exponent), gate o dout per branch
                              // with per-channel gates
    const uint16_t *gdo;      // per-channel gates only: [3][N][H][d] bf16, gate o dout (written by bwd_prep)
    float *aux;               // [3][N/32][H][64]: per query tile, 32 x (lse log2e - log2 g) then 32 x -D, rows permuted
    float *part_k, *part_v;   // [n_split][nbp][H][d] fp32 partial gradients of the pooled keys / values
    int32_t *rev_cnt, *rev_ptr, *rev_cur, *rev_idx;  // reverse routing lists
    uint16_t *dq, *dk, *dv;
    int32_t seg[kMaxSeg + 1];
    int64_t n;
    int nb, h, topk, window, n_seg;
    int nbc;        // compressed pairs (spatial blocks): nb unless blocks are grouped
    // spatial blocks of several 64-slot blocks (nullable): group of every block, its token range as the window
    // segment of the block (given only when the window is the spatial block), active tokens per group
    const int32_t *blk_grp, *blk_seg, *grp_tok;
    int own_block;  // window branch = the query's own block
    int h_kv, group;    // key/value heads; query heads per key/value head
    int gate_channels;  // gates are [N, 3, H, d]
    const int32_t *count;  // nullable [NB]: active tokens per block; the other slots are neither queries nor keys
    int nt;               // query / key tiles of 32 tokens
    int n_split, nbp, tiles_per_split;
    // token keys with grouped-query heads: the query heads of a group are dealt to hsplit workgroups, hpw heads each,
    // whose fp32 sums [hsplit][NB * 64][H_kv][d] a last pass adds up in order (hsplit == 1: no such pass)
    int hsplit, hpw;
    float *hpart_k, *hpart_v;
    const int32_t *order;  // [NB] key blocks, longest reverse list first: the order the token-key workgroups start in
    float scale, sl2;
};

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    bf16x2 p;
    p[0] = (__bf16)a;
    p[1] = (__bf16)b;
    return *reinterpret_cast<uint32_t *>(&p);
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// row permutation of the tile images: bits 2 and 3 swapped
__device__ __forceinline__ int perm32(int r) { return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1); }

union BFrag {
    bf16x8 v;
    uint32_t u[4];
};

// accumulator tile -> the two B operands (16-row slabs) of the next contraction
__device__ __forceinline__ void to_b_operand(const float (&x)[16], BFrag (&b)[2]) {
#pragma unroll
    for (int k = 0; k < 8; ++k) b[k / 4].u[k % 4] = pack_bf16(x[2 * k], x[2 * k + 1]);
}

// MFMAs whose accumulator stays in ordinary VGPRs, written as inline assembly.  A kernel compiled for one wavefront
// per SIMD (more than 256 registers) gets every MFMA builtin in the form that accumulates in AGPRs; results that the
// vector ALU must read (scores, dP) then travel through v_accvgpr_read/write, and the register allocator was seen to
// park them in the AGPRs of the long-lived dK/dV accumulators, saving and restoring those around every chain (about
// 100 register moves per step).  The hardware does not interlock "MFMA result read by a VALU instruction" and the
// compiler cannot pad what it does not see, so a chain ends with mfma_v_settle (24 wait states cover the 8 passes).
__device__ __forceinline__ void mfma_v_first(f32x16 &d, bf16x8 a, bf16x8 b) {
    asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma_v(f32x16 &d, bf16x8 a, bf16x8 b) {
    asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma_v_settle(f32x16 &d) { asm volatile("s_nop 15\n\ts_nop 7" : "+v"(d)); }

// copies n_kb KB, contiguous on both sides, global -> LDS; the two wavefronts of the workgroup split it
template <int N_KB>
__device__ __forceinline__ void copy_kb(const char *src, char *dst, int wave, uint32_t lane16) {
    static_assert(N_KB % 2 == 0, "");
    src += wave * 1024;
    dst += wave * 1024;
#pragma unroll
    for (int i = 0; i < N_KB; i += 2)
        __builtin_amdgcn_global_load_lds(GLB_PTR(src + i * 1024 + lane16), LDS_PTR(dst + i * 1024), 16, 0, 0);
}

// s_waitcnt vmcnt <= n (and lgkmcnt == 0), and a raw barrier.  Neither this barrier nor __syncthreads() waits
// for global -> LDS copies in flight: whoever issued them waits on vmcnt before the barrier that publishes them.
constexpr int vm_lgkm_imm(int n) { return (n & 0xF) | ((n >> 4) << 14) | 0x0070; }
__device__ __forceinline__ void wg_barrier() { asm volatile("s_barrier" ::: "memory"); }

// A-operand fragment of the TRANSPOSE of a tile, read out of the tile's row-order fragments in LDS with
// the transposing LDS load of gfx950 (ds_read_b64_tr_b16): within each group of 16 lanes, lane j receives
// as element e the 16-bit element j % 4 of what lane 4 e + j / 4 of the group addressed.  So a lane of the
// group addresses the four channels 4 (s % 4) .. + 3 of tile row s / 4 (s its index in the group), and
// lane j ends up with one channel of four consecutive rows -- four of the eight K-values of a fragment
// whose rows are channels.  Fragment (ks2, dt): channel 32 dt + (lane & 31), tile rows 16 ks2 + 8 hh + 0..7.
// `tr_lane_offset` is the per-lane part of the address inside the row-order fragments; the fragment adds
// dt * 2048 + ks2 * 256 and the second half of the rows another 128 (rows are stored permuted).
// This halves what a step copies into LDS: the transposed halves of the tile images stay in memory.
// In the backward's tile images the 16-byte slot of (row position r, channel half h) inside a fragment is
// h * 32 + (r ^ 4 h): without the xor the two channel halves that a group of 16 lanes addresses in one
// transposing load lie 512 bytes apart, i.e. in the same banks (measured: half the LDS cycles of these
// kernels were bank conflicts); with it the group's 16 addresses cover 32 distinct banks.
__device__ __forceinline__ uint32_t tr_lane_offset(int lane) {
    const int s = lane & 15, grp = lane >> 4;
    const int c = s & 3, k_local = s >> 2, hh = grp >> 1;
    return (uint32_t)((grp & 1) * 1024 + (c >> 1) * 512 + (4 * (hh ^ (c >> 1)) + k_local) * 16 + (c & 1) * 8);
}
// per-lane offset of this lane's 16 bytes inside a row-order fragment of such an image
__device__ __forceinline__ uint32_t row_lane_offset(int lane) {
    const int r = lane & 31, hh = lane >> 5;
    return (uint32_t)((hh * 32 + (r ^ (hh << 2))) * 16);
}
// The loads are written as inline assembly on purpose.  The compiler cannot tell that a transposing load
// (the builtin) does not touch the buffer that the global -> LDS copies of the next step are filling, and puts
// an s_waitcnt vmcnt(0) before the first of them: every step then waits for the copies it has just issued,
// and nothing is prefetched (seen in the assembly and in timestamps).  Loads it does not see get no such wait;
// in exchange their results are waited for by hand: tr_take ties a counted lgkmcnt wait to the registers of a
// fragment (LDS operations complete in order, so "at most n outstanding" covers all but the last n issued).
typedef int i32x2 __attribute__((ext_vector_type(2)));
struct TrFrag {
    i32x2 lo, hi;
};
template <int OFF>
__device__ __forceinline__ void tr_issue(TrFrag &f, uint32_t addr) {
    asm volatile("ds_read_b64_tr_b16 %0, %2 offset:%3\n\tds_read_b64_tr_b16 %1, %2 offset:%4"
                 : "=&v"(f.lo), "=&v"(f.hi)
                 : "v"(addr), "n"(OFF), "n"(OFF + 128)
                 : "memory");
}
template <int N>
__device__ __forceinline__ bf16x8 tr_take(TrFrag &f) {
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(f.lo), "+v"(f.hi) : "n"(N) : "memory");
    union {
        i32x2 h[2];
        bf16x8 v;
    } u;
    u.h[0] = f.lo;
    u.h[1] = f.hi;
    return u.v;
}

// acc[dt] += (fragment (ks2, dt) of the transposed tile) x b[ks2] for every dt and ks2: all 2 ND fragments are
// requested at once and each MFMA waits for its own.  rows: the tile's row-order fragments in LDS.
template <int ND, int... I>
__device__ __forceinline__ void mfma_tr_impl(f32x16 (&acc)[ND], uint32_t addr, const BFrag (&b)[2],
                                             std::integer_sequence<int, I...>) {
    TrFrag f[2 * ND];
    (tr_issue<(I % ND) * 2048 + (I / ND) * 256>(f[I], addr), ...);
    ((acc[I % ND] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_take<2 * (2 * ND - 1 - I)>(f[I]), b[I / ND].v,
                                                            acc[I % ND], 0, 0, 0)),
     ...);
}
template <int ND>
__device__ __forceinline__ void mfma_tr(f32x16 (&acc)[ND], const char *rows, uint32_t lane_off, const BFrag (&b)[2]) {
    // (the low 32 bits of a generic pointer into LDS are the LDS address)
    mfma_tr_impl<ND>(acc, (uint32_t)(uintptr_t)rows + lane_off, b, std::make_integer_sequence<int, 2 * ND>{});
}

// f(integral_constant<0>), ..., f(integral_constant<N - 1>), in order
template <typename F, int... K>
__device__ __forceinline__ void for_each_index_impl(F &f, std::integer_sequence<int, K...>) {
    (f(std::integral_constant<int, K>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void for_each_index(F &f) {
    for_each_index_impl(f, std::make_integer_sequence<int, N>{});
}

template <int D>
struct BGeo {
    static constexpr int NS = D / 16, ND = D / 32;
    static constexpr int ROW = 32 * D * 2;  // row-order fragments of a tile
    static constexpr int TB = D * 64;       // fragments of the transposed tile
    static constexpr int IMG = ROW;         // the backward's images hold the row-order fragments only
    static constexpr int OUT_ROW = 2 * D + 8;  // padded bf16 row of the output staging (bytes)
};

// rows of a [D x 32] accumulator pair set (transposed gradient tile) -> bf16 rows of `dst`
// (32 rows of this wavefront, row stride h*D elements), staged through LDS so that rows are
// written as whole 16-byte chunks.  x[dt][i]: channel 32 dt + (i/4)*8 + hh*4 + i%4, row lane%32.
template <int D>
__device__ __forceinline__ void store_rows_transposed(const float (&x)[D / 32][16], char *stage, uint16_t *dst,
                                                      int64_t row_stride, int lane) {
    using G = BGeo<D>;
    const int r = lane & 31, hh = lane >> 5;
#pragma unroll
    for (int dt = 0; dt < G::ND; ++dt)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            uint2 w2;
            w2.x = pack_bf16(x[dt][4 * gq + 0], x[dt][4 * gq + 1]);
            w2.y = pack_bf16(x[dt][4 * gq + 2], x[dt][4 * gq + 3]);
            *reinterpret_cast<uint2 *>(stage + r * G::OUT_ROW + (32 * dt + 8 * gq + 4 * hh) * 2) = w2;
        }
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): this wavefront's own staging writes
    constexpr int CH = D / 8, RPP = 64 / CH;
#pragma unroll
    for (int it = 0; it < 32 / RPP; ++it) {
        const int rr = it * RPP + lane / CH, ch = lane % CH;
        uint4 val = *reinterpret_cast<const uint4 *>(stage + rr * G::OUT_ROW + ch * 16);
        *reinterpret_cast<uint4 *>(dst + rr * row_stride + ch * 8) = val;
    }
}

// ---------------------------------------------------------------------------------------------
// per (token, head): the per-branch exponent offset and D = dout . o_branch, in tile-image row order
// Threads: 8 channels each.  A workgroup takes one query tile and PREP_HB heads: thread = (head, row of the tile,
// 16-byte chunk of the row), chunks fastest, so a row's d channels are read by d / 8 neighbouring lanes (16-byte
// loads, contiguous per row) and the 32 table entries of a (tile, head) are written from one wavefront, side by side.
template <int D>
struct PrepGeo {
    static constexpr int CH = D / 8;                            // chunks = lanes per (row, head)
    static constexpr int HB = CH * 32 >= 256 ? 1 : 256 / (CH * 32);  // heads per workgroup
    static constexpr int THREADS = HB * 32 * CH;
};
template <int D>
__global__ __launch_bounds__(PrepGeo<D>::THREADS) void bwd_prep(BwdArgs a) {
    using P = PrepGeo<D>;
    constexpr int CH = P::CH;
    const int c = threadIdx.x % CH, r = (threadIdx.x / CH) % 32;
    const int heads_x = (a.h + P::HB - 1) / P::HB;
    const int64_t tile = blockIdx.x / heads_x;
    const int head = (int)(blockIdx.x % heads_x) * P::HB + threadIdx.x / (CH * 32);
    if (head >= a.h) return;  // (whole groups of CH lanes leave together)
    const int64_t row = tile * 32 + r;
    float dov[8];
    {
        const uint4 w = *reinterpret_cast<const uint4 *>(a.dout + (row * a.h + head) * D + 8 * c);
        const uint32_t u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            dov[2 * j] = bf16_lo(u[j]);
            dov[2 * j + 1] = bf16_hi(u[j]);
        }
    }
    const int pr = perm32(r);
    // a padding slot is no query: zero probabilities (offset +inf) and a zero D in every branch
    const bool padding = a.count != nullptr && (int)(row & 63) >= a.count[row >> 6];
#pragma unroll
    for (int b = 0; b < 3; ++b) {
        const uint4 w = *reinterpret_cast<const uint4 *>(a.out_branch + (((int64_t)b * a.n + row) * a.h + head) * D + 8 * c);
        const uint32_t u[4] = {w.x, w.y, w.z, w.w};
        float dl = 0.f;
        if (a.gate_channels) {
            // the gradient reaching this branch is gate o dout, channel by channel: D uses it, and its
            // bf16 rounding is kept for the contractions
            const f32x4 *gch = reinterpret_cast<const f32x4 *>(a.gates + ((row * 3 + b) * a.h + head) * D + 8 * c);
            const f32x4 g_lo = gch[0], g_hi = gch[1];
            const float g[8] = {g_lo[0], g_lo[1], g_lo[2], g_lo[3], g_hi[0], g_hi[1], g_hi[2], g_hi[3]};
            uint32_t o4[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float g0 = g[2 * j] * dov[2 * j], g1 = g[2 * j + 1] * dov[2 * j + 1];
                dl += g0 * bf16_lo(u[j]) + g1 * bf16_hi(u[j]);
                o4[j] = pack_bf16(g0, g1);
            }
            *reinterpret_cast<uint4 *>(const_cast<uint16_t *>(a.gdo) + (((int64_t)b * a.n + row) * a.h + head) * D + 8 * c) =
                make_uint4(o4[0], o4[1], o4[2], o4[3]);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) dl += dov[2 * j] * bf16_lo(u[j]) + dov[2 * j + 1] * bf16_hi(u[j]);
        }
        // D of the row: the sum over its CH lanes, in a fixed order
#pragma unroll
        for (int m = 1; m < CH; m <<= 1) dl += __shfl_xor(dl, m);
        if (c != 0) continue;
        const float lse = a.lse[((int64_t)b * a.n + row) * a.h + head];
        // an empty key set (lse = -inf) or a zero gate gives zero probabilities: offset +inf
        float l2 = __builtin_inff();
        if (a.gate_channels) {
            if (lse > -__builtin_inff()) l2 = lse * kLog2e;
        } else {
            const float g = a.gates[(row * a.h + head) * 3 + b];
            if (g > 0.f && lse > -__builtin_inff()) l2 = lse * kLog2e - __log2f(g);
        }
        float *ax = a.aux + (((int64_t)b * a.nt + tile) * a.h + head) * 64;
        ax[pr] = padding ? __builtin_inff() : l2;
        ax[32 + pr] = padding ? 0.f : -dl;  // negated: the kernels start the dP accumulators from it
    }
}

// ---------------------------------------------------------------------------------------------
// reverse routing lists: for every key block the query blocks that list it, ascending
__global__ void fill_zero(int32_t *p, int n) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}
__global__ void rev_count(BwdArgs a) {
    int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= a.nb * a.topk) return;
    int v = a.idx[e];
    if (v >= 0 && v < a.nb) atomicAdd(&a.rev_cnt[v], 1);
}
__global__ __launch_bounds__(1024) void rev_scan(BwdArgs a) {
    __shared__ int part[1024];
    const int t = threadIdx.x;
    const int chunk = (a.nb + 1023) / 1024;
    const int lo = min(t * chunk, a.nb), hi = min(lo + chunk, a.nb);
    int s = 0;
    for (int i = lo; i < hi; ++i) s += a.rev_cnt[i];
    part[t] = s;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
        int x = t >= off ? part[t - off] : 0;
        __syncthreads();
        part[t] += x;
        __syncthreads();
    }
    int run = part[t] - s;  // exclusive prefix of this chunk
    for (int i = lo; i < hi; ++i) {
        a.rev_ptr[i] = run;
        a.rev_cur[i] = run;
        run += a.rev_cnt[i];
    }
    if (t == 1023) a.rev_ptr[a.nb] = part[1023];
}
// The key blocks in order of falling reverse-list length (within 1024 length classes; equal lengths in any
// order -- it only decides which workgroup starts when).  The token-key dK/dV workgroups take their block from
// this list: the long walks start first instead of forming the tail of the kernel, and the round-robin of
// workgroups over the XCDs spreads them, where a contiguous range of blocks per XCD left the popular blocks
// (say, all image blocks) to one or two XCDs.
__global__ __launch_bounds__(1024) void rev_order(BwdArgs a, int32_t *order) {
    __shared__ int bin[1024];
    const int t = threadIdx.x;
    bin[t] = 0;
    __syncthreads();
    for (int b = t; b < a.nb; b += 1024) atomicAdd(&bin[min(a.rev_cnt[b], 1023)], 1);
    __syncthreads();
    if (t == 0) {  // start of each class, longest first
        int run = 0;
        for (int c = 1023; c >= 0; --c) {
            const int n = bin[c];
            bin[c] = run;
            run += n;
        }
    }
    __syncthreads();
    for (int b = t; b < a.nb; b += 1024) order[atomicAdd(&bin[min(a.rev_cnt[b], 1023)], 1)] = b;
}
__global__ void rev_fill(BwdArgs a) {
    int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= a.nb * a.topk) return;
    int v = a.idx[e];
    if (v >= 0 && v < a.nb) a.rev_idx[atomicAdd(&a.rev_cur[v], 1)] = e / a.topk;
}
// Puts every list in ascending order (the fill order is whatever the atomics gave; a fixed order makes the
// gradients reproducible, and ascending keeps consecutive query tiles together).  The entries of a list are
// block numbers, distinct unless a row of the table repeats a block: one wavefront per key block marks them in
// a bitmap of nb bits in LDS and reads the bitmap back in order.
__global__ __launch_bounds__(64) void rev_sort(BwdArgs a) {
    extern __shared__ uint32_t bits[];  // (nb + 31) / 32 words
    const int b = blockIdx.x, lane = threadIdx.x;
    const int words = (a.nb + 31) >> 5;
    int32_t *x = a.rev_idx + a.rev_ptr[b];
    const int len = a.rev_ptr[b + 1] - a.rev_ptr[b];
    if (len <= 1) return;
    for (int w = lane; w < words; w += 64) bits[w] = 0u;
    __syncthreads();
    for (int i = lane; i < len; i += 64) atomicOr(&bits[x[i] >> 5], 1u << (x[i] & 31));
    __syncthreads();
    // a table may list a block twice in one row (it is then attended twice): the bitmap would drop the repeat,
    // so such a list is sorted the slow way
    int marked = 0;
    for (int w = lane; w < words; w += 64) marked += __popc(bits[w]);
    for (int off = 32; off > 0; off >>= 1) marked += __shfl_xor(marked, off);
    if (marked != len) {
        if (lane == 0)
            for (int i = 1; i < len; ++i) {
                int v = x[i], j = i - 1;
                while (j >= 0 && x[j] > v) {
                    x[j + 1] = x[j];
                    --j;
                }
                x[j + 1] = v;
            }
        return;
    }
    int base = 0;
    for (int w0 = 0; w0 < words; w0 += 64) {
        const int w = w0 + lane;
        uint32_t m = w < words ? bits[w] : 0u;
        const int c = __popc(m);
        int pre = c;  // inclusive prefix sum over the lanes
        for (int off = 1; off < 64; off <<= 1) {
            const int t = __shfl_up(pre, off);
            if (lane >= off) pre += t;
        }
        int at = base + pre - c;
        while (m != 0u) {
            x[at++] = (w << 5) + (__ffs(m) - 1);
            m &= m - 1u;
        }
        base += __shfl(pre, 63);
    }
}
// the same for sequences too long for the bitmap: insertion sort, one thread per list
__global__ void rev_sort_serial(BwdArgs a) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= a.nb) return;
    int32_t *x = a.rev_idx + a.rev_ptr[b];
    const int len = a.rev_ptr[b + 1] - a.rev_ptr[b];
    for (int i = 1; i < len; ++i) {
        int v = x[i], j = i - 1;
        while (j >= 0 && x[j] > v) {
            x[j + 1] = x[j];
            --j;
        }
        x[j + 1] = v;
    }
}

// Position of the n-th (from 0) set bit of m; 0 <= result <= 63 whatever n is (meaningful for n < popcount(m)).
__device__ __forceinline__ int nth_set_bit(unsigned long long m, int n) {
    int pos = 0;
#pragma unroll
    for (int w = 32; w >= 1; w >>= 1) {
        const int below = __popcll(m & ((1ull << w) - 1ull));
        if (n >= below) {
            n -= below;
            m >>= w;
            pos += w;
        }
    }
    return pos;
}

// The partial gradients of the pooled keys / values, summed over the query ranges in order into range 0's slot,
// so that the token-key workgroups read one row per pooled pair however many ranges there were.
__global__ __launch_bounds__(256) void sum_parts(float *__restrict__ part_k, float *__restrict__ part_v, int n_split,
                                                 int64_t per_split) {
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= per_split) return;
#pragma unroll
    for (int which = 0; which < 2; ++which) {
        float *part = which == 0 ? part_k : part_v;
        f32x4 acc = *reinterpret_cast<const f32x4 *>(part + i);
        for (int sp = 1; sp < n_split; ++sp) acc += *reinterpret_cast<const f32x4 *>(part + sp * per_split + i);
        *reinterpret_cast<f32x4 *>(part + i) = acc;
    }
}

// ---------------------------------------------------------------------------------------------
// dQ: one workgroup (2 wavefronts x 32 query rows) per (query block, head)
// WIDE: routing rows of 65..128 entries (two per lane of the list holder instead of one).
template <int D, bool WIDE>
__global__ __launch_bounds__(128, 2) void bwd_dq_kernel(BwdArgs a) {
    // (at d = 128 the 256-register budget of two workgroups per SIMD still holds: 64 accumulator registers)
    using G = BGeo<D>;
    constexpr int NS = G::NS, ND = G::ND;
    constexpr int TILE = 2 * G::ROW;     // K rows | V rows (K^T is read out of the K rows, see mfma_tr)
    constexpr int NBUF = kBwdNbuf;  // tile buffers: copies run NBUF - 1 tiles ahead
    static_assert((G::ROW / 1024) % 2 == 0, "");
    static_assert(2 * 32 * G::OUT_ROW <= NBUF * TILE, "output staging fits in the tile buffers");
    __shared__ __attribute__((aligned(1024))) char lds[NBUF * TILE];
    // consecutive workgroup ids go round-robin to the 8 XCDs: give each XCD a contiguous range of
    // blocks so that neighbouring blocks (overlapping windows, similar routed sets) share its L2
    const int per_xcd = (a.nb + 7) / 8;
    const int qb = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3), head = blockIdx.y;
    if (qb >= a.nb) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, hh = lane >> 5;
    const uint32_t lane16 = (uint32_t)lane * 16u;
    const int64_t row0 = (int64_t)qb * 64 + 32 * wave;
    const int half_w = a.window / 2;
    const int kvh = head / a.group;  // key/value head of this query head
    const uint32_t tr_off = tr_lane_offset(lane), row_off = row_lane_offset(lane);

    bf16x8 qf[NS], dof[NS];
    // the gradient rows of branch b: dout itself, or gate o dout with per-channel gates
    // (a padding slot reads as zeros: whatever the caller left there never reaches an MFMA)
    const bool padding = a.count != nullptr && 32 * wave + r >= a.count[qb];
    const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    auto load_dof = [&](int b) {
        const uint16_t *src = a.gate_channels ? a.gdo + (int64_t)b * a.n * a.h * D : a.dout;
        const uint16_t *drow = src + ((row0 + r) * a.h + head) * D + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < NS; ++ks) dof[ks] = padding ? zero8 : *reinterpret_cast<const bf16x8 *>(drow + 16 * ks);
    };
    {
        const uint16_t *qrow = a.q + ((row0 + r) * a.h + head) * D + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < NS; ++ks) qf[ks] = padding ? zero8 : *reinterpret_cast<const bf16x8 *>(qrow + 16 * ks);
        load_dof(0);
    }
    float l2[3], dl[3];
#pragma unroll
    for (int b = 0; b < 3; ++b) {
        const float *ax = a.aux + (((int64_t)b * a.nt + (row0 >> 5)) * a.h + head) * 64;
        l2[b] = ax[perm32(r)];
        dl[b] = ax[32 + perm32(r)];
    }
    f32x16 acc[ND];
#pragma unroll
    for (int dt = 0; dt < ND; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[dt][i] = 0.f;

    // ---- the tiles of this query block: pooled, routed, window
    const int tc = (a.nbc + 31) / 32;
    // the routing row, valid entries first: entry u sits in lane u % 64 of register u / 64.  Compacted with lane
    // permutes, not through LDS memory: with a second LDS object in the kernel the compiler can no longer tell the
    // tile buffers' reads from the copies in flight and puts a full vmcnt wait in front of the first read of every
    // step (measured: the kernel 8 % slower).
    constexpr int NR = WIDE ? 2 : 1;
    int packed[NR], pcount[NR], n_valid = 0;
    {
        int v[NR], nv[NR];
        unsigned long long bal[NR];
#pragma unroll
        for (int j = 0; j < NR; ++j) {
            const int col = lane + 64 * j;
            v[j] = col < a.topk ? a.idx[(int64_t)qb * a.topk + col] : -1;
            if (v[j] >= a.nb) v[j] = -1;
            bal[j] = __ballot(v[j] >= 0);
            nv[j] = __popcll(bal[j]);
            n_valid += nv[j];
        }
#pragma unroll
        for (int j = 0; j < NR; ++j) {
            // the entry of rank lane + 64 j: the (rank)-th valid one of register 0, or the (rank - nv[0])-th of register 1
            const int rank = lane + 64 * j;
            int val = __builtin_amdgcn_ds_bpermute(4 * nth_set_bit(bal[0], rank), v[0]);
            if constexpr (WIDE) {
                const int val1 = __builtin_amdgcn_ds_bpermute(4 * nth_set_bit(bal[1], rank - nv[0]), v[1]);
                if (rank >= nv[0]) val = val1;
            }
            packed[j] = rank < n_valid ? val : -1;
        }
    }
    // active tokens of the routed blocks, held like the list itself
#pragma unroll
    for (int j = 0; j < NR; ++j) pcount[j] = a.count != nullptr && lane + 64 * j < n_valid ? a.count[packed[j]] : 64;
    auto entry = [&](const int (&reg)[NR], int u) {  // wave-uniform u
        if constexpr (WIDE) {
            const int e0 = __builtin_amdgcn_readlane(reg[0], u & 63), e1 = __builtin_amdgcn_readlane(reg[NR - 1], u & 63);
            return u < 64 ? e0 : e1;
        } else {
            return __builtin_amdgcn_readlane(reg[0], u);
        }
    };
    const int ts = 2 * n_valid;
    int seg_lo = 0, seg_hi = 0;
    if (a.blk_seg != nullptr) {  // the query's spatial block
        seg_lo = a.blk_seg[2 * qb];
        seg_hi = a.blk_seg[2 * qb + 1];
    } else {
        for (int s = 0; s < a.n_seg; ++s)
            if (qb * 64 >= a.seg[s] && qb * 64 < a.seg[s + 1]) {
                seg_lo = a.seg[s];
                seg_hi = a.seg[s + 1];
            }
    }
    if (a.own_block) {  // window = the query's own block: the block is its own segment (a.window is 128)
        seg_lo = qb * 64;
        seg_hi = qb * 64 + 64;  // (padding slots at its end are masked per tile below)
    }
    const int k_start = max(seg_lo, qb * 64 - half_w), k_end = min(seg_hi, qb * 64 + 63 + half_w);
    const int st0 = k_start / 32;
    // active tokens of the blocks of the window range, one per lane (a range of more than 64 blocks falls back to
    // loading the count inside the loop)
    const int wcount = a.count != nullptr && (st0 >> 1) + lane < a.nb ? a.count[(st0 >> 1) + lane] : 64;
    const int tw = k_end > k_start ? (k_end - 1) / 32 + 1 - st0 : 0;
    const int T = tc + ts + tw;
    const int wlo = max(seg_lo, (int)row0 + r - half_w), whi = min(seg_hi, (int)row0 + r + half_w);

    // Two tile buffers: the copy of tile t+1 is issued behind the barrier of step t and waited for before the
    // barrier of step t+1.  The walk is one pipelined loop per branch, so that everything that depends on the
    // branch (tile lookup, image, mask rule, table entries) is fixed inside a loop; the first tile of the next
    // branch is requested in the last step of the one before it, so the pipeline never drains.
    static_assert(NBUF == 2, "");
    auto issue_tile = [&](const char *kimg, const char *vimg, int tile, char *buf) {
        const int64_t off = (int64_t)((uint32_t)tile * (uint32_t)a.h_kv + (uint32_t)kvh) * G::IMG;
        copy_kb<G::ROW / 1024>(kimg + off, buf, wave, lane16);
        copy_kb<G::ROW / 1024>(vimg + off, buf + G::ROW, wave, lane16);
    };
    // tile of step t of the whole walk (used at the branch boundaries only)
    auto issue_any = [&](int t, char *buf) {
        if (t < tc) {
            issue_tile(a.img_kc, a.img_vc, t, buf);
        } else if (t < tc + ts) {
            const int u = t - tc;
            issue_tile(a.img_k, a.img_v, 2 * entry(packed, u >> 1) + (u & 1), buf);
        } else {
            issue_tile(a.img_k, a.img_v, st0 + (t - tc - ts), buf);
        }
    };
    // steps [t0, t1) of the walk, all of branch BR.  tile_fn(u): image tile of the u-th step of the branch;
    // mask_fn(u, &j0, &lo, &hi) -> does this tile need a mask: key j0 + (position in the tile) is attended iff
    // lo <= key < hi (per lane)
    auto run_branch = [&](int t0, int t1, auto br_c, const char *kimg, const char *vimg, auto tile_fn, auto mask_fn) {
        constexpr int BR = decltype(br_c)::value;
        const float lb = l2[BR];
        f32x16 dp0;  // -D of this lane's query: the dP accumulator starts from it, so the MFMAs leave dP - D
#pragma unroll
        for (int i = 0; i < 16; ++i) dp0[i] = dl[BR];
        for (int t = t0; t < t1; ++t) {
            // tile t has landed (this wavefront's share; the barrier covers the other's); both wavefronts are done
            // with tile t-1, whose buffer takes tile t+1
            __builtin_amdgcn_s_waitcnt(vm_lgkm_imm(0));
            wg_barrier();
            char *nbuf = lds + ((t + 1) & 1) * TILE;
            const char *tile_k = lds + (t & 1) * TILE;
            const char *base = tile_k + row_off;

            // The pieces of the step in a fixed order (a wavefront issues in order: what is to overlap has to alternate
            // in the program).  K and V row fragments go through one rolling queue of QD registers sets, refilled
            // behind the MFMA that consumed a set; the score chain, then the dP chain with the tile's exponentials
            // behind its MFMAs (unmasked; edge tiles are fixed up afterwards); then the transposing loads of K^T are
            // requested, dS of the first 16-key slab is formed, and the dQ MFMAs run with the second slab's dS
            // behind the first ones.
            constexpr int QD = NS < 4 ? NS : 4;
            bf16x8 fq[QD];
            auto frag = [&](int i) {  // fragment i of the K rows (i < NS) or of the V rows
                return *reinterpret_cast<const bf16x8 *>(base + (i < NS ? i * 1024 : G::ROW + (i - NS) * 1024));
            };
#pragma unroll
            for (int i = 0; i < QD; ++i) fq[i] = frag(i);
            __builtin_amdgcn_sched_barrier(0);
            // the copies of the next tile: their address arithmetic runs while the first reads land
            if (t + 1 < t1)
                issue_tile(kimg, vimg, tile_fn(t + 1 - t0), nbuf);
            else if (t + 1 < T)
                issue_any(t + 1, nbuf);
            int j0, lo, hi;
            const bool need_mask = mask_fn(t - t0, &j0, &lo, &hi);
            f32x16 s, dp;
#pragma unroll
            for (int i = 0; i < 16; ++i) s[i] = 0.f;
            __builtin_amdgcn_sched_barrier(0);
            auto s_step = [&](auto kc) {
                constexpr int ks = decltype(kc)::value;
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[ks % QD], qf[ks], s, 0, 0, 0);
                fq[ks % QD] = frag(ks + QD);
                __builtin_amdgcn_sched_barrier(0);
            };
            for_each_index<NS>(s_step);
            constexpr int E = 16 / NS;  // exponentials per dP MFMA
            float pr[16];
            auto dp_step = [&](auto kc) {
                constexpr int ks = decltype(kc)::value;
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[ks % QD], dof[ks], ks == 0 ? dp0 : dp, 0, 0, 0);
                if constexpr (ks + QD < NS) fq[ks % QD] = frag(NS + ks + QD);
#pragma unroll
                for (int e = ks * E; e < (ks + 1) * E; ++e) {
                    pr[e] = __builtin_amdgcn_exp2f(s[e] * a.sl2 - lb);
                    asm volatile("" : "+v"(pr[e]));
                }
                __builtin_amdgcn_sched_barrier(0);
            };
            for_each_index<NS>(dp_step);
            // with per-channel gates the gradient rows change with the branch: the next branch's are requested
            // once the last dP MFMAs of this one are issued, and have arrived by the wait at the top of the next step
            if (BR < 2 && a.gate_channels && t + 1 == t1 && t + 1 < T) load_dof(t + 1 < tc + ts ? 1 : 2);
            TrFrag ft[2 * ND];
            const uint32_t tr_k = (uint32_t)(uintptr_t)tile_k + tr_off;
            auto issue_tr = [&](auto ic) {
                constexpr int I = decltype(ic)::value;
                tr_issue<(I % ND) * 2048 + (I / ND) * 256>(ft[I], tr_k);
            };
            for_each_index<2 * ND>(issue_tr);
            if (__builtin_expect(need_mask, 0)) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int j = j0 + 16 * (i / 8) + 8 * hh + (i % 8);
                    pr[i] = ((j >= lo) & (j < hi)) ? pr[i] : 0.f;
                }
            }
            BFrag dsb[2];
#pragma unroll
            for (int k = 0; k < 4; ++k) dsb[0].u[k] = pack_bf16(pr[2 * k] * dp[2 * k], pr[2 * k + 1] * dp[2 * k + 1]);
            __builtin_amdgcn_sched_barrier(0);
            constexpr int EQ = 4 / ND > 0 ? 4 / ND : 1;  // bf16 pairs of the second slab's dS per MFMA of the first slab
            auto dq_step = [&](auto ic) {
                constexpr int I = decltype(ic)::value;
                acc[I % ND] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_take<2 * (2 * ND - 1 - I)>(ft[I]), dsb[I / ND].v,
                                                                      acc[I % ND], 0, 0, 0);
                if constexpr (I < ND) {
#pragma unroll
                    for (int k = 4 + I * EQ; k < 4 + (I + 1) * EQ && k < 8; ++k) {
                        dsb[1].u[k - 4] = pack_bf16(pr[2 * k] * dp[2 * k], pr[2 * k + 1] * dp[2 * k + 1]);
                        asm volatile("" : "+v"(dsb[1].u[k - 4]));
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            };
            for_each_index<2 * ND>(dq_step);
        }
    };
    // padding slots at the end of a tile's block are no keys: valid keys of the tile, given its block's count
    auto valid_keys = [&](int cnt, int half) { return min(32, max(0, cnt - 32 * half)); };

    if (T > 0) issue_any(0, lds);
    // pooled keys: only the last tile can reach past the end
    run_branch(0, tc, std::integral_constant<int, 0>{}, a.img_kc, a.img_vc, [&](int u) { return u; },
               [&](int u, int *j0, int *lo, int *hi) {
                   *j0 = 32 * u;
                   *lo = 0;
                   *hi = a.nbc;
                   return 32 * u + 32 > a.nbc;
               });
    // routed blocks: every key counts, except padding slots
    run_branch(tc, tc + ts, std::integral_constant<int, 1>{}, a.img_k, a.img_v,
               [&](int u) { return 2 * entry(packed, u >> 1) + (u & 1); },
               [&](int u, int *j0, int *lo, int *hi) {
                   *j0 = 0;
                   *lo = 0;
                   *hi = 32;
                   if (a.count == nullptr) return false;
                   *hi = valid_keys(entry(pcount, u >> 1), u & 1);
                   return *hi < 32;
               });
    // window: the band's edges and the segment's ends, and padding slots
    const int edge_lo = max(seg_lo, (int)row0 + 31 - half_w), edge_hi = min(seg_hi, (int)row0 + half_w);
    run_branch(tc + ts, T, std::integral_constant<int, 2>{}, a.img_k, a.img_v, [&](int u) { return st0 + u; },
               [&](int u, int *j0, int *lo, int *hi) {
                   const int st = st0 + u;
                   *j0 = 32 * st;
                   *lo = wlo;
                   *hi = whi;
                   bool need = 32 * st < edge_lo || 32 * st + 32 > edge_hi;
                   if (a.count != nullptr) {
                       const int wb = (st >> 1) - (st0 >> 1);  // block of the window range
                       const int cnt = wb < 64 ? __builtin_amdgcn_readlane(wcount, wb) : a.count[st >> 1];
                       const int vld = valid_keys(cnt, st & 1);
                       if (vld < 32) {
                           need = true;
                           *hi = min(*hi, 32 * st + vld);
                       }
                   }
                   return need;
               });
    __syncthreads();  // the tile buffers become the output staging
    float x[ND][16];
#pragma unroll
    for (int dt = 0; dt < ND; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) x[dt][i] = acc[dt][i] * a.scale;
    store_rows_transposed<D>(x, lds + wave * 32 * G::OUT_ROW, a.dq + (row0 * a.h + head) * D, (int64_t)a.h * D, lane);
}

// ---------------------------------------------------------------------------------------------
// dK, dV: one workgroup (2 wavefronts x 32 keys) per (key block, head[, query range])
// blockIdx.y is the key/value head; the query tiles of each of its `group` query heads are walked in turn.
// (d = 128: the two [128 x 32] accumulator sets alone take 128 registers, so one workgroup per SIMD.)
template <int D, int MODE>
__global__ __launch_bounds__(128, (D == 128 ? 1 : 3)) void bwd_dkv_kernel(BwdArgs a) {
    using G = BGeo<D>;
    constexpr int NS = G::NS, ND = G::ND;
    constexpr int AUX = 2 * G::ROW;          // Q rows | dO rows | table (64 floats); Q^T and dO^T: see mfma_tr
    constexpr int TILE = 2 * G::ROW + 1024;  // (table padded to keep the next buffer aligned)
    static_assert(2 * 32 * G::OUT_ROW <= kBwdDkvNbuf * TILE, "output staging fits in the tile buffers");
    extern __shared__ __attribute__((aligned(1024))) char lds[];  // kBwdDkvNbuf * TILE bytes
    const int n_kb = MODE != 1 ? a.nb : a.nbp / 64;
    const int per_xcd = (n_kb + 7) / 8;
    const int head = blockIdx.y;
    int kb;
    if (MODE == 0) {  // token keys: longest walk first (see rev_order)
        if ((int)blockIdx.x >= n_kb) return;
        kb = a.order[blockIdx.x];
    } else {
        kb = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);  // (see bwd_dq_kernel)
        if (kb >= n_kb) return;
    }
    const int split = MODE == 1 ? blockIdx.z : 0;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, hh = lane >> 5;
    const uint32_t lane16 = (uint32_t)lane * 16u;
    const uint32_t tr_off = tr_lane_offset(lane), row_off = row_lane_offset(lane);
    const int64_t key0 = (int64_t)kb * 64 + 32 * wave;  // token index (MODE 0) or pooled-key index (MODE 1)
    const int64_t key = key0 + r;
    const int64_t limit = MODE != 1 ? a.n : (int64_t)a.nbc;
    const int half_w = a.window / 2;
    // MODE 0 with per-block counts: a padding slot is nobody's key (its probabilities are zeroed) and gets a zero gradient
    const int n_act = MODE != 1 && a.count != nullptr ? a.count[kb] : 64;
    const bool key_active = MODE == 1 || 32 * wave + r < n_act;

    bf16x8 kB[NS], vB[NS];
    {
        const int64_t krow_i = key < limit ? key : limit - 1;  // (rows past the end are masked below)
        const uint16_t *krow = (MODE != 1 ? a.k : a.kc) + (krow_i * a.h_kv + head) * D + 8 * hh;
        const uint16_t *vrow = (MODE != 1 ? a.v : a.vc) + (krow_i * a.h_kv + head) * D + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < NS; ++ks) {
            kB[ks] = *reinterpret_cast<const bf16x8 *>(krow + 16 * ks);
            vB[ks] = *reinterpret_cast<const bf16x8 *>(vrow + 16 * ks);
            if (!key_active) {  // a padding slot reads as zeros, whatever the caller left there
                const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
                kB[ks] = vB[ks] = zero8;
            }
        }
    }
    f32x16 acck[ND], accv[ND];
#pragma unroll
    for (int dt = 0; dt < ND; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acck[dt][i] = accv[dt][i] = 0.f;

    // ---- the query tiles that attend these keys
    int tw = 0, wt0 = 0, ts = 0, e0 = 0, T;
    if (MODE == 1) {
        wt0 = split * a.tiles_per_split;
        T = max(0, min(a.nt, wt0 + a.tiles_per_split) - wt0);
    } else {
        const int k0 = kb * 64;
        int seg_lo = 0, seg_hi = 0;
        if (a.blk_seg != nullptr) {  // the key's spatial block
            seg_lo = a.blk_seg[2 * kb];
            seg_hi = a.blk_seg[2 * kb + 1];
        } else {
            for (int s = 0; s < a.n_seg; ++s)
                if (k0 >= a.seg[s] && k0 < a.seg[s + 1]) {
                    seg_lo = a.seg[s];
                    seg_hi = a.seg[s + 1];
                }
        }
        if (a.own_block) {
            seg_lo = k0;
            seg_hi = k0 + 64;
        }
        // query i sees key j iff -W/2 <= j - i < W/2, i.e. j - W/2 < i <= j + W/2
        const int i_lo = max(seg_lo, k0 - half_w + 1), i_hi = min(seg_hi, k0 + 63 + half_w + 1);
        wt0 = i_lo / 32;
        tw = (half_w > 0 && i_hi > i_lo) ? (i_hi - 1) / 32 + 1 - wt0 : 0;
        e0 = a.rev_ptr[kb];
        ts = 2 * (a.rev_ptr[kb + 1] - e0);
        T = tw + ts;
    }
    // The walk is cut into segments with one pipelined loop each: the window tiles, then the routed tiles 64
    // reverse-list entries at a time (one entry per lane, loaded before the loop).  Inside a loop nothing is loaded
    // into registers from global memory: the wait for such a load would also wait for every tile copy in flight.
    // the query heads of the group this workgroup walks: all of them, or (token keys, heads dealt to hsplit
    // workgroups) its share
    const int gh0 = MODE == 0 && a.hsplit > 1 ? (int)blockIdx.z * a.hpw : 0;
    const int grp = MODE == 0 && a.hsplit > 1 ? min(a.group, gh0 + a.hpw) - gh0 : a.group;
    constexpr bool VGPR_CHAINS = D == 128;  // (the kernel has one wavefront per SIMD: see mfma_v)
    // the step in its interleaved form (step_interleaved below).  Not at d = 64: there it needs more than the 168
    // registers of three wavefronts per SIMD, and with two it measured slower (config 5: 1.12 -> 1.25 ms).
    constexpr bool INTERLEAVE = D != 64;
    constexpr int NB = kBwdDkvNbuf;  // tile buffers: the copies run NB - 1 steps ahead of the arithmetic
    constexpr int IPW = G::ROW / 1024;    // copy instructions per wavefront and step (wavefront 0: one more, the table)
    static_assert(NB == 2 || NB == 3, "");
    // br_c: the branch whose probabilities these are (0 compressed, 1 selected, 2 window); tile_fn(t): the t-th query
    // tile of the segment (arithmetic on registers only); every tile is met by the grp query heads of this key/value
    // head in turn
    auto run_segment = [&](int n_t, auto br_c, auto tile_fn) {
        constexpr int BR = decltype(br_c)::value;
        const int U = n_t * grp;
        if (U <= 0) return;
        const char *img_do = a.img_do[BR];
        const float *aux_br = a.aux + (int64_t)BR * a.nt * a.h * 64;  // table of this branch: [tile][head][64]
        auto issue = [&](int t, int gh, char *buf) {
            // (tile, head) index in 32 bits, byte offsets by shifts: a 64-bit multiply is several scalar instructions
            const uint32_t ih = (uint32_t)tile_fn(t) * (uint32_t)a.h + (uint32_t)(head * a.group + gh0 + gh);
            const int64_t off = (int64_t)ih * G::IMG;
            copy_kb<G::ROW / 1024>(a.img_q + off, buf, wave, lane16);
            copy_kb<G::ROW / 1024>(img_do + off, buf + G::ROW, wave, lane16);
            if (wave == 0)
                __builtin_amdgcn_global_load_lds(GLB_PTR(aux_br + (int64_t)ih * 64 + lane), LDS_PTR(buf + AUX), 4, 0, 0);
        };
        int t = 0, gh = 0, t_nxt = 0, gh_nxt = 0;  // the step being computed, the step being copied
        auto advance = [&](int &tt, int &gg) {     // (counters instead of a division per step)
            if (++gg == grp) {
                gg = 0;
                ++tt;
            }
        };
        // ---- the pieces of a step (one 32-query tile against this wavefront's 32 keys)
        struct Tile {
            const char *buf;  // its buffer: Q rows | dO rows | table
            int q0;           // first query of the tile
            bool win;         // a window tile at the band's edge: positions outside the band are masked
            f32x16 s, dp;
            float p[16];
        };
        // S = Q K^T
        auto ph_scores = [&](Tile &x, const char *buf, int tile) {
            x.buf = buf;
            x.q0 = 32 * tile;
            // window tiles away from the band's edges (and all routed tiles) need no mask
            x.win = BR == 2 && ((int)key0 - (x.q0 + 31) < -half_w || (int)key0 + 31 - x.q0 >= half_w);
            const char *base = buf + row_off;
            if constexpr (VGPR_CHAINS) {
                mfma_v_first(x.s, *reinterpret_cast<const bf16x8 *>(base), kB[0]);
#pragma unroll
                for (int ks = 1; ks < NS; ++ks) mfma_v(x.s, *reinterpret_cast<const bf16x8 *>(base + ks * 1024), kB[ks]);
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) x.s[i] = 0.f;
#pragma unroll
                for (int ks = 0; ks < NS; ++ks)
                    x.s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8 *>(base + ks * 1024),
                                                                  kB[ks], x.s, 0, 0, 0);
            }
        };
        // dP - D = dout V^T - D: the accumulator starts from -D of the 16 query rows this lane holds (second half
        // of the table, rows (i/4)*8 + hh*4 + i%4)
        auto ph_dp = [&](Tile &x) {
            const char *base = x.buf + row_off;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 y = *reinterpret_cast<const f32x4 *>(x.buf + AUX + 128 + (8 * g + 4 * hh) * 4);
#pragma unroll
                for (int j = 0; j < 4; ++j) x.dp[4 * g + j] = y[j];
            }
#pragma unroll
            for (int ks = 0; ks < NS; ++ks) {
                const bf16x8 rows = *reinterpret_cast<const bf16x8 *>(base + G::ROW + ks * 1024);
                if constexpr (VGPR_CHAINS)
                    mfma_v(x.dp, rows, vB[ks]);
                else
                    x.dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rows, vB[ks], x.dp, 0, 0, 0);
            }
        };
        // P = exp2(S scale log2e - offset), the offsets of the query rows from the first half of the table
        // (read right before their use: fewer registers live at once)
        auto ph_exp = [&](Tile &x) {
            float lv[16];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 y = *reinterpret_cast<const f32x4 *>(x.buf + AUX + (8 * g + 4 * hh) * 4);
#pragma unroll
                for (int j = 0; j < 4; ++j) lv[4 * g + j] = y[j];
            }
            // Most tiles need no mask at all (wave-uniform test): routed tiles and window tiles inside the band, of
            // blocks without padding; pooled keys before the last block.
            const bool plain = MODE == 1 ? key0 + 32 <= limit : (!x.win && n_act == 64);
            if constexpr (VGPR_CHAINS) mfma_v_settle(x.s);
            if (__builtin_expect(plain, 1)) {
#pragma unroll
                for (int i = 0; i < 16; ++i) x.p[i] = __builtin_amdgcn_exp2f(x.s[i] * a.sl2 - lv[i]);
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float pi = __builtin_amdgcn_exp2f(x.s[i] * a.sl2 - lv[i]);
                    bool ok;
                    if (MODE == 1) {
                        ok = key < limit;
                    } else {
                        const int qi = x.q0 + (i % 8) + 8 * hh + 16 * (i / 8);  // the query behind accumulator row i
                        const int dj = (int)key - qi;
                        ok = key_active & (!x.win | ((dj >= -half_w) & (dj < half_w)));
                    }
                    x.p[i] = ok ? pi : 0.f;
                }
            }
        };
        // dV^T += dout^T P
        auto ph_dv = [&](Tile &x) {
            BFrag pb[2];
            to_b_operand(x.p, pb);
            mfma_tr<ND>(accv, x.buf + G::ROW, tr_off, pb);
        };
        // dS = P o (dP - D), dK^T += Q^T dS
        auto ph_dk = [&](Tile &x) {
            if constexpr (VGPR_CHAINS) mfma_v_settle(x.dp);
            float ds[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) ds[i] = x.p[i] * x.dp[i];
            BFrag dsb[2];
            to_b_operand(ds, dsb);
            mfma_tr<ND>(acck, x.buf, tr_off, dsb);
        };

        // The interleaved form of a step (INTERLEAVE).  A wavefront issues in order, and this kernel has one wavefront
        // per SIMD at d = 128: whatever is to overlap -- vector arithmetic with MFMAs, LDS latency with either -- has to
        // alternate in the program.  Scheduling barriers fix the order of the pieces:
        //   reads of the Q rows | S#0, reads of the dout rows and of the table | S#1.. | (all reads have arrived)
        //   dP#k, each followed by its share of the exponentials (unmasked; edge tiles are fixed up afterwards) and by
        //     the transposing loads of one dout^T fragment
        //   dV#i (dout^T P), each followed by its share of dS = P o (dP - D) and by the loads of one Q^T fragment
        //   dK#i (Q^T dS)
        // The transposing loads are untracked (see tr_issue): their waits are counted by hand.  Fragment i of dout^T
        // is needed at dV#i, by when fragments i+1.. of dout^T and 0..i-1 of Q^T (two loads each) have been issued
        // behind it: at most 14 younger loads whatever i is; Q^T fragment i at dK#i has the 7-i later ones behind it.
        // The tracked reads (row fragments, table) are all waited for before the first untracked load is issued, so
        // the compiler's own counted waits never meet loads it does not know of.
        auto step_interleaved = [&](const char *buf, int tile, auto issue_next) {
            static_assert(!INTERLEAVE || 16 % NS == 0, "");
            const int q0 = 32 * tile;
            const bool win = BR == 2 && ((int)key0 - (q0 + 31) < -half_w || (int)key0 + 31 - q0 >= half_w);
            const bool plain = MODE == 1 ? key0 + 32 <= limit : (!win && n_act == 64);
            const char *base = buf + row_off;
            const uint32_t tr_q = (uint32_t)(uintptr_t)buf + tr_off, tr_do = tr_q + G::ROW;
            f32x16 sc, dp;
            float lv[16], pr[16];
            bf16x8 qr[NS], rows[NS];
#pragma unroll
            for (int ks = 0; ks < NS; ++ks) qr[ks] = *reinterpret_cast<const bf16x8 *>(base + ks * 1024);
            __builtin_amdgcn_sched_barrier(0);
            issue_next();  // the copies of the next step's tile: their address arithmetic runs while the reads land
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (VGPR_CHAINS) {
                mfma_v_first(sc, qr[0], kB[0]);
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) sc[i] = 0.f;
                sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qr[0], kB[0], sc, 0, 0, 0);
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 y = *reinterpret_cast<const f32x4 *>(buf + AUX + 128 + (8 * g + 4 * hh) * 4);
                const f32x4 z = *reinterpret_cast<const f32x4 *>(buf + AUX + (8 * g + 4 * hh) * 4);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    dp[4 * g + j] = y[j];
                    lv[4 * g + j] = z[j];
                }
            }
#pragma unroll
            for (int ks = 0; ks < NS; ++ks) rows[ks] = *reinterpret_cast<const bf16x8 *>(base + G::ROW + ks * 1024);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = 1; ks < NS; ++ks) {
                if constexpr (VGPR_CHAINS)
                    mfma_v(sc, qr[ks], kB[ks]);
                else
                    sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qr[ks], kB[ks], sc, 0, 0, 0);
            }
            // every tracked read has arrived (the empty statements make the compiler wait for them here)
#pragma unroll
            for (int ks = 0; ks < NS; ++ks) asm volatile("" : "+v"(rows[ks]));
#pragma unroll
            for (int i = 0; i < 16; ++i) asm volatile("" : "+v"(lv[i]));
            asm volatile("" : "+v"(dp));
            if constexpr (VGPR_CHAINS) mfma_v_settle(sc);
            __builtin_amdgcn_sched_barrier(0);

            TrFrag fdo[2 * ND], fq[2 * ND];
            BFrag pb[2], dsb[2];
            // dP chain with the exponentials; dout^T fragments requested on the way (fragment f after MFMA f * NS / 2ND)
            constexpr int E = 16 / NS;
            auto issue_do = [&](auto ic) {
                constexpr int I = decltype(ic)::value;
                tr_issue<(I % ND) * 2048 + (I / ND) * 256>(fdo[I], tr_do);
            };
            auto issue_q = [&](auto ic) {
                constexpr int I = decltype(ic)::value;
                tr_issue<(I % ND) * 2048 + (I / ND) * 256>(fq[I], tr_q);
            };
            auto dp_step = [&](auto kc) {
                constexpr int ks = decltype(kc)::value;
                if constexpr (VGPR_CHAINS)
                    mfma_v(dp, rows[ks], vB[ks]);
                else
                    dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rows[ks], vB[ks], dp, 0, 0, 0);
#pragma unroll
                for (int e = ks * E; e < (ks + 1) * E; ++e) {
                    pr[e] = __builtin_amdgcn_exp2f(sc[e] * a.sl2 - lv[e]);
                    if (e & 1) {
                        pb[e / 8].u[(e / 2) % 4] = pack_bf16(pr[e - 1], pr[e]);
                        asm volatile("" : "+v"(pb[e / 8].u[(e / 2) % 4]));
                    }
                    asm volatile("" : "+v"(pr[e]));
                }
                // NS MFMAs, 2 ND fragments: one fragment behind every (NS / 2ND)-th MFMA (NS = 2 ND * (NS / 2ND))
                if constexpr (ks % (NS / (2 * ND)) == 0) issue_do(std::integral_constant<int, ks / (NS / (2 * ND))>{});
                __builtin_amdgcn_sched_barrier(0);
            };
            for_each_index<NS>(dp_step);
            if constexpr (VGPR_CHAINS) mfma_v_settle(dp);
            if (__builtin_expect(!plain, 0)) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    bool ok;
                    if (MODE == 1) {
                        ok = key < limit;
                    } else {
                        const int qi = q0 + (i % 8) + 8 * hh + 16 * (i / 8);  // the query behind accumulator row i
                        const int dj = (int)key - qi;
                        ok = key_active & (!win | ((dj >= -half_w) & (dj < half_w)));
                    }
                    pr[i] = ok ? pr[i] : 0.f;
                }
                to_b_operand(pr, pb);
            }
            __builtin_amdgcn_sched_barrier(0);
            // dV with dS; Q^T fragments requested on the way
            constexpr int EV = 16 / (2 * ND);
            auto dv_step = [&](auto ic) {
                constexpr int I = decltype(ic)::value;
                // younger loads behind dout^T fragment I: its 2 ND - 1 - I successors and the I fragments of Q^T
                accv[I % ND] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_take<2 * (2 * ND - 1)>(fdo[I]), pb[I / ND].v,
                                                                       accv[I % ND], 0, 0, 0);
#pragma unroll
                for (int e = I * EV; e < (I + 1) * EV; e += 2) {
                    const float d0 = pr[e] * dp[e], d1 = pr[e + 1] * dp[e + 1];
                    dsb[e / 8].u[(e / 2) % 4] = pack_bf16(d0, d1);
                    asm volatile("" : "+v"(dsb[e / 8].u[(e / 2) % 4]));
                }
                issue_q(ic);
                __builtin_amdgcn_sched_barrier(0);
            };
            for_each_index<2 * ND>(dv_step);
            auto dk_step = [&](auto ic) {
                constexpr int I = decltype(ic)::value;
                acck[I % ND] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_take<2 * (2 * ND - 1 - I)>(fq[I]), dsb[I / ND].v,
                                                                       acck[I % ND], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            };
            for_each_index<2 * ND>(dk_step);
        };

        __builtin_amdgcn_s_waitcnt(vm_lgkm_imm(0));
        __syncthreads();  // both wavefronts are done with the buffers (previous segment)
        for (int i = 0; i < NB - 1 && i < U; ++i) {
            issue(t_nxt, gh_nxt, lds + i * TILE);
            advance(t_nxt, gh_nxt);
        }
        for (int u = 0, slot = 0; u < U; ++u, advance(t, gh), slot = slot + 1 == NB ? 0 : slot + 1) {
            // The barrier alone does not wait for copies in flight (they are counted by vmcnt, which a
            // workgroup-scope fence leaves alone): every wavefront first waits for its own share of the
            // step's tile -- the copies of the next step may stay in flight -- then the barrier publishes
            // all shares; it also tells that everyone is done with the buffer refilled next.
            if (NB == 3 && u + 1 < U) {
                if (wave == 0)
                    __builtin_amdgcn_s_waitcnt(vm_lgkm_imm(IPW + 1));
                else
                    __builtin_amdgcn_s_waitcnt(vm_lgkm_imm(IPW));
            } else {
                __builtin_amdgcn_s_waitcnt(vm_lgkm_imm(0));
            }
            wg_barrier();
            auto issue_next = [&]() {
                if (u + NB - 1 < U) {
                    const int fill = slot == 0 ? NB - 1 : slot - 1;  // the buffer of step u - 1 = that of step u + NB - 1
                    issue(t_nxt, gh_nxt, lds + fill * TILE);
                    advance(t_nxt, gh_nxt);
                }
            };
            if constexpr (INTERLEAVE) {
                step_interleaved(lds + slot * TILE, tile_fn(t), issue_next);
            } else {
                // (the plain order: scores, exponentials, dV, dP, dK; at d = 64 the interleaved one does not fit the
                // registers of three wavefronts per SIMD)
                issue_next();
                Tile x;
                ph_scores(x, lds + slot * TILE, tile_fn(t));
                ph_exp(x);
                ph_dv(x);
                ph_dp(x);
                ph_dk(x);
            }
        }
    };
    if (MODE == 1) {
        run_segment(T, std::integral_constant<int, 0>{}, [&](int t) { return wt0 + t; });
    } else if (MODE == 0) {
        run_segment(tw, std::integral_constant<int, 2>{}, [&](int t) { return wt0 + t; });
        const int n_e = ts >> 1;  // entries of the reverse list: query blocks that route to this key block
        for (int c0 = 0; c0 < n_e; c0 += 64) {
            const int rev_held = c0 + lane < n_e ? a.rev_idx[e0 + c0 + lane] : 0;
            run_segment(2 * min(64, n_e - c0), std::integral_constant<int, 1>{}, [&](int t) {
                return 2 * __builtin_amdgcn_readlane(rev_held, t >> 1) + (t & 1);
            });
        }
    }

    if (MODE == 0 && a.hsplit > 1) {
        // the sums over this workgroup's heads: [head range][key][head][channel] fp32; the last pass finishes the rows
        const int64_t o = ((((int64_t)blockIdx.z * a.nb * 64) + key) * a.h_kv + head) * D;
#pragma unroll
        for (int dt = 0; dt < ND; ++dt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 xk, xv;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    xk[j] = acck[dt][4 * g + j];
                    xv[j] = accv[dt][4 * g + j];
                }
                *reinterpret_cast<f32x4 *>(a.hpart_k + o + 32 * dt + 8 * g + 4 * hh) = xk;
                *reinterpret_cast<f32x4 *>(a.hpart_v + o + 32 * dt + 8 * g + 4 * hh) = xv;
            }
        return;
    }
    if (MODE == 2) {
        // last pass: the sums of the head ranges, added in order
        for (int z = 0; z < a.hsplit; ++z) {
            const int64_t o = ((((int64_t)z * a.nb * 64) + key) * a.h_kv + head) * D;
#pragma unroll
            for (int dt = 0; dt < ND; ++dt)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 xk = *reinterpret_cast<const f32x4 *>(a.hpart_k + o + 32 * dt + 8 * g + 4 * hh);
                    const f32x4 xv = *reinterpret_cast<const f32x4 *>(a.hpart_v + o + 32 * dt + 8 * g + 4 * hh);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        acck[dt][4 * g + j] += xk[j];
                        accv[dt][4 * g + j] += xv[j];
                    }
                }
        }
    }
    if (MODE == 1) {
        // partial sums of this query range: [split][pooled key][head][channel] fp32
        const int64_t o = (((int64_t)split * a.nbp + key) * a.h_kv + head) * D;
#pragma unroll
        for (int dt = 0; dt < ND; ++dt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 xk, xv;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    xk[j] = acck[dt][4 * g + j];
                    xv[j] = accv[dt][4 * g + j];
                }
                *reinterpret_cast<f32x4 *>(a.part_k + o + 32 * dt + 8 * g + 4 * hh) = xk;
                *reinterpret_cast<f32x4 *>(a.part_v + o + 32 * dt + 8 * g + 4 * hh) = xv;
            }
    } else {
        // add the gradient of the pooled key / value this block went into (its query ranges in order), divided by
        // the number of tokens that pair averaged: the block's, or its whole spatial block's
        const int pair = a.blk_grp != nullptr ? a.blk_grp[kb] : kb;
        const float pooled_tokens = a.grp_tok != nullptr ? (float)a.grp_tok[pair] : (float)n_act;
        float xk[ND][16], xv[ND][16];
#pragma unroll
        for (int dt = 0; dt < ND; ++dt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 pk = {0.f, 0.f, 0.f, 0.f}, pv = {0.f, 0.f, 0.f, 0.f};
                for (int sp = 0; sp < a.n_split; ++sp) {
                    const int64_t o = (((int64_t)sp * a.nbp + pair) * a.h_kv + head) * D + 32 * dt + 8 * g + 4 * hh;
                    pk += *reinterpret_cast<const f32x4 *>(a.part_k + o);
                    pv += *reinterpret_cast<const f32x4 *>(a.part_v + o);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    // the block average was taken over its n_act active tokens; a padding slot gets nothing
                    const float inv_cnt = key_active ? 1.0f / pooled_tokens : 0.f;
                    xk[dt][4 * g + j] = (acck[dt][4 * g + j] + pk[j] * inv_cnt) * a.scale;
                    xv[dt][4 * g + j] = accv[dt][4 * g + j] + pv[j] * inv_cnt;
                }
            }
        __syncthreads();  // the tile buffers become the output staging
        char *stage = lds + wave * 32 * G::OUT_ROW;
        store_rows_transposed<D>(xk, stage, a.dk + (key0 * a.h_kv + head) * D, (int64_t)a.h_kv * D, lane);
        __builtin_amdgcn_s_waitcnt(0xC07F);  // staging reads of dK done before it is overwritten
        store_rows_transposed<D>(xv, stage, a.dv + (key0 * a.h_kv + head) * D, (int64_t)a.h_kv * D, lane);
    }
}

struct WsLayout {
    size_t img_q, img_do[3], gdo, img_k, img_v, img_kc, img_vc, aux, part_k, part_v, rev_cnt, rev_ptr, rev_cur, rev_idx, total;
    int n_split, nbp, tiles_per_split, hsplit, hpw;
    size_t hpart_k, hpart_v, order, gtab;
};

WsLayout ws_layout(const Shape &s) {
    WsLayout w;
    const size_t img = (size_t)s.d * 64;  // bytes of one (tile, head) image: row-order fragments only
    const size_t nt = (size_t)s.nb * 2, ntc = (size_t)(s.nbc + 31) / 32;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off += align_up(bytes > 0 ? bytes : 1, 256);
        return at;
    };
    w.img_q = take(nt * s.h * img);
    w.img_do[0] = take(nt * s.h * img);
    if (s.gate_channels) {
        // one image of gate o dout per branch, and the rows they are packed from
        w.img_do[1] = take(nt * s.h * img);
        w.img_do[2] = take(nt * s.h * img);
        w.gdo = take((size_t)3 * s.n * s.h * s.d * 2);
    } else {
        w.img_do[1] = w.img_do[2] = w.img_do[0];
        w.gdo = 0;
    }
    w.img_k = take(nt * s.h_kv * img);
    w.img_v = take(nt * s.h_kv * img);
    w.img_kc = take(ntc * s.h_kv * img);
    w.img_vc = take(ntc * s.h_kv * img);
    w.aux = take((size_t)3 * nt * s.h * 64 * 4);
    // pooled keys: enough query ranges to fill the chip
    w.nbp = (s.nbc + 63) / 64 * 64;
    const int wgs = (w.nbp / 64) * s.h_kv;
    // The query tiles are cut into n ranges, one workgroup per (64 pooled keys, key/value head, range), all equally
    // long.  The chip runs `slots` of them at a time (256 CUs x the workgroups per CU that the kernel's registers
    // allow), so the kernel takes ceil(workgroups / slots) rounds of (tiles per range) x (query heads per key/value
    // head) steps; every range also costs its partial sums, written here and read back by the token-key kernel.
    // n minimises that: e.g. at 1680 workgroups per range and 512 slots, two ranges run 7 rounds where 6.6 would
    // do, seven ranges run 23 rounds of a seventh the length (6 % less).
    {
        const int slots = 256 * (s.d == 128 ? 2 : s.d == 64 ? 6 : 8);
        const int grp_q = s.h / s.h_kv;
        const double range_bytes = (double)w.nbp * s.h_kv * s.d * 4 * 2 * 2;
        const double step_seconds = 1.1e-6 * s.d / 128, range_steps = range_bytes / 4e12 / step_seconds;
        double best = 0;
        int best_n = 1;
        for (int n = 1; n <= 64; ++n) {
            const int64_t tiles = ((int64_t)nt + n - 1) / n;
            if (tiles <= 0) break;
            const int64_t n_eff = ((int64_t)nt + tiles - 1) / tiles;
            const int64_t rounds = ((int64_t)wgs * n_eff + slots - 1) / slots;
            const double cost = (double)rounds * tiles * grp_q + range_steps * n_eff;
            if (n == 1 || cost < best) {
                best = cost;
                best_n = n;
            }
        }
        (void)kBwdSplitTarget;
        const int n_split = best_n;
        w.tiles_per_split = (int)((nt + n_split - 1) / n_split);
        w.n_split = (int)((nt + w.tiles_per_split - 1) / (w.tiles_per_split > 0 ? w.tiles_per_split : 1));
        if (w.n_split < 1) w.n_split = 1;
    }
    w.part_k = take((size_t)w.n_split * w.nbp * s.h_kv * s.d * 4);
    w.part_v = take((size_t)w.n_split * w.nbp * s.h_kv * s.d * 4);
    // token keys: with grouped-query heads a workgroup would walk group x as many steps while there are group x
    // fewer workgroups, and the longest reverse list sets the kernel's time -- deal the heads of a group to
    // up to 8 workgroups
    // (as long as their fp32 sums stay within 2 GiB of workspace)
    const int grp = s.h / s.h_kv;
    const size_t per_range = (size_t)s.nb * 64 * s.h_kv * s.d * 4 * 2;
    const size_t fit = per_range > 0 ? ((size_t)2 << 30) / per_range : 8;
    const int ranges = (int)(fit < 8 ? (fit < 1 ? 1 : fit) : 8);
    w.hpw = (grp + ranges - 1) / ranges;
    w.hsplit = (grp + w.hpw - 1) / w.hpw;
    w.hpart_k = w.hpart_v = 0;
    if (w.hsplit > 1) {
        w.hpart_k = take((size_t)w.hsplit * s.nb * 64 * s.h_kv * s.d * 4);
        w.hpart_v = take((size_t)w.hsplit * s.nb * 64 * s.h_kv * s.d * 4);
    }
    w.rev_cnt = take((size_t)s.nb * 4);
    w.order = take((size_t)s.nb * 4);
    w.rev_ptr = take((size_t)(s.nb + 1) * 4);
    w.rev_cur = take((size_t)s.nb * 4);
    w.rev_idx = take((size_t)s.nb * (s.topk > 0 ? s.topk : 1) * 4);
    w.gtab = take(group_tables_bytes(s));
    w.total = off;
    return w;
}

template <int D>
lsrm_status launch_backward_d(const Shape &s, BwdArgs a, const WsLayout &w, char *ws, hipStream_t st, hipEvent_t ev_start,
                              hipEvent_t ev_stop) {
    using G = BGeo<D>;
    constexpr int DKV_LDS = kBwdDkvNbuf * (2 * G::ROW + 1024);
    // (set on every call: cheap, and right whichever device is current and whichever thread calls)
    LSRM_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(&bwd_dkv_kernel<D, 0>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, DKV_LDS));
    LSRM_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(&bwd_dkv_kernel<D, 1>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, DKV_LDS));
    LSRM_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(&bwd_dkv_kernel<D, 2>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, DKV_LDS));
    if (ev_start != nullptr) LSRM_HIP_CHECK(hipEventRecord(ev_start, st));
    const int ntc = (s.nbc + 31) / 32;
    lsrm_status rc;
    hipLaunchKernelGGL(bwd_prep<D>, dim3((unsigned)(a.nt * ((s.h + PrepGeo<D>::HB - 1) / PrepGeo<D>::HB))),
                       dim3(PrepGeo<D>::THREADS), 0, st, a);
    LSRM_HIP_CHECK(hipGetLastError());
    if ((rc = launch_pack_tiles(D, a.q, a.q, ws + w.img_q, s.n, s.h, a.nt, st, true, a.count)) != LSRM_OK) return rc;
    if (s.gate_channels) {
        for (int b = 0; b < 3; ++b) {
            const uint16_t *src = a.gdo + (size_t)b * s.n * s.h * D;
            if ((rc = launch_pack_tiles(D, src, src, ws + w.img_do[b], s.n, s.h, a.nt, st, true, a.count)) != LSRM_OK) return rc;
        }
    } else {
        if ((rc = launch_pack_tiles(D, a.dout, a.dout, ws + w.img_do[0], s.n, s.h, a.nt, st, true, a.count)) != LSRM_OK) return rc;
    }
    if ((rc = launch_pack_tiles(D, a.k, a.k, ws + w.img_k, s.n, s.h_kv, a.nt, st, true, a.count)) != LSRM_OK) return rc;
    if ((rc = launch_pack_tiles(D, a.v, a.v, ws + w.img_v, s.n, s.h_kv, a.nt, st, true, a.count)) != LSRM_OK) return rc;
    if ((rc = launch_pack_tiles(D, a.kc, a.kc, ws + w.img_kc, (int64_t)s.nbc, s.h_kv, ntc, st, true, nullptr)) != LSRM_OK) return rc;
    if ((rc = launch_pack_tiles(D, a.vc, a.vc, ws + w.img_vc, (int64_t)s.nbc, s.h_kv, ntc, st, true, nullptr)) != LSRM_OK) return rc;
    // reverse routing lists
    hipLaunchKernelGGL(fill_zero, dim3((s.nb + 255) / 256), dim3(256), 0, st, a.rev_cnt, s.nb);
    LSRM_HIP_CHECK(hipGetLastError());
    if (s.topk > 0) {
        hipLaunchKernelGGL(rev_count, dim3((s.nb * s.topk + 255) / 256), dim3(256), 0, st, a);
        LSRM_HIP_CHECK(hipGetLastError());
    }
    hipLaunchKernelGGL(rev_scan, dim3(1), dim3(1024), 0, st, a);
    LSRM_HIP_CHECK(hipGetLastError());
    hipLaunchKernelGGL(rev_order, dim3(1), dim3(1024), 0, st, a, const_cast<int32_t *>(a.order));
    LSRM_HIP_CHECK(hipGetLastError());
    if (s.topk > 0) {
        hipLaunchKernelGGL(rev_fill, dim3((s.nb * s.topk + 255) / 256), dim3(256), 0, st, a);
        LSRM_HIP_CHECK(hipGetLastError());
        const size_t bitmap = (size_t)((s.nb + 31) / 32) * 4;
        if (bitmap <= 48 * 1024)
            hipLaunchKernelGGL(rev_sort, dim3(s.nb), dim3(64), bitmap, st, a);
        else
            hipLaunchKernelGGL(rev_sort_serial, dim3((s.nb + 63) / 64), dim3(64), 0, st, a);
        LSRM_HIP_CHECK(hipGetLastError());
    }
    if (s.topk > 64)
        hipLaunchKernelGGL((bwd_dq_kernel<D, true>), dim3((s.nb + 7) / 8 * 8, s.h), dim3(128), 0, st, a);
    else
        hipLaunchKernelGGL((bwd_dq_kernel<D, false>), dim3((s.nb + 7) / 8 * 8, s.h), dim3(128), 0, st, a);
    LSRM_HIP_CHECK(hipGetLastError());
    hipLaunchKernelGGL((bwd_dkv_kernel<D, 1>), dim3((w.nbp / 64 + 7) / 8 * 8, s.h_kv, w.n_split), dim3(128), DKV_LDS, st,
                       a);
    LSRM_HIP_CHECK(hipGetLastError());
    if (w.n_split > 1) {
        const int64_t per_split = (int64_t)w.nbp * s.h_kv * D;
        hipLaunchKernelGGL(sum_parts, dim3((unsigned)((per_split / 4 + 255) / 256)), dim3(256), 0, st, a.part_k, a.part_v,
                           w.n_split, per_split);
        LSRM_HIP_CHECK(hipGetLastError());
        a.n_split = 1;  // (the kernels below read range 0's slot only)
    }
    hipLaunchKernelGGL((bwd_dkv_kernel<D, 0>), dim3((s.nb + 7) / 8 * 8, s.h_kv, a.hsplit), dim3(128), DKV_LDS, st, a);
    LSRM_HIP_CHECK(hipGetLastError());
    if (a.hsplit > 1) {  // add up the per-head-range sums, in order, and finish the rows
        hipLaunchKernelGGL((bwd_dkv_kernel<D, 2>), dim3((s.nb + 7) / 8 * 8, s.h_kv), dim3(128), DKV_LDS, st, a);
        LSRM_HIP_CHECK(hipGetLastError());
    }
    if (ev_stop != nullptr) LSRM_HIP_CHECK(hipEventRecord(ev_stop, st));
    return LSRM_OK;
}

}  // namespace

size_t backward_ws_bytes(const Shape &s) { return ws_layout(s).total; }

lsrm_status launch_backward(const Shape &s, const int32_t *seg_host, int n_seg, const uint16_t *d_q,
                            const uint16_t *d_k, const uint16_t *d_v, const uint16_t *d_kc, const uint16_t *d_vc,
                            const int32_t *d_idx, const float *d_gates, const float *d_lse,
                            const uint16_t *d_out_branch, const uint16_t *d_dout, uint16_t *d_dq, uint16_t *d_dk,
                            uint16_t *d_dv, void *d_ws, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
    if (s.nb == 0) return LSRM_OK;
    if (n_seg > kMaxSeg) return LSRM_ERR_UNSUPPORTED;
    const WsLayout w = ws_layout(s);
    char *ws = reinterpret_cast<char *>(d_ws);
    BwdArgs a{};
    a.q = d_q;
    a.k = d_k;
    a.v = d_v;
    a.kc = d_kc;
    a.vc = d_vc;
    a.dout = d_dout;
    a.out_branch = d_out_branch;
    a.idx = d_idx;
    a.gates = d_gates;
    a.lse = d_lse;
    a.img_q = ws + w.img_q;
    for (int b = 0; b < 3; ++b) a.img_do[b] = ws + w.img_do[b];
    a.gdo = s.gate_channels ? reinterpret_cast<const uint16_t *>(ws + w.gdo) : nullptr;
    a.img_k = ws + w.img_k;
    a.img_v = ws + w.img_v;
    a.img_kc = ws + w.img_kc;
    a.img_vc = ws + w.img_vc;
    a.aux = reinterpret_cast<float *>(ws + w.aux);
    a.part_k = reinterpret_cast<float *>(ws + w.part_k);
    a.part_v = reinterpret_cast<float *>(ws + w.part_v);
    a.rev_cnt = reinterpret_cast<int32_t *>(ws + w.rev_cnt);
    a.rev_ptr = reinterpret_cast<int32_t *>(ws + w.rev_ptr);
    a.rev_cur = reinterpret_cast<int32_t *>(ws + w.rev_cur);
    a.rev_idx = reinterpret_cast<int32_t *>(ws + w.rev_idx);
    a.dq = d_dq;
    a.dk = d_dk;
    a.dv = d_dv;
    for (int i = 0; i <= n_seg; ++i) a.seg[i] = seg_host[i];
    a.n = s.n;
    a.nb = s.nb;
    a.nbc = s.nbc;
    a.blk_grp = a.blk_seg = a.grp_tok = nullptr;
    if (s.ng > 0) {
        GroupTables gt;
        lsrm_status rc = launch_group_tables(s, reinterpret_cast<int32_t *>(ws + w.gtab), &gt, st);
        if (rc != LSRM_OK) return rc;
        a.blk_grp = gt.blk_grp;
        a.grp_tok = gt.grp_tok;
        if (s.group_window) a.blk_seg = gt.blk_seg;
    }
    a.h = s.h;
    a.h_kv = s.h_kv;
    a.group = s.h / s.h_kv;
    a.gate_channels = s.gate_channels;
    a.count = s.count;
    a.topk = s.topk;
    a.window = s.window;
    a.own_block = s.own_block;
    a.n_seg = n_seg;
    a.nt = s.nb * 2;
    a.n_split = w.n_split;
    a.hsplit = w.hsplit;
    a.hpw = w.hpw;
    a.hpart_k = reinterpret_cast<float *>(ws + w.hpart_k);
    a.hpart_v = reinterpret_cast<float *>(ws + w.hpart_v);
    a.order = reinterpret_cast<const int32_t *>(ws + w.order);
    a.nbp = w.nbp;
    a.tiles_per_split = w.tiles_per_split;
    a.scale = s.scale;
    a.sl2 = s.scale * kLog2e;
    if (s.d == 32) return launch_backward_d<32>(s, a, w, ws, st, ev_start, ev_stop);
    if (s.d == 64) return launch_backward_d<64>(s, a, w, ws, st, ev_start, ev_stop);
    return launch_backward_d<128>(s, a, w, ws, st, ev_start, ev_stop);
}

}  // namespace lsrm
