// Block compression (Sec. 3.2 "Block Partitioning and Compression"; App. A "Compressed"):
// one key/value pair per 64-token block, the in-block average.
//
// HBM-streaming kernel: every element of K and V is read exactly once (4 N h d bytes)
// and 1/64 of that is written.  One thread owns 8 consecutive channels (one 16-byte
// load per token row), consecutive threads own consecutive channels, so each row of a
// block is read with fully coalesced 16-byte accesses; the 64 rows are independent
// loads kept in flight by unrolling.  fp32 accumulation in token order, one rounding
// to bf16 at the end.
#include "lsrm_internal.h"

namespace lsrm {

namespace {

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float x) {
    uint32_t u = __float_as_uint(x);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// grid: (ceil(NB * row_chunks / 256), 2)   y = 0 -> K, y = 1 -> V
// count (nullable): block b averages its first count[b] rows only (1..64).
__global__ __launch_bounds__(256) void pool_blocks(int nb, int row_chunks /* h*d/8 */, const uint4 *__restrict__ k,
                                                   const uint4 *__restrict__ v, uint4 *__restrict__ kc,
                                                   uint4 *__restrict__ vc, const int32_t *__restrict__ count) {
    const size_t g = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t b = g / row_chunks;
    const int c = (int)(g % row_chunks);
    if (b >= (size_t)nb) return;
    const uint4 *src = (blockIdx.y == 0 ? k : v) + b * kBlock * (size_t)row_chunks + c;
    uint4 *dst = (blockIdx.y == 0 ? kc : vc) + b * (size_t)row_chunks + c;
    const int n_act = count != nullptr ? count[b] : kBlock;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
    for (int t0 = 0; t0 < kBlock; t0 += 16) {
        uint4 r[16];
#pragma unroll
        for (int t = 0; t < 16; ++t)
            r[t] = t0 + t < n_act ? src[(size_t)(t0 + t) * row_chunks] : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            acc[0] += bf16_lo(r[t].x); acc[1] += bf16_hi(r[t].x);
            acc[2] += bf16_lo(r[t].y); acc[3] += bf16_hi(r[t].y);
            acc[4] += bf16_lo(r[t].z); acc[5] += bf16_hi(r[t].z);
            acc[6] += bf16_lo(r[t].w); acc[7] += bf16_hi(r[t].w);
        }
    }
    const float den = (float)n_act;  // 64: the division is exact, as a multiplication by 1/64 would be
    uint4 o;
    o.x = f32_to_bf16_rne(acc[0] / den) | (f32_to_bf16_rne(acc[1] / den) << 16);
    o.y = f32_to_bf16_rne(acc[2] / den) | (f32_to_bf16_rne(acc[3] / den) << 16);
    o.z = f32_to_bf16_rne(acc[4] / den) | (f32_to_bf16_rne(acc[5] / den) << 16);
    o.w = f32_to_bf16_rne(acc[6] / den) | (f32_to_bf16_rne(acc[7] / den) << 16);
    *dst = o;
}

// Spatial blocks of several 64-slot blocks (Sec. 3.2: volume blocks of up to 512 active tokens): one pair per
// group, the mean over the active tokens of all its blocks.  One thread per (group, 8-channel chunk), rows in token
// order.  grid: (ceil(ng * row_chunks / 256), 2).
__global__ __launch_bounds__(256) void pool_groups(int ng, int row_chunks, const uint4 *__restrict__ k,
                                                   const uint4 *__restrict__ v, uint4 *__restrict__ kc,
                                                   uint4 *__restrict__ vc, const int32_t *__restrict__ count,
                                                   const int32_t *__restrict__ goff) {
    const size_t g = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t grp = g / row_chunks;
    const int c = (int)(g % row_chunks);
    if (grp >= (size_t)ng) return;
    const uint4 *src_all = (blockIdx.y == 0 ? k : v) + c;
    uint4 *dst = (blockIdx.y == 0 ? kc : vc) + grp * (size_t)row_chunks + c;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    int tokens = 0;
    for (int b = goff[grp]; b < goff[grp + 1]; ++b) {
        const int n_act = count != nullptr ? count[b] : kBlock;
        const uint4 *src = src_all + (size_t)b * kBlock * (size_t)row_chunks;
        for (int t = 0; t < n_act; ++t) {
            const uint4 r = src[(size_t)t * row_chunks];
            acc[0] += bf16_lo(r.x); acc[1] += bf16_hi(r.x);
            acc[2] += bf16_lo(r.y); acc[3] += bf16_hi(r.y);
            acc[4] += bf16_lo(r.z); acc[5] += bf16_hi(r.z);
            acc[6] += bf16_lo(r.w); acc[7] += bf16_hi(r.w);
        }
        tokens += n_act;
    }
    const float den = (float)(tokens > 0 ? tokens : 1);
    uint4 o;
    o.x = f32_to_bf16_rne(acc[0] / den) | (f32_to_bf16_rne(acc[1] / den) << 16);
    o.y = f32_to_bf16_rne(acc[2] / den) | (f32_to_bf16_rne(acc[3] / den) << 16);
    o.z = f32_to_bf16_rne(acc[4] / den) | (f32_to_bf16_rne(acc[5] / den) << 16);
    o.w = f32_to_bf16_rne(acc[6] / den) | (f32_to_bf16_rne(acc[7] / den) << 16);
    *dst = o;
}

__global__ __launch_bounds__(256) void fill_int(int32_t *p, size_t n, int32_t v) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// One thread per group: the tables the attention kernels look blocks up in (see GroupTables).
__global__ __launch_bounds__(256) void group_tables(int ng, int nb, const int32_t *__restrict__ goff,
                                                    const int32_t *__restrict__ count, int32_t *__restrict__ blk_grp,
                                                    int32_t *__restrict__ blk_seg, int32_t *__restrict__ grp_tok) {
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= ng) return;
    int b0 = goff[g], b1 = goff[g + 1];
    b0 = b0 < 0 ? 0 : (b0 > nb ? nb : b0);  // (never write outside the tables, whatever the offsets hold)
    b1 = b1 < b0 ? b0 : (b1 > nb ? nb : b1);
    int tokens = 0;
    for (int b = b0; b < b1; ++b) {
        blk_grp[b] = g;
        blk_seg[2 * b] = b0 * kBlock;
        blk_seg[2 * b + 1] = b1 * kBlock;
        tokens += count != nullptr ? count[b] : kBlock;
    }
    grp_tok[g] = tokens > 0 ? tokens : 1;
}

}  // namespace

lsrm_status launch_group_tables(const Shape &s, int32_t *tab, GroupTables *out, hipStream_t st) {
    out->blk_grp = out->blk_seg = out->grp_tok = nullptr;
    if (s.ng <= 0) return LSRM_OK;
    int32_t *blk_grp = tab, *blk_seg = tab + s.nb, *grp_tok = tab + 3 * (size_t)s.nb;
    // blocks that no group covers (offsets that do not reach N / 64) keep defined entries: a group of their own
    // (an empty window); a fill kernel rather than a memset, which callers that capture the stream cannot replay
    const size_t n_tab = (size_t)3 * s.nb + s.ng;
    hipLaunchKernelGGL(fill_int, dim3((unsigned)((n_tab + 255) / 256)), dim3(256), 0, st, tab, n_tab, 0);
    LSRM_HIP_CHECK(hipGetLastError());
    hipLaunchKernelGGL(group_tables, dim3((s.ng + 255) / 256), dim3(256), 0, st, s.ng, s.nb, s.goff, s.count, blk_grp,
                       blk_seg, grp_tok);
    LSRM_HIP_CHECK(hipGetLastError());
    out->blk_grp = blk_grp;
    out->blk_seg = blk_seg;
    out->grp_tok = grp_tok;
    return LSRM_OK;
}

lsrm_status launch_compress(const Shape &s, const uint16_t *d_k, const uint16_t *d_v, uint16_t *d_kc,
                            uint16_t *d_vc, hipStream_t st) {
    if (s.nb == 0) return LSRM_OK;
    int row_chunks = s.h_kv * s.d / 8;
    if (s.ng > 0) {
        dim3 grid_g((unsigned)(((size_t)s.ng * row_chunks + 255) / 256), 2);
        hipLaunchKernelGGL(pool_groups, grid_g, dim3(256), 0, st, s.ng, row_chunks, reinterpret_cast<const uint4 *>(d_k),
                           reinterpret_cast<const uint4 *>(d_v), reinterpret_cast<uint4 *>(d_kc),
                           reinterpret_cast<uint4 *>(d_vc), s.count, s.goff);
        LSRM_HIP_CHECK(hipGetLastError());
        return LSRM_OK;
    }
    dim3 grid((unsigned)(((size_t)s.nb * row_chunks + 255) / 256), 2);
    hipLaunchKernelGGL(pool_blocks, grid, dim3(256), 0, st, s.nb, row_chunks, reinterpret_cast<const uint4 *>(d_k),
                       reinterpret_cast<const uint4 *>(d_v), reinterpret_cast<uint4 *>(d_kc),
                       reinterpret_cast<uint4 *>(d_vc), s.count);
    LSRM_HIP_CHECK(hipGetLastError());
    return LSRM_OK;
}

}  // namespace lsrm
