// Payload packer and plain copies (send side bulk movers).
//
// Paper hooks: Section 1 -- only one copy of the same data is injected, so a token's row
// is written once however many ranks its bitmap names; Section 5.2 step 1 -- data is
// loaded into the pre-allocated send buffer; Section 4.3.4 (statelessness) -- the row's
// source token index and top-k ids travel with it.
//
// The packer is a row gather bound by HBM bandwidth: packed[i] = x[perm[i]].  Rows are
// multiples of 16 bytes; a group of `tpr` lanes owns one row and keeps U 16-byte loads in
// flight per lane before the first store.  Nothing is reused, so loads and stores are
// streaming (non-temporal).
#include "mw_internal.h"

namespace {

// Copy one row of (xc + sc) 16-byte chunks: chunks [0, xc) come from src_x, the rest
// from src_s (the fp8 scale tail; sc == 0 otherwise).
template <int U>
__device__ __forceinline__ void copy_row(const u32x4 *__restrict__ src_x, const u32x4 *__restrict__ src_s,
                                         int xc, int sc, u32x4 *__restrict__ dst, int lane, int tpr)
{
    const int n = xc + sc;
    for (int c0 = lane; c0 < n; c0 += U * tpr) {
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + u * tpr;
            if (c < n) v[u] = (c < xc) ? mw_ld16(src_x + c) : mw_ld16(src_s + (c - xc));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + u * tpr;
            if (c < n) mw_st16(dst + c, v[u]);
        }
    }
}

template <int U>
__global__ __launch_bounds__(256) void k_pack(const u32x4 *__restrict__ x, const u32x4 *__restrict__ scales,
                                              int xc, int sc, const int32_t *__restrict__ topk, int K,
                                              const int32_t *__restrict__ perm,
                                              const mw_send_stats *__restrict__ stats, int tpr,
                                              u32x4 *__restrict__ packed, int32_t *__restrict__ row_src_token,
                                              int32_t *__restrict__ row_topk)
{
    const int rows_per_block = blockDim.x / tpr;
    const int sub = threadIdx.x / tpr, lane = threadIdx.x - sub * tpr;
    const uint32_t i = blockIdx.x * rows_per_block + sub;
    if (sub >= rows_per_block || i >= stats->n_rows) return;
    const int32_t t = perm[i];
    copy_row<U>(x + (size_t)t * xc, scales + (size_t)t * sc, xc, sc, packed + (size_t)i * (xc + sc), lane, tpr);
    if (lane == 0) row_src_token[i] = t;
    for (int j = lane; j < K; j += tpr) row_topk[(size_t)i * K + j] = topk[(size_t)t * K + j];
}

// Flat streaming copy: a workgroup moves one contiguous tile of 256 * U chunks.
template <int U>
__global__ __launch_bounds__(256) void k_copy(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst,
                                              int64_t n_chunks)
{
    const int64_t base = (int64_t)blockIdx.x * (256 * U) + threadIdx.x;
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t c = base + u * 256;
        if (c < n_chunks) v[u] = mw_ld16(src + c);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t c = base + u * 256;
        if (c < n_chunks) mw_st16(dst + c, v[u]);
    }
}

// AllGather receive assembly: shard p goes to out + p * shard_bytes.  blockIdx.y = p.
template <int U>
__global__ __launch_bounds__(256) void k_gather_shards(const u32x4 *const *__restrict__ shards,
                                                       int64_t shard_chunks, u32x4 *__restrict__ out)
{
    const u32x4 *src = shards[blockIdx.y];
    u32x4 *dst = out + (int64_t)blockIdx.y * shard_chunks;
    const int64_t base = (int64_t)blockIdx.x * (256 * U) + threadIdx.x;
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t c = base + u * 256;
        if (c < shard_chunks) v[u] = mw_ld16(src + c);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t c = base + u * 256;
        if (c < shard_chunks) mw_st16(dst + c, v[u]);
    }
}

constexpr int kCopyU = 4;

}  // namespace

// Lanes per row: enough that U chunks per lane cover the row in one pass when possible.
static int lanes_per_row(int chunks, int U)
{
    int tpr = 64;
    while (tpr < 256 && tpr * U < chunks) tpr *= 2;
    return tpr;
}

int32_t mw_launch_pack(mw_ctx *ctx, const void *x, const float *scales, const int32_t *topk,
                       const int32_t *perm, const mw_send_stats *stats, int32_t T, void *packed,
                       int32_t *row_src_token, int32_t *row_topk, hipStream_t s)
{
    if (T == 0) return MW_OK;
    const int xc = (int)(ctx->x_row_bytes / 16), sc = (int)(ctx->s_row_bytes / 16);
    constexpr int U = 4;
    const int tpr = lanes_per_row(xc + sc, U);
    const int rows_per_block = 256 / tpr;
    const int grid = (T + rows_per_block - 1) / rows_per_block;
    hipLaunchKernelGGL(k_pack<U>, dim3(grid), dim3(256), 0, s, (const u32x4 *)x, (const u32x4 *)scales, xc, sc,
                       topk, ctx->cfg.top_k, perm, stats, tpr, (u32x4 *)packed, row_src_token, row_topk);
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

int32_t mw_launch_copy(void *dst, const void *src, int64_t n_bytes, hipStream_t s)
{
    const int64_t n_chunks = n_bytes / 16;
    if (n_chunks == 0) return MW_OK;
    const int64_t grid = (n_chunks + 256 * kCopyU - 1) / (256 * kCopyU);
    if (grid > 0x7fffffffLL) return MW_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(k_copy<kCopyU>, dim3((uint32_t)grid), dim3(256), 0, s, (const u32x4 *)src, (u32x4 *)dst,
                       n_chunks);
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

int32_t mw_launch_gather_shards(mw_ctx *ctx, const void *const *shards, int64_t shard_bytes, void *out,
                                hipStream_t s)
{
    const int64_t shard_chunks = shard_bytes / 16;
    if (shard_chunks == 0) return MW_OK;
    const int64_t gx = (shard_chunks + 256 * kCopyU - 1) / (256 * kCopyU);
    if (gx > 0x7fffffffLL) return MW_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(k_gather_shards<kCopyU>, dim3((uint32_t)gx, ctx->cfg.n_ranks), dim3(256), 0, s,
                       (const u32x4 *const *)shards, shard_chunks, (u32x4 *)out);
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}
