// Simulated network for single-GPU runs: what one destination rank receives from a
// sender's packed buffer.  Paper hook: Section 4.1 workflow step 4 -- a payload is
// delivered only to nodes named in its bitmap; bitmaps travel unchanged.
// Not part of the dispatch path proper; used to build peer receive regions.
#include "mw_internal.h"

namespace {

constexpr int kBlock = 1024;

// One workgroup: keep the groups naming dst_rank, rebase their row offsets, and record
// for every kept row which sender row it is.
__global__ __launch_bounds__(kBlock) void k_deliver_index(const mw_group_desc *__restrict__ desc,
                                                          const mw_send_stats *__restrict__ stats, int dst_rank,
                                                          uint32_t cap, mw_group_desc *__restrict__ desc_out,
                                                          int32_t *__restrict__ row_map,
                                                          uint32_t *__restrict__ counts)
{
    __shared__ uint32_t scratch[17];
    const uint32_t G = min(stats->n_groups, cap), tid = threadIdx.x;
    const uint32_t per = (G + kBlock - 1) / kBlock;
    const uint32_t g0 = min(tid * per, G), g1 = min(g0 + per, G);
    uint32_t kg = 0, kr = 0;
    for (uint32_t g = g0; g < g1; ++g)
        if ((desc[g].mask[dst_rank >> 6] >> (dst_rank & 63)) & 1ull) { ++kg; kr += desc[g].row_count; }
    uint32_t tg, tr;
    uint32_t og = mw_block_exscan(kg, scratch, &tg);
    uint32_t orow = mw_block_exscan(kr, scratch, &tr);
    for (uint32_t g = g0; g < g1; ++g) {
        mw_group_desc d = desc[g];
        if (!((d.mask[dst_rank >> 6] >> (dst_rank & 63)) & 1ull)) continue;
        for (uint32_t i = 0; i < d.row_count; ++i)
            if (orow + i < cap) row_map[orow + i] = (int32_t)(d.row_offset + i);
        d.row_offset = orow;
        desc_out[og++] = d;
        orow += d.row_count;
    }
    if (tid == 0) { counts[0] = tg; counts[1] = min(tr, cap); }
}

template <int U>
__global__ __launch_bounds__(256) void k_deliver_copy(const u32x4 *__restrict__ rows, int n_chunks, int ns,
                                                      const int32_t *__restrict__ src_token,
                                                      const int32_t *__restrict__ topk, int K,
                                                      const int32_t *__restrict__ row_map,
                                                      const uint32_t *__restrict__ counts,
                                                      u32x4 *__restrict__ rows_out,
                                                      int32_t *__restrict__ src_token_out,
                                                      int32_t *__restrict__ topk_out)
{
    const uint32_t i = blockIdx.x;
    if (i >= counts[1]) return;
    const int32_t r = row_map[i];
    const u32x4 *src = rows + (size_t)r * ns;          // ns: chunks from one row to the next, both sides
    u32x4 *dst = rows_out + (size_t)i * ns;
    for (int c0 = threadIdx.x; c0 < n_chunks; c0 += U * 256) {
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) if (c0 + u * 256 < n_chunks) v[u] = mw_ld16(src + c0 + u * 256);
#pragma unroll
        for (int u = 0; u < U; ++u) if (c0 + u * 256 < n_chunks) mw_st16(dst + c0 + u * 256, v[u]);
    }
    if (threadIdx.x == 0) src_token_out[i] = src_token[r];
    for (int j = threadIdx.x; j < K; j += 256) topk_out[(size_t)i * K + j] = topk[(size_t)r * K + j];
}

}  // namespace

int32_t mw_launch_sim_deliver(mw_ctx *ctx, const mw_group_desc *desc, const mw_send_stats *stats,
                              int32_t T, const void *rows, const int32_t *src_token, const int32_t *topk,
                              int32_t dst_rank, mw_group_desc *desc_out, void *rows_out,
                              int32_t *src_token_out, int32_t *topk_out, uint32_t *counts, hipStream_t s)
{
    hipLaunchKernelGGL(k_deliver_index, dim3(1), dim3(kBlock), 0, s, desc, stats, dst_rank, (uint32_t)T, desc_out,
                       ctx->d_row_map, counts);
    if (T > 0) {
        hipLaunchKernelGGL(k_deliver_copy<4>, dim3(T), dim3(256), 0, s, (const u32x4 *)rows,
                           (int)(ctx->row_bytes / 16), (int)(ctx->row_stride / 16), src_token, topk, ctx->cfg.top_k, ctx->d_row_map, counts,
                           (u32x4 *)rows_out, src_token_out, topk_out);
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}
