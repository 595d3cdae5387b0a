// C ABI of the MultiWrite library: context, argument validation, dispatch to the
// kernel launchers.  The contract of every entry point is in include/mw.h.
#include <new>
#include <vector>

#include "mw_internal.h"

namespace {

// A context's workspace lives on the device that was current when it was created; work for
// it enqueued with another device current would run there on foreign pointers.
#define MW_ON_DEVICE(ctx)                                               \
    do {                                                                \
        int mw_dev_now_ = -1;                                           \
        if (hipGetDevice(&mw_dev_now_) != hipSuccess) return MW_ERR_HIP; \
        if (mw_dev_now_ != (ctx)->device) return MW_ERR_INVALID_ARG;    \
    } while (0)

struct ws_layout {
    int64_t eslot, plan_cnt, plan_state, flags, cnt, base, row_base, addr_cnt, recs, hits, row_map,
        hop_bits, group_of_row, child_pos, sort_key, sort_sec, chunk_kept, row_cnt, row_start, total;
};

}  // namespace

// Derived row geometry; returns a status.
int32_t mw_row_geometry(const mw_config &c, int64_t *x_bytes, int64_t *s_bytes)
{
    switch (c.row_format) {
    case MW_ROW_BF16:
        if (c.hidden < 1) return MW_ERR_INVALID_ARG;
        *x_bytes = 2LL * c.hidden; *s_bytes = 0;
        break;
    case MW_ROW_FP8_E4M3_BLOCK128:
        if (c.hidden < 1) return MW_ERR_INVALID_ARG;
        if (c.hidden % 512 != 0) return MW_ERR_UNSUPPORTED;   // codes and scales both 16-byte multiples
        *x_bytes = c.hidden; *s_bytes = 4LL * (c.hidden / 128);
        break;
    case MW_ROW_BYTES:
        if (c.row_bytes < 16) return MW_ERR_INVALID_ARG;
        *x_bytes = c.row_bytes; *s_bytes = 0;
        break;
    default:
        return MW_ERR_INVALID_ARG;
    }
    const int64_t rb = *x_bytes + *s_bytes;
    if (rb % 16 != 0 || *x_bytes % 16 != 0) return MW_ERR_UNSUPPORTED;
    if (rb / 16 > 0x7fffffffLL) return MW_ERR_UNSUPPORTED;
    if (c.row_format != MW_ROW_BYTES && c.row_bytes != 0 && c.row_bytes != rb) return MW_ERR_INVALID_ARG;
    if (c.row_stride_bytes != 0) {
        if (c.row_stride_bytes < rb) return MW_ERR_INVALID_ARG;
        if (c.row_stride_bytes % 16 != 0 || c.row_stride_bytes / 16 > 0x7fffffffLL) return MW_ERR_UNSUPPORTED;
    }
    return MW_OK;
}

namespace {

int32_t validate(const mw_config *c, int32_t *n_local)
{
    if (!c) return MW_ERR_INVALID_ARG;
    if (c->n_ranks < 1 || c->n_experts < 0 || c->top_k < 1 || c->max_tokens < 0 || c->max_recv_rows < 0)
        return MW_ERR_INVALID_ARG;
    if (c->n_ranks > MW_MAX_RANKS || c->top_k > MW_MAX_TOPK) return MW_ERR_UNSUPPORTED;
    if (c->max_tokens > 65536 || c->n_experts > 65536) return MW_ERR_UNSUPPORTED;
    if (c->my_rank < 0 || c->my_rank >= c->n_ranks) return MW_ERR_INVALID_ARG;
    if (c->n_experts > 0 && !c->expert_to_rank) return MW_ERR_INVALID_ARG;
    if (c->max_recv_rows > (int64_t)c->n_ranks * 65536) return MW_ERR_UNSUPPORTED;
    if (c->max_hops < 0) return MW_ERR_INVALID_ARG;
    if (c->max_hops > MW_MAX_HOPS) return MW_ERR_UNSUPPORTED;
    int32_t L = 0;
    for (int32_t e = 0; e < c->n_experts; ++e) {
        if (c->expert_to_rank[e] < 0 || c->expert_to_rank[e] >= c->n_ranks) return MW_ERR_INVALID_ARG;
        L += (c->expert_to_rank[e] == c->my_rank);
    }
    if ((int64_t)L * c->n_ranks > (1 << 22)) return MW_ERR_UNSUPPORTED;   // (expert, peer) count table
    *n_local = L;
    return MW_OK;
}

ws_layout layout(const mw_config &c, int32_t L)
{
    const int64_t A = 256;
    const int64_t Kd = (c.top_k < L ? c.top_k : L) > 0 ? (c.top_k < L ? c.top_k : L) : 1;
    ws_layout w;
    int64_t o = 0;
    const int64_t ntok = c.max_tokens > 0 ? c.max_tokens : 1;
    w.eslot = o;      o += mw_align_up(4LL * (c.n_experts > 0 ? c.n_experts : 1), A);
    w.plan_cnt = o;   o += mw_align_up(8LL * ntok, A);
    w.plan_state = o; o += mw_align_up(4LL * MW_PLAN_STATE_WORDS, A);
    w.flags = o;      o += A;
    w.cnt = o;        o += mw_align_up(4LL * ((int64_t)L * c.n_ranks > 0 ? (int64_t)L * c.n_ranks : 1), A);
    w.base = o;       o += mw_align_up(4LL * ((int64_t)L * c.n_ranks > 0 ? (int64_t)L * c.n_ranks : 1), A);
    w.row_base = o;   o += mw_align_up(4LL * (c.n_ranks + 1), A);
    w.addr_cnt = o;   o += mw_align_up(4LL * c.n_ranks, A);
    w.recs = o;       o += mw_align_up((int64_t)sizeof(mw_row_rec) * (c.max_recv_rows > 0 ? c.max_recv_rows : 1), A);
    w.hits = o;       o += mw_align_up((int64_t)sizeof(mw_hit) * Kd * (c.max_recv_rows > 0 ? c.max_recv_rows : 1), A);
    w.row_map = o;    o += mw_align_up(4LL * (c.max_tokens > 0 ? c.max_tokens : 1), A);
    w.hop_bits = w.group_of_row = w.child_pos = o;
    if (c.max_hops > 0) {
        w.hop_bits = o;     o += mw_align_up(8LL * MW_MASK_WORDS * MW_MAX_HOPS + 256, A);   // + relay flags
        w.group_of_row = o; o += mw_align_up(4LL * ntok, A);
        w.child_pos = o;    o += mw_align_up(4LL * MW_MAX_HOPS * ntok, A);
    }
    // sorted chunks for the plan of large batches (only contexts that can see such batches)
    w.sort_key = w.sort_sec = w.chunk_kept = w.row_cnt = w.row_start = -1;
    if (c.max_tokens > 4096) {
        const int64_t padded = mw_align_up(ntok, 1024);
        w.sort_key = o;   o += mw_align_up(8LL * padded, A);
        w.sort_sec = o;   o += mw_align_up(4LL * padded, A);
        w.chunk_kept = o; o += mw_align_up(4LL * 64, A);
        w.row_cnt = o;    o += mw_align_up(8LL * padded, A);
        w.row_start = o;  o += mw_align_up(padded, A);
    }
    w.total = o;
    return w;
}

}  // namespace

extern "C" {

MW_API int32_t mw_workspace_bytes(const mw_config *cfg, int64_t *out_bytes)
{
    int32_t L = 0;
    if (!out_bytes) return MW_ERR_INVALID_ARG;
    int32_t rc = validate(cfg, &L);
    if (rc != MW_OK) return rc;
    int64_t xb, sb;
    rc = mw_row_geometry(*cfg, &xb, &sb);
    if (rc != MW_OK) return rc;
    *out_bytes = layout(*cfg, L).total;
    return MW_OK;
}

MW_API int32_t mw_ctx_create(const mw_config *cfg, void *workspace_dev, int64_t workspace_bytes, mw_ctx **out)
{
    if (!out) return MW_ERR_INVALID_ARG;
    *out = nullptr;
    int32_t L = 0;
    int32_t rc = validate(cfg, &L);
    if (rc != MW_OK) return rc;
    int64_t xb = 0, sb = 0;
    rc = mw_row_geometry(*cfg, &xb, &sb);
    if (rc != MW_OK) return rc;
    const ws_layout w = layout(*cfg, L);
    if (!workspace_dev || ((uintptr_t)workspace_dev & 255u) || workspace_bytes < w.total) return MW_ERR_WORKSPACE;

    mw_ctx *ctx = new (std::nothrow) mw_ctx();
    if (!ctx) return MW_ERR_INVALID_ARG;
    ctx->cfg = *cfg;
    ctx->cfg.expert_to_rank = nullptr;     // the host table is not kept
    ctx->cfg.row_bytes = xb + sb;
    ctx->n_local = L;
    ctx->hit_slots = (cfg->top_k < L ? cfg->top_k : L) > 0 ? (cfg->top_k < L ? cfg->top_k : L) : 1;
    ctx->mask_words = (cfg->n_ranks + 63) / 64;
    ctx->x_row_bytes = xb; ctx->s_row_bytes = sb; ctx->row_bytes = xb + sb;
    ctx->row_stride = cfg->row_stride_bytes != 0 ? cfg->row_stride_bytes : xb + sb;
    char *b = (char *)workspace_dev;
    ctx->d_eslot = (int32_t *)(b + w.eslot);
    ctx->d_plan_cnt = (uint64_t *)(b + w.plan_cnt);
    ctx->d_plan_state = (uint32_t *)(b + w.plan_state);
    ctx->d_sort_key = w.sort_key >= 0 ? (uint64_t *)(b + w.sort_key) : nullptr;
    ctx->d_sort_sec = w.sort_sec >= 0 ? (uint32_t *)(b + w.sort_sec) : nullptr;
    ctx->d_chunk_kept = w.chunk_kept >= 0 ? (uint32_t *)(b + w.chunk_kept) : nullptr;
    ctx->d_row_cnt = w.row_cnt >= 0 ? (uint64_t *)(b + w.row_cnt) : nullptr;
    ctx->d_row_start = w.row_start >= 0 ? (unsigned char *)(b + w.row_start) : nullptr;
    ctx->d_flags = (uint32_t *)(b + w.flags);
    ctx->d_cnt = (uint32_t *)(b + w.cnt);
    ctx->d_base = (uint32_t *)(b + w.base);
    ctx->d_recs = (mw_row_rec *)(b + w.recs);
    ctx->d_row_base = (uint32_t *)(b + w.row_base);
    ctx->d_addr_cnt = (uint32_t *)(b + w.addr_cnt);
    ctx->d_hits = (mw_hit *)(b + w.hits);
    ctx->d_row_map = (int32_t *)(b + w.row_map);
    ctx->n_hops = 0;
    ctx->recv_rows_hint = 0;
    ctx->ride_wait_limit = 1u << 21;
    ctx->options = 0;
    ctx->d_hop_bits = (uint64_t *)(b + w.hop_bits);
    ctx->d_relay_flags = (uint32_t *)(b + w.hop_bits + 8LL * MW_MASK_WORDS * MW_MAX_HOPS);
    ctx->d_group_of_row = (int32_t *)(b + w.group_of_row);
    ctx->d_child_pos = (uint32_t *)(b + w.child_pos);

    hipDeviceProp_t prop;
    if (hipGetDevice(&ctx->device) != hipSuccess || hipGetDeviceProperties(&prop, ctx->device) != hipSuccess) {
        delete ctx; return MW_ERR_HIP;
    }
    ctx->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;

    // rank table and, per expert, its slot among the experts of its own rank
    std::vector<int32_t> slot((size_t)(cfg->n_experts > 0 ? cfg->n_experts : 1), 0);
    std::vector<int32_t> seen((size_t)cfg->n_ranks, 0);
    for (int32_t e = 0; e < cfg->n_experts; ++e) {
        const int32_t r = cfg->expert_to_rank[e];
        slot[e] = (r << 16) | seen[r]++;      // slots stay below 65536 because E does
    }
    bool ok = true;
    if (cfg->n_experts > 0)
        ok = ok && hipMemcpy(ctx->d_eslot, slot.data(), 4u * (size_t)cfg->n_experts, hipMemcpyHostToDevice) == hipSuccess;
    ok = ok && hipMemset(ctx->d_flags, 0, 256) == hipSuccess;
    ok = ok && hipMemset(ctx->d_plan_cnt, 0, 8u * (size_t)(cfg->max_tokens > 0 ? cfg->max_tokens : 1)) == hipSuccess;
    ok = ok && hipMemset(ctx->d_plan_state, 0, 4u * MW_PLAN_STATE_WORDS) == hipSuccess;
    if (cfg->max_hops > 0) ok = ok && hipMemset(ctx->d_relay_flags, 0, 256) == hipSuccess;
    ok = ok && hipDeviceSynchronize() == hipSuccess;
    if (!ok) { delete ctx; return MW_ERR_HIP; }
    *out = ctx;
    return MW_OK;
}

MW_API int32_t mw_ctx_destroy(mw_ctx *ctx)
{
    if (!ctx) return MW_ERR_INVALID_ARG;
    delete ctx;
    return MW_OK;
}

MW_API int32_t mw_plan(mw_ctx *ctx, const int32_t *topk_ids_dev, int32_t n_tokens, uint64_t *mask_dev,
                int32_t *perm_dev, mw_group_desc *desc_dev, mw_send_stats *stats_dev, void *stream)
{
    if (!ctx || !stats_dev || n_tokens < 0) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (n_tokens > ctx->cfg.max_tokens) return MW_ERR_CAPACITY;
    if (n_tokens > 0 && (!topk_ids_dev || !mask_dev || !perm_dev || !desc_dev)) return MW_ERR_INVALID_ARG;
    if (ctx->cfg.n_experts == 0) return MW_ERR_INVALID_ARG;
    return mw_launch_plan(ctx, topk_ids_dev, n_tokens, mask_dev, perm_dev, desc_dev, stats_dev, (hipStream_t)stream);
}

MW_API int32_t mw_pack(mw_ctx *ctx, const void *x_dev, const float *scales_dev, const int32_t *topk_ids_dev,
                const int32_t *perm_dev, const mw_send_stats *stats_dev, int32_t n_tokens,
                void *packed_rows_dev, int32_t *row_src_token_dev, int32_t *row_topk_dev, void *stream)
{
    if (!ctx || !stats_dev || n_tokens < 0) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (n_tokens > ctx->cfg.max_tokens) return MW_ERR_CAPACITY;
    if (n_tokens == 0) return MW_OK;
    if (!x_dev || !topk_ids_dev || !perm_dev || !packed_rows_dev || !row_src_token_dev || !row_topk_dev)
        return MW_ERR_INVALID_ARG;
    if ((ctx->s_row_bytes > 0) != (scales_dev != nullptr)) return MW_ERR_INVALID_ARG;
    if (((uintptr_t)x_dev | (uintptr_t)packed_rows_dev | (uintptr_t)scales_dev) & 15u) return MW_ERR_INVALID_ARG;
    return mw_launch_pack(ctx, x_dev, scales_dev, topk_ids_dev, perm_dev, stats_dev, n_tokens, packed_rows_dev,
                          row_src_token_dev, row_topk_dev, (hipStream_t)stream);
}

MW_API int32_t mw_pack_quantize(mw_ctx *ctx, const void *x_bf16_dev, const int32_t *topk_ids_dev,
                         const int32_t *perm_dev, const mw_send_stats *stats_dev, int32_t n_tokens,
                         void *packed_rows_dev, int32_t *row_src_token_dev, int32_t *row_topk_dev, void *stream)
{
    if (!ctx || !stats_dev || n_tokens < 0) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (ctx->cfg.row_format != MW_ROW_FP8_E4M3_BLOCK128) return MW_ERR_UNSUPPORTED;
    if (n_tokens > ctx->cfg.max_tokens) return MW_ERR_CAPACITY;
    if (n_tokens == 0) return MW_OK;
    if (!x_bf16_dev || !topk_ids_dev || !perm_dev || !packed_rows_dev || !row_src_token_dev || !row_topk_dev)
        return MW_ERR_INVALID_ARG;
    if (((uintptr_t)x_bf16_dev | (uintptr_t)packed_rows_dev) & 15u) return MW_ERR_INVALID_ARG;
    return mw_launch_pack_quantize(ctx, x_bf16_dev, topk_ids_dev, perm_dev, stats_dev, n_tokens, packed_rows_dev,
                                   row_src_token_dev, row_topk_dev, (hipStream_t)stream);
}

MW_API int32_t mw_plan_pack(mw_ctx *ctx, const int32_t *topk_ids_dev, const void *x_dev, const float *scales_dev,
                     int32_t n_tokens, uint64_t *mask_dev, int32_t *perm_dev, mw_group_desc *desc_dev,
                     mw_send_stats *stats_dev, void *packed_rows_dev, int32_t *row_src_token_dev,
                     int32_t *row_topk_dev, void *stream)
{
    if (!ctx || !stats_dev || n_tokens < 0) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (n_tokens > ctx->cfg.max_tokens || n_tokens > MW_FUSED_MAX_TOKENS) return MW_ERR_CAPACITY;
    if (ctx->cfg.n_experts == 0) return MW_ERR_INVALID_ARG;
    if (n_tokens > 0) {
        if (!topk_ids_dev || !mask_dev || !perm_dev || !desc_dev || !x_dev || !packed_rows_dev || !row_src_token_dev ||
            !row_topk_dev)
            return MW_ERR_INVALID_ARG;
        if ((ctx->s_row_bytes > 0) != (scales_dev != nullptr)) return MW_ERR_INVALID_ARG;
        if (((uintptr_t)x_dev | (uintptr_t)packed_rows_dev | (uintptr_t)scales_dev) & 15u) return MW_ERR_INVALID_ARG;
    }
    return mw_launch_plan_pack(ctx, topk_ids_dev, n_tokens, x_dev, scales_dev, mask_dev, perm_dev, desc_dev, stats_dev,
                               packed_rows_dev, row_src_token_dev, row_topk_dev, (hipStream_t)stream);
}

MW_API int32_t mw_plan_allgather(mw_ctx *ctx, int64_t shard_bytes, mw_group_desc *desc_dev, mw_send_stats *stats_dev,
                          void *stream)
{
    if (!ctx || !desc_dev || !stats_dev || shard_bytes < 0) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    return mw_launch_plan_allgather(ctx, shard_bytes, desc_dev, stats_dev, (hipStream_t)stream);
}

MW_API int32_t mw_pack_allgather(mw_ctx *ctx, const void *shard_dev, int64_t shard_bytes, void *send_buf_dev,
                          void *stream)
{
    if (!ctx || shard_bytes < 0) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (shard_bytes % 16 != 0) return MW_ERR_UNSUPPORTED;
    if (shard_bytes == 0) return MW_OK;
    if (!shard_dev || !send_buf_dev || (((uintptr_t)shard_dev | (uintptr_t)send_buf_dev) & 15u))
        return MW_ERR_INVALID_ARG;
    return mw_launch_copy(ctx, send_buf_dev, shard_dev, shard_bytes, (hipStream_t)stream);
}

MW_API int32_t mw_allgather_split_point(int64_t shard_bytes, double bw_direct, double bw_relay, int32_t copies,
                                 int64_t *direct_bytes)
{
    if (!direct_bytes || shard_bytes < 0 || copies < 1 || !(bw_direct > 0.0) || !(bw_relay > 0.0))
        return MW_ERR_INVALID_ARG;
    if (shard_bytes % 16 != 0) return MW_ERR_UNSUPPORTED;
    const double f = (double)copies * bw_direct / (bw_relay + (double)copies * bw_direct);
    int64_t a = (int64_t)(f * (double)shard_bytes);
    a -= a % 16;
    if (a < 0) a = 0;
    if (a > shard_bytes) a = shard_bytes;
    *direct_bytes = a;
    return MW_OK;
}

MW_API int32_t mw_plan_allgather_split(mw_ctx *ctx, int64_t shard_bytes, int64_t direct_bytes,
                                mw_group_desc *desc_dev, mw_send_stats *stats_dev, void *stream)
{
    if (!ctx || !desc_dev || !stats_dev || shard_bytes < 0 || direct_bytes < 0 || direct_bytes > shard_bytes)
        return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (shard_bytes % 16 != 0 || direct_bytes % 16 != 0 || shard_bytes / 16 > 0xffffffffLL) return MW_ERR_UNSUPPORTED;
    return mw_launch_plan_allgather_split(ctx, shard_bytes, direct_bytes, desc_dev, stats_dev, (hipStream_t)stream);
}

MW_API int32_t mw_unpack_allgather_split(mw_ctx *ctx, const void *const *direct_dev, const void *const *relayed_dev,
                                  int64_t shard_bytes, int64_t direct_bytes, void *out_dev, void *stream)
{
    if (!ctx || shard_bytes < 0 || direct_bytes < 0 || direct_bytes > shard_bytes) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (shard_bytes % 16 != 0 || direct_bytes % 16 != 0) return MW_ERR_UNSUPPORTED;
    if (shard_bytes == 0) return MW_OK;
    if (!direct_dev || !relayed_dev || !out_dev || ((uintptr_t)out_dev & 15u)) return MW_ERR_INVALID_ARG;
    return mw_launch_gather_split(ctx, direct_dev, relayed_dev, shard_bytes, direct_bytes, out_dev,
                                  (hipStream_t)stream);
}

static int32_t check_unpack_index(mw_ctx *ctx, const void *peers_dev, int32_t n_peers,
                                  int64_t out_capacity_rows, int64_t *expert_offsets_dev, mw_recv_stats *recv_stats_dev)
{
    if (!ctx || !peers_dev || !expert_offsets_dev || !recv_stats_dev || out_capacity_rows < 0)
        return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (n_peers < 1 || n_peers > ctx->cfg.n_ranks) return MW_ERR_INVALID_ARG;
    if (ctx->cfg.n_experts == 0) return MW_ERR_INVALID_ARG;
    if (out_capacity_rows > 0xffffffffLL) return MW_ERR_UNSUPPORTED;
    return MW_OK;
}

static int32_t check_unpack_expand(mw_ctx *ctx, int32_t n_peers, void *out_rows_dev, float *out_scales_dev,
                                   int64_t out_capacity_rows, int32_t *out_src_peer_dev, int32_t *out_src_token_dev)
{
    if (!ctx || out_capacity_rows < 0) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (n_peers < 1 || n_peers > ctx->cfg.n_ranks) return MW_ERR_INVALID_ARG;
    if (ctx->cfg.n_experts == 0) return MW_ERR_INVALID_ARG;
    if (out_capacity_rows > 0 && (!out_rows_dev || !out_src_peer_dev || !out_src_token_dev))
        return MW_ERR_INVALID_ARG;
    if (out_capacity_rows > 0 && (ctx->s_row_bytes > 0) != (out_scales_dev != nullptr)) return MW_ERR_INVALID_ARG;
    if (out_capacity_rows > 0xffffffffLL) return MW_ERR_UNSUPPORTED;
    if (((uintptr_t)out_rows_dev | (uintptr_t)out_scales_dev) & 15u) return MW_ERR_INVALID_ARG;
    return MW_OK;
}

MW_API int32_t mw_unpack(mw_ctx *ctx, const mw_recv_peer *peers_dev, int32_t n_peers, void *out_rows_dev,
                  float *out_scales_dev, int64_t out_capacity_rows, int32_t *out_src_peer_dev,
                  int32_t *out_src_token_dev, int64_t *expert_offsets_dev, mw_recv_stats *recv_stats_dev,
                  void *stream)
{
    int32_t rc = check_unpack_index(ctx, peers_dev, n_peers, out_capacity_rows, expert_offsets_dev, recv_stats_dev);
    if (rc == MW_OK)
        rc = check_unpack_expand(ctx, n_peers, out_rows_dev, out_scales_dev, out_capacity_rows, out_src_peer_dev,
                                 out_src_token_dev);
    if (rc != MW_OK) return rc;
    rc = mw_launch_unpack_index(ctx, peers_dev, false, n_peers, out_capacity_rows, expert_offsets_dev, recv_stats_dev,
                                (hipStream_t)stream);
    if (rc != MW_OK) return rc;
    return mw_launch_unpack_expand(ctx, n_peers, out_rows_dev, out_scales_dev, out_capacity_rows, out_src_peer_dev,
                                   out_src_token_dev, (hipStream_t)stream);
}

MW_API int32_t mw_packet_header_bytes(int32_t top_k, int64_t *header_bytes)
{
    if (!header_bytes || top_k < 1 || top_k > MW_MAX_TOPK) return MW_ERR_INVALID_ARG;
    *header_bytes = mw_packet_header_bytes_of(top_k);
    return MW_OK;
}

MW_API int32_t mw_pack_packets(mw_ctx *ctx, const void *x_dev, const float *scales_dev, const int32_t *topk_ids_dev,
                        const uint64_t *mask_dev, const int32_t *perm_dev, const mw_send_stats *stats_dev,
                        int32_t n_tokens, void *packets_dev, void *stream)
{
    if (!ctx || !stats_dev || n_tokens < 0) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (n_tokens > ctx->cfg.max_tokens) return MW_ERR_CAPACITY;
    if (ctx->cfg.n_experts == 0) return MW_ERR_INVALID_ARG;
    if (n_tokens == 0) return MW_OK;
    if (!x_dev || !topk_ids_dev || !mask_dev || !perm_dev || !packets_dev) return MW_ERR_INVALID_ARG;
    if ((ctx->s_row_bytes > 0) != (scales_dev != nullptr)) return MW_ERR_INVALID_ARG;
    if (((uintptr_t)x_dev | (uintptr_t)packets_dev | (uintptr_t)scales_dev) & 15u) return MW_ERR_INVALID_ARG;
    return mw_launch_pack_packets(ctx, x_dev, scales_dev, topk_ids_dev, mask_dev, perm_dev, stats_dev, n_tokens,
                                  packets_dev, (hipStream_t)stream);
}

MW_API int32_t mw_unpack_packets(mw_ctx *ctx, const mw_recv_packets *peers_dev, int32_t n_peers, void *out_rows_dev,
                          float *out_scales_dev, int64_t out_capacity_rows, int32_t *out_src_peer_dev,
                          int32_t *out_src_token_dev, int64_t *expert_offsets_dev, mw_recv_stats *recv_stats_dev,
                          void *stream)
{
    int32_t rc = check_unpack_index(ctx, peers_dev, n_peers, out_capacity_rows, expert_offsets_dev, recv_stats_dev);
    if (rc == MW_OK)
        rc = check_unpack_expand(ctx, n_peers, out_rows_dev, out_scales_dev, out_capacity_rows, out_src_peer_dev,
                                 out_src_token_dev);
    if (rc != MW_OK) return rc;
    rc = mw_launch_unpack_index(ctx, peers_dev, true, n_peers, out_capacity_rows, expert_offsets_dev, recv_stats_dev,
                                (hipStream_t)stream);
    if (rc != MW_OK) return rc;
    return mw_launch_unpack_expand(ctx, n_peers, out_rows_dev, out_scales_dev, out_capacity_rows, out_src_peer_dev,
                                   out_src_token_dev, (hipStream_t)stream);
}

// the members of the three batch records, as the calls they stand for check their arguments
static int32_t check_recv_batch(mw_ctx *ctx, const mw_recv_batch *r)
{
    if (!r || r->reserved0 != 0) return MW_ERR_INVALID_ARG;
    return check_unpack_expand(ctx, r->n_peers, r->out_rows_dev, r->out_scales_dev, r->out_capacity_rows,
                               r->out_src_peer_dev, r->out_src_token_dev);
}

static int32_t check_next_batch(mw_ctx *ctx, const mw_next_batch *n, bool with_plan)
{
    if (!n || !n->ctx || n->ctx == ctx || n->ctx->device != ctx->device) return MW_ERR_INVALID_ARG;
    const int32_t rc = check_unpack_index(n->ctx, n->peers_dev, n->n_peers, n->out_capacity_rows, n->expert_offsets_dev,
                                          n->recv_stats_dev);
    if (rc != MW_OK || !with_plan) return rc;
    if (!n->send_stats_dev || n->n_tokens < 0) return MW_ERR_INVALID_ARG;
    if (n->n_tokens > n->ctx->cfg.max_tokens) return MW_ERR_CAPACITY;
    if (n->n_tokens > 0 && (!n->topk_ids_dev || !n->mask_dev || !n->perm_dev || !n->desc_dev)) return MW_ERR_INVALID_ARG;
    return MW_OK;
}

MW_API int32_t mw_unpack_expand_index_next(mw_ctx *ctx, const mw_recv_batch *recv, const mw_next_batch *next,
                                           void *stream)
{
    if (!ctx) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    int32_t rc = check_recv_batch(ctx, recv);
    if (rc == MW_OK) rc = check_next_batch(ctx, next, false);
    if (rc != MW_OK) return rc;
    return mw_launch_unpack_expand_index_next(ctx, recv->n_peers, recv->out_rows_dev, recv->out_scales_dev,
                                              recv->out_capacity_rows, recv->out_src_peer_dev, recv->out_src_token_dev,
                                              next->ctx, next->peers_dev, next->n_peers, next->out_capacity_rows,
                                              next->expert_offsets_dev, next->recv_stats_dev, (hipStream_t)stream);
}

static int32_t launch_expand_index_plan(mw_ctx *ctx, const mw_recv_batch *recv, const mw_next_batch *next,
                                        const mw_pack_call *pk, void *stream)
{
    return mw_launch_unpack_expand_index_plan_next(ctx, recv->n_peers, recv->out_rows_dev, recv->out_scales_dev,
                                                   recv->out_capacity_rows, recv->out_src_peer_dev,
                                                   recv->out_src_token_dev, next->ctx, next->peers_dev, next->n_peers,
                                                   next->out_capacity_rows, next->expert_offsets_dev,
                                                   next->recv_stats_dev, next->topk_ids_dev, next->n_tokens,
                                                   next->mask_dev, next->perm_dev, next->desc_dev, next->send_stats_dev,
                                                   pk, (hipStream_t)stream);
}

MW_API int32_t mw_unpack_expand_index_plan_next(mw_ctx *ctx, const mw_recv_batch *recv, const mw_next_batch *next,
                                                void *stream)
{
    if (!ctx) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    int32_t rc = check_recv_batch(ctx, recv);
    if (rc == MW_OK) rc = check_next_batch(ctx, next, true);
    if (rc != MW_OK) return rc;
    return launch_expand_index_plan(ctx, recv, next, nullptr, stream);
}

MW_API int32_t mw_stream_step(mw_ctx *ctx, const mw_send_batch *send, const mw_recv_batch *recv,
                              const mw_next_batch *next, void *stream)
{
    if (!ctx || !send) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    // the packer's arguments, as mw_pack checks them
    if (!send->stats_dev || send->n_tokens < 0 || send->reserved0 != 0) return MW_ERR_INVALID_ARG;
    if (send->n_tokens > ctx->cfg.max_tokens) return MW_ERR_CAPACITY;
    if (send->n_tokens > 0) {
        if (!send->x_dev || !send->topk_ids_dev || !send->perm_dev || !send->packed_rows_dev ||
            !send->row_src_token_dev || !send->row_topk_dev)
            return MW_ERR_INVALID_ARG;
        if ((ctx->s_row_bytes > 0) != (send->scales_dev != nullptr)) return MW_ERR_INVALID_ARG;
        if (((uintptr_t)send->x_dev | (uintptr_t)send->packed_rows_dev | (uintptr_t)send->scales_dev) & 15u)
            return MW_ERR_INVALID_ARG;
    }
    int32_t rc = check_recv_batch(ctx, recv);
    if (rc == MW_OK) rc = check_next_batch(ctx, next, true);
    if (rc != MW_OK) return rc;
    const mw_pack_call pk = {send->x_dev, send->scales_dev, send->topk_ids_dev, send->perm_dev, send->stats_dev,
                             send->n_tokens, send->packed_rows_dev, send->row_src_token_dev, send->row_topk_dev};
    return launch_expand_index_plan(ctx, recv, next, &pk, stream);
}

MW_API int32_t mw_combine_gather(mw_ctx *ctx, int32_t n_peers, const void *y_dev, int64_t out_capacity_rows,
                          void *ret_rows_dev, int64_t ret_capacity_rows, void *stream)
{
    if (!ctx || out_capacity_rows < 0 || ret_capacity_rows < 0) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (ctx->cfg.row_format != MW_ROW_BF16) return MW_ERR_UNSUPPORTED;
    if (n_peers < 1 || n_peers > ctx->cfg.n_ranks || ctx->cfg.n_experts == 0) return MW_ERR_INVALID_ARG;
    if (out_capacity_rows > 0xffffffffLL || ret_capacity_rows > 0xffffffffLL) return MW_ERR_UNSUPPORTED;
    if (ret_capacity_rows == 0 || out_capacity_rows == 0) return MW_OK;
    if (!y_dev || !ret_rows_dev || (((uintptr_t)y_dev | (uintptr_t)ret_rows_dev) & 15u)) return MW_ERR_INVALID_ARG;
    return mw_launch_combine(ctx, n_peers, y_dev, out_capacity_rows, ret_rows_dev, ret_capacity_rows,
                             (hipStream_t)stream);
}

MW_API int32_t mw_unpack_index(mw_ctx *ctx, const mw_recv_peer *peers_dev, int32_t n_peers, int64_t out_capacity_rows,
                        int64_t *expert_offsets_dev, mw_recv_stats *recv_stats_dev, void *stream)
{
    const int32_t rc = check_unpack_index(ctx, peers_dev, n_peers, out_capacity_rows, expert_offsets_dev, recv_stats_dev);
    if (rc != MW_OK) return rc;
    return mw_launch_unpack_index(ctx, peers_dev, false, n_peers, out_capacity_rows, expert_offsets_dev, recv_stats_dev,
                                  (hipStream_t)stream);
}

MW_API int32_t mw_unpack_expand(mw_ctx *ctx, int32_t n_peers, void *out_rows_dev, float *out_scales_dev,
                         int64_t out_capacity_rows, int32_t *out_src_peer_dev, int32_t *out_src_token_dev, void *stream)
{
    const int32_t rc = check_unpack_expand(ctx, n_peers, out_rows_dev, out_scales_dev, out_capacity_rows,
                                           out_src_peer_dev, out_src_token_dev);
    if (rc != MW_OK) return rc;
    return mw_launch_unpack_expand(ctx, n_peers, out_rows_dev, out_scales_dev, out_capacity_rows, out_src_peer_dev,
                                   out_src_token_dev, (hipStream_t)stream);
}

MW_API int32_t mw_unpack_allgather(mw_ctx *ctx, const void *const *peer_shards_dev, int64_t shard_bytes, void *out_dev,
                            void *stream)
{
    if (!ctx || shard_bytes < 0) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (shard_bytes % 16 != 0) return MW_ERR_UNSUPPORTED;
    if (shard_bytes == 0) return MW_OK;
    if (!peer_shards_dev || !out_dev || ((uintptr_t)out_dev & 15u)) return MW_ERR_INVALID_ARG;
    return mw_launch_gather_shards(ctx, peer_shards_dev, shard_bytes, out_dev, (hipStream_t)stream);
}

MW_API int32_t mw_allgather_step(mw_ctx *ctx, const void *shard_dev, int64_t shard_bytes, void *send_buf_dev,
                          mw_group_desc *desc_dev, mw_send_stats *stats_dev, const void *const *peer_shards_dev,
                          void *out_dev, void *stream)
{
    if (!ctx || !desc_dev || !stats_dev || shard_bytes < 0) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (shard_bytes % 16 != 0) return MW_ERR_UNSUPPORTED;
    if (shard_bytes > 0) {
        if (!shard_dev || !send_buf_dev || !peer_shards_dev || !out_dev) return MW_ERR_INVALID_ARG;
        if (((uintptr_t)shard_dev | (uintptr_t)send_buf_dev | (uintptr_t)out_dev) & 15u) return MW_ERR_INVALID_ARG;
    }
    return mw_launch_allgather_step(ctx, shard_dev, shard_bytes, send_buf_dev, desc_dev, stats_dev, peer_shards_dev,
                                    out_dev, (hipStream_t)stream);
}

MW_API int32_t mw_sim_deliver(mw_ctx *ctx, const mw_group_desc *desc_dev, const mw_send_stats *stats_dev,
                       int32_t n_tokens, const void *packed_rows_dev, const int32_t *row_src_token_dev,
                       const int32_t *row_topk_dev, int32_t dst_rank, mw_group_desc *desc_out_dev,
                       void *rows_out_dev, int32_t *src_token_out_dev, int32_t *topk_out_dev,
                       uint32_t *counts_out_dev, void *stream)
{
    if (!ctx || !stats_dev || !counts_out_dev || n_tokens < 0) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (n_tokens > ctx->cfg.max_tokens) return MW_ERR_CAPACITY;
    if (dst_rank < 0 || dst_rank >= ctx->cfg.n_ranks) return MW_ERR_INVALID_ARG;
    if (n_tokens > 0 && (!desc_dev || !packed_rows_dev || !row_src_token_dev || !row_topk_dev || !desc_out_dev ||
                         !rows_out_dev || !src_token_out_dev || !topk_out_dev))
        return MW_ERR_INVALID_ARG;
    if (((uintptr_t)packed_rows_dev | (uintptr_t)rows_out_dev) & 15u) return MW_ERR_INVALID_ARG;
    return mw_launch_sim_deliver(ctx, desc_dev, stats_dev, n_tokens, packed_rows_dev, row_src_token_dev,
                                 row_topk_dev, dst_rank, desc_out_dev, rows_out_dev, src_token_out_dev,
                                 topk_out_dev, counts_out_dev, (hipStream_t)stream);
}

MW_API int32_t mw_copy_bytes(void *dst_dev, const void *src_dev, int64_t n_bytes, void *stream)
{
    if (n_bytes < 0) return MW_ERR_INVALID_ARG;
    if (n_bytes % 16 != 0) return MW_ERR_UNSUPPORTED;
    if (n_bytes == 0) return MW_OK;
    if (!dst_dev || !src_dev || (((uintptr_t)dst_dev | (uintptr_t)src_dev) & 15u)) return MW_ERR_INVALID_ARG;
    return mw_launch_copy(nullptr, dst_dev, src_dev, n_bytes, (hipStream_t)stream);
}

MW_API int32_t mw_get_send_stats(mw_ctx *ctx, const mw_send_stats *stats_dev, mw_send_stats *host_out, void *stream)
{
    if (!ctx || !stats_dev || !host_out) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    MW_HIP_CHECK(hipMemcpyAsync(host_out, stats_dev, sizeof(mw_send_stats), hipMemcpyDeviceToHost, (hipStream_t)stream));
    MW_HIP_CHECK(hipStreamSynchronize((hipStream_t)stream));
    return MW_OK;
}

MW_API int32_t mw_get_recv_stats(mw_ctx *ctx, const mw_recv_stats *stats_dev, mw_recv_stats *host_out, void *stream)
{
    if (!ctx || !stats_dev || !host_out) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    MW_HIP_CHECK(hipMemcpyAsync(host_out, stats_dev, sizeof(mw_recv_stats), hipMemcpyDeviceToHost, (hipStream_t)stream));
    MW_HIP_CHECK(hipStreamSynchronize((hipStream_t)stream));
    ctx->recv_rows_hint = host_out->n_rows_seen;       // sizes the next mw_unpack's launch
    return MW_OK;
}

MW_API int32_t mw_set_forwarding(mw_ctx *ctx, const int32_t *next_hop, int32_t n_hops)
{
    if (!ctx || !next_hop) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (n_hops < 1) return MW_ERR_INVALID_ARG;
    if (n_hops > ctx->cfg.max_hops) return MW_ERR_CAPACITY;
    std::vector<uint64_t> bits((size_t)MW_MASK_WORDS * MW_MAX_HOPS, 0);
    for (int32_t r = 0; r < ctx->cfg.n_ranks; ++r) {
        const int32_t h = next_hop[r];
        if (h < 0 || h >= n_hops) return MW_ERR_INVALID_ARG;
        bits[(size_t)h * MW_MASK_WORDS + (r >> 6)] |= 1ull << (r & 63);
    }
    MW_HIP_CHECK(hipDeviceSynchronize());
    MW_HIP_CHECK(hipMemcpy(ctx->d_hop_bits, bits.data(), bits.size() * sizeof(uint64_t), hipMemcpyHostToDevice));
    MW_HIP_CHECK(hipDeviceSynchronize());
    ctx->n_hops = n_hops;
    return MW_OK;
}

MW_API int32_t mw_relay(mw_ctx *ctx, const mw_recv_peer *in_dev, const mw_relay_child *children_dev,
                 int64_t child_capacity_rows, mw_relay_stats *stats_dev, void *stream)
{
    if (!ctx || !in_dev || !children_dev || !stats_dev || child_capacity_rows < 0) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (ctx->cfg.max_hops < 1 || ctx->n_hops < 1) return MW_ERR_INVALID_ARG;      // no forwarding table
    if (child_capacity_rows > 0x7fffffffLL) return MW_ERR_UNSUPPORTED;
    return mw_launch_relay(ctx, in_dev, children_dev, child_capacity_rows, stats_dev, (hipStream_t)stream);
}

MW_API int32_t mw_relay_index(mw_ctx *ctx, const mw_recv_peer *in_dev, const mw_relay_child *children_dev,
                       int64_t child_capacity_rows, mw_relay_stats *stats_dev, void *stream)
{
    if (!ctx || !in_dev || !children_dev || !stats_dev || child_capacity_rows < 0) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (ctx->cfg.max_hops < 1 || ctx->n_hops < 1) return MW_ERR_INVALID_ARG;      // no forwarding table
    if (child_capacity_rows > 0x7fffffffLL) return MW_ERR_UNSUPPORTED;
    return mw_launch_relay_index(ctx, in_dev, children_dev, child_capacity_rows, stats_dev, (hipStream_t)stream);
}

MW_API int32_t mw_relay_copy(mw_ctx *ctx, const mw_recv_peer *in_dev, const mw_relay_child *children_dev,
                      mw_relay_stats *stats_dev, void *stream)
{
    if (!ctx || !in_dev || !children_dev || !stats_dev) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (ctx->cfg.max_hops < 1 || ctx->n_hops < 1) return MW_ERR_INVALID_ARG;
    return mw_launch_relay_copy(ctx, in_dev, children_dev, stats_dev, nullptr, nullptr, nullptr, 0, nullptr,
                                (hipStream_t)stream);
}

MW_API int32_t mw_relay_copy_index_next(mw_ctx *ctx, const mw_recv_peer *in_dev, const mw_relay_child *children_dev,
                                 mw_relay_stats *stats_dev, mw_ctx *next_ctx, const mw_recv_peer *next_in_dev,
                                 const mw_relay_child *next_children_dev, int64_t next_child_capacity_rows,
                                 mw_relay_stats *next_stats_dev, void *stream)
{
    if (!ctx || !in_dev || !children_dev || !stats_dev) return MW_ERR_INVALID_ARG;
    if (!next_ctx || next_ctx == ctx || next_ctx->device != ctx->device) return MW_ERR_INVALID_ARG;
    if (!next_in_dev || !next_children_dev || !next_stats_dev || next_child_capacity_rows < 0) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (ctx->cfg.max_hops < 1 || ctx->n_hops < 1 || next_ctx->cfg.max_hops < 1 || next_ctx->n_hops < 1)
        return MW_ERR_INVALID_ARG;
    if (next_child_capacity_rows > 0x7fffffffLL) return MW_ERR_UNSUPPORTED;
    return mw_launch_relay_copy(ctx, in_dev, children_dev, stats_dev, next_ctx, next_in_dev, next_children_dev,
                                next_child_capacity_rows, next_stats_dev, (hipStream_t)stream);
}

MW_API int32_t mw_relay_batch(const mw_relay_job *copy, int32_t n_copy, const mw_relay_job *index, int32_t n_index,
                              void *stream)
{
    if (!copy || n_copy < 1 || n_copy > MW_RELAY_BATCH_MAX || n_index < 0 || n_index > MW_RELAY_BATCH_MAX)
        return MW_ERR_INVALID_ARG;
    if (n_index > 0 && !index) return MW_ERR_INVALID_ARG;
    const mw_ctx *seen[2 * MW_RELAY_BATCH_MAX];
    int n_seen = 0;
    for (int pass = 0; pass < 2; ++pass) {
        const mw_relay_job *jobs = pass == 0 ? copy : index;
        const int n = pass == 0 ? n_copy : n_index;
        for (int j = 0; j < n; ++j) {
            const mw_relay_job &q = jobs[j];
            if (!q.ctx || !q.in_dev || !q.children_dev || !q.stats_dev) return MW_ERR_INVALID_ARG;
            if (q.ctx->device != copy[0].ctx->device) return MW_ERR_INVALID_ARG;
            if (q.ctx->cfg.max_hops < 1 || q.ctx->n_hops < 1) return MW_ERR_INVALID_ARG;       // no forwarding table
            for (int k = 0; k < n_seen; ++k) if (seen[k] == q.ctx) return MW_ERR_INVALID_ARG;
            seen[n_seen++] = q.ctx;
            if (pass == 1 && (q.child_capacity_rows < 0)) return MW_ERR_INVALID_ARG;
            if (pass == 1 && q.child_capacity_rows > 0x7fffffffLL) return MW_ERR_UNSUPPORTED;
        }
    }
    const mw_ctx *a = copy[0].ctx;
    for (int j = 1; j < n_copy; ++j) {
        const mw_ctx *x = copy[j].ctx;
        if (x->row_bytes != a->row_bytes || x->row_stride != a->row_stride || x->cfg.top_k != a->cfg.top_k ||
            x->cfg.max_tokens != a->cfg.max_tokens)
            return MW_ERR_INVALID_ARG;
    }
    MW_ON_DEVICE(copy[0].ctx);
    return mw_launch_relay_batch(copy, n_copy, index, n_index, (hipStream_t)stream);
}

MW_API int32_t mw_relay_packets(mw_ctx *ctx, const mw_recv_packets *in_dev, void *const *children_dev,
                         int64_t child_capacity_rows, mw_relay_stats *stats_dev, void *stream)
{
    if (!ctx || !in_dev || !children_dev || !stats_dev || child_capacity_rows < 0) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (ctx->cfg.max_hops < 1 || ctx->n_hops < 1) return MW_ERR_INVALID_ARG;      // no forwarding table
    if (ctx->cfg.n_experts == 0) return MW_ERR_INVALID_ARG;
    if (child_capacity_rows > 0x7fffffffLL) return MW_ERR_UNSUPPORTED;
    return mw_launch_relay_packets(ctx, in_dev, children_dev, child_capacity_rows, stats_dev, (hipStream_t)stream);
}

static int32_t relay_packets_ready(const mw_ctx *ctx)
{
    if (ctx->cfg.max_hops < 1 || ctx->n_hops < 1) return MW_ERR_INVALID_ARG;      // no forwarding table
    if (ctx->cfg.n_experts == 0) return MW_ERR_INVALID_ARG;
    return MW_OK;
}

MW_API int32_t mw_relay_packets_index(mw_ctx *ctx, const mw_recv_packets *in_dev, int64_t child_capacity_rows,
                               mw_relay_stats *stats_dev, void *stream)
{
    if (!ctx || !in_dev || !stats_dev || child_capacity_rows < 0) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (relay_packets_ready(ctx) != MW_OK) return MW_ERR_INVALID_ARG;
    if (child_capacity_rows > 0x7fffffffLL) return MW_ERR_UNSUPPORTED;
    return mw_launch_relay_packets_index(ctx, in_dev, child_capacity_rows, stats_dev, (hipStream_t)stream);
}

MW_API int32_t mw_relay_packets_copy(mw_ctx *ctx, const mw_recv_packets *in_dev, void *const *children_dev,
                              mw_relay_stats *stats_dev, void *stream)
{
    if (!ctx || !in_dev || !children_dev || !stats_dev) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (relay_packets_ready(ctx) != MW_OK) return MW_ERR_INVALID_ARG;
    return mw_launch_relay_packets_copy(ctx, in_dev, children_dev, stats_dev, nullptr, nullptr, 0, nullptr,
                                        (hipStream_t)stream);
}

MW_API int32_t mw_relay_packets_copy_index_next(mw_ctx *ctx, const mw_recv_packets *in_dev, void *const *children_dev,
                                         mw_relay_stats *stats_dev, mw_ctx *next_ctx,
                                         const mw_recv_packets *next_in_dev, int64_t next_child_capacity_rows,
                                         mw_relay_stats *next_stats_dev, void *stream)
{
    if (!ctx || !in_dev || !children_dev || !stats_dev) return MW_ERR_INVALID_ARG;
    if (!next_ctx || next_ctx == ctx || next_ctx->device != ctx->device) return MW_ERR_INVALID_ARG;
    if (!next_in_dev || !next_stats_dev || next_child_capacity_rows < 0) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    if (relay_packets_ready(ctx) != MW_OK || relay_packets_ready(next_ctx) != MW_OK) return MW_ERR_INVALID_ARG;
    if (next_child_capacity_rows > 0x7fffffffLL) return MW_ERR_UNSUPPORTED;
    return mw_launch_relay_packets_copy(ctx, in_dev, children_dev, stats_dev, next_ctx, next_in_dev,
                                        next_child_capacity_rows, next_stats_dev, (hipStream_t)stream);
}

MW_API int32_t mw_get_relay_stats(mw_ctx *ctx, const mw_relay_stats *stats_dev, mw_relay_stats *host_out, void *stream)
{
    if (!ctx || !stats_dev || !host_out) return MW_ERR_INVALID_ARG;
    MW_ON_DEVICE(ctx);
    MW_HIP_CHECK(hipMemcpyAsync(host_out, stats_dev, sizeof(mw_relay_stats), hipMemcpyDeviceToHost, (hipStream_t)stream));
    MW_HIP_CHECK(hipStreamSynchronize((hipStream_t)stream));
    return MW_OK;
}

MW_API int32_t mw_ctx_set_ride_wait_limit(mw_ctx *ctx, int64_t polls)
{
    if (!ctx || polls < 0 || polls > 0x7fffffffLL) return MW_ERR_INVALID_ARG;
    ctx->ride_wait_limit = (uint32_t)polls;
    return MW_OK;
}

MW_API int32_t mw_ctx_set_options(mw_ctx *ctx, uint32_t options)
{
    if (!ctx || (options & ~(uint32_t)(MW_OPT_RELAY_KEEP_METADATA | MW_OPT_RECV_DEDUP))) return MW_ERR_INVALID_ARG;
    ctx->options = options;
    return MW_OK;
}

MW_API int32_t mw_ctx_set_timing_events(mw_ctx *ctx, int32_t kernel, void *ev_start, void *ev_stop)
{
    if (!ctx || kernel < 0 || kernel >= MW_KERNEL_COUNT) return MW_ERR_INVALID_ARG;
    if ((ev_start == nullptr) != (ev_stop == nullptr)) return MW_ERR_INVALID_ARG;
    ctx->ev_start[kernel] = (hipEvent_t)ev_start;
    ctx->ev_stop[kernel] = (hipEvent_t)ev_stop;
    return MW_OK;
}

MW_API const char *mw_status_string(int32_t status)
{
    switch (status) {
    case MW_OK: return "ok";
    case MW_ERR_INVALID_ARG: return "invalid argument";
    case MW_ERR_CAPACITY: return "size beyond the context's capacity";
    case MW_ERR_UNSUPPORTED: return "unsupported configuration";
    case MW_ERR_HIP: return "HIP runtime error";
    case MW_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    default: return "unknown status";
    }
}

}  // extern "C"
