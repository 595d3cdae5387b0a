// Receive side: index builder and expander.
//
// Paper hooks: Section 4.1 workflow steps 3-4 -- the receiver parses the carried
// metadata and, if it is one of the destinations, delivers the payload to the target
// memory; Section 5.1 -- the receive module does reception, reassembly and delivery of
// the final buffers; Section 6.4 "Memory usage" -- one pre-allocated receive region per
// peer.  The bitmap of a row's group is the authority on whether this rank is addressed;
// which local experts get the row follows from the row's top-k ids and the rank table.
//
// Two launches on the caller's stream:
//   k_recv_index  one workgroup per peer.  Marks addressed rows from the descriptor
//                 bitmaps, then for every local expert builds an LDS bitmap over the
//                 peer's source-token indices.  A prefix of popcounts over that bitmap
//                 is the stable rank of a row among the peer's rows for that expert,
//                 whatever order the rows were packed in -- no sort, no order-dependent
//                 atomics (LDS atomic ORs only set bits).  Emits per-(expert, peer)
//                 counts and per-row (expert slot, rank) pairs.
//   k_expand      persistent workgroups.  Each first scans the (expert, peer) counts in
//                 LDS into output bases (a few hundred integers, cheaper than another
//                 launch or a grid-wide barrier), then walks received rows: a row is
//                 read once with 16-byte streaming loads and stored to each of its
//                 experts' slots.  This kernel moves ~all receive-side bytes and is
//                 bound by HBM bandwidth.
#include "mw_internal.h"

namespace {

constexpr int kIndexBlock = 1024;
constexpr int kExpandBlock = 256;

__device__ __forceinline__ bool mask_has(const uint64_t *m, int r) { return (m[r >> 6] >> (r & 63)) & 1ull; }

// Is topk_row[j] the first occurrence of its id in the row?  (duplicate ids count once)
__device__ __forceinline__ bool first_occurrence(const int32_t *topk_row, int j)
{
    const int32_t e = topk_row[j];
    for (int k = 0; k < j; ++k)
        if (topk_row[k] == e) return false;
    return true;
}

__global__ __launch_bounds__(kIndexBlock) void k_recv_index(
    const mw_recv_peer *__restrict__ peers, int P, const int32_t *__restrict__ e2r,
    const int32_t *__restrict__ local_slot, int E, int K, int Kd, int my_rank, int L, int Lc,
    uint32_t max_tokens, uint32_t wpl, uint32_t cap_rows, uint32_t *__restrict__ cnt,
    uint32_t *__restrict__ row_base, uint32_t *__restrict__ addr_cnt, mw_hit *__restrict__ hits,
    uint32_t *__restrict__ flags)
{
    extern __shared__ uint32_t lds[];
    uint32_t *addr = lds;                 // [wpl]      bit i: row i's group names this rank
    uint32_t *bits = addr + wpl;          // [Lc][wpl]  bit s of expert l: a row with source token s
    uint32_t *pre = bits + (size_t)Lc * wpl;   // [Lc][wpl] running popcount before each word
    uint32_t *scratch = pre + (size_t)Lc * wpl; // [17]

    const int tid = threadIdx.x, nthr = blockDim.x, p = blockIdx.x;
    const mw_recv_peer pr = peers[p];
    uint32_t err = 0;

    // rows of the peers before this one (each clamped to max_tokens, the total to cap_rows);
    // at most 256 peers of at most 65536 rows, so 32 bits are enough
    uint32_t part = 0;
    for (int q = tid; q < p; q += nthr) part += min(peers[q].n_rows, max_tokens);
    uint32_t before;
    mw_block_exscan(part, scratch, &before);
    const uint32_t mine = min(pr.n_rows, max_tokens);
    if (pr.n_rows > max_tokens || before + mine > cap_rows) err |= MW_FLAG_RECV_CAPACITY;
    const uint32_t rb = min(before, cap_rows);
    const uint32_t n_rows = min(before + mine, cap_rows) - rb;
    if (tid == 0) {
        row_base[p] = rb;
        if (p == P - 1) row_base[P] = rb + n_rows;
    }

    for (uint32_t w = tid; w < wpl; w += nthr) addr[w] = 0;
    for (uint32_t k = tid; k < n_rows * (uint32_t)Kd; k += nthr) hits[(size_t)rb * Kd + k] = mw_hit{-1, 0};
    __syncthreads();

    // addressed rows: groups whose bitmap has this rank's bit
    for (uint32_t g = tid; g < pr.n_desc; g += nthr) {
        const mw_group_desc *d = pr.desc + g;
        if (!mask_has(d->mask, my_rank)) continue;
        const uint64_t b = d->row_offset, e = b + d->row_count;
        if (e > n_rows) { err |= MW_FLAG_BAD_DESC; continue; }
        if (e <= b) continue;
        for (uint64_t w = b >> 5; w <= ((e - 1) >> 5); ++w) {
            const uint64_t wlo = w << 5;
            uint32_t m = 0xffffffffu;
            if (b > wlo) m &= 0xffffffffu << (b - wlo);
            if (e < wlo + 32) m &= 0xffffffffu >> (wlo + 32 - e);
            atomicOr(&addr[w], m);
        }
    }
    __syncthreads();
    {
        uint32_t a = 0, tot;
        for (uint32_t w = tid; w < wpl; w += nthr) a += __popc(addr[w]);
        mw_block_exscan(a, scratch, &tot);
        if (tid == 0) addr_cnt[p] = tot;
    }

    for (int le0 = 0; le0 < L; le0 += Lc) {
        const int lc = min(Lc, L - le0);
        const uint32_t n_words = (uint32_t)lc * wpl;
        for (uint32_t f = tid; f < n_words; f += nthr) bits[f] = 0;
        __syncthreads();

        // mark (expert, source token) pairs
        for (uint32_t i = tid; i < n_rows; i += nthr) {
            if (!((addr[i >> 5] >> (i & 31)) & 1u)) continue;
            const uint32_t s = (uint32_t)pr.row_src_token[i];
            if (s >= max_tokens) { err |= MW_FLAG_BAD_SRC_TOKEN; continue; }
            const int32_t *tk = pr.row_topk + (size_t)i * K;
            for (int j = 0; j < K; ++j) {
                const int32_t e = tk[j];
                if (e == -1) continue;
                if ((uint32_t)e >= (uint32_t)E) { err |= MW_FLAG_BAD_EXPERT; continue; }
                if (e2r[e] != my_rank) continue;
                const int l = local_slot[e] - le0;
                if (l < 0 || l >= lc || !first_occurrence(tk, j)) continue;
                const uint32_t old = atomicOr(&bits[(uint32_t)l * wpl + (s >> 5)], 1u << (s & 31));
                if ((old >> (s & 31)) & 1u) err |= MW_FLAG_DUP_SRC_TOKEN;
            }
        }
        __syncthreads();

        // running popcounts over the chunk's words (expert-major), one flat scan
        uint32_t carry = 0;
        for (uint32_t f0 = 0; f0 < n_words; f0 += nthr) {
            const uint32_t f = f0 + tid;
            const uint32_t v = (f < n_words) ? __popc(bits[f]) : 0u;
            uint32_t tot;
            const uint32_t ex = mw_block_exscan(v, scratch, &tot);
            if (f < n_words) pre[f] = carry + ex;
            carry += tot;
        }
        __syncthreads();
        for (int l = tid; l < lc; l += nthr) {
            const uint32_t end = (l + 1 < lc) ? pre[(uint32_t)(l + 1) * wpl] : carry;
            cnt[(size_t)(le0 + l) * P + p] = end - pre[(uint32_t)l * wpl];
        }

        // per row: (expert slot, stable rank) for every distinct local expert it names
        for (uint32_t i = tid; i < n_rows; i += nthr) {
            if (!((addr[i >> 5] >> (i & 31)) & 1u)) continue;
            const uint32_t s = (uint32_t)pr.row_src_token[i];
            if (s >= max_tokens) continue;
            const int32_t *tk = pr.row_topk + (size_t)i * K;
            int k = 0;
            for (int j = 0; j < K; ++j) {
                const int32_t e = tk[j];
                if (e == -1 || (uint32_t)e >= (uint32_t)E || e2r[e] != my_rank || !first_occurrence(tk, j)) continue;
                const int l = local_slot[e] - le0;
                if (l >= 0 && l < lc) {
                    const uint32_t wi = (uint32_t)l * wpl + (s >> 5);
                    const uint32_t r = pre[wi] - pre[(uint32_t)l * wpl] + __popc(bits[wi] & ((1u << (s & 31)) - 1u));
                    hits[(size_t)(rb + i) * Kd + k] = mw_hit{le0 + l, (int32_t)r};
                }
                ++k;
            }
            if (k == 0 && le0 == 0) err |= MW_FLAG_NO_LOCAL_EXPERT;
        }
        __syncthreads();
    }
    if (L == 0) {
        // no expert lives here: any addressed row is inconsistent
        for (uint32_t w = tid; w < wpl; w += nthr) if (addr[w]) err |= MW_FLAG_NO_LOCAL_EXPERT;
    }
    if (err) atomicOr(&flags[1], err);
}

template <int U>
__global__ __launch_bounds__(kExpandBlock) void k_expand(
    const mw_recv_peer *__restrict__ peers, int P, const uint32_t *__restrict__ row_base,
    const uint32_t *__restrict__ cnt, const mw_hit *__restrict__ hits, int Kd, int L, int xc, int sc, int tpr,
    u32x4 *__restrict__ out_rows, u32x4 *__restrict__ out_scales, int64_t cap,
    int32_t *__restrict__ out_src_peer, int32_t *__restrict__ out_src_token,
    int64_t *__restrict__ expert_offsets, mw_recv_stats *__restrict__ stats,
    const uint32_t *__restrict__ addr_cnt, uint32_t *flags)
{
    extern __shared__ uint32_t lds[];
    uint32_t *base = lds;                       // [L * P] first output row of (expert, peer)
    uint32_t *rbase = base + (size_t)L * P;     // [P + 1]
    uint32_t *scratch = rbase + P + 1;          // [17]
    const int tid = threadIdx.x, nthr = blockDim.x;

    const uint32_t n_lp = (uint32_t)L * P;
    uint32_t carry = 0;
    for (uint32_t f0 = 0; f0 < n_lp; f0 += nthr) {
        const uint32_t f = f0 + tid;
        const uint32_t v = (f < n_lp) ? cnt[f] : 0u;
        uint32_t tot;
        const uint32_t ex = mw_block_exscan(v, scratch, &tot);
        if (f < n_lp) base[f] = carry + ex;
        carry += tot;
    }
    const uint32_t Q = carry;
    for (int q = tid; q <= P; q += nthr) rbase[q] = row_base[q];
    __syncthreads();

    if (blockIdx.x == 0) {
        for (int le = tid; le < L; le += nthr) expert_offsets[le] = base[(uint32_t)le * P];
        if (tid == 0) {
            expert_offsets[L] = Q;
            uint64_t m = 0;
            for (int q = 0; q < P; ++q) m += addr_cnt[q];
            stats->n_recv_rows = m;
            stats->n_out_rows = Q;
            stats->error_flags = flags[1] | (((int64_t)Q > cap) ? MW_FLAG_OUT_CAPACITY : 0u);
            stats->reserved0 = 0;
            flags[1] = 0;      // ready for the next unpack
        }
    }

    const uint32_t m_total = rbase[P];
    const int rows_per_block = nthr / tpr;
    const int sub = __builtin_amdgcn_readfirstlane(tid / tpr);   // tpr is a multiple of the wave size
    const int lane = tid - sub * tpr;
    const int n = xc + sc;
    for (uint32_t g = blockIdx.x * rows_per_block + sub; g < m_total; g += gridDim.x * rows_per_block) {
        const mw_hit *h = hits + (size_t)g * Kd;
        if (h[0].le < 0) continue;              // slots fill from 0: nothing to deliver
        int lo = 0, hi = P;                     // peer of row g: last p with rbase[p] <= g
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (rbase[mid] <= g) lo = mid; else hi = mid;
        }
        const int p = lo;
        const uint32_t i = g - rbase[p];
        const u32x4 *src = (const u32x4 *)peers[p].rows + (size_t)i * n;
        for (int c0 = lane; c0 < n; c0 += U * tpr) {
            u32x4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = c0 + u * tpr;
                if (c < n) v[u] = mw_ld16(src + c);
            }
            for (int k = 0; k < Kd; ++k) {
                const mw_hit hk = h[k];
                if (hk.le < 0) break;
                const int64_t dst = (int64_t)base[(uint32_t)hk.le * P + p] + hk.rank;
                if (dst >= cap) continue;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int c = c0 + u * tpr;
                    if (c < xc) mw_st16(out_rows + (size_t)dst * xc + c, v[u]);
                    else if (c < n) mw_st16(out_scales + (size_t)dst * sc + (c - xc), v[u]);
                }
            }
        }
        if (lane == 0) {
            const int32_t stok = peers[p].row_src_token[i];
            for (int k = 0; k < Kd; ++k) {
                const mw_hit hk = h[k];
                if (hk.le < 0) break;
                const int64_t dst = (int64_t)base[(uint32_t)hk.le * P + p] + hk.rank;
                if (dst >= cap) continue;
                out_src_peer[dst] = p;
                out_src_token[dst] = stok;
            }
        }
    }
}

}  // namespace

static int lanes_per_row(int chunks, int U)
{
    int tpr = 64;
    while (tpr < kExpandBlock && tpr * U < chunks) tpr *= 2;
    return tpr;
}

int32_t mw_launch_unpack(mw_ctx *ctx, const mw_recv_peer *peers, int32_t P, void *out_rows,
                         float *out_scales, int64_t cap, int32_t *out_src_peer, int32_t *out_src_token,
                         int64_t *expert_offsets, mw_recv_stats *stats, hipStream_t s)
{
    const mw_config &c = ctx->cfg;
    const int L = ctx->n_local, Kd = ctx->hit_slots;
    const uint32_t wpl = ((uint32_t)c.max_tokens + 31u) / 32u;
    // LDS budget of the index kernel: addressed bitmap + 2 arrays per expert of the chunk
    const uint32_t budget_words = 12288 - 32;
    int Lc = (int)((budget_words - wpl) / (2 * wpl));
    if (Lc < 1) return MW_ERR_UNSUPPORTED;
    if (Lc > L) Lc = L > 0 ? L : 1;
    const size_t lds_index = ((size_t)wpl + 2 * (size_t)Lc * wpl + 32) * sizeof(uint32_t);
    hipLaunchKernelGGL(k_recv_index, dim3(P), dim3(kIndexBlock), lds_index, s, peers, P, ctx->d_e2r,
                       ctx->d_local_slot, c.n_experts, c.top_k, Kd, c.my_rank, L, Lc, (uint32_t)c.max_tokens,
                       wpl, (uint32_t)c.max_recv_rows, ctx->d_cnt, ctx->d_row_base, ctx->d_addr_cnt, ctx->d_hits,
                       ctx->d_flags);

    const int xc = (int)(ctx->x_row_bytes / 16), sc = (int)(ctx->s_row_bytes / 16);
    constexpr int U = 4;
    const int tpr = lanes_per_row(xc + sc, U);
    const size_t lds_expand = ((size_t)L * P + P + 1 + 32) * sizeof(uint32_t);
    const int grid = ctx->n_cu * 8;
    hipLaunchKernelGGL(k_expand<U>, dim3(grid), dim3(kExpandBlock), lds_expand, s, peers, P, ctx->d_row_base,
                       ctx->d_cnt, ctx->d_hits, Kd, L, xc, sc, tpr, (u32x4 *)out_rows, (u32x4 *)out_scales, cap,
                       out_src_peer, out_src_token, expert_offsets, stats, ctx->d_addr_cnt, ctx->d_flags);
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}
