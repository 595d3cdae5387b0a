// Send-side plan kernels: destination bitmaps, (bitmap, token) ordering, multicast
// groups, descriptor table and byte accounting.
//
// Paper hooks: the bitmap is Section 4.1's metadata encoding (bit r <-> rank r, ranks
// from zero, a preconfigured id -> rank table); groups are discovered per batch because
// the space of destination sets cannot be provisioned in advance (Section 2.3.2,
// C(64,8) sets at EP=64/top-8); the accounting is Section 1's "one copy however many
// destinations" against one copy per destination.
//
// Three launches on the caller's stream, no host synchronisation:
//   k_masks   one lane per token, ORs the K rank bits into four 64-bit words; wavefront
//             ballots + popcounts turn 64 tokens' bitmaps into per-rank counts.
//   k_rank    position of every kept token in (bitmap, token) order by counting its
//             predecessors.  A lane owns one token and walks a slice of all tokens whose
//             bitmaps are wave-uniform (scalar loads), so a step is a handful of 64-bit
//             compares; slices are spread over the whole chip and combined with integer
//             atomic adds (a sum, so the result does not depend on arrival order).
//             For the batch sizes of a dispatch (<= 8k tokens) this beats a multi-pass
//             radix sort of 256-bit keys, which would be launch- and barrier-bound.
//   k_groups  one workgroup: scatter perm, mark bitmap changes, scan them into group ids,
//             write descriptors and statistics.
#include "mw_internal.h"

namespace {

constexpr int kRankBlock = 256;
constexpr int kGroupsBlock = 1024;

__global__ __launch_bounds__(256) void k_masks(const int32_t *__restrict__ topk, int T, int K,
                                               const int32_t *__restrict__ e2r, int E,
                                               uint64_t *__restrict__ mask, uint32_t *__restrict__ pos,
                                               uint32_t *__restrict__ hist, uint32_t *__restrict__ flags)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = threadIdx.x & 63;
    uint64_t m[MW_MASK_WORDS] = {0, 0, 0, 0};
    bool bad = false;
    if (t < T) {
        const int32_t *row = topk + (size_t)t * K;
        for (int j = 0; j < K; ++j) {
            const int32_t e = row[j];
            if (e == -1) continue;
            if ((uint32_t)e >= (uint32_t)E) { bad = true; continue; }
            const int r = e2r[e];
            const uint64_t bit = 1ull << (r & 63);
            const int w = r >> 6;
#pragma unroll
            for (int q = 0; q < MW_MASK_WORDS; ++q) m[q] |= (w == q) ? bit : 0ull;
        }
        uint64_t *o = mask + (size_t)t * MW_MASK_WORDS;
#pragma unroll
        for (int q = 0; q < MW_MASK_WORDS; ++q) o[q] = m[q];
        pos[t] = 0;
        if (bad) atomicOr(flags, MW_FLAG_BAD_EXPERT);
    }
    // rows per destination: a wavefront ballot of bit b over 64 tokens, popcounted, is the
    // number of those tokens that name rank 64*q + b; lane b keeps it and adds it once.
#pragma unroll
    for (int q = 0; q < MW_MASK_WORDS; ++q) {
        if (__ballot(m[q] != 0) == 0) continue;      // wave-uniform
        uint32_t mine = 0;
        for (int b = 0; b < 64; ++b) {
            const uint32_t c = (uint32_t)__popcll(__ballot((m[q] >> b) & 1ull));
            if (lane == b) mine = c;
        }
        if (mine) atomicAdd(&hist[q * 64 + lane], mine);
    }
}

// pos[t] += #{u in this block's slice : (mask[u], u) < (mask[t], t)}.  Tokens with an
// empty bitmap compare below every kept token; k_groups subtracts their number.
template <int W>
__global__ __launch_bounds__(kRankBlock) void k_rank(const uint64_t *__restrict__ mask, int T, int slice,
                                                     uint32_t *__restrict__ pos)
{
    const int t = blockIdx.x * kRankBlock + threadIdx.x;
    const int u0 = blockIdx.y * slice;
    const int u1 = min(u0 + slice, T);
    uint64_t m[W];
    bool any = false;
#pragma unroll
    for (int w = 0; w < W; ++w) {
        m[w] = (t < T) ? mask[(size_t)t * MW_MASK_WORDS + w] : 0ull;
        any |= (m[w] != 0);
    }
    uint32_t c = 0;
#pragma unroll 4
    for (int u = u0; u < u1; ++u) {
        const uint64_t *q = mask + (size_t)u * MW_MASK_WORDS;   // wave-uniform address
        bool lt = false, eq = true;
#pragma unroll
        for (int w = W - 1; w >= 0; --w) {
            const uint64_t qw = q[w];
            lt = lt || (eq && qw < m[w]);
            eq = eq && (qw == m[w]);
        }
        lt = lt || (eq && u < t);
        c += lt ? 1u : 0u;
    }
    if (any && c) atomicAdd(&pos[t], c);
}

__device__ __forceinline__ bool mask_equal(const uint64_t *a, const uint64_t *b)
{
    return a[0] == b[0] && a[1] == b[1] && a[2] == b[2] && a[3] == b[3];
}

// One workgroup.  Loads are batched (independent, unrolled) and the sorted bitmaps go
// through a scratch array so that every phase costs one memory round trip, not one per row.
__global__ __launch_bounds__(kGroupsBlock) void k_groups(const uint64_t *__restrict__ mask,
                                                         const uint32_t *__restrict__ pos, int T,
                                                         uint64_t row_bytes, int32_t *__restrict__ perm,
                                                         uint64_t *__restrict__ smask, mw_group_desc *desc,
                                                         mw_send_stats *stats, uint32_t *hist, uint32_t *flags)
{
    __shared__ uint32_t scratch[17];
    const int tid = threadIdx.x;

    // kept tokens; total destinations from the histogram k_masks accumulated
    uint32_t kept = 0;
#pragma unroll 4
    for (int t = tid; t < T; t += kGroupsBlock) {
        const uint64_t *m = mask + (size_t)t * MW_MASK_WORDS;
        kept += (m[0] | m[1] | m[2] | m[3]) ? 1u : 0u;
    }
    uint32_t dests = 0;
    for (int r = tid; r < MW_MAX_RANKS; r += kGroupsBlock) {
        const uint32_t h = hist[r];
        stats->rows_per_dest[r] = h;
        dests += h;
        hist[r] = 0;           // ready for the next plan
    }
    uint32_t N, D;
    mw_block_exscan(kept, scratch, &N);
    mw_block_exscan(dests, scratch, &D);
    const uint32_t n_empty = (uint32_t)T - N;

    // perm and the bitmaps in sorted order: token t goes to its predecessor count among kept tokens
#pragma unroll 4
    for (int t = tid; t < T; t += kGroupsBlock) {
        const uint64_t *m = mask + (size_t)t * MW_MASK_WORDS;
        const uint64_t m0 = m[0], m1 = m[1], m2 = m[2], m3 = m[3];
        const uint32_t i = pos[t] - n_empty;
        if ((m0 | m1 | m2 | m3) && i < N) {
            perm[i] = t;
            uint64_t *o = smask + (size_t)i * MW_MASK_WORDS;
            o[0] = m0; o[1] = m1; o[2] = m2; o[3] = m3;
        }
    }
    __syncthreads();

    // group starts: row i opens a group when its bitmap differs from row i-1's
    const uint32_t per = (N + kGroupsBlock - 1) / kGroupsBlock;
    const uint32_t i0 = min((uint32_t)tid * per, N), i1 = min(i0 + per, N);
    uint64_t p0 = 0, p1 = 0, p2 = 0, p3 = 0;                      // bitmap of row i0 - 1, if there is one
    bool have_prev = false;
    if (i0 > 0 && i0 < i1) {
        const uint64_t *q = smask + (size_t)(i0 - 1) * MW_MASK_WORDS;
        p0 = q[0]; p1 = q[1]; p2 = q[2]; p3 = q[3];
        have_prev = true;
    }
    uint32_t starts = 0;
    {
        uint64_t a0 = p0, a1 = p1, a2 = p2, a3 = p3;
        bool hp = have_prev;
#pragma unroll 4
        for (uint32_t i = i0; i < i1; ++i) {
            const uint64_t *q = smask + (size_t)i * MW_MASK_WORDS;
            const uint64_t c0 = q[0], c1 = q[1], c2 = q[2], c3 = q[3];
            starts += (!hp || c0 != a0 || c1 != a1 || c2 != a2 || c3 != a3) ? 1u : 0u;
            a0 = c0; a1 = c1; a2 = c2; a3 = c3; hp = true;
        }
    }
    uint32_t G;
    uint32_t g = mw_block_exscan(starts, scratch, &G);
    {
        uint64_t a0 = p0, a1 = p1, a2 = p2, a3 = p3;
        bool hp = have_prev;
        for (uint32_t i = i0; i < i1; ++i) {
            const uint64_t *q = smask + (size_t)i * MW_MASK_WORDS;
            const uint64_t c0 = q[0], c1 = q[1], c2 = q[2], c3 = q[3];
            if (!hp || c0 != a0 || c1 != a1 || c2 != a2 || c3 != a3) {
                mw_group_desc d;
                d.mask[0] = c0; d.mask[1] = c1; d.mask[2] = c2; d.mask[3] = c3;
                d.row_offset = i; d.row_count = 0;
                d.n_dest = (uint32_t)(__popcll(c0) + __popcll(c1) + __popcll(c2) + __popcll(c3));
                d.reserved0 = 0;
                desc[g++] = d;
            }
            a0 = c0; a1 = c1; a2 = c2; a3 = c3; hp = true;
        }
    }
    __syncthreads();
#pragma unroll 4
    for (uint32_t k = tid; k < G; k += kGroupsBlock) {
        const uint32_t next = (k + 1 < G) ? desc[k + 1].row_offset : N;
        desc[k].row_count = next - desc[k].row_offset;
    }

    if (tid == 0) {
        stats->n_rows = N;
        stats->n_groups = G;
        stats->multicast_bytes = (uint64_t)N * row_bytes;
        stats->unicast_bytes = (uint64_t)D * row_bytes;
        stats->error_flags = flags[0];
        stats->reserved0 = 0;
        flags[0] = 0;      // ready for the next plan
    }
}

__global__ __launch_bounds__(256) void k_plan_allgather(int R, uint64_t shard_bytes, mw_group_desc *desc,
                                                        mw_send_stats *stats)
{
    const int tid = threadIdx.x;
    if (tid < MW_MAX_RANKS) stats->rows_per_dest[tid] = (tid < R) ? 1u : 0u;
    if (tid == 0) {
        mw_group_desc d;
#pragma unroll
        for (int w = 0; w < MW_MASK_WORDS; ++w) {
            const int lo = w * 64;
            d.mask[w] = (R >= lo + 64) ? ~0ull : (R > lo ? ((1ull << (R - lo)) - 1ull) : 0ull);
        }
        d.row_offset = 0; d.row_count = 1; d.n_dest = (uint32_t)R; d.reserved0 = 0;
        *desc = d;
        stats->n_rows = 1; stats->n_groups = 1;
        stats->multicast_bytes = shard_bytes;
        stats->unicast_bytes = shard_bytes * (uint64_t)R;
        stats->error_flags = 0; stats->reserved0 = 0;
    }
}

}  // namespace

int32_t mw_launch_plan(mw_ctx *ctx, const int32_t *topk, int32_t T, uint64_t *mask, int32_t *perm,
                       mw_group_desc *desc, mw_send_stats *stats, hipStream_t s)
{
    const int K = ctx->cfg.top_k, E = ctx->cfg.n_experts;
    if (T > 0) {
        {
            mw_timed tm(ctx, MW_KERNEL_PLAN_MASKS, s);
            hipLaunchKernelGGL(k_masks, dim3((T + 255) / 256), dim3(256), 0, s, topk, T, K, ctx->d_e2r, E, mask,
                               ctx->d_pos, ctx->d_hist, ctx->d_flags);
        }
        // split the predecessor walk into slices so that about 4 workgroups land on every CU
        const int tb = (T + kRankBlock - 1) / kRankBlock;
        int ns = (4 * ctx->n_cu + tb - 1) / tb;
        if (ns < 1) ns = 1;
        int slice = (T + ns - 1) / ns;
        if (slice < 64) slice = 64;
        ns = (T + slice - 1) / slice;
        const dim3 grid(tb, ns), block(kRankBlock);
        mw_timed tm(ctx, MW_KERNEL_PLAN_RANK, s);
        switch (ctx->mask_words) {
        case 1: hipLaunchKernelGGL(k_rank<1>, grid, block, 0, s, mask, T, slice, ctx->d_pos); break;
        case 2: hipLaunchKernelGGL(k_rank<2>, grid, block, 0, s, mask, T, slice, ctx->d_pos); break;
        case 3: hipLaunchKernelGGL(k_rank<3>, grid, block, 0, s, mask, T, slice, ctx->d_pos); break;
        default: hipLaunchKernelGGL(k_rank<4>, grid, block, 0, s, mask, T, slice, ctx->d_pos); break;
        }
    }
    {
        mw_timed tm(ctx, MW_KERNEL_PLAN_GROUPS, s);
        hipLaunchKernelGGL(k_groups, dim3(1), dim3(kGroupsBlock), 0, s, mask, ctx->d_pos, T,
                           (uint64_t)ctx->row_bytes, perm, ctx->d_smask, desc, stats, ctx->d_hist, ctx->d_flags);
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

int32_t mw_launch_plan_allgather(mw_ctx *ctx, int64_t shard_bytes, mw_group_desc *desc,
                                 mw_send_stats *stats, hipStream_t s)
{
    hipLaunchKernelGGL(k_plan_allgather, dim3(1), dim3(256), 0, s, ctx->cfg.n_ranks, (uint64_t)shard_bytes,
                       desc, stats);
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}
