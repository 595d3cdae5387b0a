// Send-side plan kernels: destination bitmaps, (bitmap, token) ordering, multicast
// groups, descriptor table and byte accounting.
//
// Paper hooks: the bitmap is Section 4.1's metadata encoding (bit r <-> rank r, ranks
// from zero, a preconfigured id -> rank table); groups are discovered per batch because
// the space of destination sets cannot be provisioned in advance (Section 2.3.2,
// C(64,8) sets at EP=64/top-8); the accounting is Section 1's "one copy however many
// destinations" against one copy per destination.
//
// Two launches on the caller's stream, no host synchronisation:
//   k_rank    A workgroup owns 256 tokens and a slice of all tokens.  It builds the
//             bitmaps of both from the top-k ids (one lane per token, K rank bits ORed
//             into four 64-bit words; the slice goes to LDS), then every lane counts, over
//             the slice, the tokens whose (bitmap, index) is smaller than its own, and how
//             many carry an equal bitmap before / at-or-after it.  Slices are spread over
//             the whole chip and combined with one 64-bit integer atomic add per lane (a
//             sum, so the result does not depend on arrival order).  For the batch sizes
//             of a dispatch (<= 8k tokens) this beats a multi-pass radix sort of 256-bit
//             keys, which would be launch- and barrier-bound.  The workgroups of slice 0
//             also write the bitmaps out and turn 64 tokens' bitmaps into per-rank counts
//             with wavefront ballots and popcounts.
//   k_groups  Workgroup b owns packed rows [256 b, 256 b + 256): it finds their tokens
//             from the counts (predecessor count = packed row), writes perm, ranks the
//             group starts (tokens with no equal bitmap before them) and writes their
//             descriptors; a group's row count is the number of equal bitmaps.  Writing is
//             spread over many workgroups because one CU retires only about one cache line
//             of scattered stores per cycle.
// The count and histogram buffers are zero between plans: the k_groups workgroup that is the
// last to have read them clears them, so there is no clearing launch and no host-side state
// (a captured mw_plan can be replayed).
// Batches above 8192 tokens replace k_rank by k_chunk_sort + k_merge_rank (sorted chunks,
// ranks by binary search: T log T instead of T^2); batches of at most 256 tokens can take
// k_plan_pack, which plans and packs in one launch.
#include "mw_internal.h"
#include "mw_plan_dev.h"

namespace {

constexpr int kBlock = 256;
template <int W, bool kKeyed>
__global__ __launch_bounds__(kBlock) void k_rank(const int32_t *__restrict__ topk, int T, int K,
                                                 const int32_t *__restrict__ eslot, int E, int slice,
                                                 uint64_t *__restrict__ mask_out,
                                                 unsigned long long *__restrict__ cnt,
                                                 uint32_t *__restrict__ pstate)
{
    extern __shared__ uint64_t smask[];
    mw_rank_body<W, kKeyed>(topk, T, K, eslot, E, slice, mask_out, cnt, pstate, blockIdx.x, blockIdx.y, kBlock, smask);
}

// For very large batches the walk below (every workgroup over every token's counters) is
// itself T^2 / 256 loads.  This kernel turns the counters into arrays indexed by packed row
// first -- perm, the row's counters and a "group starts here" byte -- so that k_groups<true>
// only sums the start bytes in front of its rows.
__global__ __launch_bounds__(kBlock) void k_rows_from_counters(int T, const unsigned long long *__restrict__ cnt,
                                                               const uint32_t *__restrict__ pstate,
                                                               int32_t *__restrict__ perm,
                                                               unsigned long long *__restrict__ row_cnt,
                                                               unsigned char *__restrict__ row_start)
{
    const int t = blockIdx.x * kBlock + threadIdx.x;
    if (t >= T) return;
    const uint32_t N = min(pstate[kPsKept], (uint32_t)T), n_empty = (uint32_t)T - N;
    const unsigned long long c = cnt[t];
    if ((c >> 42) == 0) return;                               // empty bitmap
    const uint32_t p = (uint32_t)(c & kField) - n_empty;
    if (p >= N) return;
    perm[p] = t;
    row_cnt[p] = c;
    row_start[p] = ((c >> 21) & kField) == 0 ? 1 : 0;
}

template <bool kByRow>
__global__ __launch_bounds__(kBlock) void k_groups(const uint64_t *__restrict__ mask, int T, uint64_t row_bytes,
                                                   unsigned long long *__restrict__ cnt,
                                                   uint32_t *__restrict__ pstate,
                                                   int32_t *__restrict__ perm, mw_group_desc *__restrict__ desc,
                                                   mw_send_stats *__restrict__ stats,
                                                   const unsigned long long *__restrict__ row_cnt,
                                                   const unsigned char *__restrict__ row_start)
{
    __shared__ int32_t tok[kBlock];
    __shared__ unsigned long long tokc[kBlock];     // the token's counters, so they are not fetched again
    __shared__ uint32_t scratch[17];
    const int tid = threadIdx.x;
    const uint32_t N = min(pstate[kPsKept], (uint32_t)T), n_empty = (uint32_t)T - N;
    const uint32_t i0 = blockIdx.x * kBlock;

    // every workgroup walks all tokens' counters (coalesced): which of them land in its rows,
    // how many groups start before its first row, how many groups there are.  Sixteen counters
    // per lane are requested before the first is looked at: one memory round trip per 4096 tokens.
    uint32_t starts_before = 0, starts_total = 0;
    if constexpr (kByRow) {
        // rows in front of this workgroup's, sixteen start bytes per load (i0 is a multiple of 256);
        // the first workgroup also counts all groups for the statistics
        const u32x4 *sb = (const u32x4 *)row_start;
        auto ones = [](u32x4 v) { return (uint32_t)(__popc(v.x) + __popc(v.y) + __popc(v.z) + __popc(v.w)); };
        for (uint32_t q = tid; q < i0 / 16; q += kBlock) starts_before += ones(sb[q]);
        if (blockIdx.x == 0) {
            for (uint32_t r = tid; r < N; r += kBlock) starts_total += row_start[r];
        }
        if (i0 + tid < N) { tok[tid] = perm[i0 + tid]; tokc[tid] = row_cnt[i0 + tid]; }
    } else
    for (int t0 = 0; t0 < T; t0 += 16 * kBlock) {
        unsigned long long cc[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int t = t0 + u * kBlock + tid;
            cc[u] = t < T ? cnt[t] : 0ull;
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const unsigned long long c = cc[u];
            if ((c >> 42) == 0) continue;                         // empty bitmap (or past the end)
            const uint32_t p = (uint32_t)(c & kField) - n_empty;  // packed row of the token
            const uint32_t st = ((c >> 21) & kField) == 0 ? 1u : 0u;
            starts_total += st;
            starts_before += (st && p < i0) ? 1u : 0u;
            if (p - i0 < (uint32_t)kBlock && p < N) { tok[p - i0] = t0 + u * kBlock + tid; tokc[p - i0] = c; }
        }
    }
    uint32_t g_base, G;
    mw_block_exscan(starts_before, scratch, &g_base);
    mw_block_exscan(starts_total, scratch, &G);                // ends with a barrier: tok[] is complete

    const uint32_t i = i0 + tid;
    uint32_t st = 0;
    int32_t t = 0;
    unsigned long long c = 0;
    if (i < N) {
        t = tok[tid];
        if ((uint32_t)t >= (uint32_t)T) t = 0;      // (only counters corrupted by overlapping plans leave a row unclaimed)
        perm[i] = t;
        c = tokc[tid];
        st = ((c >> 21) & kField) == 0 ? 1u : 0u;
    }
    uint32_t local_total;
    const uint32_t g = g_base + mw_block_exscan(st, scratch, &local_total);
    if (st) {
        const uint64_t *m = mask + (size_t)t * MW_MASK_WORDS;
        mw_group_desc d;
        uint32_t nd = 0;
#pragma unroll
        for (int w = 0; w < MW_MASK_WORDS; ++w) { d.mask[w] = m[w]; nd += (uint32_t)__popcll(m[w]); }
        d.row_offset = i;
        d.row_count = (uint32_t)((c >> 42) & kField);          // equal bitmaps, this token included
        d.n_dest = nd;
        d.reserved0 = 0;
        if (g < (uint32_t)T) desc[g] = d;                      // (always, unless the counters were corrupted)
    }

    if (blockIdx.x == 0) {
        uint32_t dests = 0;
        for (int r = tid; r < MW_MAX_RANKS; r += kBlock) {
            const uint32_t h = pstate[r];
            stats->rows_per_dest[r] = h;
            dests += h;
        }
        uint32_t D;
        mw_block_exscan(dests, scratch, &D);
        if (tid == 0) {
            stats->n_rows = N;
            stats->n_groups = G;
            stats->multicast_bytes = (uint64_t)N * row_bytes;
            stats->unicast_bytes = (uint64_t)D * row_bytes;
            stats->error_flags = pstate[kPsFlags];
            stats->reserved0 = 0;
        }
    }

    // Leave the counters and the plan state zero for the next plan.  Nobody may clear them
    // while a workgroup still reads them: every workgroup reports when it has read all it
    // needs (its loads have returned: their values were used above), and the one that reports
    // last does the clearing (publication rules in mw_internal.h: the reports order every
    // workgroup's reads before the last one's stores).  The zeros are ordinary stores, read by
    // the next plan's kernels only.  With row-indexed arrays this kernel does not read the
    // counters at all, and every workgroup clears its own slice.
    __shared__ uint32_t i_am_last;
    mw_publish_barrier();
    if (tid == 0) i_am_last = mw_report(&pstate[kPsDone]) == gridDim.x - 1u ? 1u : 0u;
    if constexpr (kByRow) {
        if (i0 + tid < (uint32_t)T) cnt[i0 + tid] = 0;
    }
    __syncthreads();
    if (!i_am_last) return;
    if constexpr (!kByRow) {
        for (int z = tid; z < T; z += kBlock) cnt[z] = 0;
    }
    for (int r = tid; r < MW_PLAN_STATE_WORDS; r += kBlock) pstate[r] = 0;
}

__global__ __launch_bounds__(256) void k_plan_allgather(int R, uint64_t shard_bytes, mw_group_desc *desc,
                                                        mw_send_stats *stats)
{
    mw_plan_allgather_body(R, shard_bytes, desc, stats);
}

// Descriptor pair of a fragment split into a direct and a relayed segment (Section 5.2),
// in units of 16 bytes.
__global__ __launch_bounds__(256) void k_plan_allgather_split(int R, uint64_t shard_bytes, uint64_t direct_bytes,
                                                              mw_group_desc *desc, mw_send_stats *stats)
{
    const int tid = threadIdx.x;
    const uint32_t units = (uint32_t)(shard_bytes / 16), d_units = (uint32_t)(direct_bytes / 16);
    if (tid < MW_MAX_RANKS) stats->rows_per_dest[tid] = (tid < R) ? units : 0u;
    if (tid < 2) {
        mw_group_desc d;
#pragma unroll
        for (int w = 0; w < MW_MASK_WORDS; ++w) {
            const int lo = w * 64;
            d.mask[w] = (R >= lo + 64) ? ~0ull : (R > lo ? ((1ull << (R - lo)) - 1ull) : 0ull);
        }
        d.row_offset = tid == 0 ? 0u : d_units;
        d.row_count = tid == 0 ? d_units : units - d_units;
        d.n_dest = (uint32_t)R; d.reserved0 = 0;
        desc[tid] = d;
    }
    if (tid == 0) {
        stats->n_rows = units; stats->n_groups = 2;
        stats->multicast_bytes = direct_bytes * (uint64_t)R + (shard_bytes - direct_bytes);
        stats->unicast_bytes = shard_bytes * (uint64_t)R;
        stats->error_flags = 0; stats->reserved0 = 0;
    }
}

// Plan and pack of a decode-sized batch (at most kFusedMax tokens) in one launch.  The results
// are those of k_rank + k_groups + the packer; what changes is the latency: three dependent
// launches and two rounds of global atomics become one launch without any global scratch.
// Workgroup b moves packed row b.  To find that row's token every workgroup builds all
// bitmaps in LDS and ranks all tokens itself (one token per lane): for so few tokens that is
// cheaper than waiting for another workgroup's result.  The first workgroup also writes the
// bitmaps, perm and the descriptors, the last one the statistics.
constexpr int kFusedMax = MW_FUSED_MAX_TOKENS;
static_assert(kFusedMax == kBlock, "one token per lane");

// kKeyed (bitmaps of more than one word, top_k <= 8): the all-pairs walk compares short keys.
template <int W, bool kKeyed>
__global__ __launch_bounds__(kBlock) void k_plan_pack(const int32_t *__restrict__ topk, int T, int K,
                                                      const int32_t *__restrict__ eslot, int E,
                                                      const u32x4 *__restrict__ x, const u32x4 *__restrict__ scales,
                                                      int xc, int sc, int ns, uint64_t row_bytes,
                                                      uint64_t *__restrict__ mask_out, int32_t *__restrict__ perm,
                                                      mw_group_desc *__restrict__ desc, mw_send_stats *__restrict__ stats,
                                                      u32x4 *__restrict__ packed, int32_t *__restrict__ row_src_token,
                                                      int32_t *__restrict__ row_topk)
{
    __shared__ uint64_t smask[kFusedMax * W];
    __shared__ int32_t tok[kFusedMax];
    __shared__ uint32_t gstart[kFusedMax + 1];
    __shared__ uint32_t hist[MW_MAX_RANKS];
    __shared__ uint32_t scratch[18];
    __shared__ mw_short_key skey[kKeyed ? kFusedMax : 1];
    const mw_small_plan_lds lds = {smask, tok, gstart, hist, scratch, skey};
    const int t = threadIdx.x;
    const mw_small_plan_rank r = mw_small_plan_ranks<W, kKeyed>(topk, T, K, eslot, E, lds);

    const uint32_t i = blockIdx.x;
    if (i < r.N) {
        const int32_t tt = tok[i];
        const int n = xc + sc;
        for (int ch = t; ch < n; ch += kBlock) {
            const u32x4 v = (ch < xc) ? mw_ld16(x + (size_t)tt * xc + ch)
                                      : mw_ld16(scales + (size_t)tt * sc + (ch - xc));
            mw_st16(packed + (size_t)i * ns + ch, v);
        }
        if (t == 0) row_src_token[i] = tt;
        for (int j = t; j < K; j += kBlock) row_topk[(size_t)i * K + j] = topk[(size_t)tt * K + j];
    }
    const bool writes_plan = blockIdx.x == 0, writes_stats = blockIdx.x == gridDim.x - 1;
    if (!writes_plan && !writes_stats) return;
    mw_small_plan_finish<W>(r, T, row_bytes, mask_out, perm, desc, stats, lds, writes_plan, writes_stats);
}

// ---- ordering of large batches: sorted chunks, then ranks by binary search ------------------
// The all-pairs walk of k_rank costs T^2 compares: 84 us at 16 k tokens, 220 us at 32 k, 700 us
// at 64 k (one-word bitmaps; 120 / 335 / 1085 us with short keys).  This path: 48 / 68 / 97 us
// (53 / 74 / 107 us).  For large batches (switch points below) whose bitmaps have a 64-bit order-preserving key (one word, or
// short keys) the same counters are produced in T log T work:
//   k_chunk_sort   one workgroup per chunk of 1024 tokens: bitmaps, keys, a bitonic sort of
//                  (key, second word) pairs in LDS; the sorted chunk goes to the workspace.
//   k_merge_rank   workgroup (c, part), one lane per sorted element of chunk c: the chunks of its
//                  part are staged through LDS in turn and searched for the element's key.  A
//                  chunk of lower index contributes its keys <= mine (ties there come before me),
//                  one of higher index its keys < mine, my own chunk my sorted position.  The
//                  parts' sums meet in one 64-bit atomic add per element, as in k_rank.
// k_groups then runs unchanged on the counters.
// Second word of a sort element: (bit-0 flag << 31) | index inside the chunk for kept tokens;
// tokens without a destination and the padding of the last chunk carry the largest key and a
// second word above every kept token's, so they sort behind all kept tokens of the chunk.
constexpr int kChunk = 1024;
// Switch points, measured: one-word bitmaps tie at 8192 tokens (35 us either way); with short
// keys (a costlier compare per pair) sorting is ahead from about 6144 (8192 tokens: 39 against 48 us).
constexpr int kChunkFromOneWord = 8193, kChunkFromKeyed = 6145;
constexpr int kRowsFrom = 24576;       // from here k_groups works on row-indexed arrays
constexpr uint32_t kSecEmpty = 0x40000000u, kSecPad = 0x7fffffffu;

template <int W>
__global__ __launch_bounds__(kChunk) void k_chunk_sort(const int32_t *__restrict__ topk, int T, int K,
                                                       const int32_t *__restrict__ eslot, int E,
                                                       uint64_t *__restrict__ mask_out, uint32_t *__restrict__ pstate,
                                                       uint64_t *__restrict__ sort_key, uint32_t *__restrict__ sort_sec,
                                                       uint32_t *__restrict__ chunk_kept)
{
    __shared__ uint64_t sk[kChunk];
    __shared__ uint32_t ss[kChunk];
    __shared__ uint32_t hist[MW_MAX_RANKS];
    __shared__ uint32_t scratch[17];
    const int tid = threadIdx.x;
    const int t = blockIdx.x * kChunk + tid;
    if (tid < MW_MAX_RANKS) hist[tid] = 0;
    bool bad = false;
    uint64_t m[MW_MASK_WORDS] = {0, 0, 0, 0};
    if (t < T) {
        token_mask(topk + (size_t)t * K, K, eslot, E, m, bad);
        uint64_t *o = mask_out + (size_t)t * MW_MASK_WORDS;
#pragma unroll
        for (int q = 0; q < MW_MASK_WORDS; ++q) o[q] = m[q];
        if (bad) atomicOr(&pstate[kPsFlags], MW_FLAG_BAD_EXPERT);
    }
    const bool any = (m[0] | m[1] | m[2] | m[3]) != 0;
    uint64_t key = ~0ull;
    uint32_t sec = t < T ? (kSecEmpty | (uint32_t)tid) : kSecPad;
    if (any) {
        if constexpr (W == 1) { key = m[0]; sec = (uint32_t)tid; }
        else { const mw_short_key k = short_key(m); key = k.key; sec = (k.flag << 31) | (uint32_t)tid; }
    }
    uint32_t kept;
    mw_block_exscan(any ? 1u : 0u, scratch, &kept);        // (its barriers also publish the cleared histogram)
    if (tid == 0) {
        chunk_kept[blockIdx.x] = kept;
        if (kept) atomicAdd(&pstate[kPsKept], kept);
    }
    // rows per destination: one LDS atomic per set bit (at most top_k per token), then one
    // global atomic per rank and chunk
#pragma unroll
    for (int q = 0; q < W; ++q) {
        uint64_t left = m[q];
        while (left) {
            const int b = __ffsll((unsigned long long)left) - 1;
            left &= left - 1;
            atomicAdd(&hist[q * 64 + b], 1u);
        }
    }

    // Bitonic network with one element per lane.  Partners closer than 64 are in the same
    // wavefront and are exchanged in registers; the ten steps with partners 64 or more apart go
    // through LDS.  Position e keeps the smaller of the pair iff it is the lower position of an
    // ascending block or the upper position of a descending one.
    const int e = tid;
    for (int k = 2; k <= kChunk; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            uint64_t pk;
            uint32_t ps;
            if (j >= 64) {
                sk[e] = key; ss[e] = sec;
                mw_lds_barrier();
                pk = sk[e ^ j]; ps = ss[e ^ j];
                mw_lds_barrier();
            } else {
                pk = __shfl_xor(key, j, 64);
                ps = __shfl_xor(sec, j, 64);
            }
            const bool mine_after = key > pk || (key == pk && sec > ps);
            const bool keep_smaller = ((e & j) == 0) == ((e & k) == 0);
            if (mine_after == keep_smaller) { key = pk; sec = ps; }
        }
    }
    sort_key[(size_t)blockIdx.x * kChunk + tid] = key;
    sort_sec[(size_t)blockIdx.x * kChunk + tid] = sec;
    mw_lds_barrier();                                       // every lane's histogram atomics are done
    if (tid < MW_MAX_RANKS && hist[tid]) atomicAdd(&pstate[tid], hist[tid]);
}

template <int W>
__global__ __launch_bounds__(kChunk) void k_merge_rank(int T, int n_chunks, const uint32_t *__restrict__ pstate,
                                                       const uint64_t *__restrict__ sort_key,
                                                       const uint32_t *__restrict__ sort_sec,
                                                       const uint32_t *__restrict__ chunk_kept,
                                                       unsigned long long *__restrict__ cnt)
{
    __shared__ uint64_t sk[kChunk];
    __shared__ uint32_t ss[kChunk];
    __shared__ uint32_t kept_of[64];                       // 65536 tokens / 1024
    const int tid = threadIdx.x, c = blockIdx.x;
    const int per = (n_chunks + (int)gridDim.y - 1) / (int)gridDim.y;
    const int c_first = blockIdx.y * per, c_end = min(n_chunks, c_first + per);
    if (c_first >= c_end) return;
    if (tid < n_chunks) kept_of[tid] = chunk_kept[tid];
    const uint64_t key = sort_key[(size_t)c * kChunk + tid];
    const uint32_t sec = sort_sec[(size_t)c * kChunk + tid];
    const uint32_t flag = sec >> 31;
    const uint32_t n_empty = blockIdx.y == 0 ? (uint32_t)T - min(pstate[kPsKept], (uint32_t)T) : 0u;
    uint64_t nk = sort_key[(size_t)c_first * kChunk + tid];  // the part's first chunk, staged below
    uint32_t ns = sort_sec[(size_t)c_first * kChunk + tid];
    uint32_t c_lt = 0, c_eqb = 0, c_eqa = 0;
    // entries of the staged chunk that are below / not above my (key, flag)
    auto below = [&](uint32_t idx) -> bool {
        const uint64_t q = sk[idx];
        if constexpr (W == 1) return q < key;
        else return q < key || (q == key && (ss[idx] >> 31) < flag);
    };
    auto not_above = [&](uint32_t idx) -> bool {
        const uint64_t q = sk[idx];
        if constexpr (W == 1) return q <= key;
        else return q < key || (q == key && (ss[idx] >> 31) <= flag);
    };
    for (int c2 = c_first; c2 < c_end; ++c2) {
        mw_lds_barrier();                                   // the previous chunk has been searched
        sk[tid] = nk; ss[tid] = ns;
        mw_lds_barrier();
        if (c2 + 1 < c_end) {                               // next chunk in flight during the search
            nk = sort_key[(size_t)(c2 + 1) * kChunk + tid];
            ns = sort_sec[(size_t)(c2 + 1) * kChunk + tid];
        }
        const uint32_t n = kept_of[c2];
        uint32_t lb = 0, ub = 0;
#pragma unroll
        for (uint32_t st = kChunk; st >= 1; st >>= 1) {
            if (lb + st <= n && below(lb + st - 1)) lb += st;
            if (ub + st <= n && not_above(ub + st - 1)) ub += st;
        }
        c_lt += lb;
        if (c2 < c) c_eqb += ub - lb;
        else if (c2 > c) c_eqa += ub - lb;
        else { c_eqb += (uint32_t)tid - lb; c_eqa += ub - (uint32_t)tid; }
    }
    if ((uint32_t)tid < kept_of[c]) {
        const int t = c * kChunk + (int)(sec & 0x3fffffffu);
        const unsigned long long add = (unsigned long long)(c_lt + c_eqb + n_empty) |
                                       ((unsigned long long)c_eqb << 21) | ((unsigned long long)c_eqa << 42);
        if (add) atomicAdd(&cnt[t], add);
    }
}

}  // namespace

int32_t mw_launch_plan_allgather_split(mw_ctx *ctx, int64_t shard_bytes, int64_t direct_bytes, mw_group_desc *desc,
                                       mw_send_stats *stats, hipStream_t s)
{
    hipLaunchKernelGGL(k_plan_allgather_split, dim3(1), dim3(256), 0, s, ctx->cfg.n_ranks, (uint64_t)shard_bytes,
                       (uint64_t)direct_bytes, desc, stats);
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

int32_t mw_launch_plan(mw_ctx *ctx, const int32_t *topk, int32_t T, uint64_t *mask, int32_t *perm,
                       mw_group_desc *desc, mw_send_stats *stats, hipStream_t s)
{
    const int K = ctx->cfg.top_k, E = ctx->cfg.n_experts;
    // both start out zero: mw_ctx_create cleared them, every plan's last kernel clears them again
    unsigned long long *cnt = (unsigned long long *)ctx->d_plan_cnt;
    uint32_t *pstate = ctx->d_plan_state;
    const int tb = (T + kBlock - 1) / kBlock;
    const bool has_key = ctx->mask_words == 1 || K <= 8;
    if (T >= (ctx->mask_words == 1 ? kChunkFromOneWord : kChunkFromKeyed) && has_key && ctx->d_sort_key) {
        const int nc = (T + kChunk - 1) / kChunk;
        // split every chunk's walk over the other chunks into parts so that the grid fills the chip
        int parts = (2 * ctx->n_cu + nc - 1) / nc;
        if (parts > nc) parts = nc;
        if (parts < 1) parts = 1;
        mw_timed tm(ctx, MW_KERNEL_PLAN_RANK, s);
        if (ctx->mask_words == 1) {
            hipLaunchKernelGGL(k_chunk_sort<1>, dim3(nc), dim3(kChunk), 0, s, topk, T, K, ctx->d_eslot, E, mask,
                               pstate, ctx->d_sort_key, ctx->d_sort_sec, ctx->d_chunk_kept);
            hipLaunchKernelGGL(k_merge_rank<1>, dim3(nc, parts), dim3(kChunk), 0, s, T, nc, pstate,
                               ctx->d_sort_key, ctx->d_sort_sec, ctx->d_chunk_kept, cnt);
        } else {
            hipLaunchKernelGGL(k_chunk_sort<4>, dim3(nc), dim3(kChunk), 0, s, topk, T, K, ctx->d_eslot, E, mask,
                               pstate, ctx->d_sort_key, ctx->d_sort_sec, ctx->d_chunk_kept);
            hipLaunchKernelGGL(k_merge_rank<4>, dim3(nc, parts), dim3(kChunk), 0, s, T, nc, pstate,
                               ctx->d_sort_key, ctx->d_sort_sec, ctx->d_chunk_kept, cnt);
        }
    } else if (T > 0) {
        // split the predecessor walk into slices so that about 2 workgroups land on every CU when
        // a compare is one word (4 when it is a key and a flag: more compare work per pair); a
        // slice's bitmaps must fit in LDS.  Fewer, longer workgroups mean fewer atomics and less
        // disturbance of a bandwidth-bound kernel running beside the plan (the expander of the
        // batch before: 88 -> 85 us per launch with fp8 rows), at the same latency.
        const int per_cu = ctx->mask_words == 1 ? 2 : 4;
        int ns = (per_cu * ctx->n_cu + tb - 1) / tb;
        if (ns < 1) ns = 1;
        int slice = (T + ns - 1) / ns;
        if (slice < 64) slice = 64;
        if (slice > 1024) slice = 1024;
        ns = (T + slice - 1) / slice;
        const dim3 grid(tb, ns), block(kBlock);
        const int W = ctx->mask_words;
        const bool keyed = W > 1 && K <= 8;         // at most eight bits per bitmap: short keys
        const size_t lds = keyed ? (size_t)slice * sizeof(mw_short_key) : (size_t)slice * W * sizeof(uint64_t);
        mw_timed tm(ctx, MW_KERNEL_PLAN_RANK, s);
#define MW_RANK(W_, KEYED_)                                                                                 \
    hipLaunchKernelGGL((k_rank<W_, KEYED_>), grid, block, lds, s, topk, T, K, ctx->d_eslot, E, slice, mask, cnt, \
                       pstate)
        if (keyed) MW_RANK(4, true);
        else if (W == 1) MW_RANK(1, false);
        else if (W == 2) MW_RANK(2, false);
        else if (W == 3) MW_RANK(3, false);
        else MW_RANK(4, false);
#undef MW_RANK
    }
    {
        mw_timed tm(ctx, MW_KERNEL_PLAN_GROUPS, s);
        if (T >= kRowsFrom && ctx->d_row_cnt) {
            hipLaunchKernelGGL(k_rows_from_counters, dim3(tb), dim3(kBlock), 0, s, T, cnt, pstate, perm,
                               (unsigned long long *)ctx->d_row_cnt, ctx->d_row_start);
            hipLaunchKernelGGL(k_groups<true>, dim3(tb), dim3(kBlock), 0, s, mask, T, (uint64_t)ctx->row_bytes, cnt,
                               pstate, perm, desc, stats, (const unsigned long long *)ctx->d_row_cnt, ctx->d_row_start);
        } else {
            hipLaunchKernelGGL(k_groups<false>, dim3(tb > 0 ? tb : 1), dim3(kBlock), 0, s, mask, T,
                               (uint64_t)ctx->row_bytes, cnt, pstate, perm, desc, stats, nullptr, nullptr);
        }
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}


int32_t mw_launch_plan_pack(mw_ctx *ctx, const int32_t *topk, int32_t T, const void *x, const float *scales,
                            uint64_t *mask, int32_t *perm, mw_group_desc *desc, mw_send_stats *stats, void *packed,
                            int32_t *row_src_token, int32_t *row_topk, hipStream_t s)
{
    static_assert(MW_MAX_RANKS == kBlock, "one lane per rank in the statistics");
    const int xc = (int)(ctx->x_row_bytes / 16), sc = (int)(ctx->s_row_bytes / 16);
    const dim3 grid(T > 0 ? T : 1), block(kBlock);
    const int K = ctx->cfg.top_k, E = ctx->cfg.n_experts;
    const uint64_t rb = (uint64_t)ctx->row_bytes;
    mw_timed tm(ctx, MW_KERNEL_PLAN_PACK, s);
#define MW_FUSED(W, KEYED)                                                                                        \
    hipLaunchKernelGGL((k_plan_pack<W, KEYED>), grid, block, 0, s, topk, T, K, ctx->d_eslot, E, (const u32x4 *)x, \
                       (const u32x4 *)scales, xc, sc, (int)(ctx->row_stride / 16), rb, mask, perm, desc, stats,       \
                       (u32x4 *)packed, row_src_token,                                                           \
                       row_topk)
    const bool keyed = K <= 8;              // at most eight bits per bitmap: short keys
    switch (ctx->mask_words) {
    case 1: MW_FUSED(1, false); break;
    case 2: if (keyed) MW_FUSED(2, true); else MW_FUSED(2, false); break;
    case 3: if (keyed) MW_FUSED(3, true); else MW_FUSED(3, false); break;
    default: if (keyed) MW_FUSED(4, true); else MW_FUSED(4, false); break;
    }
#undef MW_FUSED
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
