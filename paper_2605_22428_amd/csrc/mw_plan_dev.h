// Device code of the plan that more than one translation unit uses: the bitmap builder, the
// short keys, the all-pairs ranking of one workgroup (k_rank, and the plan that rides along
// with the expander), and the second half of that riding plan.
#ifndef MW_PLAN_DEV_H_
#define MW_PLAN_DEV_H_

#include "mw_internal.h"

namespace {

constexpr uint64_t kField = 0x1fffffull;      // 21-bit fields of the packed counter
constexpr int kPsKept = 256, kPsFlags = 257, kPsDone = 258, kPsDone2 = 259;  // plan state words after the 256 histogram bins

// Destination bitmap of one token (Section 4.1): ids are fetched in independent batches.
__device__ __forceinline__ void token_mask(const int32_t *__restrict__ row, int K,
                                           const int32_t *__restrict__ eslot, int E, uint64_t m[MW_MASK_WORDS],
                                           bool &bad)
{
#pragma unroll
    for (int q = 0; q < MW_MASK_WORDS; ++q) m[q] = 0;
    for (int j0 = 0; j0 < K; j0 += 8) {
        int32_t e[8], s[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) e[u] = (j0 + u < K) ? row[j0 + u] : -1;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const bool ok = (uint32_t)e[u] < (uint32_t)E;
            bad |= (e[u] != -1 && !ok);
            s[u] = ok ? eslot[e[u]] : -1;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (s[u] < 0) continue;
            const int r = s[u] >> 16;
            const uint64_t bit = 1ull << (r & 63);
            const int w = r >> 6;
#pragma unroll
            for (int q = 0; q < MW_MASK_WORDS; ++q) m[q] |= (w == q) ? bit : 0ull;
        }
    }
}

// Order-preserving short key of a bitmap with at most eight bits set (always the case for
// top_k <= 8): the positions of the set bits, highest first, one byte each, zero-padded.
// Comparing bitmaps as 256-bit integers is comparing these lists lexicographically; the one
// collision -- "bit 0 set" against "no further bit" -- is resolved by bit 0 itself as a second,
// less significant component.  (key, flag) pairs are equal iff the bitmaps are.  One 64-bit and
// one 32-bit compare then replace four 64-bit ones in the all-pairs walk.
struct mw_short_key { uint64_t key; uint32_t flag; uint32_t pad; };     // 16 bytes: one LDS read
__device__ __forceinline__ mw_short_key short_key(const uint64_t m[MW_MASK_WORDS])
{
    uint64_t w[MW_MASK_WORDS] = {m[0], m[1], m[2], m[3]};
    mw_short_key k = {0ull, (uint32_t)(m[0] & 1ull), 0u};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int q = w[3] ? 3 : w[2] ? 2 : w[1] ? 1 : 0;
        uint64_t cur = 0;
#pragma unroll
        for (int z = 0; z < MW_MASK_WORDS; ++z) cur = (z == q) ? w[z] : cur;
        if (cur == 0) break;
        const int b = 63 - __clzll((long long)cur);
        k.key |= (uint64_t)(q * 64 + b) << (56 - 8 * j);
#pragma unroll
        for (int z = 0; z < MW_MASK_WORDS; ++z) w[z] = (z == q) ? (cur & ~(1ull << b)) : w[z];
    }
    return k;
}

// a < b for bitmaps of W words, word W - 1 most significant
template <int W>
__device__ __forceinline__ bool mask_less(const uint64_t *a, const uint64_t *b)
{
    bool lt = false, eq = true;
#pragma unroll
    for (int w = W - 1; w >= 0; --w) {
        lt = lt || (eq && a[w] < b[w]);
        eq = eq && (a[w] == b[w]);
    }
    return lt;
}

// ---- the whole plan of a small batch inside ONE workgroup of MW_FUSED_MAX_TOKENS lanes, one token
// per lane (Section 5.1, send module: task decomposition): bitmaps, the packed order, groups and
// statistics without any global scratch or any other workgroup.  Two halves, so that a caller can
// put work between them that needs only the order (mw_plan_pack moves its row there).
// LDS of the caller: smask [MW_FUSED_MAX_TOKENS * W] bitmaps, tok [..] token of packed row i,
// gstart [.. + 1] first packed row of group g, hist [MW_MAX_RANKS], scratch [18] (17 of the scan,
// one flag word), skey [MW_FUSED_MAX_TOKENS] short keys (kKeyed only).
struct mw_small_plan_lds {
    uint64_t *smask; int32_t *tok; uint32_t *gstart; uint32_t *hist; uint32_t *scratch; mw_short_key *skey;
};
struct mw_small_plan_rank {
    uint64_t m[MW_MASK_WORDS];     // this lane's token's bitmap
    uint32_t p, N;                 // its packed row (if kept), kept tokens
    bool any;                      // the token has a destination
};

// Bitmaps and the packed order: fills smask and tok; every barrier of the workgroup is inside.
// kKeyed (bitmaps of more than one word, top_k <= 8): the all-pairs walk compares short keys.
template <int W, bool kKeyed>
__device__ __forceinline__ mw_small_plan_rank mw_small_plan_ranks(const int32_t *__restrict__ topk, int T, int K,
                                                                  const int32_t *__restrict__ eslot, int E,
                                                                  const mw_small_plan_lds &l)
{
    const int t = threadIdx.x;
    const bool slot = t < MW_FUSED_MAX_TOKENS;      // (a wider workgroup's further lanes only take part in scans and barriers)
    mw_small_plan_rank r;
    bool bad = false;
#pragma unroll
    for (int w = 0; w < MW_MASK_WORDS; ++w) r.m[w] = 0;
    if (t < T) token_mask(topk + (size_t)t * K, K, eslot, E, r.m, bad);
    mw_short_key mk = {0ull, 0u, 0u};
    if (slot) {
#pragma unroll
        for (int w = 0; w < W; ++w) l.smask[t * W + w] = r.m[w];
        if constexpr (kKeyed) { mk = short_key(r.m); l.skey[t] = mk; }
        l.hist[t] = 0;
    }
    if (t == 0) l.scratch[17] = 0;
    r.any = (r.m[0] | r.m[1] | r.m[2] | r.m[3]) != 0;
    mw_block_exscan(r.any ? 1u : 0u, l.scratch, &r.N);          // its barriers also publish smask
    if (bad) atomicOr(&l.scratch[17], 1u);

    // Packed row of token t = number of kept tokens u with (bitmap, u) < (bitmap, t).  The
    // walk takes eight tokens at a time -- eight LDS reads in flight, then eight compares --
    // because a compare is a few cycles and an LDS round trip about a hundred.  Whether u < t
    // is the same for the whole wavefront except among its own 64 tokens: "bitmap <= mine"
    // before them, the full test among them, "bitmap < mine" after them.  Slots from T up to
    // the next multiple of eight hold empty bitmaps (their lanes wrote zeros); an empty bitmap is
    // below every kept one: all of them are counted and taken off again.
    const int T8 = slot ? (T + 7) & ~7 : 0;
    const int w0 = t & ~63, w1 = w0 + 64;
    uint32_t c = 0;
    for (int u0 = 0; u0 < T8; u0 += 8) {
        bool lt[8], eq[8];
        if constexpr (kKeyed) {
            mw_short_key q[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) q[k] = l.skey[u0 + k];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const bool keq = q[k].key == mk.key;
                lt[k] = q[k].key < mk.key || (keq && q[k].flag < mk.flag);
                eq[k] = keq && q[k].flag == mk.flag;
            }
        } else {
            uint64_t q[8][W];
#pragma unroll
            for (int k = 0; k < 8; ++k)
#pragma unroll
                for (int w = 0; w < W; ++w) q[k][w] = l.smask[(u0 + k) * W + w];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                lt[k] = mask_less<W>(q[k], r.m);
                eq[k] = !lt[k] && !mask_less<W>(r.m, q[k]);
            }
        }
        if (u0 + 8 <= w0) {                         // wave-uniform: all eight before this wave's tokens
#pragma unroll
            for (int k = 0; k < 8; ++k) c += (lt[k] || eq[k]) ? 1u : 0u;
        } else if (u0 >= w1) {                      // all eight after them
#pragma unroll
            for (int k = 0; k < 8; ++k) c += lt[k] ? 1u : 0u;
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) c += (lt[k] || (eq[k] && u0 + k < t)) ? 1u : 0u;
        }
    }
    r.p = c - ((uint32_t)T8 - r.N);
    if (r.any) l.tok[r.p] = t;                      // (any: t < T <= MW_FUSED_MAX_TOKENS)
    mw_lds_barrier();
    return r;
}

// Groups, descriptors, bitmaps and perm (writes_plan) and the statistics (writes_stats).
template <int W>
__device__ __forceinline__ void mw_small_plan_finish(const mw_small_plan_rank &r, int T, uint64_t row_bytes,
                                                     uint64_t *__restrict__ mask_out, int32_t *__restrict__ perm,
                                                     mw_group_desc *__restrict__ desc, mw_send_stats *__restrict__ stats,
                                                     const mw_small_plan_lds &l, bool writes_plan, bool writes_stats)
{
    const int t = threadIdx.x, lane = t & 63;
    const uint32_t N = r.N;
    // groups: lane i looks at packed row i; a group starts where the bitmap differs from the
    // row before
    bool start = false;
    if ((uint32_t)t < N) {
        const uint64_t *q = l.smask + l.tok[t] * W;
        start = t == 0 || mask_less<W>(l.smask + l.tok[t - 1] * W, q);
    }
    uint32_t G;
    const uint32_t g = mw_block_exscan(start ? 1u : 0u, l.scratch, &G);
    if (writes_plan) {
        if (start) l.gstart[g] = (uint32_t)t;
        if (t == 0) l.gstart[G] = N;
        if (t < T) {
            uint64_t *o = mask_out + (size_t)t * MW_MASK_WORDS;
#pragma unroll
            for (int q = 0; q < MW_MASK_WORDS; ++q) o[q] = r.m[q];
        }
        if (r.any) perm[r.p] = t;
        mw_lds_barrier();
        if (start) {
            const uint64_t *q = l.smask + l.tok[t] * W;
            mw_group_desc d;
            uint32_t nd = 0;
#pragma unroll
            for (int w = 0; w < MW_MASK_WORDS; ++w) {
                d.mask[w] = (w < W) ? q[w < W ? w : 0] : 0ull;
                nd += (uint32_t)__popcll(d.mask[w]);
            }
            d.row_offset = (uint32_t)t;
            d.row_count = l.gstart[g + 1] - (uint32_t)t;
            d.n_dest = nd;
            d.reserved0 = 0;
            desc[g] = d;
        }
    }
    if (writes_stats) {
        // rows per destination: a wavefront ballot of bit b over 64 tokens, popcounted, is the
        // number of those tokens that name rank 64 q + b; lane b keeps it
#pragma unroll
        for (int q = 0; q < W; ++q) {
            if (__ballot(r.m[q] != 0) == 0) continue;      // wave-uniform
            uint32_t mine = 0;
            for (int b = 0; b < 64; ++b) {
                const uint32_t n_b = (uint32_t)__popcll(__ballot((r.m[q] >> b) & 1ull));
                if (lane == b) mine = n_b;
            }
            if (mine) atomicAdd(&l.hist[q * 64 + lane], mine);
        }
        mw_lds_barrier();
        const uint32_t h = t < MW_MAX_RANKS ? l.hist[t] : 0u;
        if (t < MW_MAX_RANKS) stats->rows_per_dest[t] = h;
        uint32_t D;
        mw_block_exscan(h, l.scratch, &D);
        if (t == 0) {
            stats->n_rows = N;
            stats->n_groups = G;
            stats->multicast_bytes = (uint64_t)N * row_bytes;
            stats->unicast_bytes = (uint64_t)D * row_bytes;
            stats->error_flags = l.scratch[17] ? MW_FLAG_BAD_EXPERT : 0u;
            stats->reserved0 = 0;
        }
    }
}

// cnt[t] += (#smaller | #equal before << 21 | #equal at-or-after << 42) over this slice, where
// "smaller" means (bitmap, index) < (bitmap[t], t).  Empty bitmaps compare below every kept
// token; k_groups subtracts their number.  A kept token always has a non-zero third field.
// kKeyed (bitmaps of more than one word, top_k <= 8): the slice holds short keys instead of bitmaps.
// Workgroup (bx, by) of `bs` lanes: tokens [bx bs, bx bs + bs) against slice by.  kAgentMask:
// the bitmaps are written through to device scope, for a reader in the same launch.
template <int W, bool kKeyed, bool kAgentMask = false>
__device__ __forceinline__ void mw_rank_body(const int32_t *__restrict__ topk, int T, int K,
                                             const int32_t *__restrict__ eslot, int E, int slice,
                                             uint64_t *__restrict__ mask_out,
                                             unsigned long long *__restrict__ cnt,
                                             uint32_t *__restrict__ pstate, int bx, int by, int bs,
                                             uint64_t *smask /* LDS: [slice][W] bitmaps, or [slice] short keys */)
{
    mw_short_key *skey = (mw_short_key *)smask;
    const int tid = threadIdx.x, lane = tid & 63;
    const int u0 = by * slice, u1 = min(u0 + slice, T);
    bool bad = false, bad_slice = false;
    for (int u = u0 + tid; u < u1; u += bs) {
        uint64_t q[MW_MASK_WORDS];
        token_mask(topk + (size_t)u * K, K, eslot, E, q, bad_slice);
        if constexpr (kKeyed) {
            skey[u - u0] = short_key(q);
        } else {
#pragma unroll
            for (int w = 0; w < W; ++w) smask[(size_t)(u - u0) * W + w] = q[w];
        }
    }
    const int t = bx * bs + tid;
    uint64_t m[MW_MASK_WORDS] = {0, 0, 0, 0};
    if (t < T) token_mask(topk + (size_t)t * K, K, eslot, E, m, bad);
    const bool any = (m[0] | m[1] | m[2] | m[3]) != 0;

    if (by == 0) {
        if (t < T) {
            uint64_t *o = mask_out + (size_t)t * MW_MASK_WORDS;
#pragma unroll
            for (int q = 0; q < MW_MASK_WORDS; ++q) {
                if constexpr (kAgentMask) __hip_atomic_store(&o[q], m[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                else o[q] = m[q];
            }
            if (bad) atomicOr(&pstate[kPsFlags], MW_FLAG_BAD_EXPERT);
        }
        const uint32_t kept = (uint32_t)__popcll(__ballot(any));
        if (lane == 0 && kept) atomicAdd(&pstate[kPsKept], kept);
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
            if (mine) atomicAdd(&pstate[q * 64 + lane], mine);
        }
    }
    mw_lds_barrier();

    // Whether a slice token u comes before token t (u < t) is the same for the whole wavefront
    // except among the wavefront's own 64 tokens: before them an equal bitmap is an "equal
    // before", after them an "equal at or after", and only inside that range the index decides.
    uint32_t c_lt = 0, c_eqb = 0, c_eqa = 0;
    const int wt0 = bx * bs + (tid & ~63);
    const int ua = min(max(u0, wt0), u1), ub = min(max(u0, wt0 + 64), u1);
    auto walk = [&](int from, int to, uint32_t &n_lt, uint32_t &n_eq_before, uint32_t &n_eq_after, bool own) {
        if constexpr (kKeyed) {
            const mw_short_key mk = short_key(m);
#pragma unroll 4
            for (int u = from; u < to; ++u) {
                const mw_short_key q = skey[u - u0];               // same address in every lane: LDS broadcast
                const bool keq = q.key == mk.key;
                const bool lt = q.key < mk.key || (keq && q.flag < mk.flag);
                const bool eq = keq && q.flag == mk.flag;
                n_lt += lt ? 1u : 0u;
                if (own) { n_eq_before += (eq && u < t) ? 1u : 0u; n_eq_after += (eq && u >= t) ? 1u : 0u; }
                else n_eq_before += eq ? 1u : 0u;
            }
        } else {
#pragma unroll 4
            for (int u = from; u < to; ++u) {
                const uint64_t *q = smask + (size_t)(u - u0) * W;  // same address in every lane: LDS broadcast
                bool lt = false, eq = true;
#pragma unroll
                for (int w = W - 1; w >= 0; --w) {
                    const uint64_t qw = q[w];
                    lt = lt || (eq && qw < m[w]);
                    eq = eq && (qw == m[w]);
                }
                n_lt += lt ? 1u : 0u;
                if (own) { n_eq_before += (eq && u < t) ? 1u : 0u; n_eq_after += (eq && u >= t) ? 1u : 0u; }
                else n_eq_before += eq ? 1u : 0u;
            }
        }
    };
    uint32_t unused = 0;
    walk(u0, ua, c_lt, c_eqb, unused, false);      // slice tokens before the wavefront's own
    walk(ua, ub, c_lt, c_eqb, c_eqa, true);        // the wavefront's own tokens, if in this slice
    walk(ub, u1, c_lt, c_eqa, unused, false);      // slice tokens after them
    if (any) {
        const unsigned long long add = (unsigned long long)(c_lt + c_eqb) | ((unsigned long long)c_eqb << 21) |
                                       ((unsigned long long)c_eqa << 42);
        if (add) atomicAdd(&cnt[t], add);
    }
}


// AllGather plan (Section 5.2): one row, one group, every rank a destination.  One workgroup
// of any size.
__device__ __forceinline__ void mw_plan_allgather_body(int R, uint64_t shard_bytes, mw_group_desc *desc,
                                                       mw_send_stats *stats)
{
    const int tid = threadIdx.x;
    for (int r = tid; r < MW_MAX_RANKS; r += (int)blockDim.x) stats->rows_per_dest[r] = (r < R) ? 1u : 0u;
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

// ---- the plan that rides along with another launch -------------------------------------
// Everything the plan of one batch needs when it runs as extra workgroups of a launch that
// does something else (one kernel argument).  The launch's workgroups `wg` = 0 .. n_rank - 1
// rank (wg = by * tb + bx), the next n_finish ones turn the counters into perm, descriptors
// and statistics.
struct mw_plan_args {
    const int32_t *topk; int T, K, E; const int32_t *eslot;
    uint64_t *mask_out; unsigned long long *cnt; uint32_t *pstate;
    int32_t *perm; mw_group_desc *desc; mw_send_stats *stats; uint64_t row_bytes;
    int tb, ns, slice;
    uint32_t n_rank, n_finish, finish_rows, wait_limit;   // finish_rows: packed rows per finishing workgroup
};

__device__ __forceinline__ unsigned long long mw_ld_agent64(const unsigned long long *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t mw_ld_agent32(const uint32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Packed rows one finishing workgroup of `bs` lanes takes (a multiple of bs), and the LDS it
// needs for them in bytes (counters, tokens, 19 scratch words).  Every finishing workgroup reads
// all tokens' counters at device scope, which is not free beside a bandwidth-bound kernel: rows
// of 512 instead of 128 per workgroup took 3 us off the launch at 4096 tokens.
static inline uint32_t mw_plan_finish_rows(int bs) { return bs >= 512 ? (uint32_t)bs : 512u / (uint32_t)bs * (uint32_t)bs; }
static inline size_t mw_plan_finish_lds(int bs) { return 12u * (size_t)mw_plan_finish_rows(bs) + 19u * sizeof(uint32_t); }

// Clears the counters of `T` tokens and the plan state: what every plan expects to find.
__device__ __forceinline__ void mw_plan_clear(unsigned long long *cnt, uint32_t *pstate, uint32_t T)
{
    for (uint32_t z = threadIdx.x; z < T; z += blockDim.x) cnt[z] = 0;
    for (uint32_t r = threadIdx.x; r < MW_PLAN_STATE_WORDS; r += blockDim.x) pstate[r] = 0;
}

// Second half of a riding plan: finishing workgroup `fb` (of n_finish, `bs` lanes each) owns
// the packed rows [fb finish_rows, (fb + 1) finish_rows) -- what k_groups does in a launch of its own.  Here the
// rank workgroups are part of the SAME launch, so:
//  * it waits until all of them have reported (pstate[kPsDone] >= n_rank).  They come before
//    it in the launch's workgroup order, are dispatched before it, and wait for nothing, so
//    the wait ends; it is bounded all the same (wait_limit polls of ~0.5 us): past the bound
//    this workgroup gives the plan up -- it raises MW_FLAG_PLAN_TIMEOUT in the plan state and
//    writes none of its rows;
//  * what those workgroups wrote is read at device scope: the counters and the state are
//    device-scope atomics anyway, the bitmaps were written through (mw_rank_body<.., true>).
// The finishing workgroup that is last to be done (a second counter) writes the statistics: the
// plan's, or -- if ANY finishing workgroup gave up -- MW_FLAG_PLAN_TIMEOUT with zero rows.  It
// also leaves the counters and the state zero for the next plan.  After a give-up some rank
// workgroups may still be running, and nobody may clear under them: the last finishing workgroup
// then adds one more report to the rank workgroups' counter, and whoever brings that counter to
// n_rank + 1 -- this workgroup if all ranks were done after all, else the rank workgroup that
// reports last (mw_plan_ride) -- does the clearing.  Either way the launch leaves the context
// ready for its next plan.
// `lds`: mw_plan_finish_lds(bs) bytes.  kInFlight: counters a lane requests before it looks at the
// first (sixteen for the shortest chain; eight where the launch has to stay small in registers).
template <int kInFlight = 16>
__device__ __forceinline__ void mw_plan_finish_ride(const mw_plan_args &a, uint32_t fb, uint64_t *lds)
{
    const uint32_t tid = threadIdx.x, bs = blockDim.x;
    const uint32_t rpw = a.finish_rows;
    unsigned long long *tokc = (unsigned long long *)lds;          // [rpw] the row's counters
    int32_t *tok = (int32_t *)(lds + rpw);                         // [rpw] token of packed row i0 + k
    uint32_t *scratch = (uint32_t *)(lds + rpw) + rpw;             // [17] scans, [18] one-lane decisions
    const uint32_t T = (uint32_t)a.T;

    if (tid == 0) {
        uint32_t polls = 0;
        while (mw_ld_agent32(&a.pstate[kPsDone]) < a.n_rank && polls < a.wait_limit) {
            __builtin_amdgcn_s_sleep(16);
            ++polls;
        }
        const bool ready = mw_ld_agent32(&a.pstate[kPsDone]) >= a.n_rank;
        if (ready) mw_acquire_after_poll();
        else __hip_atomic_fetch_or(&a.pstate[kPsFlags], MW_FLAG_PLAN_TIMEOUT, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        scratch[18] = ready ? 1u : 0u;
    }
    __syncthreads();
    const bool ready = scratch[18] != 0;
    uint32_t N = 0, G = 0;
    if (ready) {
        N = min(mw_ld_agent32(&a.pstate[kPsKept]), T);
        const uint32_t n_empty = T - N;
        const uint32_t i0 = fb * rpw;
        for (uint32_t k = tid; k < rpw; k += bs) { tok[k] = 0; tokc[k] = 0; }   // (a row no token claims -- corrupted counters only -- reads token 0)
        mw_lds_barrier();
        // all tokens' counters: which land in this workgroup's rows, how many groups start before
        // its first row, how many groups there are (sixteen counters per lane in flight)
        uint32_t starts_before = 0, starts_total = 0;
        for (uint32_t t0 = 0; t0 < T; t0 += kInFlight * bs) {
            unsigned long long cc[kInFlight];
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                const uint32_t t = t0 + u * bs + tid;
                cc[u] = t < T ? mw_ld_agent64(&a.cnt[t]) : 0ull;
            }
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                const unsigned long long c = cc[u];
                if ((c >> 42) == 0) continue;                         // empty bitmap (or past the end)
                const uint32_t p = (uint32_t)(c & kField) - n_empty;  // packed row of the token
                const uint32_t st = ((c >> 21) & kField) == 0 ? 1u : 0u;
                starts_total += st;
                starts_before += (st && p < i0) ? 1u : 0u;
                if (p - i0 < rpw && p < N) { tok[p - i0] = (int32_t)(t0 + u * bs + tid); tokc[p - i0] = c; }
            }
        }
        uint32_t g_next;
        mw_block_exscan(starts_before, scratch, &g_next);
        mw_block_exscan(starts_total, scratch, &G);                // ends with a barrier: tok[] is complete

        for (uint32_t k0 = 0; k0 < rpw && i0 + k0 < N; k0 += bs) {  // (uniform bounds: every lane takes every turn)
            const uint32_t i = i0 + k0 + tid;
            uint32_t st = 0;
            int32_t t = 0;
            unsigned long long c = 0;
            if (i < N) {
                t = tok[k0 + tid];
                if ((uint32_t)t >= T) t = 0;
                a.perm[i] = t;
                c = tokc[k0 + tid];
                st = ((c >> 21) & kField) == 0 ? 1u : 0u;
            }
            uint32_t turn_total;
            const uint32_t g = g_next + mw_block_exscan(st, scratch, &turn_total);
            g_next += turn_total;
            if (st) {
                const unsigned long long *m = (const unsigned long long *)(a.mask_out + (size_t)t * MW_MASK_WORDS);
                mw_group_desc d;
                uint32_t nd = 0;
#pragma unroll
                for (int w = 0; w < MW_MASK_WORDS; ++w) { d.mask[w] = mw_ld_agent64(m + w); nd += (uint32_t)__popcll(d.mask[w]); }
                d.row_offset = i;
                d.row_count = (uint32_t)((c >> 42) & kField);
                d.n_dest = nd;
                d.reserved0 = 0;
                if (g < T) a.desc[g] = d;
            }
        }
    }
    // Done with the counters and the state (the loads above have returned: their values were used).
    mw_publish_barrier();
    if (tid == 0) scratch[18] = mw_report(&a.pstate[kPsDone2]) == a.n_finish - 1u ? 1u : 0u;
    __syncthreads();
    if (!scratch[18]) return;

    // ---- the last finishing workgroup: statistics, then the state left zero for the next plan
    const uint32_t flags = mw_ld_agent32(&a.pstate[kPsFlags]);
    const bool gave_up = (flags & MW_FLAG_PLAN_TIMEOUT) != 0;      // (then `ready` may be false here, too)
    uint32_t dests = 0;
    for (uint32_t r = tid; r < MW_MAX_RANKS; r += bs) {
        const uint32_t h = gave_up ? 0u : mw_ld_agent32(&a.pstate[r]);
        a.stats->rows_per_dest[r] = h;
        dests += h;
    }
    uint32_t D;
    mw_block_exscan(dests, scratch, &D);
    if (tid == 0) {
        a.stats->n_rows = gave_up ? 0u : N;
        a.stats->n_groups = gave_up ? 0u : G;
        a.stats->multicast_bytes = gave_up ? 0ull : (uint64_t)N * a.row_bytes;
        a.stats->unicast_bytes = gave_up ? 0ull : (uint64_t)D * a.row_bytes;
        a.stats->error_flags = flags;
        a.stats->reserved0 = 0;
        // after a give-up: one more report on the rank workgroups' counter; n_rank reports found
        // there means every rank workgroup is done and the clearing is this workgroup's
        scratch[18] = (!gave_up || mw_report(&a.pstate[kPsDone]) == a.n_rank) ? 1u : 0u;
    }
    __syncthreads();
    if (scratch[18]) mw_plan_clear(a.cnt, a.pstate, T);
}

// One riding plan workgroup.  `lds` is the launch's dynamic LDS: the slice's keys for a rank
// workgroup, mw_plan_finish_lds(bs) bytes for a finishing one.
template <int W, bool kKeyed, int kInFlight = 16>
__device__ __forceinline__ void mw_plan_ride(const mw_plan_args &a, uint32_t wg, uint64_t *lds)
{
    if (wg < a.n_rank) {
        mw_rank_body<W, kKeyed, true>(a.topk, a.T, a.K, a.eslot, a.E, a.slice, a.mask_out, a.cnt, a.pstate,
                                      (int)(wg % (uint32_t)a.tb), (int)(wg / (uint32_t)a.tb), (int)blockDim.x, lds);
        // Reports when all its lanes are done (publication rules in mw_internal.h).  A report
        // that finds n_rank others -- all rank workgroups and the extra one of finishing
        // workgroups that gave the plan up -- comes after everybody else is done with the
        // counters and the state: this workgroup clears them (see mw_plan_finish_ride).
        uint32_t *last = (uint32_t *)lds;
        mw_publish_barrier();
        if (threadIdx.x == 0) *last = mw_report(&a.pstate[kPsDone]) == a.n_rank ? 1u : 0u;
        __syncthreads();
        if (*last) mw_plan_clear(a.cnt, a.pstate, (uint32_t)a.T);
        return;
    }
    wg -= a.n_rank;
    if (wg < a.n_finish) mw_plan_finish_ride<kInFlight>(a, wg, lds);
}

}  // namespace

#endif
