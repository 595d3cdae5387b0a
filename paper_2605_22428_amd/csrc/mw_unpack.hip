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
//                 counts and one record per received row: source address, source token,
//                 peer and (expert slot, rank) pairs.  The workgroup that finishes last
//                 (device-scope counter) scans the counts into output bases, so no
//                 third launch and no grid-wide barrier is needed.
//   k_expand      small workgroups (a single wave for long cache-line-sized rows, one
//                 workgroup per row up to 10 KiB), each moving consecutive 16-byte chunks of
//                 one received row (rows beyond 32768 by striding): a chunk is read once with
//                 a streaming load and stored to each of the row's experts' slots.  Measured
//                 on MI355X, many small waves with a single load in flight each track the
//                 plain-copy ceiling, while fewer waves with deep per-lane unrolling fall
//                 10-30 % short, and a persistent grid loses ~5 % to the hardware dispatcher.
//                 This kernel moves ~all receive-side bytes and is bound by HBM bandwidth.
// Further entry points share these bodies: k_recv_index<true> reads per-row headers (packets),
// k_expand_index_next runs the expander with the next batch's index in the same launch, and
// k_combine is the expander's mirror image for the way back.
#include "mw_internal.h"
#include "mw_plan_dev.h"
#include "mw_pack_dev.h"

namespace {

constexpr int kIndexBlock = 1024;

__device__ __forceinline__ uint32_t ld_agent(const uint32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(uint32_t *p, uint32_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// One workgroup: exclusive scan of the (expert, peer) counts in output order, expert
// offsets, totals and flags.  `scratch` is LDS scan scratch of 17 words.  Every device-scope
// read that does not depend on another is issued before the first scan.
__device__ __forceinline__ void mw_finish_counts(const uint32_t *cnt, const uint32_t *addr_cnt, uint32_t *flags,
                                                 const uint32_t *row_base, uint32_t L, uint32_t P, int64_t out_cap,
                                                 uint32_t *base, int64_t *expert_offsets, mw_recv_stats *stats,
                                                 uint32_t *scratch)
{
    const uint32_t tid = threadIdx.x, nthr = blockDim.x;
    const uint32_t n_lp = L * P;
    uint32_t m = 0;
    for (uint32_t q = tid; q < P; q += nthr) m += ld_agent(&addr_cnt[q]);
    const uint32_t err = (tid == 0) ? ld_agent(&flags[1]) : 0u;
    const uint32_t row_base_total = (tid == 0) ? ld_agent(&row_base[P]) : 0u;
    uint32_t v_next = (tid < n_lp) ? ld_agent(&cnt[tid]) : 0u;
    uint32_t carry = 0;
    for (uint32_t f0 = 0; f0 < n_lp; f0 += nthr) {          // (expert, peer) order = output order
        const uint32_t f = f0 + tid, v = v_next;
        v_next = (f + nthr < n_lp) ? ld_agent(&cnt[f + nthr]) : 0u;
        uint32_t tot;
        const uint32_t ex = mw_block_exscan(v, scratch, &tot);
        if (f < n_lp) {
            base[f] = carry + ex;
            if (f % P == 0) expert_offsets[f / P] = (int64_t)(carry + ex);
        }
        carry += tot;
    }
    uint32_t m_tot;
    mw_block_exscan(m, scratch, &m_tot);
    if (tid == 0) {
        const uint32_t Q = carry;
        expert_offsets[L] = Q;
        stats->n_recv_rows = m_tot;
        stats->n_out_rows = Q;
        stats->error_flags = err | (((int64_t)Q > out_cap) ? MW_FLAG_OUT_CAPACITY : 0u);
        stats->n_rows_seen = row_base_total;
        st_agent(&flags[1], 0u);           // ready for the next unpack
        st_agent(&flags[2], 0u);
    }
}

// kPackets: the peers' regions hold packets (mw_recv_packets): every row is its own group and
// carries its bitmap, source token and expert ids in a header in front of it; `row_bytes` is
// then the distance between packets and `header_bytes` the payload's offset inside one.
// Everything the index of one batch needs (one kernel argument; the fused launch below carries
// it beside the expander's arguments).
struct mw_index_args {
    const void *peers; int P; const int32_t *eslot;
    int E, K, Kd, my_rank, L, Lc;
    uint32_t max_tokens, wpl, cap_rows; uint64_t row_bytes; uint32_t header_bytes; int64_t out_cap;
    uint32_t *cnt, *row_base, *addr_cnt; mw_row_rec *recs; mw_hit *hits; uint32_t *base;
    int64_t *expert_offsets; mw_recv_stats *stats; uint32_t *flags;
    uint32_t dedup;     // 1: of the rows of one peer that carry the same source token only one is taken
};

// The work of workgroup `p` (peer p) of the index; any workgroup size that is a multiple of 64.
// kCache: every thread keeps its first row (ids, rank-table entries, hits, record) in registers
// from the first request to the final store, which takes two memory round trips off the chain
// -- and about thirty registers; the launches that run the index beside the row movers and
// must stay small do without (kCache = false).
template <bool kPackets, bool kCache = true>
__device__ __forceinline__ void recv_index_body(
    const void *__restrict__ peers_v, int P, const int32_t *__restrict__ eslot,
    int E, int K, int Kd, int my_rank, int L, int Lc,
    uint32_t max_tokens, uint32_t wpl, uint32_t cap_rows, uint64_t row_bytes, uint32_t header_bytes, int64_t out_cap,
    uint32_t *cnt, uint32_t *row_base, uint32_t *addr_cnt, mw_row_rec *__restrict__ recs,
    mw_hit *__restrict__ hits, uint32_t *__restrict__ base, int64_t *__restrict__ expert_offsets,
    mw_recv_stats *__restrict__ stats, uint32_t *flags, const uint32_t dedup, const int p)
{
    extern __shared__ uint32_t lds[];
    uint32_t *addr = lds;                       // [wpl]      bit i: row i's group names this rank
    uint32_t *bits = addr + wpl;                // [Lc][wpl]  bit s of expert l: a row with source token s
    uint32_t *pre = bits + (size_t)Lc * wpl;    // [Lc][wpl]  running popcount before each word
    uint32_t *scratch = pre + (size_t)Lc * wpl; // [17] scan scratch, [17] "I am last", [18] addressed rows,
                                                // [19] rows of the peers before this one, [20] repeats dropped
    uint32_t *seen = scratch + 64;              // [wpl]      (dedup only) bit s: a row with source token s was taken

    const int tid = threadIdx.x, nthr = blockDim.x;
    mw_recv_peer pr;
    if constexpr (kPackets) {
        const mw_recv_packets q = ((const mw_recv_packets *)peers_v)[p];
        const char *first_packet = (const char *)q.packets;
        pr.desc = nullptr; pr.n_desc = q.n_rows; pr.n_rows = q.n_rows;
        pr.rows = first_packet + header_bytes;
        pr.row_src_token = (const int32_t *)(first_packet + 32);
        pr.row_topk = (const int32_t *)(first_packet + 40);
    } else {
        pr = ((const mw_recv_peer *)peers_v)[p];
    }
    auto ids_of = [&](uint32_t i) -> const int32_t * {
        if constexpr (kPackets) return (const int32_t *)((const char *)pr.row_topk + (size_t)i * row_bytes);
        else return pr.row_topk + (size_t)i * K;
    };
    auto token_of = [&](uint32_t i) -> uint32_t {
        if constexpr (kPackets) return (uint32_t)*(const int32_t *)((const char *)pr.row_src_token + (size_t)i * row_bytes);
        else return (uint32_t)pr.row_src_token[i];
    };
    auto rows_of_peer = [&](int q) -> uint32_t {
        if constexpr (kPackets) return ((const mw_recv_packets *)peers_v)[q].n_rows;
        else return ((const mw_recv_peer *)peers_v)[q].n_rows;
    };
    const uint32_t mine = min(pr.n_rows, max_tokens);
    // All experts' bitmaps fit in LDS at once (the usual case): marking is fused into the row
    // parse and the thread's first row never leaves its registers.
    const bool one_chunk = Lc >= L;
    uint32_t err = 0;

    // ---- everything that depends on the peer record alone is requested before the first wait:
    // the thread's first row (source token, first eight expert ids), its first descriptor and
    // the row counts of the peers before this one.  The kernel is a chain of memory round
    // trips; beside a bandwidth-bound kernel each of them takes several times longer.
    const int32_t *tk_c = ids_of((uint32_t)tid);
    uint32_t s_c = 0;
    int32_t e_c[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) e_c[u] = -1;
    if (kCache && (uint32_t)tid < mine) {
        s_c = token_of((uint32_t)tid);
#pragma unroll
        for (int u = 0; u < 8; ++u) if (u < K) e_c[u] = tk_c[u];
    }
    uint64_t dmask_c = 0;
    uint32_t doff_c = 0, dcnt_c = 0;       // packets: dcnt_c holds the header's id count
    if ((uint32_t)tid < pr.n_desc) {
        if constexpr (kPackets) {
            const char *hd = (const char *)pr.rows - header_bytes + (size_t)tid * row_bytes;
            dmask_c = ((const uint64_t *)hd)[my_rank >> 6];
            dcnt_c = *(const uint32_t *)(hd + 36);
        } else {
            const mw_group_desc *d = pr.desc + tid;
            dmask_c = d->mask[my_rank >> 6];
            doff_c = d->row_offset;
            dcnt_c = d->row_count;
        }
    }
    uint32_t part = 0;
    for (int q = tid; q < p; q += nthr) part += min(rows_of_peer(q), max_tokens);

    for (uint32_t w = tid; w < wpl; w += nthr) addr[w] = 0;
    if (dedup) for (uint32_t w = tid; w < wpl; w += nthr) seen[w] = 0;
    if (one_chunk) for (uint32_t w = tid; w < (uint32_t)L * wpl; w += nthr) bits[w] = 0;
    if (tid < 3) scratch[18 + tid] = 0;
    mw_lds_barrier();
    // at most 256 peers of at most 65536 rows, so 32 bits are enough; a sum, so order-free
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) part += __shfl_xor(part, d, 64);
    if ((tid & 63) == 0 && part) atomicAdd(&scratch[19], part);

    // rank-table entries of the first row's ids (second round trip)
    int32_t q_c[8];
    bool bad_c = false;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const bool ok = kCache && (uint32_t)e_c[u] < (uint32_t)E;
        bad_c |= (kCache && e_c[u] != -1 && !ok);
        q_c[u] = ok ? eslot[e_c[u]] : -1;
    }
    mw_lds_barrier();
    const uint32_t before = scratch[19];
    if (pr.n_rows > max_tokens || before + mine > cap_rows) err |= MW_FLAG_RECV_CAPACITY;
    const uint32_t rb = min(before, cap_rows);
    const uint32_t n_rows = min(before + mine, cap_rows) - rb;
    if (tid == 0) {
        row_base[p] = rb;
        if (p == P - 1) st_agent(&row_base[P], rb + n_rows);    // (also read by the last workgroup)
    }

    // ---- addressed rows: groups whose bitmap has this rank's bit
    if constexpr (kPackets) {
        // one bitmap per row: 32 consecutive rows are 32 consecutive lanes, so a ballot is the
        // word of the addressed-rows bitmap and its first lane stores it (no atomics)
        for (uint32_t g0 = 0; g0 < pr.n_desc; g0 += nthr) {
            const uint32_t g = g0 + tid;
            bool a = false;
            if (g < pr.n_desc) {
                uint64_t dm = dmask_c;
                uint32_t hk = dcnt_c;
                if (g != (uint32_t)tid) {
                    const char *hd = (const char *)pr.rows - header_bytes + (size_t)g * row_bytes;
                    dm = ((const uint64_t *)hd)[my_rank >> 6];
                    hk = *(const uint32_t *)(hd + 36);
                }
                a = (dm >> (my_rank & 63)) & 1ull;
                if (a && (hk != (uint32_t)K || g >= n_rows)) { err |= MW_FLAG_BAD_DESC; a = false; }
            }
            const uint64_t bal = __ballot(a);
            if ((tid & 31) == 0 && (g >> 5) < wpl) addr[g >> 5] = (uint32_t)(bal >> (tid & 32));
        }
    } else
    for (uint32_t g = tid; g < pr.n_desc; g += nthr) {
        uint64_t dm = dmask_c;
        uint64_t b = doff_c, e = (uint64_t)doff_c + dcnt_c;
        if (g != (uint32_t)tid) {
            const mw_group_desc *d = pr.desc + g;
            dm = d->mask[my_rank >> 6];
            b = d->row_offset; e = b + d->row_count;
        }
        if (!((dm >> (my_rank & 63)) & 1ull)) continue;
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
    mw_lds_barrier();
    {
        uint32_t a = 0;
        for (uint32_t w = tid; w < wpl; w += nthr) a += __popc(addr[w]);
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) a += __shfl_xor(a, d, 64);     // one LDS atomic per wave
        if ((tid & 63) == 0 && a) atomicAdd(&scratch[18], a);
    }

    // ---- per row: its distinct local experts in top-k order (duplicate ids count once).
    // Slot k of the row's hit slots receives expert k; the first eight also stay in f[].
    // A thread always handles the same rows (i = tid, tid + nthr, ...), so what it wrote for a
    // row it may read back later without a barrier.
    auto parse = [&](uint32_t i, bool first, int (&f)[8]) -> int {
        mw_hit *h = hits + (size_t)(rb + i) * Kd;
        const int32_t *tk = ids_of(i);
        int nk = 0;
        uint64_t seen = 0;                         // (kCache) local experts below 64 the row has named so far
        constexpr int kB = kCache ? 8 : 4;         // ids looked up together
        for (int j0 = 0; j0 < K; j0 += kB) {
            int32_t q[kB];
            if (first && j0 == 0) {
#pragma unroll
                for (int u = 0; u < kB; ++u) q[u] = q_c[u];
                if (bad_c) err |= MW_FLAG_BAD_EXPERT;
            } else {
                int32_t e[kB];
#pragma unroll
                for (int u = 0; u < kB; ++u) e[u] = (j0 + u < K) ? tk[j0 + u] : -1;
#pragma unroll
                for (int u = 0; u < kB; ++u) {
                    const bool ok = (uint32_t)e[u] < (uint32_t)E;
                    if (e[u] != -1 && !ok) err |= MW_FLAG_BAD_EXPERT;
                    q[u] = ok ? eslot[e[u]] : -1;
                }
            }
#pragma unroll
            for (int u = 0; u < kB; ++u) {
                if (q[u] < 0 || (q[u] >> 16) != my_rank) continue;
                const int le = q[u] & 0xffff;
                bool dup = false;
                if (kCache && le < 64) {               // one bit test instead of a walk over the row's experts
                    dup = (seen >> le) & 1ull;
                    seen |= 1ull << le;
                } else {
#pragma unroll
                    for (int k = 0; k < 8; ++k) dup |= (k < nk && f[k] == le);
                    for (int k = 8; k < nk; ++k) dup |= (h[k].le == le);
                }
                if (dup) continue;
#pragma unroll
                for (int k = 0; k < 8; ++k) if (k == nk) f[k] = le;
                h[nk++] = mw_hit{le, 0};
            }
        }
        return nk;
    };
    // sets the (expert, source token) bits of one row for the experts [le0, le0 + lc)
    auto mark = [&](uint32_t i, uint32_t s, int nk, const int (&f)[8], int le0, int lc) {
        const mw_hit *h = hits + (size_t)(rb + i) * Kd;
        for (int k = 0; k < nk; ++k) {
            int le = 0;
#pragma unroll
            for (int k8 = 0; k8 < 8; ++k8) if (k8 == k) le = f[k8];
            if (k >= 8) le = h[k].le;
            const int l = le - le0;
            if (l < 0 || l >= lc) continue;
            const uint32_t old = atomicOr(&bits[(uint32_t)l * wpl + (s >> 5)], 1u << (s & 31));
            if ((old >> (s & 31)) & 1u) err |= MW_FLAG_DUP_SRC_TOKEN;
        }
    };
    // a row's state as the parse left it in memory
    auto reload = [&](uint32_t i, uint32_t &s, int &nk, int (&f)[8]) {
        const mw_row_rec *rc = recs + rb + i;
        const mw_hit *h = hits + (size_t)(rb + i) * Kd;
        s = (uint32_t)rc->src_token; nk = rc->n_hits;
#pragma unroll
        for (int k = 0; k < 8; ++k) f[k] = (k < nk) ? h[k].le : 0;
    };

    int nk_c = 0;
    int f_c[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    mw_row_rec rec_c = {nullptr, 0, p, 0, 0, 0, 0};
    for (uint32_t i = tid; i < n_rows; i += nthr) {
        const bool first = kCache && i == (uint32_t)tid;
        mw_row_rec rec = {nullptr, 0, p, 0, 0, 0, 0};
        if ((addr[i >> 5] >> (i & 31)) & 1u) {
            const uint32_t s = first ? s_c : token_of(i);
            if (s >= max_tokens) {
                err |= MW_FLAG_BAD_SRC_TOKEN;
            } else if (dedup && ((atomicOr(&seen[s >> 5], 1u << (s & 31)) >> (s & 31)) & 1u)) {
                // a repeat of a row already taken (a relay forwarded without updating the metadata,
                // Section 4.1): dropped.  Repeats are copies, so which of them is taken does not matter.
                err |= MW_FLAG_DUPLICATE_DROPPED;
                atomicAdd(&scratch[20], 1u);
            } else {
                int f[8] = {0, 0, 0, 0, 0, 0, 0, 0};
                const int nk = parse(i, first, f);
                if (nk == 0) err |= MW_FLAG_NO_LOCAL_EXPERT;
                rec.src = (const char *)pr.rows + (size_t)i * row_bytes;
                rec.src_token = (int32_t)s;
                rec.n_hits = nk;
                rec.le0 = f[0];
                if (one_chunk) mark(i, s, nk, f, 0, L);
                if (first) {
                    nk_c = nk;
#pragma unroll
                    for (int k = 0; k < 8; ++k) f_c[k] = f[k];
                }
            }
        }
        if (first && one_chunk) rec_c = rec;     // written once its rank is known
        else recs[rb + i] = rec;
    }

    for (int le0 = 0; le0 < L; le0 += Lc) {
        const int lc = min(Lc, L - le0);
        const uint32_t n_words = (uint32_t)lc * wpl;
        if (!one_chunk) {
            if (le0 > 0) mw_lds_barrier();           // the previous chunk's ranks have been read
            for (uint32_t f = tid; f < n_words; f += nthr) bits[f] = 0;
            mw_lds_barrier();
            for (uint32_t i = tid; i < n_rows; i += nthr) {
                uint32_t s; int nk; int f[8];
                reload(i, s, nk, f);
                mark(i, s, nk, f, le0, lc);
            }
        }
        mw_lds_barrier();

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
        mw_lds_barrier();
        for (int l = tid; l < lc; l += nthr) {
            const uint32_t end = (l + 1 < lc) ? pre[(uint32_t)(l + 1) * wpl] : carry;
            st_agent(&cnt[(size_t)(le0 + l) * P + p], end - pre[(uint32_t)l * wpl]);
        }

        // stable rank of the row among the peer's rows for each of its experts in the chunk
        for (uint32_t i = tid; i < n_rows; i += nthr) {
            const bool cached = kCache && one_chunk && i == (uint32_t)tid;
            mw_hit *h = hits + (size_t)(rb + i) * Kd;
            uint32_t s = s_c; int nk = nk_c; int f[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) f[k] = f_c[k];
            if (!cached) reload(i, s, nk, f);
            for (int k = 0; k < nk; ++k) {
                int le = 0;
#pragma unroll
                for (int k8 = 0; k8 < 8; ++k8) if (k8 == k) le = f[k8];
                if (k >= 8) le = h[k].le;
                const int l = le - le0;
                if (l < 0 || l >= lc) continue;
                const uint32_t wi = (uint32_t)l * wpl + (s >> 5);
                const int32_t rk = (int32_t)(pre[wi] - pre[(uint32_t)l * wpl] + __popc(bits[wi] & ((1u << (s & 31)) - 1u)));
                if (k > 0) h[k].rank = rk;
                else if (cached) rec_c.rank0 = rk;
                else recs[rb + i].rank0 = rk;
            }
        }
    }
    if (kCache && one_chunk && (uint32_t)tid < n_rows) recs[rb + tid] = rec_c;
    if (L == 0) {
        // no expert lives here: any addressed row is inconsistent
        for (uint32_t w = tid; w < wpl; w += nthr) if (addr[w]) err |= MW_FLAG_NO_LOCAL_EXPERT;
    }
    if (err) __hip_atomic_fetch_or(&flags[1], err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (tid == 0) st_agent(&addr_cnt[p], scratch[18] - scratch[20]);    // (both complete: barriers in between)

    // ---- the workgroup that finishes last turns the counts into output bases ----------
    // Everything the last workgroup reads (counts, addressed-row counts, flags) is written and
    // read with device-scope atomics, and every workgroup reports through one counter when all
    // its lanes are done (publication rules in mw_internal.h); the workgroup whose report is the
    // P-th has thereby acquired what all the others released.  The row records and hit slots,
    // written with ordinary stores, are read by the next kernel only.
    mw_publish_barrier();
    if (tid == 0) scratch[17] = mw_report(&flags[2]) == (uint32_t)P - 1u ? 1u : 0u;
    __syncthreads();
    if (!scratch[17]) return;
    mw_finish_counts(cnt, addr_cnt, flags, row_base, (uint32_t)L, (uint32_t)P, out_cap, base, expert_offsets, stats,
                     scratch);
}

template <bool kPackets, bool kCache = true>
__device__ __forceinline__ void recv_index_of(const mw_index_args &a, int p)
{
    recv_index_body<kPackets, kCache>(a.peers, a.P, a.eslot, a.E, a.K, a.Kd, a.my_rank, a.L, a.Lc, a.max_tokens, a.wpl,
                              a.cap_rows, a.row_bytes, a.header_bytes, a.out_cap, a.cnt, a.row_base, a.addr_cnt, a.recs,
                              a.hits, a.base, a.expert_offsets, a.stats, a.flags, a.dedup, p);
}

template <bool kPackets>
__global__ __launch_bounds__(kIndexBlock) void k_recv_index(const mw_index_args a)
{
    recv_index_of<kPackets>(a, blockIdx.x);
}

// ---- the index of a SMALL batch in one workgroup ------------------------------------------------
// With a few hundred received rows the index above is nothing but its chain of memory round
// trips, and three of them -- the wait for a workgroup's stores, its report, the last workgroup's
// reads of everybody's counts -- exist only because the peers are spread over workgroups.  Here one
// workgroup handles all peers: records, then descriptors beside the rows' tokens and ids, then the
// rank table, and the rest is LDS.  One bitmap over (expert, peer, source token) in output order
// holds a bit per delivered (row, expert) pair; a running popcount over it is every pair's output
// row at once: expert offsets, per-(expert, peer) bases and ranks are read off the same array.
// Same outputs and flags as recv_index_body + mw_finish_counts (records, not packets; no
// de-duplication); cnt and addr_cnt, which only those two exchange, are not written.
// LDS words: see mw_small_index_lds_words.  P <= blockDim.x.
constexpr int kSmallBlock = MW_FUSED_MAX_TOKENS;      // token slots of the one-workgroup plan
constexpr int kSmallLanes = 512;                      // lanes of the small launches' workgroups (index: one or two rows a lane up to 1024 rows)

static inline size_t mw_small_index_lds_words(int P, int L, uint32_t wpl, uint32_t max_tokens, uint32_t cap_rows)
{
    const uint64_t m_max = (uint64_t)P * max_tokens < cap_rows ? (uint64_t)P * max_tokens : cap_rows;
    const size_t wa = (size_t)((m_max + 31) / 32), n_w = (size_t)L * (size_t)P * wpl;
    return 10 * (size_t)P + 3 * ((size_t)P + 1) + wa + 2 * n_w + 1 + 24;
}

// kSmallRows: rows (and descriptors) a lane keeps in registers; further ones go through memory.
template <int kSmallRows>
__device__ __forceinline__ void recv_index_small(const mw_index_args &a, uint32_t *lds)
{
    const uint32_t tid = threadIdx.x, nthr = blockDim.x;
    const uint32_t P = (uint32_t)a.P, L = (uint32_t)a.L, wpl = a.wpl, K = (uint32_t)a.K, Kd = (uint32_t)a.Kd;
    const uint32_t E = (uint32_t)a.E, my_rank = (uint32_t)a.my_rank, max_tokens = a.max_tokens, cap_rows = a.cap_rows;
    const uint64_t m_max = (uint64_t)P * max_tokens < cap_rows ? (uint64_t)P * max_tokens : cap_rows;
    const uint32_t wa = (uint32_t)((m_max + 31) / 32), n_w = L * P * wpl;
    mw_recv_peer *pinfo = (mw_recv_peer *)lds;          // [P]      the peers' records
    uint32_t *rbase = lds + 10 * P;                     // [P + 1]  first row (over all peers) of peer q
    uint32_t *nrow = rbase + P + 1;                     // [P + 1]  rows taken from peer q
    uint32_t *dbase = nrow + P + 1;                     // [P + 1]  first descriptor (over all peers) of peer q
    uint32_t *addr = dbase + P + 1;                     // [wa]     bit r: row r's group names this rank
    uint32_t *bits = addr + wa;                         // [n_w]    (expert, peer, source token) in output order
    uint32_t *pre = bits + n_w;                         // [n_w + 1] running popcount in front of each word
    uint32_t *scratch = pre + n_w + 1;                  // [17] scan scratch, [17] flags, [18] addressed rows
    const mw_recv_peer *peers = (const mw_recv_peer *)a.peers;
    uint32_t err = 0;

    // ---- round trip 1: the records
    uint32_t nq = 0, dq = 0;
    if (tid < P) {
        const mw_recv_peer pr = peers[tid];
        pinfo[tid] = pr;
        nq = min(pr.n_rows, max_tokens);
        dq = min(pr.n_desc, 65536u);
        if (pr.n_rows > max_tokens) err |= MW_FLAG_RECV_CAPACITY;
    }
    for (uint32_t w = tid; w < wa; w += nthr) addr[w] = 0;
    for (uint32_t w = tid; w < n_w; w += nthr) bits[w] = 0;
    if (tid < 2) scratch[17 + tid] = 0;
    uint32_t tot;
    const uint32_t before = mw_block_exscan(nq, scratch, &tot);
    const uint32_t dbefore = mw_block_exscan(dq, scratch, &tot);
    if (tid < P) {
        if (before + nq > cap_rows) err |= MW_FLAG_RECV_CAPACITY;
        const uint32_t rb = min(before, cap_rows), nr = min(before + nq, cap_rows) - rb;
        rbase[tid] = rb; nrow[tid] = nr; dbase[tid] = dbefore;
        a.row_base[tid] = rb;
        if (tid == P - 1) { rbase[P] = rb + nr; dbase[P] = dbefore + dq; a.row_base[P] = rb + nr; }
    }
    mw_lds_barrier();
    const uint32_t M = rbase[P], D = dbase[P];
    // the peer whose range [base[q], base[q + 1]) holds v (ranges may be empty; v < base[P])
    auto peer_of = [&](const uint32_t *base, uint32_t v) -> uint32_t {
        uint32_t lo = 0, hi = P;                        // base[lo] <= v < base[hi]
        while (hi - lo > 1) {
            const uint32_t mid = (lo + hi) >> 1;
            if (base[mid] <= v) lo = mid; else hi = mid;
        }
        return lo;
    };

    // ---- round trip 2: the lane's first rows (source token, first eight ids) and descriptors, all
    // requested together; their peers by four binary searches side by side
    uint32_t q_r[kSmallRows], i_r[kSmallRows], s_r[kSmallRows];
    int32_t e_r[kSmallRows][8];
    uint32_t q_d[kSmallRows];
    uint64_t dm_d[kSmallRows];
    uint32_t off_d[kSmallRows], cnt_d[kSmallRows];
    {
        uint32_t lo[2 * kSmallRows], hi[2 * kSmallRows];
#pragma unroll
        for (int c = 0; c < 2 * kSmallRows; ++c) { lo[c] = 0; hi[c] = P; }
        // ceil(log2 P) steps: an interval of one entry stays as it is (mid == lo, and base[lo] <= v)
        for (uint32_t span = P; span > 1; span = (span + 1) >> 1) {
#pragma unroll
            for (int c = 0; c < 2 * kSmallRows; ++c) {
                const uint32_t v = tid + (uint32_t)(c % kSmallRows) * nthr, mid = (lo[c] + hi[c]) >> 1;
                const uint32_t bm = (c < kSmallRows ? rbase : dbase)[mid];
                if (bm <= v) lo[c] = mid; else hi[c] = mid;
            }
        }
#pragma unroll
        for (int j = 0; j < kSmallRows; ++j) { q_r[j] = lo[j]; q_d[j] = lo[kSmallRows + j]; }
    }
#pragma unroll
    for (int j = 0; j < kSmallRows; ++j) {
        const uint32_t r = tid + (uint32_t)j * nthr;
        i_r[j] = 0; s_r[j] = 0;
#pragma unroll
        for (int u = 0; u < 8; ++u) e_r[j][u] = -1;
        if (r < M) {
            i_r[j] = r - rbase[q_r[j]];
            const mw_recv_peer &pr = pinfo[q_r[j]];
            s_r[j] = (uint32_t)pr.row_src_token[i_r[j]];
            const int32_t *tk = pr.row_topk + (size_t)i_r[j] * K;
#pragma unroll
            for (int u = 0; u < 8; ++u) if ((uint32_t)u < K) e_r[j][u] = tk[u];
        }
        dm_d[j] = 0; off_d[j] = 0; cnt_d[j] = 0;
        if (r < D) {
            const mw_group_desc *dd = pinfo[q_d[j]].desc + (r - dbase[q_d[j]]);
            dm_d[j] = dd->mask[my_rank >> 6]; off_d[j] = dd->row_offset; cnt_d[j] = dd->row_count;
        }
    }
    // ---- round trip 3: rank-table entries of those ids, requested before the descriptors are looked at
    int32_t t_r[kSmallRows][8];
    bool bad_r[kSmallRows];
#pragma unroll
    for (int j = 0; j < kSmallRows; ++j) {
        bad_r[j] = false;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const bool ok = (uint32_t)e_r[j][u] < E;
            bad_r[j] |= (e_r[j][u] != -1 && !ok);
            t_r[j][u] = ok ? a.eslot[e_r[j][u]] : -1;
        }
    }
    // addressed rows: the row ranges of the groups whose bitmap has this rank's bit
    auto address = [&](uint32_t q, uint64_t dm, uint64_t b, uint64_t cnt) {
        const uint64_t e = b + cnt;
        if (!((dm >> (my_rank & 63u)) & 1ull)) return;
        if (e > nrow[q]) { err |= MW_FLAG_BAD_DESC; return; }
        if (e <= b) return;
        const uint64_t gb = rbase[q] + b, ge = rbase[q] + e;        // over all peers
        for (uint64_t w = gb >> 5; w <= ((ge - 1) >> 5); ++w) {
            const uint64_t wlo = w << 5;
            uint32_t m = 0xffffffffu;
            if (gb > wlo) m &= 0xffffffffu << (gb - wlo);
            if (ge < wlo + 32) m &= 0xffffffffu >> (wlo + 32 - ge);
            atomicOr(&addr[w], m);
        }
    };
#pragma unroll
    for (int j = 0; j < kSmallRows; ++j)
        if (tid + (uint32_t)j * nthr < D) address(q_d[j], dm_d[j], off_d[j], cnt_d[j]);
    for (uint32_t d = tid + kSmallRows * nthr; d < D; d += nthr) {
        const uint32_t q = peer_of(dbase, d);
        const mw_group_desc *dd = pinfo[q].desc + (d - dbase[q]);
        address(q, dd->mask[my_rank >> 6], dd->row_offset, dd->row_count);
    }
    mw_lds_barrier();
    {
        uint32_t n = 0;
        for (uint32_t w = tid; w < wa; w += nthr) n += __popc(addr[w]);
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) n += __shfl_xor(n, d, 64);
        if ((tid & 63u) == 0 && n) atomicAdd(&scratch[18], n);
        if (L == 0) for (uint32_t w = tid; w < wa; w += nthr) if (addr[w]) err |= MW_FLAG_NO_LOCAL_EXPERT;
    }

    // ---- per row: its distinct local experts in top-k order (duplicate ids count once; at most 64
    // local experts here, so "seen before" is one bit test); one bit per (expert, peer, source token).
    // Slot k of the row's hit slots receives expert k; the first eight also stay in `les`, a byte each.
    // `cached`: the row's token and the rank-table entries of its first eight ids are in registers.
    auto parse_mark = [&](uint32_t r, uint32_t q, uint32_t i, uint32_t s, bool cached, const int32_t (&tc)[8], bool badc,
                          mw_row_rec &rec, uint64_t &les) {
        rec = mw_row_rec{nullptr, 0, (int32_t)q, 0, 0, 0, 0};
        les = 0;
        if (!((addr[r >> 5] >> (r & 31u)) & 1u)) return;
        if (s >= max_tokens) { err |= MW_FLAG_BAD_SRC_TOKEN; return; }
        const mw_recv_peer &pr = pinfo[q];
        mw_hit *h = a.hits + (size_t)r * Kd;
        const int32_t *tk = pr.row_topk + (size_t)i * K;
        uint64_t seen = 0;
        int nk = 0;
        for (uint32_t j0 = 0; j0 < K; j0 += 8) {
            int32_t t8[8];
            if (cached && j0 == 0) {
#pragma unroll
                for (int u = 0; u < 8; ++u) t8[u] = tc[u];
                if (badc) err |= MW_FLAG_BAD_EXPERT;
            } else {
                int32_t e8[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) e8[u] = (j0 + u < K) ? tk[j0 + u] : -1;
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const bool ok = (uint32_t)e8[u] < E;
                    if (e8[u] != -1 && !ok) err |= MW_FLAG_BAD_EXPERT;
                    t8[u] = ok ? a.eslot[e8[u]] : -1;
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (t8[u] < 0 || (uint32_t)(t8[u] >> 16) != my_rank) continue;
                const uint32_t le = (uint32_t)t8[u] & 63u;             // (L <= 64)
                if ((seen >> le) & 1ull) continue;
                seen |= 1ull << le;
                if (nk < 8) les |= (uint64_t)le << (8 * nk);
                h[nk++] = mw_hit{(int32_t)le, 0};
            }
        }
        // the row's bits: every atomic issued before the first result is looked at
        {
            uint32_t was[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                was[k] = 0;
                if (k < nk) {
                    const uint32_t le = (uint32_t)(les >> (8 * k)) & 0xffu;
                    was[k] = atomicOr(&bits[(le * P + q) * wpl + (s >> 5)], 1u << (s & 31u));
                }
            }
            uint32_t any_was = 0;
#pragma unroll
            for (int k = 0; k < 8; ++k) any_was |= was[k];
            for (int k = 8; k < nk; ++k) any_was |= atomicOr(&bits[((uint32_t)h[k].le * P + q) * wpl + (s >> 5)], 1u << (s & 31u));
            if ((any_was >> (s & 31u)) & 1u) err |= MW_FLAG_DUP_SRC_TOKEN;
        }
        if (nk == 0) err |= MW_FLAG_NO_LOCAL_EXPERT;
        rec.src = (const char *)pr.rows + (size_t)i * a.row_bytes;
        rec.src_token = (int32_t)s;
        rec.n_hits = nk;
        rec.le0 = (int32_t)(les & 0xffu);
    };
    mw_row_rec rec_r[kSmallRows];
    uint64_t les_r[kSmallRows];
#pragma unroll
    for (int j = 0; j < kSmallRows; ++j) {
        rec_r[j] = mw_row_rec{nullptr, 0, 0, 0, 0, 0, 0};
        les_r[j] = 0;
        const uint32_t r = tid + (uint32_t)j * nthr;
        if (r < M) parse_mark(r, q_r[j], i_r[j], s_r[j], true, t_r[j], bad_r[j], rec_r[j], les_r[j]);
    }
    for (uint32_t r = tid + kSmallRows * nthr; r < M; r += nthr) {        // further rows: through memory
        const uint32_t q = peer_of(rbase, r), i = r - rbase[q];
        const uint32_t s = (uint32_t)pinfo[q].row_src_token[i];
        const int32_t none[8] = {-1, -1, -1, -1, -1, -1, -1, -1};
        mw_row_rec rec;
        uint64_t les;
        parse_mark(r, q, i, s, false, none, false, rec, les);
        a.recs[r] = rec;
    }
    mw_lds_barrier();

    // ---- running popcount over the bitmap: consecutive words per lane, one scan of the lanes' sums
    {
        const uint32_t per = (n_w + nthr - 1) / nthr;
        const uint32_t w0 = min(n_w, tid * per), w1 = min(n_w, w0 + per);
        uint32_t sum = 0;
        for (uint32_t w = w0; w < w1; ++w) sum += __popc(bits[w]);
        uint32_t run = mw_block_exscan(sum, scratch, &tot);
        for (uint32_t w = w0; w < w1; ++w) { pre[w] = run; run += __popc(bits[w]); }
        if (tid == 0) pre[n_w] = tot;
    }
    mw_lds_barrier();
    const uint32_t Q = pre[n_w];
    for (uint32_t f = tid; f < L * P; f += nthr) {
        const uint32_t b = pre[f * wpl];
        a.base[f] = b;
        if (f % P == 0) a.expert_offsets[f / P] = (int64_t)b;
    }
    // ---- ranks: output row of (row, expert) minus the base of its (expert, peer)
    auto rank_of = [&](uint32_t q, uint32_t s, int le) -> int32_t {
        const uint32_t w0 = ((uint32_t)le * P + q) * wpl, wi = w0 + (s >> 5);
        return (int32_t)(pre[wi] + __popc(bits[wi] & ((1u << (s & 31u)) - 1u)) - pre[w0]);
    };
#pragma unroll
    for (int j = 0; j < kSmallRows; ++j) {
        const uint32_t r = tid + (uint32_t)j * nthr;
        if (r >= M) continue;
        mw_hit *h = a.hits + (size_t)r * Kd;
        const int nk = rec_r[j].n_hits;
        for (int k = 0; k < nk; ++k) {
            const int le = k < 8 ? (int)((les_r[j] >> (8 * k)) & 0xffu) : h[k].le;
            const int32_t rk = rank_of(q_r[j], s_r[j], le);
            if (k == 0) rec_r[j].rank0 = rk; else h[k].rank = rk;
        }
        a.recs[r] = rec_r[j];
    }
    for (uint32_t r = tid + kSmallRows * nthr; r < M; r += nthr) {
        mw_row_rec *rc = a.recs + r;
        mw_hit *h = a.hits + (size_t)r * Kd;
        const int nk = rc->n_hits;
        const uint32_t q = (uint32_t)rc->peer, s = (uint32_t)rc->src_token;
        for (int k = 0; k < nk; ++k) {
            const int32_t rk = rank_of(q, s, h[k].le);
            if (k == 0) rc->rank0 = rk; else h[k].rank = rk;
        }
    }
    if (err) atomicOr(&scratch[17], err);
    mw_lds_barrier();
    if (tid == 0) {
        a.expert_offsets[L] = (int64_t)Q;
        a.stats->n_recv_rows = scratch[18];
        a.stats->n_out_rows = Q;
        a.stats->error_flags = scratch[17] | (((int64_t)Q > a.out_cap) ? MW_FLAG_OUT_CAPACITY : 0u);
        a.stats->n_rows_seen = M;
    }
}

// blockIdx.x selects a segment of blockDim.x chunks of the row; blockIdx.y walks rows.  All
// index reads are wave-uniform (scalar loads).  The dependent chain in front of a row's
// payload is what a one-shot workgroup cannot hide, so it is kept to two steps: the row
// record and the row count are fetched together, then the payload load and the lookup of
// the first output position are issued together; the position is there long before the
// payload is.
// g_first / g_stride: the first row of this workgroup and the distance to its next one.
__device__ __forceinline__ void expand_body(
    const mw_row_rec *__restrict__ recs, const mw_hit *__restrict__ hits, const uint32_t *__restrict__ base,
    const uint32_t *__restrict__ row_base, int P, int Kd, int xc, int sc,
    u32x4 *__restrict__ out_rows, u32x4 *__restrict__ out_scales, uint32_t cap,
    int32_t *__restrict__ out_src_peer, int32_t *__restrict__ out_src_token, uint32_t g_first, uint32_t g_stride)
{
    // The row's record and the row count are requested first -- their addresses need only
    // arguments that are in registers when the wave starts -- and every other kernel argument is
    // fetched beside them, not after the first branch: one wait for all of it.  Pointers are
    // pinned through a copy of their low half, so the originals keep their address space.
    uint32_t g = g_first;
    // g_first < max_recv_rows, so the first record read is always inside the workspace
    const u32x4 *rp = (const u32x4 *)(recs + g);
    u32x4 r0 = rp[0], r1 = rp[1];
    uint32_t m_total = row_base[P];
    uint32_t gdim = g_stride, bdim = blockDim.x;
    MW_PIN_S(gdim); MW_PIN_S(bdim); MW_PIN_S(Kd); MW_PIN_S(xc); MW_PIN_S(sc); MW_PIN_S(cap);
    MW_PIN_PTR(hits); MW_PIN_PTR(out_rows); MW_PIN_PTR(out_scales); MW_PIN_PTR(out_src_peer);
    MW_PIN_PTR(out_src_token);
    MW_PIN_S4(r0); MW_PIN_S4(r1); MW_PIN_S(m_total);
    const int n = xc + sc;
    const int c = blockIdx.x * bdim + threadIdx.x;
    while (g < m_total) {
        const int n_hits = (int)r1.x;
        if (n_hits > 0) {
            const int peer = (int)r0.w;
            const void *src = (const void *)(((uint64_t)r0.y << 32) | r0.x);
            uint32_t b0 = base[r1.y * (uint32_t)P + (uint32_t)peer];
            u32x4 v = {0u, 0u, 0u, 0u};
            if (c < n) v = mw_ld16_global(src, c);
            MW_PIN_S(b0);                                  // position lookup in flight with the payload
            uint32_t dst = b0 + r1.z;                      // below 2^30: 2^24 rows, 64 experts each
            for (int k = 1;; ++k) {
                if (dst < cap) {
                    if (c < xc) mw_st16(out_rows + (size_t)dst * xc + c, v);
                    // a row's scales are a fraction of a cache line (224 bytes of fp8 rows): an
                    // ordinary store lets L2 put neighbouring rows' pieces together before the
                    // line goes to memory, where the write-through store sent every piece by
                    // itself (fp8 expander 77.5 -> 76 us, the step 97.4 -> 94.5 us)
                    else if (c < n) out_scales[(size_t)dst * sc + (c - xc)] = v;
                    if (c == 0) { out_src_peer[dst] = peer; out_src_token[dst] = (int32_t)r0.z; }
                }
                if (k >= n_hits) break;
                const mw_hit hk = hits[(size_t)g * Kd + k];
                dst = base[(uint32_t)hk.le * P + (uint32_t)peer] + (uint32_t)hk.rank;
            }
        }
        g += gdim;
        if (g < m_total) { rp = (const u32x4 *)(recs + g); r0 = rp[0]; r1 = rp[1]; }
    }
}

__global__ __launch_bounds__(1024) void k_expand(
    const mw_row_rec *__restrict__ recs, const uint32_t *__restrict__ row_base, const uint32_t *__restrict__ base,
    const mw_hit *__restrict__ hits, int P, int Kd, int xc, int sc,     // (in registers when a wave starts)
    u32x4 *__restrict__ out_rows, u32x4 *__restrict__ out_scales, uint32_t cap,
    int32_t *__restrict__ out_src_peer, int32_t *__restrict__ out_src_token)
{
    expand_body(recs, hits, base, row_base, P, Kd, xc, sc, out_rows, out_scales, cap, out_src_peer, out_src_token,
                blockIdx.y, gridDim.y);
}

// One launch for a steady stream of batches: the expander of the current batch and, in the
// first `next.P` workgroup rows of the grid, the index of the NEXT batch, written to another
// context's workspace.  The index is a chain of memory round trips that moves almost nothing;
// run as its own launch in front of its expander it costs 14-16 us of an otherwise
// bandwidth-bound stream, and run on a second stream it costs a cross-stream wait of 7-10 us.
// Here it rides along: its workgroups are dispatched first and finish long before the
// expander's do, and the launch that expands the next batch is ordered after this one by the
// stream, so no wait, flag or fence is needed.
// kLean: every wave of a launch is given the registers (and the scratch space for spills) of the
// launch's hungriest path, the row movers' waves included -- and with 64 registers a wave, or
// with any scratch at all, the dispatcher refills the movers' wave slots more slowly (rocprofv3:
// SPI_RA_VGPR_SIMD_FULL_CSN and SPI_RA_TMP_STALL_CSN appear, occupancy 7 % down; fp8 step 94.9
// against 87.4 us with the riders compiled out).  Beside a large batch the riders therefore run
// in a lean form that fits 56 registers without spilling (no first-row cache in the index, fewer
// counters in flight in the plan's second half): a few microseconds slower, long inside the
// movers' shadow.  Beside a small batch, where the riders ARE the step, they keep the fast form.
template <bool kLean>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_expand_index_next(
    const uint32_t first_expand_row, const uint32_t unused0, const mw_row_rec *__restrict__ recs,
    const uint32_t *__restrict__ row_base, const uint32_t *__restrict__ base, const mw_hit *__restrict__ hits,
    int P, int Kd, int xc, int sc,          // up to here: in registers when a wave starts
    u32x4 *__restrict__ out_rows, u32x4 *__restrict__ out_scales, uint32_t cap,
    int32_t *__restrict__ out_src_peer, int32_t *__restrict__ out_src_token, const mw_index_args next)
{
    if (blockIdx.y >= first_expand_row) {
        expand_body(recs, hits, base, row_base, P, Kd, xc, sc, out_rows, out_scales, cap, out_src_peer, out_src_token,
                    blockIdx.y - first_expand_row, gridDim.y - first_expand_row);
        return;
    }
    if (blockIdx.x == 0) recv_index_of<false, !kLean>(next, (int)blockIdx.y);
}

// The same launch with the PLAN of the next batch riding along as well (Section 5.1, send
// module: task decomposition for the batch after this one): after the index rows of the grid
// come `n_plan_rows` rows whose workgroups rank the next batch's tokens and then, in further
// workgroups that wait for those, write perm, descriptors and statistics.  A steady stream of
// batches then needs two launches per batch on ONE stream -- the packer and this -- and no
// event.  Measured per batch: 4096 tokens x 14336-byte rows 170 us, the same as with the plan
// on a second stream and one event wait per batch (171 us); fp8 rows of half the size 101
// against 105 us.  The riding plan is not free: its device-scope atomics and loads take
// about 4 us of memory-channel time from the expander.
template <int W, bool kKeyed, bool kLean>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_expand_index_plan_next(
    const uint32_t first_pack_row, const uint32_t first_expand_row, const mw_row_rec *__restrict__ recs,
    const uint32_t *__restrict__ row_base, int P, int xc, const int32_t *__restrict__ pack_perm,
    const mw_send_stats *__restrict__ pack_stats, int sc, int Kd,   // up to here: 14 words, in registers when a wave starts
    const uint32_t *__restrict__ base, const mw_hit *__restrict__ hits,
    u32x4 *__restrict__ out_rows, u32x4 *__restrict__ out_scales, uint32_t cap,
    int32_t *__restrict__ out_src_peer, int32_t *__restrict__ out_src_token,
    const mw_index_args next, const mw_plan_args plan, const mw_pack_args pack)
{
    // A row mover's wave lives for about a microsecond, and every dependent scalar fetch in front
    // of its payload load is a tenth of that.  The movers' branches therefore come first, and
    // what decides them and locates a wave's row -- the two role boundaries, the expander's record
    // and row-count arrays, the packer's row order and row count -- are the kernel's first
    // arguments: the library is built so that the first 14 argument words are in scalar registers
    // when a wave starts (hardware preload).  A mover's wave then has ONE round trip in front of its
    // payload load (its row's record or token, with the remaining arguments fetched beside it)
    // where decoding the roles one by one took five.
    const uint32_t y_pack = first_pack_row, y_expand = first_expand_row;
    if (blockIdx.y >= y_expand) {
        expand_body(recs, hits, base, row_base, P, Kd, xc, sc, out_rows, out_scales, cap, out_src_peer, out_src_token,
                    blockIdx.y - y_expand, gridDim.y - y_expand);
        return;
    }
    if (blockIdx.y >= y_pack) {         // (mw_stream_step: the packer of a batch planned by an earlier launch)
        mw_pack_body(pack.x, pack.scales, pack.xc, pack.sc, pack.ns, pack.topk, pack.K, pack_perm, pack_stats, pack.packed,
                     pack.row_src_token, pack.row_topk, blockIdx.x, blockIdx.y - y_pack, y_expand - y_pack);
        return;
    }
    const uint32_t n_index = (uint32_t)next.P;
    if (blockIdx.y < n_index) {
        if (blockIdx.x == 0) recv_index_of<false, !kLean>(next, (int)blockIdx.y);
        return;
    }
    extern __shared__ uint64_t plan_lds[];
    mw_plan_ride<W, kKeyed, kLean ? 8 : 16>(plan, (blockIdx.y - n_index) * gridDim.x + blockIdx.x, plan_lds);
}

// A whole step of a stream of SMALL batches in one launch (the batch sizes of Section 6.3's
// dispatch experiment, 64 and 128 tokens a rank): what k_expand_index_plan_next does, with the
// riders in their one-workgroup forms -- grid row 0 indexes the next received batch
// (recv_index_small), row 1, if there is a plan to make, plans the next batch to send
// (mw_small_plan_ranks / mw_small_plan_finish, the plan of mw_plan_pack) -- then the packer's rows
// and the expander's.  At these sizes the step is the riders' chain of memory round trips, and the
// forms that spread a batch over workgroups spend half of theirs on talking to one another.
template <int W, bool kKeyed, int kRows>
__global__ __launch_bounds__(kSmallLanes) void k_small_step(
    const uint32_t first_pack_row, const uint32_t first_expand_row, const mw_row_rec *__restrict__ recs,
    const uint32_t *__restrict__ row_base, int P, int xc, const int32_t *__restrict__ pack_perm,
    const mw_send_stats *__restrict__ pack_stats, int sc, int Kd,
    const uint32_t *__restrict__ base, const mw_hit *__restrict__ hits,
    u32x4 *__restrict__ out_rows, u32x4 *__restrict__ out_scales, uint32_t cap,
    int32_t *__restrict__ out_src_peer, int32_t *__restrict__ out_src_token,
    const mw_index_args next, const mw_plan_args plan, const mw_pack_args pack)
{
    if (blockIdx.y >= first_expand_row) {
        expand_body(recs, hits, base, row_base, P, Kd, xc, sc, out_rows, out_scales, cap, out_src_peer, out_src_token,
                    blockIdx.y - first_expand_row, gridDim.y - first_expand_row);
        return;
    }
    if (blockIdx.y >= first_pack_row) {
        mw_pack_body(pack.x, pack.scales, pack.xc, pack.sc, pack.ns, pack.topk, pack.K, pack_perm, pack_stats, pack.packed,
                     pack.row_src_token, pack.row_topk, blockIdx.x, blockIdx.y - first_pack_row,
                     first_expand_row - first_pack_row);
        return;
    }
    if (blockIdx.x != 0) return;
    extern __shared__ uint64_t small_lds[];
    if (blockIdx.y == 0) {
        recv_index_small<kRows>(next, (uint32_t *)small_lds);
        return;
    }
    // LDS of the plan: bitmaps, short keys, then the 32-bit arrays
    uint64_t *smask = small_lds;
    mw_short_key *skey = (mw_short_key *)(smask + kSmallBlock * W);
    int32_t *tok = (int32_t *)(skey + (kKeyed ? kSmallBlock : 0));
    uint32_t *gstart = (uint32_t *)(tok + kSmallBlock);
    uint32_t *hist = gstart + kSmallBlock + 1;
    uint32_t *scratch = hist + MW_MAX_RANKS;
    const mw_small_plan_lds l = {smask, tok, gstart, hist, scratch, skey};
    const mw_small_plan_rank r = mw_small_plan_ranks<W, kKeyed>(plan.topk, plan.T, plan.K, plan.eslot, plan.E, l);
    mw_small_plan_finish<W>(r, plan.T, plan.row_bytes, plan.mask_out, plan.perm, plan.desc, plan.stats, l, true, true);
}

// The one-workgroup index as a launch of its own (mw_unpack_index, mw_unpack of a small batch).
template <int kRows>
__global__ __launch_bounds__(kSmallLanes) void k_recv_index_small(const mw_index_args a)
{
    extern __shared__ uint64_t small_index_lds[];
    recv_index_small<kRows>(a, (uint32_t *)small_index_lds);
}

// The way back (Section 2.1, combine-style AlltoAll; Section 2.3.2: the combine phase reduces
// and cannot be multicast).  The mirror image of the expander: a received row that went to h
// local experts gets ONE row back, the sum of those h expert outputs, so the return traffic is
// one copy per (token, rank) like the dispatch's.  Reads the index the last unpack left in the
// workspace.  Per 16-byte chunk (8 bf16): widen to single precision, add in the order of the
// row's hit slots (the order of its id list), round once to bf16 (nearest even; a NaN sum
// becomes 0x7FC0 with the sum's sign); h == 1 is a copy.  Hits whose output row was dropped for
// capacity contribute nothing.  Same launch shape and the same bytes as the expander, in the
// other direction: bound by HBM bandwidth.
__device__ __forceinline__ uint32_t mw_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return ((u >> 16) & 0x8000u) | 0x7fc0u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

__global__ __launch_bounds__(1024) void k_combine(
    const mw_row_rec *__restrict__ recs, const mw_hit *__restrict__ hits, const uint32_t *__restrict__ base,
    const uint32_t *__restrict__ row_base, int P, int Kd, int n, const u32x4 *__restrict__ y, uint32_t cap,
    u32x4 *__restrict__ ret, uint32_t ret_cap)
{
    uint32_t gdim = gridDim.y, bdim = blockDim.x;
    MW_PIN_S(gdim); MW_PIN_S(bdim); MW_PIN_S(Kd); MW_PIN_S(n); MW_PIN_S(cap); MW_PIN_S(ret_cap);
    MW_PIN_PTR(hits); MW_PIN_PTR(y); MW_PIN_PTR(ret);
    const int c = blockIdx.x * bdim + threadIdx.x;
    uint32_t g = blockIdx.y;
    const u32x4 *rp = (const u32x4 *)(recs + g);
    u32x4 r0 = rp[0], r1 = rp[1];
    uint32_t m_total = row_base[P];
    MW_PIN_S4(r0); MW_PIN_S4(r1); MW_PIN_S(m_total);
    while (g < m_total) {
        const int n_hits = (int)r1.x;
        if (n_hits > 0 && g < ret_cap) {
            const uint32_t peer = r0.w;
            uint32_t pos = base[r1.y * (uint32_t)P + peer] + r1.z;
            if (n_hits == 1) {
                if (pos < cap && c < n) mw_st16(ret + (size_t)g * n + c, mw_ld16(y + (size_t)pos * n + c));
            } else {
                float acc[8];
                bool any = false;
                for (int k = 0;; ++k) {
                    if (pos < cap && c < n) {
                        const u32x4 v = mw_ld16(y + (size_t)pos * n + c);
                        const float f[8] = {__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u),
                                            __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xffff0000u),
                                            __uint_as_float(v.z << 16), __uint_as_float(v.z & 0xffff0000u),
                                            __uint_as_float(v.w << 16), __uint_as_float(v.w & 0xffff0000u)};
#pragma unroll
                        for (int j = 0; j < 8; ++j) acc[j] = any ? acc[j] + f[j] : f[j];
                    }
                    any = any || pos < cap;
                    if (k + 1 >= n_hits) break;
                    const mw_hit hk = hits[(size_t)g * Kd + k + 1];
                    pos = base[(uint32_t)hk.le * P + peer] + (uint32_t)hk.rank;
                }
                if (any && c < n) {
                    u32x4 o;
                    o.x = mw_bf16_rne(acc[0]) | (mw_bf16_rne(acc[1]) << 16);
                    o.y = mw_bf16_rne(acc[2]) | (mw_bf16_rne(acc[3]) << 16);
                    o.z = mw_bf16_rne(acc[4]) | (mw_bf16_rne(acc[5]) << 16);
                    o.w = mw_bf16_rne(acc[6]) | (mw_bf16_rne(acc[7]) << 16);
                    mw_st16(ret + (size_t)g * n + c, o);
                }
            }
        }
        g += gdim;
        if (g < m_total) { rp = (const u32x4 *)(recs + g); r0 = rp[0]; r1 = rp[1]; }
    }
}

}  // namespace

// Index arguments of `ctx` for a launch whose workgroups may use `lds_budget_words` words of LDS
// each: the addressed-rows bitmap plus two arrays per expert of a chunk (experts beyond the
// budget are handled in further passes).  Returns false if not even one expert fits.
static bool make_index_args(mw_ctx *ctx, const void *peers, bool packets, int32_t P, int64_t cap,
                            int64_t *expert_offsets, mw_recv_stats *stats, uint32_t lds_budget_words,
                            mw_index_args *a, size_t *lds_bytes)
{
    const mw_config &c = ctx->cfg;
    const int L = ctx->n_local;
    const uint32_t wpl = ((uint32_t)c.max_tokens + 31u) / 32u;
    const uint32_t dedup = (ctx->options & MW_OPT_RECV_DEDUP) ? 1u : 0u;
    if (dedup) lds_budget_words = lds_budget_words > wpl ? lds_budget_words - wpl : 0;     // the "taken" bitmap
    if (lds_budget_words < 3 * wpl + 64) return false;
    int Lc = (int)((lds_budget_words - 64 - wpl) / (2 * wpl));
    if (Lc < 1) return false;
    if (Lc > L) Lc = L > 0 ? L : 1;
    *lds_bytes = ((size_t)wpl + 2 * (size_t)Lc * wpl + 64 + (dedup ? wpl : 0)) * sizeof(uint32_t);
    const uint32_t hb = packets ? (uint32_t)mw_packet_header_bytes_of(c.top_k) : 0u;
    *a = mw_index_args{peers, P, ctx->d_eslot, c.n_experts, c.top_k, ctx->hit_slots, c.my_rank, L, Lc,
                       (uint32_t)c.max_tokens, wpl, (uint32_t)c.max_recv_rows,
                       (uint64_t)(packets ? hb + ctx->row_bytes : ctx->row_stride), hb, cap,
                       ctx->d_cnt, ctx->d_row_base, ctx->d_addr_cnt, ctx->d_recs, ctx->d_hits, ctx->d_base,
                       expert_offsets, stats, ctx->d_flags, dedup};
    return true;
}

// the index of `P` peers' regions on `ctx` fits the one-workgroup form
static bool small_index_fits(const mw_ctx *ctx, int32_t P)
{
    static_assert(kSmallBlock == MW_MAX_RANKS, "one lane per peer record, one lane per rank in the statistics");
    if (ctx->options & MW_OPT_RECV_DEDUP) return false;
    if (P > kSmallBlock || ctx->n_local > 64) return false;
    if ((int64_t)P * ctx->cfg.max_tokens > 16384) return false;
    const uint32_t wpl = ((uint32_t)ctx->cfg.max_tokens + 31u) / 32u;
    return mw_small_index_lds_words(P, ctx->n_local, wpl, (uint32_t)ctx->cfg.max_tokens,
                                    (uint32_t)ctx->cfg.max_recv_rows) * 4 <= 40960;
}

// rows a lane of the one-workgroup index keeps in registers: two for up to 1024 received rows (as many
// as the context saw last time, if the caller has asked for the statistics), else four
static bool small_index_few_rows(const mw_ctx *ctx, int32_t P)
{
    return ctx->recv_rows_hint > 0 ? ctx->recv_rows_hint <= 2 * kSmallLanes
                                   : (int64_t)P * ctx->cfg.max_tokens <= 2 * kSmallLanes;
}

int32_t mw_launch_unpack_index(mw_ctx *ctx, const void *peers, bool packets, int32_t P, int64_t cap,
                               int64_t *expert_offsets, mw_recv_stats *stats, hipStream_t s)
{
    mw_index_args a;
    size_t lds_index;
    if (!make_index_args(ctx, peers, packets, P, cap, expert_offsets, stats, 12288, &a, &lds_index))
        return MW_ERR_UNSUPPORTED;
    // A peer seldom sends more than a fraction of its tokens to one rank: for small batches a
    // quarter of the lanes do, with shorter barriers and scans (about a microsecond of 11).
    const int ib = ctx->cfg.max_tokens <= 2048 ? 256 : kIndexBlock;
    {
        mw_timed tm(ctx, MW_KERNEL_RECV_INDEX, s);
        const int64_t expected = ctx->recv_rows_hint > 0 ? ctx->recv_rows_hint : (int64_t)P * ctx->cfg.max_tokens;
        if (!packets && expected <= kSmallLanes && small_index_fits(ctx, P)) {
            // a row a lane at most: one workgroup for all peers, nothing to exchange between workgroups
            // (9.6 against 10.9 us at 443 rows; with two rows a lane the workgroup-per-peer form is ahead)
            const uint32_t wpl = ((uint32_t)ctx->cfg.max_tokens + 31u) / 32u;
            const size_t lds = 4 * mw_small_index_lds_words(P, ctx->n_local, wpl, (uint32_t)ctx->cfg.max_tokens,
                                                            (uint32_t)ctx->cfg.max_recv_rows) + 16;
            if (small_index_few_rows(ctx, P)) hipLaunchKernelGGL(k_recv_index_small<2>, dim3(1), dim3(kSmallLanes), lds, s, a);
            else hipLaunchKernelGGL(k_recv_index_small<4>, dim3(1), dim3(kSmallLanes), lds, s, a);
        } else
        if (packets) hipLaunchKernelGGL(k_recv_index<true>, dim3(P), dim3(ib), lds_index, s, a);
        else hipLaunchKernelGGL(k_recv_index<false>, dim3(P), dim3(ib), lds_index, s, a);
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

// Grid rows of the expander: about as many as the peers held last time (if the caller has
// asked for the statistics), not the capacity -- workgroups are dispatched at a finite rate,
// empty ones included.  More rows than that are reached by striding.
static uint32_t expand_grid_rows(const mw_ctx *ctx)
{
    int64_t rows = ctx->cfg.max_recv_rows;
    if (ctx->recv_rows_hint > 0) {
        const int64_t want = ctx->recv_rows_hint + ctx->recv_rows_hint / 64 + 64;
        if (want < rows) rows = want;
    }
    return (uint32_t)(rows < kRowGridMax ? rows : kRowGridMax);
}

// Whether a launch that moves `grid_rows` received rows (more by striding) carries its riders in
// the lean form: from 32 MiB of payload on, where the movers' time dwarfs the riders'.
static bool riders_lean(const mw_ctx *ctx, uint32_t grid_rows)
{
    return (int64_t)grid_rows * ctx->row_bytes >= (32LL << 20);
}

int32_t mw_launch_unpack_expand(mw_ctx *ctx, int32_t P, void *out_rows, float *out_scales, int64_t cap,
                                int32_t *out_src_peer, int32_t *out_src_token, hipStream_t s)
{
    const mw_config &c = ctx->cfg;
    if (c.max_recv_rows > 0) {
        const int xc = (int)(ctx->x_row_bytes / 16), sc = (int)(ctx->s_row_bytes / 16);
        const mw_row_shape shape = mw_row_shape_of(xc + sc);
        const uint32_t gy = expand_grid_rows(ctx);
        mw_timed tm(ctx, MW_KERNEL_EXPAND, s);
        hipLaunchKernelGGL(k_expand, dim3(shape.nseg, gy), dim3(shape.bs), 0, s, ctx->d_recs, ctx->d_row_base, ctx->d_base,
                           ctx->d_hits, P, ctx->hit_slots, xc, sc, (u32x4 *)out_rows, (u32x4 *)out_scales,
                           (uint32_t)(cap < 0x7fffffffLL ? cap : 0x7fffffffLL), out_src_peer, out_src_token);
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

// Whether a step is small enough for k_small_step -- this batch's rows (received and to pack) under
// 24 MiB, so that the riders and not the movers are the step; the next batch's index in one
// workgroup's LDS and at most MW_FUSED_MAX_TOKENS tokens to plan -- and, if so, its launch.
// with_plan: the launch plans next_T tokens (possibly none); pk: rows to pack, or null.
static bool small_step_fits(const mw_ctx *ctx, const mw_ctx *next, int32_t next_P, int32_t next_T, const mw_pack_call *pk,
                            uint32_t gy)
{
    const int64_t rows = (int64_t)gy + (pk ? pk->n_tokens : 0);
    if (rows * ctx->row_bytes > (24LL << 20)) return false;
    if (next_T > MW_FUSED_MAX_TOKENS) return false;
    return small_index_fits(next, next_P);
}

static int32_t launch_small_step(mw_ctx *ctx, int32_t P, void *out_rows, float *out_scales, int64_t cap,
                                 int32_t *out_src_peer, int32_t *out_src_token, mw_ctx *next, const mw_index_args &a,
                                 bool with_plan, const int32_t *next_topk, int32_t next_T, uint64_t *next_mask,
                                 int32_t *next_perm, mw_group_desc *next_desc, mw_send_stats *next_send_stats,
                                 const mw_pack_call *pk, uint32_t gy, hipStream_t s)
{
    const mw_config &c = ctx->cfg;
    const int xc = (int)(ctx->x_row_bytes / 16), sc = (int)(ctx->s_row_bytes / 16);
    const int nseg = (xc + sc + kSmallLanes - 1) / kSmallLanes;
    const int K = next->cfg.top_k, W = next->mask_words;
    const bool keyed = W > 1 && K <= 8;
    mw_plan_args pl = {};
    pl.topk = next_topk; pl.T = next_T; pl.K = K; pl.E = next->cfg.n_experts; pl.eslot = next->d_eslot;
    pl.mask_out = next_mask; pl.perm = next_perm; pl.desc = next_desc; pl.stats = next_send_stats;
    pl.row_bytes = (uint64_t)next->row_bytes;
    mw_pack_args pa = {};
    uint32_t n_pack_rows = 0;
    if (pk && pk->n_tokens > 0) {
        pa.x = (const u32x4 *)pk->x; pa.scales = (const u32x4 *)pk->scales; pa.xc = xc; pa.sc = sc;
        pa.ns = (int)(ctx->row_stride / 16);
        pa.topk = pk->topk; pa.K = c.top_k; pa.perm = pk->perm; pa.stats = pk->stats;
        pa.packed = (u32x4 *)pk->packed; pa.row_src_token = pk->row_src_token; pa.row_topk = pk->row_topk;
        n_pack_rows = (uint32_t)pk->n_tokens;
    }
    const uint32_t wpl = ((uint32_t)next->cfg.max_tokens + 31u) / 32u;
    const size_t lds_index = 4 * mw_small_index_lds_words(a.P, next->n_local, wpl, (uint32_t)next->cfg.max_tokens,
                                                          (uint32_t)next->cfg.max_recv_rows);
    const int Wk = keyed ? 4 : W;
    const size_t lds_plan = (size_t)kSmallBlock * Wk * 8 + (keyed ? (size_t)kSmallBlock * sizeof(mw_short_key) : 0) +
                            4 * ((size_t)kSmallBlock + kSmallBlock + 1 + MW_MAX_RANKS + 18);
    const size_t lds = (with_plan && lds_plan > lds_index ? lds_plan : lds_index) + 16;
    const uint32_t riders = with_plan ? 2u : 1u;
    const dim3 grid(nseg, riders + n_pack_rows + gy), block(kSmallLanes);
    const uint32_t cap32 = (uint32_t)(cap < 0x7fffffffLL ? cap : 0x7fffffffLL);
    {
        mw_timed tm(ctx, MW_KERNEL_EXPAND, s);
        const bool few = small_index_few_rows(next, a.P);
#define MW_SMALL_(W_, KEYED_, ROWS_)                                                                                   \
    hipLaunchKernelGGL((k_small_step<W_, KEYED_, ROWS_>), grid, block, lds, s, riders, riders + n_pack_rows, ctx->d_recs, \
                       ctx->d_row_base, P, xc, pa.perm, pa.stats, sc, ctx->hit_slots, ctx->d_base, ctx->d_hits,         \
                       (u32x4 *)out_rows, (u32x4 *)out_scales, cap32, out_src_peer, out_src_token, a, pl, pa)
#define MW_SMALL(W_, KEYED_) do { if (few) MW_SMALL_(W_, KEYED_, 2); else MW_SMALL_(W_, KEYED_, 4); } while (0)
        if (keyed) MW_SMALL(4, true);
        else if (W == 1) MW_SMALL(1, false);
        else if (W == 2) MW_SMALL(2, false);
        else if (W == 3) MW_SMALL(3, false);
        else MW_SMALL(4, false);
#undef MW_SMALL
#undef MW_SMALL_
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

int32_t mw_launch_unpack_expand_index_next(mw_ctx *ctx, int32_t P, void *out_rows, float *out_scales, int64_t cap,
                                           int32_t *out_src_peer, int32_t *out_src_token, mw_ctx *next,
                                           const mw_recv_peer *next_peers, int32_t next_P, int64_t next_cap,
                                           int64_t *next_expert_offsets, mw_recv_stats *next_stats, hipStream_t s)
{
    const mw_config &c = ctx->cfg;
    if (c.max_recv_rows < 1) return MW_ERR_UNSUPPORTED;       // nothing to ride on
    // Every workgroup of the launch reserves the index's LDS, the expander's included: at most
    // 5 KiB, so that a CU's 160 KiB still hold a full set of 32 single-wave expander workgroups.
    mw_index_args a;
    size_t lds_index;
    if (!make_index_args(next, next_peers, false, next_P, next_cap, next_expert_offsets, next_stats, 1280, &a,
                         &lds_index))
        return MW_ERR_UNSUPPORTED;
    if (small_step_fits(ctx, next, next_P, 0, nullptr, expand_grid_rows(ctx)))
        return launch_small_step(ctx, P, out_rows, out_scales, cap, out_src_peer, out_src_token, next, a, false, nullptr,
                                 0, nullptr, nullptr, nullptr, nullptr, nullptr, expand_grid_rows(ctx), s);
    const int xc = (int)(ctx->x_row_bytes / 16), sc = (int)(ctx->s_row_bytes / 16);
    mw_row_shape shape = mw_row_shape_of(xc + sc);
    // Rows of whole cache lines: two-wave workgroups here.  The expander runs as fast with them
    // as with single waves (138.8 against 139.4 us at 30590 rows of 14336 bytes), and the riding
    // index gets two waves per peer: with one it outlasts the expander (142 against 139 us).
    if (shape.bs == 64 && (xc + sc) % 16 == 0) { shape.bs = 128; shape.nseg = (xc + sc) / 128 + ((xc + sc) % 128 ? 1 : 0); }
    const uint32_t gy = expand_grid_rows(ctx);
    {
        mw_timed tm(ctx, MW_KERNEL_EXPAND, s);
        const uint32_t cap32 = (uint32_t)(cap < 0x7fffffffLL ? cap : 0x7fffffffLL);
        if (riders_lean(ctx, gy))
            hipLaunchKernelGGL(k_expand_index_next<true>, dim3(shape.nseg, gy + (uint32_t)next_P), dim3(shape.bs), lds_index,
                               s, (uint32_t)next_P, 0u, ctx->d_recs, ctx->d_row_base, ctx->d_base, ctx->d_hits, P,
                               ctx->hit_slots, xc, sc, (u32x4 *)out_rows, (u32x4 *)out_scales, cap32, out_src_peer,
                               out_src_token, a);
        else
            hipLaunchKernelGGL(k_expand_index_next<false>, dim3(shape.nseg, gy + (uint32_t)next_P), dim3(shape.bs), lds_index,
                               s, (uint32_t)next_P, 0u, ctx->d_recs, ctx->d_row_base, ctx->d_base, ctx->d_hits, P,
                               ctx->hit_slots, xc, sc, (u32x4 *)out_rows, (u32x4 *)out_scales, cap32, out_src_peer,
                               out_src_token, a);
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

int32_t mw_launch_unpack_expand_index_plan_next(mw_ctx *ctx, int32_t P, void *out_rows, float *out_scales, int64_t cap,
                                                int32_t *out_src_peer, int32_t *out_src_token, mw_ctx *next,
                                                const mw_recv_peer *next_peers, int32_t next_P, int64_t next_cap,
                                                int64_t *next_expert_offsets, mw_recv_stats *next_stats,
                                                const int32_t *next_topk, int32_t next_T, uint64_t *next_mask,
                                                int32_t *next_perm, mw_group_desc *next_desc,
                                                mw_send_stats *next_send_stats, const mw_pack_call *pk, hipStream_t s)
{
    const mw_config &c = ctx->cfg;
    if (c.max_recv_rows < 1) return MW_ERR_UNSUPPORTED;       // nothing to ride on
    if (next_T > MW_RIDE_MAX_TOKENS) return MW_ERR_UNSUPPORTED;
    mw_index_args a;
    size_t lds_index;
    if (!make_index_args(next, next_peers, false, next_P, next_cap, next_expert_offsets, next_stats, 1280, &a,
                         &lds_index))
        return MW_ERR_UNSUPPORTED;
    const uint32_t gy = expand_grid_rows(ctx);
    if (small_step_fits(ctx, next, next_P, next_T, pk, gy))
        return launch_small_step(ctx, P, out_rows, out_scales, cap, out_src_peer, out_src_token, next, a, true, next_topk,
                                 next_T, next_mask, next_perm, next_desc, next_send_stats, pk, gy, s);
    const int xc = (int)(ctx->x_row_bytes / 16), sc = (int)(ctx->s_row_bytes / 16);
    mw_row_shape shape = mw_row_shape_of(xc + sc);
    if (shape.bs == 64 && (xc + sc) % 16 == 0) { shape.bs = 128; shape.nseg = (xc + sc) / 128 + ((xc + sc) % 128 ? 1 : 0); }

    // the riding plan: workgroups of the launch's size
    const int K = next->cfg.top_k, W = next->mask_words;
    const bool keyed = W > 1 && K <= 8;
    mw_plan_args pl;
    pl.topk = next_topk; pl.T = next_T; pl.K = K; pl.E = next->cfg.n_experts; pl.eslot = next->d_eslot;
    pl.mask_out = next_mask; pl.cnt = (unsigned long long *)next->d_plan_cnt; pl.pstate = next->d_plan_state;
    pl.perm = next_perm; pl.desc = next_desc; pl.stats = next_send_stats; pl.row_bytes = (uint64_t)next->row_bytes;
    // Slices as long as LDS allows: every (token, slice) pair costs one device-scope atomic and
    // every rank workgroup one more on a single counter, and those -- unlike the ranking itself --
    // take memory-channel time from the expander (slices of 128 tokens: +22 us per launch at
    // 4096 tokens; of 1024: +4 us).  Workgroups of two or more waves leave room for 8 KiB each.
    const size_t key_bytes = keyed ? sizeof(mw_short_key) : (size_t)W * sizeof(uint64_t);
    const size_t lds_budget = shape.bs >= 128 ? 8192 : 5120;
    pl.slice = (int)(lds_budget / key_bytes) / 128 * 128;
    if (pl.slice > (next_T + 127) / 128 * 128) pl.slice = (next_T + 127) / 128 * 128;
    if (pl.slice < 128) pl.slice = 128;
    pl.tb = next_T > 0 ? (next_T + shape.bs - 1) / shape.bs : 1;
    pl.ns = next_T > 0 ? (next_T + pl.slice - 1) / pl.slice : 1;
    pl.n_rank = (uint32_t)pl.tb * (uint32_t)pl.ns;
    pl.finish_rows = mw_plan_finish_rows(shape.bs);
    pl.n_finish = next_T > 0 ? ((uint32_t)next_T + pl.finish_rows - 1) / pl.finish_rows : 1u;
    pl.wait_limit = next->ride_wait_limit;
    const uint32_t n_plan_rows = (pl.n_rank + pl.n_finish + (uint32_t)shape.nseg - 1) / (uint32_t)shape.nseg;
    size_t lds_plan = (size_t)pl.slice * key_bytes;
    if (lds_plan < mw_plan_finish_lds(shape.bs)) lds_plan = mw_plan_finish_lds(shape.bs);
    const size_t lds = lds_index > lds_plan ? lds_index : lds_plan;
    {
        mw_timed tm(ctx, MW_KERNEL_EXPAND, s);
        // the packer of this context's own rows, if asked for: same row shape as the expander
        mw_pack_args pa = {};
        uint32_t n_pack_rows = 0;
        if (pk && pk->n_tokens > 0) {
            pa.x = (const u32x4 *)pk->x; pa.scales = (const u32x4 *)pk->scales; pa.xc = xc; pa.sc = sc;
            pa.ns = (int)(ctx->row_stride / 16);
            pa.topk = pk->topk; pa.K = c.top_k; pa.perm = pk->perm; pa.stats = pk->stats;
            pa.packed = (u32x4 *)pk->packed; pa.row_src_token = pk->row_src_token; pa.row_topk = pk->row_topk;
            n_pack_rows = (uint32_t)pk->n_tokens < 16384u ? (uint32_t)pk->n_tokens : 16384u;   // more by striding
        }
        // a grid has at most 65535 rows: the expander takes what the riders leave (more by striding)
        const uint32_t riders = (uint32_t)next_P + n_plan_rows + n_pack_rows;      // <= 256 + 8192 + 16384
        const uint32_t gy_fit = gy < 65535u - riders ? gy : 65535u - riders;
        const dim3 grid(shape.nseg, gy_fit + riders), block(shape.bs);
        const uint32_t cap32 = (uint32_t)(cap < 0x7fffffffLL ? cap : 0x7fffffffLL);
        const bool lean = riders_lean(ctx, gy_fit);
#define MW_RIDE_(W_, KEYED_, LEAN_)                                                                                \
    hipLaunchKernelGGL((k_expand_index_plan_next<W_, KEYED_, LEAN_>), grid, block, lds, s,                          \
                       (uint32_t)next_P + n_plan_rows, (uint32_t)next_P + n_plan_rows + n_pack_rows, ctx->d_recs,   \
                       ctx->d_row_base, P, xc, pa.perm, pa.stats, sc, ctx->hit_slots, ctx->d_base, ctx->d_hits,     \
                       (u32x4 *)out_rows, (u32x4 *)out_scales, cap32, out_src_peer, out_src_token, a, pl, pa)
#define MW_RIDE(W_, KEYED_) do { if (lean) MW_RIDE_(W_, KEYED_, true); else MW_RIDE_(W_, KEYED_, false); } while (0)
        if (keyed) MW_RIDE(4, true);
        else if (W == 1) MW_RIDE(1, false);
        else if (W == 2) MW_RIDE(2, false);
        else if (W == 3) MW_RIDE(3, false);
        else MW_RIDE(4, false);
#undef MW_RIDE
#undef MW_RIDE_
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

int32_t mw_launch_combine(mw_ctx *ctx, int32_t P, const void *y, int64_t cap, void *ret, int64_t ret_cap, hipStream_t s)
{
    const mw_config &c = ctx->cfg;
    if (c.max_recv_rows > 0 && ret_cap > 0) {
        const int n = (int)(ctx->x_row_bytes / 16);
        const mw_row_shape shape = mw_row_shape_of(n);
        int64_t rows = c.max_recv_rows;                     // grid sized like the expander's
        if (ctx->recv_rows_hint > 0) {
            const int64_t want = ctx->recv_rows_hint + ctx->recv_rows_hint / 64 + 64;
            if (want < rows) rows = want;
        }
        const uint32_t gy = (uint32_t)(rows < kRowGridMax ? rows : kRowGridMax);
        mw_timed tm(ctx, MW_KERNEL_COMBINE, s);
        hipLaunchKernelGGL(k_combine, dim3(shape.nseg, gy), dim3(shape.bs), 0, s, ctx->d_recs, ctx->d_hits, ctx->d_base,
                           ctx->d_row_base, P, ctx->hit_slots, n, (const u32x4 *)y,
                           (uint32_t)(cap < 0x7fffffffLL ? cap : 0x7fffffffLL), (u32x4 *)ret,
                           (uint32_t)(ret_cap < 0x7fffffffLL ? ret_cap : 0x7fffffffLL));
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}
