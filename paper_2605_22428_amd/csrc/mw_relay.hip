// Relay step: one node's part of the recursive MultiWrite execution model.
//
// Paper hooks: Section 4.3.3 -- a node holding a MultiWrite for a destination set M
// partitions M by next hop and starts one child MultiWrite per subset, a subset of one
// destination being an ordinary write; Section 4.1, "Local forwarding table" -- the next
// hop of every destination comes from the node's unicast forwarding table and the number
// of distinct next hops is the number of copies; Section 4.1, "Replication and
// forwarding" -- each copy carries updated metadata naming only the destinations served
// through its hop, so nothing is delivered twice; Section 3.2 -- the same-index device of
// the remote server replicates a token to the targets inside that server.
//
// Two launches on the caller's stream:
//   k_relay_index  workgroup h < n_hops builds child h's descriptor table: a group is kept
//                  if its bitmap intersects the hop's rank set; kept groups are ranked with
//                  block scans (group index, first row), so the child is in parent order
//                  whatever the timing.  The (group, hop) -> first child row table feeds the
//                  copy.  One more workgroup maps rows to groups and does the byte accounting.
//   k_relay_copy   small workgroups (a single wave for cache-line-sized rows), each moving
//                  consecutive 16-byte chunks of one input row: read once, stored once per next hop that keeps the row's group
//                  (lane h of every wave holds hop h's position; a ballot lists the hops).  Bound by HBM
//                  bandwidth: rows * row_bytes read, rows * copies * row_bytes written.
#include "mw_internal.h"

namespace {

constexpr int kBlock = 1024;
constexpr uint32_t kNoChild = 0xffffffffu;
constexpr uint32_t kLongGroup = 32;          // rows; longer groups are filled cooperatively

// Everything the index of one relay step needs (one kernel argument).
struct mw_relay_index_args {
    const mw_recv_peer *in; const mw_relay_child *children; int n_hops, n_ranks;
    uint32_t max_tokens, cap; uint64_t row_bytes; const uint64_t *hop_bits;
    int32_t *group_of_row; uint32_t *child_pos; uint32_t *relay_flags; mw_relay_stats *stats;
    uint32_t keep_metadata;     // 1: children carry the parent's bitmaps (Section 4.1: the update may be omitted)
};

// The bitmap of ranks below n_ranks, word w.
__device__ __forceinline__ uint64_t valid_rank_word(int n_ranks, int w)
{
    const int lo = w * 64;
    return (n_ranks >= lo + 64) ? ~0ull : (n_ranks > lo ? ((1ull << (n_ranks - lo)) - 1ull) : 0ull);
}

// Child descriptor table of next hop h, by one workgroup.  A lane takes KP consecutive groups a
// step and reads of each what the ranking needs: the NW bitmap words that can name a rank
// (ranks < 64 NW; the hop's rank set and the valid ranks have nothing above them), the row range,
// and the end of the range in front (a descriptor is valid if its row range is not empty, lies
// inside the buffer and starts at or after the end of the previous descriptor's).  All of a step's loads are
// issued before the first is used -- addresses are clamped instead of branched around -- so a
// step is one memory round trip whatever KP; then one scan of the lanes' kept groups and one
// of their rows place every kept group in parent order.
template <int NW, int KP>
__device__ __forceinline__ uint32_t relay_index_hop(
    const mw_recv_peer &src, const uint32_t G, const uint32_t n_rows, mw_group_desc *__restrict__ cdesc, const int h,
    const int n_ranks, const uint32_t cap, const uint64_t *__restrict__ hop_bits, uint32_t *__restrict__ child_pos,
    mw_relay_stats *__restrict__ stats, const uint32_t keep_metadata, uint32_t *scratch, uint32_t *fit)
{
    const uint32_t bs = blockDim.x, tid = threadIdx.x;
    uint32_t err = 0;
    uint64_t hb[NW], ok[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) { hb[w] = hop_bits[(size_t)h * MW_MASK_WORDS + w]; ok[w] = valid_rank_word(n_ranks, w); }
    if (tid < 2) fit[tid] = 0;
    mw_lds_barrier();
    uint32_t carry_g = 0, carry_r = 0;
    for (uint32_t g0 = 0; g0 < G; g0 += bs * KP) {
        const uint32_t gl = g0 + tid * KP;           // this lane's first group
        uint64_t m[KP][NW];
        uint2 oc[KP];
#pragma unroll
        for (int k = 0; k < KP; ++k) {
            const mw_group_desc *d = src.desc + min(gl + (uint32_t)k, G - 1u);
#pragma unroll
            for (int w = 0; w < NW; ++w) m[k][w] = d->mask[w];
            oc[k] = *(const uint2 *)&d->row_offset;  // (row_offset, row_count)
        }
        const uint2 po = *(const uint2 *)&src.desc[min(gl > 0 ? gl - 1u : 0u, G - 1u)].row_offset;
        uint64_t prev_end = gl > 0 ? (uint64_t)po.x + po.y : 0ull;
        bool keep[KP];
        uint32_t nd[KP], lg = 0, lr = 0;
#pragma unroll
        for (int k = 0; k < KP; ++k) {
            const uint32_t off = oc[k].x, cnt = oc[k].y;
            const bool valid = gl + k < G && cnt >= 1 && (uint64_t)off + cnt <= n_rows && off >= prev_end;
            prev_end = (uint64_t)off + cnt;
            uint32_t n = 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) n += (uint32_t)__popcll(m[k][w] & hb[w]);
            keep[k] = valid && n > 0;
            if (keep_metadata) {                     // the copy carries every destination the parent named
                n = 0;
#pragma unroll
                for (int w = 0; w < NW; ++w) { m[k][w] &= ok[w]; n += (uint32_t)__popcll(m[k][w]); }
            } else {
#pragma unroll
                for (int w = 0; w < NW; ++w) m[k][w] &= hb[w];
            }
            nd[k] = n;
            lg += keep[k] ? 1u : 0u;
            lr += keep[k] ? cnt : 0u;
        }
        uint32_t tot_g, tot_r;
        uint32_t cg = carry_g + mw_block_exscan(lg, scratch, &tot_g);
        uint32_t cr = carry_r + mw_block_exscan(lr, scratch, &tot_r);
        uint32_t fit_g = 0, fit_r = 0;
#pragma unroll
        for (int k = 0; k < KP; ++k) {
            if (gl + k >= G) continue;
            const uint32_t cnt = oc[k].y;
            uint32_t pos = kNoChild;
            if (keep[k]) {
                if ((uint64_t)cr + cnt <= cap) {
                    mw_group_desc d;
#pragma unroll
                    for (int w = 0; w < MW_MASK_WORDS; ++w) d.mask[w] = 0;
#pragma unroll
                    for (int w = 0; w < NW; ++w) d.mask[w] = m[k][w];
                    d.row_offset = cr; d.row_count = cnt; d.n_dest = nd[k]; d.reserved0 = 0;
                    cdesc[cg] = d;
                    pos = cr;
                    fit_g = cg + 1u; fit_r = cr + cnt;
                } else {
                    err |= MW_FLAG_OUT_CAPACITY;
                }
                ++cg; cr += cnt;
            }
            child_pos[(size_t)(gl + k) * MW_MAX_HOPS + h] = pos;
        }
        // kept groups that fit are a prefix of the kept groups: the largest (index + 1, end
        // row) pair describes the child.  Reduced over the wave first: same-address LDS
        // atomics of a whole workgroup would serialise.
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            fit_g = max(fit_g, (uint32_t)__shfl_xor((int)fit_g, d, 64));
            fit_r = max(fit_r, (uint32_t)__shfl_xor((int)fit_r, d, 64));
        }
        if ((tid & 63) == 0 && fit_g) { atomicMax(&fit[0], fit_g); atomicMax(&fit[1], fit_r); }
        carry_g += tot_g; carry_r += tot_r;
    }
    mw_lds_barrier();
    if (tid == 0) { stats->groups_per_hop[h] = fit[0]; stats->rows_per_hop[h] = fit[1]; }
    return err;
}

// Workgroup `wg` of the relay index: wg < n_hops builds child wg's descriptor table, wg == n_hops
// maps rows to groups and does the accounting.  Any workgroup size that is a multiple of 64.
__device__ __forceinline__ void relay_index_body(
    const mw_recv_peer *__restrict__ in, const mw_relay_child *__restrict__ children, int n_hops, int n_ranks,
    uint32_t max_tokens, uint32_t cap, uint64_t row_bytes, const uint64_t *__restrict__ hop_bits,
    int32_t *__restrict__ group_of_row, uint32_t *__restrict__ child_pos, uint32_t *relay_flags,
    mw_relay_stats *__restrict__ stats, const uint32_t keep_metadata, const int wg)
{
    const uint32_t bs = blockDim.x;
    __shared__ uint32_t scratch[17];
    __shared__ uint32_t fit[2];                  // groups, rows of the child that fit its capacity
    __shared__ unsigned long long acc[2];        // rows taken, rows * destinations
    __shared__ uint32_t n_long;
    __shared__ uint32_t long_groups[65536 / kLongGroup];
    const uint32_t tid = threadIdx.x;
    const mw_recv_peer src = in[0];
    const uint32_t G = min(src.n_desc, max_tokens), n_rows = min(src.n_rows, max_tokens);
    uint32_t err = (src.n_desc > max_tokens || src.n_rows > max_tokens) ? MW_FLAG_BAD_DESC : 0u;

    if (wg < n_hops) {
        // ---- child descriptor table of next hop wg: three groups a lane and step where one bitmap
        // word holds every rank, two for two words
        mw_group_desc *cdesc = children[wg].desc;
        if (n_ranks <= 64)
            err |= relay_index_hop<1, 3>(src, G, n_rows, cdesc, wg, n_ranks, cap, hop_bits, child_pos, stats, keep_metadata, scratch, fit);
        else if (n_ranks <= 128)
            err |= relay_index_hop<2, 2>(src, G, n_rows, cdesc, wg, n_ranks, cap, hop_bits, child_pos, stats, keep_metadata, scratch, fit);
        else
            err |= relay_index_hop<MW_MASK_WORDS, 1>(src, G, n_rows, cdesc, wg, n_ranks, cap, hop_bits, child_pos, stats, keep_metadata, scratch, fit);
    } else {
        // ---- rows -> groups, accounting, two groups a lane and step.  A group's thread writes the
        // group's index over its rows; groups longer than kLongGroup rows are queued in LDS and
        // filled by the whole workgroup.  Rows of no valid group keep whatever the array held: the
        // copy kernel checks every entry against the descriptors.
        if (tid < 2) acc[tid] = 0;
        if (tid == 0) n_long = 0;
        mw_lds_barrier();
        uint64_t valid_ranks[MW_MASK_WORDS];
#pragma unroll
        for (int w = 0; w < MW_MASK_WORDS; ++w) valid_ranks[w] = valid_rank_word(n_ranks, w);
        unsigned long long rows_in = 0, dest_rows = 0;
        uint32_t groups_in = 0;
        constexpr int KA = 2;
        for (uint32_t g0 = 0; g0 < G; g0 += bs * KA) {
            const uint32_t gl = g0 + tid * KA;
            uint64_t m[KA][MW_MASK_WORDS];
            uint2 oc[KA];
#pragma unroll
            for (int k = 0; k < KA; ++k) {
                const mw_group_desc *d = src.desc + min(gl + (uint32_t)k, G - 1u);
#pragma unroll
                for (int w = 0; w < MW_MASK_WORDS; ++w) m[k][w] = d->mask[w];
                oc[k] = *(const uint2 *)&d->row_offset;
            }
            const uint2 po = *(const uint2 *)&src.desc[min(gl > 0 ? gl - 1u : 0u, G - 1u)].row_offset;
            uint64_t prev_end = gl > 0 ? (uint64_t)po.x + po.y : 0ull;
#pragma unroll
            for (int k = 0; k < KA; ++k) {
                const uint32_t g = gl + k, off = oc[k].x, cnt = oc[k].y;
                const bool valid = cnt >= 1 && (uint64_t)off + cnt <= n_rows && off >= prev_end;
                prev_end = (uint64_t)off + cnt;
                if (g >= G) continue;
                if (!valid) { err |= MW_FLAG_BAD_DESC; continue; }
                uint32_t nd = 0;
#pragma unroll
                for (int w = 0; w < MW_MASK_WORDS; ++w) {
                    if (m[k][w] & ~valid_ranks[w]) err |= MW_FLAG_BAD_RANK;
                    nd += (uint32_t)__popcll(m[k][w] & valid_ranks[w]);
                }
                if (cnt <= kLongGroup) {
                    for (uint32_t r = 0; r < cnt; ++r) group_of_row[off + r] = (int32_t)g;
                } else {
                    long_groups[atomicAdd(&n_long, 1u)] = g;      // at most max_tokens / kLongGroup of them
                }
                rows_in += cnt; dest_rows += (unsigned long long)cnt * nd; ++groups_in;
            }
        }
        if (rows_in) atomicAdd(&acc[0], rows_in);            // integer sums: order-free
        if (dest_rows) atomicAdd(&acc[1], dest_rows);
        uint32_t tot_groups;
        mw_block_exscan(groups_in, scratch, &tot_groups);     // (its barriers also publish the queue)
        for (uint32_t q = 0; q < n_long; ++q) {
            const uint32_t g = long_groups[q];
            const uint32_t off = src.desc[g].row_offset, cnt = src.desc[g].row_count;
            for (uint32_t r = tid; r < cnt; r += bs) group_of_row[off + r] = (int32_t)g;
        }
        if (tid == 0) {
            stats->n_groups_in = tot_groups;
            stats->n_rows_in = (uint32_t)acc[0];
            stats->unicast_bytes = (uint64_t)acc[1] * row_bytes;
            stats->reserved0 = 0;
        }
        for (int h = n_hops + (int)tid; h < MW_MAX_HOPS; h += (int)bs) { stats->groups_per_hop[h] = 0; stats->rows_per_hop[h] = 0; }
    }
    if (err) atomicOr(relay_flags, err);
}

__global__ __launch_bounds__(kBlock) void k_relay_index(const mw_relay_index_args a)
{
    relay_index_body(a.in, a.children, a.n_hops, a.n_ranks, a.max_tokens, a.cap, a.row_bytes, a.hop_bits,
                     a.group_of_row, a.child_pos, a.relay_flags, a.stats, a.keep_metadata, (int)blockIdx.x);
}

// blockIdx.x selects a segment of blockDim.x chunks of a row; rows i_first, i_first + i_stride, ...
__device__ __forceinline__ void relay_copy_body(
    const mw_recv_peer *__restrict__ in, const mw_relay_child *__restrict__ children, int n_hops, int K, int n_chunks,
    int ns, uint32_t max_tokens, uint64_t row_bytes, const int32_t *__restrict__ group_of_row,
    const uint32_t *__restrict__ child_pos, uint32_t *relay_flags, mw_relay_stats *__restrict__ stats,
    const uint32_t i_first, const uint32_t i_stride)
{
    const mw_recv_peer src = in[0];
    const uint32_t n_rows = min(src.n_rows, max_tokens), n_desc = min(src.n_desc, max_tokens);
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = threadIdx.x & 63;
    for (uint32_t i = i_first; i < n_rows; i += i_stride) {
        // the payload's address depends on the row alone: requested first, the group lookups
        // (two dependent round trips) are in flight beside it
        u32x4 v = {0u, 0u, 0u, 0u};
        if (c < n_chunks) v = mw_ld16((const u32x4 *)src.rows + (size_t)i * ns + c);     // ns: chunks from row to row
        const int32_t st = src.row_src_token[i];
        const int32_t g = group_of_row[i];
        if (g < 0 || (uint32_t)g >= n_desc) continue;        // (stale or never written)
        const uint32_t off = i - src.desc[g].row_offset;
        if (off >= src.desc[g].row_count) continue;          // behind its group's end: in no valid group
        const uint32_t p = (lane < n_hops) ? child_pos[(size_t)g * MW_MAX_HOPS + lane] : kNoChild;
        int32_t tk = 0;
        if ((int)threadIdx.x < K && blockIdx.x == 0) tk = src.row_topk[(size_t)i * K + threadIdx.x];
        uint64_t hops = __ballot(p != kNoChild);              // the same in every wave
        while (hops) {
            const int h = __ffsll((unsigned long long)hops) - 1;
            hops &= hops - 1;
            const uint32_t dst = (uint32_t)__shfl((int)p, h, 64) + off;
            const mw_relay_child ch = children[h];
            if (c < n_chunks) mw_st16((u32x4 *)ch.rows + (size_t)dst * ns + c, v);
            if (blockIdx.x == 0) {
                if (threadIdx.x == 0) ch.row_src_token[dst] = st;
                if ((int)threadIdx.x < K) ch.row_topk[(size_t)dst * K + threadIdx.x] = tk;
            }
        }
    }
    if (blockIdx.x == 0 && i_first == 0 && threadIdx.x == 0) {
        unsigned long long rows_out = 0;
        for (int h = 0; h < n_hops; ++h) rows_out += stats->rows_per_hop[h];
        stats->forward_bytes = rows_out * row_bytes;
        stats->error_flags = __hip_atomic_load(relay_flags, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(relay_flags, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next relay
    }
}

__global__ __launch_bounds__(1024) void k_relay_copy(
    const mw_recv_peer *__restrict__ in, const mw_relay_child *__restrict__ children, int n_hops, int K, int n_chunks,
    int ns, uint32_t max_tokens, uint64_t row_bytes, const int32_t *__restrict__ group_of_row,
    const uint32_t *__restrict__ child_pos, uint32_t *relay_flags, mw_relay_stats *__restrict__ stats)
{
    relay_copy_body(in, children, n_hops, K, n_chunks, ns, max_tokens, row_bytes, group_of_row, child_pos, relay_flags,
                    stats, blockIdx.y, gridDim.y);
}

// A stream of relay steps on one stream (Section 4.3.3; the relay module of Section 5.1 handles
// one buffer after the other): the copy of this step's buffer and, in the first next.n_hops + 1
// workgroup rows of the grid, the index of the NEXT step's buffer, written to another context's
// workspace.  The index is a chain of memory round trips that moves almost nothing; as a launch
// of its own it costs about 15 us in front of every copy.  Held to 64 registers so that the copy
// keeps every wave slot.
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_relay_copy_index_next(
    const uint32_t first_copy_row, const uint32_t unused0,     // (the copy's arguments first: in registers when a wave starts)
    const mw_recv_peer *__restrict__ in, const mw_relay_child *__restrict__ children, int n_hops, int K, int n_chunks,
    int ns, uint32_t max_tokens, uint64_t row_bytes, const int32_t *__restrict__ group_of_row,
    const uint32_t *__restrict__ child_pos, uint32_t *relay_flags, mw_relay_stats *__restrict__ stats,
    const mw_relay_index_args next)
{
    if (blockIdx.y >= first_copy_row) {          // the copy's branch first: nothing to fetch in front of it
        relay_copy_body(in, children, n_hops, K, n_chunks, ns, max_tokens, row_bytes, group_of_row, child_pos,
                        relay_flags, stats, blockIdx.y - first_copy_row, gridDim.y - first_copy_row);
        return;
    }
    if (blockIdx.x == 0)
        relay_index_body(next.in, next.children, next.n_hops, next.n_ranks, next.max_tokens, next.cap, next.row_bytes,
                         next.hop_bits, next.group_of_row, next.child_pos, next.relay_flags, next.stats,
                         next.keep_metadata, (int)blockIdx.y);
}

// Several buffers in one launch (mw_relay_batch): the copies of n_copy buffers, `rows_per_copy`
// grid rows each, behind the index rows of n_index further buffers.  A copy workgroup finds its
// buffer by one division and reads that buffer's arguments from the kernel arguments.
struct mw_relay_copy_args {
    const mw_recv_peer *in; const mw_relay_child *children; const int32_t *group_of_row; const uint32_t *child_pos;
    uint32_t *relay_flags; mw_relay_stats *stats; int n_hops; int reserved0;
};
struct mw_relay_batch_args {
    mw_relay_copy_args copy[MW_RELAY_BATCH_MAX];
    mw_relay_index_args index[MW_RELAY_BATCH_MAX];
    uint32_t index_first_row[MW_RELAY_BATCH_MAX + 1];      // grid rows [first[k], first[k + 1]) index buffer k
};

__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_relay_batch(
    const uint32_t first_copy_row, const uint32_t rows_per_copy, int K, int n_chunks, int ns, uint32_t max_tokens,
    uint64_t row_bytes, const mw_relay_batch_args b)
{
    if (blockIdx.y >= first_copy_row) {
        const uint32_t y = blockIdx.y - first_copy_row, j = y / rows_per_copy;
        const mw_relay_copy_args &c = b.copy[j];
        relay_copy_body(c.in, c.children, c.n_hops, K, n_chunks, ns, max_tokens, row_bytes, c.group_of_row, c.child_pos,
                        c.relay_flags, c.stats, y - j * rows_per_copy, rows_per_copy);
        return;
    }
    if (blockIdx.x != 0) return;
    int k = 0;
#pragma unroll
    for (int q = 1; q < MW_RELAY_BATCH_MAX; ++q) k += (blockIdx.y >= b.index_first_row[q]) ? 1 : 0;
    const mw_relay_index_args &a = b.index[k];
    relay_index_body(a.in, a.children, a.n_hops, a.n_ranks, a.max_tokens, a.cap, a.row_bytes, a.hop_bits, a.group_of_row,
                     a.child_pos, a.relay_flags, a.stats, a.keep_metadata, (int)(blockIdx.y - b.index_first_row[k]));
}

// ---- the same step for packets (Section 4.1, "Replication and forwarding": the relay parses the
// bitmap in front of the payload, makes one copy per distinct egress port and updates the
// in-packet metadata of each copy).  Every packet is its own group, so there is no row -> group
// map: workgroup h ranks the packets that hop h keeps (child position = exclusive count), the
// extra workgroup does the accounting, and the copy kernel reads a packet once and stores it
// once per hop with the first 32 bytes -- the bitmap -- replaced by its restriction to that hop.
// Everything the index of one relay step of packets needs (one kernel argument).
struct mw_relay_packets_index_args {
    const mw_recv_packets *in; int n_hops, n_ranks; uint32_t K, max_tokens, cap; uint64_t packet_bytes;
    const uint64_t *hop_bits; uint32_t *child_pos; uint32_t *relay_flags; mw_relay_stats *stats;
};

// Positions of the packets that next hop h keeps, by one workgroup: KP consecutive packets a
// lane and step, of each header the NW bitmap words that can name a rank and the id count, all
// loads of a step issued before the first is used (as relay_index_hop).
template <int NW, int KP>
__device__ __forceinline__ uint32_t relay_packets_index_hop(
    const char *__restrict__ packets, const uint64_t packet_bytes, const uint32_t n_rows, const uint32_t K, const int h,
    const uint32_t cap, const uint64_t *__restrict__ hop_bits, uint32_t *__restrict__ child_pos,
    mw_relay_stats *__restrict__ stats, uint32_t *scratch)
{
    const uint32_t tid = threadIdx.x, bs = blockDim.x;
    uint32_t err = 0;
    uint64_t hb[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) hb[w] = hop_bits[(size_t)h * MW_MASK_WORDS + w];
    uint32_t carry = 0;
    for (uint32_t i0 = 0; i0 < n_rows; i0 += bs * KP) {
        const uint32_t il = i0 + tid * KP;
        uint64_t m[KP][NW];
        uint32_t nid[KP];
#pragma unroll
        for (int k = 0; k < KP; ++k) {
            const char *hd = packets + (size_t)min(il + (uint32_t)k, n_rows - 1u) * packet_bytes;
#pragma unroll
            for (int w = 0; w < NW; ++w) m[k][w] = *(const uint64_t *)(hd + 8 * w);
            nid[k] = *(const uint32_t *)(hd + 36);
        }
        bool keep[KP];
        uint32_t lk = 0;
#pragma unroll
        for (int k = 0; k < KP; ++k) {
            bool any = false;
#pragma unroll
            for (int w = 0; w < NW; ++w) any |= (m[k][w] & hb[w]) != 0;
            keep[k] = any && il + k < n_rows && nid[k] == K;
            lk += keep[k] ? 1u : 0u;
        }
        uint32_t tot;
        uint32_t pos = carry + mw_block_exscan(lk, scratch, &tot);
#pragma unroll
        for (int k = 0; k < KP; ++k) {
            if (il + k >= n_rows) continue;
            const bool fits = keep[k] && pos < cap;
            if (keep[k] && !fits) err |= MW_FLAG_OUT_CAPACITY;
            child_pos[(size_t)(il + k) * MW_MAX_HOPS + h] = fits ? pos : kNoChild;
            pos += keep[k] ? 1u : 0u;
        }
        carry += tot;
    }
    if (tid == 0) {
        const uint32_t fit = min(carry, cap);      // the packets that fit are a prefix of the kept ones
        stats->groups_per_hop[h] = fit; stats->rows_per_hop[h] = fit;
    }
    return err;
}

// Workgroup `wg` of the packets' relay index (wg < n_hops: hop wg's positions; wg == n_hops: the
// accounting).  Any workgroup size that is a multiple of 64.
__device__ __forceinline__ void relay_packets_index_body(
    const mw_recv_packets *__restrict__ in, int n_hops, int n_ranks, uint32_t K, uint32_t max_tokens, uint32_t cap,
    uint64_t packet_bytes, const uint64_t *__restrict__ hop_bits, uint32_t *__restrict__ child_pos,
    uint32_t *relay_flags, mw_relay_stats *__restrict__ stats, const int wg)
{
    __shared__ uint32_t scratch[17];
    __shared__ unsigned long long acc[2];        // packets taken, destinations named
    const uint32_t tid = threadIdx.x, bs = blockDim.x;
    const mw_recv_packets src = in[0];
    const char *packets = (const char *)src.packets;
    const uint32_t n_rows = min(src.n_rows, max_tokens);
    uint32_t err = src.n_rows > max_tokens ? MW_FLAG_BAD_DESC : 0u;

    if (wg < n_hops) {
        if (n_ranks <= 64)
            err |= relay_packets_index_hop<1, 4>(packets, packet_bytes, n_rows, K, wg, cap, hop_bits, child_pos, stats, scratch);
        else if (n_ranks <= 128)
            err |= relay_packets_index_hop<2, 4>(packets, packet_bytes, n_rows, K, wg, cap, hop_bits, child_pos, stats, scratch);
        else
            err |= relay_packets_index_hop<MW_MASK_WORDS, 2>(packets, packet_bytes, n_rows, K, wg, cap, hop_bits, child_pos, stats, scratch);
    } else {
        if (tid < 2) acc[tid] = 0;
        mw_lds_barrier();
        uint64_t valid_ranks[MW_MASK_WORDS];
#pragma unroll
        for (int w = 0; w < MW_MASK_WORDS; ++w) valid_ranks[w] = valid_rank_word(n_ranks, w);
        uint32_t taken = 0, dests = 0;
        constexpr int KA = 2;                       // two headers a lane in flight
        for (uint32_t i0 = 0; i0 < n_rows; i0 += bs * KA) {
            uint64_t m[KA][MW_MASK_WORDS];
            uint32_t nid[KA];
#pragma unroll
            for (int k = 0; k < KA; ++k) {
                const char *hd = packets + (size_t)min(i0 + k * bs + tid, n_rows - 1u) * packet_bytes;
#pragma unroll
                for (int w = 0; w < MW_MASK_WORDS; ++w) m[k][w] = *(const uint64_t *)(hd + 8 * w);
                nid[k] = *(const uint32_t *)(hd + 36);
            }
#pragma unroll
            for (int k = 0; k < KA; ++k) {
                if (i0 + k * bs + tid >= n_rows) continue;
                if (nid[k] != K) { err |= MW_FLAG_BAD_DESC; continue; }
#pragma unroll
                for (int w = 0; w < MW_MASK_WORDS; ++w) {
                    if (m[k][w] & ~valid_ranks[w]) err |= MW_FLAG_BAD_RANK;
                    dests += (uint32_t)__popcll(m[k][w] & valid_ranks[w]);
                }
                ++taken;
            }
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) { taken += __shfl_xor(taken, d, 64); dests += __shfl_xor(dests, d, 64); }
        if ((tid & 63) == 0) { atomicAdd(&acc[0], (unsigned long long)taken); atomicAdd(&acc[1], (unsigned long long)dests); }
        mw_lds_barrier();
        if (tid == 0) {
            stats->n_groups_in = (uint32_t)acc[0];
            stats->n_rows_in = (uint32_t)acc[0];
            stats->unicast_bytes = (uint64_t)acc[1] * packet_bytes;
            stats->reserved0 = 0;
        }
        for (int h = n_hops + (int)tid; h < MW_MAX_HOPS; h += (int)bs) { stats->groups_per_hop[h] = 0; stats->rows_per_hop[h] = 0; }
    }
    if (err) atomicOr(relay_flags, err);
}

__global__ __launch_bounds__(kBlock) void k_relay_packets_index(const mw_relay_packets_index_args a)
{
    relay_packets_index_body(a.in, a.n_hops, a.n_ranks, a.K, a.max_tokens, a.cap, a.packet_bytes, a.hop_bits,
                             a.child_pos, a.relay_flags, a.stats, (int)blockIdx.x);
}

// blockIdx.x selects a segment of blockDim.x chunks of a packet; packets i_first, i_first + i_stride, ...
__device__ __forceinline__ void relay_packets_copy_body(
    const mw_recv_packets *__restrict__ in, void *const *__restrict__ children, int n_hops, int n_chunks,
    uint32_t max_tokens, uint64_t packet_bytes, const uint64_t *__restrict__ hop_bits,
    const uint32_t *__restrict__ child_pos, uint32_t *relay_flags, mw_relay_stats *__restrict__ stats,
    const uint32_t keep_metadata, const uint32_t i_first, const uint32_t i_stride)
{
    const mw_recv_packets src = in[0];
    const uint32_t n_rows = min(src.n_rows, max_tokens);
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = threadIdx.x & 63;
    for (uint32_t i = i_first; i < n_rows; i += i_stride) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (c < n_chunks) v = mw_ld16((const u32x4 *)src.packets + (size_t)i * n_chunks + c);
        const uint32_t p = (lane < n_hops) ? child_pos[(size_t)i * MW_MAX_HOPS + lane] : kNoChild;
        uint64_t hops = __ballot(p != kNoChild);              // the same in every wave
        while (hops) {
            const int h = __ffsll((unsigned long long)hops) - 1;
            hops &= hops - 1;
            const uint32_t dst = (uint32_t)__shfl((int)p, h, 64);
            u32x4 o = v;
            if (c < 2 && !keep_metadata) {                    // chunks 0 and 1 are the bitmap: restricted to the hop's ranks
                const uint64_t b0 = hop_bits[(size_t)h * MW_MASK_WORDS + 2 * c];
                const uint64_t b1 = hop_bits[(size_t)h * MW_MASK_WORDS + 2 * c + 1];
                o.x &= (uint32_t)b0; o.y &= (uint32_t)(b0 >> 32); o.z &= (uint32_t)b1; o.w &= (uint32_t)(b1 >> 32);
            }
            if (c < n_chunks) mw_st16((u32x4 *)children[h] + (size_t)dst * n_chunks + c, o);
        }
    }
    if (blockIdx.x == 0 && i_first == 0 && threadIdx.x == 0) {
        unsigned long long rows_out = 0;
        for (int h = 0; h < n_hops; ++h) rows_out += stats->rows_per_hop[h];
        stats->forward_bytes = rows_out * packet_bytes;
        stats->error_flags = __hip_atomic_load(relay_flags, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(relay_flags, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next relay
    }
}

__global__ __launch_bounds__(1024) void k_relay_packets_copy(
    const mw_recv_packets *__restrict__ in, void *const *__restrict__ children, int n_hops, int n_chunks,
    uint32_t max_tokens, uint64_t packet_bytes, const uint64_t *__restrict__ hop_bits,
    const uint32_t *__restrict__ child_pos, uint32_t *relay_flags, mw_relay_stats *__restrict__ stats,
    const uint32_t keep_metadata)
{
    relay_packets_copy_body(in, children, n_hops, n_chunks, max_tokens, packet_bytes, hop_bits, child_pos, relay_flags,
                            stats, keep_metadata, blockIdx.y, gridDim.y);
}

// The packets' form of k_relay_copy_index_next: this buffer's copy with the next buffer's index
// (another context's workspace) in the first next.n_hops + 1 workgroup rows.  Held to 64 scalar
// registers as well: with the 69 the index's branch would take, the copy's step is 6 % longer
// (56.9 -> 60.4 us; forcing the count up with nothing else changed shows the same), the four
// values over the limit live in lanes of a vector register instead.
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(8, 8), amdgpu_num_sgpr(64))) void k_relay_packets_copy_index_next(
    const uint32_t first_copy_row, const uint32_t unused0,
    const mw_recv_packets *__restrict__ in, void *const *__restrict__ children, int n_hops, int n_chunks,
    uint32_t max_tokens, uint64_t packet_bytes, const uint64_t *__restrict__ hop_bits,
    const uint32_t *__restrict__ child_pos, uint32_t *relay_flags, mw_relay_stats *__restrict__ stats,
    const uint32_t keep_metadata, const mw_relay_packets_index_args next)
{
    if (blockIdx.y >= first_copy_row) {
        relay_packets_copy_body(in, children, n_hops, n_chunks, max_tokens, packet_bytes, hop_bits, child_pos,
                                relay_flags, stats, keep_metadata, blockIdx.y - first_copy_row,
                                gridDim.y - first_copy_row);
        return;
    }
    if (blockIdx.x == 0)
        relay_packets_index_body(next.in, next.n_hops, next.n_ranks, next.K, next.max_tokens, next.cap,
                                 next.packet_bytes, next.hop_bits, next.child_pos, next.relay_flags, next.stats,
                                 (int)blockIdx.y);
}

}  // namespace

// Workgroup shape of a copy that carries a riding index, for long rows that would otherwise move
// as single waves.  The index walks the groups a workgroup's width at a time (one memory round
// trip and two scans per step: 128 lanes took 32 steps for 4096 groups and outlasted the copy by
// half) and its 8 KiB of LDS per workgroup would leave a CU of single-wave workgroups 19 waves
// instead of 32, so the launch wants wide workgroups; the copy wants narrow ones.  Measured on
// 14336-byte rows (per step of a stream, 15 next hops): 128 lanes 80 us, 192: 67, 256: 63, 320: 55.3,
// 384: 55.8, 448: 57.4, 512: 61, 896: 57.2.  An even number of unequal segments would hand the short
// segment to the same XCDs every row (256 lanes: four segments, the last half empty).
static mw_row_shape relay_stream_shape(int n_chunks)
{
    int nseg = (n_chunks + 383) / 384;
    if (nseg > 1 && nseg % 2 == 0) ++nseg;
    return mw_row_shape{((n_chunks + nseg - 1) / nseg + 63) / 64 * 64, nseg};
}

static mw_relay_index_args relay_index_args(mw_ctx *ctx, const mw_recv_peer *in, const mw_relay_child *children,
                                            int64_t cap, mw_relay_stats *stats)
{
    mw_relay_index_args a;
    a.in = in; a.children = children; a.n_hops = ctx->n_hops; a.n_ranks = ctx->cfg.n_ranks;
    a.max_tokens = (uint32_t)ctx->cfg.max_tokens; a.cap = (uint32_t)cap; a.row_bytes = (uint64_t)ctx->row_bytes;
    a.hop_bits = ctx->d_hop_bits; a.group_of_row = ctx->d_group_of_row; a.child_pos = ctx->d_child_pos;
    a.relay_flags = ctx->d_relay_flags; a.stats = stats;
    a.keep_metadata = (ctx->options & MW_OPT_RELAY_KEEP_METADATA) ? 1u : 0u;
    return a;
}

int32_t mw_launch_relay_index(mw_ctx *ctx, const mw_recv_peer *in, const mw_relay_child *children, int64_t cap,
                              mw_relay_stats *stats, hipStream_t s)
{
    {
        mw_timed tm(ctx, MW_KERNEL_RELAY_INDEX, s);
        hipLaunchKernelGGL(k_relay_index, dim3(ctx->n_hops + 1), dim3(kBlock), 0, s,
                           relay_index_args(ctx, in, children, cap, stats));
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

// `next` != nullptr: the index of the next step's buffer rides in the same launch.
int32_t mw_launch_relay_copy(mw_ctx *ctx, const mw_recv_peer *in, const mw_relay_child *children,
                             mw_relay_stats *stats, mw_ctx *next, const mw_recv_peer *next_in,
                             const mw_relay_child *next_children, int64_t next_cap, mw_relay_stats *next_stats,
                             hipStream_t s)
{
    const mw_config &c = ctx->cfg;
    const int n_chunks = (int)(ctx->row_bytes / 16);
    mw_row_shape shape = mw_row_shape_of(n_chunks);
    uint32_t gy = (uint32_t)c.max_tokens < kRowGridMax ? (uint32_t)c.max_tokens : kRowGridMax;
    if (gy < 1) gy = 1;
    {
        mw_timed tm(ctx, MW_KERNEL_RELAY_COPY, s);
        if (!next) {
            hipLaunchKernelGGL(k_relay_copy, dim3(shape.nseg, gy), dim3(shape.bs), 0, s, in, children, ctx->n_hops,
                               c.top_k, n_chunks, (int)(ctx->row_stride / 16), (uint32_t)c.max_tokens,
                               (uint64_t)ctx->row_bytes, ctx->d_group_of_row, ctx->d_child_pos, ctx->d_relay_flags, stats);
        } else {
            if (shape.bs == 64 && n_chunks % 16 == 0) shape = relay_stream_shape(n_chunks);
            hipLaunchKernelGGL(k_relay_copy_index_next, dim3(shape.nseg, gy + (uint32_t)next->n_hops + 1u),
                               dim3(shape.bs), 0, s, (uint32_t)next->n_hops + 1u, 0u, in, children, ctx->n_hops, c.top_k, n_chunks,
                               (int)(ctx->row_stride / 16), (uint32_t)c.max_tokens, (uint64_t)ctx->row_bytes,
                               ctx->d_group_of_row, ctx->d_child_pos, ctx->d_relay_flags, stats,
                               relay_index_args(next, next_in, next_children, next_cap, next_stats));
        }
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

int32_t mw_launch_relay_batch(const mw_relay_job *copy, int32_t n_copy, const mw_relay_job *index, int32_t n_index,
                              hipStream_t s)
{
    mw_ctx *ctx = copy[0].ctx;
    const mw_config &c = ctx->cfg;
    const int n_chunks = (int)(ctx->row_bytes / 16);
    mw_row_shape shape = mw_row_shape_of(n_chunks);
    // long rows of whole cache lines: a few large workgroups per row beside a riding index (see mw_launch_relay_copy)
    if (n_index > 0 && shape.bs == 64 && n_chunks % 16 == 0) shape = relay_stream_shape(n_chunks);
    uint32_t gy = (uint32_t)c.max_tokens < 8192u ? (uint32_t)c.max_tokens : 8192u;      // per buffer; more rows by striding
    if (gy < 1) gy = 1;
    mw_relay_batch_args b = {};
    for (int j = 0; j < n_copy; ++j) {
        mw_ctx *x = copy[j].ctx;
        b.copy[j] = mw_relay_copy_args{copy[j].in_dev, copy[j].children_dev, x->d_group_of_row, x->d_child_pos,
                                       x->d_relay_flags, copy[j].stats_dev, x->n_hops, 0};
    }
    uint32_t first = 0;
    for (int k = 0; k < MW_RELAY_BATCH_MAX; ++k) {
        b.index_first_row[k] = first;
        if (k < n_index) {
            b.index[k] = relay_index_args(index[k].ctx, index[k].in_dev, index[k].children_dev,
                                          index[k].child_capacity_rows, index[k].stats_dev);
            first += (uint32_t)index[k].ctx->n_hops + 1u;
        }
    }
    b.index_first_row[MW_RELAY_BATCH_MAX] = first;
    {
        mw_timed tm(ctx, MW_KERNEL_RELAY_COPY, s);
        hipLaunchKernelGGL(k_relay_batch, dim3(shape.nseg, first + gy * (uint32_t)n_copy), dim3(shape.bs), 0, s, first, gy,
                           c.top_k, n_chunks, (int)(ctx->row_stride / 16), (uint32_t)c.max_tokens,
                           (uint64_t)ctx->row_bytes, b);
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

int32_t mw_launch_relay(mw_ctx *ctx, const mw_recv_peer *in, const mw_relay_child *children, int64_t cap,
                        mw_relay_stats *stats, hipStream_t s)
{
    const int32_t rc = mw_launch_relay_index(ctx, in, children, cap, stats, s);
    if (rc != MW_OK) return rc;
    return mw_launch_relay_copy(ctx, in, children, stats, nullptr, nullptr, nullptr, 0, nullptr, s);
}

static mw_relay_packets_index_args relay_packets_index_args(mw_ctx *ctx, const mw_recv_packets *in, int64_t cap,
                                                            mw_relay_stats *stats)
{
    mw_relay_packets_index_args a;
    a.in = in; a.n_hops = ctx->n_hops; a.n_ranks = ctx->cfg.n_ranks; a.K = (uint32_t)ctx->cfg.top_k;
    a.max_tokens = (uint32_t)ctx->cfg.max_tokens; a.cap = (uint32_t)cap;
    a.packet_bytes = (uint64_t)(mw_packet_header_bytes_of(ctx->cfg.top_k) + ctx->row_bytes);
    a.hop_bits = ctx->d_hop_bits; a.child_pos = ctx->d_child_pos; a.relay_flags = ctx->d_relay_flags; a.stats = stats;
    return a;
}

int32_t mw_launch_relay_packets_index(mw_ctx *ctx, const mw_recv_packets *in, int64_t cap, mw_relay_stats *stats,
                                      hipStream_t s)
{
    {
        mw_timed tm(ctx, MW_KERNEL_RELAY_INDEX, s);
        hipLaunchKernelGGL(k_relay_packets_index, dim3(ctx->n_hops + 1), dim3(kBlock), 0, s,
                           relay_packets_index_args(ctx, in, cap, stats));
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

// `next` != nullptr: the index of the next step's packets rides in the same launch.
int32_t mw_launch_relay_packets_copy(mw_ctx *ctx, const mw_recv_packets *in, void *const *children,
                                     mw_relay_stats *stats, mw_ctx *next, const mw_recv_packets *next_in,
                                     int64_t next_cap, mw_relay_stats *next_stats, hipStream_t s)
{
    const mw_config &c = ctx->cfg;
    const uint64_t pb = (uint64_t)(mw_packet_header_bytes_of(c.top_k) + ctx->row_bytes);
    const int n_chunks = (int)(pb / 16);
    const uint32_t keep = (ctx->options & MW_OPT_RELAY_KEEP_METADATA) ? 1u : 0u;
    mw_row_shape shape = mw_row_shape_of(n_chunks);
    uint32_t gy = (uint32_t)c.max_tokens < kRowGridMax ? (uint32_t)c.max_tokens : kRowGridMax;
    if (gy < 1) gy = 1;
    {
        mw_timed tm(ctx, MW_KERNEL_RELAY_COPY, s);
        if (!next) {
            hipLaunchKernelGGL(k_relay_packets_copy, dim3(shape.nseg, gy), dim3(shape.bs), 0, s, in, children, ctx->n_hops,
                               n_chunks, (uint32_t)c.max_tokens, pb, ctx->d_hop_bits, ctx->d_child_pos,
                               ctx->d_relay_flags, stats, keep);
        } else {
            // long packets: a few larger workgroups per packet instead of single waves, for the
            // riding index's sake (see relay_stream_shape); pieces stay whole cache lines
            if (shape.bs == 64) shape = relay_stream_shape(n_chunks);
            hipLaunchKernelGGL(k_relay_packets_copy_index_next, dim3(shape.nseg, gy + (uint32_t)next->n_hops + 1u),
                               dim3(shape.bs), 0, s, (uint32_t)next->n_hops + 1u, 0u, in, children, ctx->n_hops, n_chunks, (uint32_t)c.max_tokens, pb,
                               ctx->d_hop_bits, ctx->d_child_pos, ctx->d_relay_flags, stats, keep,
                               relay_packets_index_args(next, next_in, next_cap, next_stats));
        }
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

int32_t mw_launch_relay_packets(mw_ctx *ctx, const mw_recv_packets *in, void *const *children, int64_t cap,
                                mw_relay_stats *stats, hipStream_t s)
{
    const int32_t rc = mw_launch_relay_packets_index(ctx, in, cap, stats, s);
    if (rc != MW_OK) return rc;
    return mw_launch_relay_packets_copy(ctx, in, children, stats, nullptr, nullptr, 0, nullptr, s);
}
