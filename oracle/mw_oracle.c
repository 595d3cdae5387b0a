/*
 * mw_oracle.c -- plain, slow, single-threaded CPU oracle for one rank's share
 * of a MultiWrite dispatch (MoE AlltoAll) or AllGather.
 *
 * THIS IS TEST INFRASTRUCTURE.  Only the tests, the smoke check and the
 * cpu_baseline leg of the benchmark may build, load or call it.  It shares no
 * code, header, table or helper with the HIP library: the record layouts
 * below are typed out again here on purpose.
 *
 * What the paper fixes (and this file follows):
 *   - Section 4.3.1: MultiWrite(S, M, B_S) writes the content of the source
 *     buffer to the target buffer at every destination in M.  For a dispatch
 *     this means: every token reaches every rank that hosts one of its top-k
 *     experts, and what arrives is exactly what one unicast write per
 *     destination would have delivered (Section 4.3.4, "drop-in replacement").
 *   - Section 4.1, "Encoding scheme of metadata": destinations are a
 *     fixed-size bitmap indexed by rank, ranks numbered from zero, bit r set
 *     iff rank r is a target; a preconfigured table maps addresses (here:
 *     expert ids) to ranks.  Section 6.4 allows wider bitmaps for more than
 *     64 ranks.
 *   - Section 1 / Section 2.3.2: one copy of the data is injected however
 *     many destinations it has; unicast injects one copy per destination.
 *   - Section 4.1 workflow steps 3-4: the receiver parses the carried
 *     metadata and, if it is one of the destinations, delivers the payload.
 *   - Section 5.2: AllGather, every rank's fragment ends up at every rank.
 * What the paper leaves open (order of groups, record layouts, tie-breaks)
 * is fixed by the reading stated next to each function.
 *
 * Two independent derivations of the receive-side result live here:
 *   tier 1  ref_dispatch_plain(): the plain definition, straight from
 *           (peer, token, top-k) with no bitmaps, groups or packed buffers;
 *   tier 2  ref_plan -> ref_pack -> ref_deliver -> ref_unpack: the method's
 *           steps.  The tests require both to agree bytewise.
 *
 * Pins (tests/test_oracle_*.py): brute force on tiny inputs written
 * separately in Python, closed forms for E[popcount], the K=1 case against a
 * library stable sort (plain AlltoAllV), the all-equal-mask case against
 * memcpy, AllGather against array concatenation, the (token, destination)
 * exactly-once property, tier 1 == tier 2, and the paper's printed
 * arithmetic (C(64,8), 128 B vs 8 B metadata, 128 B / 4096 B).  The relay
 * step (ref_relay_child, ref_relay_accounting) is pinned in
 * tests/test_oracle_relay.py: children partition every parent bitmap, an
 * identity forwarding table reduces to ref_deliver with single-bit bitmaps,
 * a one-hop table returns the parent, delivery through relays equals direct
 * delivery bytewise, and the copy count against a closed form.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define REF_OK            0
#define REF_ERR_ARG      -1
#define REF_ERR_EXPERT   -2   /* expert id outside {-1} U [0, E) */
#define REF_ERR_CAPACITY -3
#define REF_ERR_INPUT    -4   /* inconsistent received buffer */

#define REF_MASK_WORDS 4      /* 256-bit destination bitmap, word w bit b <-> rank 64*w + b */
#define REF_MAX_RANKS  256

typedef struct {
    uint64_t mask[REF_MASK_WORDS];
    uint32_t row_offset;      /* first packed row of the group */
    uint32_t row_count;       /* rows in the group */
    uint32_t n_dest;          /* popcount(mask) */
    uint32_t reserved0;       /* always 0 */
} ref_group_desc;             /* 48 bytes */

typedef struct {
    uint32_t n_rows;          /* N: tokens with a non-empty destination set */
    uint32_t n_groups;        /* G */
    uint64_t multicast_bytes; /* N * row_bytes */
    uint64_t unicast_bytes;   /* row_bytes * sum over tokens of |destination set| */
    uint32_t rows_per_dest[REF_MAX_RANKS];
    uint32_t error_flags;     /* oracle: always 0 (it returns errors instead) */
    uint32_t reserved0;
} ref_send_stats;             /* 1056 bytes */

typedef struct {
    const ref_group_desc *desc;
    uint32_t n_desc;
    uint32_t n_rows;
    const uint8_t *rows;           /* [n_rows][row_bytes] */
    const int32_t *row_src_token;  /* [n_rows] */
    const int32_t *row_topk;       /* [n_rows][K] */
} ref_recv_peer;

typedef struct {
    const int32_t *topk;      /* [n_tokens][K] */
    int32_t n_tokens;
    const uint8_t *x;         /* [n_tokens][x_row_bytes]; rows not routed to this rank are never read */
    const uint8_t *scales;    /* [n_tokens][s_row_bytes] or NULL when s_row_bytes == 0 */
} ref_peer_tokens;

/* ------------------------------------------------------------------------ */
static int mask_bit(const uint64_t *m, int r) { return (int)((m[r >> 6] >> (r & 63)) & 1u); }

static int mask_popcount(const uint64_t *m)
{
    int n = 0;
    for (int r = 0; r < REF_MAX_RANKS; ++r) n += mask_bit(m, r);
    return n;
}

/* compare as unsigned 256-bit integers, word 3 most significant */
static int mask_cmp(const uint64_t *a, const uint64_t *b)
{
    for (int w = REF_MASK_WORDS - 1; w >= 0; --w) {
        if (a[w] < b[w]) return -1;
        if (a[w] > b[w]) return 1;
    }
    return 0;
}

/*
 * Destination bitmap of every token (Section 4.1, bitmap encoding): bit
 * expert_to_rank[e] is set for every valid id e in the token's top-k list.
 * -1 means "no expert" and is skipped; duplicates set the same bit again.
 */
int ref_masks(const int32_t *topk, int32_t T, int32_t K,
              const int32_t *expert_to_rank, int32_t E, int32_t R,
              uint64_t *mask /* [T][4] */)
{
    if (R < 1 || R > REF_MAX_RANKS || T < 0 || K < 1 || E < 0) return REF_ERR_ARG;
    for (int32_t e = 0; e < E; ++e)
        if (expert_to_rank[e] < 0 || expert_to_rank[e] >= R) return REF_ERR_ARG;
    for (int32_t t = 0; t < T; ++t) {
        uint64_t *m = mask + (size_t)t * REF_MASK_WORDS;
        m[0] = m[1] = m[2] = m[3] = 0;
        for (int32_t j = 0; j < K; ++j) {
            int32_t e = topk[(size_t)t * K + j];
            if (e == -1) continue;
            if (e < 0 || e >= E) return REF_ERR_EXPERT;
            int32_t r = expert_to_rank[e];
            m[r >> 6] |= (uint64_t)1 << (r & 63);
        }
    }
    return REF_OK;
}

typedef struct { const uint64_t *mask; int32_t token; } sort_item;

static int sort_item_cmp(const void *pa, const void *pb)
{
    const sort_item *a = (const sort_item *)pa, *b = (const sort_item *)pb;
    int c = mask_cmp(a->mask, b->mask);
    if (c) return c;
    return (a->token > b->token) - (a->token < b->token);
}

/*
 * Send-side plan.  Tokens with an empty destination set are dropped; the
 * others are ordered by (bitmap as an unsigned 256-bit integer, token index),
 * both ascending.  A multicast group is a maximal run of equal bitmaps in
 * that order: one descriptor per group, in that order.  Accounting follows
 * Section 1: multicast injects each packed row once, unicast once per
 * destination rank.
 */
int ref_plan(const int32_t *topk, int32_t T, int32_t K,
             const int32_t *expert_to_rank, int32_t E, int32_t R, int64_t row_bytes,
             uint64_t *mask /* [T][4] out */, int32_t *perm /* [T] out, first N used */,
             ref_group_desc *desc /* [T] out, first G used */, ref_send_stats *stats)
{
    int rc = ref_masks(topk, T, K, expert_to_rank, E, R, mask);
    if (rc != REF_OK) return rc;

    sort_item *items = (sort_item *)malloc(sizeof(sort_item) * (size_t)(T > 0 ? T : 1));
    if (!items) return REF_ERR_CAPACITY;
    int32_t N = 0;
    for (int32_t t = 0; t < T; ++t) {
        const uint64_t *m = mask + (size_t)t * REF_MASK_WORDS;
        if (m[0] | m[1] | m[2] | m[3]) { items[N].mask = m; items[N].token = t; ++N; }
    }
    qsort(items, (size_t)N, sizeof(sort_item), sort_item_cmp);   /* keys are unique: (mask, token) */

    memset(stats, 0, sizeof(*stats));
    int32_t G = 0;
    uint64_t dest_total = 0;
    for (int32_t i = 0; i < N; ++i) {
        perm[i] = items[i].token;
        if (i == 0 || mask_cmp(items[i].mask, items[i - 1].mask) != 0) {
            ref_group_desc *d = &desc[G++];
            memcpy(d->mask, items[i].mask, sizeof(d->mask));
            d->row_offset = (uint32_t)i;
            d->row_count = 0;
            d->n_dest = (uint32_t)mask_popcount(items[i].mask);
            d->reserved0 = 0;
        }
        desc[G - 1].row_count += 1;
        for (int r = 0; r < REF_MAX_RANKS; ++r)
            if (mask_bit(items[i].mask, r)) { stats->rows_per_dest[r] += 1; dest_total += 1; }
    }
    stats->n_rows = (uint32_t)N;
    stats->n_groups = (uint32_t)G;
    stats->multicast_bytes = (uint64_t)N * (uint64_t)row_bytes;
    stats->unicast_bytes = dest_total * (uint64_t)row_bytes;
    free(items);
    return REF_OK;
}

/*
 * Accounting written straight from the statement of the problem, without
 * bitmaps: for every token collect the distinct ranks of its experts.
 */
int ref_accounting_plain(const int32_t *topk, int32_t T, int32_t K,
                         const int32_t *expert_to_rank, int32_t E, int32_t R, int64_t row_bytes,
                         uint64_t *multicast_bytes, uint64_t *unicast_bytes,
                         uint32_t *rows_per_dest /* [256] */)
{
    if (R < 1 || R > REF_MAX_RANKS || K < 1) return REF_ERR_ARG;
    int32_t *seen = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);
    if (!seen) return REF_ERR_CAPACITY;
    *multicast_bytes = 0; *unicast_bytes = 0;
    memset(rows_per_dest, 0, sizeof(uint32_t) * REF_MAX_RANKS);
    for (int32_t t = 0; t < T; ++t) {
        int n = 0;
        for (int32_t j = 0; j < K; ++j) {
            int32_t e = topk[(size_t)t * K + j];
            if (e == -1) continue;
            if (e < 0 || e >= E) { free(seen); return REF_ERR_EXPERT; }
            int32_t r = expert_to_rank[e], dup = 0;
            for (int i = 0; i < n; ++i) dup |= (seen[i] == r);
            if (!dup) seen[n++] = r;
        }
        if (n > 0) *multicast_bytes += (uint64_t)row_bytes;
        *unicast_bytes += (uint64_t)n * (uint64_t)row_bytes;
        for (int i = 0; i < n; ++i) rows_per_dest[seen[i]] += 1;
    }
    free(seen);
    return REF_OK;
}

/*
 * Pack: each kept token's payload is written once, in plan order (Section 1:
 * only one copy of the same data is sent).  A packed row is the token's
 * x bytes followed by its scale bytes (fp8: H e4m3 codes then H/128 fp32
 * scales; bf16: 2H bytes and no scales).  The metadata a receiver needs
 * travels with the row (Section 4.3.4, statelessness): the source token
 * index and the token's top-k ids, copied unchanged.
 */
int ref_pack(const uint8_t *x, int64_t x_row_bytes, const uint8_t *scales, int64_t s_row_bytes,
             const int32_t *topk, int32_t K, const int32_t *perm, int32_t N,
             uint8_t *packed /* [N][x_row_bytes + s_row_bytes] */,
             int32_t *row_src_token /* [N] */, int32_t *row_topk /* [N][K] */)
{
    if (x_row_bytes < 0 || s_row_bytes < 0 || (s_row_bytes > 0 && !scales)) return REF_ERR_ARG;
    const int64_t rb = x_row_bytes + s_row_bytes;
    for (int32_t i = 0; i < N; ++i) {
        const int32_t t = perm[i];
        uint8_t *dst = packed + (size_t)i * (size_t)rb;
        memcpy(dst, x + (size_t)t * (size_t)x_row_bytes, (size_t)x_row_bytes);
        if (s_row_bytes > 0)
            memcpy(dst + x_row_bytes, scales + (size_t)t * (size_t)s_row_bytes, (size_t)s_row_bytes);
        row_src_token[i] = t;
        for (int32_t j = 0; j < K; ++j) row_topk[(size_t)i * K + j] = topk[(size_t)t * K + j];
    }
    return REF_OK;
}

/*
 * Simulated network: what rank `dst_rank` receives from one sender
 * (Section 4.1 workflow step 4: a payload is delivered only to nodes named
 * in its bitmap).  Groups whose bitmap has bit dst_rank are kept, in order,
 * their rows concatenated and row_offset rebased; bitmaps are left as sent.
 */
int ref_deliver(const ref_group_desc *desc, int32_t G, const uint8_t *rows, int64_t row_bytes,
                const int32_t *row_src_token, const int32_t *row_topk, int32_t K, int32_t dst_rank,
                ref_group_desc *desc_out, uint8_t *rows_out, int32_t *src_token_out, int32_t *topk_out,
                int32_t *G_out, int32_t *N_out)
{
    if (dst_rank < 0 || dst_rank >= REF_MAX_RANKS) return REF_ERR_ARG;
    int32_t g2 = 0, n2 = 0;
    for (int32_t g = 0; g < G; ++g) {
        if (!mask_bit(desc[g].mask, dst_rank)) continue;
        desc_out[g2] = desc[g];
        desc_out[g2].row_offset = (uint32_t)n2;
        for (uint32_t i = 0; i < desc[g].row_count; ++i) {
            const size_t s = (size_t)desc[g].row_offset + i;
            memcpy(rows_out + (size_t)n2 * (size_t)row_bytes, rows + s * (size_t)row_bytes, (size_t)row_bytes);
            src_token_out[n2] = row_src_token[s];
            for (int32_t j = 0; j < K; ++j) topk_out[(size_t)n2 * K + j] = row_topk[s * K + j];
            ++n2;
        }
        ++g2;
    }
    *G_out = g2; *N_out = n2;
    return REF_OK;
}

/* ------------------------------------------------------------------------ */
/*
 * Relay step.  Section 4.3.3 (recursive execution model): a node that holds
 * a MultiWrite for a destination set M partitions M by next hop and starts
 * one child MultiWrite per subset; |M_i| == 1 is an ordinary write.
 * Section 4.1, "Local forwarding table": the next hop of every destination
 * comes from the node's unicast forwarding table, and the number of distinct
 * next hops is the number of copies made.  Section 4.1, "Replication and
 * forwarding": the metadata of each copy is updated so that it names only
 * the destinations served through that hop -- no destination is served twice.
 *
 * Reading used here (the paper gives no buffer format): `next_hop[r]` in
 * [0, n_hops) is the forwarding table entry of destination rank r.  The child
 * for hop h keeps, in the parent's order, the groups whose bitmap names at
 * least one rank with next_hop == h; the child's bitmap is the parent's
 * restricted to those ranks, its rows are the group's rows concatenated,
 * row_offset is rebased, n_dest is the popcount of the restricted bitmap.
 * Row metadata is copied unchanged.  A destination named by a bitmap whose
 * rank is >= n_ranks is an input error.
 */
int ref_relay_child(const ref_group_desc *desc, int32_t G, const uint8_t *rows, int64_t row_bytes,
                    const int32_t *row_src_token, const int32_t *row_topk, int32_t K,
                    const int32_t *next_hop, int32_t R, int32_t n_hops, int32_t hop,
                    ref_group_desc *desc_out, uint8_t *rows_out, int32_t *src_token_out, int32_t *topk_out,
                    int32_t *G_out, int32_t *N_out)
{
    if (R < 1 || R > REF_MAX_RANKS || n_hops < 1 || hop < 0 || hop >= n_hops) return REF_ERR_ARG;
    for (int32_t r = 0; r < R; ++r)
        if (next_hop[r] < 0 || next_hop[r] >= n_hops) return REF_ERR_ARG;
    int32_t g2 = 0, n2 = 0;
    for (int32_t g = 0; g < G; ++g) {
        uint64_t sub[REF_MASK_WORDS] = {0, 0, 0, 0};
        int n_sub = 0;
        for (int r = 0; r < REF_MAX_RANKS; ++r) {
            if (!mask_bit(desc[g].mask, r)) continue;
            if (r >= R) return REF_ERR_INPUT;
            if (next_hop[r] != hop) continue;
            sub[r >> 6] |= (uint64_t)1 << (r & 63);
            ++n_sub;
        }
        if (n_sub == 0) continue;
        for (int w = 0; w < REF_MASK_WORDS; ++w) desc_out[g2].mask[w] = sub[w];
        desc_out[g2].row_offset = (uint32_t)n2;
        desc_out[g2].row_count = desc[g].row_count;
        desc_out[g2].n_dest = (uint32_t)n_sub;
        desc_out[g2].reserved0 = 0;
        for (uint32_t i = 0; i < desc[g].row_count; ++i) {
            const size_t s = (size_t)desc[g].row_offset + i;
            memcpy(rows_out + (size_t)n2 * (size_t)row_bytes, rows + s * (size_t)row_bytes, (size_t)row_bytes);
            src_token_out[n2] = row_src_token[s];
            for (int32_t j = 0; j < K; ++j) topk_out[(size_t)n2 * K + j] = row_topk[s * K + j];
            ++n2;
        }
        ++g2;
    }
    *G_out = g2; *N_out = n2;
    return REF_OK;
}

/*
 * Copies a relay makes, plainly (Section 4.1, local forwarding table): per
 * group, one copy for every distinct next hop among its destinations.
 *   forward_bytes = row_bytes * sum over groups of rows * distinct hops
 *   unicast_bytes = row_bytes * sum over groups of rows * destinations
 *   rows_per_hop[h] = rows of the groups that use hop h
 */
int ref_relay_accounting(const ref_group_desc *desc, int32_t G, int64_t row_bytes,
                         const int32_t *next_hop, int32_t R, int32_t n_hops,
                         uint64_t *forward_bytes, uint64_t *unicast_bytes, uint32_t *rows_per_hop /* [n_hops] */)
{
    if (R < 1 || R > REF_MAX_RANKS || n_hops < 1) return REF_ERR_ARG;
    for (int32_t r = 0; r < R; ++r)
        if (next_hop[r] < 0 || next_hop[r] >= n_hops) return REF_ERR_ARG;
    uint64_t fwd = 0, uni = 0;
    for (int32_t h = 0; h < n_hops; ++h) rows_per_hop[h] = 0;
    for (int32_t g = 0; g < G; ++g) {
        int n_dest = 0;
        for (int32_t h = 0; h < n_hops; ++h) {
            int used = 0;
            for (int r = 0; r < R; ++r)
                if (mask_bit(desc[g].mask, r) && next_hop[r] == h) used = 1;
            if (used) { rows_per_hop[h] += desc[g].row_count; fwd += desc[g].row_count; }
        }
        for (int r = 0; r < REF_MAX_RANKS; ++r) {
            if (!mask_bit(desc[g].mask, r)) continue;
            if (r >= R) return REF_ERR_INPUT;
            ++n_dest;
        }
        uni += (uint64_t)desc[g].row_count * (uint64_t)n_dest;
    }
    *forward_bytes = fwd * (uint64_t)row_bytes;
    *unicast_bytes = uni * (uint64_t)row_bytes;
    return REF_OK;
}

/* slot of expert e among the experts hosted by `rank`, in ascending id order; -1 if elsewhere */
static int32_t local_slot_of(const int32_t *expert_to_rank, int32_t e, int32_t rank)
{
    if (expert_to_rank[e] != rank) return -1;
    int32_t s = 0;
    for (int32_t f = 0; f < e; ++f) s += (expert_to_rank[f] == rank);
    return s;
}

/*
 * Relay step WITHOUT the metadata update (Section 4.1, last paragraph of
 * "Replication and forwarding": where routing loops cannot occur and the end
 * nodes drop repeated packets, a relay may forward the metadata as it came).
 * The child for hop h keeps the same groups, rows and row metadata as
 * ref_relay_child -- the copies made are the same -- but every kept group
 * carries the PARENT's bitmap and its popcount: a node further down sees all
 * the original destinations, the ones served over other hops included.
 */
int ref_relay_child_unmodified(const ref_group_desc *desc, int32_t G, const uint8_t *rows, int64_t row_bytes,
                               const int32_t *row_src_token, const int32_t *row_topk, int32_t K,
                               const int32_t *next_hop, int32_t R, int32_t n_hops, int32_t hop,
                               ref_group_desc *desc_out, uint8_t *rows_out, int32_t *src_token_out,
                               int32_t *topk_out, int32_t *G_out, int32_t *N_out)
{
    if (R < 1 || R > REF_MAX_RANKS || n_hops < 1 || hop < 0 || hop >= n_hops) return REF_ERR_ARG;
    for (int32_t r = 0; r < R; ++r)
        if (next_hop[r] < 0 || next_hop[r] >= n_hops) return REF_ERR_ARG;
    int32_t g2 = 0, n2 = 0;
    for (int32_t g = 0; g < G; ++g) {
        int uses_hop = 0;
        for (int r = 0; r < REF_MAX_RANKS; ++r) {
            if (!mask_bit(desc[g].mask, r)) continue;
            if (r >= R) return REF_ERR_INPUT;
            if (next_hop[r] == hop) uses_hop = 1;
        }
        if (!uses_hop) continue;
        for (int w = 0; w < REF_MASK_WORDS; ++w) desc_out[g2].mask[w] = desc[g].mask[w];
        desc_out[g2].row_offset = (uint32_t)n2;
        desc_out[g2].row_count = desc[g].row_count;
        desc_out[g2].n_dest = (uint32_t)mask_popcount(desc[g].mask);
        desc_out[g2].reserved0 = 0;
        for (uint32_t i = 0; i < desc[g].row_count; ++i) {
            const size_t s = (size_t)desc[g].row_offset + i;
            memcpy(rows_out + (size_t)n2 * (size_t)row_bytes, rows + s * (size_t)row_bytes, (size_t)row_bytes);
            src_token_out[n2] = row_src_token[s];
            for (int32_t j = 0; j < K; ++j) topk_out[(size_t)n2 * K + j] = row_topk[s * K + j];
            ++n2;
        }
        ++g2;
    }
    *G_out = g2; *N_out = n2;
    return REF_OK;
}

static int32_t local_count(const int32_t *expert_to_rank, int32_t E, int32_t rank)
{
    int32_t L = 0;
    for (int32_t e = 0; e < E; ++e) L += (expert_to_rank[e] == rank);
    return L;
}

/* does this top-k list name the local expert with slot `le`? (set semantics) */
static int row_hits(const int32_t *topk_row, int32_t K, const int32_t *expert_to_rank, int32_t E,
                    int32_t rank, int32_t le, int *bad)
{
    int hit = 0;
    for (int32_t j = 0; j < K; ++j) {
        int32_t e = topk_row[j];
        if (e == -1) continue;
        if (e < 0 || e >= E) { *bad = 1; continue; }
        if (local_slot_of(expert_to_rank, e, rank) == le) hit = 1;
    }
    return hit;
}

/*
 * Tier 2 receive side (Section 4.1 steps 3-4; Section 5.1, the receive
 * module's reception, reassembly and delivery).  For every peer in rank
 * order, rows of groups whose bitmap names this rank are delivered to each
 * local expert in the row's top-k list.  Output is expert-major; inside an
 * expert rows are ordered by (source peer, source token index) ascending,
 * whatever order they were packed in.  The output row is split back into
 * its x part and its scale part.
 */
int ref_unpack(const ref_recv_peer *peers, int32_t P, int32_t K,
               const int32_t *expert_to_rank, int32_t E, int32_t my_rank,
               int64_t x_row_bytes, int64_t s_row_bytes, int64_t out_capacity_rows,
               uint8_t *out_rows /* [cap][x_row_bytes] */, uint8_t *out_scales /* [cap][s_row_bytes] or NULL */,
               int32_t *out_src_peer, int32_t *out_src_token,
               int64_t *expert_offsets /* [L+1] */, int64_t *n_recv_rows /* rows addressed to this rank */)
{
    if (my_rank < 0 || my_rank >= REF_MAX_RANKS || P < 0) return REF_ERR_ARG;
    const int32_t L = local_count(expert_to_rank, E, my_rank);
    const int64_t rb = x_row_bytes + s_row_bytes;
    int rc = REF_OK, bad = 0;

    /* which rows are addressed to this rank, per peer */
    uint8_t **addr = (uint8_t **)calloc((size_t)(P > 0 ? P : 1), sizeof(uint8_t *));
    int64_t *cnt = (int64_t *)calloc((size_t)(L > 0 ? L : 1) * (size_t)(P > 0 ? P : 1), sizeof(int64_t));
    if (!addr || !cnt) { free(addr); free(cnt); return REF_ERR_CAPACITY; }
    int64_t M = 0;
    for (int32_t p = 0; p < P; ++p) {
        addr[p] = (uint8_t *)calloc((size_t)peers[p].n_rows + 1, 1);
        for (uint32_t g = 0; g < peers[p].n_desc; ++g) {
            const ref_group_desc *d = &peers[p].desc[g];
            if ((uint64_t)d->row_offset + d->row_count > peers[p].n_rows) { rc = REF_ERR_INPUT; goto done; }
            if (!mask_bit(d->mask, my_rank)) continue;
            for (uint32_t i = 0; i < d->row_count; ++i) addr[p][d->row_offset + i] = 1;
        }
        for (uint32_t i = 0; i < peers[p].n_rows; ++i) {
            if (!addr[p][i]) continue;
            ++M;
            int any = 0;
            for (int32_t le = 0; le < L; ++le)
                if (row_hits(peers[p].row_topk + (size_t)i * K, K, expert_to_rank, E, my_rank, le, &bad)) {
                    cnt[(size_t)le * P + p] += 1; any = 1;
                }
            if (!any) { rc = REF_ERR_INPUT; goto done; }   /* bitmap names us but no local expert does */
        }
    }
    if (bad) { rc = REF_ERR_EXPERT; goto done; }
    *n_recv_rows = M;

    /* expert-major, then peer-major bases */
    {
        int64_t run = 0;
        for (int32_t le = 0; le < L; ++le) {
            expert_offsets[le] = run;
            for (int32_t p = 0; p < P; ++p) run += cnt[(size_t)le * P + p];
        }
        expert_offsets[L] = run;
        if (run > out_capacity_rows) { rc = REF_ERR_CAPACITY; goto done; }
    }

    for (int32_t le = 0; le < L; ++le) {
        int64_t base = expert_offsets[le];
        for (int32_t p = 0; p < P; ++p) {
            const ref_recv_peer *pr = &peers[p];
            for (uint32_t i = 0; i < pr->n_rows; ++i) {
                if (!addr[p][i]) continue;
                if (!row_hits(pr->row_topk + (size_t)i * K, K, expert_to_rank, E, my_rank, le, &bad)) continue;
                /* rank of this row's source token among the peer's rows for this expert */
                int64_t before = 0;
                for (uint32_t i2 = 0; i2 < pr->n_rows; ++i2) {
                    if (!addr[p][i2] || i2 == i) continue;
                    if (!row_hits(pr->row_topk + (size_t)i2 * K, K, expert_to_rank, E, my_rank, le, &bad)) continue;
                    if (pr->row_src_token[i2] == pr->row_src_token[i]) { rc = REF_ERR_INPUT; goto done; }
                    before += (pr->row_src_token[i2] < pr->row_src_token[i]);
                }
                const int64_t pos = base + before;
                const uint8_t *src = pr->rows + (size_t)i * (size_t)rb;
                memcpy(out_rows + (size_t)pos * (size_t)x_row_bytes, src, (size_t)x_row_bytes);
                if (s_row_bytes > 0)
                    memcpy(out_scales + (size_t)pos * (size_t)s_row_bytes, src + x_row_bytes, (size_t)s_row_bytes);
                out_src_peer[pos] = p;
                out_src_token[pos] = pr->row_src_token[i];
            }
            base += cnt[(size_t)le * P + p];
        }
    }
done:
    for (int32_t p = 0; p < P; ++p) free(addr[p]);
    free(addr); free(cnt);
    return rc;
}

/*
 * Receive side with de-duplication (Section 4.1, last paragraph of
 * "Replication and forwarding": end nodes that drop repeated packets).  A
 * packet of this path is a (source peer, source token) pair; a peer's region
 * may hold it more than once when relays forwarded without updating the
 * metadata.  Reading used here: inside one peer's region, among the rows
 * whose group names this rank, the FIRST row (lowest row index) of every
 * source token is taken and the later ones are dropped; what is taken is
 * then delivered as in ref_unpack: expert-major, inside an expert by (source
 * peer, source token) ascending.  n_recv_rows counts the rows taken,
 * n_dropped the repeats.  Written on its own, from the definition: for every
 * local expert and peer, the taken rows that name the expert are put out in
 * ascending source-token order.
 */
int ref_unpack_dedup(const ref_recv_peer *peers, int32_t P, int32_t K,
                     const int32_t *expert_to_rank, int32_t E, int32_t my_rank,
                     int64_t x_row_bytes, int64_t s_row_bytes, int64_t out_capacity_rows,
                     uint8_t *out_rows, uint8_t *out_scales, int32_t *out_src_peer, int32_t *out_src_token,
                     int64_t *expert_offsets /* [L+1] */, int64_t *n_recv_rows, int64_t *n_dropped)
{
    if (my_rank < 0 || my_rank >= REF_MAX_RANKS || P < 0) return REF_ERR_ARG;
    const int32_t L = local_count(expert_to_rank, E, my_rank);
    const int64_t rb = x_row_bytes + s_row_bytes;
    int rc = REF_OK, bad = 0;
    /* taken[p][i] = 1: row i of peer p is addressed to this rank and is the first row of its token */
    uint8_t **taken = (uint8_t **)calloc((size_t)(P > 0 ? P : 1), sizeof(uint8_t *));
    if (!taken) return REF_ERR_CAPACITY;
    int64_t M = 0, D = 0, Q = 0;
    for (int32_t p = 0; p < P; ++p) {
        const ref_recv_peer *pr = &peers[p];
        taken[p] = (uint8_t *)calloc((size_t)pr->n_rows + 1, 1);
        for (uint32_t g = 0; g < pr->n_desc; ++g) {
            const ref_group_desc *d = &pr->desc[g];
            if ((uint64_t)d->row_offset + d->row_count > pr->n_rows) { rc = REF_ERR_INPUT; goto done; }
            if (!mask_bit(d->mask, my_rank)) continue;
            for (uint32_t i = 0; i < d->row_count; ++i) taken[p][d->row_offset + i] = 1;
        }
        for (uint32_t i = 0; i < pr->n_rows; ++i) {
            if (!taken[p][i]) continue;
            for (uint32_t i2 = 0; i2 < i; ++i2)
                if (taken[p][i2] && pr->row_src_token[i2] == pr->row_src_token[i]) { taken[p][i] = 0; break; }
            if (taken[p][i]) ++M; else ++D;
        }
    }
    for (int32_t le = 0; le < L; ++le) {
        expert_offsets[le] = Q;
        for (int32_t p = 0; p < P; ++p) {
            const ref_recv_peer *pr = &peers[p];
            /* the taken rows of this peer that name expert le, smallest source token first */
            int32_t last = INT32_MIN;
            for (;;) {
                int64_t best = -1;
                for (uint32_t i = 0; i < pr->n_rows; ++i) {
                    if (!taken[p][i] || pr->row_src_token[i] <= last) continue;
                    if (!row_hits(pr->row_topk + (size_t)i * K, K, expert_to_rank, E, my_rank, le, &bad)) continue;
                    if (best < 0 || pr->row_src_token[i] < pr->row_src_token[best]) best = (int64_t)i;
                }
                if (best < 0) break;
                if (Q >= out_capacity_rows) { rc = REF_ERR_CAPACITY; goto done; }
                const uint8_t *src = pr->rows + (size_t)best * (size_t)rb;
                memcpy(out_rows + (size_t)Q * (size_t)x_row_bytes, src, (size_t)x_row_bytes);
                if (s_row_bytes > 0)
                    memcpy(out_scales + (size_t)Q * (size_t)s_row_bytes, src + x_row_bytes, (size_t)s_row_bytes);
                out_src_peer[Q] = p;
                out_src_token[Q] = pr->row_src_token[best];
                last = pr->row_src_token[best];
                ++Q;
            }
        }
    }
    expert_offsets[L] = Q;
    if (bad) rc = REF_ERR_EXPERT;
    *n_recv_rows = M; *n_dropped = D;
done:
    for (int32_t p = 0; p < P; ++p) free(taken[p]);
    free(taken);
    return rc;
}

/*
 * Tier 1: the plain definition of what a dispatch delivers to this rank
 * (Section 4.3.1 applied to every token; Section 2.1, dispatch-style
 * AlltoAll).  No bitmaps, groups or packed buffers: for each local expert in
 * ascending id order, for each peer in rank order, for each of its tokens in
 * index order, the token is delivered iff the expert is in its top-k set.
 */
int ref_dispatch_plain(const ref_peer_tokens *peers, int32_t P, int32_t K,
                       const int32_t *expert_to_rank, int32_t E, int32_t my_rank,
                       int64_t x_row_bytes, int64_t s_row_bytes, int64_t out_capacity_rows,
                       uint8_t *out_rows, uint8_t *out_scales,
                       int32_t *out_src_peer, int32_t *out_src_token, int64_t *expert_offsets)
{
    int64_t pos = 0;
    int32_t le = 0;
    for (int32_t e = 0; e < E; ++e) {
        if (expert_to_rank[e] != my_rank) continue;
        expert_offsets[le++] = pos;
        for (int32_t p = 0; p < P; ++p)
            for (int32_t t = 0; t < peers[p].n_tokens; ++t) {
                int in_set = 0;
                for (int32_t j = 0; j < K; ++j) in_set |= (peers[p].topk[(size_t)t * K + j] == e);
                if (!in_set) continue;
                if (pos >= out_capacity_rows) return REF_ERR_CAPACITY;
                memcpy(out_rows + (size_t)pos * (size_t)x_row_bytes,
                       peers[p].x + (size_t)t * (size_t)x_row_bytes, (size_t)x_row_bytes);
                if (s_row_bytes > 0)
                    memcpy(out_scales + (size_t)pos * (size_t)s_row_bytes,
                           peers[p].scales + (size_t)t * (size_t)s_row_bytes, (size_t)s_row_bytes);
                out_src_peer[pos] = p;
                out_src_token[pos] = t;
                ++pos;
            }
    }
    expert_offsets[le] = pos;
    return REF_OK;
}

/*
 * AllGather as a MultiWrite with a static destination set (Section 2.3.3,
 * Section 5.2): the shard is one packed row, one group, bitmap = all R ranks
 * (this rank included).
 */
int ref_plan_allgather(int32_t R, int64_t shard_bytes, ref_group_desc *desc, ref_send_stats *stats)
{
    if (R < 1 || R > REF_MAX_RANKS || shard_bytes < 0) return REF_ERR_ARG;
    memset(desc, 0, sizeof(*desc));
    memset(stats, 0, sizeof(*stats));
    for (int32_t r = 0; r < R; ++r) {
        desc->mask[r >> 6] |= (uint64_t)1 << (r & 63);
        stats->rows_per_dest[r] = 1;
    }
    desc->row_offset = 0; desc->row_count = 1; desc->n_dest = (uint32_t)R;
    stats->n_rows = 1; stats->n_groups = 1;
    stats->multicast_bytes = (uint64_t)shard_bytes;
    stats->unicast_bytes = (uint64_t)shard_bytes * (uint64_t)R;
    return REF_OK;
}

/* Section 5.2 step 1: the local fragment is loaded into the send buffer. */
int ref_pack_allgather(const uint8_t *shard, int64_t shard_bytes, uint8_t *send_buf)
{
    memcpy(send_buf, shard, (size_t)shard_bytes);
    return REF_OK;
}

/* Result of AllGather: the fragments of ranks 0..R-1 side by side in rank order. */
int ref_unpack_allgather(const uint8_t *const *peer_shards, int32_t R, int64_t shard_bytes, uint8_t *out)
{
    for (int32_t p = 0; p < R; ++p)
        memcpy(out + (size_t)p * (size_t)shard_bytes, peer_shards[p], (size_t)shard_bytes);
    return REF_OK;
}

/* ------------------------------------------------------------------------ */
/*
 * AllGather with a two-segment fragment (Section 5.2, modified workflow
 * step 1 and 2): every node splits its fragment into a segment sent over the
 * direct links by plain writes (one copy per destination) and a segment sent
 * once through the relay path as a MultiWrite; the split ratio is chosen from
 * the bandwidths of the two paths so that both segments arrive together.
 *
 * Section 3.1's model, written out: with the direct fraction f, the direct
 * path takes f*s/w_direct and the relay path (1-f)*s*copies/w_relay, where
 * `copies` is how often the relayed segment crosses the link to the relay
 * (1 with multicast, one per final destination with unicast multi-path).
 * Both are equal at
 *     f = copies*w_direct / (w_relay + copies*w_direct).
 * Equal bandwidths: f = 1/2 and latency s/(2w) with multicast, f = 3/4 and
 * 3s/(4w) with unicast to three destinations -- the paper's two figures.
 *
 * Reading used here: the split point is f*s rounded down to a multiple of 16
 * bytes.  Descriptors count 16-byte units: desc[0] = units [0, a/16) (direct
 * segment), desc[1] = units [a/16, s/16) (relayed segment), both naming all R
 * ranks; an empty segment still gets its (empty) descriptor.  multicast_bytes
 * is what this node injects with the split, a*R + (s-a), unicast_bytes = s*R
 * (this rank's own copy counted, as in ref_plan_allgather).
 */
int ref_allgather_split_point(int64_t shard_bytes, double w_direct, double w_relay, int32_t copies,
                              int64_t *direct_bytes)
{
    if (shard_bytes < 0 || shard_bytes % 16 != 0 || !(w_direct > 0.0) || !(w_relay > 0.0) || copies < 1)
        return REF_ERR_ARG;
    const double f = (double)copies * w_direct / (w_relay + (double)copies * w_direct);
    int64_t a = (int64_t)(f * (double)shard_bytes);
    a -= a % 16;
    if (a < 0) a = 0;
    if (a > shard_bytes) a = shard_bytes;
    *direct_bytes = a;
    return REF_OK;
}

int ref_plan_allgather_split(int32_t R, int64_t shard_bytes, int64_t direct_bytes,
                             ref_group_desc *desc /* [2] */, ref_send_stats *stats)
{
    if (R < 1 || R > REF_MAX_RANKS || shard_bytes < 0 || shard_bytes % 16 != 0) return REF_ERR_ARG;
    if (direct_bytes < 0 || direct_bytes > shard_bytes || direct_bytes % 16 != 0) return REF_ERR_ARG;
    if (shard_bytes / 16 > 0xffffffffLL) return REF_ERR_ARG;
    memset(desc, 0, 2 * sizeof(*desc));
    memset(stats, 0, sizeof(*stats));
    for (int q = 0; q < 2; ++q)
        for (int32_t r = 0; r < R; ++r) desc[q].mask[r >> 6] |= (uint64_t)1 << (r & 63);
    desc[0].row_offset = 0;
    desc[0].row_count = (uint32_t)(direct_bytes / 16);
    desc[1].row_offset = (uint32_t)(direct_bytes / 16);
    desc[1].row_count = (uint32_t)((shard_bytes - direct_bytes) / 16);
    desc[0].n_dest = desc[1].n_dest = (uint32_t)R;
    for (int32_t r = 0; r < R; ++r) stats->rows_per_dest[r] = (uint32_t)(shard_bytes / 16);
    stats->n_rows = (uint32_t)(shard_bytes / 16);
    stats->n_groups = 2;
    stats->multicast_bytes = (uint64_t)direct_bytes * (uint64_t)R + (uint64_t)(shard_bytes - direct_bytes);
    stats->unicast_bytes = (uint64_t)shard_bytes * (uint64_t)R;
    return REF_OK;
}

/* Result: rank p's fragment = its direct piece followed by its relayed piece, ranks side by side. */
int ref_unpack_allgather_split(const uint8_t *const *direct, const uint8_t *const *relayed, int32_t R,
                               int64_t shard_bytes, int64_t direct_bytes, uint8_t *out)
{
    if (direct_bytes < 0 || direct_bytes > shard_bytes) return REF_ERR_ARG;
    for (int32_t p = 0; p < R; ++p) {
        uint8_t *o = out + (size_t)p * (size_t)shard_bytes;
        memcpy(o, direct[p], (size_t)direct_bytes);
        memcpy(o + direct_bytes, relayed[p], (size_t)(shard_bytes - direct_bytes));
    }
    return REF_OK;
}

/* ------------------------------------------------------------------------ */
/*
 * Packets: the bitmap embedded in the payload (Section 6.4, "Metadata
 * overhead", second option: for more ranks than a protocol field holds, the
 * metadata travels in front of the data) together with the rest of what a
 * receiver needs (Section 4.3.4, statelessness: all mapping information is in
 * the packet).  The paper fixes no layout; this reading:
 *   packet = header | row,   header_bytes = 40 + 4K rounded up to 128
 *   header: bytes  0..31  destination bitmap, 4 little-endian 64-bit words
 *           bytes 32..35  index of the token at its source (int32)
 *           bytes 36..39  K (uint32)
 *           bytes 40..    the token's K expert ids (int32 each), as the gate
 *                         emitted them; the rest of the header is zero.
 * 128 bytes in front of a 4096-byte payload is the paper's own example of the
 * cost (1024 bit per 4096 byte = 3.13 %).
 */
int64_t ref_packet_header_bytes(int32_t K)
{
    if (K < 0) return REF_ERR_ARG;
    return ((int64_t)40 + 4 * (int64_t)K + 127) / 128 * 128;
}

static void put_le(uint8_t *dst, uint64_t v, int n_bytes)
{
    for (int b = 0; b < n_bytes; ++b) dst[b] = (uint8_t)(v >> (8 * b));
}

static uint64_t get_le(const uint8_t *src, int n_bytes)
{
    uint64_t v = 0;
    for (int b = 0; b < n_bytes; ++b) v |= (uint64_t)src[b] << (8 * b);
    return v;
}

/* packet i = header of token perm[i] followed by its row (x part, then scales) */
int ref_pack_packets(const uint8_t *x, int64_t x_row_bytes, const uint8_t *scales, int64_t s_row_bytes,
                     const int32_t *topk, int32_t K, const uint64_t *mask /* [T][4] */,
                     const int32_t *perm, int32_t N, uint8_t *packets /* [N][header + row bytes] */)
{
    if (x_row_bytes < 0 || s_row_bytes < 0 || (s_row_bytes > 0 && !scales) || K < 0) return REF_ERR_ARG;
    const int64_t hb = ref_packet_header_bytes(K), pb = hb + x_row_bytes + s_row_bytes;
    for (int32_t i = 0; i < N; ++i) {
        const int32_t t = perm[i];
        uint8_t *h = packets + (size_t)i * (size_t)pb;
        memset(h, 0, (size_t)hb);
        for (int w = 0; w < REF_MASK_WORDS; ++w) put_le(h + 8 * w, mask[(size_t)t * REF_MASK_WORDS + w], 8);
        put_le(h + 32, (uint32_t)t, 4);
        put_le(h + 36, (uint32_t)K, 4);
        for (int32_t j = 0; j < K; ++j) put_le(h + 40 + 4 * j, (uint32_t)topk[(size_t)t * K + j], 4);
        memcpy(h + hb, x + (size_t)t * (size_t)x_row_bytes, (size_t)x_row_bytes);
        if (s_row_bytes > 0)
            memcpy(h + hb + x_row_bytes, scales + (size_t)t * (size_t)s_row_bytes, (size_t)s_row_bytes);
    }
    return REF_OK;
}

/* Simulated network for packets (Section 4.1 step 4): the packets whose bitmap names dst_rank,
 * in order, unchanged.  Returns how many were kept through *n_kept. */
int ref_deliver_packets(const uint8_t *packets, int64_t n_packets, int64_t packet_bytes, int32_t dst_rank,
                        uint8_t *out, int64_t *n_kept)
{
    if (dst_rank < 0 || dst_rank >= REF_MAX_RANKS || packet_bytes < 128) return REF_ERR_ARG;
    int64_t n = 0;
    for (int64_t i = 0; i < n_packets; ++i) {
        const uint8_t *h = packets + (size_t)i * (size_t)packet_bytes;
        const uint64_t word = get_le(h + 8 * (dst_rank >> 6), 8);
        if (!((word >> (dst_rank & 63)) & 1u)) continue;
        memcpy(out + (size_t)n * (size_t)packet_bytes, h, (size_t)packet_bytes);
        ++n;
    }
    *n_kept = n;
    return REF_OK;
}

typedef struct {
    const uint8_t *packets;   /* [n_rows][packet_bytes] */
    uint32_t n_rows;
    uint32_t reserved0;
} ref_recv_packets;

typedef struct { int32_t token; int64_t packet; } token_at;

static int token_at_cmp(const void *pa, const void *pb)
{
    const token_at *a = (const token_at *)pa, *b = (const token_at *)pb;
    return (a->token > b->token) - (a->token < b->token);
}

/*
 * Receive side for packets (Section 4.1 steps 3-4): every packet is parsed on
 * its own.  If its bitmap names this rank, its row is delivered to each local
 * expert among its ids.  Same output as ref_unpack: expert-major, inside an
 * expert ordered by (source peer, source token index), whatever order the
 * packets arrived in.
 */
int ref_unpack_packets(const ref_recv_packets *peers, int32_t P, int32_t K,
                       const int32_t *expert_to_rank, int32_t E, int32_t my_rank,
                       int64_t x_row_bytes, int64_t s_row_bytes, int64_t out_capacity_rows,
                       uint8_t *out_rows, uint8_t *out_scales, int32_t *out_src_peer, int32_t *out_src_token,
                       int64_t *expert_offsets /* [L+1] */, int64_t *n_recv_rows)
{
    if (my_rank < 0 || my_rank >= REF_MAX_RANKS || P < 0 || K < 0) return REF_ERR_ARG;
    const int32_t L = local_count(expert_to_rank, E, my_rank);
    const int64_t hb = ref_packet_header_bytes(K), pb = hb + x_row_bytes + s_row_bytes;
    int bad = 0;
    int64_t pos = 0, M = 0, most = 1;
    for (int32_t p = 0; p < P; ++p) if ((int64_t)peers[p].n_rows > most) most = peers[p].n_rows;
    token_at *list = (token_at *)malloc((size_t)most * sizeof(token_at));
    int32_t *ids = (int32_t *)malloc((size_t)(K > 0 ? K : 1) * sizeof(int32_t));
    if (!list || !ids) { free(list); free(ids); return REF_ERR_CAPACITY; }
    int rc = REF_OK;

    for (int32_t p = 0; p < P; ++p)
        for (uint32_t i = 0; i < peers[p].n_rows; ++i) {
            const uint8_t *h = peers[p].packets + (size_t)i * (size_t)pb;
            if ((int64_t)get_le(h + 36, 4) != K) { rc = REF_ERR_INPUT; goto done; }
            if ((get_le(h + 8 * (my_rank >> 6), 8) >> (my_rank & 63)) & 1u) ++M;
        }
    *n_recv_rows = M;

    for (int32_t le = 0; le < L; ++le) {
        expert_offsets[le] = pos;
        for (int32_t p = 0; p < P; ++p) {
            int64_t n = 0;
            for (uint32_t i = 0; i < peers[p].n_rows; ++i) {
                const uint8_t *h = peers[p].packets + (size_t)i * (size_t)pb;
                if (!((get_le(h + 8 * (my_rank >> 6), 8) >> (my_rank & 63)) & 1u)) continue;
                for (int32_t j = 0; j < K; ++j) ids[j] = (int32_t)(uint32_t)get_le(h + 40 + 4 * j, 4);
                if (!row_hits(ids, K, expert_to_rank, E, my_rank, le, &bad)) continue;
                list[n].token = (int32_t)(uint32_t)get_le(h + 32, 4);
                list[n].packet = i;
                ++n;
            }
            qsort(list, (size_t)n, sizeof(token_at), token_at_cmp);
            for (int64_t k = 0; k < n; ++k) {
                if (k > 0 && list[k].token == list[k - 1].token) { rc = REF_ERR_INPUT; goto done; }
                if (pos >= out_capacity_rows) { rc = REF_ERR_CAPACITY; goto done; }
                const uint8_t *row = peers[p].packets + (size_t)list[k].packet * (size_t)pb + hb;
                memcpy(out_rows + (size_t)pos * (size_t)x_row_bytes, row, (size_t)x_row_bytes);
                if (s_row_bytes > 0)
                    memcpy(out_scales + (size_t)pos * (size_t)s_row_bytes, row + x_row_bytes, (size_t)s_row_bytes);
                out_src_peer[pos] = p;
                out_src_token[pos] = list[k].token;
                ++pos;
            }
        }
    }
    expert_offsets[L] = pos;
    if (bad) rc = REF_ERR_EXPERT;
done:
    free(list); free(ids);
    return rc;
}

/* ------------------------------------------------------------------------ */
/*
 * Quantise-in-pack: the packer takes bf16 rows and writes fp8 rows
 * (H e4m3 codes, then H/128 fp32 scales), so the quantised copy is never
 * written to memory on its own.  Not in the paper (its payload is opaque
 * bytes); the arithmetic is the usual block-wise fp8 recipe, and this is the
 * contract both sides follow, in IEEE single precision with round to nearest
 * even and no fused or reordered operations:
 *   per block of 128 consecutive elements of a row
 *     a   = max |x_j|                       (bf16 widened to fp32, exact)
 *     a_c = max(a, 2^-20)                   (never zero, never subnormal)
 *     s   = a_c / 448                       -> the block's stored scale
 *     inv = 448 / a_c
 *     y_j = x_j * inv, limited to [-448, 448]
 *     code_j = the OCP e4m3 ("fn": no infinities, largest finite 448) value
 *              nearest to y_j; a tie goes to the code with an even mantissa;
 *              the sign is kept (a negative y_j that rounds to zero is -0).
 * Inputs must be finite.
 * The nearest code is found by definition: the 127 non-negative finite codes
 * are decoded from the format (exponent bias 7, three mantissa bits,
 * subnormals at exponent field 0) and searched.
 */
static double e4m3_value(int code /* 0..126 */)
{
    const int e = code >> 3, m = code & 7;
    return e == 0 ? ldexp((double)m, -9) : ldexp((double)(8 + m), e - 10);
}

static uint8_t e4m3_nearest(float y /* finite, |y| <= 448 */)
{
    uint32_t bits;
    memcpy(&bits, &y, 4);
    const uint8_t sign = (uint8_t)((bits >> 24) & 0x80u);
    const double a = fabs((double)y);
    int lo = 0;                                  /* largest code whose value is <= a */
    while (lo < 126 && e4m3_value(lo + 1) <= a) ++lo;
    if (lo == 126) return (uint8_t)(sign | 126);
    const double d_lo = a - e4m3_value(lo), d_hi = e4m3_value(lo + 1) - a;   /* exact in double */
    int code = lo;
    if (d_hi < d_lo || (d_hi == d_lo && (lo & 1))) code = lo + 1;
    return (uint8_t)(sign | code);
}

static float bf16_value(uint16_t b)
{
    const uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

int ref_quantize_e4m3_block128(const uint16_t *x /* [n_rows][H] bf16 bit patterns */, int64_t n_rows, int32_t H,
                               uint8_t *codes /* [n_rows][H] */, float *scales /* [n_rows][H/128] */)
{
    if (n_rows < 0 || H < 0 || H % 128 != 0) return REF_ERR_ARG;
    const int32_t nb = H / 128;
    for (int64_t r = 0; r < n_rows; ++r)
        for (int32_t b = 0; b < nb; ++b) {
            const uint16_t *xb = x + (size_t)r * (size_t)H + (size_t)b * 128;
            volatile float a = 0.0f;             /* volatile: every step is rounded to single precision */
            for (int j = 0; j < 128; ++j) {
                const float v = fabsf(bf16_value(xb[j]));
                if (!(v <= 3.4028234663852886e38f)) return REF_ERR_INPUT;      /* not finite */
                if (v > a) a = v;
            }
            volatile float a_c = a > 0x1p-20f ? a : 0x1p-20f;
            volatile float s = a_c / 448.0f;
            volatile float inv = 448.0f / a_c;
            scales[(size_t)r * (size_t)nb + b] = s;
            for (int j = 0; j < 128; ++j) {
                volatile float y = bf16_value(xb[j]) * inv;
                if (y > 448.0f) y = 448.0f;
                if (y < -448.0f) y = -448.0f;
                codes[(size_t)r * (size_t)H + (size_t)b * 128 + j] = e4m3_nearest(y);
            }
        }
    return REF_OK;
}

/* ------------------------------------------------------------------------ */
/*
 * The way back (Section 2.1, combine-style AlltoAll; Section 2.3.2 notes that
 * the combine phase reduces and cannot use multicast).  What this rank can do
 * locally is the mirror image of MultiWrite's "one copy per destination
 * set": a token that reached h of this rank's experts gets ONE row back, the
 * sum of those h expert outputs, instead of h rows.
 *
 * Reading (the paper does not define the step):
 *   y [Q][H] bf16 is laid out exactly like the dispatch output (expert-major,
 *   then source peer, then source token).  For source peer p and token t with
 *   at least one local expert in its id list,
 *     ret(p, t) = bf16( ((y[q_1] + y[q_2]) + ...) + y[q_h] )
 *   summed in single precision in the order the distinct local experts appear
 *   in the token's id list (first occurrences), one rounding to bf16 (nearest,
 *   ties to even) at the end; h = 1 is a plain copy of the 16-bit patterns.
 *   A NaN sum becomes the quiet NaN 0x7FC0 with the sum's sign bit.
 * Row (p, t) is written to return row i of peer p's return region, where i is
 * the row's position in what the peer sent (row_src_token[i] == t): the peer
 * gets its rows back in the order it packed them.  Rows that were not
 * addressed to this rank are left untouched.
 */
static uint16_t bf16_round(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)(((u >> 16) & 0x8000u) | 0x7fc0u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

int ref_combine_gather(const ref_recv_peer *peers, int32_t P, int32_t K,
                       const int32_t *expert_to_rank, int32_t E, int32_t my_rank, int32_t H,
                       const uint16_t *y /* [Q][H] */, const int32_t *out_src_peer, const int32_t *out_src_token,
                       const int64_t *expert_offsets /* [L+1] */,
                       uint16_t *const *ret /* [P] -> [n_rows of that peer][H] */)
{
    if (my_rank < 0 || my_rank >= REF_MAX_RANKS || P < 0 || H < 0) return REF_ERR_ARG;
    int bad = 0;
    float *acc = (float *)malloc((size_t)(H > 0 ? H : 1) * sizeof(float));
    if (!acc) return REF_ERR_CAPACITY;
    int rc = REF_OK;
    for (int32_t p = 0; p < P && rc == REF_OK; ++p) {
        const ref_recv_peer *pr = &peers[p];
        uint8_t *addr = (uint8_t *)calloc((size_t)pr->n_rows + 1, 1);
        for (uint32_t g = 0; g < pr->n_desc; ++g) {
            const ref_group_desc *d = &pr->desc[g];
            if ((uint64_t)d->row_offset + d->row_count > pr->n_rows) { rc = REF_ERR_INPUT; break; }
            if (!mask_bit(d->mask, my_rank)) continue;
            for (uint32_t i = 0; i < d->row_count; ++i) addr[d->row_offset + i] = 1;
        }
        for (uint32_t i = 0; i < pr->n_rows && rc == REF_OK; ++i) {
            if (!addr[i]) continue;
            const int32_t *ids = pr->row_topk + (size_t)i * K;
            const int32_t t = pr->row_src_token[i];
            int h = 0;
            const uint16_t *only = NULL;
            for (int32_t j = 0; j < K; ++j) {
                const int32_t e = ids[j];
                if (e == -1) continue;
                if (e < 0 || e >= E) { bad = 1; continue; }
                if (expert_to_rank[e] != my_rank) continue;
                int seen = 0;
                for (int32_t j2 = 0; j2 < j; ++j2) seen |= (ids[j2] == e);
                if (seen) continue;
                const int32_t le = local_slot_of(expert_to_rank, e, my_rank);
                int64_t q = -1;
                for (int64_t c = expert_offsets[le]; c < expert_offsets[le + 1]; ++c)
                    if (out_src_peer[c] == p && out_src_token[c] == t) { q = c; break; }
                if (q < 0) { rc = REF_ERR_INPUT; break; }
                const uint16_t *row = y + (size_t)q * (size_t)H;
                for (int32_t c = 0; c < H; ++c) {
                    volatile float sum = (h == 0) ? bf16_value(row[c]) : acc[c] + bf16_value(row[c]);
                    acc[c] = sum;
                }
                only = row;
                ++h;
            }
            if (rc != REF_OK) break;
            if (h == 0) { rc = REF_ERR_INPUT; break; }
            uint16_t *dst = ret[p] + (size_t)i * (size_t)H;
            if (h == 1) memcpy(dst, only, (size_t)H * 2);
            else for (int32_t c = 0; c < H; ++c) dst[c] = bf16_round(acc[c]);
        }
        free(addr);
    }
    free(acc);
    if (rc == REF_OK && bad) rc = REF_ERR_EXPERT;
    return rc;
}

/* ------------------------------------------------------------------------ */
/*
 * Relay of packets: the paper's own form of the step (Section 4.1,
 * "Replication and forwarding": the relay buffers the payload, parses the
 * bitmap, makes one copy per distinct egress port and updates the in-packet
 * metadata of each copy so that downstream nodes do not replicate again;
 * Section 4.3.3, the recursive model).  Reading, as for ref_relay_child with
 * every packet its own group: the child for hop h keeps, in order, the
 * packets whose bitmap names at least one rank with next_hop == h; the
 * header's bitmap becomes the parent's restricted to those ranks; everything
 * else in the packet is copied unchanged.
 * Also returns the accounting of the whole relay step through `copies`
 * (packets written over all hops: one per distinct next hop, Section 4.1)
 * and `dests` (one per destination: what unicast would send); both may be
 * NULL.
 */
int ref_relay_packets_child(const uint8_t *packets, int64_t n_packets, int64_t packet_bytes,
                            const int32_t *next_hop, int32_t R, int32_t n_hops, int32_t hop,
                            uint8_t *out, int64_t *n_out, uint64_t *copies, uint64_t *dests)
{
    if (R < 1 || R > REF_MAX_RANKS || n_hops < 1 || hop < 0 || hop >= n_hops || packet_bytes < 128) return REF_ERR_ARG;
    for (int32_t r = 0; r < R; ++r)
        if (next_hop[r] < 0 || next_hop[r] >= n_hops) return REF_ERR_ARG;
    int64_t n = 0;
    uint64_t n_copies = 0, n_dests = 0;
    for (int64_t i = 0; i < n_packets; ++i) {
        const uint8_t *pk = packets + (size_t)i * (size_t)packet_bytes;
        uint64_t mask[REF_MASK_WORDS], sub[REF_MASK_WORDS] = {0, 0, 0, 0};
        for (int w = 0; w < REF_MASK_WORDS; ++w) mask[w] = get_le(pk + 8 * w, 8);
        int n_sub = 0;
        for (int32_t h = 0; h < n_hops; ++h) {
            int used = 0;
            for (int r = 0; r < REF_MAX_RANKS; ++r) {
                if (!mask_bit(mask, r)) continue;
                if (r >= R) return REF_ERR_INPUT;
                if (next_hop[r] == h) used = 1;
            }
            n_copies += (uint64_t)used;
        }
        for (int r = 0; r < R; ++r) {
            if (!mask_bit(mask, r)) continue;
            ++n_dests;
            if (next_hop[r] != hop) continue;
            sub[r >> 6] |= (uint64_t)1 << (r & 63);
            ++n_sub;
        }
        if (n_sub == 0) continue;
        uint8_t *dst = out + (size_t)n * (size_t)packet_bytes;
        memcpy(dst, pk, (size_t)packet_bytes);
        for (int w = 0; w < REF_MASK_WORDS; ++w) put_le(dst + 8 * w, sub[w], 8);
        ++n;
    }
    *n_out = n;
    if (copies) *copies = n_copies;
    if (dests) *dests = n_dests;
    return REF_OK;
}

/*
 * Relay of packets WITHOUT the metadata update (Section 4.1, last paragraph
 * of "Replication and forwarding"; see ref_relay_child_unmodified).  The
 * child for hop h holds, in order, the packets ref_relay_packets_child keeps
 * for it, each one byte for byte as it arrived: header bitmap included.
 */
int ref_relay_packets_child_unmodified(const uint8_t *packets, int64_t n_packets, int64_t packet_bytes,
                                       const int32_t *next_hop, int32_t R, int32_t n_hops, int32_t hop,
                                       uint8_t *out, int64_t *n_out)
{
    if (R < 1 || R > REF_MAX_RANKS || n_hops < 1 || hop < 0 || hop >= n_hops || packet_bytes < 128) return REF_ERR_ARG;
    for (int32_t r = 0; r < R; ++r)
        if (next_hop[r] < 0 || next_hop[r] >= n_hops) return REF_ERR_ARG;
    int64_t n = 0;
    for (int64_t i = 0; i < n_packets; ++i) {
        const uint8_t *pk = packets + (size_t)i * (size_t)packet_bytes;
        uint64_t mask[REF_MASK_WORDS];
        for (int w = 0; w < REF_MASK_WORDS; ++w) mask[w] = get_le(pk + 8 * w, 8);
        int wanted = 0;
        for (int r = 0; r < REF_MAX_RANKS; ++r) {
            if (!mask_bit(mask, r)) continue;
            if (r >= R) return REF_ERR_INPUT;
            if (next_hop[r] == hop) wanted = 1;
        }
        if (!wanted) continue;
        memcpy(out + (size_t)n * (size_t)packet_bytes, pk, (size_t)packet_bytes);
        ++n;
    }
    *n_out = n;
    return REF_OK;
}
