/*
 * mw.h -- C ABI of the MI355X (gfx950) MultiWrite dispatch / AllGather hot path.
 *
 * One rank's local share of a MultiWrite many-to-many operation
 * (paper Section 4.3.1: MultiWrite(S, M, B_S) delivers the source buffer to
 * every destination in M, injecting it once).  The send side turns each
 * token's top-k expert ids into a destination-rank bitmap (Section 4.1,
 * "Encoding scheme of metadata"), groups tokens by bitmap into multicast
 * groups, packs every payload row once per group and writes a group
 * descriptor table (the batched form of Section 4.3.2's "array of remote
 * buffers").  The receive side parses the carried metadata and delivers each
 * row to the local experts it names (Section 4.1 workflow steps 3-4;
 * Section 5.1, receive module).  The network and the other ranks are not
 * part of this library.
 *
 * Conventions for every entry point
 *   - extern "C"; returns an int32 status: MW_OK (0) or a negative MW_ERR_*.
 *   - pointers named *_dev are DEVICE pointers (hipMalloc'd memory of the
 *     current device); everything else is a HOST pointer.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Calls only enqueue work; they never synchronise the stream unless the
 *     entry point says so, never allocate or free device memory, and never
 *     take ownership of a caller buffer.  Buffers must stay valid until the
 *     enqueued work has completed.
 *   - Entry points that take a stream launch kernels only (no memory-set or
 *     copy nodes, no synchronisation) and keep nothing on the host that a
 *     later call depends on, so a sequence of them can be captured into a HIP
 *     graph and replayed; the statistics read-backs (mw_get_*_stats),
 *     mw_ctx_create and mw_set_forwarding synchronise and stay outside.
 *   - Errors the host can see (null pointers, sizes out of range, misaligned
 *     rows) are returned synchronously and nothing is enqueued.  Errors only
 *     visible on the device (bad expert id, capacity overflow, inconsistent
 *     received metadata) set MW_FLAG_* bits in the statistics block, the
 *     offending item is left out, and all kernels still terminate normally.
 *   - Work enqueued for one context shares its workspace in four parts:
 *     (1) mw_plan (and the plan half of mw_unpack_expand_index_plan_next,
 *     in next_ctx); (2) mw_unpack, mw_unpack_packets, mw_unpack_index,
 *     mw_unpack_expand, mw_unpack_expand_index[_plan]_next (the part of `ctx` and,
 *     for the index, of `next_ctx`) and mw_combine_gather; (3) mw_relay,
 *     mw_relay_index, mw_relay_copy, mw_relay_copy_index_next (the part of `ctx`
 *     and, for the index, of `next_ctx`), mw_relay_packets and its three forms
 *     of the same names; (4)
 *     mw_sim_deliver.  Calls of one part race if they
 *     overlap on the device; calls of different parts, and the packers
 *     (mw_pack, mw_pack_quantize, mw_pack_packets, mw_plan_pack, the
 *     AllGather calls), which use no workspace, may run on different streams
 *     at once.  The host-side context is not locked: one host thread at a
 *     time per context.
 *   - A context belongs to the device that was current at mw_ctx_create; an
 *     entry point called with another device current returns
 *     MW_ERR_INVALID_ARG and enqueues nothing.
 */
#ifndef MW_H_
#define MW_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MW_API __attribute__((visibility("default")))

#define MW_MASK_WORDS 4          /* 256-bit destination bitmap */
#define MW_MAX_RANKS  256        /* Section 6.4: bitmaps wider than 64 bit; 256 ranks here */
#define MW_MAX_TOPK   64
#define MW_MAX_HOPS   64         /* next hops (egress ports) a relay's forwarding table may name */
#define MW_FUSED_MAX_TOKENS 256  /* largest batch mw_plan_pack takes */
#define MW_RIDE_MAX_TOKENS 8192  /* largest next batch mw_unpack_expand_index_plan_next plans */
#define MW_STATIC_MAX_TOKENS 8192   /* largest batch mw_plan_static takes */
#define MW_STATIC_MAX_EXPERTS 1024  /* most experts mw_plan_static takes */

/* status codes */
#define MW_OK                 0
#define MW_ERR_INVALID_ARG   -1  /* null pointer, negative size, value out of range */
#define MW_ERR_CAPACITY      -2  /* n_tokens / sizes beyond what the context was created for */
#define MW_ERR_UNSUPPORTED   -3  /* more than 256 ranks, row not a multiple of 16 bytes, ... */
#define MW_ERR_HIP           -4  /* a HIP runtime call failed */
#define MW_ERR_WORKSPACE     -5  /* workspace missing, misaligned or too small */

/* row formats */
#define MW_ROW_BF16             0  /* row = hidden bf16 values, 2*hidden bytes */
#define MW_ROW_FP8_E4M3_BLOCK128 1 /* row = hidden e4m3 codes then hidden/128 fp32 scales */
#define MW_ROW_BYTES            2  /* row = row_bytes opaque bytes (AllGather shards, tests) */

/* device-side error flags (mw_send_stats.error_flags / mw_recv_stats.error_flags) */
#define MW_FLAG_BAD_EXPERT       0x01u  /* expert id outside {-1} U [0, n_experts): entry ignored */
#define MW_FLAG_OUT_CAPACITY     0x02u  /* more output rows than out_capacity_rows: surplus rows dropped */
#define MW_FLAG_NO_LOCAL_EXPERT  0x04u  /* row's group names this rank but none of its experts is local */
#define MW_FLAG_BAD_SRC_TOKEN    0x08u  /* row_src_token outside [0, max_tokens): row dropped */
#define MW_FLAG_BAD_DESC         0x10u  /* descriptor row range outside the peer's rows: group dropped */
#define MW_FLAG_RECV_CAPACITY    0x20u  /* peers hold more rows than max_recv_rows (or one more than max_tokens):
                                           surplus rows dropped; a group cut by the limit is dropped whole and
                                           sets MW_FLAG_BAD_DESC too */
#define MW_FLAG_DUP_SRC_TOKEN    0x40u  /* two rows of one peer carry the same source token for one expert */
#define MW_FLAG_PLAN_TIMEOUT     0x100u /* mw_unpack_expand_index_plan_next, mw_stream_step: the riding plan gave up waiting (see there) */
#define MW_FLAG_BAD_RANK         0x80u  /* relay: a bitmap names a rank >= n_ranks: that bit is not forwarded */
#define MW_FLAG_DUPLICATE_DROPPED 0x200u /* with MW_OPT_RECV_DEDUP: a repeated row was dropped (information, not an error) */

/*
 * Destination bitmap, Section 4.1: ranks are numbered from zero and bit r says
 * whether rank r is a target.  Fixed width of 4 x 64 bit (Section 6.4 allows
 * wider fields for more than 64 ranks): rank r <-> mask[r / 64] bit (r % 64);
 * bits at and above n_ranks are zero.
 */
typedef struct mw_group_desc {
    uint64_t mask[MW_MASK_WORDS];
    uint32_t row_offset;   /* index of the group's first packed row */
    uint32_t row_count;    /* rows in the group (>= 1) */
    uint32_t n_dest;       /* popcount(mask) */
    uint32_t reserved0;    /* written as 0 */
} mw_group_desc;           /* 48 bytes, little endian, no padding */

/* Send-side statistics, written by mw_plan / mw_plan_allgather (device resident). */
typedef struct mw_send_stats {
    uint32_t n_rows;            /* N: tokens with a non-empty destination set = packed rows */
    uint32_t n_groups;          /* G: distinct destination sets */
    uint64_t multicast_bytes;   /* N * row_bytes: every row injected once (Section 1) */
    uint64_t unicast_bytes;     /* row_bytes * sum over tokens of |destination set| */
    uint32_t rows_per_dest[MW_MAX_RANKS]; /* rows whose set names rank r (this rank included) */
    uint32_t error_flags;       /* MW_FLAG_* */
    uint32_t reserved0;
} mw_send_stats;                /* 1056 bytes */

/* Receive-side statistics, written by mw_unpack (device resident). */
typedef struct mw_recv_stats {
    uint64_t n_recv_rows;       /* M: received rows whose group bitmap names this rank */
    uint64_t n_out_rows;        /* Q: (row, local expert) pairs = rows of the expert-major output */
    uint32_t error_flags;       /* MW_FLAG_* */
    uint32_t n_rows_seen;       /* rows in the peers' buffers, addressed to this rank or not */
} mw_recv_stats;                /* 24 bytes */

/*
 * What one peer wrote into this rank's pre-allocated receive region
 * (Section 6.4, "Memory usage": one region per peer).  The array of these
 * records lives in device memory; so does everything they point to.
 * Rows are laid out as mw_pack writes them.  A sender's complete buffer is
 * accepted as well: groups whose bitmap does not name this rank are skipped.
 */
typedef struct mw_recv_peer {
    const mw_group_desc *desc;      /* [n_desc], row ranges ascending and inside [0, n_rows) */
    uint32_t n_desc;
    uint32_t n_rows;                /* <= max_tokens */
    const void *rows;               /* [n_rows] rows, row_stride_bytes apart, 16-byte aligned */
    const int32_t *row_src_token;   /* [n_rows] index of the row's token at the sender */
    const int32_t *row_topk;        /* [n_rows][top_k] the token's expert ids as the gate emitted them */
} mw_recv_peer;                     /* 40 bytes */

/*
 * Context configuration (Section 5.1, initialisation module: topology and
 * node configuration; Section 4.1: the table that maps addresses -- here
 * expert ids -- to ranks).  Immutable after mw_ctx_create.
 */
typedef struct mw_config {
    int32_t n_ranks;        /* R, 1..256 */
    int32_t n_experts;      /* E >= 0 (0: AllGather-only context) */
    int32_t top_k;          /* K, 1..64 */
    int32_t my_rank;        /* 0..R-1 */
    int32_t hidden;         /* H elements per token (ignored for MW_ROW_BYTES) */
    int32_t row_format;     /* MW_ROW_* */
    int64_t row_bytes;      /* MW_ROW_BYTES: given.  Otherwise 0 or the derived value:
                               bf16 2*H; fp8 H + 4*(H/128).  Must be a multiple of 16;
                               fp8 additionally needs H % 512 == 0 so both parts are. */
    int32_t max_tokens;     /* capacity for n_tokens and bound on any peer's token indices */
    int32_t max_hops;       /* 0..MW_MAX_HOPS: next hops mw_relay may fan out to (0: relay not used) */
    int64_t max_recv_rows;  /* capacity for the sum of the peers' n_rows in mw_unpack */
    const int32_t *expert_to_rank; /* HOST, [E], values in [0, R); copied at create */
    int64_t row_stride_bytes; /* bytes from the start of one row to the start of the next in every array
                               * of packed or received rows (see below); 0 = row_bytes, rows back to back */
} mw_config;

/*
 * Row stride.  Arrays of rows on the wire side of the path -- what mw_pack, mw_pack_quantize,
 * mw_plan_pack and mw_stream_step write, what mw_sim_deliver and mw_relay read and write, the
 * `rows` of an mw_recv_peer -- hold row i at byte offset i * row_stride_bytes.  The stride is at
 * least row_bytes and a multiple of 16; the bytes between the end of a row and the start of
 * the next are never read and never written.  It is a matter of layout only: a row's content,
 * the byte accounting (which counts row_bytes per row) and every output of mw_unpack are the
 * same for any stride.  Rows that are not whole 128-byte cache lines move faster with a
 * stride that is (fp8 rows of 7392 bytes at a stride of 7424: the expander reads them 9 %
 * faster).  The packet forms (mw_pack_packets, mw_unpack_packets, mw_relay_packets) have
 * their own fixed packet size and do not use it.
 */

typedef struct mw_ctx mw_ctx;

/* Bytes of device workspace a context for `cfg` needs. */
MW_API int32_t mw_workspace_bytes(const mw_config *cfg, int64_t *out_bytes);

/*
 * Create a context on the current device.  `workspace_dev` (256-byte aligned,
 * at least mw_workspace_bytes) stays owned by the caller and must outlive the
 * context.  Copies the rank table to the device and SYNCHRONISES the device
 * once.  The library owns only the small host-side mw_ctx.
 */
MW_API int32_t mw_ctx_create(const mw_config *cfg, void *workspace_dev, int64_t workspace_bytes, mw_ctx **out);
MW_API int32_t mw_ctx_destroy(mw_ctx *ctx);

/*
 * Number of polls (about half a microsecond each) the second half of a plan riding in
 * mw_unpack_expand_index_plan_next or mw_stream_step waits for its first half before it gives
 * up; default 2097152.
 * 0 makes it give up unless the first half is already complete when it looks: for tests of
 * that path.  Applies to later calls that plan with this context.
 */
MW_API int32_t mw_ctx_set_ride_wait_limit(mw_ctx *ctx, int64_t polls);

/*
 * Options of a context (Section 4.1, last paragraph of "Replication and forwarding": where routing
 * loops cannot occur and the end nodes drop repeated packets, a relay may omit the update of the
 * in-packet metadata; whether to do so is a deployment decision).  Host only; applies to later
 * calls; 0 (the default) is the behaviour described at the entry points.
 *   MW_OPT_RELAY_KEEP_METADATA  mw_relay, mw_relay_index and the packets' forms: every child keeps the
 *       groups, rows and row metadata it would keep anyway -- the copies made are the same -- but its
 *       bitmaps (and n_dest) are the parent's, not the parent's restricted to the hop's ranks.
 *   MW_OPT_RECV_DEDUP  mw_unpack, mw_unpack_index, mw_unpack_packets and the launches that carry
 *       the index: of the rows of one peer's region that are addressed to this rank and carry the
 *       same source token, one is taken and the others are dropped (they are copies of one another,
 *       so it does not matter which).  n_recv_rows counts the rows taken; MW_FLAG_DUPLICATE_DROPPED
 *       says that something was dropped; MW_FLAG_DUP_SRC_TOKEN is never raised.
 * Deployments of the first option need the second at the destinations, relays that forward once,
 * and end nodes that never forward: a node further down sees destinations that were served
 * over other hops as well.
 */
#define MW_OPT_RELAY_KEEP_METADATA 0x1u
#define MW_OPT_RECV_DEDUP          0x2u
MW_API int32_t mw_ctx_set_options(mw_ctx *ctx, uint32_t options);

/* ---- send side (Section 5.1, send module: task decomposition) -------------------------- */

/*
 * mw_plan: destination bitmaps, multicast groups, descriptor table.
 *   mask[t]  = OR over the token's valid expert ids e of bit expert_to_rank[e]
 *              (Section 4.1); id -1 means "no expert"; duplicates count once.
 *   perm     = tokens with a non-empty bitmap ordered by (bitmap as unsigned
 *              256-bit integer with word 3 most significant, token index),
 *              both ascending; perm[i] = token of packed row i.
 *   desc[g]  = one record per maximal run of equal bitmaps, in that order.
 *   stats    = counts and the multicast / unicast byte accounting.
 * topk_ids_dev [n_tokens][top_k] int32 row-major; mask_dev [n_tokens][4];
 * perm_dev and desc_dev have room for n_tokens entries (first N / G are
 * written, the rest is left untouched).  0 <= n_tokens <= max_tokens.
 */
MW_API int32_t mw_plan(mw_ctx *ctx, const int32_t *topk_ids_dev, int32_t n_tokens,
                uint64_t *mask_dev, int32_t *perm_dev, mw_group_desc *desc_dev,
                mw_send_stats *stats_dev, void *stream);

/*
 * mw_plan_static: mw_plan for callers that cannot allocate device memory or keep a workspace
 * around -- code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * No context and no workspace: the plan's scratch memory (per-token counters, plan state, the
 * expert table; 70912 bytes) is one array inside the library's device image, which every GPU the
 * library runs on holds until the process ends.  The call allocates and frees nothing, on the
 * host or on the device, and enqueues kernels only (one small one that clears the scratch and
 * builds the expert table, then mw_plan's own).
 *   cfg                 HOST; n_ranks, n_experts, top_k and the row format fields (hidden,
 *                       row_format, row_bytes: for the byte accounting) are used as in mw_ctx_create,
 *                       the other fields -- expert_to_rank included -- are ignored.
 *   expert_to_rank_dev  DEVICE, [n_experts] int32, read by the enqueued work.  An entry outside
 *                       [0, n_ranks) names no rank: that expert is ignored and the statistics carry
 *                       MW_FLAG_BAD_EXPERT.
 *   the other arguments, the outputs and the device-side flags are mw_plan's, bit for bit.
 * Limits: n_tokens <= MW_STATIC_MAX_TOKENS and n_experts <= MW_STATIC_MAX_EXPERTS, else
 * MW_ERR_CAPACITY and nothing is enqueued.  Every call on one GPU shares that GPU's array:
 * calls that overlap on one GPU (two streams, two threads) race; calls on one stream do not.
 */
MW_API int32_t mw_plan_static(const mw_config *cfg, const int32_t *expert_to_rank_dev,
                              const int32_t *topk_ids_dev, int32_t n_tokens, uint64_t *mask_dev,
                              int32_t *perm_dev, mw_group_desc *desc_dev, mw_send_stats *stats_dev, void *stream);

/*
 * mw_pack: every kept token's payload written once, in plan order
 * (Section 1: only one copy of the same data is sent; Section 5.2 step 1:
 * load the data into the pre-allocated send buffer), together with the
 * metadata a receiver needs (Section 4.3.4, statelessness):
 *   packed[i]        = x[perm[i]]  (fp8: the H codes followed by the H/128 scales)
 *   row_src_token[i] = perm[i]
 *   row_topk[i][:]   = topk_ids[perm[i]][:]   unchanged
 * for i < stats->n_rows (read on the device).  x_dev [n_tokens][H] bf16 or
 * e4m3 bytes, or [n_tokens][row_bytes] for MW_ROW_BYTES; scales_dev
 * [n_tokens][H/128] fp32 for fp8, else NULL.  Outputs have room for n_tokens
 * rows.  All payload pointers 16-byte aligned.
 */
MW_API int32_t mw_pack(mw_ctx *ctx, const void *x_dev, const float *scales_dev,
                const int32_t *topk_ids_dev, const int32_t *perm_dev,
                const mw_send_stats *stats_dev, int32_t n_tokens,
                void *packed_rows_dev, int32_t *row_src_token_dev, int32_t *row_topk_dev,
                void *stream);

/*
 * mw_pack_quantize: mw_pack for a context of MW_ROW_FP8_E4M3_BLOCK128 rows whose input is
 * still bf16: x_bf16_dev [n_tokens][H] bf16, packed rows = H e4m3 codes then H/128 fp32 scales,
 * quantised on the way (the paper's payload is opaque bytes, Section 4.3.1; this only changes
 * what the send module loads into the send buffer, Section 5.2 step 1).  Contract, in IEEE
 * single precision with round to nearest even, one rounding per operation, per block of 128
 * consecutive elements of a row:
 *   a = max |x_j|;  a_c = max(a, 2^-20);  scale = a_c / 448 (stored);
 *   code_j = the OCP e4m3 value (no infinities, largest finite 448) nearest to
 *            x_j * (448 / a_c) limited to [-448, 448]; ties to the even mantissa; sign kept.
 * Inputs must be finite: a block holding an infinity or a NaN gets unspecified codes and
 * scale (nothing faults, no flag).  Other arguments, metadata outputs and errors as mw_pack;
 * MW_ERR_UNSUPPORTED for a context of another row format.
 */
MW_API int32_t mw_pack_quantize(mw_ctx *ctx, const void *x_bf16_dev, const int32_t *topk_ids_dev,
                         const int32_t *perm_dev, const mw_send_stats *stats_dev, int32_t n_tokens,
                         void *packed_rows_dev, int32_t *row_src_token_dev, int32_t *row_topk_dev, void *stream);

/*
 * mw_plan_pack: mw_plan followed by mw_pack for a decode-sized batch, as one kernel launch.
 * Section 6.3 (AlltoAll dispatch over batch sizes): at 64 and 128 tokens per rank the fixed
 * cost of a MultiWrite, not the bytes, decides; here that cost is launches and their
 * dependencies.  Every output is byte for byte what the two calls write (same argument
 * meaning, layout and error flags).  0 <= n_tokens <= min(max_tokens, MW_FUSED_MAX_TOKENS);
 * more returns MW_ERR_CAPACITY and nothing is enqueued.  Uses no workspace, so it may overlap
 * other calls on the same context.
 */
MW_API int32_t mw_plan_pack(mw_ctx *ctx, const int32_t *topk_ids_dev, const void *x_dev, const float *scales_dev,
                     int32_t n_tokens, uint64_t *mask_dev, int32_t *perm_dev, mw_group_desc *desc_dev,
                     mw_send_stats *stats_dev, void *packed_rows_dev, int32_t *row_src_token_dev,
                     int32_t *row_topk_dev, void *stream);

/*
 * AllGather as a MultiWrite with a static destination set (Section 2.3.3,
 * Section 5.2): the shard is one row, one group, bitmap = ranks 0..R-1
 * (this rank included).  Writes one descriptor and the statistics.
 */
MW_API int32_t mw_plan_allgather(mw_ctx *ctx, int64_t shard_bytes, mw_group_desc *desc_dev,
                          mw_send_stats *stats_dev, void *stream);

/* Section 5.2 step 1: load the local fragment into the send buffer (16-byte multiple). */
MW_API int32_t mw_pack_allgather(mw_ctx *ctx, const void *shard_dev, int64_t shard_bytes,
                          void *send_buf_dev, void *stream);

/* ---- receive side (Section 5.1, receive module: reception, reassembly, delivery) ------- */

/*
 * mw_unpack: expand the peers' packed buffers into per-local-expert
 * contiguous layouts.  Local experts are the ids e with expert_to_rank[e] ==
 * my_rank, in ascending id order (slot le = 0..L-1).  A row is delivered to
 * local expert le iff its group's bitmap names this rank and le's id is in
 * its row_topk list (set semantics).  Output is expert-major; inside an
 * expert rows are ordered by (source peer, source token index) ascending,
 * independent of packing order:
 *   out_rows[pos]      = the row's x part   ([out_capacity_rows][x bytes per row])
 *   out_scales[pos]    = the row's scales   (fp8 only, else NULL)
 *   out_src_peer[pos], out_src_token[pos]
 *   expert_offsets[le] = first output row of expert le; expert_offsets[L] = Q
 * peers_dev: device array of n_peers records, 1 <= n_peers <= n_ranks.
 */
MW_API int32_t mw_unpack(mw_ctx *ctx, const mw_recv_peer *peers_dev, int32_t n_peers,
                  void *out_rows_dev, float *out_scales_dev, int64_t out_capacity_rows,
                  int32_t *out_src_peer_dev, int32_t *out_src_token_dev,
                  int64_t *expert_offsets_dev, mw_recv_stats *recv_stats_dev, void *stream);

/*
 * The two halves of mw_unpack as separate calls, so that a caller with several batches in
 * flight can run the latency-bound half of the next batch beside the bandwidth-bound half of
 * the current one.  mw_unpack_index reads the peers' metadata, writes expert_offsets and the
 * statistics and leaves one record per received row in the context's workspace;
 * mw_unpack_expand moves the payload as those records say.  mw_unpack(...) is exactly
 * mw_unpack_index(...) followed by mw_unpack_expand(...) with the same arguments on the same
 * stream.  The expand must be ordered after its index (same stream, or an event), the peers'
 * buffers must stay unchanged in between, and a context's workspace holds one index at a
 * time: batches in flight at once need one context each.
 */
MW_API int32_t mw_unpack_index(mw_ctx *ctx, const mw_recv_peer *peers_dev, int32_t n_peers, int64_t out_capacity_rows,
                        int64_t *expert_offsets_dev, mw_recv_stats *recv_stats_dev, void *stream);
MW_API int32_t mw_unpack_expand(mw_ctx *ctx, int32_t n_peers, void *out_rows_dev, float *out_scales_dev,
                         int64_t out_capacity_rows, int32_t *out_src_peer_dev, int32_t *out_src_token_dev, void *stream);

/*
 * Batches of a steady stream, as the launches that handle several batches at once take them:
 * three small records the caller fills in host memory (read during the call only; every *_dev
 * member points to device memory and has the meaning, layout and ownership of the argument of
 * the same name of the call named beside it; reserved members are zero).
 */
typedef struct mw_send_batch {       /* this rank's batch to send: the arguments of mw_pack */
    const void *x_dev;
    const float *scales_dev;
    const int32_t *topk_ids_dev;
    const int32_t *perm_dev;             /* from a plan that an EARLIER launch completed */
    const mw_send_stats *stats_dev;      /* ditto */
    void *packed_rows_dev;
    int32_t *row_src_token_dev;
    int32_t *row_topk_dev;
    int32_t n_tokens;
    int32_t reserved0;
} mw_send_batch;

typedef struct mw_recv_batch {       /* the received batch whose index the context holds: the arguments of mw_unpack_expand */
    void *out_rows_dev;
    float *out_scales_dev;
    int32_t *out_src_peer_dev;
    int32_t *out_src_token_dev;
    int64_t out_capacity_rows;
    int32_t n_peers;
    int32_t reserved0;
} mw_recv_batch;

typedef struct mw_next_batch {       /* the batch after: the arguments of mw_unpack_index and of mw_plan on `ctx` */
    mw_ctx *ctx;                         /* another context on the same device: its workspace takes the index (and the plan) */
    const mw_recv_peer *peers_dev;       /* mw_unpack_index ... */
    int64_t *expert_offsets_dev;
    mw_recv_stats *recv_stats_dev;
    int64_t out_capacity_rows;
    int32_t n_peers;
    int32_t n_tokens;                    /* mw_plan ... (the five members from here on are read by the calls that plan only) */
    const int32_t *topk_ids_dev;
    uint64_t *mask_dev;
    int32_t *perm_dev;
    mw_group_desc *desc_dev;
    mw_send_stats *send_stats_dev;
} mw_next_batch;

/*
 * mw_unpack_expand_index_next: for a steady stream of batches.  One launch does what
 * mw_unpack_expand(ctx, recv->...) does for the batch whose index `ctx` holds, and what
 * mw_unpack_index(next->ctx, next->peers_dev, ...) does for the NEXT batch: the index, a
 * latency-bound kernel that moves almost nothing, rides along with the bandwidth-bound
 * expander of the batch before it instead of standing in front of its own.  The call after
 * this one on the same stream (with the roles of the two contexts exchanged) finds the next
 * batch's index complete: launches on a stream are ordered.  Outputs of both halves are
 * exactly those of the separate calls.  `ctx` and `next->ctx` must be different contexts on
 * the same device (each holds one index in its workspace); arguments as for the two calls
 * (the plan members of `next` are not read).
 * MW_ERR_UNSUPPORTED if the next context's index needs more than 5 KiB of LDS per workgroup
 * (max_tokens above about 8000 with several local experts): use the separate calls then.
 */
MW_API int32_t mw_unpack_expand_index_next(mw_ctx *ctx, const mw_recv_batch *recv, const mw_next_batch *next,
                                           void *stream);

/*
 * mw_unpack_expand_index_plan_next: mw_unpack_expand_index_next with the send-side plan of the
 * next batch in the same launch as well -- what mw_plan(next->ctx, next->topk_ids_dev,
 * next->n_tokens, next->mask_dev, next->perm_dev, next->desc_dev, next->send_stats_dev) does,
 * with exactly its outputs (Section 5.1, send module).  The plan, too, is a chain of memory round
 * trips that moves almost nothing; here it runs in the shadow of the expander.  A steady
 * stream of batches is then two launches per batch on ONE stream, with no event between them:
 *     mw_pack(batch n);  mw_unpack_expand_index_plan_next(expand n; index n+1; plan n+1);
 *     mw_pack(batch n+1);  ...
 * The plan uses the plan part of next->ctx's workspace (see the conventions above); its outputs
 * are complete when this launch is, i.e. for every later call on the same stream.  The riding
 * plan ranks tokens all-pairs (as mw_plan does up to about 8000 tokens): it stays in the
 * expander's shadow while that takes less time than the expander -- 4096 tokens beside 30000
 * received rows of 14 KiB do, 8192 tokens over 256 ranks beside 20000 such rows do not (use
 * mw_plan on a second stream there).
 * Inside the launch the plan's second half waits for its first half (workgroups that come
 * earlier in the same launch and wait for nothing themselves); the wait is bounded (about a
 * second by default, mw_ctx_set_ride_wait_limit).  Past the bound -- not observed, and not
 * expected on hardware that starts a launch's workgroups in order -- the plan is given up:
 * next->send_stats_dev reports MW_FLAG_PLAN_TIMEOUT with zero rows and the other plan outputs
 * are undefined.  Nothing else is lost: the receive side of the launch is unaffected, the launch
 * itself leaves the plan part of next->ctx's workspace clean once its last workgroup is done with
 * it, and the next plan on next->ctx (riding or not) works as usual.
 * MW_ERR_UNSUPPORTED if next->n_tokens > MW_RIDE_MAX_TOKENS (larger batches: mw_plan), or where
 * mw_unpack_expand_index_next returns it; MW_ERR_CAPACITY if next->n_tokens > max_tokens of
 * next->ctx.
 */
MW_API int32_t mw_unpack_expand_index_plan_next(mw_ctx *ctx, const mw_recv_batch *recv, const mw_next_batch *next,
                                                void *stream);

/*
 * mw_stream_step: a whole step of a steady stream of batches in ONE launch -- what
 *     mw_pack(ctx, send->...)   and   mw_unpack_expand_index_plan_next(ctx, recv, next)
 * do, with exactly their outputs: this rank's next batch to send is packed (Section 5.1, send
 * module) while an earlier received batch is expanded, the batch received after that is indexed
 * (receive module) and the batch to send after this one is planned.  The two bandwidth-bound
 * parts then run as one stream of small workgroups with no launch boundary between them, and
 * the latency-bound parts ride along.  send->perm_dev and send->stats_dev must come from a plan
 * that an EARLIER launch completed (mw_plan, or the plan half of the previous mw_stream_step);
 * the payload rows (send->x_dev, send->scales_dev) and the row format are those of `ctx`.
 * Errors as for the two calls.
 */
MW_API int32_t mw_stream_step(mw_ctx *ctx, const mw_send_batch *send, const mw_recv_batch *recv,
                              const mw_next_batch *next, void *stream);

/*
 * mw_combine_gather: the way back (Section 2.1, combine-style AlltoAll).  The paper notes that
 * the combine phase reduces and cannot use multicast (Section 2.3.2); what a rank can do
 * locally is the mirror image of "one copy per destination set": a token that reached h of
 * this rank's experts gets ONE row back, the sum of those h expert outputs.
 *   y_dev [out_capacity_rows][H] bf16: the experts' outputs, laid out exactly like the
 *   out_rows of the last mw_unpack / mw_unpack_index / mw_unpack_packets on this context
 *   (same n_peers, same out_capacity_rows); the peers' receive regions are not read again.
 *   ret_rows_dev [ret_capacity_rows][H] bf16: return row b_p + i belongs to row i of peer p's
 *   region, b_p = sum of the n_rows of the peers before p; peer p's return region is
 *   rows [b_p, b_p + n_rows_p): the peer gets its rows back in the order it packed them.
 *     ret = bf16(((y[q_1] + y[q_2]) + ...) + y[q_h]), single precision, summed in the order the
 *     distinct local experts appear in the row's id list, one rounding to bf16 (nearest, ties
 *     to even) at the end; a NaN sum gives 0x7FC0 with the sum's sign; h = 1 copies the row
 *     unchanged.  Outputs of rows dropped for capacity contribute nothing.
 *   Rows of a region that were not addressed to this rank, and rows at or beyond
 *   ret_capacity_rows, are not written.
 * bf16 contexts only (MW_ERR_UNSUPPORTED otherwise).  Races with a later unpack on the same
 * context, whose index it reads.
 */
MW_API int32_t mw_combine_gather(mw_ctx *ctx, int32_t n_peers, const void *y_dev, int64_t out_capacity_rows,
                          void *ret_rows_dev, int64_t ret_capacity_rows, void *stream);

/*
 * AllGather result (Section 5.2): out = shard of rank 0, rank 1, ... rank R-1
 * side by side.  peer_shards_dev: device array of n_ranks device pointers.
 */
MW_API int32_t mw_unpack_allgather(mw_ctx *ctx, const void *const *peer_shards_dev, int64_t shard_bytes,
                            void *out_dev, void *stream);

/*
 * mw_allgather_step: for a steady stream of AllGathers, one launch that does what
 *     mw_unpack_allgather(ctx, peer_shards_dev, shard_bytes, out_dev),
 *     mw_pack_allgather(ctx, shard_dev, shard_bytes, send_buf_dev) and
 *     mw_plan_allgather(ctx, shard_bytes, desc_dev, stats_dev)
 * do, with exactly their outputs: the shards received for one operation are assembled while
 * this rank's shard of the next one is loaded into its send buffer (Section 5.2, steps 1 and
 * 4) and its one-row plan is written.  Arguments and errors as for the three calls.
 */
MW_API int32_t mw_allgather_step(mw_ctx *ctx, const void *shard_dev, int64_t shard_bytes, void *send_buf_dev,
                          mw_group_desc *desc_dev, mw_send_stats *stats_dev, const void *const *peer_shards_dev,
                          void *out_dev, void *stream);

/*
 * AllGather with a two-segment fragment (Section 5.2, modified workflow): each node splits
 * its fragment into a segment sent over the direct links by plain writes and a segment sent
 * once through the relay path as a MultiWrite; the ratio follows from the bandwidths of the
 * two paths so that both segments arrive together (Section 3.1's model).
 *
 * mw_allgather_split_point (HOST only, no context): direct_bytes = f * shard_bytes rounded
 * down to a multiple of 16 with f = copies * bw_direct / (bw_relay + copies * bw_direct),
 * where `copies` is how often the relayed segment crosses the link to the relay (1 with
 * MultiWrite; the number of final destinations with unicast multi-path).
 */
MW_API int32_t mw_allgather_split_point(int64_t shard_bytes, double bw_direct, double bw_relay, int32_t copies,
                                 int64_t *direct_bytes);

/*
 * Descriptor pair for a split fragment, in units of 16 bytes: desc[0] = units
 * [0, direct_bytes / 16) (direct segment), desc[1] = the rest (relayed segment), both naming
 * ranks 0..R-1.  stats: n_rows = units, n_groups = 2, multicast_bytes = direct_bytes * R +
 * (shard_bytes - direct_bytes) (what this node injects), unicast_bytes = shard_bytes * R.
 * The send buffer is the one mw_pack_allgather fills; the segments are byte ranges of it.
 */
MW_API int32_t mw_plan_allgather_split(mw_ctx *ctx, int64_t shard_bytes, int64_t direct_bytes,
                                mw_group_desc *desc_dev, mw_send_stats *stats_dev, void *stream);

/*
 * Assembly of split fragments: out = for p = 0..R-1: direct_dev[p][0, direct_bytes) followed by
 * relayed_dev[p][0, shard_bytes - direct_bytes).  Two device arrays of n_ranks device pointers
 * (the pieces of one rank arrive in different receive regions).  A pointer may be NULL when its
 * piece is empty.
 */
MW_API int32_t mw_unpack_allgather_split(mw_ctx *ctx, const void *const *direct_dev, const void *const *relayed_dev,
                                  int64_t shard_bytes, int64_t direct_bytes, void *out_dev, void *stream);

/* ---- packets: bitmap and row metadata in front of every row ------------------------------
 *
 * Section 6.4, "Metadata overhead": when the bitmap does not fit a protocol field it is
 * embedded in the payload (the paper's example: 1024 bit in front of 4096 byte, 3.13 %).
 * Together with the source token and the expert ids this makes every row self-describing
 * (Section 4.3.4, statelessness), so no descriptor table and no side arrays travel with it and
 * a receiver can take packets in any order.  Layout of this build (the paper fixes none):
 *   packet = header | row;  header_bytes = 40 + 4 * top_k rounded up to 128 (128 for top_k <= 22)
 *   header: bytes  0..31  destination bitmap, mask[0..3] little endian
 *           bytes 32..35  row_src_token (int32)
 *           bytes 36..39  top_k (uint32)
 *           bytes 40..    the token's top_k expert ids (int32), then zeros
 * Packets are 16-byte aligned; a whole number of 128-byte lines in front of the row keeps
 * the row's alignment.
 */
MW_API int32_t mw_packet_header_bytes(int32_t top_k, int64_t *header_bytes);   /* HOST only */

/*
 * mw_pack_packets: mw_pack with that layout.  packets[i] = header(perm[i]) | row(perm[i]) for
 * i < stats->n_rows, with mask_dev, perm_dev and stats_dev as mw_plan wrote them.
 * packets_dev has room for n_tokens packets of header_bytes + row_bytes.  Other arguments as
 * mw_pack.
 */
MW_API int32_t mw_pack_packets(mw_ctx *ctx, const void *x_dev, const float *scales_dev,
                        const int32_t *topk_ids_dev, const uint64_t *mask_dev, const int32_t *perm_dev,
                        const mw_send_stats *stats_dev, int32_t n_tokens, void *packets_dev, void *stream);

/* What one peer wrote into this rank's receive region, as packets. */
typedef struct mw_recv_packets {
    const void *packets;    /* [n_rows][header_bytes + row_bytes], 16-byte aligned */
    uint32_t n_rows;        /* <= max_tokens */
    uint32_t reserved0;
} mw_recv_packets;          /* 16 bytes */

/*
 * mw_unpack_packets: mw_unpack for regions of packets; same outputs, same order (by source
 * peer and source token, whatever order the packets lie in), same flags.  A packet is taken
 * iff its bitmap names this rank; a header whose id count is not top_k sets MW_FLAG_BAD_DESC
 * and the packet is left out.  mw_unpack_expand is not used with it: this call does both halves.
 */
MW_API int32_t mw_unpack_packets(mw_ctx *ctx, const mw_recv_packets *peers_dev, int32_t n_peers,
                          void *out_rows_dev, float *out_scales_dev, int64_t out_capacity_rows,
                          int32_t *out_src_peer_dev, int32_t *out_src_token_dev,
                          int64_t *expert_offsets_dev, mw_recv_stats *recv_stats_dev, void *stream);

/* ---- relay (Section 4.3.3, recursive execution model; Section 4.1, local forwarding table,
 *      replication and forwarding, update of in-packet metadata) ------------------------------ */

/*
 * Where mw_relay writes the child MultiWrite of one next hop: the same layout mw_pack
 * writes and mw_unpack / mw_relay read.  Device array of n_hops records; every buffer has
 * room for child_capacity_rows rows (descriptors: as many entries).
 */
typedef struct mw_relay_child {
    mw_group_desc *desc;
    void *rows;                 /* [capacity][row_bytes], 16-byte aligned */
    int32_t *row_src_token;     /* [capacity] */
    int32_t *row_topk;          /* [capacity][top_k] */
} mw_relay_child;               /* 32 bytes */

typedef struct mw_relay_stats {
    uint32_t n_groups_in;       /* groups of the input taken (row range valid) */
    uint32_t n_rows_in;         /* their rows */
    uint64_t forward_bytes;     /* row_bytes * rows written to all children: one copy per distinct next hop */
    uint64_t unicast_bytes;     /* row_bytes * sum over groups of rows * destinations: one copy per destination */
    uint32_t groups_per_hop[MW_MAX_HOPS];
    uint32_t rows_per_hop[MW_MAX_HOPS];
    uint32_t error_flags;       /* MW_FLAG_BAD_DESC | MW_FLAG_OUT_CAPACITY | MW_FLAG_BAD_RANK */
    uint32_t reserved0;
} mw_relay_stats;               /* 544 bytes */

/*
 * The node's unicast forwarding table (Section 4.1): next_hop[r] in [0, n_hops) is the egress
 * port / next-hop id towards destination rank r, for every r < n_ranks.  HOST array, copied;
 * 1 <= n_hops <= max_hops.  SYNCHRONISES the device.  Must not be called while work of this
 * context is in flight.
 */
MW_API int32_t mw_set_forwarding(mw_ctx *ctx, const int32_t *next_hop, int32_t n_hops);

/*
 * mw_relay: one step of the recursive model.  The node holds a MultiWrite buffer `in_dev`
 * (one device record: what mw_pack wrote at the source, or what a previous relay wrote)
 * and starts one child MultiWrite per next hop:
 *   child h keeps, in order, the groups whose bitmap names a rank with next_hop == h;
 *   its bitmap is the parent's restricted to those ranks (so no destination is served
 *   twice, Section 4.1), n_dest its popcount, rows concatenated, row_offset rebased;
 *   row_src_token and row_topk travel unchanged.
 * A group's rows are read once and written once per distinct next hop (the number of
 * unique egress ports is the number of copies, Section 4.1).  A child with one destination
 * left is an ordinary write of that buffer (Section 4.3.3 rule 2); a child for this rank
 * itself is what mw_unpack takes as a peer region.  Groups must have ascending, disjoint
 * row ranges inside [0, n_rows); others are dropped with MW_FLAG_BAD_DESC.  Groups that do
 * not fit child_capacity_rows are dropped from that child with MW_FLAG_OUT_CAPACITY.
 * The input's n_desc and n_rows may not exceed max_tokens.
 */
MW_API int32_t mw_relay(mw_ctx *ctx, const mw_recv_peer *in_dev, const mw_relay_child *children_dev,
                 int64_t child_capacity_rows, mw_relay_stats *stats_dev, void *stream);

/*
 * mw_relay as its two halves, for a node that relays one buffer after the other (Section 4.3.3;
 * Section 5.1, relay module).  mw_relay_index builds the children's descriptor tables, the
 * statistics except forward_bytes and error_flags, and -- in the context's workspace -- what
 * the copy needs; mw_relay_copy moves the rows and completes the statistics.  mw_relay is
 * mw_relay_index followed by mw_relay_copy with the same arguments.
 * mw_relay_copy_index_next is mw_relay_copy(ctx, in_dev, children_dev, stats_dev) and
 * mw_relay_index(next_ctx, next_in_dev, next_children_dev, next_child_capacity_rows,
 * next_stats_dev) in ONE launch, with identical results: the index of the next buffer is a
 * chain of memory round trips that moves almost nothing and runs beside the copy of this one.
 * `next_ctx` is another context on the same device (its workspace holds the next index),
 * with its own forwarding table; the two steps' children and statistics must not overlap.
 * A stream of buffers alternates between two contexts:
 *   mw_relay_index(A, buf0); mw_relay_copy_index_next(A, buf0, B, buf1);
 *   mw_relay_copy_index_next(B, buf1, A, buf2); ... ; mw_relay_copy(last).
 */
MW_API int32_t mw_relay_index(mw_ctx *ctx, const mw_recv_peer *in_dev, const mw_relay_child *children_dev,
                       int64_t child_capacity_rows, mw_relay_stats *stats_dev, void *stream);
MW_API int32_t mw_relay_copy(mw_ctx *ctx, const mw_recv_peer *in_dev, const mw_relay_child *children_dev,
                      mw_relay_stats *stats_dev, void *stream);
MW_API int32_t mw_relay_copy_index_next(mw_ctx *ctx, const mw_recv_peer *in_dev, const mw_relay_child *children_dev,
                                 mw_relay_stats *stats_dev, mw_ctx *next_ctx, const mw_recv_peer *next_in_dev,
                                 const mw_relay_child *next_children_dev, int64_t next_child_capacity_rows,
                                 mw_relay_stats *next_stats_dev, void *stream);

/*
 * mw_relay_batch: for a relay that has more than one buffer waiting (Section 5.1, relay module:
 * buffers are relayed one after the other; Section 4.3.3).  ONE launch does
 *     mw_relay_copy(copy[j].ctx, copy[j].in_dev, copy[j].children_dev, copy[j].stats_dev)   for j < n_copy
 * and
 *     mw_relay_index(index[k].ctx, index[k].in_dev, index[k].children_dev,
 *                    index[k].child_capacity_rows, index[k].stats_dev)                      for k < n_index
 * with identical results.  A relay's copy of a 50-megabyte buffer is short enough for what a
 * launch costs by itself (its first waves' dependent fetches, its last waves' tail, the gap to
 * the next launch) to be a sixth of it; with two buffers per launch that cost is paid once for
 * both.  The price is latency: the first buffer of a batch waits for the second.
 * copy, index: HOST arrays (read during the call only) of at most MW_RELAY_BATCH_MAX jobs each;
 * 1 <= n_copy, 0 <= n_index.  All contexts are distinct, on one device, have a forwarding table,
 * and the copy jobs' contexts have the same row size, row stride, top_k and max_tokens.  Every
 * copy job's index must have been made by an EARLIER launch (mw_relay_index, or the index part
 * of an earlier mw_relay_batch or mw_relay_copy_index_next); child_capacity_rows of a copy job
 * is not read.  A stream of buffers over four contexts, two buffers a launch:
 *     mw_relay_index(A, b0); mw_relay_index(B, b1);
 *     mw_relay_batch(copy {A b0, B b1}, index {C b2, D b3}); mw_relay_batch(copy {C, D}, index {A b4, B b5}); ...
 */
#define MW_RELAY_BATCH_MAX 4
typedef struct mw_relay_job {
    mw_ctx *ctx;
    const mw_recv_peer *in_dev;
    const mw_relay_child *children_dev;
    int64_t child_capacity_rows;
    mw_relay_stats *stats_dev;
} mw_relay_job;
MW_API int32_t mw_relay_batch(const mw_relay_job *copy, int32_t n_copy, const mw_relay_job *index, int32_t n_index,
                              void *stream);

/*
 * mw_relay_packets: the relay step for packets -- the paper's own form of it (Section 4.1,
 * "Replication and forwarding": the relay parses the bitmap in front of the payload, makes one
 * copy per distinct egress port and updates the in-packet metadata of each copy so that
 * downstream nodes do not replicate again).  in_dev: one device record.  children_dev: device
 * array of n_hops device pointers, child h a buffer of child_capacity_rows packets.  Child h
 * keeps, in order, the packets whose bitmap names a rank with next_hop == h; the first 32
 * bytes of each copy (the bitmap) are the parent's restricted to those ranks, the rest of the
 * packet is unchanged.  Statistics as mw_relay with every packet its own group; forward_bytes
 * and unicast_bytes count whole packets (header + row).  A header whose id count is not top_k
 * drops the packet (MW_FLAG_BAD_DESC); packets beyond a child's capacity are dropped from that
 * child (MW_FLAG_OUT_CAPACITY); n_rows may not exceed max_tokens.
 */
MW_API int32_t mw_relay_packets(mw_ctx *ctx, const mw_recv_packets *in_dev, void *const *children_dev,
                         int64_t child_capacity_rows, mw_relay_stats *stats_dev, void *stream);

/*
 * mw_relay_packets as its two halves and, for a stream of packet buffers, with the next
 * buffer's index in the copy's launch: the packets' forms of mw_relay_index, mw_relay_copy and
 * mw_relay_copy_index_next (Section 4.1, replication and forwarding; Section 5.1, relay
 * module), with the same rules -- mw_relay_packets is the index followed by the copy, the
 * one-launch form gives identical results, `next_ctx` is another context on the same device
 * with its own forwarding table, and two contexts take turns.
 */
MW_API int32_t mw_relay_packets_index(mw_ctx *ctx, const mw_recv_packets *in_dev, int64_t child_capacity_rows,
                               mw_relay_stats *stats_dev, void *stream);
MW_API int32_t mw_relay_packets_copy(mw_ctx *ctx, const mw_recv_packets *in_dev, void *const *children_dev,
                              mw_relay_stats *stats_dev, void *stream);
MW_API int32_t mw_relay_packets_copy_index_next(mw_ctx *ctx, const mw_recv_packets *in_dev, void *const *children_dev,
                                         mw_relay_stats *stats_dev, mw_ctx *next_ctx,
                                         const mw_recv_packets *next_in_dev, int64_t next_child_capacity_rows,
                                         mw_relay_stats *next_stats_dev, void *stream);

/* ---- simulation and measurement helpers (not part of the dispatch path) ---------------- */

/*
 * Simulated network (Section 4.1 workflow step 4: a payload reaches only the
 * nodes named in its bitmap): from a sender's mw_plan/mw_pack output keep the
 * groups that name dst_rank, in order, rows concatenated, row_offset rebased,
 * bitmaps unchanged.  counts_out_dev[0] = groups kept, [1] = rows kept.
 * Outputs have room for n_tokens entries.
 */
MW_API int32_t mw_sim_deliver(mw_ctx *ctx, const mw_group_desc *desc_dev, const mw_send_stats *stats_dev,
                       int32_t n_tokens, const void *packed_rows_dev,
                       const int32_t *row_src_token_dev, const int32_t *row_topk_dev, int32_t dst_rank,
                       mw_group_desc *desc_out_dev, void *rows_out_dev, int32_t *src_token_out_dev,
                       int32_t *topk_out_dev, uint32_t *counts_out_dev, void *stream);

/* Plain streaming device copy of n_bytes (multiple of 16): the copy ceiling the
 * row movers are compared with, and the reference kernel for counter scaling. */
MW_API int32_t mw_copy_bytes(void *dst_dev, const void *src_dev, int64_t n_bytes, void *stream);

/* Copy a statistics block to the host.  SYNCHRONISES `stream`.  mw_get_recv_stats also lets
 * the context remember how many rows the peers' buffers held, and the next mw_unpack sizes its
 * launch for about that many rows instead of max_recv_rows (a hint only: any number of rows
 * up to max_recv_rows is still handled). */
MW_API int32_t mw_get_send_stats(mw_ctx *ctx, const mw_send_stats *stats_dev, mw_send_stats *host_out, void *stream);
MW_API int32_t mw_get_recv_stats(mw_ctx *ctx, const mw_recv_stats *stats_dev, mw_recv_stats *host_out, void *stream);
MW_API int32_t mw_get_relay_stats(mw_ctx *ctx, const mw_relay_stats *stats_dev, mw_relay_stats *host_out, void *stream);

/*
 * Measurement hook.  While a pair of hipEvent_t handles (created by the caller with
 * timing enabled, passed as void*) is set for a kernel, every launch of that kernel by
 * this context records `ev_start` just before it and `ev_stop` just after it on the
 * call's stream, so the caller can read the kernel's own duration with
 * hipEventElapsedTime.  NULL, NULL switches the hook off (the default).
 */
#define MW_KERNEL_PLAN_RANK    0
#define MW_KERNEL_PLAN_GROUPS  1
#define MW_KERNEL_PACK         2
#define MW_KERNEL_RECV_INDEX   3
#define MW_KERNEL_EXPAND       4
#define MW_KERNEL_AG_PACK      5   /* mw_pack_allgather's copy */
#define MW_KERNEL_AG_GATHER    6   /* mw_unpack_allgather's shard assembly */
#define MW_KERNEL_RELAY_INDEX  7
#define MW_KERNEL_RELAY_COPY   8
#define MW_KERNEL_PLAN_PACK    9   /* mw_plan_pack's single kernel */
#define MW_KERNEL_PACK_QUANT   10  /* mw_pack_quantize's kernel */
#define MW_KERNEL_COMBINE      11  /* mw_combine_gather's kernel */
#define MW_KERNEL_COUNT        12
MW_API int32_t mw_ctx_set_timing_events(mw_ctx *ctx, int32_t kernel, void *ev_start, void *ev_stop);

MW_API const char *mw_status_string(int32_t status);

#ifdef __cplusplus
}
#endif
#endif /* MW_H_ */
