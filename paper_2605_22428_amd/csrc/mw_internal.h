// Internal declarations shared by the HIP sources of the MultiWrite library.
// Not installed; the public C ABI is include/mw.h.
#ifndef MW_INTERNAL_H_
#define MW_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mw.h"

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

#define MW_PLAN_STATE_WORDS 264   // 256 histogram bins + kept tokens + flags + two counts of workgroups done (+ padding)

// (local expert slot, rank among the peer's rows for that expert); le < 0 = unused slot
struct mw_hit { int32_t le; int32_t rank; };

// One received row as the expander needs it, in one 32-byte record: where it lies, its
// source token and peer, how many local experts it goes to and the first of them.  Further
// (expert slot, rank) pairs are in the row's hit slots 1 .. n_hits - 1.
struct mw_row_rec {
    const void *src;
    int32_t src_token;
    int32_t peer;
    int32_t n_hits;     // 0: nothing to deliver
    int32_t le0;        // first local expert slot
    int32_t rank0;      // rank among the peer's rows for that expert
    int32_t reserved0;
};

// Launch shape of the row movers: one 16-byte chunk per lane, grid x = segment of `bs` chunks
// of a row, grid y = row, so workgroups are dispatched in address order along a row and then
// row by row.  Measured on MI355X (expander, 30590 received rows, GB/s of HBM traffic):
//
//   row bytes              2048  4096  7168  8192  10240  12288  14336  16384  24576
//   single-wave segments   4413  4753  4848  4872   5879   6470   6485   6350   6427
//   one workgroup per row  5824  6194  6158  6332   5976   6225   6073   6225   6448
//
// Rows of up to 10 KiB are moved by one workgroup each (a wave per KiB).  Longer rows that are
// whole 128-byte cache lines (bf16 rows of 14336 bytes) are cut into single-wave workgroups:
// whole-row workgroups of 14 waves leave an eighth of a CU's wave slots empty, and several
// chunks per lane, or all rows' first segments first, are slower still.  Rows that are not whole
// cache lines (fp8 rows of 7392 bytes start and end inside lines) are never cut into single
// waves, so the lines two pieces share are touched from one CU: cut, such rows were 40 % slower.
constexpr uint32_t kRowGridMax = 32768;       // grid y; further rows by striding
struct mw_row_shape { int bs; int nseg; };
static inline mw_row_shape mw_row_shape_of(int chunks)
{
    if (chunks < 1) return mw_row_shape{64, 1};
    if (chunks % 8 == 0 && chunks > 640) return mw_row_shape{64, (chunks + 63) / 64};
    int b = (chunks + 63) / 64 * 64;
    if (b > 1024) b = 1024;
    return mw_row_shape{b, (chunks + b - 1) / b};
}

// Host-side context.  Every d_* pointer is a slice of the caller's workspace.
struct mw_ctx {
    mw_config cfg;
    int32_t n_local;        // L: experts hosted by my_rank
    int32_t hit_slots;      // Kd = max(1, min(K, L)): local experts one row can name
    int32_t mask_words;     // ceil(R / 64): bitmap words that can be non-zero
    int64_t x_row_bytes;    // payload part of a row
    int64_t s_row_bytes;    // scale part of a row (fp8) or 0
    int64_t row_bytes;
    int64_t row_stride;     // bytes from one row to the next in packed / received row arrays (>= row_bytes)
    int device;
    int n_cu;
    // workspace slices
    int32_t *d_eslot;       // [E] (rank << 16) | slot of expert e among the experts of its rank
    uint64_t *d_plan_cnt;       // [max_tokens] packed per-token counters; zero between plans
    uint32_t *d_plan_state;     // [MW_PLAN_STATE_WORDS] rows per destination, kept tokens, flags, workgroups done; zero between plans
    uint64_t *d_sort_key;       // [max_tokens rounded up to 1024] sorted chunks of the large-batch plan (or null)
    uint32_t *d_sort_sec;       // same count: second sort word
    uint32_t *d_chunk_kept;     // [64] kept tokens per chunk
    uint64_t *d_row_cnt;        // [max_tokens] a packed row's counters (large-batch plan, or null)
    unsigned char *d_row_start; // [max_tokens] 1: a group starts at this packed row
    uint32_t ride_wait_limit;   // polls a riding plan's second half waits for its first
    uint32_t options;           // MW_OPT_*
    uint32_t *d_flags;      // [4] 1: receive flags, 2: receive workgroups done
    uint32_t *d_base;       // [L][R] first output row of (local expert, peer)
    mw_row_rec *d_recs;     // [max_recv_rows]
    uint32_t *d_cnt;        // [L][R] rows of peer p delivered to local expert le
    uint32_t *d_row_base;   // [R + 1] exclusive prefix of the peers' n_rows
    uint32_t *d_addr_cnt;   // [R] rows of peer p whose group names this rank
    mw_hit *d_hits;         // [max_recv_rows][Kd]
    int32_t *d_row_map;     // [max_tokens] mw_sim_deliver: kept row -> sender row
    int64_t recv_rows_hint; // rows the peers' buffers held at the last mw_get_recv_stats (0: unknown)
    // relay (only with cfg.max_hops > 0)
    int32_t n_hops;         // 0 until mw_set_forwarding
    uint64_t *d_hop_bits;   // [MW_MAX_HOPS][4] ranks served through each next hop
    int32_t *d_group_of_row;// [max_tokens]
    uint32_t *d_child_pos;  // [max_tokens][MW_MAX_HOPS] first child row of (group, hop) or kNoChild
    uint32_t *d_relay_flags;// [1]
    // measurement hook: optional event pairs recorded around single kernels
    hipEvent_t ev_start[MW_KERNEL_COUNT];
    hipEvent_t ev_stop[MW_KERNEL_COUNT];
};

// Records the context's timing events (if set) around one kernel launch.
struct mw_timed {
    mw_ctx *ctx; int k; hipStream_t s;
    mw_timed(mw_ctx *c, int kernel, hipStream_t st) : ctx(c), k(kernel), s(st)
    {
        if (ctx->ev_start[k]) (void)hipEventRecord(ctx->ev_start[k], s);
    }
    ~mw_timed()
    {
        if (ctx->ev_stop[k]) (void)hipEventRecord(ctx->ev_stop[k], s);
    }
};

#define MW_HIP_CHECK(expr)                         \
    do {                                           \
        hipError_t e_ = (expr);                    \
        if (e_ != hipSuccess) return MW_ERR_HIP;   \
    } while (0)

static inline int64_t mw_align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

// Header in front of a packet's row: 4 bitmap words, source token, id count, the ids; whole
// 128-byte lines so that the row behind it starts on a cache line.
static inline int64_t mw_packet_header_bytes_of(int32_t top_k) { return mw_align_up(40 + 4 * (int64_t)top_k, 128); }

// ---- device helpers ---------------------------------------------------------------------
#ifdef __HIPCC__
// Streaming 16-byte accesses: payload rows are touched once, keep them out of the way of
// the small, reused index arrays.
__device__ __forceinline__ u32x4 mw_ld16(const u32x4 *p) { return __builtin_nontemporal_load(p); }
// The store is streaming and written through (sc0 sc1 nt): the lines leave the L2 as they are
// written, so the end of the kernel has nothing left to write back and the next launch on the
// stream starts about two microseconds sooner than with a plain non-temporal store.
__device__ __forceinline__ void mw_st16(u32x4 *p, u32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt" ::"v"(p), "v"(v) : "memory");
}
// The same load through a pointer that was read from memory: saying that it is a global
// address keeps it off the flat path, whose loads also count as LDS traffic and would make
// every later wait for a scalar load wait for the payload too.
typedef const __attribute__((address_space(1))) u32x4 *mw_gptr16;
__device__ __forceinline__ u32x4 mw_ld16_global(const void *row, int chunk)
{
    return __builtin_nontemporal_load((mw_gptr16)row + chunk);
}

// Wave-uniform values: "the value is needed in scalar registers here".  The compiler
// otherwise sinks every scalar load to its first use, one wait per load; pinning several
// values side by side makes it issue their loads together and wait once.
#define MW_PIN_S(x) asm volatile("" : "+s"(x))
#define MW_PIN_PTR(p) do { uint32_t lo_ = (uint32_t)(uintptr_t)(p); asm volatile("" : "+s"(lo_)); } while (0)
#define MW_PIN_S4(v) asm volatile("" : "+s"((v).x), "+s"((v).y), "+s"((v).z), "+s"((v).w))

// Workgroup barrier for data exchanged through LDS only.  __syncthreads() also waits until
// every global load and store of the wave has completed (about a microsecond each time a
// store or a prefetch is outstanding); this one orders LDS accesses and nothing else.
__device__ __forceinline__ void mw_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---- publication between workgroups of ONE launch ------------------------------------------
// A workgroup that has produced (or finished reading) data another workgroup of the same launch
// depends on reports through a counter; the other side reads the counter and then the data.
//   producer   every lane: its stores / atomics;  mw_publish_barrier();  one lane: mw_report(counter)
//   consumer   one lane: reads the counter (mw_report's return value, or a poll followed by
//              mw_acquire_after_poll());  workgroup barrier;  every lane: reads the data
// In memory-model terms: the barrier orders every lane's accesses before the reporting lane's
// (workgroup scope); the report is a release (and, as a read-modify-write whose value decides who
// is last, an acquire) at agent scope; the consumer's counter read is an acquire at agent scope;
// happens-before is transitive over the two scopes, so everything the producer's lanes did is
// visible to every lane of the consumer after its barrier, whatever cache either side runs behind.
// The data itself is additionally written and read with agent-scope atomics, which are performed
// at the device's coherence point, so the release and acquire fences find next to nothing to
// write back or invalidate on their own account.
// MW_PUBLISH_FENCES 0 builds the same protocol from relaxed atomics and an explicit wait for all
// outstanding memory operations of every lane (s_waitcnt vmcnt(0)) in front of the barrier:
// correct on gfx950, where an agent-scope atomic or a write-through store is complete once
// acknowledged, but an argument about this hardware rather than about the memory model.
#ifndef MW_PUBLISH_FENCES
#define MW_PUBLISH_FENCES 0
#endif
__device__ __forceinline__ void mw_publish_barrier()
{
#if !MW_PUBLISH_FENCES
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#endif
    __syncthreads();
}
__device__ __forceinline__ uint32_t mw_report(uint32_t *counter)
{
#if MW_PUBLISH_FENCES
    return __hip_atomic_fetch_add(counter, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
#else
    return __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#endif
}
__device__ __forceinline__ void mw_acquire_after_poll()
{
#if MW_PUBLISH_FENCES
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
#endif
}

// Exclusive prefix sum over one value per thread of a block (blockDim.x multiple of 64,
// at most 1024).  `wave_tot` is LDS scratch of 17 words.  Returns the exclusive prefix;
// *total receives the block total.  Ends with a barrier so the scratch can be reused.  The
// barriers order LDS only.  Every wave adds up the waves' totals for itself (one LDS read a
// lane and a 16-lane scan): a single thread walking them took a dependent LDS round trip per
// wave, a microsecond for 1024 lanes.
__device__ __forceinline__ uint32_t mw_block_exscan(uint32_t v, uint32_t *wave_tot, uint32_t *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_wave = blockDim.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t o = __shfl_up(inc, d, 64);
        if (lane >= d) inc += o;
    }
    if (lane == 63) wave_tot[wave] = inc;
    mw_lds_barrier();
    uint32_t t = (lane < n_wave) ? wave_tot[lane] : 0u;
#pragma unroll
    for (int d = 1; d < 16; d <<= 1) {
        uint32_t o = __shfl_up(t, d, 64);
        if (lane >= d) t += o;
    }
    const uint32_t before = (wave > 0) ? (uint32_t)__shfl((int)t, wave - 1, 64) : 0u;
    *total = (uint32_t)__shfl((int)t, n_wave - 1, 64);
    mw_lds_barrier();
    return before + inc - v;
}
#endif

// payload and scale bytes of a row of `c` (checks the row format's constraints); returns a status
int32_t mw_row_geometry(const mw_config &c, int64_t *x_bytes, int64_t *s_bytes);

// kernels' host launchers (one per source file)
int32_t mw_launch_plan(mw_ctx *ctx, const int32_t *topk, int32_t T, uint64_t *mask, int32_t *perm,
                       mw_group_desc *desc, mw_send_stats *stats, hipStream_t s);
int32_t mw_launch_pack(mw_ctx *ctx, const void *x, const float *scales, const int32_t *topk,
                       const int32_t *perm, const mw_send_stats *stats, int32_t T, void *packed,
                       int32_t *row_src_token, int32_t *row_topk, hipStream_t s);
int32_t mw_launch_plan_pack(mw_ctx *ctx, const int32_t *topk, int32_t T, const void *x, const float *scales,
                            uint64_t *mask, int32_t *perm, mw_group_desc *desc, mw_send_stats *stats, void *packed,
                            int32_t *row_src_token, int32_t *row_topk, hipStream_t s);
int32_t mw_launch_unpack_index(mw_ctx *ctx, const void *peers, bool packets, int32_t P, int64_t cap,
                               int64_t *expert_offsets, mw_recv_stats *stats, hipStream_t s);
int32_t mw_launch_pack_quantize(mw_ctx *ctx, const void *x_bf16, const int32_t *topk, const int32_t *perm,
                                const mw_send_stats *stats, int32_t T, void *packed, int32_t *row_src_token,
                                int32_t *row_topk, hipStream_t s);
int32_t mw_launch_pack_packets(mw_ctx *ctx, const void *x, const float *scales, const int32_t *topk,
                               const uint64_t *mask, const int32_t *perm, const mw_send_stats *stats, int32_t T,
                               void *packets, hipStream_t s);
int32_t mw_launch_unpack_expand(mw_ctx *ctx, int32_t P, void *out_rows, float *out_scales, int64_t cap,
                                int32_t *out_src_peer, int32_t *out_src_token, hipStream_t s);
int32_t mw_launch_unpack_expand_index_next(mw_ctx *ctx, int32_t P, void *out_rows, float *out_scales, int64_t cap,
                                           int32_t *out_src_peer, int32_t *out_src_token, mw_ctx *next,
                                           const mw_recv_peer *next_peers, int32_t next_P, int64_t next_cap,
                                           int64_t *next_expert_offsets, mw_recv_stats *next_stats, hipStream_t s);
int32_t mw_launch_allgather_step(mw_ctx *ctx, const void *own_shard, int64_t shard_bytes, void *send_buf,
                                 mw_group_desc *desc, mw_send_stats *stats, const void *const *shards, void *out,
                                 hipStream_t s);
// the arguments of an mw_pack that rides in another launch (mw_stream_step)
struct mw_pack_call {
    const void *x; const float *scales; const int32_t *topk; const int32_t *perm; const mw_send_stats *stats;
    int32_t n_tokens; void *packed; int32_t *row_src_token; int32_t *row_topk;
};
int32_t mw_launch_unpack_expand_index_plan_next(mw_ctx *ctx, int32_t P, void *out_rows, float *out_scales, int64_t cap,
                                                int32_t *out_src_peer, int32_t *out_src_token, mw_ctx *next,
                                                const mw_recv_peer *next_peers, int32_t next_P, int64_t next_cap,
                                                int64_t *next_expert_offsets, mw_recv_stats *next_stats,
                                                const int32_t *next_topk, int32_t next_T, uint64_t *next_mask,
                                                int32_t *next_perm, mw_group_desc *next_desc,
                                                mw_send_stats *next_send_stats, const mw_pack_call *pack, hipStream_t s);
int32_t mw_launch_combine(mw_ctx *ctx, int32_t P, const void *y, int64_t cap, void *ret, int64_t ret_cap, hipStream_t s);
int32_t mw_launch_plan_allgather(mw_ctx *ctx, int64_t shard_bytes, mw_group_desc *desc,
                                 mw_send_stats *stats, hipStream_t s);
int32_t mw_launch_plan_allgather_split(mw_ctx *ctx, int64_t shard_bytes, int64_t direct_bytes, mw_group_desc *desc,
                                       mw_send_stats *stats, hipStream_t s);
int32_t mw_launch_gather_split(mw_ctx *ctx, const void *const *direct, const void *const *relayed,
                               int64_t shard_bytes, int64_t direct_bytes, void *out, hipStream_t s);
int32_t mw_launch_copy(mw_ctx *ctx, void *dst, const void *src, int64_t n_bytes, hipStream_t s);
int32_t mw_launch_gather_shards(mw_ctx *ctx, const void *const *shards, int64_t shard_bytes, void *out,
                                hipStream_t s);
int32_t mw_launch_relay_batch(const mw_relay_job *copy, int32_t n_copy, const mw_relay_job *index, int32_t n_index,
                              hipStream_t s);
int32_t mw_launch_relay(mw_ctx *ctx, const mw_recv_peer *in, const mw_relay_child *children, int64_t cap,
                        mw_relay_stats *stats, hipStream_t s);
int32_t mw_launch_relay_index(mw_ctx *ctx, const mw_recv_peer *in, const mw_relay_child *children, int64_t cap,
                              mw_relay_stats *stats, hipStream_t s);
int32_t mw_launch_relay_copy(mw_ctx *ctx, const mw_recv_peer *in, const mw_relay_child *children,
                             mw_relay_stats *stats, mw_ctx *next, const mw_recv_peer *next_in,
                             const mw_relay_child *next_children, int64_t next_cap, mw_relay_stats *next_stats,
                             hipStream_t s);
int32_t mw_launch_relay_packets_index(mw_ctx *ctx, const mw_recv_packets *in, int64_t cap, mw_relay_stats *stats,
                                      hipStream_t s);
int32_t mw_launch_relay_packets_copy(mw_ctx *ctx, const mw_recv_packets *in, void *const *children,
                                     mw_relay_stats *stats, mw_ctx *next, const mw_recv_packets *next_in,
                                     int64_t next_cap, mw_relay_stats *next_stats, hipStream_t s);
int32_t mw_launch_relay_packets(mw_ctx *ctx, const mw_recv_packets *in, void *const *children, int64_t cap,
                                mw_relay_stats *stats, hipStream_t s);
int32_t mw_launch_sim_deliver(mw_ctx *ctx, const mw_group_desc *desc, const mw_send_stats *stats,
                              int32_t T, const void *rows, const int32_t *src_token, const int32_t *topk,
                              int32_t dst_rank, mw_group_desc *desc_out, void *rows_out,
                              int32_t *src_token_out, int32_t *topk_out, uint32_t *counts, hipStream_t s);

#endif  // MW_INTERNAL_H_
