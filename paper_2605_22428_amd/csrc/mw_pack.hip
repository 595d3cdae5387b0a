// Payload packer and plain copies (send side bulk movers).
//
// Paper hooks: Section 1 -- only one copy of the same data is injected, so a token's row
// is written once however many ranks its bitmap names; Section 5.2 step 1 -- data is
// loaded into the pre-allocated send buffer; Section 4.3.4 (statelessness) -- the row's
// source token index and top-k ids travel with it.
//
// The packer is a row gather bound by HBM bandwidth: packed[i] = x[perm[i]].  Rows are
// multiples of 16 bytes.  Small workgroups, each moving consecutive 16-byte chunks of one
// row with a single streaming load and store per lane: on MI355X many light waves
// follow the plain-copy ceiling more closely than fewer waves with several loads in flight.
// Nothing is reused, so accesses are non-temporal.
#include "mw_internal.h"
#include "mw_pack_dev.h"
#include "mw_plan_dev.h"

namespace {

// blockIdx.x = segment of blockDim.x chunks, blockIdx.y walks packed rows.
__global__ __launch_bounds__(1024) void k_pack(const int32_t *__restrict__ perm, const mw_send_stats *__restrict__ stats,
                                               const u32x4 *__restrict__ x, const u32x4 *__restrict__ scales,
                                               int xc, int sc, int ns, int K,      // (in registers when a wave starts)
                                               const int32_t *__restrict__ topk, u32x4 *__restrict__ packed,
                                               int32_t *__restrict__ row_src_token, int32_t *__restrict__ row_topk)
{
    mw_pack_body(x, scales, xc, sc, ns, topk, K, perm, stats, packed, row_src_token, row_topk, blockIdx.x, blockIdx.y,
                 gridDim.y);
}

// The packer for packets (Section 6.4: the bitmap embedded in front of the payload): packet i =
// header | row of token perm[i], `hc` header chunks then the row's chunks.  Same launch shape
// as k_pack; the workgroup of the row's first segment also writes the header, one 32-bit word
// per lane: words 0..7 the bitmap, 8 the token index, 9 the id count, then the ids, then zeros.
__global__ __launch_bounds__(1024) void k_pack_packets(const u32x4 *__restrict__ x, const u32x4 *__restrict__ scales,
                                                       int xc, int sc, int hc, const int32_t *__restrict__ topk, int K,
                                                       const uint64_t *__restrict__ mask,
                                                       const int32_t *__restrict__ perm,
                                                       const mw_send_stats *__restrict__ stats,
                                                       u32x4 *__restrict__ packets)
{
    uint32_t gdim = gridDim.y, bdim = blockDim.x;
    MW_PIN_S(gdim); MW_PIN_S(bdim); MW_PIN_S(xc); MW_PIN_S(sc); MW_PIN_S(hc); MW_PIN_S(K);
    MW_PIN_PTR(x); MW_PIN_PTR(scales); MW_PIN_PTR(topk); MW_PIN_PTR(mask); MW_PIN_PTR(packets);
    uint32_t i = blockIdx.y;
    int32_t t = perm[i];
    uint32_t n_rows = stats->n_rows;
    MW_PIN_S(t); MW_PIN_S(n_rows);
    const int n = xc + sc;
    const int c = blockIdx.x * bdim + threadIdx.x;
    while (i < n_rows) {
        u32x4 *pk = packets + (size_t)i * (hc + n);
        if (c < n) {
            const u32x4 v = (c < xc) ? mw_ld16(x + (size_t)t * xc + c) : mw_ld16(scales + (size_t)t * sc + (c - xc));
            mw_st16(pk + hc + c, v);
        }
        if (blockIdx.x == 0) {
            uint32_t *hw = (uint32_t *)pk;
            const uint32_t *mw = (const uint32_t *)(mask + (size_t)t * MW_MASK_WORDS);
            for (int j = threadIdx.x; j < hc * 4; j += bdim) {
                uint32_t v = 0;
                if (j < 2 * MW_MASK_WORDS) v = mw[j];
                else if (j == 8) v = (uint32_t)t;
                else if (j == 9) v = (uint32_t)K;
                else if (j < 10 + K) v = (uint32_t)topk[(size_t)t * K + (j - 10)];
                hw[j] = v;
            }
        }
        i += gdim;
        if (i < n_rows) t = perm[i];
    }
}

// Quantise-in-pack: the packer for fp8 rows fed with bf16 rows, so the quantised copy of the
// batch is never written and read back on its own (a separate quantiser would add
// 2 * N * (H + H / 32) bytes of traffic to the 2 H + H + H / 32 per row moved here).
// Contract, in IEEE single precision, one rounding per operation:
//   per 128 consecutive elements: a = max |x|, a_c = max(a, 2^-20), scale = a_c / 448 (stored),
//   code = e4m3 (OCP "fn", largest finite 448) nearest to x * (448 / a_c) limited to +-448,
//   ties to the even mantissa, sign kept.  Inputs must be finite.
// One workgroup per packed row, one 16-byte chunk (8 elements) per lane: a block of 128 elements
// is 16 neighbouring lanes, whose maxima meet by four exchanges inside the wave.  The
// conversion is the hardware's (round to nearest even); the limit to +-448 in front of it means
// it never sees a value it would have to saturate.
__device__ __forceinline__ float mw_bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float mw_bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

template <int U>
__global__ __launch_bounds__(1024) void k_pack_quant(const u32x4 *__restrict__ x, int ic, int H,
                                                     const int32_t *__restrict__ topk, int K,
                                                     const int32_t *__restrict__ perm,
                                                     const mw_send_stats *__restrict__ stats,
                                                     unsigned char *__restrict__ packed, uint64_t row_stride,
                                                     int32_t *__restrict__ row_src_token, int32_t *__restrict__ row_topk)
{
    const uint32_t gdim = gridDim.x, bdim = blockDim.x;
    uint32_t i = blockIdx.x;
    int32_t t = perm[i];
    const uint32_t n_rows = stats->n_rows;
    while (i < n_rows) {
        unsigned char *row = packed + (size_t)i * row_stride;
        // ic is a multiple of 64: whole waves.  A lane's U chunks are requested together.
        for (int c0 = threadIdx.x; c0 < ic; c0 += U * bdim) {
            u32x4 vv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = c0 + u * bdim;
                if (c < ic) vv[u] = mw_ld16(x + (size_t)t * ic + c);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = c0 + u * bdim;
                if (c >= ic) break;
                const u32x4 v = vv[u];
                float f[8] = {mw_bf16_lo(v.x), mw_bf16_hi(v.x), mw_bf16_lo(v.y), mw_bf16_hi(v.y),
                              mw_bf16_lo(v.z), mw_bf16_hi(v.z), mw_bf16_lo(v.w), mw_bf16_hi(v.w)};
                float a = 0.0f;
#pragma unroll
                for (int j = 0; j < 8; ++j) a = fmaxf(a, fabsf(f[j]));
#pragma unroll
                for (int d = 1; d < 16; d <<= 1) a = fmaxf(a, __shfl_xor(a, d, 64));
                const float a_c = fmaxf(a, 0x1p-20f);
                const float scale = a_c / 448.0f, inv = 448.0f / a_c;
#pragma unroll
                for (int j = 0; j < 8; ++j) f[j] = fminf(fmaxf(f[j] * inv, -448.0f), 448.0f);
                uint32_t lo = 0, hi = 0;
                lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[0], f[1], lo, false);
                lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[2], f[3], lo, true);
                hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[4], f[5], hi, false);
                hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[6], f[7], hi, true);
                __builtin_nontemporal_store(((unsigned long long)hi << 32) | lo,
                                            (unsigned long long *)(row + 8 * (size_t)c));
                if ((c & 15) == 0) *(float *)(row + H + 4 * (c >> 4)) = scale;
            }
        }
        if (threadIdx.x == 0) row_src_token[i] = t;
        for (int j = threadIdx.x; j < K; j += bdim) row_topk[(size_t)i * K + j] = topk[(size_t)t * K + j];
        i += gdim;
        if (i < n_rows) t = perm[i];
    }
}

// Lanes per workgroup of the flat copies below: single waves (a plain copy of several hundred
// megabytes runs about 2 % faster with 64-lane workgroups than with 256-lane ones).
constexpr int kFlat = 64;

// Flat streaming copy, one chunk per lane.
__global__ __launch_bounds__(kFlat) void k_copy(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst,
                                              int64_t n_chunks)
{
    const int64_t c = (int64_t)blockIdx.x * kFlat + threadIdx.x;
    if (c < n_chunks) mw_st16(dst + c, mw_ld16(src + c));
}

// AllGather receive assembly: shard p goes to out + p * shard_bytes.  blockIdx.y = p.
__global__ __launch_bounds__(kFlat) void k_gather_shards(const u32x4 *const *__restrict__ shards,
                                                       int64_t shard_chunks, u32x4 *__restrict__ out)
{
    const u32x4 *src = shards[blockIdx.y];
    u32x4 *dst = out + (int64_t)blockIdx.y * shard_chunks;
    const int64_t c = (int64_t)blockIdx.x * kFlat + threadIdx.x;
    if (c < shard_chunks) mw_st16(dst + c, mw_ld16(src + c));
}

// A whole AllGather step of a stream of them in one launch (Section 5.2, steps 1 and 4, for two
// consecutive operations): rows y < R of the grid assemble the shards received for one
// operation, row R copies this rank's shard of the next one into its send buffer, and the first
// workgroup of row R + 1 writes that operation's one-row plan.
__global__ __launch_bounds__(kFlat) void k_allgather_step(const u32x4 *const *__restrict__ shards,
                                                        int64_t shard_chunks, u32x4 *__restrict__ out, int R,
                                                        const u32x4 *__restrict__ own, u32x4 *__restrict__ send_buf,
                                                        mw_group_desc *desc, mw_send_stats *stats)
{
    const int64_t c = (int64_t)blockIdx.x * kFlat + threadIdx.x;
    if ((int)blockIdx.y < R) {
        if (c < shard_chunks) mw_st16(out + (int64_t)blockIdx.y * shard_chunks + c, mw_ld16(shards[blockIdx.y] + c));
    } else if ((int)blockIdx.y == R) {
        if (c < shard_chunks) mw_st16(send_buf + c, mw_ld16(own + c));
    } else if (blockIdx.x == 0) {
        mw_plan_allgather_body(R, (uint64_t)shard_chunks * 16u, desc, stats);
    }
}

// AllGather assembly of split fragments (Section 5.2): chunk c of shard p comes from the
// direct piece while c < direct_chunks, else from the relayed piece.  blockIdx.y = p.
__global__ __launch_bounds__(kFlat) void k_gather_split(const u32x4 *const *__restrict__ direct,
                                                      const u32x4 *const *__restrict__ relayed,
                                                      int64_t shard_chunks, int64_t direct_chunks,
                                                      u32x4 *__restrict__ out)
{
    const int64_t c = (int64_t)blockIdx.x * kFlat + threadIdx.x;
    if (c >= shard_chunks) return;
    const u32x4 *src = (c < direct_chunks) ? direct[blockIdx.y] + c : relayed[blockIdx.y] + (c - direct_chunks);
    mw_st16(out + (int64_t)blockIdx.y * shard_chunks + c, mw_ld16(src));
}

}  // namespace

int32_t mw_launch_gather_split(mw_ctx *ctx, const void *const *direct, const void *const *relayed,
                               int64_t shard_bytes, int64_t direct_bytes, void *out, hipStream_t s)
{
    const int64_t shard_chunks = shard_bytes / 16;
    if (shard_chunks == 0) return MW_OK;
    const int64_t gx = (shard_chunks + kFlat - 1) / kFlat;
    if (gx > 0x7fffffffLL) return MW_ERR_UNSUPPORTED;
    {
        mw_timed tm(ctx, MW_KERNEL_AG_GATHER, s);
        hipLaunchKernelGGL(k_gather_split, dim3((uint32_t)gx, ctx->cfg.n_ranks), dim3(kFlat), 0, s,
                           (const u32x4 *const *)direct, (const u32x4 *const *)relayed, shard_chunks, direct_bytes / 16,
                           (u32x4 *)out);
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

int32_t mw_launch_pack(mw_ctx *ctx, const void *x, const float *scales, const int32_t *topk,
                       const int32_t *perm, const mw_send_stats *stats, int32_t T, void *packed,
                       int32_t *row_src_token, int32_t *row_topk, hipStream_t s)
{
    if (T == 0) return MW_OK;
    const int xc = (int)(ctx->x_row_bytes / 16), sc = (int)(ctx->s_row_bytes / 16);
    const mw_row_shape shape = mw_row_shape_of(xc + sc);
    const uint32_t gy = (uint32_t)T < kRowGridMax ? (uint32_t)T : kRowGridMax;
    {
        mw_timed tm(ctx, MW_KERNEL_PACK, s);
        hipLaunchKernelGGL(k_pack, dim3(shape.nseg, gy), dim3(shape.bs), 0, s, perm, stats, (const u32x4 *)x,
                           (const u32x4 *)scales, xc, sc, (int)(ctx->row_stride / 16), ctx->cfg.top_k, topk,
                           (u32x4 *)packed, row_src_token, row_topk);
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

int32_t mw_launch_pack_packets(mw_ctx *ctx, const void *x, const float *scales, const int32_t *topk,
                               const uint64_t *mask, const int32_t *perm, const mw_send_stats *stats, int32_t T,
                               void *packets, hipStream_t s)
{
    if (T == 0) return MW_OK;
    const int xc = (int)(ctx->x_row_bytes / 16), sc = (int)(ctx->s_row_bytes / 16);
    const int hc = (int)(mw_packet_header_bytes_of(ctx->cfg.top_k) / 16);
    const mw_row_shape shape = mw_row_shape_of(xc + sc);      // the header is whole cache lines
    const uint32_t gy = (uint32_t)T < kRowGridMax ? (uint32_t)T : kRowGridMax;
    {
        mw_timed tm(ctx, MW_KERNEL_PACK, s);
        hipLaunchKernelGGL(k_pack_packets, dim3(shape.nseg, gy), dim3(shape.bs), 0, s, (const u32x4 *)x,
                           (const u32x4 *)scales, xc, sc, hc, topk, ctx->cfg.top_k, mask, perm, stats, (u32x4 *)packets);
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

int32_t mw_launch_pack_quantize(mw_ctx *ctx, const void *x_bf16, const int32_t *topk, const int32_t *perm,
                                const mw_send_stats *stats, int32_t T, void *packed, int32_t *row_src_token,
                                int32_t *row_topk, hipStream_t s)
{
    if (T == 0) return MW_OK;
    const int H = ctx->cfg.hidden, ic = H / 8;                  // H % 512 == 0 for fp8 rows
    // Two chunks per lane, both requested before either is processed: unlike the plain row
    // movers this kernel has a long chain behind every load (exchanges, two divisions, the
    // conversions), and a second load in flight hides it (23 -> 17 us at 4096 x 7168; four are
    // no better).
    constexpr int U = 2;
    int bs = (ic / U + 63) / 64 * 64;
    if (bs > 1024) bs = 1024;
    const uint32_t gx = (uint32_t)T < kRowGridMax ? (uint32_t)T : kRowGridMax;
    {
        mw_timed tm(ctx, MW_KERNEL_PACK_QUANT, s);
        hipLaunchKernelGGL(k_pack_quant<U>, dim3(gx), dim3(bs), 0, s, (const u32x4 *)x_bf16, ic, H, topk, ctx->cfg.top_k,
                           perm, stats, (unsigned char *)packed, (uint64_t)ctx->row_stride, row_src_token, row_topk);
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

int32_t mw_launch_copy(mw_ctx *ctx, void *dst, const void *src, int64_t n_bytes, hipStream_t s)
{
    const int64_t n_chunks = n_bytes / 16;
    if (n_chunks == 0) return MW_OK;
    const int64_t grid = (n_chunks + kFlat - 1) / kFlat;
    if (grid > 0x7fffffffLL) return MW_ERR_UNSUPPORTED;
    if (ctx) {
        mw_timed tm(ctx, MW_KERNEL_AG_PACK, s);
        hipLaunchKernelGGL(k_copy, dim3((uint32_t)grid), dim3(kFlat), 0, s, (const u32x4 *)src, (u32x4 *)dst, n_chunks);
    } else {
        hipLaunchKernelGGL(k_copy, dim3((uint32_t)grid), dim3(kFlat), 0, s, (const u32x4 *)src, (u32x4 *)dst, n_chunks);
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

int32_t mw_launch_gather_shards(mw_ctx *ctx, const void *const *shards, int64_t shard_bytes, void *out,
                                hipStream_t s)
{
    const int64_t shard_chunks = shard_bytes / 16;
    if (shard_chunks == 0) return MW_OK;
    const int64_t gx = (shard_chunks + kFlat - 1) / kFlat;
    if (gx > 0x7fffffffLL) return MW_ERR_UNSUPPORTED;
    {
        mw_timed tm(ctx, MW_KERNEL_AG_GATHER, s);
        hipLaunchKernelGGL(k_gather_shards, dim3((uint32_t)gx, ctx->cfg.n_ranks), dim3(kFlat), 0, s,
                           (const u32x4 *const *)shards, shard_chunks, (u32x4 *)out);
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}

int32_t mw_launch_allgather_step(mw_ctx *ctx, const void *own_shard, int64_t shard_bytes, void *send_buf,
                                 mw_group_desc *desc, mw_send_stats *stats, const void *const *shards, void *out,
                                 hipStream_t s)
{
    const int64_t shard_chunks = shard_bytes / 16;
    const int64_t gx = shard_chunks > 0 ? (shard_chunks + kFlat - 1) / kFlat : 1;
    if (gx > 0x7fffffffLL) return MW_ERR_UNSUPPORTED;
    {
        mw_timed tm(ctx, MW_KERNEL_AG_GATHER, s);
        hipLaunchKernelGGL(k_allgather_step, dim3((uint32_t)gx, ctx->cfg.n_ranks + 2), dim3(kFlat), 0, s,
                           (const u32x4 *const *)shards, shard_chunks, (u32x4 *)out, ctx->cfg.n_ranks,
                           (const u32x4 *)own_shard, (u32x4 *)send_buf, desc, stats);
    }
    MW_HIP_CHECK(hipGetLastError());
    return MW_OK;
}
