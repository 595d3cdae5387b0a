// Device code of the packer that more than one translation unit uses (k_pack, and the launch
// that carries a whole step of a stream of batches).
#ifndef MW_PACK_DEV_H_
#define MW_PACK_DEV_H_

#include "mw_internal.h"

namespace {

// Workgroup `seg` of a packed row's segments (blockDim.x chunks each), rows i_first, i_first +
// i_stride, ...  Chunks [0, xc) come from x, chunks [xc, xc + sc) from the fp8 scale rows
// (sc == 0 otherwise); packed row i starts ns chunks after row i - 1.  The row count and the row's token are wave-uniform and fetched
// together (perm has room for every row the grid can reach, so the read is in bounds even
// past the last kept row).
struct mw_pack_args {
    const u32x4 *x, *scales; int xc, sc, ns; const int32_t *topk; int K;     // ns: chunks from one packed row to the next
    const int32_t *perm; const mw_send_stats *stats;
    u32x4 *packed; int32_t *row_src_token, *row_topk;
};

__device__ __forceinline__ void mw_pack_body(const u32x4 *__restrict__ x, const u32x4 *__restrict__ scales,
                                             int xc, int sc, int ns, const int32_t *__restrict__ topk, int K,
                                             const int32_t *__restrict__ perm,
                                             const mw_send_stats *__restrict__ stats,
                                             u32x4 *__restrict__ packed, int32_t *__restrict__ row_src_token,
                                             int32_t *__restrict__ row_topk, uint32_t seg, uint32_t i_first,
                                             uint32_t i_stride)
{
    // the row's token and the row count are requested first, the remaining arguments beside them
    uint32_t i = i_first;
    int32_t t = perm[i];
    uint32_t n_rows = stats->n_rows;
    uint32_t gdim = i_stride, bdim = blockDim.x;
    MW_PIN_S(gdim); MW_PIN_S(bdim); MW_PIN_S(xc); MW_PIN_S(sc); MW_PIN_S(ns); MW_PIN_S(K);
    MW_PIN_PTR(x); MW_PIN_PTR(scales); MW_PIN_PTR(topk); MW_PIN_PTR(packed); MW_PIN_PTR(row_src_token);
    MW_PIN_PTR(row_topk);
    MW_PIN_S(t); MW_PIN_S(n_rows);
    const int n = xc + sc;
    const int c = seg * bdim + threadIdx.x;
    while (i < n_rows) {
        if (c < n) {
            const u32x4 v = (c < xc) ? mw_ld16(x + (size_t)t * xc + c) : mw_ld16(scales + (size_t)t * sc + (c - xc));
            mw_st16(packed + (size_t)i * ns + c, v);
        }
        if (seg == 0) {
            if (threadIdx.x == 0) row_src_token[i] = t;
            for (int j = threadIdx.x; j < K; j += bdim) row_topk[(size_t)i * K + j] = topk[(size_t)t * K + j];
        }
        i += gdim;
        if (i < n_rows) t = perm[i];
    }
}

}  // namespace

#endif
