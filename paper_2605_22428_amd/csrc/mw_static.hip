// mw_plan_static: the send-side plan for callers that cannot allocate device memory -- code
// under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  mw_plan keeps
// its counters, its plan state and the expert table in a workspace the caller allocated; here
// the same three live in one file-scope device array, so the call needs no context and no
// workspace.  The kernels are mw_plan's own (mw_launch_plan): they get the array's device
// address the way they get the workspace's.
//
// The array's name is a host-side stand-in for the symbol, not a device address: the address
// is looked up once per device (hipGetSymbolAddress, with that device current) and only the
// looked-up pointer is ever handed to a kernel.  Every GPU the library runs on holds its own
// copy of the array until the process ends.
#include <mutex>

#include "mw_internal.h"

namespace {

constexpr int64_t kCntBytes = 8LL * MW_STATIC_MAX_TOKENS;            // packed per-token counters
constexpr int64_t kStateBytes = (4LL * MW_PLAN_STATE_WORDS + 255) / 256 * 256;
constexpr int64_t kSlotBytes = 4LL * MW_STATIC_MAX_EXPERTS;          // (rank << 16) | slot per expert
constexpr int64_t kScratchBytes = kCntBytes + kStateBytes + kSlotBytes;   // 70912 bytes

static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
struct device_slot { unsigned char *ptr; int n_cu; };
device_slot g_slot[kMaxDevices];          // ptr == nullptr: not looked up yet
std::mutex g_slot_lock;

// The device address of `scratch` on the current device (looked up on the first call there).
int32_t scratch_of_current_device(device_slot *out, int *device)
{
    int dev = -1;
    MW_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return MW_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> hold(g_slot_lock);
    if (!g_slot[dev].ptr) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MW_ERR_HIP;
        hipDeviceProp_t prop;
        MW_HIP_CHECK(hipGetDeviceProperties(&prop, dev));
        g_slot[dev].n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
        g_slot[dev].ptr = (unsigned char *)p;
    }
    *out = g_slot[dev];
    *device = dev;
    return MW_OK;
}

// One workgroup.  The array keeps what the last call left in it: the counters of the tokens
// this plan uses and the plan state are cleared, and the expert table is rebuilt from the
// caller's rank table (slot of expert e = experts of the same rank with a smaller id).  An
// entry outside [0, R) names no rank: its expert is ignored and the plan reports
// MW_FLAG_BAD_EXPERT.
constexpr int kPrepBlock = 1024;
constexpr int kStateFlagsWord = 257;      // the plan state's flag word (256 histogram bins, kept tokens, flags, ...)
__global__ __launch_bounds__(kPrepBlock) void k_static_prepare(const int32_t *__restrict__ e2r, int E, int R, int T,
                                                               unsigned long long *__restrict__ cnt,
                                                               uint32_t *__restrict__ pstate,
                                                               int32_t *__restrict__ eslot)
{
    __shared__ int32_t rank_of[MW_STATIC_MAX_EXPERTS];
    const int tid = threadIdx.x;
    for (int e = tid; e < E; e += kPrepBlock) rank_of[e] = e2r[e];
    for (int t = tid; t < T; t += kPrepBlock) cnt[t] = 0;
    for (int w = tid; w < MW_PLAN_STATE_WORDS; w += kPrepBlock) pstate[w] = 0;
    __syncthreads();
    bool bad = false;
    for (int e = tid; e < E; e += kPrepBlock) {
        const int32_t r = rank_of[e];
        int32_t v = -1;
        if (r >= 0 && r < R) {
            int slot = 0;
            for (int q = 0; q < e; ++q) slot += rank_of[q] == r ? 1 : 0;
            v = (r << 16) | slot;
        } else {
            bad = true;
        }
        eslot[e] = v;
    }
    if (bad) atomicOr(&pstate[kStateFlagsWord], MW_FLAG_BAD_EXPERT);
}

}  // namespace

extern "C" MW_API int32_t mw_plan_static(const mw_config *cfg, const int32_t *expert_to_rank_dev,
                                         const int32_t *topk_ids_dev, int32_t n_tokens, uint64_t *mask_dev,
                                         int32_t *perm_dev, mw_group_desc *desc_dev, mw_send_stats *stats_dev,
                                         void *stream)
{
    if (!cfg || !stats_dev || n_tokens < 0) return MW_ERR_INVALID_ARG;
    if (cfg->n_ranks < 1 || cfg->n_experts < 1 || cfg->top_k < 1) return MW_ERR_INVALID_ARG;
    if (cfg->n_ranks > MW_MAX_RANKS || cfg->top_k > MW_MAX_TOPK) return MW_ERR_UNSUPPORTED;
    if (cfg->n_experts > MW_STATIC_MAX_EXPERTS || n_tokens > MW_STATIC_MAX_TOKENS) return MW_ERR_CAPACITY;
    if (!expert_to_rank_dev) return MW_ERR_INVALID_ARG;
    if (n_tokens > 0 && (!topk_ids_dev || !mask_dev || !perm_dev || !desc_dev)) return MW_ERR_INVALID_ARG;
    int64_t xb = 0, sb = 0;
    const int32_t rc = mw_row_geometry(*cfg, &xb, &sb);
    if (rc != MW_OK) return rc;
    device_slot slot;
    int dev = -1;
    const int32_t rs = scratch_of_current_device(&slot, &dev);
    if (rs != MW_OK) return rs;

    // a context on the stack whose plan slices are the device's array (nothing else is used by the plan)
    mw_ctx tmp = {};
    tmp.cfg = *cfg;
    tmp.cfg.expert_to_rank = nullptr;
    tmp.cfg.max_tokens = MW_STATIC_MAX_TOKENS;
    tmp.mask_words = (cfg->n_ranks + 63) / 64;
    tmp.x_row_bytes = xb; tmp.s_row_bytes = sb; tmp.row_bytes = xb + sb;
    tmp.row_stride = xb + sb;
    tmp.device = dev;
    tmp.n_cu = slot.n_cu;
    tmp.d_plan_cnt = (uint64_t *)slot.ptr;
    tmp.d_plan_state = (uint32_t *)(slot.ptr + kCntBytes);
    tmp.d_eslot = (int32_t *)(slot.ptr + kCntBytes + kStateBytes);

    const hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(k_static_prepare, dim3(1), dim3(kPrepBlock), 0, s, expert_to_rank_dev, cfg->n_experts,
                       cfg->n_ranks, n_tokens, (unsigned long long *)tmp.d_plan_cnt, tmp.d_plan_state, tmp.d_eslot);
    MW_HIP_CHECK(hipGetLastError());
    return mw_launch_plan(&tmp, topk_ids_dev, n_tokens, mask_dev, perm_dev, desc_dev, stats_dev, s);
}
