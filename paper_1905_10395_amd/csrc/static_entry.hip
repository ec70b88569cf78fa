// lsgd_select_pull_static: leader selection + pull update for callers that cannot allocate device
// memory.  The bookkeeping the population handle normally keeps in the caller's workspace (group
// table, leader indices, re-selection flags) lives in a file-scope device array instead, so the
// call needs no handle, no workspace and no allocation of any kind.
#include <cmath>
#include <mutex>

#include "common.h"

using namespace lsgd;

namespace {

// int32 words: offsets[G+1] | group_of[W] | lead[G] | glead[1] | refreshed[G+1] | plan[W] (8 words each)
constexpr int kOffOffsets = 0;
constexpr int kOffGroupOf = kOffOffsets + LSGD_STATIC_MAX_GROUPS + 1;
constexpr int kOffLead = kOffGroupOf + LSGD_STATIC_MAX_WORKERS;
constexpr int kOffGlead = kOffLead + LSGD_STATIC_MAX_GROUPS;
constexpr int kOffRefreshed = kOffGlead + 1;
constexpr int kOffPlan = (kOffRefreshed + LSGD_STATIC_MAX_GROUPS + 1 + 7) / 8 * 8;         // 32-byte aligned records
constexpr int kScratchWords = kOffPlan + LSGD_STATIC_MAX_WORKERS * (int)(sizeof(RowPlan) / sizeof(int32_t));

// One copy per GPU the library is loaded on, held until the process ends.
static __device__ __align__(256) int32_t scratch[(kScratchWords + 63) / 64 * 64];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
int32_t* g_scratch_ptr[kMaxDevices] = {};

// Device address of this GPU's copy of the array (looked up once per device, with that device current).
lsgd_status scratch_for_current_device(int32_t** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return set_error(LSGD_ERR_HIP, "select_pull_static: hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return set_error(LSGD_ERR_UNSUPPORTED, "select_pull_static: device index %d outside [0,%d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return set_error(LSGD_ERR_HIP, "select_pull_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = static_cast<int32_t*>(p);
    }
    *out = g_scratch_ptr[dev];
    return LSGD_OK;
}

struct GroupTable {
    int32_t off[LSGD_STATIC_MAX_GROUPS + 1];
};

// Writes the group table of this call into the scratch array (it arrives by value as a kernel
// argument, so no host-to-device copy is involved).
__global__ __launch_bounds__(256) void static_setup_kernel(GroupTable t, int W, int G, int32_t* offsets, int32_t* group_of)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i <= G) offsets[i] = t.off[i];
    if (i < W) {
        int j = 0;
        while (j + 1 < G && t.off[j + 1] <= i) ++j;
        group_of[i] = j;
    }
}

} // namespace

extern "C" lsgd_status lsgd_select_pull_static(int32_t W, int64_t P, int64_t ld, int32_t n_groups, const int32_t* group_offsets,
                                               float* x, const float* g, float* m, const float* losses, int32_t* leaders,
                                               float eta, float lambda_L, float lambda_G, float momentum, float weight_decay,
                                               int32_t flags, void* hip_stream)
{
    if (W <= 0 || W > LSGD_STATIC_MAX_WORKERS)
        return set_error(LSGD_ERR_SHAPE, "select_pull_static: W=%d outside [1,%d] (the static scratch holds at most %d workers)", W,
                         LSGD_STATIC_MAX_WORKERS, LSGD_STATIC_MAX_WORKERS);
    if (n_groups <= 0 || n_groups > LSGD_STATIC_MAX_GROUPS || n_groups > W)
        return set_error(LSGD_ERR_SHAPE, "select_pull_static: n_groups=%d outside [1,min(W,%d)] (the static scratch holds at most %d groups)",
                         n_groups, LSGD_STATIC_MAX_GROUPS, LSGD_STATIC_MAX_GROUPS);
    if (P <= 0) return set_error(LSGD_ERR_SHAPE, "select_pull_static: P=%lld must be positive", (long long)P);
    if (ld < P) return set_error(LSGD_ERR_SHAPE, "select_pull_static: ld=%lld < P=%lld", (long long)ld, (long long)P);
    if (!x || !g || !losses) return set_error(LSGD_ERR_INVALID_ARG, "select_pull_static: x, g and losses are required");
    if (!std::isfinite(momentum) || momentum < 0.0f) return set_error(LSGD_ERR_INVALID_ARG, "select_pull_static: momentum must be finite and >= 0");
    if (momentum != 0.0f && !m) return set_error(LSGD_ERR_INVALID_ARG, "select_pull_static: momentum != 0 needs the m buffer");
    if (!std::isfinite(eta) || !std::isfinite(lambda_L) || !std::isfinite(lambda_G) || !std::isfinite(weight_decay))
        return set_error(LSGD_ERR_INVALID_ARG, "select_pull_static: eta, lambda_L, lambda_G, weight_decay must be finite");
    const int known = LSGD_NESTEROV | LSGD_LEADER_EXEMPT | LSGD_PULL_UNSCALED_BY_ETA | LSGD_MOMENTUM_GRAD_ONLY;
    if (flags & ~known) return set_error(LSGD_ERR_INVALID_ARG, "select_pull_static: flag bits 0x%x are not available here", flags & ~known);
    if ((flags & LSGD_PULL_UNSCALED_BY_ETA) && (lambda_L != 0.0f || lambda_G != 0.0f) && eta == 0.0f)
        return set_error(LSGD_ERR_INVALID_ARG, "select_pull_static: unscaled pulls need eta != 0");
    GroupTable tab;
    if (group_offsets) {
        for (int j = 0; j <= n_groups; ++j) tab.off[j] = group_offsets[j];
        if (tab.off[0] != 0 || tab.off[n_groups] != W) return set_error(LSGD_ERR_SHAPE, "select_pull_static: group_offsets must start at 0 and end at W");
        for (int j = 0; j < n_groups; ++j)
            if (tab.off[j + 1] <= tab.off[j]) return set_error(LSGD_ERR_SHAPE, "select_pull_static: group %d is empty or offsets decrease", j);
    } else {
        if (W % n_groups) return set_error(LSGD_ERR_SHAPE, "select_pull_static: W=%d not divisible by n_groups=%d and no group_offsets", W, n_groups);
        for (int j = 0; j <= n_groups; ++j) tab.off[j] = j * (W / n_groups);
    }
    for (int j = n_groups + 1; j <= LSGD_STATIC_MAX_GROUPS; ++j) tab.off[j] = W;
    int group_size = tab.off[1] - tab.off[0];
    for (int j = 0; j < n_groups; ++j)
        if (tab.off[j + 1] - tab.off[j] != tab.off[1] - tab.off[0]) group_size = 0;

    int32_t* base = nullptr;
    lsgd_status st = scratch_for_current_device(&base);
    if (st != LSGD_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);

    DeviceState ds{};
    ds.offsets = base + kOffOffsets;
    ds.group_of = base + kOffGroupOf;
    ds.lead = leaders ? leaders : base + kOffLead;
    ds.glead = leaders ? leaders + n_groups : base + kOffGlead;
    ds.refreshed = base + kOffRefreshed;
    ds.plan = reinterpret_cast<RowPlan*>(base + kOffPlan);

    // every word of the scratch that this call reads is written by this call first: the group table
    // here, the leaders and the re-selection flags by the selection kernel
    const int setup_threads = W > n_groups + 1 ? W : n_groups + 1;
    hipLaunchKernelGGL(static_setup_kernel, dim3((unsigned)((setup_threads + 255) / 256)), dim3(256), 0, s, tab, (int)W, (int)n_groups,
                       ds.offsets, ds.group_of);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return set_error(LSGD_ERR_HIP, "select_pull_static: setup: %s", hipGetErrorString(e));

    RefreshBits all;
    for (size_t k = 0; k < sizeof(all.w) / sizeof(all.w[0]); ++k) all.w[k] = 0;
    for (int j = 0; j < n_groups; ++j) all.w[j >> 6] |= 1ull << (j & 63);
    e = launch_select_leaders(losses, W, n_groups, ds, all, all, 1, 1, s);
    if (e != hipSuccess) return set_error(LSGD_ERR_HIP, "select_pull_static: select_leaders: %s", hipGetErrorString(e));

    PullParams q{};
    q.x = x; q.g = g; q.m = momentum != 0.0f ? m : nullptr; q.Z = nullptr; q.xb = nullptr;
    q.P = P; q.ld = ld; q.W = W; q.G = n_groups;
    q.eta = eta; q.mu = momentum; q.wd = weight_decay;
    q.lamL = lambda_L; q.lamG = lambda_G;
    if (flags & LSGD_PULL_UNSCALED_BY_ETA) {
        if (lambda_L != 0.0f) q.lamL = lambda_L / eta;
        if (lambda_G != 0.0f) q.lamG = lambda_G / eta;
    }
    q.flags = flags;
    q.use_refreshed = 1;
    q.clear_refreshed = 0;
    q.group_size = group_size;
    q.comm_pull = 0;
    e = launch_pull_update(q, ds, s);
    if (e != hipSuccess) return set_error(LSGD_ERR_HIP, "select_pull_static: pull_update: %s", hipGetErrorString(e));
    return LSGD_OK;
}
