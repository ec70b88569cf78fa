// Leader selection: segmented argmin of the workers' losses (Eq. 1 / Eq. 2 of
// arXiv 1905.10395; the steps of Algorithm 1 that pick the best worker of each
// group and of all groups).  Ties resolve to the lowest worker index and NaN
// counts as +infinity.
//
// A loss and its worker index are packed into one 64-bit key whose unsigned
// order is (loss ascending, index ascending), so a plain integer minimum is
// the argmin with the required tie-break.
#include "common.h"

namespace lsgd {

__device__ __forceinline__ uint64_t loss_key(float v, int idx)
{
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) u = 0x7F800000u; // NaN -> +inf
    if (u == 0x80000000u) u = 0u;                         // -0 ties with +0
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);       // monotone map to unsigned
    return ((uint64_t)u << 32) | (uint32_t)idx;
}

__device__ __forceinline__ uint64_t shfl_up_u64(uint64_t v, int d)
{
    uint32_t lo = __shfl_up((uint32_t)v, d, kWave);
    uint32_t hi = __shfl_up((uint32_t)(v >> 32), d, kWave);
    return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ uint64_t shfl_xor_u64(uint64_t v, int d)
{
    uint32_t lo = __shfl_xor((uint32_t)v, d, kWave);
    uint32_t hi = __shfl_xor((uint32_t)(v >> 32), d, kWave);
    return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ uint64_t wave_min_u64(uint64_t k)
{
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        uint64_t o = shfl_xor_u64(k, d);
        k = o < k ? o : k;
    }
    return k;
}

constexpr int kSelThreads = 256;

__device__ __forceinline__ void write_plan_rows(int tid, int nthreads, int W, int G, const int32_t* group_of, const int32_t* lead,
                                                const int32_t* glead, const int32_t* refreshed, RowPlan* plan)
{
    for (int i = tid; i < W; i += nthreads) {
        const int j = group_of[i];
        RowPlan r;
        r.ll = lead[j]; r.gl = glead[0]; r.freshL = refreshed[j]; r.freshG = refreshed[G]; r.j = j;
        r.pad[0] = r.pad[1] = r.pad[2] = 0;
        plan[i] = r;
    }
}

__global__ __launch_bounds__(kSelThreads) void select_leaders_kernel(
    const float* __restrict__ losses, int W, int G, const int32_t* __restrict__ offsets,
    const int32_t* __restrict__ group_of, RefreshBits bits, RefreshBits capture, int refresh_global,
    int capture_global, int32_t* lead, int32_t* glead, int32_t* refreshed, RowPlan* __restrict__ plan)
{
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const uint64_t kNone = ~0ull;

    // every leader's "re-selected since the last update" flag is rewritten on each call
    for (int j = tid; j <= G; j += kSelThreads) {
        int r = (j < G) ? (int)((capture.w[j >> 6] >> (j & 63)) & 1ull) : (capture_global != 0);
        refreshed[j] = r;
    }

    if (W <= kWave) {
        // One wavefront holds the whole population: segmented inclusive min-scan
        // over lanes (a lane only accepts keys from lanes of its own group), so
        // the last lane of every segment ends with the segment's minimum.
        if (wave == 0) {
            uint64_t key = kNone;
            int gid = -1;
            if (lane < W) {
                key = loss_key(losses[lane], lane);
                gid = group_of[lane];
            }
            uint64_t seg = key;
#pragma unroll
            for (int d = 1; d < kWave; d <<= 1) {
                uint64_t ok = shfl_up_u64(seg, d);
                int og = __shfl_up(gid, d, kWave);
                if (lane >= d && og == gid && ok < seg) seg = ok;
            }
            if (lane < W) {
                bool last = (lane == W - 1) || (group_of[lane + 1] != gid);
                if (last && ((bits.w[gid >> 6] >> (gid & 63)) & 1ull)) lead[gid] = (int32_t)(uint32_t)seg;
            }
            if (refresh_global) {
                uint64_t all = wave_min_u64(key);
                if (lane == 0) glead[0] = (int32_t)(uint32_t)all;
            }
        }
    } else {
        // General case: one wavefront per group (groups strided over the waves of
        // the block), lanes stride over the group's rows, butterfly minimum.
        constexpr int kWaves = kSelThreads / kWave;
        for (int j = wave; j < G; j += kWaves) {
            if (!((bits.w[j >> 6] >> (j & 63)) & 1ull)) continue;
            uint64_t key = kNone;
            for (int i = offsets[j] + lane; i < offsets[j + 1]; i += kWave) {
                uint64_t k = loss_key(losses[i], i);
                key = k < key ? k : key;
            }
            key = wave_min_u64(key);
            if (lane == 0) lead[j] = (int32_t)(uint32_t)key;
        }
        if (refresh_global) {
            __shared__ uint64_t part[kWaves];
            uint64_t key = kNone;
            for (int i = tid; i < W; i += kSelThreads) {
                uint64_t k = loss_key(losses[i], i);
                key = k < key ? k : key;
            }
            key = wave_min_u64(key);
            if (lane == 0) part[wave] = key;
            __syncthreads();
            if (tid == 0) {
                uint64_t k = part[0];
                for (int w = 1; w < kWaves; ++w) k = part[w] < k ? part[w] : k;
                glead[0] = (int32_t)(uint32_t)k;
            }
        }
    }
    // every row's view of the result, for the update kernel (the block's own global writes above are
    // visible to all its threads after the barrier)
    __threadfence_block();
    __syncthreads();
    write_plan_rows(tid, kSelThreads, W, G, group_of, lead, glead, refreshed, plan);
}

__global__ void init_state_kernel(int32_t* lead, int32_t* glead, int32_t* refreshed, int G)
{
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < G) lead[t] = -1;
    if (t <= G) refreshed[t] = 0;
    if (t == 0) glead[0] = -1;
}

__global__ void init_refreshed_kernel(int32_t* refreshed, int G)
{
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t <= G) refreshed[t] = 0;
}

hipError_t launch_init_refreshed(const DeviceState& st, int G, hipStream_t s)
{
    hipLaunchKernelGGL(init_refreshed_kernel, dim3((unsigned)((G + 1 + 255) / 256)), dim3(256), 0, s, st.refreshed, G);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void write_plan_kernel(int W, int G, const int32_t* group_of, const int32_t* lead, const int32_t* glead,
                                                         const int32_t* refreshed, RowPlan* plan)
{
    write_plan_rows(blockIdx.x * blockDim.x + threadIdx.x, gridDim.x * blockDim.x, W, G, group_of, lead, glead, refreshed, plan);
}

hipError_t launch_init_state(const DeviceState& st, int W, int G, hipStream_t s)
{
    int threads = 256;
    int blocks = (G + 1 + threads - 1) / threads;
    hipLaunchKernelGGL(init_state_kernel, dim3(blocks), dim3(threads), 0, s, st.lead, st.glead, st.refreshed, G);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_write_plan(st, W, G, s);
}

hipError_t launch_write_plan(const DeviceState& st, int W, int G, hipStream_t s)
{
    hipLaunchKernelGGL(write_plan_kernel, dim3((unsigned)((W + 255) / 256)), dim3(256), 0, s, W, G, st.group_of, st.lead, st.glead,
                       st.refreshed, st.plan);
    return hipGetLastError();
}

hipError_t launch_select_leaders(const float* losses, int W, int G, const DeviceState& st,
                                 const RefreshBits& bits, const RefreshBits& capture, int refresh_global,
                                 int capture_global, hipStream_t s)
{
    hipLaunchKernelGGL(select_leaders_kernel, dim3(1), dim3(kSelThreads), 0, s, losses, W, G, st.offsets,
                       st.group_of, bits, capture, refresh_global, capture_global, st.lead, st.glead,
                       st.refreshed, st.plan);
    return hipGetLastError();
}

} // namespace lsgd
