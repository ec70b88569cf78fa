// lsgd_stream_probe: plain streams of known size, for measuring what the memory system of the
// GPU at hand gives the access shapes the update kernels use.  Not part of the method: the
// benchmark reports these rates beside the update's own, as measured ceilings.
#include "common.h"

using namespace lsgd;

namespace {

typedef float v2f __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
constexpr int kThreads = 256;

// 256-thread workgroups, workgroup b on block b of the arrays in memory order.  Lane width per kind as it
// streams fastest on this chip: 16-byte lanes for the read-only and copy streams, 8-byte lanes (2 KB of each
// stream per workgroup) for the 3-read/2-write update.
template <int KIND, class V>
__global__ __launch_bounds__(kThreads) void stream_probe_kernel(V* __restrict__ a, V* __restrict__ b, V* __restrict__ c, int64_t nv,
                                                                float mu, float eta)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= nv) return;
    if (KIND == LSGD_PROBE_READ) {
        const V v = __builtin_nontemporal_load(a + i);
        if (v.x == 1.2345678e-30f && v.y == 8.7654321e-30f) b[i] = v;        // keeps the load; practically never taken
    } else if (KIND == LSGD_PROBE_COPY) {
        __builtin_nontemporal_store(__builtin_nontemporal_load(a + i), b + i);
    } else {
        V x = __builtin_nontemporal_load(a + i);
        const V g = __builtin_nontemporal_load(b + i);
        V m = __builtin_nontemporal_load(c + i);
        m = mu * m + g;
        x = x - eta * m;
        __builtin_nontemporal_store(x, a + i);
        __builtin_nontemporal_store(m, c + i);
    }
}

template <int KIND, class V>
hipError_t launch_probe(float* a, float* b, float* c, int64_t n, hipStream_t s)
{
    const int64_t nv = n / (int64_t)(sizeof(V) / sizeof(float));
    const int64_t blocks = (nv + kThreads - 1) / kThreads;
    hipLaunchKernelGGL((stream_probe_kernel<KIND, V>), dim3((unsigned)blocks), dim3(kThreads), 0, s, reinterpret_cast<V*>(a),
                       reinterpret_cast<V*>(b), reinterpret_cast<V*>(c), nv, 0.9f, 1e-3f);
    return hipGetLastError();
}

} // namespace

extern "C" lsgd_status lsgd_stream_probe(int32_t kind, float* a, float* b, float* c, int64_t n, void* hip_stream)
{
    if (kind != LSGD_PROBE_READ && kind != LSGD_PROBE_COPY && kind != LSGD_PROBE_UPDATE)
        return set_error(LSGD_ERR_INVALID_ARG, "stream_probe: unknown kind %d", (int)kind);
    if (!a || !b || (kind == LSGD_PROBE_UPDATE && !c)) return set_error(LSGD_ERR_INVALID_ARG, "stream_probe: NULL buffer");
    if (n <= 0 || n % 2) return set_error(LSGD_ERR_SHAPE, "stream_probe: n = %lld must be positive and even", (long long)n);
    if ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b) | reinterpret_cast<uintptr_t>(c)) & 7u)
        return set_error(LSGD_ERR_INVALID_ARG, "stream_probe: buffers must be 8-byte aligned");
    if (n / 2 / kThreads > 0x7fffffff) return set_error(LSGD_ERR_SHAPE, "stream_probe: n too large for one launch");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const bool wide = n % 4 == 0 && !((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b)) & 15u);
    hipError_t e;
    if (kind == LSGD_PROBE_READ)
        e = wide ? launch_probe<LSGD_PROBE_READ, v4f>(a, b, c, n, s) : launch_probe<LSGD_PROBE_READ, v2f>(a, b, c, n, s);
    else if (kind == LSGD_PROBE_COPY)
        e = wide ? launch_probe<LSGD_PROBE_COPY, v4f>(a, b, c, n, s) : launch_probe<LSGD_PROBE_COPY, v2f>(a, b, c, n, s);
    else
        e = launch_probe<LSGD_PROBE_UPDATE, v2f>(a, b, c, n, s);
    if (e != hipSuccess) return set_error(LSGD_ERR_HIP, "stream_probe: %s", hipGetErrorString(e));
    return LSGD_OK;
}
