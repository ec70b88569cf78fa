// Smoothed selection loss and center variable (Section 4.1, experimental
// setup: leaders are chosen from the training loss averaged over the last
// few minibatches; the model reported at test time is the average of all
// workers' parameters).
#include "common.h"

namespace lsgd {

typedef float v4f __attribute__((ext_vector_type(4)));

// One thread per worker: store the new loss into ring slot t % K, then average
// the filled slots in slot order with a double accumulator, so that the value
// leaders are chosen from does not depend on the launch shape.
__global__ __launch_bounds__(256) void smooth_losses_kernel(float* __restrict__ window, int K, int slot, int filled,
                                                            const float* losses, int W, float* out)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= W) return;
    const float cur = losses[i];
    window[(int64_t)slot * W + i] = cur;
    double s = 0.0;
    for (int q = 0; q < filled; ++q) s += (double)(q == slot ? cur : window[(int64_t)q * W + i]);
    out[i] = (float)(s / (double)filled);
}

// Column mean over the W rows.  A thread owns VEC adjacent columns and walks
// the rows in order, kRows loads in flight; the sum is carried in double (the
// adds hide behind the row reads), so the result is the correctly ordered sum
// rounded once.
constexpr int kCenterThreads = 256;
constexpr int kRows = 8;

template <int VEC>
__global__ __launch_bounds__(kCenterThreads) void center_kernel(const float* __restrict__ x, int W, int64_t col0, int64_t col1,
                                                                int64_t ld, float* __restrict__ out)
{
    const int64_t col = col0 + ((int64_t)blockIdx.x * kCenterThreads + threadIdx.x) * VEC;
    if (col >= col1) return;
    double s[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) s[v] = 0.0;
    const float* p = x + col;
    int i = 0;
    if (VEC == 4) {
        for (; i + kRows <= W; i += kRows) {
            v4f r[kRows];
#pragma unroll
            for (int u = 0; u < kRows; ++u)
                r[u] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p + (int64_t)(i + u) * ld));
#pragma unroll
            for (int u = 0; u < kRows; ++u) {
                s[0] += (double)r[u].x; s[1 % VEC] += (double)r[u].y; s[2 % VEC] += (double)r[u].z; s[3 % VEC] += (double)r[u].w;
            }
        }
        for (; i < W; ++i) {
            const v4f r = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p + (int64_t)i * ld));
            s[0] += (double)r.x; s[1 % VEC] += (double)r.y; s[2 % VEC] += (double)r.z; s[3 % VEC] += (double)r.w;
        }
        v4f o;
        o.x = (float)(s[0] / (double)W); o.y = (float)(s[1 % VEC] / (double)W);
        o.z = (float)(s[2 % VEC] / (double)W); o.w = (float)(s[3 % VEC] / (double)W);
        *reinterpret_cast<v4f*>(out + col) = o;
    } else {
        for (; i < W; ++i) s[0] += (double)p[(int64_t)i * ld];
        out[col] = (float)(s[0] / (double)W);
    }
}

// Elastic-averaging center (the comparison method of the paper, supplement "Low-Rank Matrix Completion
// Experiments"): center <- (1 - a) center + a * mean_i x[i], a = W*eta*lambda, with the mean taken in
// double in row order as above; the center as it was goes to old_center (the workers' step pulls to it).
// In place on center: a thread reads its columns of center before it writes them.
template <int VEC>
__global__ __launch_bounds__(kCenterThreads) void easgd_center_kernel(const float* __restrict__ x, int W, int64_t col0, int64_t col1,
                                                                      int64_t ld, float* __restrict__ center,
                                                                      float* __restrict__ old_center, double a)
{
#pragma clang fp contract(off)      // (1-a)*c + a*mean as two products and a sum, rounded like the plain expression
    const int64_t col = col0 + ((int64_t)blockIdx.x * kCenterThreads + threadIdx.x) * VEC;
    if (col >= col1) return;
    double s[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) s[v] = 0.0;
    const float* p = x + col;
    int i = 0;
    if (VEC == 4) {
        const v4f c = *reinterpret_cast<const v4f*>(center + col);
        for (; i + kRows <= W; i += kRows) {
            v4f r[kRows];
#pragma unroll
            for (int u = 0; u < kRows; ++u) r[u] = *reinterpret_cast<const v4f*>(p + (int64_t)(i + u) * ld);
#pragma unroll
            for (int u = 0; u < kRows; ++u) {
                s[0] += (double)r[u].x; s[1 % VEC] += (double)r[u].y; s[2 % VEC] += (double)r[u].z; s[3 % VEC] += (double)r[u].w;
            }
        }
        for (; i < W; ++i) {
            const v4f r = *reinterpret_cast<const v4f*>(p + (int64_t)i * ld);
            s[0] += (double)r.x; s[1 % VEC] += (double)r.y; s[2 % VEC] += (double)r.z; s[3 % VEC] += (double)r.w;
        }
        v4f o;
        o.x = (float)((1.0 - a) * (double)c.x + a * (s[0] / (double)W));
        o.y = (float)((1.0 - a) * (double)c.y + a * (s[1 % VEC] / (double)W));
        o.z = (float)((1.0 - a) * (double)c.z + a * (s[2 % VEC] / (double)W));
        o.w = (float)((1.0 - a) * (double)c.w + a * (s[3 % VEC] / (double)W));
        *reinterpret_cast<v4f*>(old_center + col) = c;
        *reinterpret_cast<v4f*>(center + col) = o;
    } else {
        const float c = center[col];
        for (; i < W; ++i) s[0] += (double)p[(int64_t)i * ld];
        old_center[col] = c;
        center[col] = (float)((1.0 - a) * (double)c + a * (s[0] / (double)W));
    }
}

hipError_t launch_easgd_center(const float* x, int W, int64_t P, int64_t ld, float* center, float* old_center, double a, hipStream_t s)
{
    auto aligned16 = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
    const bool vec_ok = (ld % 4 == 0) && aligned16(x) && aligned16(center) && aligned16(old_center);
    const int64_t P4 = vec_ok ? (P & ~(int64_t)3) : 0;
    if (P4 > 0) {
        const int64_t blocks = (P4 / 4 + kCenterThreads - 1) / kCenterThreads;
        hipLaunchKernelGGL((easgd_center_kernel<4>), dim3((unsigned)blocks), dim3(kCenterThreads), 0, s, x, W, (int64_t)0, P4, ld, center,
                           old_center, a);
    }
    if (P > P4) {
        const int64_t blocks = (P - P4 + kCenterThreads - 1) / kCenterThreads;
        hipLaunchKernelGGL((easgd_center_kernel<1>), dim3((unsigned)blocks), dim3(kCenterThreads), 0, s, x, W, P4, P, ld, center,
                           old_center, a);
    }
    return hipGetLastError();
}

hipError_t launch_smooth_losses(float* window, int K, int64_t t, const float* losses, int W, float* out, hipStream_t s)
{
    const int slot = (int)(t % K);
    const int filled = (int)(t + 1 < (int64_t)K ? t + 1 : (int64_t)K);
    hipLaunchKernelGGL(smooth_losses_kernel, dim3((unsigned)((W + 255) / 256)), dim3(256), 0, s, window, K, slot, filled, losses,
                       W, out);
    return hipGetLastError();
}

hipError_t launch_center(const float* x, int W, int64_t P, int64_t ld, float* out, hipStream_t s)
{
    auto aligned16 = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
    const bool vec_ok = (ld % 4 == 0) && aligned16(x) && aligned16(out);
    const int64_t P4 = vec_ok ? (P & ~(int64_t)3) : 0;
    if (P4 > 0) {
        const int64_t blocks = (P4 / 4 + kCenterThreads - 1) / kCenterThreads;
        hipLaunchKernelGGL((center_kernel<4>), dim3((unsigned)blocks), dim3(kCenterThreads), 0, s, x, W, (int64_t)0, P4, ld, out);
    }
    if (P > P4) {
        const int64_t blocks = (P - P4 + kCenterThreads - 1) / kCenterThreads;
        hipLaunchKernelGGL((center_kernel<1>), dim3((unsigned)blocks), dim3(kCenterThreads), 0, s, x, W, P4, P, ld, out);
    }
    return hipGetLastError();
}

} // namespace lsgd
