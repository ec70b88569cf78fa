// Per-worker gradient and loss of low-rank matrix completion on a batch of
// observed entries (the problem family of the motivating example and of the
// supplement's "Low-Rank Matrix Completion Experiments" in arXiv 1905.10395,
// in rectangular, partially observed form).
//
//   e_k = <U[a_k], V[b_k]> - M_k ;  loss = c * sum_k e_k^2
//   dU[a] = 2c * sum_{k: a_k = a} e_k V[b_k] ;  dV[b] = 2c * sum_{k: b_k = b} e_k U[a_k]
//
// Worker row of x and of g: [U (m x r) | V (n x r)], row-major factors.
#include "common.h"

namespace lsgd {

constexpr int kMcThreads = 256;
constexpr int kMcEntriesPerBlock = 256;

__global__ __launch_bounds__(256) void fill_zero_kernel(float* __restrict__ g, int64_t ld)
{
    float* row = g + (int64_t)blockIdx.y * ld;
    const int64_t n4 = ld >> 2;
    float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; c < n4; c += (int64_t)gridDim.x * blockDim.x)
        reinterpret_cast<float4*>(row)[c] = z;
    if (blockIdx.x == 0 && threadIdx.x < (ld & 3)) row[(n4 << 2) + threadIdx.x] = 0.f;
}
__global__ __launch_bounds__(256) void fill_zero_scalar_kernel(float* __restrict__ g, int64_t ld)
{
    float* row = g + (int64_t)blockIdx.y * ld;
    for (int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; c < ld; c += (int64_t)gridDim.x * blockDim.x)
        row[c] = 0.f;
}

// General path: S lanes cooperate on one entry (S = power of two >= min(r, 64)),
// residual by a lane butterfly, gradient rows accumulated with hardware fp32
// atomics into the zero-filled g.  Any r, m, n.
template <int S>
__global__ __launch_bounds__(kMcThreads) void mc_grad_atomic_kernel(
    const float* __restrict__ x, float* __restrict__ g, int64_t ld, int m, int n, int r,
    const int32_t* __restrict__ rows, const int32_t* __restrict__ cols, const float* __restrict__ vals,
    const int32_t* __restrict__ batch_idx, int64_t nb, float two_c, float* __restrict__ partials, int nblk)
{
    const int w = blockIdx.y;
    const float* U = x + (int64_t)w * ld;
    const float* V = U + (int64_t)m * r;
    float* gU = g + (int64_t)w * ld;
    float* gV = gU + (int64_t)m * r;
    const int sub = threadIdx.x / S, q0 = threadIdx.x % S;
    constexpr int kSubs = kMcThreads / S;
    const int64_t k0 = (int64_t)blockIdx.x * kMcEntriesPerBlock;
    const int64_t k1 = (k0 + kMcEntriesPerBlock < nb) ? k0 + kMcEntriesPerBlock : nb;
    float sq = 0.f;
    for (int64_t k = k0 + sub; k < k1; k += kSubs) {
        const int64_t s = batch_idx ? (int64_t)batch_idx[(int64_t)w * nb + k] : k;
        const int a = rows[s], b = cols[s];
        const float* ua = U + (int64_t)a * r;
        const float* vb = V + (int64_t)b * r;
        float dot = 0.f;
        for (int q = q0; q < r; q += S) dot = fmaf(ua[q], vb[q], dot);
#pragma unroll
        for (int d = 1; d < S; d <<= 1) dot += __shfl_xor(dot, d, S);
        const float e = dot - vals[s];
        if (q0 == 0) sq = fmaf(e, e, sq);
        const float f = two_c * e;
        for (int q = q0; q < r; q += S) {
            unsafeAtomicAdd(gU + (int64_t)a * r + q, f * vb[q]);
            unsafeAtomicAdd(gV + (int64_t)b * r + q, f * ua[q]);
        }
    }
    // block sum of squared residuals in a fixed order
    __shared__ float red[kMcThreads];
    red[threadIdx.x] = sq;
    __syncthreads();
    for (int d = kMcThreads / 2; d > 0; d >>= 1) {
        if (threadIdx.x < d) red[threadIdx.x] += red[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) partials[(int64_t)w * nblk + blockIdx.x] = red[0];
}

// losses[w] = c * sum of the worker's partial sums, accumulated in fp64 in a fixed order.
__global__ __launch_bounds__(256) void mc_loss_finish_kernel(const float* __restrict__ partials, int nblk, float c,
                                                             float* __restrict__ losses)
{
    const int w = blockIdx.x;
    double acc = 0.0;
    for (int i = threadIdx.x; i < nblk; i += 256) acc += (double)partials[(int64_t)w * nblk + i];
    __shared__ double red[256];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int d = 128; d > 0; d >>= 1) {
        if (threadIdx.x < d) red[threadIdx.x] += red[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) losses[w] = (float)((double)c * red[0]);
}

static int64_t mc_entries(const lsgd_mc_batch& b) { return b.batch_idx ? b.B : b.n_obs; }

size_t mc_partials(int W, const lsgd_mc_batch& b)
{
    const int64_t nblk = (mc_entries(b) + kMcEntriesPerBlock - 1) / kMcEntriesPerBlock;
    return (size_t)W * (size_t)(nblk > 0 ? nblk : 1);
}

size_t mc_scratch_bytes(int W, const lsgd_mc_batch& b)
{
    (void)W; (void)b;
    return 0;
}

hipError_t launch_mc_grad_loss(const float* x, float* g, float* losses, int W, int64_t P, int64_t ld,
                               const lsgd_mc_batch& b, const DeviceState& st, hipStream_t s)
{
    (void)P;
    const int64_t nb = mc_entries(b);
    const int nblk = (int)((nb + kMcEntriesPerBlock - 1) / kMcEntriesPerBlock);
    // zero the whole rows (padding included)
    {
        const bool v4 = (reinterpret_cast<uintptr_t>(g) & 15u) == 0 && (ld % 4 == 0);
        int64_t blocks = ((v4 ? ld / 4 : ld) + 255) / 256;
        if (blocks > 2048) blocks = 2048;
        if (blocks < 1) blocks = 1;
        if (v4) hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks, (unsigned)W), dim3(256), 0, s, g, ld);
        else hipLaunchKernelGGL(fill_zero_scalar_kernel, dim3((unsigned)blocks, (unsigned)W), dim3(256), 0, s, g, ld);
    }
    if (nblk > 0) {
        dim3 grid((unsigned)nblk, (unsigned)W);
        const float two_c = 2.0f * b.c;
#define LSGD_MC_LAUNCH(S)                                                                                     \
    hipLaunchKernelGGL((mc_grad_atomic_kernel<S>), grid, dim3(kMcThreads), 0, s, x, g, ld, b.m, b.n, b.r,     \
                       b.rows, b.cols, b.vals, b.batch_idx, nb, two_c, st.partials, nblk)
        if (b.r <= 1) LSGD_MC_LAUNCH(1);
        else if (b.r <= 2) LSGD_MC_LAUNCH(2);
        else if (b.r <= 4) LSGD_MC_LAUNCH(4);
        else if (b.r <= 8) LSGD_MC_LAUNCH(8);
        else if (b.r <= 16) LSGD_MC_LAUNCH(16);
        else if (b.r <= 32) LSGD_MC_LAUNCH(32);
        else LSGD_MC_LAUNCH(64);
#undef LSGD_MC_LAUNCH
    }
    hipLaunchKernelGGL(mc_loss_finish_kernel, dim3((unsigned)W), dim3(256), 0, s, st.partials, nblk, b.c, losses);
    return hipGetLastError();
}

} // namespace lsgd
