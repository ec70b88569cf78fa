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

// (a, b, M) of observed entry s, from the 16-byte records when the caller supplied them
__device__ __forceinline__ void fetch_entry(const lsgd_mc_entry* __restrict__ entries, const int32_t* __restrict__ rows,
                                            const int32_t* __restrict__ cols, const float* __restrict__ vals, int64_t s,
                                            int& a, int& b, float& v)
{
    if (entries) {
        const int4 e = reinterpret_cast<const int4*>(entries)[s];
        a = e.x; b = e.y; v = __int_as_float(e.z);
    } else {
        a = rows[s]; b = cols[s]; v = vals[s];
    }
}

// General path: S lanes cooperate on one entry (S = power of two >= min(r, 64)),
// residual by a lane butterfly, gradient rows accumulated with hardware fp32
// atomics into the zero-filled g.  Any r, m, n.
template <int S>
__global__ __launch_bounds__(kMcThreads) void mc_grad_atomic_kernel(
    const float* __restrict__ x, float* __restrict__ g, int64_t ld, int m, int n, int r,
    const int32_t* __restrict__ rows, const int32_t* __restrict__ cols, const float* __restrict__ vals,
    const int32_t* __restrict__ batch_idx, int64_t nb, float two_c, float* __restrict__ partials, int nblk,
    const lsgd_mc_entry* __restrict__ entries)
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
        int a, b;
        float mv;
        fetch_entry(entries, rows, cols, vals, s, a, b, mv);
        const float* ua = U + (int64_t)a * r;
        const float* vb = V + (int64_t)b * r;
        float dot = 0.f;
        for (int q = q0; q < r; q += S) dot = fmaf(ua[q], vb[q], dot);
#pragma unroll
        for (int d = 1; d < S; d <<= 1) dot += __shfl_xor(dot, d, S);
        const float e = dot - mv;
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

// ------------------------------------------------------------------------------------------
// Binned path (r % 4 == 0, 16-byte aligned rows): no global floating-point atomics.
// Factor rows are grouped in bins of 64 consecutive rows (U bins, then V bins).
//   1. residual kernel (1024 entries per workgroup): fetches each entry's (a, b, M), computes
//      e_k with a lane group per entry, and ranks the entries of the workgroup inside their U bin
//      and V bin with LDS counters; writes the workgroup's bin histogram.
//   2. scan kernel: per worker, bin totals -> bin starts, and the start of every workgroup's
//      share inside each bin.
//   3. scatter kernel: entry -> record (row inside the bin, other factor's row, e_k) at
//      bin start + workgroup share + rank, once for the U side and once for the V side.
//   4. reduce kernel: one workgroup per (worker, bin) sorts the bin's records by row in LDS, then
//      each lane group sums e_k * other_row over the records of its rows in registers and writes
//      the gradient row once, scaled by 2c; rows without entries come out as zeros, so there is
//      no separate zero fill.
// Workgroups of one worker are numbered so that they land on one die (workgroup id modulo 8),
// which keeps the worker's factors, 5 MB at rank 32, in that die's L2.  This placement only
// affects speed, never results.
// ------------------------------------------------------------------------------------------
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kBinRows = 64;          // factor rows per bin
constexpr int kResEntries = 1024;     // entries per workgroup in the residual kernel
constexpr int kMaxBins = 8192;        // LDS histogram capacity (U bins + V bins)
constexpr int kXcd = 8;

struct McBinned {
    int32_t* hist;   // [W][nblk][nbins] per-workgroup bin counts, then the bin's records before this workgroup
    int32_t* bstart; // [W][nbins+1] bin starts
    int32_t* ea;     // [W][nb] a_k
    int32_t* eb;     // [W][nb] b_k
    float* ee;       // [W][nb] e_k
    uint32_t* rk;    // [W][nb] rank in U bin (low 16 bits) | rank in V bin (high 16 bits), within the workgroup
    int2* rec;       // [W][2*nb] (row-in-bin << 26 | other row, e bits): U bins then V bins
    int nbinsU, nbins, nblk;
};

// maps a linear workgroup id to (worker, chunk) with all chunks of a worker on the same die
__device__ __forceinline__ bool xcd_map(int64_t id, int W, int nchunk, int& w, int& chunk)
{
    const int xcd = (int)(id % kXcd);
    const int64_t t = id / kXcd;
    w = (int)(t / nchunk) * kXcd + xcd;
    chunk = (int)(t % nchunk);
    return w < W;
}

template <int LPE>
__global__ __launch_bounds__(kResEntries) void mc_residual_kernel(
    const float* __restrict__ x, int64_t ld, int m, int n, int r, const int32_t* __restrict__ rows,
    const int32_t* __restrict__ cols, const float* __restrict__ vals, const int32_t* __restrict__ batch_idx,
    int64_t nb, McBinned S, float* __restrict__ partials, int W, const lsgd_mc_entry* __restrict__ entries)
{
    int w, blk;
    if (!xcd_map(blockIdx.x, W, S.nblk, w, blk)) return;
    const float* U = x + (int64_t)w * ld;
    const float* V = U + (int64_t)m * r;
    extern __shared__ int lhist[];                 // [nbins]
    __shared__ int sa[kResEntries], sb[kResEntries];
    __shared__ float sv[kResEntries];
    __shared__ float red[kResEntries / 64];
    const int t = threadIdx.x;
    const int64_t k0 = (int64_t)blk * kResEntries;
    const int cnt_here = (int)((nb - k0 < kResEntries) ? nb - k0 : kResEntries);
    for (int i = t; i < S.nbins; i += kResEntries) lhist[i] = 0;
    // phase 1: thread t fetches entry t's (a, b, M): all index chasing of the workgroup is in flight at once
    if (t < cnt_here) {
        const int64_t s = batch_idx ? (int64_t)batch_idx[(int64_t)w * nb + k0 + t] : k0 + t;
        int a, b;
        float mv;
        fetch_entry(entries, rows, cols, vals, s, a, b, mv);
        sa[t] = a; sb[t] = b; sv[t] = mv;
    }
    __syncthreads();
    // phase 2: LPE lanes per entry, two entries per lane group in flight; sv[] becomes e_k
    const int sub = t / LPE, q0 = t % LPE;
    constexpr int kSubs = kResEntries / LPE;
    const int r4 = r >> 2;
    for (int e0 = sub; e0 < cnt_here; e0 += 2 * kSubs) {
        const int e1 = e0 + kSubs;
        const bool two = e1 < cnt_here;
        const v4f* ua0 = reinterpret_cast<const v4f*>(U + (int64_t)sa[e0] * r);
        const v4f* vb0 = reinterpret_cast<const v4f*>(V + (int64_t)sb[e0] * r);
        const v4f* ua1 = reinterpret_cast<const v4f*>(U + (int64_t)sa[two ? e1 : e0] * r);
        const v4f* vb1 = reinterpret_cast<const v4f*>(V + (int64_t)sb[two ? e1 : e0] * r);
        float d0 = 0.f, d1 = 0.f;
        for (int q = q0; q < r4; q += LPE) {
            const v4f u0 = ua0[q], v0 = vb0[q], u1 = ua1[q], v1 = vb1[q];
            d0 += u0.x * v0.x + u0.y * v0.y + u0.z * v0.z + u0.w * v0.w;
            d1 += u1.x * v1.x + u1.y * v1.y + u1.z * v1.z + u1.w * v1.w;
        }
#pragma unroll
        for (int d = 1; d < LPE; d <<= 1) { d0 += __shfl_xor(d0, d, LPE); d1 += __shfl_xor(d1, d, LPE); }
        if (q0 == 0) {
            sv[e0] = d0 - sv[e0];
            if (two) sv[e1] = d1 - sv[e1];
        }
    }
    __syncthreads();
    // phase 3: thread t records entry t (coalesced stores) and takes its ranks from the LDS counters
    float sq = 0.f;
    if (t < cnt_here) {
        const float e = sv[t];
        sq = e * e;
        const int a = sa[t], b = sb[t];
        const int64_t o = (int64_t)w * nb + k0 + t;
        const uint32_t ru = (uint32_t)atomicAdd(&lhist[a / kBinRows], 1);
        const uint32_t rv = (uint32_t)atomicAdd(&lhist[S.nbinsU + b / kBinRows], 1);
        S.ea[o] = a; S.eb[o] = b; S.ee[o] = e;
        S.rk[o] = ru | (rv << 16);
    }
    // squared-error partial of the workgroup, in a fixed order
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) sq += __shfl_xor(sq, d, 64);
    if ((t & 63) == 0) red[t >> 6] = sq;
    __syncthreads();
    if (t == 0) {
        float tot = 0.f;
        for (int i = 0; i < kResEntries / 64; ++i) tot += red[i];
        partials[(int64_t)w * S.nblk + blk] = tot;
    }
    int32_t* gh = S.hist + ((int64_t)w * S.nblk + blk) * S.nbins;
    for (int i = t; i < S.nbins; i += kResEntries) gh[i] = lhist[i];
}

// One workgroup per worker.  Thread per bin: walks the bin's column of the histogram matrix once
// (coalesced across bins, sixteen loads in flight), replacing each workgroup's count by the number of
// the bin's records that precede it; then an exclusive scan of the bin totals gives the bin starts.
__global__ __launch_bounds__(1024) void mc_scan_kernel(McBinned S)
{
    const int w = blockIdx.x, t = threadIdx.x, lane = t & 63, wv = t >> 6;
    int32_t* hist = S.hist + (int64_t)w * S.nblk * S.nbins;
    int32_t* bstart = S.bstart + (int64_t)w * (S.nbins + 1);
    __shared__ int wsum[16];
    __shared__ int carry_s;
    if (t == 0) carry_s = 0;
    __syncthreads();
    for (int base = 0; base < S.nbins; base += 1024) {
        const int bin = base + t;
        int total = 0;
        if (bin < S.nbins) {
            for (int b0 = 0; b0 < S.nblk; b0 += 16) {
                int c[16];
#pragma unroll
                for (int q = 0; q < 16; ++q) c[q] = (b0 + q < S.nblk) ? hist[(int64_t)(b0 + q) * S.nbins + bin] : 0;
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    if (b0 + q < S.nblk) hist[(int64_t)(b0 + q) * S.nbins + bin] = total;
                    total += c[q];
                }
            }
        }
        int inc = total;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) { const int v = __shfl_up(inc, d, 64); if (lane >= d) inc += v; }
        if (lane == 63) wsum[wv] = inc;
        __syncthreads();
        int before = carry_s;
        for (int q = 0; q < wv; ++q) before += wsum[q];
        if (bin < S.nbins) bstart[bin] = before + inc - total;
        __syncthreads();
        if (t == 1023) carry_s = before + inc;
        __syncthreads();
    }
    if (t == 0) bstart[S.nbins] = carry_s;
}

__global__ __launch_bounds__(256) void mc_scatter_kernel(McBinned S, int64_t nb)
{
    const int w = blockIdx.y;
    const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k >= nb) return;
    const int blk = (int)(k / kResEntries);
    const int32_t* share = S.hist + ((int64_t)w * S.nblk + blk) * S.nbins;
    const int64_t o = (int64_t)w * nb + k;
    const int a = S.ea[o], b = S.eb[o];
    const int eb = __float_as_int(S.ee[o]);
    const uint32_t rk = S.rk[o];
    int2* rec = S.rec + (int64_t)w * 2 * nb;
    const int32_t* bstart = S.bstart + (int64_t)w * (S.nbins + 1);
    const int bu = a / kBinRows, bv = S.nbinsU + b / kBinRows;
    rec[bstart[bu] + share[bu] + (int)(rk & 0xFFFFu)] = make_int2(((a % kBinRows) << 26) | b, eb);
    rec[bstart[bv] + share[bv] + (int)(rk >> 16)] = make_int2(((b % kBinRows) << 26) | a, eb);
}

// One workgroup per (worker, bin).  The bin's records are staged in LDS and counting-sorted by their
// row inside the bin (64 integer LDS counters), so that each lane group owns whole rows: it walks the
// row's records, four gathers of the other factor's rows in flight, accumulates in registers and writes
// the gradient row once (scaled by 2c).  Rows without records are written as zeros.
constexpr int kRedCap = 2048;                     // records staged per pass

template <int LPE>
__global__ __launch_bounds__(kMcThreads) void mc_reduce_kernel(const float* __restrict__ x, float* __restrict__ g, int64_t ld,
                                                               int m, int n, int r, McBinned S, int64_t nb, float two_c, int W)
{
    constexpr int kSubs = kMcThreads / LPE;                          // lane groups per workgroup
    constexpr int RPG = (kBinRows + kSubs - 1) / kSubs;              // rows per lane group
    constexpr int PER = kRedCap / kMcThreads;                        // records per thread and pass
    int w, bin;
    if (!xcd_map(blockIdx.x, W, S.nbins, w, bin)) return;
    __shared__ int2 sorted[kRedCap];
    __shared__ int cnt[kBinRows], start[kBinRows + 1];
    const int t = threadIdx.x;
    const bool uside = bin < S.nbinsU;
    const int row0 = (uside ? bin : bin - S.nbinsU) * kBinRows;       // first factor row of the bin
    const int nrows = uside ? m : n;
    const float* xw = x + (int64_t)w * ld;
    const float* other = uside ? xw + (int64_t)m * r : xw;             // U rows gather V rows and vice versa
    const int2* rec = S.rec + (int64_t)w * 2 * nb;
    const int32_t* bstart = S.bstart + (int64_t)w * (S.nbins + 1);
    const int j0 = bstart[bin], j1 = bstart[bin + 1];
    const int sub = t / LPE, q0 = t % LPE;
    const bool lane_live = q0 < (r >> 2);
    v4f acc[RPG];
#pragma unroll
    for (int i = 0; i < RPG; ++i) acc[i] = (v4f)(0.f);

    for (int c0 = j0; c0 < j1; c0 += kRedCap) {
        const int nrec = (j1 - c0 < kRedCap) ? j1 - c0 : kRedCap;
        if (t < kBinRows) cnt[t] = 0;
        __syncthreads();
        int2 mine[PER];
        int rank[PER];
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int i = t + u * kMcThreads;
            if (i < nrec) {
                mine[u] = rec[c0 + i];
                rank[u] = atomicAdd(&cnt[(uint32_t)mine[u].x >> 26], 1);
            }
        }
        __syncthreads();
        if (t < 64) {                                                 // exclusive scan of the 64 row counts
            const int c = cnt[t];
            int inc = c;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) { const int v = __shfl_up(inc, d, 64); if (t >= d) inc += v; }
            start[t] = inc - c;
            if (t == 63) start[64] = inc;
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int i = t + u * kMcThreads;
            if (i < nrec) sorted[start[(uint32_t)mine[u].x >> 26] + rank[u]] = mine[u];
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < RPG; ++i) {
            const int row = sub + i * kSubs;
            if (row < kBinRows && lane_live) {
                const int s0 = start[row], s1 = start[row + 1];
                for (int sidx = s0; sidx < s1; sidx += 4) {
                    int2 rc[4];
                    v4f ov[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) rc[u] = sorted[(sidx + u < s1) ? sidx + u : sidx];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        ov[u] = reinterpret_cast<const v4f*>(other + (int64_t)(rc[u].x & 0x3FFFFFF) * r)[q0];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (sidx + u < s1) acc[i] += __int_as_float(rc[u].y) * ov[u];
                }
            }
        }
        __syncthreads();
    }
    float* out = g + (int64_t)w * ld + (uside ? (int64_t)0 : (int64_t)m * r) + (int64_t)row0 * r;
#pragma unroll
    for (int i = 0; i < RPG; ++i) {
        const int row = sub + i * kSubs;
        if (row < kBinRows && row0 + row < nrows && lane_live)
            reinterpret_cast<v4f*>(out + (int64_t)row * r)[q0] = two_c * acc[i];
    }
}

__global__ __launch_bounds__(256) void mc_zero_pad_kernel(float* __restrict__ g, int64_t P, int64_t ld)
{
    const int64_t c = P + (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (c < ld) g[(int64_t)blockIdx.y * ld + c] = 0.f;
}

__global__ __launch_bounds__(256) void mc_pack_kernel(const int32_t* __restrict__ rows, const int32_t* __restrict__ cols,
                                                      const float* __restrict__ vals, int64_t n, lsgd_mc_entry* __restrict__ out)
{
    for (int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x; k < n; k += (int64_t)gridDim.x * 256) {
        int4 e = make_int4(rows[k], cols[k], __float_as_int(vals[k]), 0);
        reinterpret_cast<int4*>(out)[k] = e;
    }
}

hipError_t launch_mc_pack(const int32_t* rows, const int32_t* cols, const float* vals, int64_t n, lsgd_mc_entry* out, hipStream_t s)
{
    int64_t blocks = (n + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(mc_pack_kernel, dim3((unsigned)blocks), dim3(256), 0, s, rows, cols, vals, n, out);
    return hipGetLastError();
}

static int64_t mc_entries(const lsgd_mc_batch& b) { return b.batch_idx ? b.B : b.n_obs; }

static size_t up256(size_t v) { return (v + 255) / 256 * 256; }

static int mc_bins_u(const lsgd_mc_batch& b) { return (b.m + kBinRows - 1) / kBinRows; }
static int mc_bins(const lsgd_mc_batch& b) { return mc_bins_u(b) + (b.n + kBinRows - 1) / kBinRows; }
static int mc_res_blocks(const lsgd_mc_batch& b) { return (int)((mc_entries(b) + kResEntries - 1) / kResEntries); }

static bool mc_binned_ok(const lsgd_mc_batch& b)
{
    const int64_t nb = mc_entries(b);
    return b.r % 4 == 0 && nb > 0 && nb < ((int64_t)1 << 30) && mc_bins(b) <= kMaxBins && b.m < (1 << 26) && b.n < (1 << 26) &&
           (size_t)kBinRows * b.r * 4 <= 64 * 1024 && (int64_t)mc_res_blocks(b) * mc_bins(b) <= ((int64_t)1 << 22);
}

size_t mc_partials(int W, const lsgd_mc_batch& b)
{
    const int64_t nblk = (mc_entries(b) + kMcEntriesPerBlock - 1) / kMcEntriesPerBlock;
    return (size_t)W * (size_t)(nblk > 0 ? nblk : 1);
}

size_t mc_scratch_bytes(int W, const lsgd_mc_batch& b)
{
    if (!mc_binned_ok(b)) return 0;
    const size_t nb = (size_t)mc_entries(b);
    return up256((size_t)W * mc_res_blocks(b) * mc_bins(b) * 4) + up256((size_t)W * (mc_bins(b) + 1) * 4) +
           4 * up256((size_t)W * nb * 4) + up256((size_t)W * 2 * nb * 8);
}

template <int LPE>
static void launch_binned(const float* x, float* g, int W, int64_t ld, const lsgd_mc_batch& b, int64_t nb,
                          const McBinned& S, float* partials, hipStream_t s)
{
    const int rounds = (W + kXcd - 1) / kXcd;
    hipLaunchKernelGGL((mc_residual_kernel<LPE>), dim3((unsigned)((int64_t)rounds * kXcd * S.nblk)), dim3(kResEntries),
                       (size_t)S.nbins * 4, s, x, ld, b.m, b.n, b.r, b.rows, b.cols, b.vals, b.batch_idx, nb, S, partials, W, b.entries);
    hipLaunchKernelGGL(mc_scan_kernel, dim3((unsigned)W), dim3(1024), 0, s, S);
    hipLaunchKernelGGL(mc_scatter_kernel, dim3((unsigned)((nb + 255) / 256), (unsigned)W), dim3(256), 0, s, S, nb);
    hipLaunchKernelGGL((mc_reduce_kernel<LPE>), dim3((unsigned)((int64_t)rounds * kXcd * S.nbins)), dim3(kMcThreads),
                       0, s, x, g, ld, b.m, b.n, b.r, S, nb, 2.0f * b.c, W);
}

hipError_t launch_mc_grad_loss(const float* x, float* g, float* losses, int W, int64_t P, int64_t ld,
                               const lsgd_mc_batch& b, const DeviceState& st, hipStream_t s)
{
    const int64_t nb = mc_entries(b);
    const bool aligned = (reinterpret_cast<uintptr_t>(x) & 15u) == 0 && (reinterpret_cast<uintptr_t>(g) & 15u) == 0 && ld % 4 == 0;
    const bool binned = mc_binned_ok(b) && aligned && st.scratch_bytes >= mc_scratch_bytes(W, b);
    if (binned) {
        McBinned S;
        S.nbinsU = mc_bins_u(b); S.nbins = mc_bins(b); S.nblk = mc_res_blocks(b);
        char* p = st.scratch;
        const size_t nbw = up256((size_t)W * (size_t)nb * 4);
        S.hist = reinterpret_cast<int32_t*>(p); p += up256((size_t)W * S.nblk * S.nbins * 4);
        S.bstart = reinterpret_cast<int32_t*>(p); p += up256((size_t)W * (S.nbins + 1) * 4);
        S.ea = reinterpret_cast<int32_t*>(p); p += nbw;
        S.eb = reinterpret_cast<int32_t*>(p); p += nbw;
        S.ee = reinterpret_cast<float*>(p); p += nbw;
        S.rk = reinterpret_cast<uint32_t*>(p); p += nbw;
        S.rec = reinterpret_cast<int2*>(p);
        const int r4 = b.r / 4;
        if (r4 <= 1) launch_binned<1>(x, g, W, ld, b, nb, S, st.partials, s);
        else if (r4 <= 2) launch_binned<2>(x, g, W, ld, b, nb, S, st.partials, s);
        else if (r4 <= 4) launch_binned<4>(x, g, W, ld, b, nb, S, st.partials, s);
        else if (r4 <= 8) launch_binned<8>(x, g, W, ld, b, nb, S, st.partials, s);
        else if (r4 <= 16) launch_binned<16>(x, g, W, ld, b, nb, S, st.partials, s);
        else if (r4 <= 32) launch_binned<32>(x, g, W, ld, b, nb, S, st.partials, s);
        else launch_binned<64>(x, g, W, ld, b, nb, S, st.partials, s);
        if (ld > P)
            hipLaunchKernelGGL(mc_zero_pad_kernel, dim3((unsigned)((ld - P + 255) / 256), (unsigned)W), dim3(256), 0, s, g, P, ld);
        hipLaunchKernelGGL(mc_loss_finish_kernel, dim3((unsigned)W), dim3(256), 0, s, st.partials, S.nblk, b.c, losses);
        return hipGetLastError();
    }
    const int nblk = (int)((nb + kMcEntriesPerBlock - 1) / kMcEntriesPerBlock);
    // general path: zero the whole rows (padding included), then atomics
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
                       b.rows, b.cols, b.vals, b.batch_idx, nb, two_c, st.partials, nblk, b.entries)
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
