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
// atomics into the zero-filled g.  Any r, m, n.  GRAD = false evaluates the
// squared residuals only (g may be NULL).
template <int S, bool GRAD>
__global__ __launch_bounds__(kMcThreads) void mc_grad_atomic_kernel(
    const float* __restrict__ x, float* __restrict__ g, int64_t ld, int m, int n, int r,
    const int32_t* __restrict__ rows, const int32_t* __restrict__ cols, const float* __restrict__ vals,
    const int32_t* __restrict__ batch_idx, int64_t nb, float two_c, float* __restrict__ partials, int nblk,
    const lsgd_mc_entry* __restrict__ entries)
{
    const int w = blockIdx.y;
    const float* U = x + (int64_t)w * ld;
    const float* V = U + (int64_t)m * r;
    float* gU = GRAD ? g + (int64_t)w * ld : nullptr;
    float* gV = GRAD ? gU + (int64_t)m * r : nullptr;
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
        if (GRAD) {
            const float f = two_c * e;
            for (int q = q0; q < r; q += S) {
                unsafeAtomicAdd(gU + (int64_t)a * r + q, f * vb[q]);
                unsafeAtomicAdd(gV + (int64_t)b * r + q, f * ua[q]);
            }
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

// Objective only, rank a multiple of 4 and 16-byte aligned rows: LPE lanes share an entry with one float4
// of each factor row per lane, and four entries per lane group are in flight (index, record and both rows
// of each are fetched before the first product), since nothing but gathers happens here.
template <int LPE>
__global__ __launch_bounds__(kMcThreads) void mc_loss_vec_kernel(
    const float* __restrict__ x, int64_t ld, int m, int n, int r,
    const int32_t* __restrict__ rows, const int32_t* __restrict__ cols, const float* __restrict__ vals,
    const int32_t* __restrict__ batch_idx, int64_t nb, float* __restrict__ partials, int nblk,
    const lsgd_mc_entry* __restrict__ entries)
{
    constexpr int kSubs = kMcThreads / LPE, kFly = 4;
    const int w = blockIdx.y;
    const float* U = x + (int64_t)w * ld;
    const float* V = U + (int64_t)m * r;
    const int sub = threadIdx.x / LPE, q0 = threadIdx.x % LPE;
    const bool lane_on = q0 < (r >> 2);
    const int64_t k0 = (int64_t)blockIdx.x * kMcEntriesPerBlock;
    const int64_t k1 = (k0 + kMcEntriesPerBlock < nb) ? k0 + kMcEntriesPerBlock : nb;
    float sq = 0.f;
    for (int64_t kb = k0; kb < k1; kb += kSubs * kFly) {
        float4 ua[kFly], vb[kFly];
        float mv[kFly];
        bool live[kFly];
#pragma unroll
        for (int u = 0; u < kFly; ++u) {
            const int64_t k = kb + (int64_t)u * kSubs + sub;
            live[u] = k < k1;
            const int64_t kc = live[u] ? k : k1 - 1;           // a lane group past the end repeats the last entry
            const int64_t s = batch_idx ? (int64_t)batch_idx[(int64_t)w * nb + kc] : kc;
            int a, b;
            fetch_entry(entries, rows, cols, vals, s, a, b, mv[u]);
            ua[u] = vb[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (lane_on) {
                ua[u] = reinterpret_cast<const float4*>(U + (int64_t)a * r)[q0];
                vb[u] = reinterpret_cast<const float4*>(V + (int64_t)b * r)[q0];
            }
        }
#pragma unroll
        for (int u = 0; u < kFly; ++u) {
            float dot = ua[u].x * vb[u].x;
            dot = fmaf(ua[u].y, vb[u].y, dot);
            dot = fmaf(ua[u].z, vb[u].z, dot);
            dot = fmaf(ua[u].w, vb[u].w, dot);
#pragma unroll
            for (int d = 1; d < LPE; d <<= 1) dot += __shfl_xor(dot, d, LPE);
            const float e = dot - mv[u];
            if (q0 == 0 && live[u]) sq = fmaf(e, e, sq);
        }
    }
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
// Binned path (r % 4 == 0, 16-byte aligned rows): no global floating-point atomics, and each
// factor row an entry touches is gathered once per side.
// Factor rows are grouped in bins of 128 consecutive rows (U bins, then V bins).
//   1. prepare kernel (1024 threads, E = 1024..4096 entries per workgroup): fetches each entry's
//      (a, b, M), ranks the workgroup's entries inside their U bin and V bin with LDS counters,
//      scans the counters, and writes every entry twice into the workgroup's own region of 2E
//      records: as (row of a inside its bin, b, M) grouped by U bin, and as (row of b inside its
//      bin, a, M) grouped by V bin, plus the table of where each bin starts in that region.  No
//      factor row is read here, and no pass over all workgroups is needed: a bin's records are
//      the union of one short segment per workgroup.
//   2. side kernel: one workgroup per (worker, bin), U and V bins alike, in one launch.  It
//      collects the bin's segments and sorts the records by row in LDS; a lane group takes its own
//      row from an LDS copy of the bin's rows, gathers the other factor's row for each record,
//      forms e = <U[a], V[b]> - M and adds e times the gathered row to its row's gradient.  Both
//      sides form e with the same lane partition and reduction tree, so they get the same bits.
//      U bins also sum e^2 (double per lane, fixed tree over the workgroup).
//   3. loss: c * the U bins' sums, added in bin order in double.
// Gradient rows are written once, scaled by 2c; rows without entries come out as zeros, so
// there is no separate zero fill.  The order of a row's records follows LDS rank order, so the
// last bits of a gradient row (fp32 sums) can differ between runs; the loss is summed in double,
// where a different order changes the rounded fp32 result only in freak cases.
// Workgroups of one worker are numbered so that they land on one die (workgroup id modulo 8),
// which keeps the worker's factors, 5 MB at rank 32, in that die's L2.  This placement only
// affects speed, never results.
// ------------------------------------------------------------------------------------------
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kBinRows = 128;         // factor rows per bin (64, 128 or 256)
constexpr int kKeyShift = (kBinRows == 64) ? 26 : (kBinRows == 128) ? 25 : 24;   // record key: row in bin above, other row below
constexpr int kKeyMask = (1 << kKeyShift) - 1;
constexpr int kPrepThreads = 1024;    // threads per workgroup in the prepare kernel
constexpr int kMaxBins = 8192;        // LDS histogram capacity (U bins + V bins)
constexpr int kXcd = 8;

struct McBinned {
    int32_t* segs;   // [W][nblk][nbins+1] first record of each bin inside the workgroup's region
                     // (U bins fill [0, count), V bins [count, 2 count); entry nbins = 2 count)
    int2* rec;       // [W][nblk][2E] (row-in-bin << kKeyShift | other factor's row, M bits)
    int nbinsU, nbins, nblk, E;
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

template <int EPT>
__global__ __launch_bounds__(kPrepThreads) void mc_prep_kernel(
    const int32_t* __restrict__ rows, const int32_t* __restrict__ cols, const float* __restrict__ vals,
    const int32_t* __restrict__ batch_idx, int64_t nb, McBinned S, const lsgd_mc_entry* __restrict__ entries)
{
    constexpr int E = EPT * kPrepThreads;
    const int w = blockIdx.y, blk = blockIdx.x, t = threadIdx.x, lane = t & 63, wv = t >> 6;
    extern __shared__ int lhist[];                 // [nbins + 1]
    __shared__ int wsum[kPrepThreads / 64];
    for (int i = t; i <= S.nbins; i += kPrepThreads) lhist[i] = 0;
    const int64_t k0 = (int64_t)blk * E;
    const int cnt_here = (int)((nb - k0 < E) ? nb - k0 : E);
    // every index chase of the workgroup is in flight at once
    int64_t src[EPT];
#pragma unroll
    for (int u = 0; u < EPT; ++u) {
        const int i = u * kPrepThreads + t;
        src[u] = (i < cnt_here) ? (batch_idx ? (int64_t)batch_idx[(int64_t)w * nb + k0 + i] : k0 + i) : 0;
    }
    int a[EPT], b[EPT];
    float mv[EPT];
#pragma unroll
    for (int u = 0; u < EPT; ++u) {
        a[u] = b[u] = 0; mv[u] = 0.f;
        if (u * kPrepThreads + t < cnt_here) fetch_entry(entries, rows, cols, vals, src[u], a[u], b[u], mv[u]);
    }
    __syncthreads();
    int ru[EPT], rv[EPT];
#pragma unroll
    for (int u = 0; u < EPT; ++u) {
        if (u * kPrepThreads + t < cnt_here) {
            ru[u] = atomicAdd(&lhist[a[u] / kBinRows], 1);
            rv[u] = atomicAdd(&lhist[S.nbinsU + b[u] / kBinRows], 1);
        }
    }
    __syncthreads();
    // exclusive scan of the counters in place: thread t owns `per` consecutive bins
    const int per = (S.nbins + kPrepThreads - 1) / kPrepThreads;     // <= kMaxBins / 1024
    int loc[kMaxBins / kPrepThreads];
    int tot = 0;
#pragma unroll
    for (int q = 0; q < kMaxBins / kPrepThreads; ++q) {
        const int i = t * per + q;
        loc[q] = (q < per && i < S.nbins) ? lhist[i] : 0;
        tot += loc[q];
    }
    int inc = tot;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) { const int v = __shfl_up(inc, d, 64); if (lane >= d) inc += v; }
    if (lane == 63) wsum[wv] = inc;
    __syncthreads();
    int run = inc - tot;
    for (int q = 0; q < wv; ++q) run += wsum[q];
#pragma unroll
    for (int q = 0; q < kMaxBins / kPrepThreads; ++q) {
        const int i = t * per + q;
        if (q < per && i < S.nbins) { lhist[i] = run; run += loc[q]; }
    }
    if (t == 0) lhist[S.nbins] = 2 * cnt_here;
    __syncthreads();
    int32_t* seg = S.segs + ((int64_t)w * S.nblk + blk) * (S.nbins + 1);
    for (int i = t; i <= S.nbins; i += kPrepThreads) seg[i] = lhist[i];
    // the records take their sorted places in LDS first, so that they leave as one contiguous run
    int2* stage = reinterpret_cast<int2*>(lhist + ((S.nbins + 2) & ~1));     // [2 E], 8-byte aligned behind the counters
#pragma unroll
    for (int u = 0; u < EPT; ++u) {
        if (u * kPrepThreads + t < cnt_here) {
            const int mb = __float_as_int(mv[u]);
            stage[lhist[a[u] / kBinRows] + ru[u]] = make_int2(((a[u] % kBinRows) << kKeyShift) | b[u], mb);
            stage[lhist[S.nbinsU + b[u] / kBinRows] + rv[u]] = make_int2(((b[u] % kBinRows) << kKeyShift) | a[u], mb);
        }
    }
    __syncthreads();
    int2* rec = S.rec + ((int64_t)w * S.nblk + blk) * (2 * E);
    for (int i = t; i < 2 * cnt_here; i += kPrepThreads) rec[i] = stage[i];
}

// Sum over the LPE adjacent lanes of a lane group, result in every lane of the group.  Steps inside a
// row of 16 lanes are data-parallel-primitive adds (swap neighbours, swap pairs, mirror 8, mirror 16:
// after the first two steps every lane of a quad holds the quad's sum, and a mirror maps each quad onto
// a different one); wider groups finish with lane shuffles.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v)
{
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
template <int LPE>
__device__ __forceinline__ float group_sum(float v)
{
    if (LPE >= 2) v = dpp_add<0xB1>(v);       // quad_perm [1,0,3,2]
    if (LPE >= 4) v = dpp_add<0x4E>(v);       // quad_perm [2,3,0,1]
    if (LPE >= 8) v = dpp_add<0x141>(v);      // row_half_mirror
    if (LPE >= 16) v = dpp_add<0x140>(v);     // row_mirror
    if (LPE >= 32) v += __shfl_xor(v, 16, 64);
    if (LPE >= 64) v += __shfl_xor(v, 32, 64);
    return v;
}

// One workgroup per (worker, bin).  The bin's records (one segment per prepare workgroup) are
// staged in LDS and counting-sorted by their row inside the bin (one integer LDS counter per row), so that
// each lane group owns whole rows: it walks the row's records, four gathers of the other factor's
// rows in flight, forms each record's residual against its own row, accumulates in registers and
// writes the gradient row once (scaled by 2c).  Rows without records are written as zeros.
constexpr int kSideThreads = 256;
constexpr int kRedCap = 1024;                     // records staged per pass
constexpr int kSegCap = kSideThreads;             // segments collected at a time

// EXACT: r == 4 * LPE, every lane of a group holds part of the row.
template <int LPE, bool EXACT>
__global__ __launch_bounds__(kSideThreads) void mc_side_kernel(const float* __restrict__ x, float* __restrict__ g, int64_t ld,
                                                             int m, int n, int r, McBinned S, float two_c,
                                                             float* __restrict__ partials, int W)
{
    constexpr int kSubs = kSideThreads / LPE;                          // lane groups per workgroup
    constexpr int RPG = (kBinRows + kSubs - 1) / kSubs;              // rows per lane group
    constexpr int PER = kRedCap / kSideThreads;                        // records per thread and pass
    int w, gbin;
    if (!xcd_map(blockIdx.x, W, S.nbins, w, gbin)) return;
    extern __shared__ v4f tile[];                                     // the bin's own rows [kBinRows][r]
    __shared__ int2 sorted[kRedCap];
    __shared__ int cnt[kBinRows], start[kBinRows + 1];
    __shared__ int segoff[kSegCap + 1], segbase[kSegCap], wtot[kSideThreads / 64];
    __shared__ double sqred[kSideThreads / 64];
    const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const bool uside = gbin < S.nbinsU;
    const int row0 = (uside ? gbin : gbin - S.nbinsU) * kBinRows;     // first factor row of the bin
    const int nrows = uside ? m : n;
    const float* xw = x + (int64_t)w * ld;
    const float* own = uside ? xw : xw + (int64_t)m * r;
    const float* other = uside ? xw + (int64_t)m * r : xw;            // U rows gather V rows and vice versa
    const int r4 = r >> 2;
    {
        const int live = (nrows - row0 < kBinRows ? nrows - row0 : kBinRows) * r4;
        const v4f* src = reinterpret_cast<const v4f*>(own + (int64_t)row0 * r);
        for (int i = t; i < live; i += kSideThreads) tile[i] = src[i];
    }
    const int2* rec = S.rec + (int64_t)w * S.nblk * (2 * S.E);
    const int32_t* segs = S.segs + (int64_t)w * S.nblk * (S.nbins + 1) + gbin;
    const int sub = t / LPE, q0 = t % LPE;
    const bool lane_live = EXACT || q0 < r4;
    const float* obase = other + q0 * 4;                              // this lane's four columns of a gathered row
    v4f acc[RPG];
#pragma unroll
    for (int i = 0; i < RPG; ++i) acc[i] = (v4f)(0.f);
    double sq = 0.0;

    for (int blk0 = 0; blk0 < S.nblk; blk0 += kSegCap) {
        const int nseg = (S.nblk - blk0 < kSegCap) ? S.nblk - blk0 : kSegCap;
        // these segments: thread t takes segment t, counts are scanned into segoff
        int c = 0;
        if (t < nseg) {
            const int blk = blk0 + t;
            const int32_t* sp = segs + (int64_t)blk * (S.nbins + 1);
            const int s0 = sp[0];
            c = sp[1] - s0;
            segbase[t] = blk * (2 * S.E) + s0;
        }
        int inc = c;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) { const int v = __shfl_up(inc, d, 64); if (lane >= d) inc += v; }
        if (lane == 63) wtot[wv] = inc;
        __syncthreads();
        int before = 0;
        for (int q = 0; q < wv; ++q) before += wtot[q];
        segoff[t + 1] = before + inc;
        if (t == 0) segoff[0] = 0;
        __syncthreads();
        const int total = segoff[kSideThreads];

        for (int c0 = 0; c0 < total; c0 += kRedCap) {
            const int nrec = (total - c0 < kRedCap) ? total - c0 : kRedCap;
            if (t < kBinRows) cnt[t] = 0;
            __syncthreads();
            int2 mine[PER];
            int rank[PER];
#pragma unroll
            for (int u = 0; u < PER; ++u) {
                const int i = t + u * kSideThreads;
                if (i < nrec) {
                    // segment holding record c0 + i: the s with segoff[s] <= c0 + i < segoff[s + 1]
                    const int key = c0 + i;
                    int lo = 0, hi = nseg;
                    while (hi - lo > 1) {
                        const int mid = (lo + hi) >> 1;
                        if (segoff[mid] <= key) lo = mid; else hi = mid;
                    }
                    mine[u] = rec[segbase[lo] + (key - segoff[lo])];
                    rank[u] = atomicAdd(&cnt[(uint32_t)mine[u].x >> kKeyShift], 1);
                }
            }
            __syncthreads();
            if (kBinRows > 64 || t < 64) {                            // exclusive scan of the row counts
                const int cc = (t < kBinRows) ? cnt[t] : 0;
                int in2 = cc;
#pragma unroll
                for (int d = 1; d < 64; d <<= 1) { const int v = __shfl_up(in2, d, 64); if (lane >= d) in2 += v; }
                if (kBinRows > 64) {
                    if (lane == 63) wtot[wv] = in2;
                    __syncthreads();
                    for (int q = 0; q < wv; ++q) in2 += wtot[q];
                }
                if (t < kBinRows) start[t] = in2 - cc;
                if (t == kBinRows - 1) start[kBinRows] = in2;
            }
            __syncthreads();
#pragma unroll
            for (int u = 0; u < PER; ++u) {
                const int i = t + u * kSideThreads;
                if (i < nrec) sorted[start[(uint32_t)mine[u].x >> kKeyShift] + rank[u]] = mine[u];
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < RPG; ++i) {
                const int row = sub + i * kSubs;
                if (row < kBinRows) {
                    const int s0 = start[row], s1 = start[row + 1];
                    if (s0 < s1) {
                        const v4f mine_row = lane_live ? tile[row * r4 + q0] : (v4f)(0.f);
                        float rowsq = 0.f;
                        for (int sidx = s0; sidx < s1; sidx += 4) {
                            // straight-line body: slots past the row's end repeat its last record with weight zero
                            int2 rc[4];
                            v4f ov[4];
#pragma unroll
                            for (int u = 0; u < 4; ++u) rc[u] = sorted[(sidx + u < s1) ? sidx + u : s1 - 1];
#pragma unroll
                            for (int u = 0; u < 4; ++u)
                                ov[u] = lane_live ? *reinterpret_cast<const v4f*>(obase + (uint64_t)(uint32_t)(rc[u].x & kKeyMask) * (uint32_t)r)
                                                  : (v4f)(0.f);
                            float d[4];
#pragma unroll
                            for (int u = 0; u < 4; ++u)
                                d[u] = group_sum<LPE>(mine_row.x * ov[u].x + mine_row.y * ov[u].y + mine_row.z * ov[u].z + mine_row.w * ov[u].w);
#pragma unroll
                            for (int u = 0; u < 4; ++u) {
                                const float e = (sidx + u < s1) ? d[u] - __int_as_float(rc[u].y) : 0.f;
                                acc[i] += e * ov[u];
                                rowsq = fmaf(e, e, rowsq);
                            }
                        }
                        if (q0 == 0) sq += (double)rowsq;
                    }
                }
            }
            __syncthreads();
        }
    }
    float* out = g + (int64_t)w * ld + (uside ? (int64_t)0 : (int64_t)m * r) + (int64_t)row0 * r;
#pragma unroll
    for (int i = 0; i < RPG; ++i) {
        const int row = sub + i * kSubs;
        if (row < kBinRows && row0 + row < nrows && lane_live)
            reinterpret_cast<v4f*>(out + (int64_t)row * r)[q0] = two_c * acc[i];
    }
    if (uside) {                                                      // sum of squared residuals of this U bin
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) sq += __shfl_xor(sq, d, 64);
        if (lane == 0) sqred[wv] = sq;
        __syncthreads();
        if (t == 0) {
            double tot = 0.0;
            for (int q = 0; q < kSideThreads / 64; ++q) tot += sqred[q];
            partials[(int64_t)w * S.nbinsU + gbin] = (float)tot;
        }
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
// entries per prepare workgroup: as many as keeps at least ~2 workgroups per compute unit busy,
// more when the segment table would otherwise outgrow its bound
static int mc_ept(int W, const lsgd_mc_batch& b)
{
    const int64_t nb = mc_entries(b);
    int ept = 4;
    while (ept > 1 && (int64_t)W * ((nb + (int64_t)ept * kPrepThreads - 1) / ((int64_t)ept * kPrepThreads)) < 512) ept >>= 1;
    while (ept < 4 && ((nb + (int64_t)ept * kPrepThreads - 1) / ((int64_t)ept * kPrepThreads)) * (mc_bins(b) + 1) > ((int64_t)1 << 22))
        ept <<= 1;
    return ept;
}
static int mc_prep_blocks(int W, const lsgd_mc_batch& b)
{
    const int64_t E = (int64_t)mc_ept(W, b) * kPrepThreads;
    return (int)((mc_entries(b) + E - 1) / E);
}
static bool mc_binned_ok(int W, const lsgd_mc_batch& b)
{
    const int64_t nb = mc_entries(b);
    if (!(b.r % 4 == 0 && nb > 0 && nb < ((int64_t)1 << 30) && mc_bins(b) <= kMaxBins && b.m < (1 << kKeyShift) && b.n < (1 << kKeyShift) &&
          (size_t)kBinRows * b.r * 4 <= 64 * 1024))
        return false;
    return (int64_t)mc_prep_blocks(W, b) * (mc_bins(b) + 1) <= ((int64_t)1 << 22);
}

size_t mc_partials(int W, const lsgd_mc_batch& b)
{
    int64_t nblk = (mc_entries(b) + kMcEntriesPerBlock - 1) / kMcEntriesPerBlock;   // general path: one per workgroup
    if (nblk < mc_bins_u(b)) nblk = mc_bins_u(b);                                  // binned path: one per U bin
    return (size_t)W * (size_t)(nblk > 0 ? nblk : 1);
}

size_t mc_scratch_bytes(int W, const lsgd_mc_batch& b)
{
    if (!mc_binned_ok(W, b)) return 0;
    const size_t slots = (size_t)mc_prep_blocks(W, b) * mc_ept(W, b) * kPrepThreads;
    return up256((size_t)W * mc_prep_blocks(W, b) * (mc_bins(b) + 1) * 4) + up256((size_t)W * 2 * slots * 8);
}

template <int LPE>
static void launch_binned(const float* x, float* g, int W, int64_t ld, const lsgd_mc_batch& b, int64_t nb,
                          const McBinned& S, float* partials, hipStream_t s)
{
    const int rounds = (W + kXcd - 1) / kXcd;
    const dim3 pgrid((unsigned)S.nblk, (unsigned)W);
    const size_t plds = (size_t)((S.nbins + 2) & ~1) * 4 + (size_t)2 * S.E * 8;     // counters, then the staged records
    static bool big_lds = false;
    if (!big_lds) {                                   // 4096 entries per workgroup stage 64 KB of records
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&mc_prep_kernel<4>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)((kMaxBins + 2) * 4 + 2 * 4 * kPrepThreads * 8));
        big_lds = true;
    }
    if (S.E == kPrepThreads)
        hipLaunchKernelGGL((mc_prep_kernel<1>), pgrid, dim3(kPrepThreads), plds, s, b.rows, b.cols, b.vals, b.batch_idx, nb, S, b.entries);
    else if (S.E == 2 * kPrepThreads)
        hipLaunchKernelGGL((mc_prep_kernel<2>), pgrid, dim3(kPrepThreads), plds, s, b.rows, b.cols, b.vals, b.batch_idx, nb, S, b.entries);
    else
        hipLaunchKernelGGL((mc_prep_kernel<4>), pgrid, dim3(kPrepThreads), plds, s, b.rows, b.cols, b.vals, b.batch_idx, nb, S, b.entries);
    if (b.r == 4 * LPE)
        hipLaunchKernelGGL((mc_side_kernel<LPE, true>), dim3((unsigned)((int64_t)rounds * kXcd * S.nbins)), dim3(kSideThreads),
                           (size_t)kBinRows * b.r * 4, s, x, g, ld, b.m, b.n, b.r, S, 2.0f * b.c, partials, W);
    else
        hipLaunchKernelGGL((mc_side_kernel<LPE, false>), dim3((unsigned)((int64_t)rounds * kXcd * S.nbins)), dim3(kSideThreads),
                           (size_t)kBinRows * b.r * 4, s, x, g, ld, b.m, b.n, b.r, S, 2.0f * b.c, partials, W);
}

hipError_t launch_mc_grad_loss(const float* x, float* g, float* losses, int W, int64_t P, int64_t ld,
                               const lsgd_mc_batch& b, const DeviceState& st, hipStream_t s)
{
    const int64_t nb = mc_entries(b);
    const bool aligned = (reinterpret_cast<uintptr_t>(x) & 15u) == 0 && (reinterpret_cast<uintptr_t>(g) & 15u) == 0 && ld % 4 == 0;
    const bool binned = mc_binned_ok(W, b) && aligned && st.scratch_bytes >= mc_scratch_bytes(W, b);
    if (binned) {
        McBinned S;
        S.nbinsU = mc_bins_u(b); S.nbins = mc_bins(b); S.nblk = mc_prep_blocks(W, b); S.E = mc_ept(W, b) * kPrepThreads;
        char* p = st.scratch;
        S.segs = reinterpret_cast<int32_t*>(p); p += up256((size_t)W * S.nblk * (S.nbins + 1) * 4);
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
        hipLaunchKernelGGL(mc_loss_finish_kernel, dim3((unsigned)W), dim3(256), 0, s, st.partials, S.nbinsU, b.c, losses);
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
#define LSGD_MC_LAUNCH(S)                                                                                       \
    hipLaunchKernelGGL((mc_grad_atomic_kernel<S, true>), grid, dim3(kMcThreads), 0, s, x, g, ld, b.m, b.n, b.r, \
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

// Objective values only: the residual pass of the general path without its atomics, one partial sum per
// block of entries, then the same fixed-order finish.
hipError_t launch_mc_loss(const float* x, float* losses, int W, int64_t ld, const lsgd_mc_batch& b, const DeviceState& st,
                          hipStream_t s)
{
    const int64_t nb = mc_entries(b);
    const int nblk = (int)((nb + kMcEntriesPerBlock - 1) / kMcEntriesPerBlock);
    const bool vec = b.r % 4 == 0 && b.r <= 256 && (reinterpret_cast<uintptr_t>(x) & 15u) == 0 && ld % 4 == 0;
    if (nblk > 0 && vec) {
        dim3 grid((unsigned)nblk, (unsigned)W);
#define LSGD_MC_LAUNCH(LPE)                                                                                      \
    hipLaunchKernelGGL((mc_loss_vec_kernel<LPE>), grid, dim3(kMcThreads), 0, s, x, ld, b.m, b.n, b.r, b.rows,   \
                       b.cols, b.vals, b.batch_idx, nb, st.partials, nblk, b.entries)
        const int r4 = b.r / 4;
        if (r4 <= 1) LSGD_MC_LAUNCH(1);
        else if (r4 <= 2) LSGD_MC_LAUNCH(2);
        else if (r4 <= 4) LSGD_MC_LAUNCH(4);
        else if (r4 <= 8) LSGD_MC_LAUNCH(8);
        else if (r4 <= 16) LSGD_MC_LAUNCH(16);
        else if (r4 <= 32) LSGD_MC_LAUNCH(32);
        else LSGD_MC_LAUNCH(64);
#undef LSGD_MC_LAUNCH
    } else if (nblk > 0) {
        dim3 grid((unsigned)nblk, (unsigned)W);
#define LSGD_MC_LAUNCH(S)                                                                                              \
    hipLaunchKernelGGL((mc_grad_atomic_kernel<S, false>), grid, dim3(kMcThreads), 0, s, x, (float*)nullptr, ld, b.m, b.n, \
                       b.r, b.rows, b.cols, b.vals, b.batch_idx, nb, 0.0f, st.partials, nblk, b.entries)
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
