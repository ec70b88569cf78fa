// Fused leader-pull (+ momentum) update of the whole population, one pass.
//
//   d   = g + wd*x + lam_L (x - z_local) + lam_G (x - z_global)
//   mu = 0:  x <- x - eta*d            mu > 0:  m <- mu*m + d ; x <- x - eta*m
//
// (arXiv 1905.10395: supplement B.1 for the eta-scaled step, Eq. 3 for the two
// pulls, Algorithm 1 for leader copies kept between communications.)
//
// Geometry.  The update is independent per parameter column and bound by HBM
// traffic: 20 B per parameter with momentum (read x, g, m; write x, m), 12 B
// without.  It runs in place.  The only rows another row ever reads are the
// leaders, so the work is split in two launches:
//   1. pull_rows_kernel streams every row that is not being captured as a
//      leader, in plain row-major order (sequential x, g, m streams); it
//      reads the leader tiles it needs from x (leaders re-selected since the
//      last update, which this launch never writes) or from the kept-copy
//      buffer Z (Algorithm 1's stored leaders).
//   2. pull_leaders_kernel then updates the captured leader rows; there a
//      workgroup owns a column tile for all of them and takes its copies
//      before it stores anything, and writes the copies to Z.
// A re-selected leader therefore costs no extra pass over memory: the
// "broadcast" of the paper is two rows that stay in the memory-side cache.
#include "common.h"
#include "update_math.h"

namespace lsgd {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));

template <int VEC> struct Vec;
template <> struct Vec<4> { using type = v4f; };
template <> struct Vec<2> { using type = v2f; };
template <> struct Vec<1> { using type = float; };

template <int VEC> __device__ __forceinline__ typename Vec<VEC>::type ld_vec(const float* p)
{
    return *reinterpret_cast<const typename Vec<VEC>::type*>(p);
}
template <int VEC> __device__ __forceinline__ typename Vec<VEC>::type ld_stream(const float* p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const typename Vec<VEC>::type*>(p));
}

__device__ __forceinline__ void st_vec(float* p, v4f v) { *reinterpret_cast<v4f*>(p) = v; }
__device__ __forceinline__ void st_vec(float* p, v2f v) { *reinterpret_cast<v2f*>(p) = v; }
__device__ __forceinline__ void st_vec(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_stream(float* p, v4f v) { __builtin_nontemporal_store(v, reinterpret_cast<v4f*>(p)); }
__device__ __forceinline__ void st_stream(float* p, v2f v) { __builtin_nontemporal_store(v, reinterpret_cast<v2f*>(p)); }
__device__ __forceinline__ void st_stream(float* p, float v) { __builtin_nontemporal_store(v, p); }

__device__ __forceinline__ void st_bf16(uint16_t* p, v4f v)
{
    typedef unsigned int v2u __attribute__((ext_vector_type(2)));
    const v2u o = {f32x2_to_bf16x2(v.x, v.y), f32x2_to_bf16x2(v.z, v.w)};
    *reinterpret_cast<v2u*>(p) = o;
}
__device__ __forceinline__ void st_bf16(uint16_t* p, v2f v) { *reinterpret_cast<unsigned int*>(p) = f32x2_to_bf16x2(v.x, v.y); }
__device__ __forceinline__ void st_bf16(uint16_t* p, float v) { *p = f32_to_bf16_rne(v); }

__device__ __forceinline__ v4f zero_of(v4f) { return (v4f)(0.f); }
__device__ __forceinline__ v2f zero_of(v2f) { return (v2f)(0.f); }
__device__ __forceinline__ float zero_of(float) { return 0.f; }

constexpr int kPullThreads = 256;

struct PullDev {
    float* x;
    const float* g;
    float* m;
    float* Z;
    uint16_t* xb;
    int64_t col0, col1, ld; // columns [col0, col1)
    int row0;               // first row of this launch of the streaming kernel
    int W, G;
    float eta, lamL, lamG, mu, wd;
    int flags, use_refreshed;
    int group_size;     // l when all groups have l rows (group = row / l), else 0: look the group up
    const int32_t* offsets;
    const int32_t* group_of;
    const int32_t* lead;
    const int32_t* glead;
    const int32_t* refreshed;
    const RowPlan* plan;
};

template <class V>
__device__ __forceinline__ Coef make_coef(const PullDev& a)
{
    Coef c;
    c.eta = a.eta; c.mu = a.mu; c.wd = a.wd; c.cL = a.lamL; c.cG = a.lamG;
    c.nesterov = (a.flags & LSGD_NESTEROV) != 0;
    c.grad_only = (a.flags & LSGD_MOMENTUM_GRAD_ONLY) != 0;
    return c;
}

template <int VEC, int KIND>
__device__ __forceinline__ void apply_row(const PullDev& a, int64_t o, typename Vec<VEC>::type xv, typename Vec<VEC>::type gv,
                                          typename Vec<VEC>::type mv, const typename Vec<VEC>::type zl,
                                          const typename Vec<VEC>::type zg, const Coef& c)
{
    using V = typename Vec<VEC>::type;
    update_vec<KIND, V>(xv, gv, mv, zl, zg, c);
    st_stream(a.x + o, xv);
    if (KIND == 1) st_stream(a.m + o, mv);
    if (a.xb) st_bf16(a.xb + o, xv);
}

template <int VEC, int KIND>
__device__ __forceinline__ void update_row(const PullDev& a, int64_t o, typename Vec<VEC>::type xv,
                                           const typename Vec<VEC>::type zl, const typename Vec<VEC>::type zg, const Coef& c)
{
    using V = typename Vec<VEC>::type;
    V gv = (KIND != 2) ? ld_stream<VEC>(a.g + o) : zero_of(V());
    V mv = (KIND == 1) ? ld_stream<VEC>(a.m + o) : zero_of(V());
    apply_row<VEC, KIND>(a, o, xv, gv, mv, zl, zg, c);
}

// Kernel 1: every row that nobody reads as a freshly selected leader.  One
// workgroup per (row, column tile).  Workgroups are numbered so that they are
// dispatched chunk by chunk: the columns are cut into chunks of kChunkBytes
// (4 MB of one row); inside a chunk the order is plain row-major.  The
// x, g, m streams are then long sequential runs in memory, while the leader
// tiles of the chunk, which every row of a group re-reads, stay in the L2
// of the die that reads them instead of being fetched again for each row.
constexpr int64_t kChunkBytes = 4 << 20;

// VEC adjacent columns of one row, starting at col.  Everything the row needs to know about its leaders comes
// from its 32-byte plan record (one scalar load), so that the streams' loads are issued as early as possible.
template <int VEC, int KIND>
__device__ __forceinline__ void pull_rows_body(const PullDev& a, int row, int64_t col)
{
    using V = typename Vec<VEC>::type;
    constexpr bool COMM = KIND == 2;       // communication pull: every re-selected leader is captured
    bool pullG = COMM || a.lamG != 0.0f, pullL = COMM || a.lamL != 0.0f;
    RowPlan pl;
    pl.ll = pl.gl = -1; pl.freshL = pl.freshG = 0; pl.j = 0;
    if (pullL || pullG) pl = a.plan[row];
    const int j = pl.j;
    const int ll = pullL ? pl.ll : -1;
    const int gl = pullG ? pl.gl : -1;
    const bool freshL = pullL && a.use_refreshed && pl.freshL;
    const bool freshG = pullG && a.use_refreshed && pl.freshG;
    // rows captured as leaders in this update are handled by pull_leaders_kernel afterwards
    if ((freshL && row == ll) || (freshG && row == gl)) return;
    Coef c = make_coef<V>(a);
    if (COMM) {                            // only leaders selected just now pull
        if (!freshL) { c.cL = 0.0f; pullL = false; }
        if (!freshG) { c.cG = 0.0f; pullG = false; }
        if (c.cL == 0.0f && c.cG == 0.0f) return;
    }

    const int64_t o = (int64_t)row * a.ld + col;
    V xv = ld_stream<VEC>(a.x + o);
    V zl = zero_of(V()), zg = zero_of(V());
    if (pullL) zl = ld_vec<VEC>((freshL ? a.x + (int64_t)ll * a.ld : a.Z + (int64_t)j * a.ld) + col);
    if (pullG) zg = ld_vec<VEC>((freshG ? a.x + (int64_t)gl * a.ld : a.Z + (int64_t)a.G * a.ld) + col);
    if (!COMM && (a.flags & LSGD_LEADER_EXEMPT)) {
        if (row == ll) c.cL = 0.0f;
        if (row == gl) c.cG = 0.0f;
    }
    update_row<VEC, KIND>(a, o, xv, zl, zg, c);
}

// Grid: x = tile inside the chunk, y = row, z = chunk, which is the dispatch order described above without any
// index arithmetic in the kernel.  A thread whose group of columns straddles the end of the row takes them one by one.
template <int VEC, int KIND>
__global__ __launch_bounds__(kPullThreads) void pull_rows_kernel(PullDev a, int tpc)
{
    const int row = a.row0 + blockIdx.y;
    const int64_t tile = (int64_t)blockIdx.z * tpc + blockIdx.x;
    const int64_t col = a.col0 + (tile * kPullThreads + threadIdx.x) * VEC;
    if (col >= a.col1) return;
    if (VEC == 1 || col + VEC <= a.col1) {
        pull_rows_body<VEC, KIND>(a, row, col);
    } else {
        for (int64_t cc = col; cc < a.col1; ++cc) pull_rows_body<1, KIND>(a, row, cc);
    }
}

// Kernel 2 (runs after kernel 1): the rows that were captured as leaders.  A
// workgroup owns a column tile for all of them, so it can take every copy it
// needs before it stores anything: first the global leader's tile, whose own
// row is updated at once (its local pull still sees its group's leader
// untouched), then each re-selected local leader, whose pull to itself is
// exactly zero.  Captured tiles are also written to the kept-copy buffer Z.
template <int VEC, int KIND>
__device__ __forceinline__ void pull_leaders_body(const PullDev& a, int64_t col)
{
    using V = typename Vec<VEC>::type;
    constexpr bool COMM = KIND == 2;
    const bool pullG = COMM ? a.refreshed[a.G] != 0 : a.lamG != 0.0f, pullL = COMM || a.lamL != 0.0f;
    const bool exempt = !COMM && (a.flags & LSGD_LEADER_EXEMPT) != 0;
    const bool freshG = pullG && a.refreshed[a.G];
    const int gl = pullG ? a.glead[0] : -1;
    Coef c = make_coef<V>(a);
    if (COMM && !freshG) c.cG = 0.0f;

    V zg = zero_of(V());
    if (pullG) zg = ld_vec<VEC>((freshG ? a.x + (int64_t)gl * a.ld : a.Z + (int64_t)a.G * a.ld) + col);
    if (freshG) {
        if (a.Z) st_vec(a.Z + (int64_t)a.G * a.ld + col, zg);
        const int j = a.group_of[gl];
        const int ll = pullL ? a.lead[j] : -1;
        V zl = zero_of(V());
        Coef cg = c;
        if (COMM && !a.refreshed[j]) cg.cL = 0.0f;       // its group did not communicate: no local pull
        // its group's leader copy: the live row only when that group re-selected too (then a row
        // equal to gl is this very tile); a group that kept its leader pulls to the stored copy,
        // also when the kept leader is gl itself (the copy taken at the start of the period)
        if (pullL && cg.cL != 0.0f) {
            const bool freshL = a.refreshed[j] != 0;
            zl = (freshL && ll == gl) ? zg : ld_vec<VEC>((freshL ? a.x + (int64_t)ll * a.ld : a.Z + (int64_t)j * a.ld) + col);
        } else {
            cg.cL = 0.0f;
        }
        if (exempt) { cg.cG = 0.0f; if (ll == gl) cg.cL = 0.0f; }
        if (!(COMM && cg.cL == 0.0f && cg.cG == 0.0f))           // capture only: the row does not move
            update_row<VEC, KIND>(a, (int64_t)gl * a.ld + col, zg, zl, zg, cg);
    }
    if (!pullL) return;
    // re-selected local leaders, four at a time so that their loads are all in flight together
    constexpr int kBatch = 4;
    int j = 0;
    while (j < a.G) {
        int row[kBatch], grp[kBatch], cnt = 0;
        for (; j < a.G && cnt < kBatch; ++j) {
            if (!a.refreshed[j]) continue;
            const int ll = a.lead[j];
            if (freshG && ll == gl) {      // already updated above; its pre-update tile is zg
                if (a.Z) st_vec(a.Z + (int64_t)j * a.ld + col, zg);
                continue;
            }
            row[cnt] = ll; grp[cnt] = j; ++cnt;
        }
        V xv[kBatch], gv[kBatch], mv[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            if (u < cnt) {
                const int64_t o = (int64_t)row[u] * a.ld + col;
                xv[u] = ld_vec<VEC>(a.x + o);
                gv[u] = (KIND != 2) ? ld_stream<VEC>(a.g + o) : zero_of(V());
                mv[u] = (KIND == 1) ? ld_stream<VEC>(a.m + o) : zero_of(V());
            }
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            if (u < cnt) {
                const int64_t o = (int64_t)row[u] * a.ld + col;
                if (a.Z) st_vec(a.Z + (int64_t)grp[u] * a.ld + col, xv[u]);
                Coef cl = c;
                if (exempt) { cl.cL = 0.0f; if (row[u] == gl) cl.cG = 0.0f; }
                if (!(COMM && cl.cG == 0.0f))                         // a leader's pull to itself is zero
                    apply_row<VEC, KIND>(a, o, xv[u], gv[u], mv[u], xv[u], zg, cl);
            }
        }
    }
}

template <int VEC, int KIND>
__global__ __launch_bounds__(kPullThreads) void pull_leaders_kernel(PullDev a)
{
    const int64_t col = a.col0 + ((int64_t)blockIdx.x * kPullThreads + threadIdx.x) * VEC;
    if (col >= a.col1) return;
    if (VEC == 1 || col + VEC <= a.col1) {
        pull_leaders_body<VEC, KIND>(a, col);
    } else {
        for (int64_t cc = col; cc < a.col1; ++cc) pull_leaders_body<1, KIND>(a, cc);
    }
}

// VR: columns per thread of the streaming kernel, VL: of the leader-rows kernel.
template <int VR, int VL, int KIND>
static void launch_range(PullDev a, bool leaders, hipStream_t s)
{
    const int64_t cols = a.col1 - a.col0;
    if (cols <= 0) return;
    const int64_t per_block = (int64_t)kPullThreads * VR;
    const int64_t tiles = (cols + per_block - 1) / per_block;
    const int64_t chunk_tiles = kChunkBytes / (per_block * (int64_t)sizeof(float));
    const int tpc = (int)(tiles < chunk_tiles ? tiles : chunk_tiles);
    const int64_t chunks = (tiles + tpc - 1) / tpc;
    if (!(KIND == 2 && a.lamL == 0.0f && a.lamG == 0.0f)) {            // (capture only: no row moves)
        // grid.y and grid.z hold at most 65535 each: rows and chunks beyond that go to further launches
        for (int row0 = 0; row0 < a.W; row0 += 65535) {
            const int nrows = a.W - row0 < 65535 ? a.W - row0 : 65535;
            for (int64_t c0 = 0; c0 < chunks; c0 += 65535) {
                const int64_t nch = chunks - c0 < 65535 ? chunks - c0 : 65535;
                PullDev part = a;
                part.row0 = row0;
                part.col0 = a.col0 + c0 * tpc * per_block;
                hipLaunchKernelGGL((pull_rows_kernel<VR, KIND>), dim3((unsigned)tpc, (unsigned)nrows, (unsigned)nch), dim3(kPullThreads), 0, s,
                                   part, tpc);
            }
        }
    }
    if (leaders) {
        const int64_t lper = (int64_t)kPullThreads * VL;
        hipLaunchKernelGGL((pull_leaders_kernel<VL, KIND>), dim3((unsigned)((cols + lper - 1) / lper)), dim3(kPullThreads), 0, s, a);
    }
}

hipError_t launch_pull_update(const PullParams& p, const DeviceState& st, hipStream_t s)
{
    PullDev a;
    a.x = p.x; a.g = p.g; a.m = p.m; a.Z = p.Z; a.xb = p.xb;
    a.ld = p.ld; a.W = p.W; a.G = p.G;
    a.eta = p.eta; a.lamL = p.lamL; a.lamG = p.lamG; a.mu = p.mu; a.wd = p.wd;
    a.flags = p.flags; a.use_refreshed = p.use_refreshed; a.group_size = p.group_size;
    a.offsets = st.offsets; a.group_of = st.group_of; a.lead = st.lead; a.glead = st.glead; a.refreshed = st.refreshed;
    a.plan = st.plan;
    const bool comm = p.comm_pull != 0;
    const bool mom = !comm && p.mu != 0.0f;
    const bool leaders = p.use_refreshed && (comm || p.lamL != 0.0f || p.lamG != 0.0f);

    auto aligned = [](const void* q, unsigned n) { return (reinterpret_cast<uintptr_t>(q) & (n - 1u)) == 0; };
    auto layout_ok = [&](unsigned v) {      // every row start and every thread's group of v columns is v*4-byte aligned
        return (p.ld % v == 0) && aligned(p.x, 4 * v) && (comm || aligned(p.g, 4 * v)) && (!mom || aligned(p.m, 4 * v)) &&
               (!p.Z || aligned(p.Z, 4 * v)) && (!p.xb || aligned(p.xb, 2 * v));
    };
    // The streaming kernel moves 8 bytes per lane: on this chip a 3-read/2-write stream runs fastest with narrow
    // per-lane accesses and 2 KB of each stream per workgroup (16-byte lanes: 6.0 TB/s, 8-byte lanes: 6.7 TB/s).
    // The leader-rows kernel keeps 16-byte lanes when the layout allows.  A ragged last group of columns is
    // finished element-wise by its thread; layouts with odd strides or unaligned bases go element-wise altogether.
    a.col0 = 0; a.col1 = p.P; a.row0 = 0;
#define LSGD_PULL_DISPATCH(VR, VL) \
    do { if (comm) launch_range<VR, VL, 2>(a, leaders, s); else if (mom) launch_range<VR, VL, 1>(a, leaders, s); else launch_range<VR, VL, 0>(a, leaders, s); } while (0)
    if (layout_ok(4)) LSGD_PULL_DISPATCH(2, 4);
    else if (layout_ok(2)) LSGD_PULL_DISPATCH(2, 2);
    else LSGD_PULL_DISPATCH(1, 1);
#undef LSGD_PULL_DISPATCH
    return hipGetLastError();
}

// ---- whole-matrix fp32 -> bf16 cast (initial fill of the shadow) ----
__global__ __launch_bounds__(256) void cast_shadow_kernel(const float* __restrict__ x, uint16_t* __restrict__ xb,
                                                          int64_t P, int64_t ld)
{
    const int64_t row = blockIdx.y;
    for (int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; c < P; c += (int64_t)gridDim.x * blockDim.x)
        xb[row * ld + c] = f32_to_bf16_rne(x[row * ld + c]);
}

hipError_t launch_cast_shadow(const float* x, uint16_t* xb, int W, int64_t P, int64_t ld, hipStream_t s)
{
    int64_t blocks = (P + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(cast_shadow_kernel, dim3((unsigned)blocks, (unsigned)W), dim3(256), 0, s, x, xb, P, ld);
    return hipGetLastError();
}

} // namespace lsgd
