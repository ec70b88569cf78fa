// Per-worker gradient and loss of a fully connected ReLU classifier with softmax
// cross-entropy, for all W workers of the population at once (each worker has
// its own weights).  This is the stochastic gradient g_t^{j,i} that a worker
// takes on its own minibatch in arXiv 1905.10395 (Section 2), for the MLP
// workload: bf16 matrix operands, fp32 accumulation, fp32 gradients.
//
//   forward   z_k = h_{k-1} W_k^T + b_k ; h_k = bf16(relu(z_k)) ; logits fp32
//   loss      mean_b (logsumexp(z_L) - z_L[y_b]) ; delta_L = bf16((softmax - onehot)/B)
//   backward  dW_k = delta_k^T h_{k-1} ; db_k = sum_b delta_k ;
//             delta_{k-1} = bf16((delta_k W_k) .* [h_{k-1} > 0])
//
// The three matrix products are dense contractions and run on the matrix
// cores (v_mfma_f32_32x32x16_bf16) whenever the shapes are multiples of the
// tile sizes; a plain vector-ALU path covers every other shape, including
// the narrow classifier layer.
//
// Operand layouts for the MFMA kernel.  A lane feeds the matrix core eight
// consecutive values along the contraction index:
//   forward : A = h_{k-1} [B][d_in]   B-operand = W_k [d_out][d_in]    both contiguous in d_in
//   d-input : A = delta_k [B][d_out]  B-operand = W_k [d_out][d_in]    contraction over d_out: rows of W
//   d-weight: A = delta_k^T [d_out][B] B-operand = h_{k-1} [B][d_in]   contraction over B: rows of h
// In the last two the B-operand is contiguous along the *output* column.  Its
// tile is staged in LDS as it lies in memory and the fragments are fetched
// with the LDS transposing read (see lds_read_tr).  delta_k is stored in both
// layouts by the kernel that produces it.
#include "common.h"
#include "update_math.h"

namespace lsgd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

enum { EPI_FWD = 0, EPI_DX = 1, EPI_DW = 2, EPI_DWU = 3 };   // DWU: d-weight with the update applied in place of the store

struct GemmArgs {
    const uint16_t* A; int64_t sA; int64_t lda;   // [M][K], per-worker stride sA (elements)
    const uint16_t* B; int64_t sB; int64_t ldb;   // TRANS_B ? [K][N] : [N][K]
    int M, N, K;
    const float* bias; int64_t sBias;             // EPI_FWD: fp32 [N]
    const uint16_t* mask; int64_t sMask; int64_t ldmask; // EPI_DX: h_{k-1} [M][N]
    uint16_t* out; int64_t sOut; int64_t ldout;   // EPI_FWD: h [M][N]; EPI_DX: delta [M][N]
    uint16_t* outT; int64_t sOutT; int64_t ldoutT;// EPI_DX: delta^T [N][M]
    float* C; int64_t sC; int64_t ldc;            // EPI_DW: fp32 [M][N]
    FusedUpdate fu; int64_t colC;                 // EPI_DWU: update state; column of C[0][0] in the parameter row
};

// Per-worker view of the fused update: coefficients (with the leader exemption resolved) and row pointers.
struct FusedRow {
    Coef c;
    float* x;
    float* m;
    uint16_t* xb;
    const float* zl;
    const float* zg;
};

__device__ __forceinline__ FusedRow fused_row(const FusedUpdate& u, int w, int64_t ld)
{
    FusedRow r;
    r.c.eta = u.eta; r.c.mu = u.mu; r.c.wd = u.wd; r.c.cL = u.lamL; r.c.cG = u.lamG;
    r.c.nesterov = (u.flags & LSGD_NESTEROV) != 0;
    r.c.grad_only = (u.flags & LSGD_MOMENTUM_GRAD_ONLY) != 0;
    const int j = u.group_of[w];
    if (u.flags & LSGD_LEADER_EXEMPT) {
        if (u.lamL != 0.0f && u.lead[j] == w) r.c.cL = 0.0f;
        if (u.lamG != 0.0f && u.glead[0] == w) r.c.cG = 0.0f;
    }
    r.x = u.x + (int64_t)w * ld;
    r.m = u.m ? u.m + (int64_t)w * ld : nullptr;
    r.xb = u.xb + (int64_t)w * ld;
    r.zl = (u.lamL != 0.0f) ? u.Z + (int64_t)j * ld : nullptr;
    r.zg = (u.lamG != 0.0f) ? u.Z + (int64_t)u.G * ld : nullptr;
    return r;
}

// N parameters at columns base + off[0..N) of the worker's row, gradient values gv: all loads first,
// then the arithmetic, then the stores (x, m, bf16 copy).
template <int N>
__device__ __forceinline__ void fused_apply(const FusedRow& r, int64_t base, const int (&off)[N], const float (&gv)[N])
{
    float* xp = r.x + base;
    float* mp = r.m ? r.m + base : nullptr;
    const float* lp = r.zl ? r.zl + base : nullptr;
    const float* gp = r.zg ? r.zg + base : nullptr;
    uint16_t* bp = r.xb + base;
    float xv[N], mv[N], zl[N], zg[N];
#pragma unroll
    for (int v = 0; v < N; ++v) xv[v] = xp[off[v]];
#pragma unroll
    for (int v = 0; v < N; ++v) mv[v] = mp ? mp[off[v]] : 0.f;
#pragma unroll
    for (int v = 0; v < N; ++v) zl[v] = lp ? lp[off[v]] : 0.f;
#pragma unroll
    for (int v = 0; v < N; ++v) zg[v] = gp ? gp[off[v]] : 0.f;
#pragma unroll
    for (int v = 0; v < N; ++v) {
        if (mp) update_vec<1, float>(xv[v], gv[v], mv[v], zl[v], zg[v], r.c);
        else update_vec<0, float>(xv[v], gv[v], mv[v], zl[v], zg[v], r.c);
    }
#pragma unroll
    for (int v = 0; v < N; ++v) {
        xp[off[v]] = xv[v];
        if (mp) mp[off[v]] = mv[v];
        bp[off[v]] = f32_to_bf16_rne(xv[v]);
    }
}

// R groups of four adjacent parameters (columns multiples of 4, rows 16-byte aligned) at element offsets
// `off` of the worker's row: the loads of one batch are issued as a block, so that they are in flight while the previous batch is updated and stored.
template <int R>
struct FusedBatch {
    int64_t off[R];
    f32x4 xv[R], mv[R], zl[R], zg[R];
};

template <int R>
__device__ __forceinline__ void fused_load4(const FusedRow& r, FusedBatch<R>& b)
{
    const f32x4 zero = (f32x4)(0.f);
#pragma unroll
    for (int q = 0; q < R; ++q) b.xv[q] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(r.x + b.off[q]));
#pragma unroll
    for (int q = 0; q < R; ++q) b.mv[q] = r.m ? __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(r.m + b.off[q])) : zero;
#pragma unroll
    for (int q = 0; q < R; ++q) b.zl[q] = r.zl ? *reinterpret_cast<const f32x4*>(r.zl + b.off[q]) : zero;
#pragma unroll
    for (int q = 0; q < R; ++q) b.zg[q] = r.zg ? *reinterpret_cast<const f32x4*>(r.zg + b.off[q]) : zero;
}

template <int R>
__device__ __forceinline__ void fused_store4(const FusedRow& r, FusedBatch<R>& b, const f32x4 (&gv)[R])
{
#pragma unroll
    for (int q = 0; q < R; ++q) {
        if (r.m) update_vec<1, f32x4>(b.xv[q], gv[q], b.mv[q], b.zl[q], b.zg[q], r.c);
        else update_vec<0, f32x4>(b.xv[q], gv[q], b.mv[q], b.zl[q], b.zg[q], r.c);
    }
#pragma unroll
    for (int q = 0; q < R; ++q) {
        __builtin_nontemporal_store(b.xv[q], reinterpret_cast<f32x4*>(r.x + b.off[q]));
        if (r.m) __builtin_nontemporal_store(b.mv[q], reinterpret_cast<f32x4*>(r.m + b.off[q]));
        const u32x2 o = {f32x2_to_bf16x2(b.xv[q].x, b.xv[q].y), f32x2_to_bf16x2(b.xv[q].z, b.xv[q].w)};
        *reinterpret_cast<u32x2*>(r.xb + b.off[q]) = o;
    }
}

constexpr int kBK = 64;          // contraction tile
constexpr int kLdk = kBK + 8;    // padded LDS row (bf16 elements): 144 B

// An operand given as [k][n] (n contiguous: the weights in the d-input product, the activations in the
// d-weight product) is staged in LDS as it lies in memory, 64 k-rows of BN + kPadN elements: the padding shifts
// consecutive rows by 64 bytes, i.e. a quarter of the banks, so that the four rows one transposing read touches
// cover all banks once.  The matrix cores want, per lane, eight consecutive k of one column n; the LDS
// transposing read delivers that: in every group of 16 lanes, lane i supplies the address of four consecutive
// elements, the 16 x 4 elements are taken as a 4 x 16 matrix (lanes 4r .. 4r+3 hold row r), and lane i receives
// column i.  With lanes 4r .. 4r+3 pointing at k-row r, columns n0 .. n0+15, lane i gets (k0 .. k0+3, n0 + i).
constexpr int kPadN = 32;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ s16x4 lds_read_tr(const uint16_t* p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
}

// BM x BN output tile per workgroup, WVM x WVN wavefronts, each owning (BM/WVM) x (BN/WVN).
// 128x128 / 128x64 with 2x2 wavefronts run two workgroups per CU; 256x256 with 2x4 wavefronts
// (128x64 per wavefront, all 147 KB of LDS) moves half the bytes through LDS per flop.
template <int BM, int BN, int WVM, int WVN, bool TRANS_B, int EPI>
__global__ __launch_bounds__(64 * WVM * WVN, (WVM * WVN > 4) ? 1 : 2) void gemm_bf16_kernel(GemmArgs g)  // min. workgroups per CU
{
    constexpr int kGemmThreads = 64 * WVM * WVN;
    constexpr int WTM = BM / WVM, WTN = BN / WVN;
    constexpr int TM = WTM / 32, TN = WTN / 32;      // 32x32 MFMA tiles per wavefront
    constexpr int A_CHUNKS = BM * (kBK / 8) / kGemmThreads; // 16-byte chunks per thread
    constexpr int B_CHUNKS = BN * (kBK / 8) / kGemmThreads;
    constexpr int LDN = BN + kPadN;                  // row of a [k][n]-staged tile
    constexpr int B_TILE = TRANS_B ? kBK * LDN : BN * kLdk;   // elements of one B buffer
    constexpr int STAGES = (TM * TN > 4) ? 1 : 2;    // register stages of global prefetch (one beside 128 accumulator registers)

    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t* As = smem;                              // [2][BM][kLdk]
    uint16_t* Bs = smem + 2 * BM * kLdk;              // [2][BN][kLdk], or [2][kBK][LDN] for a [k][n] operand

    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    const int wm = wid / WVN, wn = wid % WVN;
    // Fused update: a die (workgroup id modulo 8) owns every eighth tile column, and visits its tiles
    // row by row with the workers varying fastest.  All workers' workgroups for one tile then run
    // together on one die, so the tile of the leader copies they share is fetched into that die's L2
    // once; a worker's delta^T tile is reused across the die's columns and its h tiles across rows.
    int w, tm, tn;
    if (EPI == EPI_DWU) {
        const int W = (int)gridDim.z, tiles_n = (int)gridDim.x;
        const int64_t id = ((int64_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
        if (tiles_n % 8 == 0) {
            const int xcd = (int)(id & 7);
            int64_t s = id >> 3;
            w = (int)(s % W); s /= W;
            const int per = tiles_n / 8;
            tn = (int)(s % per) * 8 + xcd;
            tm = (int)(s / per);
        } else {
            w = (int)(id % W);
            const int64_t tile = id / W;
            tn = (int)(tile % tiles_n); tm = (int)(tile / tiles_n);
        }
    } else {
        w = blockIdx.z; tm = blockIdx.y; tn = blockIdx.x;
    }
    const int m0 = tm * BM, n0 = tn * BN;
    const uint16_t* A = g.A + (int64_t)w * g.sA + (int64_t)m0 * g.lda;
    const uint16_t* B = g.B + (int64_t)w * g.sB;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // two register stages: the loads of k-steps kt+1 and kt+2 are in flight while kt is multiplied
    constexpr int RB = B_CHUNKS;
    u32x4 ra0[A_CHUNKS], ra1[STAGES == 2 ? A_CHUNKS : 1];
    u32x4 rb0[RB], rb1[STAGES == 2 ? RB : 1];

    auto load_global = [&](int kt, u32x4* ra, u32x4* rb) {
        const int k0 = kt * kBK;
#pragma unroll
        for (int c = 0; c < A_CHUNKS; ++c) {
            const int id = tid + c * kGemmThreads, row = id >> 3, ch = id & 7;
            ra[c] = *reinterpret_cast<const u32x4*>(A + (int64_t)row * g.lda + k0 + ch * 8);
        }
        if (TRANS_B) {
#pragma unroll
            for (int c = 0; c < B_CHUNKS; ++c) {
                const int id = tid + c * kGemmThreads, row = id / (BN / 8), ch = id % (BN / 8);
                rb[c] = *reinterpret_cast<const u32x4*>(B + (int64_t)(k0 + row) * g.ldb + n0 + ch * 8);
            }
        } else {
#pragma unroll
            for (int c = 0; c < B_CHUNKS; ++c) {
                const int id = tid + c * kGemmThreads, row = id >> 3, ch = id & 7;
                rb[c] = *reinterpret_cast<const u32x4*>(B + (int64_t)(n0 + row) * g.ldb + k0 + ch * 8);
            }
        }
    };
    auto store_lds = [&](int buf, const u32x4* ra, const u32x4* rb) {
        uint16_t* as = As + buf * BM * kLdk;
        uint16_t* bs = Bs + buf * B_TILE;
#pragma unroll
        for (int c = 0; c < A_CHUNKS; ++c) {
            const int id = tid + c * kGemmThreads, row = id >> 3, ch = id & 7;
            *reinterpret_cast<u32x4*>(as + row * kLdk + ch * 8) = ra[c];
        }
        if (TRANS_B) {
#pragma unroll
            for (int c = 0; c < B_CHUNKS; ++c) {
                const int id = tid + c * kGemmThreads, row = id / (BN / 8), ch = id % (BN / 8);
                *reinterpret_cast<u32x4*>(bs + row * LDN + ch * 8) = rb[c];
            }
        } else {
#pragma unroll
            for (int c = 0; c < B_CHUNKS; ++c) {
                const int id = tid + c * kGemmThreads, row = id >> 3, ch = id & 7;
                *reinterpret_cast<u32x4*>(bs + row * kLdk + ch * 8) = rb[c];
            }
        }
    };

    auto compute = [&](int buf) {
        const uint16_t* as = As + buf * BM * kLdk;
        const uint16_t* bs = Bs + buf * B_TILE;
#pragma unroll
        for (int kk = 0; kk < kBK / 16; ++kk) {
            bf16x8 af[TM], bfr[TN];
            const int ch = kk * 2 + (lane >> 5);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = wm * WTM + i * 32 + (lane & 31);
                af[i] = *reinterpret_cast<const bf16x8*>(as + row * kLdk + ch * 8);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (TRANS_B) {
                    // lane (n = lane % 32, k-half = lane / 32): k = 16 kk + 8 (lane / 32) + 0..7 of column n
                    const int i = lane & 15;
                    const int col = wn * WTN + j * 32 + (lane & 16) + 4 * (i & 3);
                    const int row = kk * 16 + 8 * (lane >> 5) + (i >> 2);
                    const s16x4 lo = lds_read_tr(bs + row * LDN + col);
                    const s16x4 hi = lds_read_tr(bs + (row + 4) * LDN + col);
                    const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    bfr[j] = __builtin_bit_cast(bf16x8, v);
                } else {
                    const int row = wn * WTN + j * 32 + (lane & 31);
                    bfr[j] = *reinterpret_cast<const bf16x8*>(bs + row * kLdk + ch * 8);
                }
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
    };

    // Pipeline.  LDS holds k-steps kt (being multiplied) and kt+1.  Each iteration first hands the
    // register stage that has arrived to LDS (into the buffer nobody reads now) and re-issues it for
    // a later k-step, then multiplies: LDS writes and global loads drain underneath the MFMAs.
    // Two register stages (k-steps kt+1 and kt+2 in flight) where registers allow, else one.
    const int nk = g.K / kBK;
    if (STAGES == 2) {
        load_global(0, ra0, rb0);
        if (nk > 1) load_global(1, ra1, rb1);
        store_lds(0, ra0, rb0);
        if (nk > 2) load_global(2, ra0, rb0);
        __syncthreads();
        int kt = 0;
        for (; kt + 1 < nk; kt += 2) {                    // both halves always run: no exit in the middle of the body
            store_lds(1, ra1, rb1);
            if (kt + 3 < nk) load_global(kt + 3, ra1, rb1);
            compute(0);
            __syncthreads();
            if (kt + 2 < nk) store_lds(0, ra0, rb0);
            if (kt + 4 < nk) load_global(kt + 4, ra0, rb0);
            compute(1);
            __syncthreads();
        }
        if (kt < nk) {                                    // odd number of k-steps: the last one sits in buffer 0
            compute(0);
            __syncthreads();
        }
    } else {
        load_global(0, ra0, rb0);
        store_lds(0, ra0, rb0);
        if (nk > 1) load_global(1, ra0, rb0);
        __syncthreads();
        for (int kt = 0; kt < nk; ++kt) {
            const int buf = kt & 1;
            if (kt + 1 < nk) store_lds(buf ^ 1, ra0, rb0);
            if (kt + 2 < nk) load_global(kt + 2, ra0, rb0);
            compute(buf);
            __syncthreads();
        }
    }

    // epilogue: lane holds column n = lane%32 and rows (lane/32)*4 + 8*(v/4) + v%4 of each 32x32 tile
    if (EPI == EPI_DWU) {
        // The update streams x, m and the leader copies, so it wants whole rows per wavefront: the
        // accumulators go through LDS (reusing the operand buffers), 32 rows of every wavefront row at a
        // time, and come back as float4 per thread with a wavefront covering contiguous row segments.
        constexpr int LDC = BN + 4;                       // padded fp32 row
        constexpr int CH_ROWS = WVM * 32;                 // rows staged at a time
        constexpr int C4 = BN / 4;                        // float4 per row
        constexpr int RPP = kGemmThreads / C4;            // rows covered by one pass of all threads
        constexpr int PASSES = CH_ROWS / RPP;
        constexpr int R = PASSES < 4 ? PASSES : 4;        // rows in flight per thread
        static_assert(CH_ROWS % RPP == 0 && PASSES % R == 0, "tile shape");
        float* stage = reinterpret_cast<float*>(smem);
        const FusedRow fr = fused_row(g.fu, w, g.sC);
        const int c4 = tid % C4, r0 = tid / C4;
        constexpr int BPR = PASSES / R;                   // batches per staged block of rows
        constexpr int NB = TM * BPR;
        FusedBatch<R> fb[2];
        auto set_cols = [&](int bi, FusedBatch<R>& b) {   // batch bi = (staged block, pass group)
            const int i = bi / BPR, p0 = (bi % BPR) * R;
#pragma unroll
            for (int q = 0; q < R; ++q) {
                const int rr = r0 + (p0 + q) * RPP;        // row inside the staged block
                const int m = m0 + (rr >> 5) * WTM + i * 32 + (rr & 31);
                b.off[q] = g.colC + (int64_t)m * g.ldc + n0 + c4 * 4;
            }
        };
        set_cols(0, fb[0]);
        fused_load4<R>(fr, fb[0]);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            __syncthreads();                              // operand buffers / previous block no longer read
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int rl = wm * 32 + (lane >> 5) * 4 + 8 * (v >> 2) + (v & 3);
                    stage[rl * LDC + wn * WTN + j * 32 + (lane & 31)] = acc[i][j][v];
                }
            __syncthreads();
#pragma unroll
            for (int qb = 0; qb < BPR; ++qb) {
                const int bi = i * BPR + qb;
                if (bi + 1 < NB) {                        // next batch's loads fly while this one is finished
                    set_cols(bi + 1, fb[(bi + 1) & 1]);
                    fused_load4<R>(fr, fb[(bi + 1) & 1]);
                }
                f32x4 gv[R];
#pragma unroll
                for (int q = 0; q < R; ++q) {
                    const int rr = r0 + (qb * R + q) * RPP;
                    gv[q] = *reinterpret_cast<const f32x4*>(stage + rr * LDC + c4 * 4);
                }
                fused_store4<R>(fr, fb[bi & 1], gv);
            }
        }
        return;
    }
    if (EPI == EPI_FWD || EPI == EPI_DX) {
        // bf16 results leave through LDS (the operand buffers are free now): lanes hold single columns, a
        // row-major tile in LDS turns them into 16-byte pieces of rows, 256 contiguous bytes per 16 lanes.
        constexpr int LDT = BN + kPadN;                   // rows shift by 64 bytes, as for the transposing read
        constexpr int T_CHUNKS = BM * (BN / 8) / kGemmThreads;
        static_assert((size_t)BM * LDT <= (size_t)2 * (BM * kLdk + B_TILE), "result tile fits the operand buffers");
        uint16_t* T = smem;
        uint16_t* out = g.out + (int64_t)w * g.sOut;
        if (EPI == EPI_DX) {
            // the ReLU mask (h_{k-1} != 0) arrives as 16-byte pieces too and is read back per lane with the
            // transposing read: rows R .. R+3 of the lane's own column, the layout of four accumulators
            const uint16_t* mask = g.mask + (int64_t)w * g.sMask;
            u32x4 mk[T_CHUNKS];
#pragma unroll
            for (int c = 0; c < T_CHUNKS; ++c) {
                const int id = tid + c * kGemmThreads, row = id / (BN / 8), ch = id % (BN / 8);
                mk[c] = *reinterpret_cast<const u32x4*>(mask + (int64_t)(m0 + row) * g.ldmask + n0 + ch * 8);
            }
#pragma unroll
            for (int c = 0; c < T_CHUNKS; ++c) {
                const int id = tid + c * kGemmThreads, row = id / (BN / 8), ch = id % (BN / 8);
                *reinterpret_cast<u32x4*>(T + row * LDT + ch * 8) = mk[c];
            }
            __syncthreads();
        }
        uint16_t* outT = (EPI == EPI_DX) ? g.outT + (int64_t)w * g.sOutT : nullptr;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int nl = wn * WTN + j * 32 + (lane & 31);               // column inside the tile
                const int rb = wm * WTM + i * 32 + (lane >> 5) * 4;            // first row inside the tile
                if (EPI == EPI_FWD) {
                    const float b = g.bias[(int64_t)w * g.sBias + n0 + nl];
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const float z = acc[i][j][v] + b;
                        T[(rb + 8 * (v >> 2) + (v & 3)) * LDT + nl] = f32_to_bf16_rne(z > 0.f ? z : 0.f);
                    }
                } else {
                    const int l16 = lane & 15;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        // every 4 x 16 block of the tile is read and then overwritten by the same 16 lanes
                        const s16x4 on = lds_read_tr(T + (rb + 8 * q + (l16 >> 2)) * LDT + wn * WTN + j * 32 + (lane & 16) + 4 * (l16 & 3));
                        uint32_t pk[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const uint16_t d = on[r] != 0 ? f32_to_bf16_rne(acc[i][j][q * 4 + r]) : (uint16_t)0;
                            T[(rb + 8 * q + r) * LDT + nl] = d;
                            pk[r] = d;
                        }
                        // the transposed copy: the lane's four rows are 8 contiguous bytes of it
                        const u32x2 o = {pk[0] | (pk[1] << 16), pk[2] | (pk[3] << 16)};
                        *reinterpret_cast<u32x2*>(outT + (int64_t)(n0 + nl) * g.ldoutT + m0 + rb + 8 * q) = o;
                    }
                }
            }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < T_CHUNKS; ++c) {
            const int id = tid + c * kGemmThreads, row = id / (BN / 8), ch = id % (BN / 8);
            *reinterpret_cast<u32x4*>(out + (int64_t)(m0 + row) * g.ldout + n0 + ch * 8) = *reinterpret_cast<const u32x4*>(T + row * LDT + ch * 8);
        }
        return;
    }
    float* C = g.C + (int64_t)w * g.sC;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n0 + wn * WTN + j * 32 + (lane & 31);
            const int mb = m0 + wm * WTM + i * 32 + (lane >> 5) * 4;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = mb + 8 * (v >> 2) + (v & 3);
                C[(int64_t)m * g.ldc + n] = acc[i][j][v];
            }
        }
}

template <int BM, int BN, int WVM, int WVN, bool TRANS_B, int EPI>
static void launch_gemm(const GemmArgs& g, int W, hipStream_t s)
{
    const size_t lds = (size_t)2 * (BM * kLdk + (TRANS_B ? kBK * (BN + kPadN) : BN * kLdk)) * sizeof(uint16_t);
    static bool configured = false;
    if (!configured) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_kernel<BM, BN, WVM, WVN, TRANS_B, EPI>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        configured = true;
    }
    dim3 grid((unsigned)(g.N / BN), (unsigned)(g.M / BM), (unsigned)W);
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WVM, WVN, TRANS_B, EPI>), grid, dim3(64 * WVM * WVN), lds, s, g);
}

static bool aligned_for_mfma(const GemmArgs& g)
{
    auto a16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
    return a16(g.A) && a16(g.B) && g.lda % 8 == 0 && g.ldb % 8 == 0 && g.sA % 8 == 0 && g.sB % 8 == 0;
}

// Picks the largest tile whose grid still fills the chip; returns false when no MFMA tile fits the shape.
template <bool TRANS_B, int EPI>
static bool try_mfma(const GemmArgs& g, int W, hipStream_t s)
{
    if (g.K % kBK || g.M % 128 || g.N % 64 || !aligned_for_mfma(g)) return false;
    if (EPI == EPI_DX && (g.ldoutT % 4 || (reinterpret_cast<uintptr_t>(g.outT) & 7u) || g.sOutT % 4)) return false;
    if (EPI == EPI_FWD || EPI == EPI_DX) {                 // 16-byte pieces of the result rows (and of the mask rows)
        auto a16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
        if (!a16(g.out) || g.ldout % 8 || g.sOut % 8) return false;
        if (EPI == EPI_DX && (!a16(g.mask) || g.ldmask % 8 || g.sMask % 8)) return false;
    }
    if (EPI == EPI_DWU) {                                  // float4 rows of x, m, Z; 8-byte groups of the bf16 copy
        auto a16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
        if (g.colC % 4 || g.ldc % 4 || g.sC % 4 || !a16(g.fu.x) || !a16(g.fu.m) || !a16(g.fu.Z) ||
            (reinterpret_cast<uintptr_t>(g.fu.xb) & 7u))
            return false;
    }
    const int64_t blocks256 = (g.M % 256 == 0 && g.N % 256 == 0) ? (int64_t)(g.M / 256) * (g.N / 256) * W : 0;
    const int64_t blocks128 = (int64_t)(g.M / 128) * (g.N / 128) * W;
    // the fused update keeps two batches of x, m and leader values in registers: no room beside a 256x256 tile
    // a 256-row tile covers a whole batch of 256: the weight operand is then read once instead of twice
    const int64_t blocks_tall = (g.M % 256 == 0 && g.N % 128 == 0) ? (int64_t)(g.M / 256) * (g.N / 128) * W : 0;
    if (blocks256 >= 256 && EPI != EPI_DWU) launch_gemm<256, 256, 2, 4, TRANS_B, EPI>(g, W, s);
    else if ((EPI == EPI_FWD || EPI == EPI_DX) && blocks_tall >= 256) launch_gemm<256, 128, 4, 2, TRANS_B, EPI>(g, W, s);
    else if (g.N % 128 == 0 && blocks128 >= 256) launch_gemm<128, 128, 2, 2, TRANS_B, EPI>(g, W, s);
    else launch_gemm<128, 64, 2, 2, TRANS_B, EPI>(g, W, s);
    return true;
}

// ------------------------------------------------------------------------------------------
// Vector-ALU kernels: any shape.  They are the path of the narrow classifier layer and the
// fallback of shapes the MFMA tiles do not divide.
// ------------------------------------------------------------------------------------------

// out[b][o] = sum_i h[b][i] * Wq[o][i] + bias[o].  One wavefront per (b, worker); lanes stride over i.
// HIDDEN: relu + bf16 store; else fp32 logits.
template <bool HIDDEN>
__global__ __launch_bounds__(256) void fwd_valu_kernel(const uint16_t* __restrict__ H, int64_t sH, int64_t ldh,
                                                       const uint16_t* __restrict__ Wq, int64_t sW, const float* __restrict__ bias,
                                                       int64_t sBias, int B, int din, int dout, uint16_t* __restrict__ out,
                                                       float* __restrict__ logits, int64_t sOut, int64_t ldout)
{
    const int lane = threadIdx.x & 63;
    const int b = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int w = blockIdx.y;
    if (b >= B) return;
    const uint16_t* h = H + (int64_t)w * sH + (int64_t)b * ldh;
    const uint16_t* Wm = Wq + (int64_t)w * sW;
    for (int o = 0; o < dout; ++o) {
        const uint16_t* wr = Wm + (int64_t)o * din;
        float acc = 0.f;
        for (int i = lane; i < din; i += 64) acc = fmaf(bf16_to_f32(h[i]), bf16_to_f32(wr[i]), acc);
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) acc += __shfl_xor(acc, d, 64);
        if (lane == 0) {
            const float z = acc + bias[(int64_t)w * sBias + o];
            if (HIDDEN) out[(int64_t)w * sOut + (int64_t)b * ldout + o] = f32_to_bf16_rne(z > 0.f ? z : 0.f);
            else logits[(int64_t)w * sOut + (int64_t)b * ldout + o] = z;
        }
    }
}

// Softmax cross-entropy of one worker's batch: loss = mean_b(lse - z[y]); delta = bf16((p - onehot)/B),
// stored as [B][C] and [C][B].  One workgroup per worker.
__global__ __launch_bounds__(256) void loss_delta_kernel(const float* __restrict__ logits, int64_t sLogits, const int32_t* __restrict__ y,
                                                         int B, int C, uint16_t* __restrict__ delta, uint16_t* __restrict__ deltaT,
                                                         int64_t sDelta, float* __restrict__ losses)
{
    const int w = blockIdx.x;
    const float* lg = logits + (int64_t)w * sLogits;
    uint16_t* d = delta + (int64_t)w * sDelta;
    uint16_t* dT = deltaT + (int64_t)w * sDelta;
    const float invB = 1.0f / (float)B;
    double part = 0.0;
    for (int b = threadIdx.x; b < B; b += 256) {
        const float* z = lg + (int64_t)b * C;
        float mx = z[0];
        for (int c = 1; c < C; ++c) mx = fmaxf(mx, z[c]);
        float se = 0.f;
        for (int c = 0; c < C; ++c) se += expf(z[c] - mx);
        const float lse = mx + logf(se);
        const int yb = y[(int64_t)w * B + b];
        part += (double)(lse - z[yb]);
        for (int c = 0; c < C; ++c) {
            const float p = expf(z[c] - lse);
            const uint16_t q = f32_to_bf16_rne((p - (c == yb ? 1.f : 0.f)) * invB);
            d[(int64_t)b * C + c] = q;
            dT[(int64_t)c * B + b] = q;
        }
    }
    __shared__ double red[256];
    red[threadIdx.x] = part;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) losses[w] = (float)(red[0] / (double)B);
}

// dW[o][i] = sum_b deltaT[o][b] * h[b][i].  One thread per (o, i).
__global__ __launch_bounds__(256) void dw_valu_kernel(const uint16_t* __restrict__ deltaT, int64_t sD, const uint16_t* __restrict__ H,
                                                      int64_t sH, int64_t ldh, int B, int din, int dout, float* __restrict__ g, int64_t sG,
                                                      FusedUpdate fu, int64_t col0)
{
    const int w = blockIdx.z, o = blockIdx.y;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= din) return;
    const uint16_t* dt = deltaT + (int64_t)w * sD + (int64_t)o * B;
    const uint16_t* h = H + (int64_t)w * sH;
    float acc = 0.f;
    for (int b = 0; b < B; ++b) acc = fmaf(bf16_to_f32(dt[b]), bf16_to_f32(h[(int64_t)b * ldh + i]), acc);
    if (fu.enabled) {
        const int off[1] = {0};
        const float gv[1] = {acc};
        fused_apply<1>(fused_row(fu, w, sG), col0 + (int64_t)o * din + i, off, gv);
    } else {
        g[(int64_t)w * sG + (int64_t)o * din + i] = acc;
    }
}

// db[o] = sum_b deltaT[o][b].  One wavefront per o.
__global__ __launch_bounds__(256) void db_kernel(const uint16_t* __restrict__ deltaT, int64_t sD, int B, int dout, float* __restrict__ g, int64_t sG,
                                                 FusedUpdate fu, int64_t col0)
{
    const int lane = threadIdx.x & 63;
    const int o = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int w = blockIdx.y;
    if (o >= dout) return;
    const uint16_t* dt = deltaT + (int64_t)w * sD + (int64_t)o * B;
    float acc = 0.f;
    for (int b = lane; b < B; b += 64) acc += bf16_to_f32(dt[b]);
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) acc += __shfl_xor(acc, d, 64);
    if (lane == 0) {
        if (fu.enabled) {
            const int off[1] = {0};
            const float gv[1] = {acc};
            fused_apply<1>(fused_row(fu, w, sG), col0 + o, off, gv);
        } else {
            g[(int64_t)w * sG + o] = acc;
        }
    }
}

// dprev[b][i] = bf16((sum_o delta[b][o] * Wq[o][i]) * [h[b][i] > 0]), also stored transposed.  One thread per (b, i).
__global__ __launch_bounds__(256) void dx_valu_kernel(const uint16_t* __restrict__ delta, int64_t sD, const uint16_t* __restrict__ Wq, int64_t sW,
                                                      const uint16_t* __restrict__ H, int64_t sH, int64_t ldh, int B, int din, int dout,
                                                      uint16_t* __restrict__ dprev, uint16_t* __restrict__ dprevT, int64_t sP)
{
    const int w = blockIdx.z, b = blockIdx.y;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= din) return;
    const uint16_t* d = delta + (int64_t)w * sD + (int64_t)b * dout;
    const uint16_t* Wm = Wq + (int64_t)w * sW;
    float acc = 0.f;
    for (int o = 0; o < dout; ++o) acc = fmaf(bf16_to_f32(d[o]), bf16_to_f32(Wm[(int64_t)o * din + i]), acc);
    const bool on = H[(int64_t)w * sH + (int64_t)b * ldh + i] != 0;
    const uint16_t q = on ? f32_to_bf16_rne(acc) : (uint16_t)0;
    dprev[(int64_t)w * sP + (int64_t)b * din + i] = q;
    dprevT[(int64_t)w * sP + (int64_t)i * B + b] = q;
}

// ---- narrow-layer kernels: the classifier layer (a handful of classes) with 16-byte loads ----
__device__ __forceinline__ void unpack8(const u32x4 v, float* f)
{
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        f[2 * q] = __uint_as_float(v[q] << 16);
        f[2 * q + 1] = __uint_as_float(v[q] & 0xFFFF0000u);
    }
}

// One wavefront per output (b, o): out = <h[b,:], Wq[o,:]> + bias[o].  d_in % 8 == 0, rows 16-byte aligned.
template <bool HIDDEN>
__global__ __launch_bounds__(256) void fwd_narrow_kernel(const uint16_t* __restrict__ H, int64_t sH, int64_t ldh,
                                                         const uint16_t* __restrict__ Wq, int64_t sW, const float* __restrict__ bias,
                                                         int64_t sBias, int B, int din, int dout, uint16_t* __restrict__ out,
                                                         float* __restrict__ logits, int64_t sOut, int64_t ldout)
{
    const int lane = threadIdx.x & 63;
    const int64_t idx = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int w = blockIdx.y;
    if (idx >= (int64_t)B * dout) return;
    const int b = (int)(idx / dout), o = (int)(idx % dout);
    const u32x4* h = reinterpret_cast<const u32x4*>(H + (int64_t)w * sH + (int64_t)b * ldh);
    const u32x4* wr = reinterpret_cast<const u32x4*>(Wq + (int64_t)w * sW + (int64_t)o * din);
    float acc = 0.f;
    for (int c = lane; c < din / 8; c += 64) {
        float a[8], q[8];
        unpack8(h[c], a); unpack8(wr[c], q);
#pragma unroll
        for (int t = 0; t < 8; ++t) acc = fmaf(a[t], q[t], acc);
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) acc += __shfl_xor(acc, d, 64);
    if (lane == 0) {
        const float z = acc + bias[(int64_t)w * sBias + o];
        if (HIDDEN) out[(int64_t)w * sOut + (int64_t)b * ldout + o] = f32_to_bf16_rne(z > 0.f ? z : 0.f);
        else logits[(int64_t)w * sOut + (int64_t)b * ldout + o] = z;
    }
}

// Bias gradients of all layers in one launch: db_k[o] = sum_b deltaT_k[o][b] with 16-byte loads, half a
// wavefront per output, eight outputs per workgroup.  B % 8 == 0, rows 16-byte aligned.
struct BiasLayers {
    int n;                    // layers
    int first_block[65];      // workgroups of layer i: first_block[i] .. first_block[i+1]
    int dout[64];
    int64_t dT[64];           // delta^T of the layer, element offset in a worker's scratch
    int64_t col[64];          // column of the layer's bias in the parameter row
};

__global__ __launch_bounds__(256) void db_all_kernel(const uint16_t* __restrict__ scratch, int64_t sD, int B, BiasLayers t,
                                                     float* __restrict__ g, int64_t sG, FusedUpdate fu)
{
    int layer = 0;
    while (layer + 1 < t.n && (int)blockIdx.x >= t.first_block[layer + 1]) ++layer;   // uniform
    const int lane = threadIdx.x & 63, l = lane & 31;
    const int o = (((int)blockIdx.x - t.first_block[layer]) * 4 + (threadIdx.x >> 6)) * 2 + (lane >> 5);
    const int w = blockIdx.y;
    const int dout = t.dout[layer];
    float acc = 0.f;
    if (o < dout) {
        const u32x4* dt = reinterpret_cast<const u32x4*>(scratch + (int64_t)w * sD + t.dT[layer] + (int64_t)o * B);
        for (int c = l; c < B / 8; c += 32) {
            float a[8];
            unpack8(dt[c], a);
#pragma unroll
            for (int q = 0; q < 8; ++q) acc += a[q];
        }
    }
#pragma unroll
    for (int d = 1; d < 32; d <<= 1) acc += __shfl_xor(acc, d, 64);
    if (l == 0 && o < dout) {
        const int64_t col = t.col[layer] + o;
        if (fu.enabled) {
            const int off[1] = {0};
            const float gv[1] = {acc};
            fused_apply<1>(fused_row(fu, w, sG), col, off, gv);
        } else {
            g[(int64_t)w * sG + col] = acc;
        }
    }
}

// dW[o][i..i+7] for one output row o and 512 columns per workgroup; the four wavefronts split the batch
// and combine through LDS in a fixed order.  d_in % 8 == 0.
__global__ __launch_bounds__(256) void dw_narrow_kernel(const uint16_t* __restrict__ deltaT, int64_t sD, const uint16_t* __restrict__ H,
                                                        int64_t sH, int64_t ldh, int B, int din, int dout, float* __restrict__ g, int64_t sG,
                                                        FusedUpdate fu, int64_t col0)
{
    const int w = blockIdx.z, o = blockIdx.y;
    const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + lane;            // 16-byte chunk (8 columns)
    const bool live = c < din / 8;
    const uint16_t* dt = deltaT + (int64_t)w * sD + (int64_t)o * B;
    const uint16_t* h = H + (int64_t)w * sH;
    float acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[t] = 0.f;
    const int b0 = (int)((int64_t)B * q / 4), b1 = (int)((int64_t)B * (q + 1) / 4);
    if (live) {
        int b = b0;
        for (; b + 8 <= b1; b += 8) {                     // eight rows of h in flight
            u32x4 hv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) hv[u] = *reinterpret_cast<const u32x4*>(h + (int64_t)(b + u) * ldh + (int64_t)c * 8);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float d = bf16_to_f32(dt[b + u]);
                float a[8];
                unpack8(hv[u], a);
#pragma unroll
                for (int t = 0; t < 8; ++t) acc[t] = fmaf(d, a[t], acc[t]);
            }
        }
        for (; b < b1; ++b) {
            const float d = bf16_to_f32(dt[b]);
            float a[8];
            unpack8(*reinterpret_cast<const u32x4*>(h + (int64_t)b * ldh + (int64_t)c * 8), a);
#pragma unroll
            for (int t = 0; t < 8; ++t) acc[t] = fmaf(d, a[t], acc[t]);
        }
    }
    __shared__ float red[4][64][9];
#pragma unroll
    for (int t = 0; t < 8; ++t) red[q][lane][t] = acc[t];
    __syncthreads();
    if (q == 0 && live) {
        float sum[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) sum[t] = ((red[0][lane][t] + red[1][lane][t]) + red[2][lane][t]) + red[3][lane][t];
        if (fu.enabled) {
            const int off[8] = {0, 1, 2, 3, 4, 5, 6, 7};
            fused_apply<8>(fused_row(fu, w, sG), col0 + (int64_t)o * din + (int64_t)c * 8, off, sum);
        } else {
            float* dst = g + (int64_t)w * sG + (int64_t)o * din + (int64_t)c * 8;
#pragma unroll
            for (int t = 0; t < 8; ++t) dst[t] = sum[t];
        }
    }
}

// dprev[b][i..i+7] = bf16(sum_o delta[b][o] Wq[o][i..i+7]) .* [h > 0] for a narrow delta (few classes).
// A workgroup owns 64 samples x 64 columns: thread (b, 8-column chunk).  The row-major result is
// stored directly (128 contiguous bytes per sample); the transposed copy goes through an LDS tile so
// that it too leaves as 128-byte runs (64 samples of one column).
__global__ __launch_bounds__(512) void dx_narrow_kernel(const uint16_t* __restrict__ delta, int64_t sD, const uint16_t* __restrict__ Wq, int64_t sW,
                                                        const uint16_t* __restrict__ H, int64_t sH, int64_t ldh, int B, int din, int dout,
                                                        uint16_t* __restrict__ dprev, uint16_t* __restrict__ dprevT, int64_t sP)
{
    constexpr int kLd = 72;                                   // padded tile row (bf16), 144 B
    __shared__ __attribute__((aligned(16))) uint16_t tile[64 * kLd];   // [column][sample]
    const int w = blockIdx.z;
    const int t = threadIdx.x, cl = t & 7, bl = t >> 3;
    const int b = blockIdx.y * 64 + bl;
    const int c = blockIdx.x * 8 + cl;                        // 16-byte chunk = 8 columns
    const bool live = b < B && c < din / 8;
    uint32_t pk[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) pk[q] = 0;
    if (live) {
        const uint16_t* d = delta + (int64_t)w * sD + (int64_t)b * dout;
        const uint16_t* Wm = Wq + (int64_t)w * sW + (int64_t)c * 8;
        float acc[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[q] = 0.f;
        for (int o = 0; o < dout; ++o) {
            const float dv = bf16_to_f32(d[o]);
            float a[8];
            unpack8(*reinterpret_cast<const u32x4*>(Wm + (int64_t)o * din), a);
#pragma unroll
            for (int q = 0; q < 8; ++q) acc[q] = fmaf(dv, a[q], acc[q]);
        }
        const u32x4 hm = *reinterpret_cast<const u32x4*>(H + (int64_t)w * sH + (int64_t)b * ldh + (int64_t)c * 8);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const uint32_t hb = (q & 1) ? (hm[q >> 1] >> 16) : (hm[q >> 1] & 0xFFFFu);
            pk[q] = hb ? (uint32_t)f32_to_bf16_rne(acc[q]) : 0u;
        }
        u32x4 o4 = {pk[0] | (pk[1] << 16), pk[2] | (pk[3] << 16), pk[4] | (pk[5] << 16), pk[6] | (pk[7] << 16)};
        *reinterpret_cast<u32x4*>(dprev + (int64_t)w * sP + (int64_t)b * din + (int64_t)c * 8) = o4;
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) tile[(cl * 8 + q) * kLd + bl] = (uint16_t)pk[q];
    __syncthreads();
    // thread (column il, 8-sample chunk): 16 bytes of the transposed copy
    const int il = t >> 3, bc = t & 7;
    const int col = blockIdx.x * 64 + il;
    const int b0 = blockIdx.y * 64 + bc * 8;
    if (col < din && b0 < B) {
        uint16_t* dst = dprevT + (int64_t)w * sP + (int64_t)col * B + b0;
        const uint16_t* src = tile + il * kLd + bc * 8;
        if (b0 + 8 <= B && (B & 7) == 0) {
            *reinterpret_cast<u32x4*>(dst) = *reinterpret_cast<const u32x4*>(src);
        } else {
            for (int q = 0; q < 8 && b0 + q < B; ++q) dst[q] = src[q];
        }
    }
}

// h_0 = bf16(X) for fp32 inputs: n values per worker, rounded to nearest even
__global__ __launch_bounds__(256) void cast_input_kernel(const float* __restrict__ X, int64_t n, uint16_t* __restrict__ out, int64_t sOut)
{
    const int w = blockIdx.y;
    const float* src = X + (int64_t)w * n;
    uint16_t* dst = out + (int64_t)w * sOut;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) dst[i] = f32_to_bf16_rne(src[i]);
}

__global__ __launch_bounds__(256) void zero_pad_kernel(float* __restrict__ g, int64_t P, int64_t ld)
{
    const int64_t c = P + (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (c < ld) g[(int64_t)blockIdx.y * ld + c] = 0.f;
}

// ------------------------------------------------------------------------------------------
// Host orchestration
// ------------------------------------------------------------------------------------------
namespace {

struct MlpPlan {
    int L;
    std::size_t bytes;
    // per-worker element offsets inside the scratch (bf16 elements unless noted)
    int64_t h[64];      // h[k], k = 1..L-1  [B][d_k]
    int64_t d[64];      // delta[k], k = 1..L [B][d_k]
    int64_t dT[64];     // delta^T[k]         [d_k][B]
    int64_t logits;     // fp32 [B][C], offset in bytes from the worker's base
    int64_t x0;         // bf16 copy of fp32 inputs [B][d_0] (only when the batch brings fp32 inputs)
    int64_t per_worker; // bytes per worker
};

inline int64_t up16(int64_t v) { return (v + 15) / 16 * 16; }

MlpPlan make_plan(const lsgd_mlp_batch& b, int W)
{
    MlpPlan p{};
    p.L = b.n_layers;
    int64_t o = 0; // bytes
    for (int k = 1; k <= p.L; ++k) {
        const int64_t n = (int64_t)b.B * b.dims[k] * 2;
        if (k < p.L) { p.h[k] = o / 2; o = up16(o + n); }
        p.d[k] = o / 2; o = up16(o + n);
        p.dT[k] = o / 2; o = up16(o + n);
    }
    p.logits = o; o = up16(o + (int64_t)b.B * b.dims[p.L] * 4);
    if (b.x_is_fp32) { p.x0 = o / 2; o = up16(o + (int64_t)b.B * b.dims[0] * 2); }
    p.per_worker = (o + 255) / 256 * 256;
    p.bytes = (std::size_t)p.per_worker * (std::size_t)W;
    return p;
}

} // namespace

bool mlp_shape_supported(const lsgd_mlp_batch& b, const char** why)
{
    if (b.n_layers > 60) { *why = "more than 60 layers"; return false; }
    if (b.dims[b.n_layers] > 4096) { *why = "more than 4096 classes"; return false; }
    return true;
}

size_t mlp_scratch_bytes(int W, const lsgd_mlp_batch& b) { return make_plan(b, W).bytes; }

hipError_t launch_mlp_grad_loss(const uint16_t* xb, const float* x, float* g, float* losses, int W, int64_t P,
                                int64_t ld, const lsgd_mlp_batch& b, const DeviceState& st, hipStream_t s)
{
    hipError_t e = launch_mlp_forward(xb, x, losses, W, P, ld, b, st, s);
    if (e != hipSuccess) return e;
    return launch_mlp_backward(xb, x, g, W, P, ld, b, st, nullptr, s);
}

hipError_t launch_mlp_forward(const uint16_t* xb, const float* x, float* losses, int W, int64_t P, int64_t ld,
                              const lsgd_mlp_batch& b, const DeviceState& st, hipStream_t s)
{
    const MlpPlan p = make_plan(b, W);
    const int L = p.L, B = b.B;
    uint16_t* sc16 = reinterpret_cast<uint16_t*>(st.scratch);
    const int64_t sW16 = p.per_worker / 2;     // per-worker stride in bf16 elements
    const int64_t sW32 = p.per_worker / 4;     // ... in fp32 elements
    float* logits = reinterpret_cast<float*>(st.scratch + p.logits);

    int64_t woff[64];
    { int64_t o = 0; for (int k = 1; k <= L; ++k) { woff[k] = o; o += (int64_t)b.dims[k] * b.dims[k - 1] + b.dims[k]; } }

    // ---- forward ----
    const uint16_t* X0 = static_cast<const uint16_t*>(b.X);
    int64_t sX0 = (int64_t)B * b.dims[0];
    if (b.x_is_fp32) {                                     // the bf16 copy both passes read
        const int64_t n = (int64_t)B * b.dims[0];
        int64_t blocks = (n + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(cast_input_kernel, dim3((unsigned)blocks, (unsigned)W), dim3(256), 0, s, static_cast<const float*>(b.X), n,
                           sc16 + p.x0, sW16);
        X0 = sc16 + p.x0; sX0 = sW16;
    }
    for (int k = 1; k <= L; ++k) {
        const int din = b.dims[k - 1], dout = b.dims[k];
        const uint16_t* Hin = (k == 1) ? X0 : sc16 + p.h[k - 1];
        const int64_t sHin = (k == 1) ? sX0 : sW16;
        const float* bias = x + woff[k] + (int64_t)dout * din;
        bool done = false;
        if (k < L) {
            GemmArgs a{};
            a.A = Hin; a.sA = sHin; a.lda = din;
            a.B = xb + woff[k]; a.sB = ld; a.ldb = din;
            a.M = B; a.N = dout; a.K = din;
            a.bias = bias; a.sBias = ld;
            a.out = sc16 + p.h[k]; a.sOut = sW16; a.ldout = dout;
            done = try_mfma<false, EPI_FWD>(a, W, s);
        }
        auto a16 = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
        const bool vec8 = din % 8 == 0 && ld % 8 == 0 && woff[k] % 8 == 0 && a16(xb) && a16(Hin) && sHin % 8 == 0;
        if (!done && vec8 && dout <= 64) {
            dim3 grid((unsigned)(((int64_t)B * dout + 3) / 4), (unsigned)W);
            if (k < L)
                hipLaunchKernelGGL(fwd_narrow_kernel<true>, grid, dim3(256), 0, s, Hin, sHin, (int64_t)din, xb + woff[k], ld, bias, ld,
                                   B, din, dout, sc16 + p.h[k], (float*)nullptr, sW16, (int64_t)dout);
            else
                hipLaunchKernelGGL(fwd_narrow_kernel<false>, grid, dim3(256), 0, s, Hin, sHin, (int64_t)din, xb + woff[k], ld, bias, ld,
                                   B, din, dout, (uint16_t*)nullptr, logits, sW32, (int64_t)dout);
            done = true;
        }
        if (!done) {
            dim3 grid((unsigned)((B + 3) / 4), (unsigned)W);
            if (k < L)
                hipLaunchKernelGGL(fwd_valu_kernel<true>, grid, dim3(256), 0, s, Hin, sHin, (int64_t)din, xb + woff[k], ld, bias, ld,
                                   B, din, dout, sc16 + p.h[k], (float*)nullptr, sW16, (int64_t)dout);
            else
                hipLaunchKernelGGL(fwd_valu_kernel<false>, grid, dim3(256), 0, s, Hin, sHin, (int64_t)din, xb + woff[k], ld, bias, ld,
                                   B, din, dout, (uint16_t*)nullptr, logits, sW32, (int64_t)dout);
        }
    }
    // ---- loss and output delta ----
    hipLaunchKernelGGL(loss_delta_kernel, dim3((unsigned)W), dim3(256), 0, s, logits, sW32, b.y, B, b.dims[L],
                       sc16 + p.d[L], sc16 + p.dT[L], sW16, losses);
    return hipGetLastError();
}

// Backward pass.  Per layer, from the top: delta_{k-1} first (it reads W_k, which the fused update
// of dW_k overwrites), then dW_k and db_k.
hipError_t launch_mlp_backward(const uint16_t* xb, const float* x, float* g, int W, int64_t P, int64_t ld,
                               const lsgd_mlp_batch& b, const DeviceState& st, const FusedUpdate* fu_in, hipStream_t s)
{
    const MlpPlan p = make_plan(b, W);
    const int L = p.L, B = b.B;
    uint16_t* sc16 = reinterpret_cast<uint16_t*>(st.scratch);
    const int64_t sW16 = p.per_worker / 2;     // per-worker stride in bf16 elements
    FusedUpdate fu{};
    if (fu_in) fu = *fu_in;
    const bool fused = fu.enabled != 0;

    int64_t woff[64];
    { int64_t o = 0; for (int k = 1; k <= L; ++k) { woff[k] = o; o += (int64_t)b.dims[k] * b.dims[k - 1] + b.dims[k]; } }

    // fp32 inputs: the forward pass of this step left their bf16 copy in the scratch
    const uint16_t* X0 = b.x_is_fp32 ? sc16 + p.x0 : static_cast<const uint16_t*>(b.X);
    const int64_t sX0 = b.x_is_fp32 ? sW16 : (int64_t)B * b.dims[0];
    for (int k = L; k >= 1; --k) {
        const int din = b.dims[k - 1], dout = b.dims[k];
        const uint16_t* Hin = (k == 1) ? X0 : sc16 + p.h[k - 1];
        const int64_t sHin = (k == 1) ? sX0 : sW16;
        // delta_{k-1}
        if (k > 1) {
            GemmArgs a{};
            a.A = sc16 + p.d[k]; a.sA = sW16; a.lda = dout;
            a.B = xb + woff[k]; a.sB = ld; a.ldb = din;
            a.M = B; a.N = din; a.K = dout;
            a.mask = Hin; a.sMask = sHin; a.ldmask = din;
            a.out = sc16 + p.d[k - 1]; a.sOut = sW16; a.ldout = din;
            a.outT = sc16 + p.dT[k - 1]; a.sOutT = sW16; a.ldoutT = B;
            auto a16 = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
            const bool vec8 = din % 8 == 0 && ld % 8 == 0 && woff[k] % 8 == 0 && a16(xb) && a16(Hin) && sHin % 8 == 0;
            if (try_mfma<true, EPI_DX>(a, W, s)) {
            } else if (vec8 && dout <= 64) {
                dim3 grid((unsigned)((din / 8 + 7) / 8), (unsigned)((B + 63) / 64), (unsigned)W);
                hipLaunchKernelGGL(dx_narrow_kernel, grid, dim3(512), 0, s, sc16 + p.d[k], sW16, xb + woff[k], ld, Hin, sHin,
                                   (int64_t)din, B, din, dout, sc16 + p.d[k - 1], sc16 + p.dT[k - 1], sW16);
            } else {
                dim3 grid((unsigned)((din + 255) / 256), (unsigned)B, (unsigned)W);
                hipLaunchKernelGGL(dx_valu_kernel, grid, dim3(256), 0, s, sc16 + p.d[k], sW16, xb + woff[k], ld, Hin, sHin,
                                   (int64_t)din, B, din, dout, sc16 + p.d[k - 1], sc16 + p.dT[k - 1], sW16);
            }
        }
        // dW_k
        {
            GemmArgs a{};
            a.A = sc16 + p.dT[k]; a.sA = sW16; a.lda = B;
            a.B = Hin; a.sB = sHin; a.ldb = din;
            a.M = dout; a.N = din; a.K = B;
            a.C = g + woff[k]; a.sC = ld; a.ldc = din;
            a.fu = fu; a.colC = woff[k];
            auto a16 = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
            const bool vec8 = din % 8 == 0 && a16(Hin) && sHin % 8 == 0;
            if (fused ? try_mfma<true, EPI_DWU>(a, W, s) : try_mfma<true, EPI_DW>(a, W, s)) {
            } else if (vec8 && dout <= 64) {
                dim3 grid((unsigned)((din / 8 + 63) / 64), (unsigned)dout, (unsigned)W);
                hipLaunchKernelGGL(dw_narrow_kernel, grid, dim3(256), 0, s, sc16 + p.dT[k], sW16, Hin, sHin, (int64_t)din, B, din,
                                   dout, g + woff[k], ld, fu, woff[k]);
            } else {
                dim3 grid((unsigned)((din + 255) / 256), (unsigned)dout, (unsigned)W);
                hipLaunchKernelGGL(dw_valu_kernel, grid, dim3(256), 0, s, sc16 + p.dT[k], sW16, Hin, sHin, (int64_t)din, B, din,
                                   dout, g + woff[k], ld, fu, woff[k]);
            }
        }
    }
    // db_k of every layer (delta^T_k is complete once layer k+1 has been processed; the biases' columns
    // are nobody else's): one launch when the rows allow 16-byte loads, else one per layer
    if (B % 8 == 0 && sW16 % 8 == 0 && (reinterpret_cast<uintptr_t>(sc16) & 15u) == 0) {
        BiasLayers t{};
        t.n = L;
        int blocks = 0;
        for (int k = 1; k <= L; ++k) {
            t.first_block[k - 1] = blocks;
            t.dout[k - 1] = b.dims[k];
            t.dT[k - 1] = p.dT[k];
            t.col[k - 1] = woff[k] + (int64_t)b.dims[k] * b.dims[k - 1];
            blocks += (b.dims[k] + 7) / 8;
        }
        t.first_block[L] = blocks;
        hipLaunchKernelGGL(db_all_kernel, dim3((unsigned)blocks, (unsigned)W), dim3(256), 0, s, sc16, sW16, B, t, g, ld, fu);
    } else {
        for (int k = L; k >= 1; --k) {
            const int din = b.dims[k - 1], dout = b.dims[k];
            hipLaunchKernelGGL(db_kernel, dim3((unsigned)((dout + 3) / 4), (unsigned)W), dim3(256), 0, s, sc16 + p.dT[k], sW16, B, dout,
                               g + woff[k] + (int64_t)dout * din, ld, fu, woff[k] + (int64_t)dout * din);
        }
    }
    if (fused) return hipGetLastError();          // g is not written, so there is no padding to clear
    if (ld > P)
        hipLaunchKernelGGL(zero_pad_kernel, dim3((unsigned)((ld - P + 255) / 256), (unsigned)W), dim3(256), 0, s, g, P, ld);
    return hipGetLastError();
}

} // namespace lsgd
