/*
 * lsgd.h - C boundary of the batched Leader-SGD step for one AMD MI355X (gfx950).
 *
 * A population of W workers lives on one GPU as a row-major fp32 matrix
 * x[W, ld] (row i = parameters of worker i, P <= ld used columns).  Workers are
 * partitioned into n contiguous groups (Eq. 2 of arXiv 1905.10395: n groups of
 * l workers, each with a local leader, plus one global leader).  One step is
 *
 *   1. lsgd_grad_loss       g_i, loss_i of every worker on its own minibatch
 *                           (Section 2: stochastic gradient g_t^{j,i}; Section
 *                           3.1.3: one loss sample per worker)
 *   2. lsgd_select_leaders  segmented argmin of the losses (Eq. 1 / Eq. 2;
 *                           the leader-picking steps of Algorithm 1)
 *   3. lsgd_pull_update     x_i <- x_i - eta*(g_i + lam_L (x_i - z_local)
 *                                              + lam_G (x_i - z_global))
 *                           (supplement B.1; Eq. 3), optional momentum
 *   lsgd_step               1-3 on the population's stream, no host sync.
 *
 * General rules
 *   - Pointers marked "device" are device memory owned by the caller for the
 *     life of the handle; the library never allocates, frees or resizes them.
 *     Pointers marked "host" are read during the call only.
 *   - Every call validates its arguments first; a failing call enqueues no
 *     device work.  Calls return an lsgd_status and never abort or throw;
 *     lsgd_last_error() gives a message for the last failure on this thread.
 *   - All device work is enqueued on the stream given at creation.  Only
 *     lsgd_get_leaders / lsgd_get_losses synchronise that stream.
 *   - Worker indices returned are global, in [0, W).
 */
#ifndef LSGD_H
#define LSGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lsgd_population lsgd_population; /* opaque host object */

typedef enum {
    LSGD_OK = 0,
    LSGD_ERR_INVALID_ARG = 1, /* NULL where a pointer is required, bad enum, non-finite scalar */
    LSGD_ERR_SHAPE = 2,       /* W<=0, ld<P, offsets not covering [0,W], sizes not matching P  */
    LSGD_ERR_STATE = 3,       /* call order: pull with lam>0 before any selection, missing buffer */
    LSGD_ERR_UNSUPPORTED = 4, /* shape outside what the kernels implement                       */
    LSGD_ERR_HIP = 5,         /* a HIP runtime call failed                                      */
    LSGD_ERR_NOMEM = 6        /* workspace too small / host allocation failed                   */
} lsgd_status;

/* lsgd_config.flags */
enum {
    LSGD_NESTEROV = 1,            /* x <- x - eta*(d + mu*m) instead of x <- x - eta*m            */
    LSGD_LEADER_EXEMPT = 2,       /* a leader is not pulled to a (stale) copy of itself:
                                     supplement, lemma on leader descent                          */
    LSGD_PULL_UNSCALED_BY_ETA = 4,/* Eq. 3 as printed: pulls are not multiplied by eta            */
    LSGD_MOMENTUM_GRAD_ONLY = 8,  /* momentum buffer accumulates g only; pulls applied outside it */
    LSGD_WRITE_BF16_SHADOW = 16,  /* pull_update also writes bf16(x) to x_bf16 (MLP operands)     */
    LSGD_FUSED_MLP_UPDATE = 32    /* lsgd_step on LSGD_BATCH_MLP applies the update inside the
                                     backward kernels (the gradient never goes through memory):
                                     g is not written and holds unspecified values afterwards,
                                     x_bf16 is always kept current.  Same results as the
                                     three-call sequence up to fp32 rounding.  Needs z_snapshot
                                     when a lambda is non-zero.  Other batch kinds and the
                                     separate calls are unaffected.                              */
};

#define LSGD_MAX_WORKERS 32768
#define LSGD_MAX_GROUPS 1024

typedef struct {
    int32_t W;                    /* workers = rows                                              */
    int64_t P;                    /* parameters per worker                                       */
    int64_t ld;                   /* row stride in elements, ld >= P                             */
    int32_t n_groups;             /* n of Eq. 2                                                  */
    const int32_t* group_offsets; /* host [n_groups+1], strictly increasing, [0]=0, [n]=W;
                                     NULL: W % n_groups == 0 and equal contiguous groups          */
    float momentum;               /* mu; 0 disables the momentum buffer                          */
    int32_t flags;                /* LSGD_* bits above                                           */
    float weight_decay;           /* g <- g + wd*x inside the update; 0 = none                   */
} lsgd_config;

/* ---- minibatch descriptors (host structs; the arrays they point to are device memory) ---- */
typedef enum { LSGD_BATCH_EXTERNAL = 0, LSGD_BATCH_MC = 1, LSGD_BATCH_MLP = 2 } lsgd_batch_kind;

/* Gradient and losses were produced by the caller: g (given at creation) is
 * already filled; losses is device [W].                                        */
typedef struct {
    const float* losses; /* device [W] */
} lsgd_external_batch;

/* Low-rank matrix completion on observed entries (the problem family of the
 * paper's motivating example and supplement, rectangular form).  Worker row =
 * [U (m x r, row-major) | V (n x r, row-major)], P = (m+n)*r.  For each batch
 * entry k = (a_k, b_k, M_k): e_k = <U[a_k],V[b_k]> - M_k;
 * loss = c*sum e_k^2; dU[a] = 2c*sum_{a_k=a} e_k V[b_k]; dV[b] likewise.
 * Entries drawn more than once count each time.                                */
typedef struct {
    int32_t row, col; /* a, b                                                       */
    float val;        /* M_ab                                                       */
    int32_t reserved; /* keeps the record at 16 bytes                               */
} lsgd_mc_entry;

typedef struct {
    int32_t m, n, r;
    const int32_t* rows;      /* device [n_obs] row index a of each observed entry  */
    const int32_t* cols;      /* device [n_obs] column index b                      */
    const float* vals;        /* device [n_obs] observed value M_ab                 */
    int64_t n_obs;
    const int32_t* batch_idx; /* device [W, B] indices into the observed list, or
                                 NULL: every worker uses all n_obs entries (batch
                                 gradient, "LGD")                                   */
    int64_t B;                /* entries per worker when batch_idx != NULL          */
    float c;                  /* loss normalisation                                 */
    const lsgd_mc_entry* entries; /* device [n_obs], optional: the same observed list with
                                 one 16-byte record per entry (see lsgd_mc_pack_entries).
                                 When non-NULL it is read instead of rows/cols/vals:
                                 one random access per batch element instead of three */
} lsgd_mc_batch;

/* Fully connected ReLU classifier with softmax cross-entropy, mean over the
 * batch.  Worker row = [W_1 (d1 x d0 row-major) | b_1 | W_2 | b_2 | ...].
 * Matrix operands (inputs, weights, stored activations, back-propagated
 * deltas) are bf16, accumulation and everything else fp32.                     */
typedef struct {
    int32_t n_layers;    /* number of weight matrices                              */
    const int32_t* dims; /* host [n_layers+1]: d0 (input) ... d_L (classes)        */
    const void* X;       /* device [W, B, d0]: bf16 bit patterns (uint16), or fp32
                            values when x_is_fp32 (rounded to bf16, to nearest even,
                            on the way in: a copy in the workspace)                */
    const int32_t* y;    /* device [W, B] class labels in [0, d_L)                 */
    int32_t B;           /* samples per worker                                     */
    int32_t x_is_fp32;   /* 0: X holds bf16 bit patterns; 1: X holds fp32 values   */
} lsgd_mlp_batch;

typedef struct {
    int32_t kind;     /* lsgd_batch_kind                                            */
    const void* desc; /* host pointer to the matching struct above                  */
} lsgd_batch;

/* Bytes of device workspace lsgd_create_population needs for this population
 * and for gradient calls shaped like `largest` (NULL: selection and update
 * only).  Returns 0 on invalid arguments (see lsgd_last_error).               */
size_t lsgd_workspace_bytes(const lsgd_config* cfg, const lsgd_batch* largest);

/* Binds caller-owned device buffers into a population handle.
 *   x, g       device [W, ld] fp32, required
 *   m          device [W, ld] fp32, required iff cfg->momentum != 0; the caller zeroes it
 *   z_snapshot device [(n_groups+1), ld] fp32 leader copies kept between
 *              communications (Algorithm 1; supplement B.1).  NULL is allowed
 *              when every update follows a full refresh.
 *   x_bf16     device [W, ld] bf16, required for LSGD_BATCH_MLP and for
 *              LSGD_WRITE_BF16_SHADOW, else NULL
 *   workspace  device, >= lsgd_workspace_bytes(...), 256-byte aligned
 *   hip_stream a hipStream_t (NULL = default stream)
 * The fast update path needs x, g, m, z_snapshot 16-byte aligned and ld % 4 == 0;
 * other layouts take a scalar path.                                            */
lsgd_status lsgd_create_population(const lsgd_config* cfg, float* x, float* g, float* m,
                                   float* z_snapshot, uint16_t* x_bf16, void* workspace,
                                   size_t workspace_bytes, void* hip_stream,
                                   lsgd_population** out);

/* Frees the host object only. */
lsgd_status lsgd_destroy_population(lsgd_population* pop);

/* Writes g[W, ld] (unused padding columns zeroed) and losses (device [W]; NULL =
 * the population's own loss buffer, the one lsgd_step uses).  For
 * LSGD_BATCH_EXTERNAL copies the given losses into the population's buffer when
 * `losses` is NULL, otherwise into `losses`.                                   */
lsgd_status lsgd_grad_loss(lsgd_population* pop, const lsgd_batch* batch, float* losses);

/* Objective values only: losses[i] = f_i(x_i) on worker i's part of the batch at
 * the current parameters (device [W]; NULL = the population's own loss buffer);
 * g is neither read nor written.  This is what choosing a leader costs (Section
 * 3.1.3: the leader is the worker whose estimate of the objective, one draw per
 * worker, is smallest; Algorithm 1 determines the best workers after the local
 * step, at the parameters that step produced, on the sample of the iteration
 * that follows).  lsgd_step and
 * lsgd_step_alg1 select from the losses of their own gradient pass, i.e. at the
 * parameters before the step; the printed order is
 *   lsgd_step_alg1(..., comm = 0); lsgd_loss(next batch, NULL);
 *   lsgd_select_leaders(NULL, mask, global); lsgd_leader_pull(lambda, lambda_G).
 * Same batch kinds, checks and workspace as lsgd_grad_loss.  For LSGD_BATCH_MC
 * the squared residuals are summed in another order than in lsgd_grad_loss, so
 * the two values can differ in the last bits; for LSGD_BATCH_MLP it is the
 * forward pass of lsgd_grad_loss (bit-identical losses).                        */
lsgd_status lsgd_loss(lsgd_population* pop, const lsgd_batch* batch, float* losses);

/* Segmented argmin.  For each group j with refresh_local[j] != 0 (host
 * [n_groups]; NULL = all) the local leader becomes the lowest index attaining the
 * group's minimum loss; if refresh_global the global leader becomes the lowest
 * index attaining the minimum over all workers.  NaN counts as +infinity.  The
 * leaders refreshed here are captured (copied from x before any row changes) by
 * the next lsgd_pull_update; the others keep their stored copies.
 * losses: device [W]; NULL = the population's own buffer (LSGD_ERR_STATE if
 * nothing has written it yet).                                                  */
lsgd_status lsgd_select_leaders(lsgd_population* pop, const float* losses,
                                const uint8_t* refresh_local, int refresh_global);

/* d = g + wd*x + lam_L (x - z_local) + lam_G (x - z_global);
 * mu = 0: x <- x - eta*d;  mu > 0: m <- mu*m + d, x <- x - eta*m (flags modify).
 * In place on x and m; every row is computed from pre-update values.  A term
 * whose coefficient is exactly 0 is skipped and its leader copy is neither read
 * nor written.  LSGD_ERR_STATE if a needed leader was never selected, or a kept
 * copy is needed and z_snapshot is NULL.  A leader re-selected since the last
 * update whose coefficient is 0 in this call is not captured; its kept copy is
 * then no longer valid (LSGD_ERR_STATE for a later update that would need it
 * before the next selection).                                                   */
lsgd_status lsgd_pull_update(lsgd_population* pop, float eta, float lambda_L, float lambda_G);

/* grad_loss -> select_leaders -> pull_update with the population's own loss
 * buffer.  The first step of a population must refresh everything.  With
 * LSGD_FUSED_MLP_UPDATE and an LSGD_BATCH_MLP batch the same three stages run as
 * forward pass + losses -> select_leaders -> kept copies brought up to date ->
 * backward pass that applies the update (see the flag); the state afterwards is
 * the same up to fp32 rounding, except that g is left unspecified.             */
lsgd_status lsgd_step(lsgd_population* pop, const lsgd_batch* batch, float eta, float lambda_L,
                      float lambda_G, const uint8_t* refresh_local, int refresh_global);

/* Communication pull of Algorithm 1 (its two blocks that pick the best
 * workers and move everyone towards them): captures every leader
 * re-selected since the last update (copied from x before any row changes, and
 * written to z_snapshot when it exists, also when its coefficient is 0), then
 *   groups whose local leader was re-selected:  x <- x - lambda_L (x - z_local)
 *   if the global leader was re-selected:        x <- x - lambda_G (x - z_global)
 * in that order, element-wise, with no gradient, learning rate or momentum
 * involved.  Groups (or the global term) with nothing re-selected are left
 * alone.  LSGD_ERR_STATE if nothing was re-selected since the last update.     */
lsgd_status lsgd_leader_pull(lsgd_population* pop, float lambda_L, float lambda_G);

/* lsgd_step_alg1.comm bits */
enum {
    LSGD_COMM_LOCAL = 1,  /* local communication at this step  (n l tau   divides the iteration count) */
    LSGD_COMM_GLOBAL = 2  /* global communication at this step (n l tau_G divides the iteration count) */
};

/* One iteration of Algorithm 1 for every worker at once:
 *   grad_loss;  x <- x - eta g - gamma_L (x - z_local) - gamma_G (x - z_global)
 *   with the kept leader copies (gamma_L = gamma/tau, gamma_G = gamma_G/tau_G,
 *   not multiplied by eta; momentum, weight decay and flags of the population
 *   apply to the gradient part as in lsgd_pull_update);
 *   then, when comm has LSGD_COMM_LOCAL / LSGD_COMM_GLOBAL: select_leaders from
 *   this iteration's losses (comm_local_mask: host [n_groups] choosing the
 *   groups that communicate, NULL = all) followed by lsgd_leader_pull.
 * Before the first iteration the caller initialises the leaders (the
 * initialisation block of Algorithm 1): grad_loss, select_leaders(all), lsgd_leader_pull(0, 0).
 * Needs z_snapshot.  eta must be non-zero when a gamma is.                      */
lsgd_status lsgd_step_alg1(lsgd_population* pop, const lsgd_batch* batch, float eta, float gamma_L,
                           float gamma_G, float lambda_L, float lambda_G, int comm,
                           const uint8_t* comm_local_mask);

/* Selection loss averaged over the last K minibatches (Section 4.1: leaders are
 * determined from the average training loss over the last 10 or 64 batches).
 *   window device [K, W] fp32 ring owned by the caller; slot t % K receives the
 *          new losses (no initialisation needed: only filled slots are read)
 *   t      0-based count of calls so far on this ring
 *   losses device [W] new losses; NULL = the population's own buffer
 *   out    device [W] mean over the min(t+1, K) newest slots, summed in slot
 *          order in double; NULL = the population's own buffer (so that a
 *          following lsgd_select_leaders(pop, NULL, ...) uses it); may alias losses. */
lsgd_status lsgd_smooth_losses(lsgd_population* pop, float* window, int32_t K, int64_t t,
                               const float* losses, float* out);

/* Center variable (Section 4.1: the model reported at test time is the average
 * of all workers' parameters): out[p] = (1/W) sum_i x[i, p], summed over i in
 * order in double and rounded once.  out: device [P] (16-byte aligned for the
 * fast path), must not overlap x.                                              */
lsgd_status lsgd_center(lsgd_population* pop, float* out);

/* Elastic averaging (EAGD / EASGD), the method the paper compares with, as a variant of the same update
 * (supplement, "Low-Rank Matrix Completion Experiments": both methods are X+ = (1 - eta lam) X + eta lam Z -
 * eta grad, with Z the leader for LGD and the center for EAGD):
 *   center+ = (1 - W eta lam) center + W eta lam * (1/W) sum_i x_i       (mean in double, rounded once)
 *   x_i+    = x_i - eta (g_i + lam (x_i - center))                        for every worker,
 * both from the values before the call; momentum, weight decay and the Nesterov / grad-only flags of the
 * population apply to the workers' step as in lsgd_pull_update; no leaders are involved.
 *   center device [ld] fp32 owned by the caller (16-byte aligned for the fast path), updated in place; the
 *          caller initialises it (the paper does not say how; e.g. with lsgd_center)
 * The pre-update center is kept in the global row of z_snapshot during the call, which therefore must exist
 * and afterwards no longer holds a global leader copy.  LSGD_ERR_STATE while a leader selection is pending.
 * lsgd_easgd_step = lsgd_grad_loss into the population's own buffers, then lsgd_easgd_update.            */
lsgd_status lsgd_easgd_update(lsgd_population* pop, float* center, float eta, float lambda);
lsgd_status lsgd_easgd_step(lsgd_population* pop, const lsgd_batch* batch, float* center, float eta, float lambda);

/* Builds the 16-byte-record form of an observed-entry list (device to device, on
 * hip_stream): out[k] = {rows[k], cols[k], vals[k], 0}.  The list of observed
 * entries is fixed across steps (the paper's M and its observed set), so this is
 * done once by the caller.  All pointers device, [n_obs].                          */
lsgd_status lsgd_mc_pack_entries(const int32_t* rows, const int32_t* cols, const float* vals,
                                 int64_t n_obs, lsgd_mc_entry* out, void* hip_stream);

/* Recomputes the whole bf16 shadow from x (after the caller changed x). */
lsgd_status lsgd_sync_shadow(lsgd_population* pop);

/* Synchronise the stream and read back.  local_leaders: host [n_groups];
 * global_leader: host [1]; either may be NULL.  Leaders never selected read -1. */
lsgd_status lsgd_get_leaders(lsgd_population* pop, int32_t* local_leaders, int32_t* global_leader);
/* Restores leader indices read earlier with lsgd_get_leaders (checkpoint / resume: the state of a run is
 * x, m, z_snapshot and these G+1 indices; x_bf16 is rebuilt from x by the next gradient call).  The rows of
 * z_snapshot are taken to be the copies that belong to these leaders, no re-selection is pending afterwards.
 * local_leaders: host [n_groups], each a row of its group or -1 (never selected); global_leader: a row or -1.
 * Synchronises the stream.                                                                                */
lsgd_status lsgd_set_leaders(lsgd_population* pop, const int32_t* local_leaders, int32_t global_leader);
/* losses_host: host [W], the population's own loss buffer. */
lsgd_status lsgd_get_losses(lsgd_population* pop, float* losses_host);

/* For callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  One leader selection over all groups and
 * the global leader followed by one pull update, i.e. what lsgd_step does for an
 * LSGD_BATCH_EXTERNAL batch with a full refresh, without a population handle or workspace:
 * the group table, leader indices and re-selection flags that the handle keeps in the
 * caller's workspace live in a static device array inside the library (38 KB per GPU, held
 * until the process ends), and the call itself allocates nothing on the host or the device.
 *   W <= LSGD_STATIC_MAX_WORKERS, n_groups <= LSGD_STATIC_MAX_GROUPS: larger shapes are
 *            rejected with LSGD_ERR_SHAPE
 *   group_offsets host [n_groups+1] or NULL (equal groups), as in lsgd_config
 *   x, g, m  device [W, ld] fp32 as in lsgd_create_population (m may be NULL when
 *            momentum == 0); updated in place exactly as lsgd_pull_update does
 *   losses   device [W]
 *   leaders  device [n_groups+1] int32 or NULL: receives the local leaders and, last, the
 *            global leader
 *   flags    LSGD_NESTEROV | LSGD_LEADER_EXEMPT | LSGD_PULL_UNSCALED_BY_ETA |
 *            LSGD_MOMENTUM_GRAD_ONLY
 * Every leader is re-selected at every call, so no leader copies are kept.  Work is enqueued
 * on hip_stream of the current device; nothing synchronises.  All calls on one GPU share
 * that GPU's array: calls that may overlap there (different streams, different threads)
 * race and must be ordered by the caller.  Every word a call reads it writes first, so the
 * contents left by an earlier call never matter.                                          */
#define LSGD_STATIC_MAX_WORKERS 1024
#define LSGD_STATIC_MAX_GROUPS 64
lsgd_status lsgd_select_pull_static(int32_t W, int64_t P, int64_t ld, int32_t n_groups,
                                    const int32_t* group_offsets, float* x, const float* g, float* m,
                                    const float* losses, int32_t* leaders, float eta, float lambda_L,
                                    float lambda_G, float momentum, float weight_decay, int32_t flags,
                                    void* hip_stream);

/* Measurement aid, not part of the method: one pass of a plain stream over n floats per buffer, in
 * memory order, so that a benchmark can report what the memory system at hand gives the access
 * shapes the update uses, beside the update's own rate.
 *   LSGD_PROBE_READ    reads a                              (4 n bytes)
 *   LSGD_PROBE_COPY    b <- a                               (8 n bytes)
 *   LSGD_PROBE_UPDATE  c <- 0.9 c + b ; a <- a - 1e-3 c     (20 n bytes: the momentum update without
 *                      leader rows, 3 reads and 2 writes per element)
 * a, b, c: device [n] fp32, 8-byte aligned, n even (c may be NULL except for LSGD_PROBE_UPDATE).     */
enum { LSGD_PROBE_READ = 0, LSGD_PROBE_COPY = 1, LSGD_PROBE_UPDATE = 2 };
lsgd_status lsgd_stream_probe(int32_t kind, float* a, float* b, float* c, int64_t n, void* hip_stream);

/* Message for the last failing call on this thread ("" if none).  Static storage. */
const char* lsgd_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LSGD_H */
