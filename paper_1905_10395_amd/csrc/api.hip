// Host side of the C boundary declared in lsgd.h: argument validation, the
// population object, workspace carving and kernel dispatch.  No arithmetic of
// the method lives here.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "common.h"

using namespace lsgd;

namespace {
thread_local char g_err[512] = "";
}

namespace lsgd {
lsgd_status set_error(lsgd_status st, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}
} // namespace lsgd

namespace {

#define fail(...) lsgd::set_error(__VA_ARGS__)

constexpr size_t kAlign = 256;
size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Layout {
    size_t lead, glead, refreshed, offsets, group_of, plan, losses, partials, scratch, total;
    size_t partials_cap, scratch_bytes;
};

Layout make_layout(int W, int G, size_t partials_cap, size_t scratch_bytes)
{
    Layout L;
    size_t o = 0;
    L.lead = o;      o = align_up(o + sizeof(int32_t) * (size_t)G);
    L.glead = o;     o = align_up(o + sizeof(int32_t));
    L.refreshed = o; o = align_up(o + sizeof(int32_t) * (size_t)(G + 1));
    L.offsets = o;   o = align_up(o + sizeof(int32_t) * (size_t)(G + 1));
    L.group_of = o;  o = align_up(o + sizeof(int32_t) * (size_t)W);
    L.plan = o;      o = align_up(o + sizeof(RowPlan) * (size_t)W);
    L.losses = o;    o = align_up(o + sizeof(float) * (size_t)W);
    L.partials = o;  o = align_up(o + sizeof(float) * partials_cap);
    L.scratch = o;   o = align_up(o + scratch_bytes);
    L.total = o;
    L.partials_cap = partials_cap;
    L.scratch_bytes = scratch_bytes;
    return L;
}

lsgd_status check_config(const lsgd_config* cfg, std::vector<int32_t>* offsets_out)
{
    if (!cfg) return fail(LSGD_ERR_INVALID_ARG, "config is NULL");
    if (cfg->W <= 0 || cfg->W > LSGD_MAX_WORKERS) return fail(LSGD_ERR_SHAPE, "W=%d outside [1,%d]", cfg->W, LSGD_MAX_WORKERS);
    if (cfg->P <= 0) return fail(LSGD_ERR_SHAPE, "P=%lld must be positive", (long long)cfg->P);
    if (cfg->ld < cfg->P) return fail(LSGD_ERR_SHAPE, "ld=%lld < P=%lld", (long long)cfg->ld, (long long)cfg->P);
    if (cfg->n_groups <= 0 || cfg->n_groups > LSGD_MAX_GROUPS || cfg->n_groups > cfg->W)
        return fail(LSGD_ERR_SHAPE, "n_groups=%d outside [1,min(W,%d)]", cfg->n_groups, LSGD_MAX_GROUPS);
    if (!std::isfinite(cfg->momentum) || cfg->momentum < 0.0f) return fail(LSGD_ERR_INVALID_ARG, "momentum must be finite and >= 0");
    if (!std::isfinite(cfg->weight_decay)) return fail(LSGD_ERR_INVALID_ARG, "weight_decay must be finite");
    const int known = LSGD_NESTEROV | LSGD_LEADER_EXEMPT | LSGD_PULL_UNSCALED_BY_ETA | LSGD_MOMENTUM_GRAD_ONLY | LSGD_WRITE_BF16_SHADOW |
                      LSGD_FUSED_MLP_UPDATE;
    if (cfg->flags & ~known) return fail(LSGD_ERR_INVALID_ARG, "unknown flag bits 0x%x", cfg->flags & ~known);
    std::vector<int32_t> off((size_t)cfg->n_groups + 1);
    if (cfg->group_offsets) {
        for (int j = 0; j <= cfg->n_groups; ++j) off[(size_t)j] = cfg->group_offsets[j];
        if (off.front() != 0 || off.back() != cfg->W) return fail(LSGD_ERR_SHAPE, "group_offsets must start at 0 and end at W");
        for (int j = 0; j < cfg->n_groups; ++j)
            if (off[(size_t)j + 1] <= off[(size_t)j]) return fail(LSGD_ERR_SHAPE, "group %d is empty or offsets decrease", j);
    } else {
        if (cfg->W % cfg->n_groups) return fail(LSGD_ERR_SHAPE, "W=%d not divisible by n_groups=%d and no group_offsets", cfg->W, cfg->n_groups);
        for (int j = 0; j <= cfg->n_groups; ++j) off[(size_t)j] = j * (cfg->W / cfg->n_groups);
    }
    if (offsets_out) offsets_out->swap(off);
    return LSGD_OK;
}

int64_t mlp_params(const lsgd_mlp_batch& b)
{
    int64_t P = 0;
    for (int k = 0; k < b.n_layers; ++k) P += (int64_t)b.dims[k + 1] * b.dims[k] + b.dims[k + 1];
    return P;
}

// Shape/pointer checks of a batch against a population shape; also sizes its scratch needs.
lsgd_status check_batch(const lsgd_batch* batch, int W, int64_t P, size_t* partials, size_t* scratch)
{
    if (partials) *partials = 0;
    if (scratch) *scratch = 0;
    if (!batch) return fail(LSGD_ERR_INVALID_ARG, "batch is NULL");
    if (!batch->desc) return fail(LSGD_ERR_INVALID_ARG, "batch->desc is NULL");
    switch (batch->kind) {
    case LSGD_BATCH_EXTERNAL: {
        const auto* d = static_cast<const lsgd_external_batch*>(batch->desc);
        if (!d->losses) return fail(LSGD_ERR_INVALID_ARG, "external batch: losses is NULL");
        return LSGD_OK;
    }
    case LSGD_BATCH_MC: {
        const auto* d = static_cast<const lsgd_mc_batch*>(batch->desc);
        if (d->m <= 0 || d->n <= 0 || d->r <= 0) return fail(LSGD_ERR_SHAPE, "matrix completion: m, n, r must be positive");
        if ((int64_t)(d->m + (int64_t)d->n) * d->r != P)
            return fail(LSGD_ERR_SHAPE, "matrix completion: (m+n)*r = %lld != P = %lld", (long long)((int64_t)(d->m + (int64_t)d->n) * d->r), (long long)P);
        if (d->n_obs < 0 || d->B < 0) return fail(LSGD_ERR_SHAPE, "matrix completion: negative n_obs or B");
        if (d->n_obs > 0 && !d->entries && (!d->rows || !d->cols || !d->vals))
            return fail(LSGD_ERR_INVALID_ARG, "matrix completion: rows/cols/vals is NULL and no packed entries given");
        if (d->entries && (reinterpret_cast<uintptr_t>(d->entries) & 15u))
            return fail(LSGD_ERR_INVALID_ARG, "matrix completion: entries must be 16-byte aligned");
        if (d->batch_idx && d->B > 0 && d->n_obs == 0) return fail(LSGD_ERR_SHAPE, "matrix completion: batch indices into an empty list");
        if (!std::isfinite(d->c)) return fail(LSGD_ERR_INVALID_ARG, "matrix completion: c must be finite");
        if (partials) *partials = mc_partials(W, *d);
        if (scratch) *scratch = mc_scratch_bytes(W, *d);
        return LSGD_OK;
    }
    case LSGD_BATCH_MLP: {
        const auto* d = static_cast<const lsgd_mlp_batch*>(batch->desc);
        if (d->n_layers <= 0 || !d->dims) return fail(LSGD_ERR_INVALID_ARG, "MLP: n_layers must be positive and dims non-NULL");
        for (int k = 0; k <= d->n_layers; ++k)
            if (d->dims[k] <= 0) return fail(LSGD_ERR_SHAPE, "MLP: dims[%d] must be positive", k);
        if (mlp_params(*d) != P) return fail(LSGD_ERR_SHAPE, "MLP: layer sizes give %lld parameters, P = %lld", (long long)mlp_params(*d), (long long)P);
        if (d->B <= 0) return fail(LSGD_ERR_SHAPE, "MLP: B must be positive");
        if (!d->X || !d->y) return fail(LSGD_ERR_INVALID_ARG, "MLP: X or y is NULL");
        const char* why = "";
        if (!mlp_shape_supported(*d, &why)) return fail(LSGD_ERR_UNSUPPORTED, "MLP: %s", why);
        if (scratch) *scratch = mlp_scratch_bytes(W, *d);
        return LSGD_OK;
    }
    default:
        return fail(LSGD_ERR_INVALID_ARG, "unknown batch kind %d", batch->kind);
    }
}

} // namespace

struct lsgd_population {
    lsgd_config cfg;
    std::vector<int32_t> offsets, group_of;
    float *x, *g, *m, *Z;
    uint16_t* xb;
    hipStream_t stream;
    Layout layout;
    DeviceState st;
    std::vector<uint8_t> local_selected, pending_local, z_valid; // z_valid: [G+1]
    bool global_selected, pending_global;
    bool shadow_valid;
    bool losses_valid; // the population's own loss buffer has been written (grad_loss / smooth_losses into it)
    int group_size; // rows per group if all groups are equal, else 0
};

extern "C" {

const char* lsgd_last_error(void) { return g_err; }

size_t lsgd_workspace_bytes(const lsgd_config* cfg, const lsgd_batch* largest)
{
    if (check_config(cfg, nullptr) != LSGD_OK) return 0;
    size_t partials = 0, scratch = 0;
    if (largest && check_batch(largest, cfg->W, cfg->P, &partials, &scratch) != LSGD_OK) return 0;
    // fixed part (with a W-float partials slot), then oversized partials, then workload scratch
    size_t total = make_layout(cfg->W, cfg->n_groups, (size_t)cfg->W, 0).total;
    if (partials > (size_t)cfg->W) total += align_up(sizeof(float) * partials);
    return total + align_up(scratch);
}

lsgd_status lsgd_create_population(const lsgd_config* cfg, float* x, float* g, float* m, float* z_snapshot,
                                   uint16_t* x_bf16, void* workspace, size_t workspace_bytes, void* hip_stream,
                                   lsgd_population** out)
{
    if (!out) return fail(LSGD_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    std::vector<int32_t> off;
    lsgd_status st = check_config(cfg, &off);
    if (st != LSGD_OK) return st;
    if (!x || !g) return fail(LSGD_ERR_INVALID_ARG, "x and g are required");
    if (cfg->momentum != 0.0f && !m) return fail(LSGD_ERR_INVALID_ARG, "momentum != 0 needs the m buffer");
    if ((cfg->flags & LSGD_WRITE_BF16_SHADOW) && !x_bf16) return fail(LSGD_ERR_INVALID_ARG, "LSGD_WRITE_BF16_SHADOW needs x_bf16");
    if (!workspace) return fail(LSGD_ERR_INVALID_ARG, "workspace is NULL");
    if (reinterpret_cast<uintptr_t>(workspace) % kAlign) return fail(LSGD_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    const size_t fixed = make_layout(cfg->W, cfg->n_groups, (size_t)cfg->W, 0).total;
    if (workspace_bytes < fixed) return fail(LSGD_ERR_NOMEM, "workspace of %zu bytes < %zu needed", workspace_bytes, fixed);

    lsgd_population* p = new (std::nothrow) lsgd_population();
    if (!p) return fail(LSGD_ERR_NOMEM, "host allocation failed");
    p->cfg = *cfg;
    p->cfg.group_offsets = nullptr;
    p->offsets = off;
    p->group_of.resize((size_t)cfg->W);
    for (int j = 0; j < cfg->n_groups; ++j)
        for (int i = off[(size_t)j]; i < off[(size_t)j + 1]; ++i) p->group_of[(size_t)i] = j;
    p->x = x; p->g = g; p->m = m; p->Z = z_snapshot; p->xb = x_bf16;
    p->stream = static_cast<hipStream_t>(hip_stream);
    // everything past the fixed part is split between loss partials and workload scratch on demand
    const size_t spare = workspace_bytes - fixed;
    p->layout = make_layout(cfg->W, cfg->n_groups, (size_t)cfg->W, 0);
    char* base = static_cast<char*>(workspace);
    p->st.lead = reinterpret_cast<int32_t*>(base + p->layout.lead);
    p->st.glead = reinterpret_cast<int32_t*>(base + p->layout.glead);
    p->st.refreshed = reinterpret_cast<int32_t*>(base + p->layout.refreshed);
    p->st.offsets = reinterpret_cast<int32_t*>(base + p->layout.offsets);
    p->st.group_of = reinterpret_cast<int32_t*>(base + p->layout.group_of);
    p->st.plan = reinterpret_cast<RowPlan*>(base + p->layout.plan);
    p->st.losses = reinterpret_cast<float*>(base + p->layout.losses);
    p->st.partials = reinterpret_cast<float*>(base + p->layout.partials);
    p->st.partials_cap = (size_t)cfg->W;
    p->st.scratch = base + p->layout.total;
    p->st.scratch_bytes = spare;
    p->local_selected.assign((size_t)cfg->n_groups, 0);
    p->pending_local.assign((size_t)cfg->n_groups, 0);
    p->z_valid.assign((size_t)cfg->n_groups + 1, 0);
    p->global_selected = p->pending_global = false;
    p->shadow_valid = false;
    p->losses_valid = false;
    p->group_size = off[1] - off[0];
    for (int j = 0; j < cfg->n_groups; ++j)
        if (off[(size_t)j + 1] - off[(size_t)j] != off[1] - off[0]) p->group_size = 0;

    hipError_t e = hipMemcpyAsync(p->st.offsets, p->offsets.data(), sizeof(int32_t) * p->offsets.size(), hipMemcpyHostToDevice, p->stream);
    if (e == hipSuccess) e = hipMemcpyAsync(p->st.group_of, p->group_of.data(), sizeof(int32_t) * p->group_of.size(), hipMemcpyHostToDevice, p->stream);
    if (e == hipSuccess) e = launch_init_state(p->st, cfg->W, cfg->n_groups, p->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(p->stream); // host vectors were the copy source
    if (e != hipSuccess) {
        delete p;
        return fail(LSGD_ERR_HIP, "create: %s", hipGetErrorString(e));
    }
    *out = p;
    return LSGD_OK;
}

lsgd_status lsgd_destroy_population(lsgd_population* pop)
{
    delete pop;
    return LSGD_OK;
}

} // extern "C"

namespace {

lsgd_status do_grad_loss(lsgd_population* p, const lsgd_batch* batch, float* losses_out)
{
    float* losses = losses_out ? losses_out : p->st.losses;
    hipError_t e = hipSuccess;
    switch (batch->kind) {
    case LSGD_BATCH_EXTERNAL: {
        const auto* d = static_cast<const lsgd_external_batch*>(batch->desc);
        if (d->losses != losses)
            e = hipMemcpyAsync(losses, d->losses, sizeof(float) * (size_t)p->cfg.W, hipMemcpyDeviceToDevice, p->stream);
        break;
    }
    case LSGD_BATCH_MC: {
        const auto* d = static_cast<const lsgd_mc_batch*>(batch->desc);
        // loss partials live at the start of the spare region when they outgrow the fixed slot
        DeviceState st = p->st;
        const size_t need = mc_partials(p->cfg.W, *d);
        size_t used = 0;
        if (need > (size_t)p->cfg.W) {
            st.partials = reinterpret_cast<float*>(p->st.scratch);
            used = align_up(sizeof(float) * need);
        }
        st.scratch = p->st.scratch + used;
        st.scratch_bytes = p->st.scratch_bytes - used;
        e = launch_mc_grad_loss(p->x, p->g, losses, p->cfg.W, p->cfg.P, p->cfg.ld, *d, st, p->stream);
        break;
    }
    case LSGD_BATCH_MLP: {
        const auto* d = static_cast<const lsgd_mlp_batch*>(batch->desc);
        if (!p->shadow_valid) {
            e = launch_cast_shadow(p->x, p->xb, p->cfg.W, p->cfg.P, p->cfg.ld, p->stream);
            if (e != hipSuccess) break;
            p->shadow_valid = true;
        }
        e = launch_mlp_grad_loss(p->xb, p->x, p->g, losses, p->cfg.W, p->cfg.P, p->cfg.ld, *d, p->st, p->stream);
        break;
    }
    default: break;
    }
    if (e != hipSuccess) return fail(LSGD_ERR_HIP, "grad_loss: %s", hipGetErrorString(e));
    if (!losses_out) p->losses_valid = true;
    return LSGD_OK;
}

// objective values only, at the current parameters; g is left alone
lsgd_status do_loss(lsgd_population* p, const lsgd_batch* batch, float* losses_out)
{
    float* losses = losses_out ? losses_out : p->st.losses;
    hipError_t e = hipSuccess;
    switch (batch->kind) {
    case LSGD_BATCH_EXTERNAL: {
        const auto* d = static_cast<const lsgd_external_batch*>(batch->desc);
        if (d->losses != losses)
            e = hipMemcpyAsync(losses, d->losses, sizeof(float) * (size_t)p->cfg.W, hipMemcpyDeviceToDevice, p->stream);
        break;
    }
    case LSGD_BATCH_MC: {
        const auto* d = static_cast<const lsgd_mc_batch*>(batch->desc);
        DeviceState st = p->st;
        if (mc_partials(p->cfg.W, *d) > (size_t)p->cfg.W) st.partials = reinterpret_cast<float*>(p->st.scratch);
        e = launch_mc_loss(p->x, losses, p->cfg.W, p->cfg.ld, *d, st, p->stream);
        break;
    }
    case LSGD_BATCH_MLP: {
        const auto* d = static_cast<const lsgd_mlp_batch*>(batch->desc);
        if (!p->shadow_valid) {
            e = launch_cast_shadow(p->x, p->xb, p->cfg.W, p->cfg.P, p->cfg.ld, p->stream);
            if (e != hipSuccess) break;
            p->shadow_valid = true;
        }
        e = launch_mlp_forward(p->xb, p->x, losses, p->cfg.W, p->cfg.P, p->cfg.ld, *d, p->st, p->stream);
        break;
    }
    default: break;
    }
    if (e != hipSuccess) return fail(LSGD_ERR_HIP, "loss: %s", hipGetErrorString(e));
    if (!losses_out) p->losses_valid = true;
    return LSGD_OK;
}

lsgd_status check_grad_loss(lsgd_population* p, const lsgd_batch* batch)
{
    size_t partials = 0, scratch = 0;
    lsgd_status st = check_batch(batch, p->cfg.W, p->cfg.P, &partials, &scratch);
    if (st != LSGD_OK) return st;
    if (batch->kind == LSGD_BATCH_MLP && !p->xb) return fail(LSGD_ERR_STATE, "MLP batches need the x_bf16 buffer");
    size_t need = scratch;
    if (partials > (size_t)p->cfg.W) need += align_up(sizeof(float) * partials);
    if (need > p->st.scratch_bytes)
        return fail(LSGD_ERR_NOMEM, "workspace too small for this batch: %zu spare bytes, %zu needed", p->st.scratch_bytes, need);
    return LSGD_OK;
}

lsgd_status check_scalars(float eta, float lamL, float lamG)
{
    if (!std::isfinite(eta) || !std::isfinite(lamL) || !std::isfinite(lamG))
        return fail(LSGD_ERR_INVALID_ARG, "eta, lambda_L, lambda_G must be finite");
    return LSGD_OK;
}

// Would an update with these coefficients find every leader it needs, given
// what is selected / pending / kept (optionally after a selection with this mask)?
lsgd_status check_pull_state(const lsgd_population* p, float eta, float lamL, float lamG,
                             const uint8_t* extra_local, bool extra_all_local, bool extra_global)
{
    if ((p->cfg.flags & LSGD_PULL_UNSCALED_BY_ETA) && (lamL != 0.0f || lamG != 0.0f) && eta == 0.0f)
        return fail(LSGD_ERR_INVALID_ARG, "unscaled pulls need eta != 0");
    const int G = p->cfg.n_groups;
    if (lamL != 0.0f) {
        for (int j = 0; j < G; ++j) {
            const bool fresh = p->pending_local[(size_t)j] || extra_all_local || (extra_local && extra_local[j]);
            if (fresh) continue;
            if (!p->Z) return fail(LSGD_ERR_STATE, "group %d keeps its leader but z_snapshot is NULL", j);
            if (!p->z_valid[(size_t)j]) return fail(LSGD_ERR_STATE, "group %d has no selected leader copy", j);
        }
    }
    if (lamG != 0.0f) {
        const bool fresh = p->pending_global || extra_global;
        if (!fresh) {
            if (!p->Z) return fail(LSGD_ERR_STATE, "global leader is kept but z_snapshot is NULL");
            if (!p->z_valid[(size_t)G]) return fail(LSGD_ERR_STATE, "no global leader copy has been selected");
        }
    }
    return LSGD_OK;
}

lsgd_status do_select(lsgd_population* p, const float* losses, const uint8_t* refresh_local, int refresh_global)
{
    const int G = p->cfg.n_groups;
    RefreshBits sel, cap;
    std::memset(&sel, 0, sizeof(sel));
    std::memset(&cap, 0, sizeof(cap));
    for (int j = 0; j < G; ++j) {
        const bool r = !refresh_local || refresh_local[j];
        if (r) {
            sel.w[j >> 6] |= 1ull << (j & 63);
            p->pending_local[(size_t)j] = 1;
            p->local_selected[(size_t)j] = 1;
        }
        if (p->pending_local[(size_t)j]) cap.w[j >> 6] |= 1ull << (j & 63);
    }
    if (refresh_global) { p->pending_global = true; p->global_selected = true; }
    hipError_t e = launch_select_leaders(losses ? losses : p->st.losses, p->cfg.W, G, p->st, sel, cap,
                                         refresh_global != 0, p->pending_global, p->stream);
    if (e != hipSuccess) return fail(LSGD_ERR_HIP, "select_leaders: %s", hipGetErrorString(e));
    return LSGD_OK;
}

bool any_pending(const lsgd_population* p)
{
    bool any = p->pending_global;
    for (int j = 0; j < p->cfg.n_groups; ++j) any = any || p->pending_local[(size_t)j];
    return any;
}

// comm: Algorithm 1's communication pull (lamL, lamG are its lambdas; eta unused).
// unscaled: the pulls of a gradient step are not multiplied by eta.
lsgd_status do_pull(lsgd_population* p, float eta, float lamL, float lamG, bool unscaled, bool comm)
{
    const int G = p->cfg.n_groups;
    PullParams q;
    q.x = p->x; q.g = p->g; q.m = p->m; q.Z = p->Z;
    q.xb = (p->cfg.flags & LSGD_WRITE_BF16_SHADOW) ? p->xb : nullptr;
    q.P = p->cfg.P; q.ld = p->cfg.ld; q.W = p->cfg.W; q.G = G;
    q.eta = eta; q.mu = p->cfg.momentum; q.wd = p->cfg.weight_decay;
    q.lamL = lamL; q.lamG = lamG;
    if (unscaled && !comm) {
        if (lamL != 0.0f) q.lamL = lamL / eta;
        if (lamG != 0.0f) q.lamG = lamG / eta;
    }
    q.flags = p->cfg.flags;
    q.use_refreshed = any_pending(p) ? 1 : 0;
    q.clear_refreshed = 0;
    q.group_size = p->group_size;
    q.comm_pull = comm ? 1 : 0;
    hipError_t e = launch_pull_update(q, p->st, p->stream);
    if (e != hipSuccess) return fail(LSGD_ERR_HIP, "%s: %s", comm ? "leader_pull" : "pull_update", hipGetErrorString(e));
    // a refreshed leader whose term was active has now been captured (and kept, if Z exists);
    // the communication pull captures every refreshed leader
    // (a re-selected leader whose coefficient was exactly 0 was not captured: its kept copy, if any, still
    // belongs to the previous leader, so it stops being valid until the next selection)
    for (int j = 0; j < G; ++j) {
        if (p->pending_local[(size_t)j]) p->z_valid[(size_t)j] = (comm || lamL != 0.0f) && p->Z != nullptr;
        p->pending_local[(size_t)j] = 0;
    }
    if (p->pending_global) p->z_valid[(size_t)G] = (comm || lamG != 0.0f) && p->Z != nullptr;
    p->pending_global = false;
    if (!(p->cfg.flags & LSGD_WRITE_BF16_SHADOW)) p->shadow_valid = false;
    return LSGD_OK;
}

lsgd_status do_pull(lsgd_population* p, float eta, float lamL, float lamG)
{
    return do_pull(p, eta, lamL, lamG, (p->cfg.flags & LSGD_PULL_UNSCALED_BY_ETA) != 0, false);
}

// forward + losses -> leaders -> kept copies brought up to date -> backward pass that applies the update
lsgd_status do_fused_mlp_step(lsgd_population* p, const lsgd_batch* batch, float eta, float lamL, float lamG,
                              const uint8_t* refresh_local, int refresh_global)
{
    const auto* d = static_cast<const lsgd_mlp_batch*>(batch->desc);
    if ((lamL != 0.0f || lamG != 0.0f) && !p->Z) return fail(LSGD_ERR_STATE, "the fused MLP update reads leaders from z_snapshot, which is NULL");
    hipError_t e = hipSuccess;
    if (!p->shadow_valid) {
        e = launch_cast_shadow(p->x, p->xb, p->cfg.W, p->cfg.P, p->cfg.ld, p->stream);
        if (e != hipSuccess) return fail(LSGD_ERR_HIP, "cast_shadow: %s", hipGetErrorString(e));
        p->shadow_valid = true;
    }
    e = launch_mlp_forward(p->xb, p->x, p->st.losses, p->cfg.W, p->cfg.P, p->cfg.ld, *d, p->st, p->stream);
    if (e != hipSuccess) return fail(LSGD_ERR_HIP, "mlp forward: %s", hipGetErrorString(e));
    p->losses_valid = true;
    lsgd_status st = do_select(p, nullptr, refresh_local, refresh_global);
    if (st != LSGD_OK) return st;
    if (any_pending(p)) {
        if (lamL != 0.0f || lamG != 0.0f) {
            st = do_pull(p, 0.0f, 0.0f, 0.0f, false, true);            // capture only: nobody moves
            if (st != LSGD_OK) return st;
        } else {                                                       // nothing is captured: old copies go stale
            for (int j = 0; j < p->cfg.n_groups; ++j)
                if (p->pending_local[(size_t)j]) { p->z_valid[(size_t)j] = 0; p->pending_local[(size_t)j] = 0; }
            if (p->pending_global) { p->z_valid[(size_t)p->cfg.n_groups] = 0; p->pending_global = false; }
        }
    }
    FusedUpdate fu{};
    fu.enabled = 1;
    fu.x = p->x; fu.m = (p->cfg.momentum != 0.0f) ? p->m : nullptr; fu.xb = p->xb; fu.Z = p->Z;
    fu.lead = p->st.lead; fu.glead = p->st.glead; fu.group_of = p->st.group_of; fu.G = p->cfg.n_groups;
    fu.eta = eta; fu.mu = p->cfg.momentum; fu.wd = p->cfg.weight_decay; fu.flags = p->cfg.flags;
    fu.lamL = lamL; fu.lamG = lamG;
    if (p->cfg.flags & LSGD_PULL_UNSCALED_BY_ETA) {
        if (lamL != 0.0f) fu.lamL = lamL / eta;
        if (lamG != 0.0f) fu.lamG = lamG / eta;
    }
    e = launch_mlp_backward(p->xb, p->x, p->g, p->cfg.W, p->cfg.P, p->cfg.ld, *d, p->st, &fu, p->stream);
    if (e != hipSuccess) return fail(LSGD_ERR_HIP, "mlp backward: %s", hipGetErrorString(e));
    p->shadow_valid = true;
    return LSGD_OK;
}

} // namespace

extern "C" {

lsgd_status lsgd_grad_loss(lsgd_population* pop, const lsgd_batch* batch, float* losses)
{
    if (!pop) return fail(LSGD_ERR_INVALID_ARG, "population is NULL");
    lsgd_status st = check_grad_loss(pop, batch);
    if (st != LSGD_OK) return st;
    return do_grad_loss(pop, batch, losses);
}

lsgd_status lsgd_loss(lsgd_population* pop, const lsgd_batch* batch, float* losses)
{
    if (!pop) return fail(LSGD_ERR_INVALID_ARG, "population is NULL");
    lsgd_status st = check_grad_loss(pop, batch);
    if (st != LSGD_OK) return st;
    return do_loss(pop, batch, losses);
}

lsgd_status lsgd_select_leaders(lsgd_population* pop, const float* losses, const uint8_t* refresh_local, int refresh_global)
{
    if (!pop) return fail(LSGD_ERR_INVALID_ARG, "population is NULL");
    if (!losses && !pop->losses_valid)
        return fail(LSGD_ERR_STATE, "select_leaders: losses is NULL and the population's own loss buffer was never written "
                                    "(no lsgd_grad_loss / lsgd_smooth_losses into it yet)");
    return do_select(pop, losses, refresh_local, refresh_global);
}

lsgd_status lsgd_pull_update(lsgd_population* pop, float eta, float lambda_L, float lambda_G)
{
    if (!pop) return fail(LSGD_ERR_INVALID_ARG, "population is NULL");
    lsgd_status st = check_scalars(eta, lambda_L, lambda_G);
    if (st != LSGD_OK) return st;
    st = check_pull_state(pop, eta, lambda_L, lambda_G, nullptr, false, false);
    if (st != LSGD_OK) return st;
    return do_pull(pop, eta, lambda_L, lambda_G);
}

lsgd_status lsgd_step(lsgd_population* pop, const lsgd_batch* batch, float eta, float lambda_L, float lambda_G,
                      const uint8_t* refresh_local, int refresh_global)
{
    if (!pop) return fail(LSGD_ERR_INVALID_ARG, "population is NULL");
    lsgd_status st = check_scalars(eta, lambda_L, lambda_G);
    if (st != LSGD_OK) return st;
    st = check_grad_loss(pop, batch);
    if (st != LSGD_OK) return st;
    st = check_pull_state(pop, eta, lambda_L, lambda_G, refresh_local, refresh_local == nullptr, refresh_global != 0);
    if (st != LSGD_OK) return st;
    if ((pop->cfg.flags & LSGD_FUSED_MLP_UPDATE) && batch->kind == LSGD_BATCH_MLP)
        return do_fused_mlp_step(pop, batch, eta, lambda_L, lambda_G, refresh_local, refresh_global);
    st = do_grad_loss(pop, batch, nullptr);
    if (st != LSGD_OK) return st;
    st = do_select(pop, nullptr, refresh_local, refresh_global);
    if (st != LSGD_OK) return st;
    return do_pull(pop, eta, lambda_L, lambda_G);
}

lsgd_status lsgd_leader_pull(lsgd_population* pop, float lambda_L, float lambda_G)
{
    if (!pop) return fail(LSGD_ERR_INVALID_ARG, "population is NULL");
    lsgd_status st = check_scalars(0.0f, lambda_L, lambda_G);
    if (st != LSGD_OK) return st;
    if (!any_pending(pop)) return fail(LSGD_ERR_STATE, "leader_pull: no leader was re-selected since the last update");
    return do_pull(pop, 0.0f, lambda_L, lambda_G, false, true);
}

lsgd_status lsgd_step_alg1(lsgd_population* pop, const lsgd_batch* batch, float eta, float gamma_L, float gamma_G,
                           float lambda_L, float lambda_G, int comm, const uint8_t* comm_local_mask)
{
    if (!pop) return fail(LSGD_ERR_INVALID_ARG, "population is NULL");
    lsgd_status st = check_scalars(eta, gamma_L, gamma_G);
    if (st != LSGD_OK) return st;
    st = check_scalars(eta, lambda_L, lambda_G);
    if (st != LSGD_OK) return st;
    if (comm & ~(LSGD_COMM_LOCAL | LSGD_COMM_GLOBAL)) return fail(LSGD_ERR_INVALID_ARG, "step_alg1: unknown comm bits %d", comm);
    if (!pop->Z) return fail(LSGD_ERR_STATE, "step_alg1 needs the z_snapshot buffer");
    if ((gamma_L != 0.0f || gamma_G != 0.0f) && eta == 0.0f) return fail(LSGD_ERR_INVALID_ARG, "unscaled pulls need eta != 0");
    st = check_grad_loss(pop, batch);
    if (st != LSGD_OK) return st;
    // the every-iteration pulls read kept copies (or leaders still pending from an explicit selection)
    st = check_pull_state(pop, eta, gamma_L, gamma_G, nullptr, false, false);
    if (st != LSGD_OK) return st;
    const int G = pop->cfg.n_groups;
    bool any_local = false;
    if (comm & LSGD_COMM_LOCAL) {
        for (int j = 0; j < G; ++j) any_local = any_local || !comm_local_mask || comm_local_mask[j];
    }
    st = do_grad_loss(pop, batch, nullptr);
    if (st != LSGD_OK) return st;
    st = do_pull(pop, eta, gamma_L, gamma_G, true, false);
    if (st != LSGD_OK) return st;
    if (!any_local && !(comm & LSGD_COMM_GLOBAL)) return LSGD_OK;
    std::vector<uint8_t> none;
    const uint8_t* mask = comm_local_mask;
    if (!(comm & LSGD_COMM_LOCAL)) {
        none.assign((size_t)G, 0);
        mask = none.data();
    }
    st = do_select(pop, nullptr, mask, (comm & LSGD_COMM_GLOBAL) != 0);
    if (st != LSGD_OK) return st;
    return do_pull(pop, 0.0f, lambda_L, lambda_G, false, true);
}

lsgd_status lsgd_smooth_losses(lsgd_population* pop, float* window, int32_t K, int64_t t, const float* losses, float* out)
{
    if (!pop) return fail(LSGD_ERR_INVALID_ARG, "population is NULL");
    if (!window) return fail(LSGD_ERR_INVALID_ARG, "smooth_losses: window is NULL");
    if (K <= 0 || K > 65536) return fail(LSGD_ERR_SHAPE, "smooth_losses: K = %d outside [1, 65536]", (int)K);
    if (t < 0) return fail(LSGD_ERR_INVALID_ARG, "smooth_losses: t is negative");
    if (!losses && !pop->losses_valid)
        return fail(LSGD_ERR_STATE, "smooth_losses: losses is NULL and the population's own loss buffer was never written");
    hipError_t e = launch_smooth_losses(window, K, t, losses ? losses : pop->st.losses, pop->cfg.W,
                                        out ? out : pop->st.losses, pop->stream);
    if (e != hipSuccess) return fail(LSGD_ERR_HIP, "smooth_losses: %s", hipGetErrorString(e));
    if (!out) pop->losses_valid = true;
    return LSGD_OK;
}

lsgd_status lsgd_center(lsgd_population* pop, float* out)
{
    if (!pop) return fail(LSGD_ERR_INVALID_ARG, "population is NULL");
    if (!out) return fail(LSGD_ERR_INVALID_ARG, "center: out is NULL");
    hipError_t e = launch_center(pop->x, pop->cfg.W, pop->cfg.P, pop->cfg.ld, out, pop->stream);
    if (e != hipSuccess) return fail(LSGD_ERR_HIP, "center: %s", hipGetErrorString(e));
    return LSGD_OK;
}

lsgd_status lsgd_easgd_update(lsgd_population* pop, float* center, float eta, float lambda)
{
    if (!pop) return fail(LSGD_ERR_INVALID_ARG, "population is NULL");
    if (!center) return fail(LSGD_ERR_INVALID_ARG, "easgd_update: center is NULL");
    lsgd_status st = check_scalars(eta, lambda, 0.0f);
    if (st != LSGD_OK) return st;
    if (!pop->Z) return fail(LSGD_ERR_STATE, "easgd_update keeps the pre-update center in z_snapshot, which is NULL");
    if (any_pending(pop)) return fail(LSGD_ERR_STATE, "easgd_update: a leader selection is pending; elastic averaging uses no leaders");
    const int G = pop->cfg.n_groups;
    // center first (it reads the workers before they move); the old center lands in the global row of Z
    const double a = (double)pop->cfg.W * (double)eta * (double)lambda;
    hipError_t e = launch_easgd_center(pop->x, pop->cfg.W, pop->cfg.P, pop->cfg.ld, center, pop->Z + (int64_t)G * pop->cfg.ld, a, pop->stream);
    if (e != hipSuccess) return fail(LSGD_ERR_HIP, "easgd_update: center: %s", hipGetErrorString(e));
    pop->z_valid[(size_t)G] = 0;             // that row no longer holds a leader
    PullParams q;
    q.x = pop->x; q.g = pop->g; q.m = pop->m; q.Z = pop->Z;
    q.xb = (pop->cfg.flags & LSGD_WRITE_BF16_SHADOW) ? pop->xb : nullptr;
    q.P = pop->cfg.P; q.ld = pop->cfg.ld; q.W = pop->cfg.W; q.G = G;
    q.eta = eta; q.mu = pop->cfg.momentum; q.wd = pop->cfg.weight_decay;
    q.lamL = 0.0f; q.lamG = lambda;
    q.flags = pop->cfg.flags & ~LSGD_LEADER_EXEMPT;        // nobody is a leader here
    q.use_refreshed = 0; q.clear_refreshed = 0;
    q.group_size = pop->group_size;
    q.comm_pull = 0;
    e = launch_pull_update(q, pop->st, pop->stream);
    if (e != hipSuccess) return fail(LSGD_ERR_HIP, "easgd_update: %s", hipGetErrorString(e));
    if (!(pop->cfg.flags & LSGD_WRITE_BF16_SHADOW)) pop->shadow_valid = false;
    return LSGD_OK;
}

lsgd_status lsgd_easgd_step(lsgd_population* pop, const lsgd_batch* batch, float* center, float eta, float lambda)
{
    if (!pop) return fail(LSGD_ERR_INVALID_ARG, "population is NULL");
    if (!center) return fail(LSGD_ERR_INVALID_ARG, "easgd_step: center is NULL");
    lsgd_status st = check_scalars(eta, lambda, 0.0f);
    if (st != LSGD_OK) return st;
    if (!pop->Z) return fail(LSGD_ERR_STATE, "easgd_step keeps the pre-update center in z_snapshot, which is NULL");
    if (any_pending(pop)) return fail(LSGD_ERR_STATE, "easgd_step: a leader selection is pending; elastic averaging uses no leaders");
    st = check_grad_loss(pop, batch);
    if (st != LSGD_OK) return st;
    st = do_grad_loss(pop, batch, nullptr);
    if (st != LSGD_OK) return st;
    return lsgd_easgd_update(pop, center, eta, lambda);
}

lsgd_status lsgd_mc_pack_entries(const int32_t* rows, const int32_t* cols, const float* vals, int64_t n_obs,
                                 lsgd_mc_entry* out, void* hip_stream)
{
    if (n_obs < 0) return fail(LSGD_ERR_SHAPE, "n_obs is negative");
    if (n_obs == 0) return LSGD_OK;
    if (!rows || !cols || !vals || !out) return fail(LSGD_ERR_INVALID_ARG, "pack_entries: NULL pointer");
    if (reinterpret_cast<uintptr_t>(out) & 15u) return fail(LSGD_ERR_INVALID_ARG, "pack_entries: out must be 16-byte aligned");
    hipError_t e = launch_mc_pack(rows, cols, vals, n_obs, out, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(LSGD_ERR_HIP, "pack_entries: %s", hipGetErrorString(e));
    return LSGD_OK;
}

lsgd_status lsgd_sync_shadow(lsgd_population* pop)
{
    if (!pop) return fail(LSGD_ERR_INVALID_ARG, "population is NULL");
    if (!pop->xb) return fail(LSGD_ERR_STATE, "no x_bf16 buffer was given");
    hipError_t e = launch_cast_shadow(pop->x, pop->xb, pop->cfg.W, pop->cfg.P, pop->cfg.ld, pop->stream);
    if (e != hipSuccess) return fail(LSGD_ERR_HIP, "sync_shadow: %s", hipGetErrorString(e));
    pop->shadow_valid = true;
    return LSGD_OK;
}

lsgd_status lsgd_get_leaders(lsgd_population* pop, int32_t* local_leaders, int32_t* global_leader)
{
    if (!pop) return fail(LSGD_ERR_INVALID_ARG, "population is NULL");
    hipError_t e = hipSuccess;
    if (local_leaders)
        e = hipMemcpyAsync(local_leaders, pop->st.lead, sizeof(int32_t) * (size_t)pop->cfg.n_groups, hipMemcpyDeviceToHost, pop->stream);
    if (e == hipSuccess && global_leader)
        e = hipMemcpyAsync(global_leader, pop->st.glead, sizeof(int32_t), hipMemcpyDeviceToHost, pop->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(pop->stream);
    if (e != hipSuccess) return fail(LSGD_ERR_HIP, "get_leaders: %s", hipGetErrorString(e));
    return LSGD_OK;
}

lsgd_status lsgd_set_leaders(lsgd_population* pop, const int32_t* local_leaders, int32_t global_leader)
{
    if (!pop) return fail(LSGD_ERR_INVALID_ARG, "population is NULL");
    if (!local_leaders) return fail(LSGD_ERR_INVALID_ARG, "set_leaders: local_leaders is NULL");
    const int G = pop->cfg.n_groups;
    for (int j = 0; j < G; ++j) {
        const int32_t v = local_leaders[j];
        if (v != -1 && (v < pop->offsets[(size_t)j] || v >= pop->offsets[(size_t)j + 1]))
            return fail(LSGD_ERR_INVALID_ARG, "set_leaders: leader %d is not a row of group %d", (int)v, j);
    }
    if (global_leader != -1 && (global_leader < 0 || global_leader >= pop->cfg.W))
        return fail(LSGD_ERR_INVALID_ARG, "set_leaders: global leader %d outside [0, W)", (int)global_leader);
    // staged through the host object so that the source outlives the asynchronous copy
    std::vector<int32_t> stage(local_leaders, local_leaders + G);
    stage.push_back(global_leader);
    hipError_t e = hipMemcpyAsync(pop->st.lead, stage.data(), sizeof(int32_t) * (size_t)G, hipMemcpyHostToDevice, pop->stream);
    if (e == hipSuccess) e = hipMemcpyAsync(pop->st.glead, stage.data() + G, sizeof(int32_t), hipMemcpyHostToDevice, pop->stream);
    if (e == hipSuccess) e = launch_init_refreshed(pop->st, G, pop->stream);
    if (e == hipSuccess) e = launch_write_plan(pop->st, pop->cfg.W, G, pop->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(pop->stream);
    if (e != hipSuccess) return fail(LSGD_ERR_HIP, "set_leaders: %s", hipGetErrorString(e));
    for (int j = 0; j < G; ++j) {
        pop->local_selected[(size_t)j] = stage[(size_t)j] != -1;
        pop->pending_local[(size_t)j] = 0;
        pop->z_valid[(size_t)j] = stage[(size_t)j] != -1 && pop->Z != nullptr;
    }
    pop->global_selected = global_leader != -1;
    pop->pending_global = false;
    pop->z_valid[(size_t)G] = global_leader != -1 && pop->Z != nullptr;
    return LSGD_OK;
}

lsgd_status lsgd_get_losses(lsgd_population* pop, float* losses_host)
{
    if (!pop || !losses_host) return fail(LSGD_ERR_INVALID_ARG, "population or output is NULL");
    hipError_t e = hipMemcpyAsync(losses_host, pop->st.losses, sizeof(float) * (size_t)pop->cfg.W, hipMemcpyDeviceToHost, pop->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(pop->stream);
    if (e != hipSuccess) return fail(LSGD_ERR_HIP, "get_losses: %s", hipGetErrorString(e));
    return LSGD_OK;
}

} // extern "C"
