// Internal declarations shared by the HIP translation units of liblsgd.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lsgd.h"

namespace lsgd {

constexpr int kWave = 64;

// What a row of the population needs to know about its leaders, gathered in one 32-byte record so that the
// streaming update kernel finds it with a single scalar load (written by the selection kernel and by whatever
// else changes lead / glead / refreshed).
struct RowPlan {
    int32_t ll;      // local leader of the row's group (-1 = never selected)
    int32_t gl;      // global leader
    int32_t freshL;  // the group's leader was re-selected since the last update
    int32_t freshG;  // the global leader was
    int32_t j;       // the row's group
    int32_t pad[3];
};

// Device-side bookkeeping placed at the start of the caller's workspace.
struct DeviceState {
    int32_t* lead;      // [G]   local leader of each group (-1 = never selected)
    int32_t* glead;     // [1]   global leader
    int32_t* refreshed; // [G+1] 1 = leader re-selected since the last update (capture from x)
    int32_t* offsets;   // [G+1] group j owns rows [offsets[j], offsets[j+1])
    int32_t* group_of;  // [W]
    RowPlan* plan;      // [W]   lead / glead / refreshed as seen from each row
    float* losses;      // [W]   the population's own loss buffer
    float* partials;    // scratch for loss partial sums
    size_t partials_cap;
    char* scratch;      // workload scratch (activations, sort buffers ...)
    size_t scratch_bytes;
};

struct RefreshBits {
    uint64_t w[LSGD_MAX_GROUPS / 64];
};

// Records the message lsgd_last_error() returns on this thread and hands the status back.
lsgd_status set_error(lsgd_status st, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// ---- kernels' host launchers (each returns the hipError_t of its launches) ----
hipError_t launch_init_state(const DeviceState& st, int W, int G, hipStream_t s);
// clears the "re-selected since the last update" flags
hipError_t launch_init_refreshed(const DeviceState& st, int G, hipStream_t s);
// rewrites plan[W] from lead, glead, refreshed, group_of (after the host changed any of them)
hipError_t launch_write_plan(const DeviceState& st, int W, int G, hipStream_t s);

hipError_t launch_select_leaders(const float* losses, int W, int G, const DeviceState& st,
                                 const RefreshBits& bits, const RefreshBits& capture, int refresh_global,
                                 int capture_global, hipStream_t s);

struct PullParams {
    float* x;
    const float* g;
    float* m;           // may be NULL when mu == 0
    float* Z;           // may be NULL
    uint16_t* xb;       // bf16 shadow or NULL
    int64_t P, ld;
    int W, G;
    float eta, lamL, lamG, mu, wd;
    int flags;          // LSGD_NESTEROV | LSGD_LEADER_EXEMPT | LSGD_MOMENTUM_GRAD_ONLY
    int use_refreshed;  // 0: treat every leader as kept (read Z)
    int clear_refreshed;
    int group_size;     // rows per group when all groups are equal, else 0
    int comm_pull;      // 1: Algorithm 1's communication pull (no gradient, no momentum)
};
hipError_t launch_pull_update(const PullParams& p, const DeviceState& st, hipStream_t s);

hipError_t launch_smooth_losses(float* window, int K, int64_t t, const float* losses, int W, float* out, hipStream_t s);
hipError_t launch_easgd_center(const float* x, int W, int64_t P, int64_t ld, float* center, float* old_center, double a, hipStream_t s);
hipError_t launch_center(const float* x, int W, int64_t P, int64_t ld, float* out, hipStream_t s);

hipError_t launch_cast_shadow(const float* x, uint16_t* xb, int W, int64_t P, int64_t ld, hipStream_t s);

size_t mc_scratch_bytes(int W, const lsgd_mc_batch& b);
size_t mc_partials(int W, const lsgd_mc_batch& b);
hipError_t launch_mc_grad_loss(const float* x, float* g, float* losses, int W, int64_t P, int64_t ld,
                               const lsgd_mc_batch& b, const DeviceState& st, hipStream_t s);
// objective values only (no gradient); needs the same loss-partial slots as launch_mc_grad_loss
hipError_t launch_mc_loss(const float* x, float* losses, int W, int64_t ld, const lsgd_mc_batch& b, const DeviceState& st,
                          hipStream_t s);

hipError_t launch_mc_pack(const int32_t* rows, const int32_t* cols, const float* vals, int64_t n, lsgd_mc_entry* out, hipStream_t s);

// When `enabled`, the kernels that produce gradient values apply the update to x (and m, and the
// bf16 copy) themselves instead of writing g.  Leader parameters are always read from the kept
// copies Z, which the caller has brought up to date beforehand.
struct FusedUpdate {
    int enabled;
    float* x;
    float* m;               // NULL when mu == 0
    uint16_t* xb;
    const float* Z;         // [(G+1)][ld]; may be NULL when both coefficients are 0
    const int32_t* lead;
    const int32_t* glead;
    const int32_t* group_of;
    int G;
    float eta, lamL, lamG, mu, wd;   // lamL, lamG as the kernel applies them (already divided by eta if unscaled)
    int flags;
};

size_t mlp_scratch_bytes(int W, const lsgd_mlp_batch& b);
// returns LSGD_OK / LSGD_ERR_UNSUPPORTED through *status for shapes the kernels do not cover
hipError_t launch_mlp_grad_loss(const uint16_t* xb, const float* x, float* g, float* losses, int W,
                                int64_t P, int64_t ld, const lsgd_mlp_batch& b, const DeviceState& st,
                                hipStream_t s);
// the two halves of launch_mlp_grad_loss: forward pass + losses (+ output delta), then the backward pass,
// which writes g, or applies the update when fu->enabled
hipError_t launch_mlp_forward(const uint16_t* xb, const float* x, float* losses, int W, int64_t P, int64_t ld,
                              const lsgd_mlp_batch& b, const DeviceState& st, hipStream_t s);
hipError_t launch_mlp_backward(const uint16_t* xb, const float* x, float* g, int W, int64_t P, int64_t ld,
                               const lsgd_mlp_batch& b, const DeviceState& st, const FusedUpdate* fu, hipStream_t s);
bool mlp_shape_supported(const lsgd_mlp_batch& b, const char** why);

// ---- small device helpers ----
// fp32 -> bf16, round to nearest even, by the hardware conversion (two values per instruction)
typedef __bf16 lsgd_bf16x2 __attribute__((ext_vector_type(2)));
typedef float lsgd_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi)
{
    const lsgd_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, lsgd_bf16x2));
}
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float v) { return (uint16_t)(f32x2_to_bf16x2(v, 0.f) & 0xFFFFu); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

} // namespace lsgd
