// Advantage estimators, clipped policy objective and log-probability aggregation on the device
// (fp32): the consumers of vla_logprob_recompute's outputs in the PPO / GRPO update.  All of it is
// a few bytes per step, so the kernels are simple and deterministic (fixed-order reductions, no
// atomics); one workgroup-level tree per trajectory, one final workgroup over trajectories.
#include "vla_internal.h"

namespace {

__device__ __forceinline__ float block_sum_256(float v, float *red) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// One thread per trajectory walks it backwards: A_t = delta_t + gamma * lambda * (1 - done_t) * A_{t+1}.
__global__ void gae_kernel(const float *rewards, const float *values, const int32_t *dones, int n, int T,
                           float gamma, float lambda, float *adv, float *returns) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float *r = rewards + (size_t)i * T, *v = values + (size_t)i * (T + 1);
    const int32_t *d = dones ? dones + (size_t)i * T : nullptr;
    float next = 0.f;
    for (int t = T - 1; t >= 0; t--) {
        const float cont = (d && d[t]) ? 0.f : 1.f;
        const float delta = r[t] + gamma * v[t + 1] * cont - v[t];
        next = delta + gamma * lambda * cont * next;
        adv[(size_t)i * T + t] = next;
        if (returns) returns[(size_t)i * T + t] = next + v[t];
    }
}

// One thread per group: population mean / standard deviation of its G returns.
__global__ void grpo_advantage_kernel(const float *R, int n_groups, int G, float *adv, int32_t *keep) {
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= n_groups) return;
    const float *r = R + (size_t)g * G;
    float mean = 0.f, lo = r[0], hi = r[0];
    for (int i = 0; i < G; i++) { mean += r[i]; lo = fminf(lo, r[i]); hi = fmaxf(hi, r[i]); }
    mean /= (float)G;
    float var = 0.f;
    for (int i = 0; i < G; i++) var += (r[i] - mean) * (r[i] - mean);
    const float sd = sqrtf(var / (float)G);
    // a group of identical returns is recognised by max == min: the rounded mean of equal values that fp32 does
    // not represent exactly (0.1 x G) can differ from them and leave a tiny non-zero deviation
    const bool spread = hi > lo && sd > 0.f;
    for (int i = 0; i < G; i++) adv[(size_t)g * G + i] = spread ? (r[i] - mean) / sd : 0.f;
    if (keep) keep[g] = spread ? 1 : 0;
}

// One workgroup per trajectory: sums of the masked surrogate, the valid count and the clipped count.
__global__ void __launch_bounds__(256) objective_rows_kernel(const float *logp_new, const float *logp_old,
                                                            const float *adv, int adv_per_step,
                                                            const int32_t *mask, int T, float lo, float hi,
                                                            float *per_step, float *rows /*[n][3]*/) {
    __shared__ float red[4];
    const int i = blockIdx.x;
    float s = 0.f, cnt = 0.f, clipped = 0.f;
    for (int t = threadIdx.x; t < T; t += 256) {
        const size_t o = (size_t)i * T + t;
        // a masked step is never read: padding may hold anything (NaN, inf), and NaN * 0 would poison the sums
        if (mask && !mask[o]) {
            if (per_step) per_step[o] = 0.f;
            continue;
        }
        const float a = adv_per_step ? adv[o] : adv[i];
        const float rho = expf(logp_new[o] - logp_old[o]);
        const float u = rho * a, c = fminf(fmaxf(rho, lo), hi) * a;
        const float v = fminf(u, c);
        if (per_step) per_step[o] = v;
        s += v; cnt += 1.f; clipped += (c < u) ? 1.f : 0.f;
    }
    s = block_sum_256(s, red);
    cnt = block_sum_256(cnt, red);
    clipped = block_sum_256(clipped, red);
    if (threadIdx.x == 0) { rows[i * 3] = s; rows[i * 3 + 1] = cnt; rows[i * 3 + 2] = clipped; }
}

// One workgroup combines the trajectories in a fixed order.
__global__ void __launch_bounds__(256) objective_final_kernel(const float *rows, int n, int per_trajectory,
                                                             float *objective, float *clip_frac) {
    __shared__ float red[4];
    float s = 0.f, cnt = 0.f, clipped = 0.f;
    for (int i = threadIdx.x; i < n; i += 256) {
        const float si = rows[i * 3], ci = rows[i * 3 + 1];
        s += per_trajectory ? (ci > 0.f ? si / ci : 0.f) : si;
        cnt += ci; clipped += rows[i * 3 + 2];
    }
    s = block_sum_256(s, red);
    cnt = block_sum_256(cnt, red);
    clipped = block_sum_256(clipped, red);
    if (threadIdx.x == 0) {
        *objective = per_trajectory ? s / (float)n : (cnt > 0.f ? s / cnt : 0.f);
        if (clip_frac) *clip_frac = cnt > 0.f ? clipped / cnt : 0.f;
    }
}

__global__ void logp_aggregate_kernel(const float *logp, size_t n_out, int inner, float *out) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_out) return;
    float s = 0.f;
    for (int j = 0; j < inner; j++) s += logp[i * inner + j];
    out[i] = s;
}

// Scratch of vla_policy_objective_noalloc: the per-trajectory partial sums [n][3] that the workspace argument of
// vla_policy_objective otherwise brings in.  One copy per GPU that loads the library, held until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress; kernels are handed the address it returns.
constexpr int NOALLOC_MAX_TRAJ = 65536;
__device__ __align__(256) float scratch[NOALLOC_MAX_TRAJ * 3];

constexpr int MAX_DEVICES = 64;
float *g_scratch_ptr[MAX_DEVICES] = {};          // device address of `scratch` on each GPU, looked up on first use

// Device address of this GPU's copy of `scratch` (the current device's), or NULL with the error set.
float *scratch_of_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        vla_set_error("policy_objective_noalloc: cannot identify the current device");
        return nullptr;
    }
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            vla_set_error("policy_objective_noalloc: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
            return nullptr;
        }
        g_scratch_ptr[dev] = (float *)p;
    }
    return g_scratch_ptr[dev];
}

int policy_objective_launch(const float *logp_new, const float *logp_old, const float *adv, int adv_per_step,
                            const int32_t *mask, int n_traj, int T, float clip_low, float clip_high, int per_trajectory,
                            float *rows, float *objective, float *per_step, float *clip_frac, hipStream_t st) {
    objective_rows_kernel<<<n_traj, 256, 0, st>>>(logp_new, logp_old, adv, adv_per_step, mask, T, 1.0f - clip_low,
                                                  1.0f + clip_high, per_step, rows);
    int rc = vla_check_launch("policy_objective_rows");
    if (rc) return rc;
    objective_final_kernel<<<1, 256, 0, st>>>(rows, n_traj, per_trajectory, objective, clip_frac);
    return vla_check_launch("policy_objective_final");
}

}  // namespace

extern "C" {

int vla_gae(const float *rewards, const float *values, const int32_t *dones, int n, int T, float gamma,
            float lambda, float *adv, float *returns, void *stream) {
    if (!rewards || !values || !adv) { vla_set_error("gae: rewards, values or adv is NULL"); return VLA_EINVAL; }
    if (n <= 0 || T <= 0) { vla_set_error("gae: n and T must be positive"); return VLA_EINVAL; }
    gae_kernel<<<(n + 63) / 64, 64, 0, (hipStream_t)stream>>>(rewards, values, dones, n, T, gamma, lambda, adv, returns);
    return vla_check_launch("gae");
}

int vla_grpo_advantage(const float *total_reward, int n_groups, int G, float *adv, int32_t *keep, void *stream) {
    if (!total_reward || !adv) { vla_set_error("grpo_advantage: total_reward or adv is NULL"); return VLA_EINVAL; }
    if (n_groups <= 0 || G <= 0) { vla_set_error("grpo_advantage: n_groups and G must be positive"); return VLA_EINVAL; }
    grpo_advantage_kernel<<<(n_groups + 63) / 64, 64, 0, (hipStream_t)stream>>>(total_reward, n_groups, G, adv, keep);
    return vla_check_launch("grpo_advantage");
}

size_t vla_policy_objective_workspace_bytes(int n_traj) { return n_traj > 0 ? (size_t)n_traj * 3 * sizeof(float) : 0; }

int vla_policy_objective(const float *logp_new, const float *logp_old, const float *adv, int adv_per_step,
                         const int32_t *mask, int n_traj, int T, float clip_low, float clip_high,
                         int per_trajectory, void *ws, size_t ws_bytes, float *objective, float *per_step,
                         float *clip_frac, void *stream) {
    if (!logp_new || !logp_old || !adv || !objective || !ws) {
        vla_set_error("policy_objective: logp_new, logp_old, adv, objective or ws is NULL");
        return VLA_EINVAL;
    }
    if (n_traj <= 0 || T <= 0 || !(clip_low >= 0.f) || !(clip_high >= 0.f)) {
        vla_set_error("policy_objective: sizes must be positive and clip ratios non-negative");
        return VLA_EINVAL;
    }
    if (ws_bytes < vla_policy_objective_workspace_bytes(n_traj)) {
        vla_set_error("policy_objective: workspace %zu bytes, need %zu", ws_bytes, vla_policy_objective_workspace_bytes(n_traj));
        return VLA_EWORKSPACE;
    }
    return policy_objective_launch(logp_new, logp_old, adv, adv_per_step, mask, n_traj, T, clip_low, clip_high,
                                   per_trajectory, (float *)ws, objective, per_step, clip_frac, (hipStream_t)stream);
}

int vla_policy_objective_noalloc_max_traj(void) { return NOALLOC_MAX_TRAJ; }

int vla_policy_objective_noalloc(const float *logp_new, const float *logp_old, const float *adv, int adv_per_step,
                                 const int32_t *mask, int n_traj, int T, float clip_low, float clip_high,
                                 int per_trajectory, float *objective, float *per_step, float *clip_frac, void *stream) {
    if (!logp_new || !logp_old || !adv || !objective) {
        vla_set_error("policy_objective_noalloc: logp_new, logp_old, adv or objective is NULL");
        return VLA_EINVAL;
    }
    if (n_traj <= 0 || T <= 0 || !(clip_low >= 0.f) || !(clip_high >= 0.f)) {
        vla_set_error("policy_objective_noalloc: sizes must be positive and clip ratios non-negative");
        return VLA_EINVAL;
    }
    if (n_traj > NOALLOC_MAX_TRAJ) {
        vla_set_error("policy_objective_noalloc: %d trajectories exceed the built-in scratch of %d; use "
                      "vla_policy_objective with a workspace", n_traj, NOALLOC_MAX_TRAJ);
        return VLA_ESHAPE;
    }
    float *rows = scratch_of_current_device();
    if (!rows) return VLA_EHIP;
    // every slot below n_traj is written by the first kernel before the second reads it, so what an earlier call
    // left in the array is never seen and nothing has to be cleared
    return policy_objective_launch(logp_new, logp_old, adv, adv_per_step, mask, n_traj, T, clip_low, clip_high,
                                   per_trajectory, rows, objective, per_step, clip_frac, (hipStream_t)stream);
}

int vla_logp_aggregate(const float *logp, size_t n_out, int inner, float *out, void *stream) {
    if (!logp || !out) { vla_set_error("logp_aggregate: logp or out is NULL"); return VLA_EINVAL; }
    if (n_out == 0 || inner <= 0) { vla_set_error("logp_aggregate: sizes must be positive"); return VLA_EINVAL; }
    logp_aggregate_kernel<<<(unsigned)((n_out + 255) / 256), 256, 0, (hipStream_t)stream>>>(logp, n_out, inner, out);
    return vla_check_launch("logp_aggregate");
}

}  // extern "C"
