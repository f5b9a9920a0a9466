// Host-side arithmetic of the GPU allocation modes (section IV-A): rollout time of the collocated mode
// and of the hybrid mode with two-stage fine-grained pipelining, profile lookup, and the search over
// (k, N_G, N_S).  No device work.
#include "../../include/vla.h"
#include "vla_internal.h"

#include <cmath>

extern "C" {

// k = 1: the two components alternate, m (t_G + t_S).  k = 2: two sub-batches take turns; after its
// first start the slower component never idles, the faster one adds one step at the start (generation)
// or the end (simulation): 2 m max(t_G, t_S) + min(t_G, t_S).
int vla_pipeline_time(double t_gen, double t_sim, int k, int m_chunks, double *out) {
    if (!out) { vla_set_error("vla_pipeline_time: out is NULL"); return VLA_EINVAL; }
    if (!(t_gen >= 0) || !(t_sim >= 0) || m_chunks < 0) {
        vla_set_error("vla_pipeline_time: negative or NaN time, or negative step count");
        return VLA_EINVAL;
    }
    if (k != 1 && k != 2) { vla_set_error("vla_pipeline_time: k = %d unsupported (1 or 2 pipeline stages)", k); return VLA_EINVAL; }
    if (m_chunks == 0) { *out = 0.0; return VLA_OK; }
    if (k == 1) *out = m_chunks * (t_gen + t_sim);
    else *out = 2.0 * m_chunks * std::fmax(t_gen, t_sim) + std::fmin(t_gen, t_sim);
    return VLA_OK;
}

int vla_profile_lookup(const double *profile, int n_prof, double batch, double *out) {
    if (!profile || !out || n_prof < 1 || n_prof > 30) { vla_set_error("vla_profile_lookup: NULL pointer or n_prof outside 1..30"); return VLA_EINVAL; }
    const double top = (double)(1u << (n_prof - 1));
    if (!(batch >= 1.0) || batch > top) {
        vla_set_error("vla_profile_lookup: batch %g outside the profiled range 1..%g", batch, top);
        return VLA_ESHAPE;
    }
    int i = 0;
    while (i + 1 < n_prof && (double)(1u << (i + 1)) <= batch) i++;
    const double lo = (double)(1u << i);
    if (batch == lo) { *out = profile[i]; return VLA_OK; }
    const double hi = (double)(1u << (i + 1));
    const double w = (batch - lo) / (hi - lo);
    *out = profile[i] * (1.0 - w) + profile[i + 1] * w;
    return VLA_OK;
}

int vla_auto_placement(const double *t_gen, const double *t_sim, int n_prof, int n_envs, int n_gpus, int m_chunks,
                       vla_placement *best, vla_placement *all, int all_cap, int *n_all) {
    if (!t_gen || !t_sim || !best) { vla_set_error("vla_auto_placement: NULL pointer"); return VLA_EINVAL; }
    if (n_prof < 1 || n_prof > 30 || n_envs < 1 || n_gpus < 1 || m_chunks < 1 || all_cap < 0 || (all_cap > 0 && !all)) {
        vla_set_error("vla_auto_placement: non-positive size");
        return VLA_EINVAL;
    }
    int count = 0, rc;
    bool have = false;
    auto consider = [&](int k, int n_g, int n_s, double g, double s) -> int {
        vla_placement c{k, n_g, n_s, 0.0};
        if ((rc = vla_pipeline_time(g, s, k, m_chunks, &c.time))) return rc;
        if (all && count < all_cap) all[count] = c;
        count++;
        if (!have || c.time < best->time) { *best = c; have = true; }
        return VLA_OK;
    };
    auto per_gpu = [&](int parts) { return (n_envs + parts - 1) / parts; };
    if (n_envs >= n_gpus) {
        double g, s;
        if ((rc = vla_profile_lookup(t_gen, n_prof, per_gpu(n_gpus), &g))) return rc;
        if ((rc = vla_profile_lookup(t_sim, n_prof, per_gpu(n_gpus), &s))) return rc;
        if ((rc = consider(1, n_gpus, n_gpus, g, s))) return rc;
    }
    for (int n_g = 1; n_g < n_gpus; n_g++) {
        const int n_s = n_gpus - n_g;
        if (n_envs < 2 * n_g || n_envs < 2 * n_s) continue;
        double g, s;
        if ((rc = vla_profile_lookup(t_gen, n_prof, per_gpu(2 * n_g), &g))) return rc;
        if ((rc = vla_profile_lookup(t_sim, n_prof, per_gpu(2 * n_s), &s))) return rc;
        if ((rc = consider(2, n_g, n_s, g, s))) return rc;
    }
    if (n_all) *n_all = count;
    if (!have) { vla_set_error("vla_auto_placement: no feasible placement (fewer environments than GPUs)"); return VLA_ESHAPE; }
    return VLA_OK;
}

}  // extern "C"
