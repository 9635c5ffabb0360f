// Host side of the C ABI declared in include/kvm.h: argument validation, workspace
// carving, error strings and kernel dispatch.  No allocation, no synchronisation.
#include <math.h>
#include <algorithm>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include "kvm_common.h"

namespace kvm {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

kvm_status check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("%s: launch failed: %s", what, hipGetErrorString(e));
        return KVM_ERR_LAUNCH;
    }
    return KVM_OK;
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- optional per-kernel timing ---------------------------------------------------------
struct ProfState {
    bool on = false;
    int cap = 0, used = 0;
    hipEvent_t *ev = nullptr;        // 2 per timed launch
    const char **names = nullptr;    // kernel name per timed launch (string literals)
};
static ProfState g_prof;

ProfScope::ProfScope(const char *name, hipStream_t s) : slot(-1), st(s)
{
    if (!g_prof.on || g_prof.used >= g_prof.cap) return;
    // a stream that is being captured into a graph is not timed: the event records would become
    // nodes of the caller's graph
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) return;
    slot = g_prof.used++;
    g_prof.names[slot] = name;
    (void)hipEventRecord(g_prof.ev[2 * slot], st);
}

ProfScope::~ProfScope()
{
    if (slot >= 0) (void)hipEventRecord(g_prof.ev[2 * slot + 1], st);
}

static kvm_status check_shape(const kvm_shape *sh, const char *fn)
{
    if (!sh) { set_error("%s: shape is NULL", fn); return KVM_ERR_INVALID_ARG; }
    if (sh->B < 0 || sh->H_kv < 1 || sh->G < 1 || sh->N < 0) {
        set_error("%s: invalid sizes B=%d H_kv=%d G=%d N=%d", fn, sh->B, sh->H_kv, sh->G, sh->N);
        return KVM_ERR_INVALID_ARG;
    }
    if (sh->d != HEAD_DIM) { set_error("%s: head dimension %d is not supported (only %d)", fn, sh->d, HEAD_DIM); return KVM_ERR_UNSUPPORTED; }
    if (sh->dtype != KVM_F32 && sh->dtype != KVM_F16 && sh->dtype != KVM_BF16) {
        set_error("%s: unknown dtype %d", fn, sh->dtype);
        return KVM_ERR_UNSUPPORTED;
    }
    // grids and int32 offsets inside a slice
    const long long slices = (long long)sh->B * sh->H_kv * sh->G;
    if (slices > (1ll << 24) || (long long)sh->N > (1ll << 22)) {
        set_error("%s: shape too large (B*H_kv*G=%lld, N=%d)", fn, slices, sh->N);
        return KVM_ERR_UNSUPPORTED;
    }
    return KVM_OK;
}

static kvm_status check_params(const kvm_params *pr, const char *fn)
{
    if (!pr) { set_error("%s: params is NULL", fn); return KVM_ERR_INVALID_ARG; }
    const bool ok = pr->budget >= 0.0 && pr->budget <= 1.0 && pr->recent_ratio >= 0.0 && pr->recent_ratio <= 1.0 &&
                    pr->heavy_ratio >= 0.0 && pr->heavy_ratio <= 1.0;
    if (!ok) {
        set_error("%s: budget/recent_ratio/heavy_ratio must lie in [0,1] (%g, %g, %g)", fn, pr->budget,
                  pr->recent_ratio, pr->heavy_ratio);
        return KVM_ERR_INVALID_ARG;
    }
    if (pr->enforce_budget && pr->recent_ratio + pr->heavy_ratio > pr->budget) {
        set_error("%s: recent_ratio + heavy_ratio = %g exceeds the budget %g", fn, pr->recent_ratio + pr->heavy_ratio,
                  pr->budget);
        return KVM_ERR_INVALID_ARG;
    }
    if (!(pr->threshold == pr->threshold)) { set_error("%s: threshold is NaN", fn); return KVM_ERR_INVALID_ARG; }
    if (pr->sigma_mode != KVM_SIGMA_MEAN_DIST && pr->sigma_mode != KVM_SIGMA_FIXED) {
        set_error("%s: unknown sigma_mode %d", fn, pr->sigma_mode);
        return KVM_ERR_UNSUPPORTED;
    }
    if (pr->weights != KVM_WEIGHTS_GAUSSIAN && pr->weights != KVM_WEIGHTS_AVERAGE) {
        set_error("%s: unknown weights %d", fn, pr->weights);
        return KVM_ERR_UNSUPPORTED;
    }
    if (pr->set_rule != KVM_SETS_ADJACENT && pr->set_rule != KVM_SETS_ANCHOR) {
        set_error("%s: unknown set_rule %d", fn, pr->set_rule);
        return KVM_ERR_UNSUPPORTED;
    }
    if (pr->pivot_rule < KVM_PIVOT_MAX_SCORE || pr->pivot_rule > KVM_PIVOT_RANDOM) {
        set_error("%s: unknown pivot_rule %d", fn, pr->pivot_rule);
        return KVM_ERR_UNSUPPORTED;
    }
    if (pr->sigma_mode == KVM_SIGMA_FIXED && !(pr->sigma > 0.f)) {
        set_error("%s: fixed sigma must be > 0 (%g)", fn, (double)pr->sigma);
        return KVM_ERR_INVALID_ARG;
    }
    return KVM_OK;
}

static int capacity(const kvm_shape *sh, const kvm_params *pr)
{
    return pr->enforce_budget ? (int)floor(pr->budget * (double)sh->N) : sh->N;
}

static size_t ws_attn(const kvm_shape *sh)
{
    // row statistics, then one flag per (query slice, row tile); the decode-time update keeps its
    // scores in the first part and two floats per (query slice, 64 keys) in the second, which is
    // the larger need
    const size_t q_slices = (size_t)sh->B * sh->H_kv * sh->G;
    const size_t second = std::max((size_t)attn_row_tiles(sh->N), (size_t)attn_lse_stride(sh->N) / 64 * 2);
    return align_up(q_slices * attn_lse_stride(sh->N) * sizeof(float) + q_slices * second * sizeof(float), 256);
}
static size_t ws_identify(const kvm_shape *sh)
{
    const size_t tok = (size_t)sh->B * sh->H_kv * sh->N;
    // adjacent similarities, inverse key norms, run lengths of the anchor rule, flag bytes
    return 3 * align_up(tok * sizeof(float), 256) + align_up(tok, 256);
}

}  // namespace kvm

using namespace kvm;

extern "C" {

kvm_status kvm_params_for_budget(double budget, kvm_params *out)
{
    if (!out || !(budget > 0.0 && budget <= 1.0)) {
        set_error("kvm_params_for_budget: need out != NULL and 0 < budget <= 1");
        return KVM_ERR_INVALID_ARG;
    }
    memset(out, 0, sizeof(*out));
    out->budget = budget;
    if (budget == 0.5) { out->recent_ratio = 0.17; out->heavy_ratio = 0.12; }
    else if (budget == 0.35) { out->recent_ratio = 0.08; out->heavy_ratio = 0.02; }
    else { out->recent_ratio = 0.34 * budget; out->heavy_ratio = 0.24 * budget; }
    out->threshold = 0.75f;
    out->sigma_mode = KVM_SIGMA_MEAN_DIST;
    out->sigma = 0.f;
    out->value_scale_by_set_size = 1;
    out->enforce_budget = 1;
    out->weights = KVM_WEIGHTS_GAUSSIAN;
    out->pivot_rule = KVM_PIVOT_MAX_SCORE;
    out->pivot_seed = 0;
    out->set_rule = KVM_SETS_ADJACENT;
    out->sim_given = 0;
    return KVM_OK;
}

int32_t kvm_out_capacity(const kvm_shape *shape, const kvm_params *params)
{
    if (check_shape(shape, "kvm_out_capacity") != KVM_OK || check_params(params, "kvm_out_capacity") != KVM_OK) return -1;
    return capacity(shape, params);
}

size_t kvm_workspace_bytes(const kvm_shape *shape, const kvm_params *params)
{
    if (check_shape(shape, "kvm_workspace_bytes") != KVM_OK) return 0;
    // (the refresh of a compacted cache needs two ints per output row on top of the merge plan; without
    // params the capacity is taken as N)
    const int cap = params && check_params(params, "kvm_workspace_bytes") == KVM_OK ? capacity(shape, params) : shape->N;
    const size_t a = ws_attn(shape), b = ws_identify(shape), c = merge_refresh_workspace_bytes(*shape, cap);
    return (a > b ? (a > c ? a : c) : (b > c ? b : c)) + 256;
}

static kvm_status attn_mass_entry(const char *who, const kvm_shape *shape, const void *Q, const void *K, const float *row_lse,
                                  bool with_lse, float *mass, float *sim, bool with_sim, void *ws, size_t ws_bytes,
                                  void *stream)
{
    kvm_status rc = check_shape(shape, who);
    if (rc != KVM_OK) return rc;
    const bool empty = (long long)shape->B * shape->N == 0;
    if (!empty && (!Q || !K || !mass || (with_lse && !row_lse))) {
        set_error("%s: Q, K%s and mass must not be NULL", who, with_lse ? ", row_lse" : "");
        return KVM_ERR_INVALID_ARG;
    }
    if (!empty && with_sim && !sim) {
        set_error("%s: sim must not be NULL", who);
        return KVM_ERR_INVALID_ARG;
    }
    if (empty) return KVM_OK;
    if (!ws || ws_bytes < ws_attn(shape)) {
        set_error("%s: workspace of %zu bytes needed, %zu given", who, ws_attn(shape), ws ? ws_bytes : (size_t)0);
        return KVM_ERR_WORKSPACE;
    }
    return launch_attn_mass(*shape, Q, K, with_lse ? row_lse : nullptr, mass, (float *)ws, with_sim ? sim : nullptr,
                            (hipStream_t)stream);
}

kvm_status kvm_attn_mass(const kvm_shape *shape, const void *Q, const void *K, float *mass, void *ws, size_t ws_bytes,
                         void *stream)
{
    return attn_mass_entry("kvm_attn_mass", shape, Q, K, nullptr, false, mass, nullptr, false, ws, ws_bytes, stream);
}

kvm_status kvm_attn_mass_sim(const kvm_shape *shape, const void *Q, const void *K, float *mass, float *sim, void *ws,
                             size_t ws_bytes, void *stream)
{
    return attn_mass_entry("kvm_attn_mass_sim", shape, Q, K, nullptr, false, mass, sim, true, ws, ws_bytes, stream);
}

kvm_status kvm_attn_mass_from_lse(const kvm_shape *shape, const void *Q, const void *K, const float *row_lse, float *mass,
                                  void *ws, size_t ws_bytes, void *stream)
{
    return attn_mass_entry("kvm_attn_mass_from_lse", shape, Q, K, row_lse, true, mass, nullptr, false, ws, ws_bytes, stream);
}

kvm_status kvm_attn_mass_append(const kvm_shape *shape, const void *q_new, const void *K, float *mass, void *ws,
                                size_t ws_bytes, void *stream)
{
    kvm_status rc = check_shape(shape, "kvm_attn_mass_append");
    if (rc != KVM_OK) return rc;
    if ((long long)shape->B * shape->N == 0) return KVM_OK;
    if (!q_new || !K || !mass) { set_error("kvm_attn_mass_append: q_new, K and mass must not be NULL"); return KVM_ERR_INVALID_ARG; }
    if (!ws || ws_bytes < ws_attn(shape)) {
        set_error("kvm_attn_mass_append: workspace of %zu bytes needed, %zu given", ws_attn(shape), ws ? ws_bytes : (size_t)0);
        return KVM_ERR_WORKSPACE;
    }
    return launch_attn_append(*shape, q_new, K, mass, (float *)ws, (hipStream_t)stream);
}

kvm_status kvm_sim_append(const kvm_shape *shape, const void *K, float *sim, void *stream)
{
    kvm_status rc = check_shape(shape, "kvm_sim_append");
    if (rc != KVM_OK) return rc;
    if ((long long)shape->B * shape->N == 0) return KVM_OK;
    if (!K || !sim) { set_error("kvm_sim_append: K and sim must not be NULL"); return KVM_ERR_INVALID_ARG; }
    return launch_sim_append(*shape, K, sim, (hipStream_t)stream);
}

kvm_status kvm_identify_sets(const kvm_shape *shape, const kvm_params *params, const void *K, const float *mass,
                             int32_t *set_id, int32_t *set_start, int32_t *pivot, int32_t *n_sets, float *sim_opt,
                             int32_t *slice_status, void *ws, size_t ws_bytes, void *stream)
{
    kvm_status rc = check_shape(shape, "kvm_identify_sets");
    if (rc != KVM_OK) return rc;
    rc = check_params(params, "kvm_identify_sets");
    if (rc != KVM_OK) return rc;
    if (shape->B == 0) return KVM_OK;
    if (!set_start || !n_sets || !slice_status || (capacity(shape, params) > 0 && !pivot) ||
        (shape->N > 0 && ((!K && !params->sim_given) || !mass || !set_id))) {
        set_error("kvm_identify_sets: a required pointer is NULL");
        return KVM_ERR_INVALID_ARG;
    }
    if (params->sim_given && (!sim_opt || params->set_rule != KVM_SETS_ADJACENT)) {
        set_error("kvm_identify_sets: sim_given needs sim_opt and the adjacent set rule");
        return KVM_ERR_INVALID_ARG;
    }
    if (ws_identify(shape) > 0 && (!ws || ws_bytes < ws_identify(shape))) {
        set_error("kvm_identify_sets: workspace of %zu bytes needed, %zu given", ws_identify(shape), ws ? ws_bytes : (size_t)0);
        return KVM_ERR_WORKSPACE;
    }
    const size_t tok = (size_t)shape->B * shape->H_kv * shape->N;
    float *sim = sim_opt ? sim_opt : (float *)ws;
    const size_t stride = align_up(tok * sizeof(float), 256);
    float *inv_norm = (float *)((uint8_t *)ws + stride);
    int32_t *run = (int32_t *)((uint8_t *)ws + 2 * stride);
    uint8_t *flags = (uint8_t *)ws + 3 * stride;
    return launch_identify(*shape, *params, capacity(shape, params), K, mass, set_id, set_start, pivot, n_sets, sim,
                           inv_norm, run, flags, slice_status, (hipStream_t)stream);
}

static kvm_status evict_common(const char *fn, bool merge_values, const kvm_shape *shape, const kvm_params *params, const void *K,
                               const void *V, const float *mass, int32_t *kept, int32_t *n_kept, void *K_out, void *V_out,
                               void *ws, size_t ws_bytes, void *stream)
{
    kvm_status rc = check_shape(shape, fn);
    if (rc != KVM_OK) return rc;
    rc = check_params(params, fn);
    if (rc != KVM_OK) return rc;
    if (shape->B == 0) return KVM_OK;
    const int cap = capacity(shape, params);
    if (!n_kept || (cap > 0 && (!kept || !K_out || !V_out)) || (shape->N > 0 && (!K || !V || !mass))) {
        set_error("%s: a required pointer is NULL", fn);
        return KVM_ERR_INVALID_ARG;
    }
    if (ws_identify(shape) > 0 && (!ws || ws_bytes < ws_identify(shape))) {
        set_error("%s: workspace of %zu bytes needed, %zu given", fn, ws_identify(shape), ws ? ws_bytes : (size_t)0);
        return KVM_ERR_WORKSPACE;
    }
    const size_t tok = (size_t)shape->B * shape->H_kv * shape->N;
    uint8_t *flags = (uint8_t *)ws + 3 * align_up(tok * sizeof(float), 256);
    return launch_evict(*shape, *params, cap, K, V, mass, kept, n_kept, K_out, V_out, flags, merge_values, (hipStream_t)stream);
}

kvm_status kvm_evict(const kvm_shape *shape, const kvm_params *params, const void *K, const void *V, const float *mass,
                     int32_t *kept, int32_t *n_kept, void *K_out, void *V_out, void *ws, size_t ws_bytes, void *stream)
{
    return evict_common("kvm_evict", false, shape, params, K, V, mass, kept, n_kept, K_out, V_out, ws, ws_bytes, stream);
}

kvm_status kvm_evict_merge_values(const kvm_shape *shape, const kvm_params *params, const void *K, const void *V,
                                  const float *mass, int32_t *kept, int32_t *n_kept, void *K_out, void *V_out, void *ws,
                                  size_t ws_bytes, void *stream)
{
    return evict_common("kvm_evict_merge_values", true, shape, params, K, V, mass, kept, n_kept, K_out, V_out, ws, ws_bytes,
                        stream);
}

kvm_status kvm_merge(const kvm_shape *shape, const kvm_params *params, const void *K, const void *V,
                     const int32_t *set_start, const int32_t *pivot, const int32_t *n_sets, void *K_out, void *V_out,
                     float *w_opt, void *ws, size_t ws_bytes, void *stream)
{
    kvm_status rc = check_shape(shape, "kvm_merge");
    if (rc != KVM_OK) return rc;
    rc = check_params(params, "kvm_merge");
    if (rc != KVM_OK) return rc;
    const int cap = capacity(shape, params);
    if ((long long)shape->B * shape->N == 0 || cap == 0) return KVM_OK;
    if (!K || !V || !set_start || !pivot || !n_sets || !K_out || !V_out) {
        set_error("kvm_merge: a required pointer is NULL");
        return KVM_ERR_INVALID_ARG;
    }
    if (!ws || ws_bytes < merge_workspace_bytes(*shape)) {
        set_error("kvm_merge: workspace of %zu bytes needed, %zu given", merge_workspace_bytes(*shape), ws ? ws_bytes : (size_t)0);
        return KVM_ERR_WORKSPACE;
    }
    return launch_merge(*shape, *params, cap, K, V, set_start, pivot, n_sets, K_out, V_out, w_opt, (int32_t *)ws,
                        (hipStream_t)stream);
}

kvm_status kvm_merge_refresh(const kvm_shape *shape, const kvm_params *params, const void *K, const void *V,
                             const int32_t *prev_set_id, const int32_t *prev_set_start, const int32_t *prev_pivot,
                             const int32_t *prev_n_sets, const int32_t *set_start, const int32_t *pivot, const int32_t *n_sets,
                             void *K_out, void *V_out, int32_t *n_changed_opt, void *ws, size_t ws_bytes, void *stream)
{
    kvm_status rc = check_shape(shape, "kvm_merge_refresh");
    if (rc != KVM_OK) return rc;
    rc = check_params(params, "kvm_merge_refresh");
    if (rc != KVM_OK) return rc;
    const int cap = capacity(shape, params);
    if ((long long)shape->B * shape->N == 0 || cap == 0) return KVM_OK;
    if (!K || !V || !prev_set_id || !prev_set_start || !prev_pivot || !prev_n_sets || !set_start || !pivot || !n_sets || !K_out ||
        !V_out) {
        set_error("kvm_merge_refresh: a required pointer is NULL");
        return KVM_ERR_INVALID_ARG;
    }
    if (prev_set_start == set_start || prev_pivot == pivot || prev_n_sets == n_sets) {
        set_error("kvm_merge_refresh: the previous and the new maps must be different buffers");
        return KVM_ERR_INVALID_ARG;
    }
    const size_t need = merge_refresh_workspace_bytes(*shape, cap);
    if (!ws || ws_bytes < need) {
        set_error("kvm_merge_refresh: workspace of %zu bytes needed, %zu given", need, ws ? ws_bytes : (size_t)0);
        return KVM_ERR_WORKSPACE;
    }
    return launch_merge_refresh(*shape, *params, cap, K, V, prev_set_id, prev_set_start, prev_pivot, prev_n_sets, set_start, pivot,
                                n_sets, K_out, V_out, n_changed_opt, (int32_t *)ws, (hipStream_t)stream);
}

kvm_status kvm_merge_static(const kvm_shape *shape, const kvm_params *params, const void *K, const void *V,
                            const int32_t *set_start, const int32_t *pivot, const int32_t *n_sets, void *K_out, void *V_out,
                            float *w_opt, void *stream)
{
    kvm_status rc = check_shape(shape, "kvm_merge_static");
    if (rc != KVM_OK) return rc;
    rc = check_params(params, "kvm_merge_static");
    if (rc != KVM_OK) return rc;
    const int cap = capacity(shape, params);
    if ((long long)shape->B * shape->N == 0 || cap == 0) return KVM_OK;
    if (!K || !V || !set_start || !pivot || !n_sets || !K_out || !V_out) {
        set_error("kvm_merge_static: a required pointer is NULL");
        return KVM_ERR_INVALID_ARG;
    }
    return launch_merge_static(*shape, *params, cap, K, V, set_start, pivot, n_sets, K_out, V_out, w_opt, (hipStream_t)stream);
}

kvm_status kvm_profile_disable(void)
{
    if (g_prof.ev) {
        for (int i = 0; i < 2 * g_prof.cap; ++i) (void)hipEventDestroy(g_prof.ev[i]);
        delete[] g_prof.ev;
        delete[] g_prof.names;
    }
    g_prof = ProfState();
    return KVM_OK;
}

kvm_status kvm_profile_enable(int32_t max_launches)
{
    kvm_profile_disable();
    if (max_launches < 1 || max_launches > (1 << 20)) {
        set_error("kvm_profile_enable: max_launches must lie in [1, 2^20]");
        return KVM_ERR_INVALID_ARG;
    }
    g_prof.ev = new hipEvent_t[2 * (size_t)max_launches];
    g_prof.names = new const char *[max_launches];
    for (int i = 0; i < 2 * max_launches; ++i) {
        if (hipEventCreate(&g_prof.ev[i]) != hipSuccess) {
            for (int j = 0; j < i; ++j) (void)hipEventDestroy(g_prof.ev[j]);   // cap is still 0: disable frees the arrays only
            kvm_profile_disable();
            set_error("kvm_profile_enable: hipEventCreate failed");
            return KVM_ERR_LAUNCH;
        }
    }
    g_prof.cap = max_launches;
    g_prof.used = 0;
    g_prof.on = true;
    return KVM_OK;
}

int32_t kvm_profile_collect(kvm_kernel_time *out, int32_t max_records)
{
    if (!g_prof.on || !out || max_records < 1) return 0;
    int n = 0;
    for (int i = 0; i < g_prof.used; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(g_prof.ev[2 * i + 1]) != hipSuccess) continue;
        if (hipEventElapsedTime(&ms, g_prof.ev[2 * i], g_prof.ev[2 * i + 1]) != hipSuccess) continue;
        int r = 0;
        while (r < n && strcmp(out[r].name, g_prof.names[i]) != 0) ++r;
        if (r == n) {
            if (n == max_records) continue;
            memset(&out[n], 0, sizeof(out[n]));
            strncpy(out[n].name, g_prof.names[i], sizeof(out[n].name) - 1);
            ++n;
        }
        out[r].launches += 1;
        out[r].total_ms += ms;
    }
    g_prof.used = 0;
    return n;
}

const char *kvm_last_error(void) { return g_err; }

const char *kvm_version(void) { return "0.1.0"; }

}  // extern "C"
