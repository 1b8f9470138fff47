// C-ABI entry points of libppow: host-side validation and kernel launches.
// Nothing here allocates device memory or synchronises.
#include <stdarg.h>
#include <stdio.h>

#include "ppow_device.h"

#include <math.h>

#include <mutex>

// ---- scratch of the entry point that allocates nothing -----------------------------------
// Same layout as the caller-supplied workspace of ppow_score_windows: the cluster kernel's
// exchange words, then one record per (window, position).  Every device the library runs on
// holds its own copy of the array, at its own address, until the process ends.  In host code
// the name `scratch` is only a handle for hipGetSymbolAddress, never a device address.
constexpr size_t kStaticScratchBytes =
    ppow::kClusterScratchBytes + static_cast<size_t>(PPOW_STATIC_MAX_ROWS) * sizeof(ppow::RowRecord);
static_assert(kStaticScratchBytes == PPOW_STATIC_SCRATCH_BYTES, "header states the size");
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

thread_local char g_error[256] = "";
thread_local const char *g_row_kernel = "none";

int fail(ppow_status code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof g_error, fmt, ap);
    va_end(ap);
    return code;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool sizes_ok(int64_t B, int32_t K, int64_t V, int32_t dtype) {
    if (B < 0 || K < 1 || K > PPOW_MAX_K || V < 2 || V > INT32_MAX) return false;
    if (dtype != PPOW_F32 && dtype != PPOW_BF16) return false;
    if (B > INT32_MAX / K) return false;            // B*K positions are indexed with 32 bits
    return true;
}

}  // namespace

extern "C" {

const char *ppow_last_error(void) { return g_error; }

const char *ppow_version(void) { return "0.3.0"; }

const char *ppow_last_row_kernel(void) { return g_row_kernel; }

size_t ppow_score_workspace_bytes(int64_t B, int32_t K, int64_t V, int32_t dtype, uint32_t flags) {
    (void)flags;
    if (!sizes_ok(B, K, V, dtype)) return 0;
    // [scratch of the cluster kernel][one record per (window, position)]
    return ppow::kClusterScratchBytes +
           static_cast<size_t>(B) * static_cast<size_t>(K) * sizeof(ppow::RowRecord);
}

}  // extern "C"

namespace {

// Everything of a scoring call the host can check without the workspace.
int validate_score_args(const void *draft_logits, const void *target_logits,
                        const int32_t *draft_tokens, const float *uniforms, int64_t B, int32_t K,
                        int64_t V, int32_t dtype, const ppow_params *params,
                        const ppow_outputs *out) {
    if (!params || !out) return fail(PPOW_ERR_INVALID_ARG, "params and out must not be NULL");
    if (!sizes_ok(B, K, V, dtype))
        return fail(PPOW_ERR_INVALID_ARG,
                    "sizes out of range: B=%lld K=%d V=%lld dtype=%d (need B>=0, 1<=K<=%d, "
                    "2<=V<2^31, B*K<2^31, dtype f32|bf16)",
                    (long long)B, K, (long long)V, dtype, PPOW_MAX_K);
    if (params->verify != PPOW_VERIFY_REJECTION && params->verify != PPOW_VERIFY_GREEDY)
        return fail(PPOW_ERR_INVALID_ARG, "unknown verify mode %d", params->verify);
    if (params->flags & ~static_cast<uint32_t>(PPOW_FLAG_EXPECTED_ACCEPT | PPOW_FLAG_POLICY_TERMS))
        return fail(PPOW_ERR_INVALID_ARG, "unknown flag bits 0x%x", params->flags);
    if (!(params->cost_ratio > 0.f) || !isfinite(params->cost_ratio))
        return fail(PPOW_ERR_INVALID_ARG, "cost_ratio must be a positive finite number");
    if (!isfinite(params->prox_eps) || !isfinite(params->prox_eta))
        return fail(PPOW_ERR_INVALID_ARG, "prox_eps and prox_eta must be finite");
    if (B == 0) return PPOW_OK;                     // nothing to score: pointers may be NULL
    if (!draft_logits || !target_logits || !draft_tokens)
        return fail(PPOW_ERR_INVALID_ARG, "logits and draft_tokens must not be NULL");
    if (!aligned16(draft_logits) || !aligned16(target_logits))
        return fail(PPOW_ERR_INVALID_ARG, "logit base pointers must be 16-byte aligned");
    if (params->verify == PPOW_VERIFY_REJECTION && !uniforms)
        return fail(PPOW_ERR_INVALID_ARG, "uniforms must be given for rejection verification");
    if (!out->accepted_len || !out->r_speedup || !out->r_proximity || !out->adaw_score)
        return fail(PPOW_ERR_INVALID_ARG,
                    "accepted_len, r_speedup, r_proximity and adaw_score outputs are required");
    const bool second_pass = (params->flags & PPOW_FLAG_EXPECTED_ACCEPT) != 0;
    if (out->expected_accept && !second_pass)
        return fail(PPOW_ERR_INVALID_ARG,
                    "expected_accept output needs PPOW_FLAG_EXPECTED_ACCEPT");
    if (second_pass && !out->expected_accept)
        return fail(PPOW_ERR_INVALID_ARG,
                    "PPOW_FLAG_EXPECTED_ACCEPT needs the expected_accept output");
    const bool policy_terms = (params->flags & PPOW_FLAG_POLICY_TERMS) != 0;
    if (!policy_terms && (out->reverse_kl || out->alignment || out->reverse_kl_mean ||
                          out->alignment_mean))
        return fail(PPOW_ERR_INVALID_ARG,
                    "reverse_kl / alignment outputs need PPOW_FLAG_POLICY_TERMS");
    const bool group_outputs = out->advantage || out->group_best_len || out->group_best_index;
    if (group_outputs) {
        if (params->rollout_group < 1 || B % params->rollout_group != 0)
            return fail(PPOW_ERR_INVALID_ARG,
                        "group outputs need rollout_group >= 1 dividing B (got %d, B=%lld)",
                        params->rollout_group, (long long)B);
        if (out->advantage && (!(params->adv_delta >= 0.f) || !isfinite(params->adv_delta)))
            return fail(PPOW_ERR_INVALID_ARG, "adv_delta must be a finite number >= 0");
    }
    return PPOW_OK;
}

// The launches of a scoring call; arguments validated, B > 0, `workspace` large enough.
int enqueue_score(const void *draft_logits, const void *target_logits,
                  const int32_t *draft_tokens, const float *uniforms, const float *ref_logprob,
                  int64_t B, int32_t K, int64_t V, int32_t dtype, const ppow_params *params,
                  const ppow_outputs *out, void *workspace, hipStream_t stream) {
    const int64_t rows = B * K;
    const bool second_pass = (params->flags & PPOW_FLAG_EXPECTED_ACCEPT) != 0;
    const bool policy_terms = (params->flags & PPOW_FLAG_POLICY_TERMS) != 0;
    const bool group_outputs = out->advantage || out->group_best_len || out->group_best_index;

    ppow::RowArgs ra;
    ra.target = target_logits;
    ra.draft = draft_logits;
    ra.tokens = draft_tokens;
    ra.uniforms = uniforms;
    ra.records = reinterpret_cast<ppow::RowRecord *>(static_cast<char *>(workspace) +
                                                      ppow::kClusterScratchBytes);
    ra.kl = out->kl;
    ra.confidence = out->confidence;
    ra.accept_prob = out->accept_prob;
    ra.expected_accept = out->expected_accept;
    ra.logp_target_tok = out->logp_target_tok;
    ra.logp_draft_tok = out->logp_draft_tok;
    ra.V = V;
    ra.inv_ln_V = 1.0 / log(static_cast<double>(V));
    ra.greedy = params->verify == PPOW_VERIFY_GREEDY;
    ra.reverse_kl = out->reverse_kl;
    ra.alignment = out->alignment;
    ra.second_pass = second_pass;
    ra.want_policy_terms = policy_terms;
    hipError_t err = hipSuccess;
    bool launched = false;
    if (second_pass) {
        // preferred: second pass from LDS; falls through when the device or sizes rule it out
        err = ppow::launch_row_cluster(ra, rows, dtype, workspace, stream, &launched);
        if (err != hipSuccess)
            return fail(PPOW_ERR_DEVICE, "cluster row kernel launch failed: %s",
                        hipGetErrorString(err));
    }
    g_row_kernel = launched ? "cluster" : "row";
    if (!launched) {
        err = ppow::launch_row_stats(ra, rows, dtype, stream);
        if (err != hipSuccess)
            return fail(PPOW_ERR_DEVICE, "row kernel launch failed: %s", hipGetErrorString(err));
    }

    ppow::WindowArgs wa;
    wa.records = ra.records;
    wa.ref_logprob = ref_logprob;
    wa.accepted_len = out->accepted_len;
    wa.r_speedup = out->r_speedup;
    wa.r_proximity = out->r_proximity;
    wa.adaw_score = out->adaw_score;
    wa.delta = out->delta;
    wa.reverse_kl_mean = out->reverse_kl_mean;
    wa.alignment_mean = out->alignment_mean;
    wa.status_clear = launched ? nullptr : static_cast<uint32_t *>(workspace);
    wa.status_check = launched ? static_cast<const uint32_t *>(workspace) : nullptr;
    wa.B = B;
    wa.K = K;
    wa.cost_ratio = params->cost_ratio;
    wa.prox_eps = params->prox_eps;
    wa.prox_eta = params->prox_eta;
    err = ppow::launch_window_epilogue(wa, stream);
    if (err != hipSuccess)
        return fail(PPOW_ERR_DEVICE, "window kernel launch failed: %s", hipGetErrorString(err));

    if (group_outputs) {
        ppow::GroupArgs ga;
        ga.r_speedup = out->r_speedup;
        ga.r_proximity = out->r_proximity;
        ga.accepted_len = out->accepted_len;
        ga.advantage = out->advantage;
        ga.best_len = out->group_best_len;
        ga.best_index = out->group_best_index;
        ga.group = params->rollout_group;
        ga.groups = B / params->rollout_group;
        ga.delta_stab = params->adv_delta;
        err = ppow::launch_group_epilogue(ga, stream);
        if (err != hipSuccess)
            return fail(PPOW_ERR_DEVICE, "group kernel launch failed: %s", hipGetErrorString(err));
    }
    return PPOW_OK;
}

struct StaticScratch {
    std::mutex lock;
    void *ptr[64] = {};        // device address of `scratch` on each device, once resolved
};
StaticScratch &static_scratch() {
    static StaticScratch s;
    return s;
}

// Device address of this device's copy of `scratch`.  The array's name is only a host-side
// handle: the address comes from hipGetSymbolAddress, once per device, with that device
// current; the same set-up creates the event that chains cluster launches, so that later
// calls create nothing at all.
int static_scratch_for_current_device(void **out_ptr) {
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess)
        return fail(PPOW_ERR_DEVICE, "hipGetDevice failed: %s", hipGetErrorString(err));
    if (dev < 0 || dev >= 64)
        return fail(PPOW_ERR_UNSUPPORTED, "device ordinal %d is beyond the 64 the library tracks", dev);
    StaticScratch &s = static_scratch();
    std::lock_guard<std::mutex> guard(s.lock);
    if (!s.ptr[dev]) {
        void *p = nullptr;
        err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err != hipSuccess || !p) {
            (void)hipGetLastError();
            return fail(PPOW_ERR_DEVICE, "hipGetSymbolAddress(scratch) failed on device %d: %s", dev,
                        hipGetErrorString(err));
        }
        err = ppow::prepare_cluster_chain();
        if (err != hipSuccess)
            return fail(PPOW_ERR_DEVICE, "event creation failed on device %d: %s", dev,
                        hipGetErrorString(err));
        s.ptr[dev] = p;
    }
    *out_ptr = s.ptr[dev];
    return PPOW_OK;
}

}  // namespace

extern "C" {

int ppow_score_windows(const void *draft_logits, const void *target_logits,
                       const int32_t *draft_tokens, const float *uniforms,
                       const float *ref_logprob, int64_t B, int32_t K, int64_t V, int32_t dtype,
                       const ppow_params *params, const ppow_outputs *out, void *workspace,
                       size_t workspace_bytes, void *hip_stream) {
    const int status = validate_score_args(draft_logits, target_logits, draft_tokens, uniforms, B, K,
                                           V, dtype, params, out);
    if (status != PPOW_OK || B == 0) return status;
    const size_t need = ppow_score_workspace_bytes(B, K, V, dtype, params->flags);
    if (!workspace || !aligned16(workspace) || workspace_bytes < need)
        return fail(PPOW_ERR_WORKSPACE, "workspace must be 16-byte aligned and hold %zu bytes", need);
    return enqueue_score(draft_logits, target_logits, draft_tokens, uniforms, ref_logprob, B, K, V,
                         dtype, params, out, workspace, static_cast<hipStream_t>(hip_stream));
}

int ppow_score_windows_static(const void *draft_logits, const void *target_logits,
                              const int32_t *draft_tokens, const float *uniforms,
                              const float *ref_logprob, int64_t B, int32_t K, int64_t V,
                              int32_t dtype, const ppow_params *params, const ppow_outputs *out,
                              void *hip_stream) {
    const int status = validate_score_args(draft_logits, target_logits, draft_tokens, uniforms, B, K,
                                           V, dtype, params, out);
    if (status != PPOW_OK || B == 0) return status;
    if (B * K > PPOW_STATIC_MAX_ROWS)
        return fail(PPOW_ERR_UNSUPPORTED,
                    "B*K = %lld positions exceed the %d the built-in scratch holds; use "
                    "ppow_score_windows with a workspace", (long long)(B * K), PPOW_STATIC_MAX_ROWS);
    void *ptr = nullptr;
    const int ready = static_scratch_for_current_device(&ptr);
    if (ready != PPOW_OK) return ready;
    return enqueue_score(draft_logits, target_logits, draft_tokens, uniforms, ref_logprob, B, K, V,
                         dtype, params, out, ptr, static_cast<hipStream_t>(hip_stream));
}

int ppow_release(void) {
    const hipError_t err = ppow::release_cluster_chain();
    if (err != hipSuccess) {
        (void)hipGetLastError();
        return fail(PPOW_ERR_DEVICE, "hipEventDestroy failed: %s", hipGetErrorString(err));
    }
    return PPOW_OK;
}

void ppow_debug_cluster_wait_limit(uint32_t looks) { ppow::set_cluster_spin_limit(looks); }

size_t ppow_adaw_sequence_workspace_bytes(int64_t N, int32_t T, int64_t V, int32_t dtype) {
    if (N < 0 || T < 1 || V < 2 || V > INT32_MAX || N > INT32_MAX / T) return 0;
    if (dtype != PPOW_F32 && dtype != PPOW_BF16) return 0;
    return ppow::kClusterScratchBytes +
           static_cast<size_t>(N) * static_cast<size_t>(T) * sizeof(ppow::RowRecord);
}

int ppow_adaw_sequence(const void *draft_logits, const void *target_logits, int64_t N, int32_t T,
                       int64_t V, int32_t dtype, int32_t K, const float *uniforms,
                       float adaw_fraction, const float *mix_uniforms,
                       float *criticality, float *window_score, int32_t *sampled_start,
                       void *workspace, size_t workspace_bytes, void *hip_stream) {
    const size_t need = ppow_adaw_sequence_workspace_bytes(N, T, V, dtype);
    if (need == 0 || K < 1 || K > T)
        return fail(PPOW_ERR_INVALID_ARG,
                    "sizes out of range: N=%lld T=%d V=%lld K=%d dtype=%d (need N>=0, 1<=K<=T, "
                    "N*T<2^31, 2<=V<2^31, dtype f32|bf16)",
                    (long long)N, T, (long long)V, K, dtype);
    if (N == 0) return PPOW_OK;
    if (!draft_logits || !target_logits || !window_score)
        return fail(PPOW_ERR_INVALID_ARG, "logits and window_score must not be NULL");
    if (!aligned16(draft_logits) || !aligned16(target_logits))
        return fail(PPOW_ERR_INVALID_ARG, "logit base pointers must be 16-byte aligned");
    if (sampled_start && !uniforms)
        return fail(PPOW_ERR_INVALID_ARG, "sampled_start needs uniforms");
    if (sampled_start && !(adaw_fraction >= 0.f && adaw_fraction <= 1.f))
        return fail(PPOW_ERR_INVALID_ARG, "adaw_fraction must lie in [0, 1]");
    if (sampled_start && adaw_fraction < 1.f && !mix_uniforms)
        return fail(PPOW_ERR_INVALID_ARG, "an adaw_fraction below 1 needs mix_uniforms");
    if (!workspace || !aligned16(workspace) || workspace_bytes < need)
        return fail(PPOW_ERR_WORKSPACE, "workspace must be 16-byte aligned and hold %zu bytes", need);

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    ppow::RowArgs ra = {};
    ra.target = target_logits;
    ra.draft = draft_logits;
    ra.records = reinterpret_cast<ppow::RowRecord *>(static_cast<char *>(workspace) +
                                                      ppow::kClusterScratchBytes);
    ra.V = V;
    ra.inv_ln_V = 1.0 / log(static_cast<double>(V));
    g_row_kernel = "row";
    hipError_t err = ppow::launch_row_stats(ra, N * T, dtype, stream);
    if (err != hipSuccess)
        return fail(PPOW_ERR_DEVICE, "row kernel launch failed: %s", hipGetErrorString(err));

    ppow::SequenceArgs sa;
    sa.records = ra.records;
    sa.uniforms = uniforms;
    sa.mix_uniforms = adaw_fraction < 1.f ? mix_uniforms : nullptr;
    sa.adaw_fraction = adaw_fraction;
    sa.criticality = criticality;
    sa.window_score = window_score;
    sa.sampled_start = sampled_start;
    sa.N = N;
    sa.T = T;
    sa.K = K;
    err = ppow::launch_sequence_windows(sa, stream);
    if (err != hipSuccess)
        return fail(PPOW_ERR_DEVICE, "sequence kernel launch failed: %s", hipGetErrorString(err));
    return PPOW_OK;
}

size_t ppow_select_workspace_bytes(int64_t B, int32_t M) {
    if (B < 1 || B > INT32_MAX || M < 1 || M > B) return 0;
    return ppow::select_workspace_bytes(B, M);
}

int ppow_select_windows(const float *adaw_score, int64_t B, int32_t M, int32_t *indices,
                        float *scores, void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (B < 1 || B > INT32_MAX || M < 1 || M > B)
        return fail(PPOW_ERR_INVALID_ARG, "need 1 <= M <= B < 2^31 (B=%lld, M=%d)", (long long)B, M);
    if (!adaw_score || !indices)
        return fail(PPOW_ERR_INVALID_ARG, "adaw_score and indices must not be NULL");
    const size_t need = ppow::select_workspace_bytes(B, M);
    if (!workspace || !aligned16(workspace) || workspace_bytes < need)
        return fail(PPOW_ERR_WORKSPACE, "workspace must be 16-byte aligned and hold %zu bytes", need);
    const hipError_t err = ppow::launch_select(adaw_score, B, M, indices, scores, workspace,
                                               static_cast<hipStream_t>(hip_stream));
    if (err != hipSuccess)
        return fail(PPOW_ERR_DEVICE, "select kernel launch failed: %s", hipGetErrorString(err));
    return PPOW_OK;
}

}  // extern "C"
