// Internal declarations shared by the HIP translation units of libppow.
// Not part of the public interface (that is include/ppow.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ppow.h"

namespace ppow {

// What the row kernel leaves for the window epilogue: one record per (window, position).
struct RowRecord {
    float criticality;   // v_t = C(P_t) * KL(P_t || Q_t)            (Section 4.2)
    float gap;           // max_y a_t[y] - a_t[tok_t]                 (Section 4.3.2, same-context reference)
    float logp_tok;      // log P_t(tok_t)
    int32_t accept;      // verification outcome of this position     (Appendix C.1)
    float reverse_kl;    // KL(Q_t || P_t)                            (Section 4.1, Appendix A.2)
    float alignment;     // exp(d) - d - 1, d = log P_t(tok) - log Q_t(tok)   (Appendix E)
    uint32_t bad_token;  // bit 0: the drafted token of this position was outside [0, V);
                         // bit 1: the logit rows of this position were not all finite
    float pad1;
};
static_assert(sizeof(RowRecord) == 32, "records are 32 bytes");

struct RowArgs {
    const void *target;          // [rows, V]
    const void *draft;           // [rows, V]
    const int32_t *tokens;       // [rows]
    const float *uniforms;       // [rows] or nullptr (greedy)
    RowRecord *records;          // [rows]
    float *kl;                   // optional per-row outputs, nullptr = skip
    float *confidence;
    float *accept_prob;
    float *expected_accept;
    float *logp_target_tok;
    float *logp_draft_tok;
    float *reverse_kl;
    float *alignment;
    int64_t V;
    double inv_ln_V;             // 1 / ln V
    int32_t greedy;              // 1: accept iff token == argmax target
    int32_t second_pass;         // 1: compute sum_y min(P, Q)
    int32_t want_policy_terms;   // 1: compute KL(Q||P) and the alignment metric
};

struct WindowArgs {
    const RowRecord *records;    // [B*K]
    const float *ref_logprob;    // [B] or nullptr
    int32_t *accepted_len;       // [B]
    float *r_speedup;            // [B]
    float *r_proximity;          // [B]
    float *adaw_score;           // [B]
    float *delta;                // [B] or nullptr
    float *reverse_kl_mean;      // [B] or nullptr
    float *alignment_mean;       // [B] or nullptr
    uint32_t *status_clear;      // workspace status word to zero, or nullptr (cluster path owns it)
    const uint32_t *status_check; // status word the cluster kernel may have set, or nullptr
    int64_t B;
    int32_t K;
    float cost_ratio, prox_eps, prox_eta;
};

struct GroupArgs {
    const float *r_speedup;      // [B]
    const float *r_proximity;    // [B]
    const int32_t *accepted_len; // [B]
    float *advantage;            // [B] or nullptr
    int32_t *best_len;           // [B / group] or nullptr
    int32_t *best_index;         // [B / group] or nullptr
    int64_t groups;              // B / group
    int32_t group;               // rollout / candidate group size G
    float delta_stab;            // small positive constant of the normalisation
};

struct SequenceArgs {
    const RowRecord *records;    // [N*T]
    const float *uniforms;       // [N] or nullptr
    const float *mix_uniforms;   // [N] curriculum draws, or nullptr: every start is ADAW-selected
    float adaw_fraction;         // share of ADAW-selected starts (Appendix A.3)
    float *criticality;          // [N*T] or nullptr
    float *window_score;         // [N*(T-K+1)]
    int32_t *sampled_start;      // [N] or nullptr
    int64_t N;
    int32_t T, K;
};

// Scratch words of the cluster variant of the row kernel, kept in front of the records.
constexpr size_t kClusterScratchBytes = 1u << 20;

hipError_t launch_row_stats(const RowArgs &args, int64_t rows, int32_t dtype, hipStream_t stream);
hipError_t launch_row_cluster(const RowArgs &args, int64_t rows, int32_t dtype, void *scratch,
                              hipStream_t stream, bool *launched);
hipError_t prepare_cluster_chain();
hipError_t release_cluster_chain();
void set_cluster_spin_limit(uint32_t spins);   // 0 restores the default
hipError_t launch_window_epilogue(const WindowArgs &args, hipStream_t stream);
hipError_t launch_group_epilogue(const GroupArgs &args, hipStream_t stream);
hipError_t launch_sequence_windows(const SequenceArgs &args, hipStream_t stream);

size_t select_workspace_bytes(int64_t B, int32_t M);
hipError_t launch_select(const float *score, int64_t B, int32_t M, int32_t *indices, float *scores,
                         void *workspace, hipStream_t stream);

}  // namespace ppow
