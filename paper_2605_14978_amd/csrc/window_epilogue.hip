// Window epilogue: from the per-position records of the row kernel to the four
// per-window outputs.  Lane t of a group of G = 2^ceil(log2 K) consecutive lanes
// holds position t of one window, so a wavefront carries 64/G windows.
//   accepted length  k = number of leading accepted positions: the first zero of
//                    the group's slice of the wavefront ballot (Appendix C.1: the
//                    sum over n of the product over t <= n of the accept bits)
//   R_speedup        k / (k*gamma + 1)                          (Section 4.3.1)
//   delta            sum_t gap_t, or ref - sum_t log P_t(tok_t) (Section 4.3.2)
//   r_proximity      eta * [k == 0] * [delta < eps]             (Algorithm 1)
//   ADAW score       (1/K) sum_t v_t over all K positions       (Section 4.2)
//   window means of KL(Q_t||P_t) (the target-anchored regulariser of Appendix A.2) and of
//   the alignment metric of Appendix E, when asked for
// Sums use a fixed xor-shuffle tree, so results do not depend on scheduling.
#include "ppow_device.h"

namespace ppow {
namespace {

constexpr int kThreads = 256;

__global__ __launch_bounds__(kThreads) void window_epilogue_kernel(WindowArgs args, int log2_group) {
    const int group = 1 << log2_group;
    const int lane = threadIdx.x & 63;
    const int64_t gid = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    const int64_t window = gid >> log2_group;
    const int t = static_cast<int>(gid & (group - 1));
    const bool active = (window < args.B) && (t < args.K);
    if (gid == 0 && args.status_clear) *args.status_clear = 0u;
    // A bounded wait of the cluster kernel that expired left records unwritten: every window
    // of the call is then marked instead of being given plausible-looking numbers.
    const bool expired = args.status_check && *args.status_check != 0u;

    float v = 0.f, gap = 0.f, logp = 0.f, rkl = 0.f, align = 0.f;
    int accept = 0;
    bool bad_token = false, bad_logits = false;
    if (active) {
        const RowRecord rec = args.records[window * args.K + t];
        bad_token = (rec.bad_token & 1u) != 0u;
        bad_logits = (rec.bad_token & 2u) != 0u;
        v = rec.criticality;
        gap = rec.gap;
        logp = rec.logp_tok;
        accept = rec.accept;
        rkl = rec.reverse_kl;
        align = rec.alignment;
    }

    // first rejected position of this window
    const unsigned long long ballot = __ballot(active && accept != 0);
    const int group_base = lane & ~(group - 1);
    unsigned long long bits = ballot >> group_base;
    unsigned long long rejected = ~bits;
    if (args.K < 64) rejected |= (1ull << args.K);          // position K always "rejects"
    int k = rejected ? __builtin_ctzll(rejected) : 64;
    // a drafted token outside [0, V) anywhere in the window: no accepted length, no reward
    const unsigned long long group_mask = group == 64 ? ~0ull : ((1ull << group) - 1ull);
    const bool not_finite = ((__ballot(active && bad_logits) >> group_base) & group_mask) != 0ull;
    const bool invalid = not_finite ||
                         ((__ballot(active && bad_token) >> group_base) & group_mask) != 0ull;
    if (invalid) k = not_finite ? -2 : -1;      // logits that are not finite: no score either
    if (expired) k = -3;

    // fixed-order sums over the group
    for (int off = group >> 1; off > 0; off >>= 1) {
        v += __shfl_xor(v, off, 64);
        gap += __shfl_xor(gap, off, 64);
        logp += __shfl_xor(logp, off, 64);
        rkl += __shfl_xor(rkl, off, 64);
        align += __shfl_xor(align, off, 64);
    }

    if (active && t == 0) {
        const float kf = static_cast<float>(k);
        const float delta = args.ref_logprob ? (args.ref_logprob[window] - logp) : gap;
        args.accepted_len[window] = k;
        args.r_speedup[window] = (invalid || expired) ? 0.f : kf / fmaf(kf, args.cost_ratio, 1.0f);
        args.r_proximity[window] = (k == 0 && delta < args.prox_eps) ? args.prox_eta : 0.f;
        args.adaw_score[window] = (not_finite || expired) ? 0.f : v / static_cast<float>(args.K);
        if (args.delta) args.delta[window] = delta;
        if (args.reverse_kl_mean) args.reverse_kl_mean[window] = rkl / static_cast<float>(args.K);
        if (args.alignment_mean) args.alignment_mean[window] = align / static_cast<float>(args.K);
    }
}

// Per group of G consecutive windows, one thread per group, everything in index order:
//  * group-relative advantage (Section 4.1): A_i = (R_i - mean) / (std + delta) with
//    R_i = r_speedup + r_proximity (Algorithm 1's reward), std the population standard deviation.
//    Mean and variance are formed in double: a group whose rewards are all equal (every window
//    fully accepted, say) then has R_i - mean exactly 0, where an fp32 mean leaves a residue of
//    an ulp or two that the division by std + delta (delta ~ 1e-6) would blow up to ~0.1;
//  * best candidate (multi-candidate decoding, Table 2): the largest accepted length of the
//    group and the index of the first window attaining it.
__global__ __launch_bounds__(kThreads) void group_epilogue_kernel(GroupArgs args) {
    const int64_t g = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (g >= args.groups) return;
    const int64_t base = g * args.group;
    if (args.advantage) {
        auto reward = [&](int i) {
            return static_cast<double>(args.r_speedup[base + i]) +
                   static_cast<double>(args.r_proximity[base + i]);
        };
        const double count = static_cast<double>(args.group);
        double mean = 0.0;
        for (int i = 0; i < args.group; ++i) mean += reward(i);
        mean /= count;
        double var = 0.0;
        for (int i = 0; i < args.group; ++i) {
            const double d = reward(i) - mean;
            var += d * d;
        }
        const double inv = 1.0 / (sqrt(var / count) + static_cast<double>(args.delta_stab));
        for (int i = 0; i < args.group; ++i)
            args.advantage[base + i] = static_cast<float>((reward(i) - mean) * inv);
    }
    if (args.best_len || args.best_index) {
        int best = 0, best_k = args.accepted_len[base];
        for (int i = 1; i < args.group; ++i) {
            const int k = args.accepted_len[base + i];
            if (k > best_k) { best_k = k; best = i; }
        }
        if (args.best_len) args.best_len[g] = best_k;
        if (args.best_index) args.best_index[g] = best;
    }
}

// Sequence-mode ADAW (Algorithm 1): one workgroup per sequence of T scored positions.
//   window_score[j] = (1/K) sum_{t=j}^{j+K-1} v_t, summed in index order;
//   sampled start: under the hard-window curriculum (Appendix A.3, Table 5) the window is an
//   ADAW-selected one when the sequence's mixing draw is below the ADAW fraction, else an
//   ordinary one, floor(u * W).  An ADAW-selected start inverts the cumulative distribution
//   of the window scores at the draw u: the smallest j whose running sum reaches u times the
//   total; all-zero scores fall back to floor(u * W).  The running sums are double: wavefront
//   0 splits the scores into 64 contiguous segments, each lane adds up its own, a wavefront
//   scan of the 64 segment sums gives every lane the sum before its segment, and the lane
//   whose segment contains the crossing walks it again.  (A double sum of fp32 scores is
//   exact or within 2^-53 of exact whatever its order, so the decision is the one an
//   index-order double sum takes, up to draws within ~1e-16 of a boundary.)
constexpr int kSeqLdsScores = 8192;        // window scores of one sequence staged in LDS
__device__ __forceinline__ int padded(int j) { return j + (j >> 5); }   // segment starts in distinct banks

__device__ __forceinline__ double shuffle_up(double x, int delta) {
    const long long bits = __builtin_bit_cast(long long, x);
    const int lo = __shfl_up(static_cast<int>(bits), delta, 64);
    const int hi = __shfl_up(static_cast<int>(bits >> 32), delta, 64);
    return __builtin_bit_cast(double, (static_cast<long long>(hi) << 32) |
                                          static_cast<long long>(static_cast<unsigned>(lo)));
}
__device__ __forceinline__ double broadcast(double x, int lane) {
    const long long bits = __builtin_bit_cast(long long, x);
    const int lo = __shfl(static_cast<int>(bits), lane, 64);
    const int hi = __shfl(static_cast<int>(bits >> 32), lane, 64);
    return __builtin_bit_cast(double, (static_cast<long long>(hi) << 32) |
                                          static_cast<long long>(static_cast<unsigned>(lo)));
}

__global__ __launch_bounds__(kThreads) void sequence_windows_kernel(SequenceArgs args) {
    __shared__ float sh_score[kSeqLdsScores + kSeqLdsScores / 32 + 1];
    const int64_t n = blockIdx.x;
    const int T = args.T, K = args.K, W = T - K + 1;
    const RowRecord *rec = args.records + n * T;
    if (args.criticality)
        for (int t = threadIdx.x; t < T; t += kThreads) args.criticality[n * T + t] = rec[t].criticality;
    float *score = args.window_score + n * W;
    for (int j = threadIdx.x; j < W; j += kThreads) {
        float sum = 0.f;
        for (int t = 0; t < K; ++t) sum += rec[j + t].criticality;
        const float s = sum / static_cast<float>(K);
        score[j] = s;
        if (j < kSeqLdsScores) sh_score[padded(j)] = s;
    }
    if (!args.sampled_start) return;
    __syncthreads();                        // the scores of this sequence are all written
    if (threadIdx.x >= 64) return;
    const int lane = threadIdx.x;
    const double u = static_cast<double>(args.uniforms[n]);
    const int uniform_pick = min(static_cast<int>(floor(u * static_cast<double>(W))), W - 1);
    const bool adaw = !args.mix_uniforms || args.mix_uniforms[n] < args.adaw_fraction;
    if (!adaw) {                            // uniform over the wavefront: an ordinary window
        if (lane == 0) args.sampled_start[n] = uniform_pick;
        return;
    }
    auto score_at = [&](int j) { return j < kSeqLdsScores ? sh_score[padded(j)] : score[j]; };
    const int per = (W + 63) / 64;          // lane l owns scores [l*per, min(W, (l+1)*per))
    const int j0 = min(lane * per, W), j1 = min(j0 + per, W);
    double mine = 0.0;
    for (int j = j0; j < j1; ++j) mine += static_cast<double>(score_at(j));
    double upto = mine;                     // inclusive scan over the lanes
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const double prev = shuffle_up(upto, off);
        if (lane >= off) upto += prev;
    }
    const double total = broadcast(upto, 63);
    int pick = uniform_pick;                // all-zero scores: the weights are undefined
    if (total > 0.0) {
        const double threshold = u * total;
        const unsigned long long reached = __ballot(upto >= threshold);
        // first lane whose running sum reaches the threshold; rounding may leave none
        const int owner = reached ? __builtin_ctzll(reached) : 63;
        const double before = shuffle_up(upto, 1);      // sum of the scores before this segment
        int first = j1 - 1;                 // if rounding leaves the walk short: the segment's end
        if (lane == owner) {
            double c = lane == 0 ? 0.0 : before;
            for (int j = j0; j < j1; ++j) {
                c += static_cast<double>(score_at(j));
                if (c >= threshold) { first = j; break; }
            }
        }
        pick = __shfl(first, owner, 64);
    }
    if (lane == 0) args.sampled_start[n] = pick;
}

}  // namespace

hipError_t launch_window_epilogue(const WindowArgs &args, hipStream_t stream) {
    if (args.B == 0) return hipSuccess;
    int log2_group = 0;
    while ((1 << log2_group) < args.K) ++log2_group;
    const int64_t threads = args.B << log2_group;
    const int64_t blocks = (threads + kThreads - 1) / kThreads;
    hipLaunchKernelGGL(window_epilogue_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0,
                       stream, args, log2_group);
    return hipGetLastError();
}

hipError_t launch_group_epilogue(const GroupArgs &args, hipStream_t stream) {
    if (args.groups == 0) return hipSuccess;
    const int64_t blocks = (args.groups + kThreads - 1) / kThreads;
    hipLaunchKernelGGL(group_epilogue_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0,
                       stream, args);
    return hipGetLastError();
}

hipError_t launch_sequence_windows(const SequenceArgs &args, hipStream_t stream) {
    if (args.N == 0) return hipSuccess;
    hipLaunchKernelGGL(sequence_windows_kernel, dim3(static_cast<unsigned>(args.N)), dim3(kThreads), 0,
                       stream, args);
    return hipGetLastError();
}

}  // namespace ppow
