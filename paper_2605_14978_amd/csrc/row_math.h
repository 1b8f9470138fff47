// Device-side arithmetic shared by the two row kernels (one workgroup per row pair, and a
// cluster of workgroups per row pair): storage unpacking, the per-lane online softmax state,
// wave reductions and the per-position epilogue.
//
// With P = softmax(a), Q = softmax(b) (Section 4.2) a lane accumulates, relative to its own
// references rho (log2 units; rho <= lane max <= rho + gap):
//     Z_a = sum 2^t,  S1 = sum 2^t * t,  S2 = sum 2^t * (a - b),    t  = a*log2(e) - rho_a
//     Z_b = sum 2^tb,                    S2r = sum 2^tb * (b - a),  tb = b*log2(e) - rho_b
// from which  H(P)     = ln2' * (log2 Z_a - S1 / Z_a)
//             KL(P||Q) = S2  / Z_a - ln2' * ((rho_a - rho_b) + log2(Z_a / Z_b))
//             KL(Q||P) = S2r / Z_b + ln2' * ((rho_a - rho_b) + log2(Z_a / Z_b))
// with ln2' = 1 / float(log2 e), so that the constant used going in is undone coming out;
// the few per-row operations that subtract nearly equal numbers are done in double.
// Identical rows give exactly zero divergence.  The lanes of a wavefront start from a common
// reference, the largest logit among the wavefront's first chunks (start_reference), and a
// lane's reference only moves when a chunk maximum exceeds it by more than a gap: a few
// times per row, which keeps the rescale off the streaming path.  The gap also bounds the
// rounding of the exponents: t is rounded to 2^-23 * |t|, so an element that carries much of
// the probability must not sit far above the reference -- with |t| <= 8 its exponential is
// good to 2e-7, where |t| ~ 24 would cost 1e-6 of absolute error in the divergences of nearly
// identical rows (the two rows round differently).  The exact row maximum and its first index
// are tracked separately, branch-free.
#pragma once

#include <limits.h>
#include <math.h>

#include "ppow_device.h"

namespace ppow {

constexpr float kLog2e = 1.44269504088896340736f;
// Rescale gaps in log2 units (partial sums stay below 2^gap * count).  The one-workgroup-per-row
// kernel starts its wavefronts near the top of the row and can afford the tight gap.  The
// cluster kernel keeps the wide one and per-lane starting references: there the cross-lane
// maximum at the start of a row sits on the critical path of a whole cluster (1.5 % of its
// throughput when measured), and a rebase has to rescale what the lane has kept; on that path
// the divergences of nearly identical rows carry up to ~1.5e-6 of absolute error.
#ifndef PPOW_RESCALE_GAP
#define PPOW_RESCALE_GAP 8.0f
#endif
// How a kernel folds: its rescale gap, and whether a chunk's exponentials are added in a tree
// before they reach the running partition sums (eight more live registers, which the cluster
// kernel -- it keeps a slice of both rows in registers -- cannot spare).
struct RowFold {
    static constexpr float gap = PPOW_RESCALE_GAP;
    static constexpr bool tree = true;
    static constexpr bool double_log = true;    // log2(Z_a / Z_b) of the epilogue in double
};
struct ClusterFold {
    static constexpr float gap = 24.0f;
    static constexpr bool tree = false;
    static constexpr bool double_log = false;   // (the software double logarithm is register-hungry)
};
#define PPOW_NEG_INF (-__builtin_huge_valf())

#ifndef PPOW_ROW_NONTEMPORAL
#define PPOW_ROW_NONTEMPORAL 1
#endif

typedef uint32_t raw4 __attribute__((ext_vector_type(4)));   // one 128-bit load

// Streaming load: logits that will not be read again should not displace other lines in
// cache (STREAM); a row that a second pass re-reads from memory is loaded normally.
template <bool STREAM>
__device__ __forceinline__ raw4 load_chunk(const raw4 *p) {
#if PPOW_ROW_NONTEMPORAL
    if (STREAM) return __builtin_nontemporal_load(p);
#endif
    return *p;
}

__device__ __forceinline__ float as_float(uint32_t bits) { return __builtin_bit_cast(float, bits); }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

template <int DTYPE>
struct Storage;

template <>
struct Storage<PPOW_F32> {
    using elem = float;
    static constexpr int VEC = 4;
    static __device__ __forceinline__ void unpack(const raw4 &r, float (&x)[VEC]) {
        x[0] = as_float(r.x); x[1] = as_float(r.y); x[2] = as_float(r.z); x[3] = as_float(r.w);
    }
    static __device__ __forceinline__ float load1(const elem *p) { return *p; }
    static __device__ __forceinline__ raw4 pack(const float (&x)[VEC]) {
        raw4 r;
        r.x = __builtin_bit_cast(uint32_t, x[0]); r.y = __builtin_bit_cast(uint32_t, x[1]);
        r.z = __builtin_bit_cast(uint32_t, x[2]); r.w = __builtin_bit_cast(uint32_t, x[3]);
        return r;
    }
};

template <>
struct Storage<PPOW_BF16> {
    using elem = uint16_t;
    static constexpr int VEC = 8;
    // a bfloat16 is the upper half of a binary32; element 2i sits in the low half of word i
    static __device__ __forceinline__ void unpack(const raw4 &r, float (&x)[VEC]) {
        x[0] = as_float(r.x << 16); x[1] = as_float(r.x & 0xffff0000u);
        x[2] = as_float(r.y << 16); x[3] = as_float(r.y & 0xffff0000u);
        x[4] = as_float(r.z << 16); x[5] = as_float(r.z & 0xffff0000u);
        x[6] = as_float(r.w << 16); x[7] = as_float(r.w & 0xffff0000u);
    }
    static __device__ __forceinline__ float load1(const elem *p) {
        return as_float(static_cast<uint32_t>(*p) << 16);
    }
};

// The vector body of a row starts at the first address of the row that is a multiple of this
// (a cache line, so that a wave's 1 KiB reads do not straddle lines); the elements before it
// and after the last whole 16-byte chunk go through scalar loads.  PPOW_ROW_ALIGN >= 16.
#ifndef PPOW_ROW_ALIGN
#define PPOW_ROW_ALIGN 128
#endif
constexpr unsigned kRowAlign = PPOW_ROW_ALIGN;

struct LaneState {
    float rho_a, z_a, s1, s2;   // target side
    float rho_b, z_b, s2r;      // draft side (s2r only when the reverse divergence is wanted)
    float m_a;                  // exact maximum of the target logits this lane has seen
    int best;                   // body chunk in which m_a was first reached (-1: none yet)

    __device__ __forceinline__ void reset() {
        rho_a = PPOW_NEG_INF; z_a = 0.f; s1 = 0.f; s2 = 0.f;
        rho_b = PPOW_NEG_INF; z_b = 0.f; s2r = 0.f;
        m_a = PPOW_NEG_INF; best = -1;
    }
};

__device__ __forceinline__ void rebase_target(LaneState &s, float new_rho) {
    if (s.rho_a == PPOW_NEG_INF) {
        s.z_a = 0.f; s.s1 = 0.f; s.s2 = 0.f;
    } else {
        const float d = s.rho_a - new_rho;
        const float sc = fast_exp2(d);
        s.s1 = sc * fmaf(d, s.z_a, s.s1);     // every t shifts by d
        s.z_a *= sc;
        s.s2 *= sc;
    }
    s.rho_a = new_rho;
}

__device__ __forceinline__ void rebase_draft(LaneState &s, float new_rho) {
    const float sc = (s.rho_b == PPOW_NEG_INF) ? 0.f : fast_exp2(s.rho_b - new_rho);
    s.z_b *= sc;
    s.s2r *= sc;
    s.rho_b = new_rho;
}

// Fold VEC element pairs into the running sums (no argmax bookkeeping).  With KEEP the two
// exponentials of every pair, 2^(a*log2e - rho_a) and 2^(b*log2e - rho_b) relative to the
// references as they stand after this call, are handed back for a later pass.
template <class POLICY, int VEC, bool REV, bool KEEP>
__device__ __forceinline__ void fold_impl(LaneState &s, const float (&a)[VEC], const float (&b)[VEC],
                                          float cma, float cmb, float *ea, float *eb_out) {
    const float ta_max = fmaf(cma, kLog2e, -s.rho_a);
    const float tb_max = fmaf(cmb, kLog2e, -s.rho_b);
    if (fmaxf(ta_max, tb_max) > POLICY::gap) {      // rare: the reference lags too far behind
        if (ta_max > POLICY::gap) rebase_target(s, cma * kLog2e);
        if (tb_max > POLICY::gap) rebase_draft(s, cmb * kLog2e);
    }
    // The two partition sums carry the log-sum-exps, whose difference is what is left of the
    // divergence of nearly identical rows: with POLICY::tree the chunk's exponentials are added
    // in a tree and reach the running sum with one addition (same count of additions as adding
    // them one by one, an eighth of the roundings against the large running sum).
    float za[VEC], zb[VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
        const float t = fmaf(a[j], kLog2e, -s.rho_a);
        const float e = fast_exp2(t);
        const float d = a[j] - b[j];
        if (POLICY::tree) za[j] = e; else s.z_a += e;
        s.s1 = fmaf(e, t, s.s1);
        s.s2 = fmaf(e, d, s.s2);
        const float tb = fmaf(b[j], kLog2e, -s.rho_b);
        const float eb = fast_exp2(tb);
        if (POLICY::tree) zb[j] = eb; else s.z_b += eb;
        if (REV) s.s2r = fmaf(eb, -d, s.s2r);
        if (KEEP) { ea[j] = e; eb_out[j] = eb; }
    }
    if (POLICY::tree) {
#pragma unroll
        for (int w = 1; w < VEC; w <<= 1) {
#pragma unroll
            for (int j = 0; j + w < VEC; j += 2 * w) { za[j] += za[j + w]; zb[j] += zb[j + w]; }
        }
        s.z_a += za[0];
        s.z_b += zb[0];
    }
}

template <class POLICY, int VEC, bool REV>
__device__ __forceinline__ void fold(LaneState &s, const float (&a)[VEC], const float (&b)[VEC],
                                     float cma, float cmb) {
    fold_impl<POLICY, VEC, REV, false>(s, a, b, cma, cmb, nullptr, nullptr);
}

template <class POLICY, int VEC, bool REV>
__device__ __forceinline__ void fold_chunk(LaneState &s, const float (&a)[VEC],
                                           const float (&b)[VEC], int chunk) {
    float cma = a[0], cmb = b[0];
#pragma unroll
    for (int j = 1; j < VEC; ++j) {
        cma = fmaxf(cma, a[j]);
        cmb = fmaxf(cmb, b[j]);
    }
    s.best = (cma > s.m_a) ? chunk : s.best;       // strict: the first chunk keeps a tie
    s.m_a = fmaxf(s.m_a, cma);
    fold<POLICY, VEC, REV>(s, a, b, cma, cmb);
}

// As fold_chunk, but the raw logits will not be looked at again: the exponentials are kept in
// their place (ea, eb), and the position of the lane's maximum is tracked to the element
// (first_elem = chunk * VEC + first j of the chunk that reaches the chunk maximum).
template <class POLICY, int VEC, bool REV>
__device__ __forceinline__ void fold_chunk_keep(LaneState &s, const float (&a)[VEC],
                                                const float (&b)[VEC], int chunk, int &first_elem,
                                                float (&ea)[VEC], float (&eb)[VEC]) {
    float cma = a[0], cmb = b[0];
#pragma unroll
    for (int j = 1; j < VEC; ++j) {
        cma = fmaxf(cma, a[j]);
        cmb = fmaxf(cmb, b[j]);
    }
    int jf = VEC - 1;
#pragma unroll
    for (int j = VEC - 2; j >= 0; --j) jf = (a[j] == cma) ? j : jf;
    const bool better = cma > s.m_a;                // strict: the first chunk keeps a tie
    s.best = better ? chunk : s.best;
    first_elem = better ? chunk * VEC + jf : first_elem;
    s.m_a = fmaxf(s.m_a, cma);
    fold_impl<POLICY, VEC, REV, true>(s, a, b, cma, cmb, ea, eb);
}

// Pass-2 contribution of VEC pairs from kept exponentials: scale_a = 2^(rho_a - lam_a) etc.
template <int VEC>
__device__ __forceinline__ float min_prob_sum_kept(const float (&ea)[VEC], const float (&eb)[VEC],
                                                   float scale_a, float scale_b) {
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc += fminf(ea[j] * scale_a, eb[j] * scale_b);
    return acc;
}

// sum_y min(P(y), Q(y)) contribution of VEC pairs; lam = log2-domain log-sum-exp.  The
// exponential is monotone, so the smaller probability is the exponential of the smaller
// exponent: one v_exp_f32 per pair instead of two.
template <int VEC>
__device__ __forceinline__ float min_prob_sum(const float (&a)[VEC], const float (&b)[VEC],
                                              float lam_a, float lam_b) {
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < VEC; ++j)
        acc += fast_exp2(fminf(fmaf(a[j], kLog2e, -lam_a), fmaf(b[j], kLog2e, -lam_b)));
    return acc;
}

// Wave-wide reductions without LDS traffic: four data-parallel-primitive steps reduce each row
// of 16 lanes (lane i pairs with i^1, i^2, then with the mirrored lane of its half row and of
// its row, which by then hold the partner quad's / half row's value), and the four row results
// are read out as scalars.  Every lane returns the same bits; the order of the additions is
// fixed, so results repeat from run to run.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(
        0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ int dpp_move(int x) {
    return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xF, 0xF, true);
}
constexpr int kDppXor1 = 0xB1;          // quad_perm:[1,0,3,2]
constexpr int kDppXor2 = 0x4E;          // quad_perm:[2,3,0,1]
constexpr int kDppHalfMirror = 0x141;   // row_half_mirror
constexpr int kDppMirror = 0x140;       // row_mirror

__device__ __forceinline__ float row_lane(float x, int lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), lane));
}

__device__ __forceinline__ float wave_max(float x) {
    x = fmaxf(x, dpp_move<kDppXor1>(x));
    x = fmaxf(x, dpp_move<kDppXor2>(x));
    x = fmaxf(x, dpp_move<kDppHalfMirror>(x));
    x = fmaxf(x, dpp_move<kDppMirror>(x));
    return fmaxf(fmaxf(row_lane(x, 0), row_lane(x, 16)), fmaxf(row_lane(x, 32), row_lane(x, 48)));
}

__device__ __forceinline__ float wave_sum(float x) {
    x += dpp_move<kDppXor1>(x);
    x += dpp_move<kDppXor2>(x);
    x += dpp_move<kDppHalfMirror>(x);
    x += dpp_move<kDppMirror>(x);
    return (row_lane(x, 0) + row_lane(x, 16)) + (row_lane(x, 32) + row_lane(x, 48));
}

__device__ __forceinline__ int wave_min(int x) {
    x = min(x, dpp_move<kDppXor1>(x));
    x = min(x, dpp_move<kDppXor2>(x));
    x = min(x, dpp_move<kDppHalfMirror>(x));
    x = min(x, dpp_move<kDppMirror>(x));
    return min(min(__builtin_amdgcn_readlane(x, 0), __builtin_amdgcn_readlane(x, 16)),
               min(__builtin_amdgcn_readlane(x, 32), __builtin_amdgcn_readlane(x, 48)));
}

// Common starting references of a wavefront: the maxima of its lanes' first chunks (-inf for a
// lane without one).  Every lane of the wavefront must call this, before its first fold.
__device__ __forceinline__ void start_reference(LaneState &s, float first_max_a, float first_max_b) {
#ifdef PPOW_NO_START_REFERENCE          // tuning build: every lane finds its own first reference
    (void)s; (void)first_max_a; (void)first_max_b;
    return;
#endif
    const float wa = wave_max(first_max_a);
    const float wb = wave_max(first_max_b);
    if (wa != PPOW_NEG_INF) {                 // some lane has a chunk: both rows have elements
        s.rho_a = wa * kLog2e;
        s.rho_b = wb * kLog2e;
    }
}

template <int VEC>
__device__ __forceinline__ float chunk_max(const float (&x)[VEC]) {
    float m = x[0];
#pragma unroll
    for (int j = 1; j < VEC; ++j) m = fmaxf(m, x[j]);
    return m;
}

// Sums of one row pair relative to the references ref_a / ref_b, plus the exact target maximum.
struct RowTotals {
    float ref_a, ref_b;
    float z_a, s1, s2, z_b, s2r;
    float row_max;
    int arg_i;
};

// A lane's (or a partial result's) sums re-expressed relative to common references.
__device__ __forceinline__ void to_common_reference(float rho_a, float rho_b, float ref_a,
                                                    float ref_b, float &z_a, float &s1, float &s2,
                                                    float &z_b, float &s2r) {
    if (rho_a != PPOW_NEG_INF) {            // whoever saw any element saw both rows
        const float da = rho_a - ref_a;
        const float sa = fast_exp2(da);
        const float sb = fast_exp2(rho_b - ref_b);
        s1 = sa * fmaf(da, z_a, s1);
        z_a *= sa;
        s2 *= sa;
        z_b *= sb;
        s2r *= sb;
    } else {
        z_a = 0.f; s1 = 0.f; s2 = 0.f; z_b = 0.f; s2r = 0.f;
    }
}

// Per-position scalars from the row totals (Sections 4.2, 4.3.2; Appendices C.1 and E), run
// by one lane: writes the record for the window epilogue and the optional per-position outputs.
// The drafted token of a row and the two logits it selects, loaded ahead of finish_row.
struct DraftedToken {
    int tok;
    float a_tok, b_tok;
};

template <int DTYPE>
__device__ __forceinline__ DraftedToken load_drafted_token(const RowArgs &args, int64_t row) {
    using S = Storage<DTYPE>;
    using elem = typename S::elem;
    DraftedToken d;
    if (!args.tokens) {                   // sequence mode: no drafted token to verify
        d.tok = -1; d.a_tok = 0.f; d.b_tok = 0.f;
        return d;
    }
    // A token outside [0, V) must not become an address: element 0 is read in its place and
    // the position is marked (tok = -2), which the window epilogue turns into accepted_len = -1.
    const int tok = args.tokens[row];
    const bool in_range = static_cast<uint32_t>(tok) < static_cast<uint32_t>(args.V);
    const int at = in_range ? tok : 0;
    d.tok = in_range ? tok : -2;
    d.a_tok = S::load1(static_cast<const elem *>(args.target) + row * args.V + at);
    d.b_tok = S::load1(static_cast<const elem *>(args.draft) + row * args.V + at);
    return d;
}

template <int DTYPE, class POLICY>
__device__ __forceinline__ void finish_row(const RowArgs &args, int64_t row, const RowTotals &t,
                                           float expected, const DraftedToken &drafted) {
    const float log2_za = fast_log2(t.z_a);
    const float log2_zb = fast_log2(t.z_b);
    const double ln2p_d = 1.0 / static_cast<double>(kLog2e);
    const float ln2p = static_cast<float>(ln2p_d);
    const double inv_za = 1.0 / static_cast<double>(t.z_a);
    const double entropy = ln2p_d * (static_cast<double>(log2_za) - t.s1 * inv_za);
    const double log2_ratio_z = POLICY::double_log
        ? log2(static_cast<double>(t.z_a) / static_cast<double>(t.z_b))
        : static_cast<double>(fast_log2(t.z_a / t.z_b));
    const double lse_diff = ln2p_d * ((static_cast<double>(t.ref_a) - static_cast<double>(t.ref_b)) +
                                      log2_ratio_z);
    const float kl = fmaxf(static_cast<float>(t.s2 * inv_za - lse_diff), 0.f);
    float conf = static_cast<float>(1.0 - entropy * args.inv_ln_V);
    conf = fminf(fmaxf(conf, 0.f), 1.f);

    const int tok = drafted.tok;
    const float a_tok = drafted.a_tok;
    const float b_tok = drafted.b_tok;
    // log-probabilities relative to the references: the error then scales with |log p|,
    // not with the magnitude of the logits
    const float xa = fmaf(a_tok, kLog2e, -t.ref_a) - log2_za;    // log2 P(tok)
    const float xb = fmaf(b_tok, kLog2e, -t.ref_b) - log2_zb;    // log2 Q(tok)
    const float logp = ln2p * xa;
    const float logq = ln2p * xb;
    // the ratio from the difference itself: exactly 0 when the rows are identical
    const float log2_ratio = xa - xb;
    const float alpha = fast_exp2(fminf(log2_ratio, 0.f));

    int accept = 0;
    if (tok >= 0) {
        if (args.greedy) accept = (tok == t.arg_i);
        else accept = (args.uniforms[row] <= alpha);
    }

    float reverse_kl = 0.f, alignment = 0.f;
    if (args.want_policy_terms) {
        const double inv_zb = 1.0 / static_cast<double>(t.z_b);
        reverse_kl = fmaxf(static_cast<float>(t.s2r * inv_zb + lse_diff), 0.f);
        // exp(d) - d - 1 with d = log P(tok) - log Q(tok), in double: it cancels for small d
        const double d = ln2p_d * static_cast<double>(log2_ratio);
        alignment = static_cast<float>(expm1(d) - d);
    }

    RowRecord rec;
    rec.criticality = conf * kl;
    rec.gap = t.row_max - a_tok;
    rec.logp_tok = logp;
    rec.accept = accept;
    rec.reverse_kl = reverse_kl;
    rec.alignment = alignment;
    // A NaN or an infinity anywhere in either row ends up in one of the row sums.  The test is
    // on bit patterns the compiler cannot trace back to a float: the build lets it assume that
    // floats are never NaN, and it would fold a test it recognised as one for NaN away.
    auto opaque_bits = [](float x) {
        uint32_t u = __builtin_bit_cast(uint32_t, x);
        asm volatile("" : "+v"(u));
        return u;
    };
    const uint32_t exponent_bits = 0x7f800000u;
    const bool finite = (opaque_bits(t.z_a) & exponent_bits) != exponent_bits &&
                        (opaque_bits(t.z_b) & exponent_bits) != exponent_bits &&
                        (opaque_bits(t.s1) & exponent_bits) != exponent_bits &&
                        (opaque_bits(t.s2) & exponent_bits) != exponent_bits;
    rec.bad_token = ((tok == -2) ? 1u : 0u) | (finite ? 0u : 2u);
    rec.pad1 = 0.f;
    args.records[row] = rec;

    if (args.kl) args.kl[row] = kl;
    if (args.confidence) args.confidence[row] = conf;
    if (args.accept_prob) args.accept_prob[row] = alpha;
    if (args.expected_accept) args.expected_accept[row] = expected;
    if (args.logp_target_tok) args.logp_target_tok[row] = logp;
    if (args.logp_draft_tok) args.logp_draft_tok[row] = logq;
    if (args.reverse_kl) args.reverse_kl[row] = reverse_kl;
    if (args.alignment) args.alignment[row] = alignment;
}

}  // namespace ppow
