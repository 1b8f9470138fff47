// Row-pair streaming reduction: the only kernel of the scoring pass that touches
// the logits.  One 256-thread workgroup reads one target row a[0..V) and the
// paired draft row b[0..V) exactly once, with 128-bit loads, and reduces them to
// the per-position scalars the window epilogue needs.
//
// With P = softmax(a), Q = softmax(b) (Section 4.2) it accumulates, relative to
// a per-lane reference rho (in log2 units, rho <= lane max <= rho + kRescaleGap):
//     Z_a  = sum 2^t,  S1 = sum 2^t * t,  S2 = sum 2^t * (a - b),   t  = a*log2(e) - rho_a
//     Z_b  = sum 2^tb,                                             tb = b*log2(e) - rho_b
// from which  H(P)     = ln2' * (log2 Z_a - S1 / Z_a)
//             KL(P||Q) = S2 / Z_a - ln2' * ((rho_a - rho_b) + log2(Z_a / Z_b))
// with ln2' = 1 / float(log2 e), so that the constant used going in is undone
// coming out; the few per-row operations that subtract nearly equal numbers are
// done in double.  Identical rows give exactly zero divergence.  The reference only moves when a chunk maximum exceeds it
// by more than kRescaleGap, which keeps the rescale off the streaming path; the
// exact row maximum and its first index are tracked separately, branch-free.
#include "ppow_device.h"

#include <limits.h>
#include <math.h>

namespace ppow {
namespace {

// Launch shape of the streaming kernel; the defaults are the measured best on MI355X.
#ifndef PPOW_ROW_THREADS
#define PPOW_ROW_THREADS 256
#endif
#ifndef PPOW_ROW_UNROLL
#define PPOW_ROW_UNROLL 4
#endif
#ifndef PPOW_ROW_NONTEMPORAL
#define PPOW_ROW_NONTEMPORAL 1
#endif
constexpr int kThreads = PPOW_ROW_THREADS;
constexpr int kWaves = kThreads / 64;
constexpr int kUnroll = PPOW_ROW_UNROLL;
constexpr float kLog2e = 1.44269504088896340736f;
constexpr float kRescaleGap = 24.0f;   // log2 units: partial sums stay below 2^24 * count
#define PPOW_NEG_INF (-__builtin_huge_valf())

typedef uint32_t raw4 __attribute__((ext_vector_type(4)));   // one 128-bit load

// Streaming load: logits that will not be read again should not displace other lines in
// cache (STREAM); a row that the second pass re-reads is loaded normally the first time.
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

struct LaneState {
    float rho_a, z_a, s1, s2;   // target side
    float rho_b, z_b;           // draft side
    float m_a;                  // exact maximum of the target logits this lane has seen
    int best;                   // body chunk in which m_a was first reached (-1: none yet)
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
    s.z_b = (s.rho_b == PPOW_NEG_INF) ? 0.f : s.z_b * fast_exp2(s.rho_b - new_rho);
    s.rho_b = new_rho;
}

// Fold VEC element pairs into the running sums (no argmax bookkeeping).
template <int VEC>
__device__ __forceinline__ void fold(LaneState &s, const float (&a)[VEC], const float (&b)[VEC],
                                     float cma, float cmb) {
    const float ta_max = fmaf(cma, kLog2e, -s.rho_a);
    const float tb_max = fmaf(cmb, kLog2e, -s.rho_b);
    if (fmaxf(ta_max, tb_max) > kRescaleGap) {      // rare: the reference lags too far behind
        if (ta_max > kRescaleGap) rebase_target(s, cma * kLog2e);
        if (tb_max > kRescaleGap) rebase_draft(s, cmb * kLog2e);
    }
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
        const float t = fmaf(a[j], kLog2e, -s.rho_a);
        const float e = fast_exp2(t);
        s.z_a += e;
        s.s1 = fmaf(e, t, s.s1);
        s.s2 = fmaf(e, a[j] - b[j], s.s2);
        const float tb = fmaf(b[j], kLog2e, -s.rho_b);
        s.z_b += fast_exp2(tb);
    }
}

template <int VEC>
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
    fold<VEC>(s, a, b, cma, cmb);
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off, 64));
    return x;
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

template <int DTYPE, bool SECOND>
__global__ __launch_bounds__(kThreads) void row_stats_kernel(RowArgs args) {
    using S = Storage<DTYPE>;
    using elem = typename S::elem;
    constexpr int VEC = S::VEC;

    __shared__ float sh_f[kWaves][6];
    __shared__ int sh_i[kWaves];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int64_t row = blockIdx.x;
    const int V = static_cast<int>(args.V);

    const elem *row_a = static_cast<const elem *>(args.target) + row * args.V;
    const elem *row_b = static_cast<const elem *>(args.draft) + row * args.V;

    // Elements before the first 16-byte boundary of the row (both rows share the
    // misalignment because both base pointers are 16-byte aligned).
    const uintptr_t addr = reinterpret_cast<uintptr_t>(row_a);
    int head = static_cast<int>(((16u - (addr & 15u)) & 15u) / sizeof(elem));
    head = head < V ? head : V;
    const int nchunks = (V - head) / VEC;
    const int tail_begin = head + nchunks * VEC;

    const raw4 *pa = reinterpret_cast<const raw4 *>(row_a + head);
    const raw4 *pb = reinterpret_cast<const raw4 *>(row_b + head);

    LaneState s;
    s.rho_a = PPOW_NEG_INF; s.z_a = 0.f; s.s1 = 0.f; s.s2 = 0.f;
    s.rho_b = PPOW_NEG_INF; s.z_b = 0.f;
    s.m_a = PPOW_NEG_INF; s.best = -1;

    int c = tid;
    for (; c + (kUnroll - 1) * kThreads < nchunks; c += kUnroll * kThreads) {
        raw4 ra[kUnroll], rb[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            ra[u] = load_chunk<!SECOND>(pa + c + u * kThreads);
            rb[u] = load_chunk<!SECOND>(pb + c + u * kThreads);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            float a[VEC], b[VEC];
            S::unpack(ra[u], a);
            S::unpack(rb[u], b);
            fold_chunk<VEC>(s, a, b, c + u * kThreads);
        }
    }
    for (; c < nchunks; c += kThreads) {
        float a[VEC], b[VEC];
        S::unpack(load_chunk<!SECOND>(pa + c), a);
        S::unpack(load_chunk<!SECOND>(pb + c), b);
        fold_chunk<VEC>(s, a, b, c);
    }

    // Ragged ends: at most VEC-1 elements before and after the vector body.
    const int ragged = head + (V - tail_begin);
    float rag_v = PPOW_NEG_INF;
    int rag_i = INT_MAX;
    if (tid < ragged) {
        rag_i = (tid < head) ? tid : tail_begin + (tid - head);
        const float a1[1] = {S::load1(row_a + rag_i)};
        const float b1[1] = {S::load1(row_b + rag_i)};
        fold<1>(s, a1, b1, a1[0], b1[0]);
        rag_v = a1[0];
    }

    // ---- workgroup combine --------------------------------------------------------------
    // 1. common references and the exact row maximum
    float ref_a = wave_max(s.rho_a);
    float ref_b = wave_max(s.rho_b);
    float row_max = wave_max(fmaxf(s.m_a, rag_v));
    if (lane == 0) { sh_f[wave][0] = ref_a; sh_f[wave][1] = ref_b; sh_f[wave][2] = row_max; }
    __syncthreads();
    ref_a = sh_f[0][0]; ref_b = sh_f[0][1]; row_max = sh_f[0][2];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) {
        ref_a = fmaxf(ref_a, sh_f[w][0]);
        ref_b = fmaxf(ref_b, sh_f[w][1]);
        row_max = fmaxf(row_max, sh_f[w][2]);
    }
    __syncthreads();

    // First index of the row maximum: only lanes that hold it re-read their one chunk.
    int arg_i = (rag_v == row_max) ? rag_i : INT_MAX;
    if (s.best >= 0 && s.m_a == row_max) {
        float a[VEC];
        S::unpack(pa[s.best], a);
        int first = VEC - 1;
#pragma unroll
        for (int j = VEC - 2; j >= 0; --j) first = (a[j] == row_max) ? j : first;
        const int idx = head + s.best * VEC + first;
        arg_i = idx < arg_i ? idx : arg_i;
    }

    // 2. bring every lane to the common references, then plain sums in a fixed tree
    float z_a = 0.f, s1 = 0.f, s2 = 0.f, z_b = 0.f;
    if (s.rho_a != PPOW_NEG_INF) {          // a lane that saw any element saw both rows
        const float da = s.rho_a - ref_a;
        const float sc = fast_exp2(da);
        z_a = s.z_a * sc;
        s1 = sc * fmaf(da, s.z_a, s.s1);
        s2 = s.s2 * sc;
        z_b = s.z_b * fast_exp2(s.rho_b - ref_b);
    }

    z_a = wave_sum(z_a); s1 = wave_sum(s1); s2 = wave_sum(s2); z_b = wave_sum(z_b);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const int other = __shfl_xor(arg_i, off, 64);
        arg_i = other < arg_i ? other : arg_i;
    }
    if (lane == 0) {
        sh_f[wave][0] = z_a; sh_f[wave][1] = s1; sh_f[wave][2] = s2; sh_f[wave][3] = z_b;
        sh_i[wave] = arg_i;
    }
    __syncthreads();
    z_a = sh_f[0][0]; s1 = sh_f[0][1]; s2 = sh_f[0][2]; z_b = sh_f[0][3];
    arg_i = sh_i[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) {
        z_a += sh_f[w][0]; s1 += sh_f[w][1]; s2 += sh_f[w][2]; z_b += sh_f[w][3];
        arg_i = sh_i[w] < arg_i ? sh_i[w] : arg_i;
    }
    const float arg_v = row_max;

    const float log2_za = fast_log2(z_a);
    const float log2_zb = fast_log2(z_b);

    // ---- optional second pass: sum_y min(P(y), Q(y))  (Appendix B.1) ----------------------
    float expected = 0.f;
    if (SECOND) {
        // The row is walked backwards: its end was read last and is the most likely part to
        // still sit in the L2 / memory-side cache.
        const float lam_a = ref_a + log2_za;      // log2-domain log-sum-exp
        const float lam_b = ref_b + log2_zb;
        float acc = 0.f;
        int cc = nchunks - 1 - tid;
        for (; cc - (kUnroll - 1) * kThreads >= 0; cc -= kUnroll * kThreads) {
            raw4 ra[kUnroll], rb[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                ra[u] = load_chunk<true>(pa + cc - u * kThreads);
                rb[u] = load_chunk<true>(pb + cc - u * kThreads);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                float a[VEC], b[VEC];
                S::unpack(ra[u], a);
                S::unpack(rb[u], b);
#pragma unroll
                for (int j = 0; j < VEC; ++j)
                    acc += fminf(fast_exp2(fmaf(a[j], kLog2e, -lam_a)),
                                 fast_exp2(fmaf(b[j], kLog2e, -lam_b)));
            }
        }
        for (; cc >= 0; cc -= kThreads) {
            float a[VEC], b[VEC];
            S::unpack(load_chunk<true>(pa + cc), a);
            S::unpack(load_chunk<true>(pb + cc), b);
#pragma unroll
            for (int j = 0; j < VEC; ++j)
                acc += fminf(fast_exp2(fmaf(a[j], kLog2e, -lam_a)),
                             fast_exp2(fmaf(b[j], kLog2e, -lam_b)));
        }
        if (tid < ragged) {
            const int y = (tid < head) ? tid : tail_begin + (tid - head);
            acc += fminf(fast_exp2(fmaf(S::load1(row_a + y), kLog2e, -lam_a)),
                         fast_exp2(fmaf(S::load1(row_b + y), kLog2e, -lam_b)));
        }
        acc = wave_sum(acc);
        __syncthreads();
        if (lane == 0) sh_f[wave][5] = acc;
        __syncthreads();
        expected = sh_f[0][5];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) expected += sh_f[w][5];
    }

    // ---- per-position scalars (Sections 4.2, 4.3.2; Appendix C.1) -------------------------
    if (tid == 0) {
        const double ln2p_d = 1.0 / static_cast<double>(kLog2e);
        const float ln2p = static_cast<float>(ln2p_d);
        const double inv_za = 1.0 / static_cast<double>(z_a);
        const double entropy = ln2p_d * (static_cast<double>(log2_za) - s1 * inv_za);
        const double lse_diff = ln2p_d * (static_cast<double>(ref_a - ref_b) +
                                          static_cast<double>(fast_log2(z_a / z_b)));
        const float kl = fmaxf(static_cast<float>(s2 * inv_za - lse_diff), 0.f);
        float conf = static_cast<float>(1.0 - entropy * args.inv_ln_V);
        conf = fminf(fmaxf(conf, 0.f), 1.f);

        const int tok = args.tokens[row];
        const float a_tok = S::load1(row_a + tok);
        const float b_tok = S::load1(row_b + tok);
        // log-probabilities relative to the running references: the error then scales
        // with |log p|, not with the magnitude of the logits
        const float xa = fmaf(a_tok, kLog2e, -ref_a) - log2_za;    // log2 P(tok)
        const float xb = fmaf(b_tok, kLog2e, -ref_b) - log2_zb;    // log2 Q(tok)
        const float logp = ln2p * xa;
        const float logq = ln2p * xb;
        // the ratio from the difference itself: exactly 0 when the rows are identical
        const float alpha = fast_exp2(fminf(xa - xb, 0.f));

        int accept;
        if (args.greedy) accept = (tok == arg_i);
        else accept = (args.uniforms[row] <= alpha);

        RowRecord rec;
        rec.criticality = conf * kl;
        rec.gap = arg_v - a_tok;
        rec.logp_tok = logp;
        rec.accept = accept;
        args.records[row] = rec;

        if (args.kl) args.kl[row] = kl;
        if (args.confidence) args.confidence[row] = conf;
        if (args.accept_prob) args.accept_prob[row] = alpha;
        if (args.expected_accept) args.expected_accept[row] = expected;
        if (args.logp_target_tok) args.logp_target_tok[row] = logp;
        if (args.logp_draft_tok) args.logp_draft_tok[row] = logq;
    }
}

}  // namespace

// Dynamic LDS requested only to cap how many two-pass workgroups share a CU, so that the rows
// in flight fit the memory-side cache when they are read the second time.
#ifndef PPOW_PASS2_LDS_BYTES
#define PPOW_PASS2_LDS_BYTES 0
#endif

hipError_t launch_row_stats(const RowArgs &args, int64_t rows, int32_t dtype, hipStream_t stream) {
    if (rows == 0) return hipSuccess;
    const dim3 grid(static_cast<unsigned>(rows)), block(kThreads);
    if (args.second_pass) {
        const size_t lds = PPOW_PASS2_LDS_BYTES;
        if (dtype == PPOW_BF16) {
            if (lds > 65536)
                (void)hipFuncSetAttribute(reinterpret_cast<const void *>(row_stats_kernel<PPOW_BF16, true>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
            hipLaunchKernelGGL((row_stats_kernel<PPOW_BF16, true>), grid, block, lds, stream, args);
        } else {
            if (lds > 65536)
                (void)hipFuncSetAttribute(reinterpret_cast<const void *>(row_stats_kernel<PPOW_F32, true>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
            hipLaunchKernelGGL((row_stats_kernel<PPOW_F32, true>), grid, block, lds, stream, args);
        }
    } else if (dtype == PPOW_BF16) {
        hipLaunchKernelGGL((row_stats_kernel<PPOW_BF16, false>), grid, block, 0, stream, args);
    } else {
        hipLaunchKernelGGL((row_stats_kernel<PPOW_F32, false>), grid, block, 0, stream, args);
    }
    return hipGetLastError();
}

}  // namespace ppow
