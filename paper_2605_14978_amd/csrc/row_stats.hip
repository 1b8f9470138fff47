// Row-pair streaming reduction, one workgroup per row pair: the kernel of the scoring pass
// that touches the logits.  A 256-thread workgroup reads one target row a[0..V) and the paired
// draft row b[0..V) once, with 128-bit loads, and reduces them to the per-position scalars the
// window epilogue needs (arithmetic in row_math.h).  With the second-pass flag it then re-reads
// the row pair from memory for sum_y min(P, Q) (Appendix B.1); the cluster kernel in
// row_cluster.hip does that pass from LDS instead and is preferred when it can be launched.
#include "row_math.h"

namespace ppow {
namespace {

// Launch shape of the streaming kernel; the defaults are the measured best on MI355X.
#ifndef PPOW_ROW_THREADS
#define PPOW_ROW_THREADS 256
#endif
#ifndef PPOW_ROW_UNROLL
#define PPOW_ROW_UNROLL 4
#endif
constexpr int kThreads = PPOW_ROW_THREADS;
constexpr int kWaves = kThreads / 64;
constexpr int kUnroll = PPOW_ROW_UNROLL;

// Tuning build (PPOW_ROW_TRACE=1): thread 0 records when its workgroup began and ended (100 MHz
// clock) and where it ran (hardware id, XCD), for the first 40 000 rows, in the part of the
// scratch in front of the records that this kernel does not use (bytes 4096 .. 4096 + 20 * 40000
// of the workspace).
#ifndef PPOW_ROW_TRACE
#define PPOW_ROW_TRACE 0
#endif
#if PPOW_ROW_TRACE
__device__ __forceinline__ void trace_row(const RowArgs &args, int64_t row, unsigned long long begin) {
    if (row >= 40000) return;
    char *base = reinterpret_cast<char *>(args.records) - kClusterScratchBytes + 4096;
    unsigned long long *when = reinterpret_cast<unsigned long long *>(base);
    when[2 * row] = begin;
    when[2 * row + 1] = wall_clock64();
    unsigned hw, xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    reinterpret_cast<unsigned *>(base + 16 * 40000)[row] = (hw & 0xffffu) | (xcc << 16);
}
#endif

template <int DTYPE, bool SECOND, bool REV>
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
#if PPOW_ROW_TRACE
    const unsigned long long trace_begin = wall_clock64();
#endif

    const elem *row_a = static_cast<const elem *>(args.target) + row * args.V;
    const elem *row_b = static_cast<const elem *>(args.draft) + row * args.V;

    // Elements before the first kRowAlign-byte boundary of the target row.  Both base pointers
    // are 16-byte aligned and both rows start at the same element offset, so the draft row is
    // 16-byte aligned at the same element (its own line boundary may fall elsewhere).
    const uintptr_t addr = reinterpret_cast<uintptr_t>(row_a);
    int head = static_cast<int>(((kRowAlign - (addr & (kRowAlign - 1u))) & (kRowAlign - 1u)) / sizeof(elem));
    head = head < V ? head : V;
    const int nchunks = (V - head) / VEC;
    const int tail_begin = head + nchunks * VEC;

    const raw4 *pa = reinterpret_cast<const raw4 *>(row_a + head);
    const raw4 *pb = reinterpret_cast<const raw4 *>(row_b + head);

    LaneState s;
    s.reset();

    // Prologue: every lane's first chunk, which also gives the wavefront its starting references.
    {
        float a[VEC], b[VEC];
        float first_a = PPOW_NEG_INF, first_b = PPOW_NEG_INF;
        if (tid < nchunks) {
            S::unpack(load_chunk<!SECOND>(pa + tid), a);
            S::unpack(load_chunk<!SECOND>(pb + tid), b);
            first_a = chunk_max<VEC>(a);
            first_b = chunk_max<VEC>(b);
        }
        start_reference(s, first_a, first_b);
        if (tid < nchunks) fold_chunk<RowFold, VEC, REV>(s, a, b, tid);
    }

    int c = tid + kThreads;
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
            fold_chunk<RowFold, VEC, REV>(s, a, b, c + u * kThreads);
        }
    }
    for (; c < nchunks; c += kThreads) {
        float a[VEC], b[VEC];
        S::unpack(load_chunk<!SECOND>(pa + c), a);
        S::unpack(load_chunk<!SECOND>(pb + c), b);
        fold_chunk<RowFold, VEC, REV>(s, a, b, c);
    }

    // Ragged ends: fewer than kRowAlign bytes of elements before the vector body and at most
    // VEC-1 elements after it (63 + 7 bf16 elements at most), one per lane.
    const int ragged = head + (V - tail_begin);
    float rag_v = PPOW_NEG_INF;
    int rag_i = INT_MAX;
    if (tid < ragged) {
        rag_i = (tid < head) ? tid : tail_begin + (tid - head);
        const float a1[1] = {S::load1(row_a + rag_i)};
        const float b1[1] = {S::load1(row_b + rag_i)};
        fold<RowFold, 1, REV>(s, a1, b1, a1[0], b1[0]);
        rag_v = a1[0];
    }

    // ---- workgroup combine --------------------------------------------------------------
    // 1. common references and the exact row maximum
    RowTotals t;
    t.ref_a = wave_max(s.rho_a);
    t.ref_b = wave_max(s.rho_b);
    t.row_max = wave_max(fmaxf(s.m_a, rag_v));
    if (lane == 0) { sh_f[wave][0] = t.ref_a; sh_f[wave][1] = t.ref_b; sh_f[wave][2] = t.row_max; }
    __syncthreads();
    t.ref_a = sh_f[0][0]; t.ref_b = sh_f[0][1]; t.row_max = sh_f[0][2];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) {
        t.ref_a = fmaxf(t.ref_a, sh_f[w][0]);
        t.ref_b = fmaxf(t.ref_b, sh_f[w][1]);
        t.row_max = fmaxf(t.row_max, sh_f[w][2]);
    }
    __syncthreads();

    // First index of the row maximum: only lanes that hold it re-read their one chunk.
    int arg_i = (rag_v == t.row_max) ? rag_i : INT_MAX;
    if (s.best >= 0 && s.m_a == t.row_max) {
        float a[VEC];
        S::unpack(pa[s.best], a);
        int first = VEC - 1;
#pragma unroll
        for (int j = VEC - 2; j >= 0; --j) first = (a[j] == t.row_max) ? j : first;
        const int idx = head + s.best * VEC + first;
        arg_i = idx < arg_i ? idx : arg_i;
    }

    // 2. bring every lane to the common references, then plain sums in a fixed tree
    to_common_reference(s.rho_a, s.rho_b, t.ref_a, t.ref_b, s.z_a, s.s1, s.s2, s.z_b, s.s2r);
    t.z_a = wave_sum(s.z_a); t.s1 = wave_sum(s.s1); t.s2 = wave_sum(s.s2); t.z_b = wave_sum(s.z_b);
    t.s2r = REV ? wave_sum(s.s2r) : 0.f;
    arg_i = wave_min(arg_i);
    if (lane == 0) {
        sh_f[wave][0] = t.z_a; sh_f[wave][1] = t.s1; sh_f[wave][2] = t.s2; sh_f[wave][3] = t.z_b;
        sh_f[wave][4] = t.s2r; sh_i[wave] = arg_i;
    }
    __syncthreads();
    t.z_a = sh_f[0][0]; t.s1 = sh_f[0][1]; t.s2 = sh_f[0][2]; t.z_b = sh_f[0][3]; t.s2r = sh_f[0][4];
    t.arg_i = sh_i[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) {
        t.z_a += sh_f[w][0]; t.s1 += sh_f[w][1]; t.s2 += sh_f[w][2]; t.z_b += sh_f[w][3];
        t.s2r += sh_f[w][4];
        t.arg_i = sh_i[w] < t.arg_i ? sh_i[w] : t.arg_i;
    }

    // ---- optional second pass: sum_y min(P(y), Q(y))  (Appendix B.1) ----------------------
    float expected = 0.f;
    if (SECOND) {
        // The row is walked backwards: its end was read last and is the most likely part to
        // still sit in cache.
        const float lam_a = t.ref_a + fast_log2(t.z_a);      // log2-domain log-sum-exp
        const float lam_b = t.ref_b + fast_log2(t.z_b);
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
                acc += min_prob_sum<VEC>(a, b, lam_a, lam_b);
            }
        }
        for (; cc >= 0; cc -= kThreads) {
            float a[VEC], b[VEC];
            S::unpack(load_chunk<true>(pa + cc), a);
            S::unpack(load_chunk<true>(pb + cc), b);
            acc += min_prob_sum<VEC>(a, b, lam_a, lam_b);
        }
        if (tid < ragged) {
            const float a1[1] = {S::load1(row_a + rag_i)};
            const float b1[1] = {S::load1(row_b + rag_i)};
            acc += min_prob_sum<1>(a1, b1, lam_a, lam_b);
        }
        acc = wave_sum(acc);
        __syncthreads();
        if (lane == 0) sh_f[wave][5] = acc;
        __syncthreads();
        expected = sh_f[0][5];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) expected += sh_f[w][5];
    }

    if (tid == 0) finish_row<DTYPE, RowFold>(args, row, t, expected, load_drafted_token<DTYPE>(args, row));
#if PPOW_ROW_TRACE
    if (tid == 0) trace_row(args, row, trace_begin);
#endif
}

template <int DTYPE, bool SECOND>
void launch_one(const RowArgs &args, dim3 grid, dim3 block, hipStream_t stream) {
    if (args.want_policy_terms)
        hipLaunchKernelGGL((row_stats_kernel<DTYPE, SECOND, true>), grid, block, 0, stream, args);
    else
        hipLaunchKernelGGL((row_stats_kernel<DTYPE, SECOND, false>), grid, block, 0, stream, args);
}

}  // namespace

hipError_t launch_row_stats(const RowArgs &args, int64_t rows, int32_t dtype, hipStream_t stream) {
    if (rows == 0) return hipSuccess;
    const dim3 grid(static_cast<unsigned>(rows)), block(kThreads);
    if (dtype == PPOW_BF16) {
        if (args.second_pass) launch_one<PPOW_BF16, true>(args, grid, block, stream);
        else launch_one<PPOW_BF16, false>(args, grid, block, stream);
    } else {
        if (args.second_pass) launch_one<PPOW_F32, true>(args, grid, block, stream);
        else launch_one<PPOW_F32, false>(args, grid, block, stream);
    }
    return hipGetLastError();
}

}  // namespace ppow
