// Top-M window selection (Section 4.2: windows with larger s_j are prioritised).
//
// Every window gets a 64-bit composite  (order-preserving image of its fp32
// score) << 32 | ~index.  Composites are distinct, a larger composite means
// "larger score, or equal score and smaller index", so the answer is simply the
// M largest composites in descending order.  One workgroup:
//   1. radix select, 8 bits a pass from the top: LDS digit histograms narrow
//      down the M-th largest composite (index digits that cannot vary are skipped);
//   2. compaction of the composites at or above it into a sort buffer (LDS, or
//      the workspace when M exceeds the LDS capacity);
//   3. bitonic sort of the buffer, descending; decode indices and scores.
// Integer work throughout: the result is exact and independent of scheduling.
#include "ppow_device.h"

namespace ppow {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kLdsSortCap = 8192;          // composites the LDS sort buffer holds (64 KiB)
constexpr int kBatch = 4;                  // scores a lane fetches before it processes them

__device__ __forceinline__ uint32_t ordered_bits(float x) {
    uint32_t u = __builtin_bit_cast(uint32_t, x);
    u = (u == 0x80000000u) ? 0u : u;                 // -0.0 and +0.0 are the same score
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float from_ordered_bits(uint32_t k) {
    const uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    return __builtin_bit_cast(float, u);
}

__device__ __forceinline__ uint64_t composite(float score, int index) {
    return (static_cast<uint64_t>(ordered_bits(score)) << 32) | (~static_cast<uint32_t>(index));
}

template <bool SORT_IN_LDS>
__global__ __launch_bounds__(kThreads) void select_kernel(const float *__restrict__ score, int B, int M,
                                                          int sort_len, int index_bits,
                                                          int32_t *indices, float *scores_out,
                                                          uint64_t *global_buf) {
    __shared__ uint64_t lds_buf[SORT_IN_LDS ? kLdsSortCap : 1];
    __shared__ uint32_t hist[kWaves][256];
    __shared__ uint32_t sh_digit, sh_need, sh_count, sh_bin;
    uint64_t *buf = SORT_IN_LDS ? lds_buf : global_buf;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    // ---- 1. radix select of the M-th largest composite ------------------------------------
    uint64_t prefix = 0, prefix_mask = 0;
    uint32_t need = static_cast<uint32_t>(M);
    for (int shift = 56; shift >= 0; shift -= 8) {
        if (shift < 32 && shift >= index_bits) {
            // ~index has only ones up here: nothing to decide
            prefix |= 0xffull << shift;
            prefix_mask |= 0xffull << shift;
            continue;
        }
        for (int i = tid; i < kWaves * 256; i += kThreads) (&hist[0][0])[i] = 0;
        __syncthreads();
        for (int i0 = 0; i0 < B; i0 += kBatch * kThreads) {
            float key[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {               // kBatch independent loads in flight
                const int i = i0 + u * kThreads + tid;
                key[u] = i < B ? score[i] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int i = i0 + u * kThreads + tid;
                const bool valid = i < B;
                const uint64_t c = valid ? composite(key[u], i) : 0;
                const bool match = valid && (c & prefix_mask) == prefix;
                const uint32_t digit = static_cast<uint32_t>(c >> shift) & 0xffu;
                // Scores crowd into few leading digits: the lanes that share the digit of the
                // first matching lane are counted with one LDS atomic instead of up to 64
                // colliding ones.
                const unsigned long long matching = __ballot(match);
                if (matching) {
                    const int leader = __ffsll(static_cast<long long>(matching)) - 1;
                    const uint32_t d0 = __shfl(digit, leader, 64);
                    const unsigned long long same = __ballot(match && digit == d0);
                    if (lane == leader)
                        atomicAdd(&hist[wave][d0], static_cast<uint32_t>(__popcll(same)));
                    else if (match && digit != d0)
                        atomicAdd(&hist[wave][digit], 1u);
                }
            }
        }
        __syncthreads();
        if (tid < 256) {
            uint32_t total = 0;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) total += hist[w][tid];
            hist[0][tid] = total;
        }
        __syncthreads();
        if (wave == 0) {
            // lane l owns digits 4l..4l+3; find the digit where the count from the top reaches `need`
            uint32_t h[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) h[j] = hist[0][lane * 4 + j];
            const uint32_t local = h[0] + h[1] + h[2] + h[3];
            uint32_t incl = local;                     // inclusive sum over lanes >= this one
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t up = __shfl_down(incl, off, 64);
                if (lane + off < 64) incl += up;
            }
            const uint32_t above = incl - local;
            if (above < need && need <= above + local) {
                uint32_t cum = above;
                int digit = lane * 4;
                uint32_t remaining = need, in_bin = 0;
#pragma unroll
                for (int j = 3; j >= 0; --j) {
                    if (cum + h[j] >= need) {
                        digit = lane * 4 + j; remaining = need - cum; in_bin = h[j];
                        break;
                    }
                    cum += h[j];
                }
                sh_digit = static_cast<uint32_t>(digit);
                sh_need = remaining;
                sh_bin = in_bin;
            }
        }
        __syncthreads();
        prefix |= static_cast<uint64_t>(sh_digit) << shift;
        prefix_mask |= 0xffull << shift;
        need = sh_need;
        const bool take_all = sh_bin == need;
        __syncthreads();
        // Once every window that still matches the prefix is wanted, the remaining digits
        // decide nothing: the threshold is the smallest composite with this prefix.  This is
        // the usual case after the score digits, where a tie at the boundary is rare.
        if (take_all) break;
    }
    const uint64_t threshold = prefix;      // the M-th largest composite itself

    // ---- 2. compaction -------------------------------------------------------------------
    if (tid == 0) sh_count = 0;
    for (int i = tid; i < sort_len; i += kThreads) buf[i] = 0;   // 0 sorts below every composite
    __syncthreads();
    for (int i0 = 0; i0 < B; i0 += kThreads) {
        const int i = i0 + tid;
        const uint64_t c = i < B ? composite(score[i], i) : 0;
        const bool keep = i < B && c >= threshold;
        const unsigned long long kept = __ballot(keep);           // one counter update per wave
        if (kept) {
            const int leader = __ffsll(static_cast<long long>(kept)) - 1;
            uint32_t base = 0;
            if (lane == leader) base = atomicAdd(&sh_count, static_cast<uint32_t>(__popcll(kept)));
            base = __shfl(base, leader, 64);
            if (keep)       // slot order is settled by the sort
                buf[base + __popcll(kept & ((1ull << lane) - 1ull))] = c;
        }
    }
    __syncthreads();

    // ---- 3. bitonic sort, descending ------------------------------------------------------
    for (int k = 2; k <= sort_len; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = tid; i < sort_len; i += kThreads) {
                const int partner = i ^ j;
                if (partner > i) {
                    const uint64_t x = buf[i], y = buf[partner];
                    const bool descending = (i & k) == 0;
                    if ((x < y) == descending) { buf[i] = y; buf[partner] = x; }
                }
            }
            __syncthreads();
        }
    }

    for (int i = tid; i < M; i += kThreads) {
        const uint64_t c = buf[i];
        indices[i] = static_cast<int32_t>(~static_cast<uint32_t>(c));
        if (scores_out) scores_out[i] = from_ordered_bits(static_cast<uint32_t>(c >> 32));
    }
}

int next_pow2(int x) {
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

}  // namespace

size_t select_workspace_bytes(int64_t B, int32_t M) {
    (void)B;
    const int sort_len = next_pow2(M);
    const size_t need = sort_len > kLdsSortCap ? static_cast<size_t>(sort_len) * sizeof(uint64_t) : 0;
    return need < 256 ? 256 : need;
}

hipError_t launch_select(const float *score, int64_t B, int32_t M, int32_t *indices, float *scores,
                         void *workspace, hipStream_t stream) {
    const int sort_len = next_pow2(M);
    int index_bits = 0;
    while ((int64_t{1} << index_bits) < B) ++index_bits;
    index_bits = ((index_bits + 7) / 8) * 8;          // whole 8-bit digits
    if (sort_len <= kLdsSortCap)
        hipLaunchKernelGGL(select_kernel<true>, dim3(1), dim3(kThreads), 0, stream, score,
                           static_cast<int>(B), M, sort_len, index_bits, indices, scores,
                           static_cast<uint64_t *>(nullptr));
    else
        hipLaunchKernelGGL(select_kernel<false>, dim3(1), dim3(kThreads), 0, stream, score,
                           static_cast<int>(B), M, sort_len, index_bits, indices, scores,
                           static_cast<uint64_t *>(workspace));
    return hipGetLastError();
}

}  // namespace ppow
