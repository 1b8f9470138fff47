// Top-M window selection (Section 4.2: windows with larger s_j are prioritised).
//
// Every window gets a 64-bit composite  (order-preserving image of its fp32
// score) << 32 | ~index.  Composites are distinct, a larger composite means
// "larger score, or equal score and smaller index", so the answer is simply the
// M largest composites in descending order.  The steps, all in one workgroup:
//   1. radix select, 8 bits a pass from the top: LDS digit histograms narrow
//      down the M-th largest composite (index digits that cannot vary are skipped);
//   2. compaction of the composites at or above it into a sort buffer (LDS, or
//      the workspace when M exceeds the LDS capacity);
//   3. bitonic sort of the buffer, descending; decode indices and scores.
// Up to 32 768 windows a workgroup keeps every composite in registers: one read of the
// scores; the passes of step 1 touch LDS only, step 3 becomes a bitonic network over
// registers, lane exchanges and, for the widest steps only, LDS.  More windows than that are cut into
// slices of 16 384: one workgroup per slice keeps the slice's own M largest (step 1 and 2),
// and a last workgroup selects and sorts among the survivors -- the global M largest are
// among them.  What fits neither scheme (M above the LDS sort buffer, too many survivors)
// takes the general kernel that re-reads the scores from memory in every pass.
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
__global__ __launch_bounds__(kThreads) void select_general_kernel(const float *__restrict__ score, int B, int M,
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


// ---- register-resident selection --------------------------------------------------------

// Optional phase timing for tuning (off in the product build): thread 0 of workgroup 0 leaves
// shader-clock readings at the phase boundaries of the resident kernel.
#ifndef PPOW_SELECT_FEW_DIGITS
#define PPOW_SELECT_FEW_DIGITS 8
#endif
#ifndef PPOW_SELECT_TIMING
#define PPOW_SELECT_TIMING 0
#endif
#if PPOW_SELECT_TIMING
__device__ long long g_select_ticks[8];
#define PPOW_SELECT_TICK(i) do { if (threadIdx.x == 0 && blockIdx.x == 0) g_select_ticks[i] = clock64(); } while (0)
#else
#define PPOW_SELECT_TICK(i) do { } while (0)
#endif

constexpr uint32_t kFewDigits = PPOW_SELECT_FEW_DIGITS;   // digit span counted with ballots

struct SelectShared {
    uint32_t hist[2][256];          // double-buffered by pass: the next pass's bins are cleared
    uint32_t digit[2], need[2], bin[2];   // while this pass's are read
    uint32_t count;
};

// ---- cross-lane helpers: xor exchanges inside a 16-lane row are data-parallel-primitive
//      moves (no LDS round trip), wider ones go through ds_bpermute ------------------------
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t x) {
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), CTRL, 0xF, 0xF, true));
}
template <int D>
__device__ __forceinline__ uint32_t lane_xor(uint32_t x) {
    if constexpr (D == 1) return dpp_mov<0xB1>(x);                      // quad_perm [1,0,3,2]
    else if constexpr (D == 2) return dpp_mov<0x4E>(x);                 // quad_perm [2,3,0,1]
    else if constexpr (D == 4) return dpp_mov<0x1B>(dpp_mov<0x141>(x)); // i^7 (half mirror) then i^3
    else if constexpr (D == 8) return dpp_mov<0x141>(dpp_mov<0x140>(x));// i^15 (row mirror) then i^7
    else return static_cast<uint32_t>(__shfl_xor(static_cast<int>(x), D, 64));
}
template <int D>
__device__ __forceinline__ uint64_t lane_xor(uint64_t x) {
    const uint32_t lo = lane_xor<D>(static_cast<uint32_t>(x));
    const uint32_t hi = lane_xor<D>(static_cast<uint32_t>(x >> 32));
    return (static_cast<uint64_t>(hi) << 32) | lo;
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t x) {
    x = min(x, lane_xor<1>(x)); x = min(x, lane_xor<2>(x)); x = min(x, lane_xor<4>(x)); x = min(x, lane_xor<8>(x));
    return min(min(static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(x), 0)),
                   static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(x), 16))),
               min(static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(x), 32)),
                   static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(x), 48))));
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x) {
    x = max(x, lane_xor<1>(x)); x = max(x, lane_xor<2>(x)); x = max(x, lane_xor<4>(x)); x = max(x, lane_xor<8>(x));
    return max(max(static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(x), 0)),
                   static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(x), 16))),
               max(static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(x), 32)),
                   static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(x), 48))));
}

// Inclusive sum over lanes 0..l: four shifts inside each row of 16 lanes, then the last lane
// of row 0 (2) is added to row 1 (3), and the last lane of the lower half to the upper half.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_add(uint32_t x) {
    return x + static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), CTRL, ROW_MASK, 0xF, true));
}
__device__ __forceinline__ uint32_t wave_inclusive_scan_u32(uint32_t x) {
    x = dpp_add<0x111, 0xF>(x);       // row_shr:1 (lanes shifted in from outside the row read 0)
    x = dpp_add<0x112, 0xF>(x);       // row_shr:2
    x = dpp_add<0x114, 0xF>(x);       // row_shr:4
    x = dpp_add<0x118, 0xF>(x);       // row_shr:8
    x = dpp_add<0x142, 0xA>(x);       // row_bcast:15 into rows 1 and 3
    x = dpp_add<0x143, 0xC>(x);       // row_bcast:31 into rows 2 and 3
    return x;
}

// The `need`-th largest of the workgroup's composites (E per thread in registers; 0 marks an
// empty slot and is below every composite).  All threads return the same value.  Radix select,
// 8 bits a pass from the top; two barriers a pass: bins and results are double-buffered, so
// clearing the next pass's bins and reading this pass's result need no barrier of their own.
template <int E>
__device__ __forceinline__ uint64_t radix_select(const uint64_t (&key)[E], uint32_t need,
                                                 int index_bits, SelectShared &sh) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint64_t prefix = 0, prefix_mask = 0;
    if (tid < 256) sh.hist[0][tid] = 0;
    __syncthreads();
    int pass = 0;
    for (int shift = 56; shift >= 0; shift -= 8) {
        if (shift < 32 && shift >= index_bits) {
            // ~index has only ones up here: nothing to decide
            prefix |= 0xffull << shift;
            prefix_mask |= 0xffull << shift;
            continue;
        }
        uint32_t *hist = sh.hist[pass & 1];
        if (tid < 256) sh.hist[(pass & 1) ^ 1][tid] = 0;          // for the next pass
        // Scores crowd into few leading digits: LDS atomics on one bin are served one lane at a
        // time, so a wavefront whose matching composites span few digits (the rule in the first
        // passes) counts them digit by digit with ballots and adds each count with one atomic;
        // one whose digits are spread (the rule later) adds its composites one by one.
        uint32_t lo = 256u, hi = 0u;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const uint64_t c = key[e];
            const bool match = c != 0 && (c & prefix_mask) == prefix;
            const uint32_t digit = static_cast<uint32_t>(c >> shift) & 0xffu;
            lo = match ? min(lo, digit) : lo;
            hi = match ? max(hi, digit) : hi;
        }
        const uint32_t wave_lo = wave_min_u32(lo), wave_hi = wave_max_u32(hi);
        if (wave_lo <= wave_hi) {                                   // some composite matches
            if (wave_hi - wave_lo < kFewDigits) {
                for (uint32_t d = wave_lo; d <= wave_hi; ++d) {     // the same trip count in every lane
                    uint32_t count = 0;
#pragma unroll
                    for (int e = 0; e < E; ++e) {
                        const uint64_t c = key[e];
                        const bool here = c != 0 && (c & prefix_mask) == prefix &&
                                          (static_cast<uint32_t>(c >> shift) & 0xffu) == d;
                        count += static_cast<uint32_t>(__popcll(__ballot(here)));
                    }
                    if (lane == 0 && count != 0) atomicAdd(&hist[d], count);
                }
            } else {
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const uint64_t c = key[e];
                    if (c != 0 && (c & prefix_mask) == prefix)
                        atomicAdd(&hist[static_cast<uint32_t>(c >> shift) & 0xffu], 1u);
                }
            }
        }
        __syncthreads();
        if (wave == 0) {
            // lane l owns digits 4l..4l+3; find the digit where the count from the top reaches `need`
            uint32_t h[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) h[j] = hist[lane * 4 + j];
            const uint32_t local = h[0] + h[1] + h[2] + h[3];
            const uint32_t upto = wave_inclusive_scan_u32(local);       // lanes 0..l
            const uint32_t all = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(upto), 63));
            const uint32_t above = all - upto;                          // lanes l+1..63
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
                sh.digit[pass & 1] = static_cast<uint32_t>(digit);
                sh.need[pass & 1] = remaining;
                sh.bin[pass & 1] = in_bin;
            }
        }
        __syncthreads();
        prefix |= static_cast<uint64_t>(sh.digit[pass & 1]) << shift;
        prefix_mask |= 0xffull << shift;
        need = sh.need[pass & 1];
        const bool take_all = sh.bin[pass & 1] == need;
        ++pass;
        // every composite that still matches the prefix is wanted: the rest decides nothing
        if (take_all) break;
    }
    return prefix;
}

// Composites at or above the threshold go to `out` (LDS or global), in no particular order;
// returns how many there were (the same value in every thread).  A thread counts its own, a
// wavefront scan places them, one atomic per wavefront reserves the space.
template <int E>
__device__ __forceinline__ uint32_t compact_above(const uint64_t (&key)[E], uint64_t threshold,
                                                  uint64_t *out, SelectShared &sh) {
    const int lane = threadIdx.x & 63;
    if (threadIdx.x == 0) sh.count = 0;
    __syncthreads();
    uint32_t mine = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) mine += (key[e] != 0 && key[e] >= threshold) ? 1u : 0u;
    const uint32_t incl = wave_inclusive_scan_u32(mine);
    uint32_t base = 0;
    if (lane == 63 && incl != 0) base = atomicAdd(&sh.count, incl);
    base = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(base), 63));
    uint32_t at = base + incl - mine;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        if (key[e] != 0 && key[e] >= threshold) out[at++] = key[e];
    }
    __syncthreads();
    return sh.count;
}

// Bitonic sort, descending, of sort_len = R * (active threads) composites held R per thread:
// element i = t*R + r sits in register r of thread t.  A step with partner distance J is done
// inside the thread (J < R), by a lane exchange (partner thread in the same wavefront) or
// through LDS (partner in another wavefront: 10 of the 66 steps of a 2048-element sort).
// Stages and steps are unrolled at compile time, so a step is straight-line code.
// (The LDS steps alternate between the two halves of the buffer when the sort fits one half,
// which saves the barrier that would otherwise protect the previous step's readers.)
template <int R, int K, int J>
__device__ __forceinline__ void bitonic_step(uint64_t (&key)[R], int t, bool active, uint64_t *lds,
                                             bool two_halves, int &parity) {
    if constexpr (J < R) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if ((r & J) == 0) {
                const uint64_t x = key[r], y = key[r | J];
                const bool descending = ((t * R + r) & K) == 0;
                const bool swap = (x < y) == descending;
                key[r] = swap ? y : x;
                key[r | J] = swap ? x : y;
            }
        }
    } else {
        constexpr int D = J / R;                   // partner thread: t ^ D
        // the thread with the clear bit holds the lower-numbered elements of its pairs
        const bool want_max = ((t & D) == 0) == (((t * R) & K) == 0);
        uint64_t theirs[R];
        if constexpr (D < 64) {
#pragma unroll
            for (int r = 0; r < R; ++r) theirs[r] = lane_xor<D>(key[r]);
        } else {
            uint64_t *half = lds;
            if (two_halves) { half += parity * (kLdsSortCap / 2); parity ^= 1; }
            else __syncthreads();                  // earlier readers of the buffer are done
            if (active) {
#pragma unroll
                for (int r = 0; r < R; ++r) half[t * R + r] = key[r];
            }
            __syncthreads();
#pragma unroll
            for (int r = 0; r < R; ++r) theirs[r] = active ? half[(t ^ D) * R + r] : 0;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const bool take = want_max ? (theirs[r] > key[r]) : (theirs[r] < key[r]);
            key[r] = take ? theirs[r] : key[r];
        }
    }
}

template <int R, int K, int J>
__device__ __forceinline__ void bitonic_stage(uint64_t (&key)[R], int t, bool active, uint64_t *lds,
                                              bool two_halves, int &parity) {
    bitonic_step<R, K, J>(key, t, active, lds, two_halves, parity);
    if constexpr (J > 1) bitonic_stage<R, K, J / 2>(key, t, active, lds, two_halves, parity);
}

template <int R, int K>
__device__ __forceinline__ void bitonic_stages(uint64_t (&key)[R], int sort_len, int t, bool active,
                                               uint64_t *lds, bool two_halves, int &parity) {
    if (K > sort_len) return;                      // uniform over the workgroup
    bitonic_stage<R, K, K / 2>(key, t, active, lds, two_halves, parity);
    if constexpr (K < kLdsSortCap && K < R * kThreads)
        bitonic_stages<R, K * 2>(key, sort_len, t, active, lds, two_halves, parity);
}

// `lds` holds kLdsSortCap composites and is free for the sort's use (every thread has taken its
// composites out of it; the caller has a barrier between that and this call).
template <int R>
__device__ __forceinline__ void bitonic_sort_registers(uint64_t (&key)[R], int sort_len, uint64_t *lds) {
    const int t = threadIdx.x;
    int parity = 0;
    bitonic_stages<R, 2>(key, sort_len, t, t * R < sort_len, lds, sort_len <= kLdsSortCap / 2, parity);
}

// One workgroup selects and sorts the M largest of n inputs: fp32 scores with their position
// as index (FROM_SCORES) or ready-made composites (0 = none).  n <= E * 1024,
// M <= sort_len <= min(R * 1024, 8192), sort_len a power of two; sort_len / R threads sort.
template <int E, int R, bool FROM_SCORES>
__global__ __launch_bounds__(kThreads) void select_resident_kernel(const void *__restrict__ input, int n,
                                                                   int M, int sort_len, int index_bits,
                                                                   int32_t *indices, float *scores_out) {
    __shared__ uint64_t buf[kLdsSortCap];
    __shared__ SelectShared sh;
    const int tid = threadIdx.x;
    uint64_t key[E];
    PPOW_SELECT_TICK(0);
    if (FROM_SCORES) {
        float x[E];
#pragma unroll
        for (int e = 0; e < E; ++e)              // every load in flight before the first use
            x[e] = static_cast<const float *>(input)[min(e * kThreads + tid, n - 1)];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int i = e * kThreads + tid;
            key[e] = i < n ? composite(x[e], i) : 0;
        }
    } else {
#pragma unroll
        for (int e = 0; e < E; ++e)
            key[e] = static_cast<const uint64_t *>(input)[min(e * kThreads + tid, n - 1)];
#pragma unroll
        for (int e = 0; e < E; ++e) key[e] = (e * kThreads + tid) < n ? key[e] : 0;
    }
    PPOW_SELECT_TICK(1);
    const uint64_t threshold = radix_select<E>(key, static_cast<uint32_t>(M), index_bits, sh);
    PPOW_SELECT_TICK(2);
    for (int i = tid; i < sort_len; i += kThreads) buf[i] = 0;    // 0 sorts below every composite
    compact_above<E>(key, threshold, buf, sh);                    // its first barrier orders the fill
    PPOW_SELECT_TICK(3);
    uint64_t mine[R];
#pragma unroll
    for (int r = 0; r < R; ++r) mine[r] = (tid * R + r) < sort_len ? buf[tid * R + r] : 0;
    __syncthreads();                                              // the buffer now serves the sort
    bitonic_sort_registers<R>(mine, sort_len, buf);
    PPOW_SELECT_TICK(4);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int i = tid * R + r;
        if (i < M) {
            indices[i] = static_cast<int32_t>(~static_cast<uint32_t>(mine[r]));
            if (scores_out) scores_out[i] = from_ordered_bits(static_cast<uint32_t>(mine[r] >> 32));
        }
    }
    PPOW_SELECT_TICK(5);
}

// One workgroup per slice of kSliceLen scores: the slice's own `keep` largest composites (all
// of them if the slice has no more), unsorted, zero-padded to `keep`, to candidates[slice].
constexpr int kSliceE = 16;
constexpr int kSliceLen = kSliceE * kThreads;
__global__ __launch_bounds__(kThreads) void select_slice_kernel(const float *__restrict__ score, int B,
                                                                int keep, int index_bits,
                                                                uint64_t *candidates) {
    __shared__ SelectShared sh;
    const int tid = threadIdx.x;
    const int base = blockIdx.x * kSliceLen;
    const int valid = min(B - base, kSliceLen);
    float x[kSliceE];
#pragma unroll
    for (int e = 0; e < kSliceE; ++e) x[e] = score[base + min(e * kThreads + tid, valid - 1)];
    uint64_t key[kSliceE];
#pragma unroll
    for (int e = 0; e < kSliceE; ++e) {
        const int i = e * kThreads + tid;
        key[e] = i < valid ? composite(x[e], base + i) : 0;
    }
    uint64_t *out = candidates + static_cast<size_t>(blockIdx.x) * keep;
    uint64_t threshold = 1;                                      // everything there is
    if (valid > keep) threshold = radix_select<kSliceE>(key, static_cast<uint32_t>(keep), index_bits, sh);
    const uint32_t count = compact_above<kSliceE>(key, threshold, out, sh);
    for (int i = static_cast<int>(count) + tid; i < keep; i += kThreads) out[i] = 0;
}

int next_pow2(int x) {
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

// How a request is served.
struct SelectPlan {
    enum { kResident, kSliced, kGeneral } kind;
    int sort_len;
    int slices;        // kSliced: workgroups of the first kernel
    int keep;          // kSliced: survivors per slice
};

SelectPlan plan_select(int64_t B, int32_t M) {
    SelectPlan p;
    p.sort_len = next_pow2(M);
    p.slices = 0;
    p.keep = 0;
    p.kind = SelectPlan::kGeneral;
    if (p.sort_len > kLdsSortCap) return p;
    if (B <= 32 * kThreads) {
        p.kind = SelectPlan::kResident;
        return p;
    }
    const int64_t slices = (B + kSliceLen - 1) / kSliceLen;
    const int64_t keep = M < kSliceLen ? M : kSliceLen;
    if (slices * keep <= 32 * kThreads) {
        p.kind = SelectPlan::kSliced;
        p.slices = static_cast<int>(slices);
        p.keep = static_cast<int>(keep);
    }
    return p;
}

template <int E, bool FROM_SCORES>
void launch_resident_e(const void *input, int n, int M, int sort_len, int index_bits, int32_t *indices,
                       float *scores, hipStream_t stream) {
    // composites per thread in the sort: as few as the sort's length allows, so that all 16
    // wavefronts share the work and hide each other's exchange latencies (8 per thread on a
    // quarter of the threads measured 2.5 times slower)
    if (sort_len <= 2 * kThreads)
        hipLaunchKernelGGL((select_resident_kernel<E, 2, FROM_SCORES>), dim3(1), dim3(kThreads), 0, stream,
                           input, n, M, sort_len, index_bits, indices, scores);
    else if (sort_len <= 4 * kThreads)
        hipLaunchKernelGGL((select_resident_kernel<E, 4, FROM_SCORES>), dim3(1), dim3(kThreads), 0, stream,
                           input, n, M, sort_len, index_bits, indices, scores);
    else
        hipLaunchKernelGGL((select_resident_kernel<E, 8, FROM_SCORES>), dim3(1), dim3(kThreads), 0, stream,
                           input, n, M, sort_len, index_bits, indices, scores);
}

template <bool FROM_SCORES>
void launch_resident(const void *input, int n, int M, int sort_len, int index_bits, int32_t *indices,
                     float *scores, hipStream_t stream) {
    if (n <= 4 * kThreads)
        launch_resident_e<4, FROM_SCORES>(input, n, M, sort_len, index_bits, indices, scores, stream);
    else if (n <= 16 * kThreads)
        launch_resident_e<16, FROM_SCORES>(input, n, M, sort_len, index_bits, indices, scores, stream);
    else
        launch_resident_e<32, FROM_SCORES>(input, n, M, sort_len, index_bits, indices, scores, stream);
}

}  // namespace

#if PPOW_SELECT_TIMING
extern "C" void ppow_debug_select_ticks(long long *out) {
    (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_select_ticks), sizeof(long long) * 8);
}
#endif

size_t select_workspace_bytes(int64_t B, int32_t M) {
    const SelectPlan p = plan_select(B, M);
    size_t need = 0;
    if (p.kind == SelectPlan::kGeneral && p.sort_len > kLdsSortCap)
        need = static_cast<size_t>(p.sort_len) * sizeof(uint64_t);
    if (p.kind == SelectPlan::kSliced)
        need = static_cast<size_t>(p.slices) * p.keep * sizeof(uint64_t);
    return need < 256 ? 256 : need;
}

hipError_t launch_select(const float *score, int64_t B, int32_t M, int32_t *indices, float *scores,
                         void *workspace, hipStream_t stream) {
    const SelectPlan p = plan_select(B, M);
    int index_bits = 0;
    while ((int64_t{1} << index_bits) < B) ++index_bits;
    index_bits = ((index_bits + 7) / 8) * 8;          // whole 8-bit digits
    switch (p.kind) {
    case SelectPlan::kResident:
        launch_resident<true>(score, static_cast<int>(B), M, p.sort_len, index_bits, indices, scores, stream);
        break;
    case SelectPlan::kSliced: {
        uint64_t *candidates = static_cast<uint64_t *>(workspace);
        hipLaunchKernelGGL(select_slice_kernel, dim3(p.slices), dim3(kThreads), 0, stream, score,
                           static_cast<int>(B), p.keep, index_bits, candidates);
        const hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
        launch_resident<false>(candidates, p.slices * p.keep, M, p.sort_len, index_bits, indices, scores,
                               stream);
        break;
    }
    case SelectPlan::kGeneral:
        if (p.sort_len <= kLdsSortCap)
            hipLaunchKernelGGL(select_general_kernel<true>, dim3(1), dim3(kThreads), 0, stream, score,
                               static_cast<int>(B), M, p.sort_len, index_bits, indices, scores,
                               static_cast<uint64_t *>(nullptr));
        else
            hipLaunchKernelGGL(select_general_kernel<false>, dim3(1), dim3(kThreads), 0, stream, score,
                               static_cast<int>(B), M, p.sort_len, index_bits, indices, scores,
                               static_cast<uint64_t *>(workspace));
        break;
    }
    return hipGetLastError();
}

}  // namespace ppow
