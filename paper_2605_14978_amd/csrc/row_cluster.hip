// Row-pair reduction with the second pass served from on-chip memory: a cluster of S workgroups
// shares one row pair, each member streams its slice of both rows from HBM once, keeps the raw
// 128-bit chunks in registers and LDS, and after the members have exchanged their partial
// softmax sums it computes its share of sum_y min(P(y), Q(y)) (Appendix B.1) from that copy.
// Every logit is fetched from HBM once, where the one-workgroup-per-row kernel has to read
// the row pair twice.  A CU holds 2 workgroups x (80 KB of VGPRs + 76 KB of LDS) of logits, so
// 256 CUs keep about 64 fp32 rows of 152K logits (or 150 bf16 rows of 128K) in flight.
//
// The kernel is persistent and its grid is never larger than what the device holds at once
// (occupancy of this kernel x compute units), so every workgroup becomes resident as soon as
// whatever else runs on the device has made room, and the one wait of a member -- for the
// partial sums of the other members of its own cluster, which each of them publishes
// unconditionally -- always ends.  (Two such kernels at once could each hold half the device
// and wait for the other half: launches are therefore chained, see ClusterChain below.)  The
// wait is bounded all the same: if it ever expired the kernel would set the status word and
// leave, and the window epilogue then marks every window of the call (accepted_len = -3)
// instead of publishing numbers made from records that were never written.
//
// Exchange protocol per row (epoch e of the cluster, slots double-buffered by e & 1).  Every
// exchanged value is one 64-bit word {tag = e+1, fp32 bits}, written and read with agent-scope
// atomics, so a reader recognises the word of the right epoch by itself and no ordering
// between different addresses -- hence no cache-wide fence -- is needed:
//   member: publish its partial sums;
//           wave 0 polls the S members' words until all carry the tag, combines them in
//           member order and hands the row totals to the workgroup through LDS;
//           pass 2 from registers/LDS; publish the partial min-sum;
//           member (e mod S) polls the S min-sums, adds them in member order and finishes
//           the row.  Fixed order => bitwise reproducible.
#include <atomic>
#include <mutex>

#include "row_math.h"

namespace ppow {
namespace {

#ifndef PPOW_CLUSTER_THREADS
#define PPOW_CLUSTER_THREADS 512
#endif
#ifndef PPOW_CLUSTER_WAVES_PER_EU
#define PPOW_CLUSTER_WAVES_PER_EU 4            // 2 workgroups of 8 waves per CU -> 128 VGPRs
#endif
#ifndef PPOW_CLUSTER_REG_CHUNKS
#define PPOW_CLUSTER_REG_CHUNKS 5              // 128-bit chunks per row side a lane keeps in VGPRs
#endif
#ifndef PPOW_CLUSTER_LDS_BYTES
#define PPOW_CLUSTER_LDS_BYTES (76 * 1024)     // two workgroups per CU out of 160 KB
#endif
constexpr int kThreads = PPOW_CLUSTER_THREADS;
constexpr int kWaves = kThreads / 64;
constexpr int kRegChunks = PPOW_CLUSTER_REG_CHUNKS;
constexpr int kMaxMembers = 64;                // one lane of a wavefront per member
constexpr int kExchanged = 10;                 // words a member publishes per row
constexpr unsigned kDefaultMaxSpins = 1u << 24; // many seconds: members may be kept off the GPU for a
                                                // while by other streams' kernels, never this long

// scratch layout (bytes): [0,4) status | [256, ...) slots
constexpr size_t kSlotOffset = 256;
constexpr size_t kSlotLimit = 768 * 1024;      // slots end here (phase timings of a tuning build follow)
static_assert(kSlotLimit + 256 * 1024 <= kClusterScratchBytes, "scratch layout");
constexpr int kMaxClusters = 4096;

struct ClusterArgs {
    RowArgs row;
    int64_t rows;
    int32_t members;        // S
    int32_t clusters;
    int32_t slice_chunks;   // LDS part of a slice per row side, in 128-bit chunks
    uint32_t *status;
    uint64_t *slots;        // [clusters][2][kExchanged][stride]: word i of all members side by
                            // side, so the wavefront that collects them (member l on lane l)
                            // reads each word of the whole cluster with one coalesced request
    int32_t stride;         // S rounded up to a multiple of 8 (64 bytes)
    uint32_t max_spins;     // looks at a slot before a wait gives up
};

// 128-bit load from global memory straight into LDS: lane i of the wave writes 16 bytes at
// lds_wave_base + 16*i (lds_wave_base must be wave-uniform).  Streaming cache policy.
__device__ __forceinline__ void direct_to_lds(const raw4 *src, raw4 *lds_wave_base) {
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void *)(src),
        (__attribute__((address_space(3))) void *)(lds_wave_base), 16, 0,
        PPOW_ROW_NONTEMPORAL ? 2 : 0);
}

__device__ __forceinline__ void publish(uint64_t *p, uint32_t tag, uint32_t bits) {
    __hip_atomic_store(p, (static_cast<uint64_t>(tag) << 32) | bits, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void publish(uint64_t *p, uint32_t tag, float v) {
    publish(p, tag, __builtin_bit_cast(uint32_t, v));
}
__device__ __forceinline__ uint64_t observe(const uint64_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ bool tagged(uint64_t w, uint32_t tag) {
    return static_cast<uint32_t>(w >> 32) == tag;
}
__device__ __forceinline__ float value_of(uint64_t w) { return as_float(static_cast<uint32_t>(w)); }

__global__ void zero_words_kernel(uint32_t *p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// Two workgroups per CU: the register allocation is held to 128 VGPRs (4 waves per SIMD).
// Optional phase timing for tuning (off in the product build): thread 0 of each workgroup adds
// up shader-clock cycles per phase and stores them behind the exchange slots.
#ifndef PPOW_CLUSTER_TIMING
#define PPOW_CLUSTER_TIMING 0
#endif
#if PPOW_CLUSTER_TIMING
#define PPOW_TICK(i) do { if (tid == 0) { const long long now_ = clock64(); phase_[i] += now_ - last_; last_ = now_; } } while (0)
#else
#define PPOW_TICK(i) do { } while (0)
#endif
#if PPOW_CLUSTER_TIMING
constexpr size_t kTimingOffset = kSlotLimit;
#endif

// What the closing member keeps of a row until it closes it (in LDS: it outlives the row by
// most of the next one, and registers are what limits how much of a slice stays on chip).
struct PendingClose {
    int64_t row;
    uint32_t tag;
    const uint64_t *slot_base;
    RowTotals totals;
    DraftedToken drafted;
};

// Wave 0 of the closing member: add the S partial min-sums in member order, finish the row.
template <int DTYPE>
__device__ __forceinline__ void close_row(const ClusterArgs &ca, const PendingClose &p, int lane) {
    const bool has = lane < ca.members;
    const uint64_t *word = p.slot_base + 9 * ca.stride + (has ? lane : 0);
    uint64_t w = 0;
    unsigned spins = 0;
    for (;;) {
        w = observe(word);
        if (__all(tagged(w, p.tag) || !has)) break;
        __builtin_amdgcn_s_sleep(1);
        if (++spins > ca.max_spins) {            // never expected: report, do not hang
            if (lane == 0)
                __hip_atomic_fetch_or(ca.status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            break;
        }
    }
    const float expected = wave_sum(has ? value_of(w) : 0.f);
    if (lane == 0) finish_row<DTYPE, ClusterFold>(ca.row, p.row, p.totals, expected, p.drafted);
}

template <int DTYPE, bool REV>
__global__ __launch_bounds__(kThreads)
__attribute__((amdgpu_waves_per_eu(PPOW_CLUSTER_WAVES_PER_EU, PPOW_CLUSTER_WAVES_PER_EU)))
void row_cluster_kernel(ClusterArgs ca) {
    using S = Storage<DTYPE>;
    using elem = typename S::elem;
    constexpr int VEC = S::VEC;
    constexpr int kRegSpan = kRegChunks * kThreads;       // chunks of a slice kept in registers
    constexpr bool KEEP = DTYPE == PPOW_F32;              // 4 fp32 per chunk: room for the exponentials

    extern __shared__ raw4 lds[];
    __shared__ float sh_m[kWaves][3];
    __shared__ float sh_f[kWaves][6];
    __shared__ int sh_i[kWaves];
    __shared__ int sh_abort;
    __shared__ float sh_g[9];

    const RowArgs &args = ca.row;
    const int members = ca.members;
    const int cluster = blockIdx.x / members;
    const int member = blockIdx.x - cluster * members;
    if (cluster >= ca.clusters) return;                 // whole workgroup leaves together

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int V = static_cast<int>(args.V);
    raw4 *lds_a = lds;
    raw4 *lds_b = lds + ca.slice_chunks;

    __shared__ PendingClose pending;
    bool pending_open = false;
#if PPOW_CLUSTER_TIMING
    long long phase_[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    long long last_ = clock64();
#endif

    uint32_t epoch = 0;
    for (int64_t row = cluster; row < ca.rows; row += ca.clusters, ++epoch) {
        const elem *row_a = static_cast<const elem *>(args.target) + row * args.V;
        const elem *row_b = static_cast<const elem *>(args.draft) + row * args.V;
        const uintptr_t addr = reinterpret_cast<uintptr_t>(row_a);
        int head = static_cast<int>(((kRowAlign - (addr & (kRowAlign - 1u))) & (kRowAlign - 1u)) / sizeof(elem));
        head = head < V ? head : V;
        const int nchunks = (V - head) / VEC;
        const int tail_begin = head + nchunks * VEC;

        // this member's slice of the vector body: the first kRegSpan chunks stay in registers,
        // the rest (at most slice_chunks) in LDS
        const int per = ((nchunks + members - 1) / members + 7) & ~7;   // whole cache lines
        const int c0 = member * per;
        int n = nchunks - c0;
        n = n < per ? n : per;
        n = n > 0 ? n : 0;
        const raw4 *pa = reinterpret_cast<const raw4 *>(row_a + head) + c0;
        const raw4 *pb = reinterpret_cast<const raw4 *>(row_b + head) + c0;

        // the member that will close this row fetches the drafted token's logits early
        const bool closer = member == static_cast<int>(epoch % static_cast<uint32_t>(members));
        DraftedToken drafted = {0, 0.f, 0.f};
        if (closer && tid == 0) drafted = load_drafted_token<DTYPE>(args, row);

        // ---- pass 1: HBM -> registers (-> LDS) + running sums ------------------------------
        raw4 ka[kRegChunks], kb[kRegChunks];
#pragma unroll
        for (int k = 0; k < kRegChunks; ++k) {
            const int c = tid + k * kThreads;
            if (c < n) {
                ka[k] = load_chunk<true>(pa + c);
                kb[k] = load_chunk<true>(pb + c);
            }
        }
        // the LDS part goes from HBM straight into LDS (no registers in between), lane i of a
        // wave landing at base + 16*i, so every load of the slice is in flight at once
        for (int c = tid + kRegSpan; c < n; c += kThreads) {
            const int wave_first = c - lane - kRegSpan;            // wave-uniform LDS chunk index
            direct_to_lds(pa + c, lds_a + wave_first);
            direct_to_lds(pb + c, lds_b + wave_first);
        }
        LaneState s;
        s.reset();
        // fp32 rows: the raw logits are not needed after this pass, so the two exponentials of
        // every pair take their place in the registers / LDS and pass 2 only rescales them
        // (the position of the lane's maximum is tracked to the element instead of re-scanned).
        // If a lane's reference moves (rare), what it has kept so far is rescaled to the new one.
        int first_elem = -1;
        auto rescale_kept = [&](int regs_upto, int lds_upto, float fa, float fb) {
#pragma unroll
            for (int k = 0; k < kRegChunks; ++k) {
                if (k < regs_upto && tid + k * kThreads < n) {
                    float ea[VEC], eb[VEC];
                    S::unpack(ka[k], ea);
                    S::unpack(kb[k], eb);
#pragma unroll
                    for (int j = 0; j < VEC; ++j) { ea[j] *= fa; eb[j] *= fb; }
                    if constexpr (KEEP) { ka[k] = S::pack(ea); kb[k] = S::pack(eb); }
                }
            }
            for (int c = tid + kRegSpan; c < lds_upto; c += kThreads) {
                float ea[VEC], eb[VEC];
                S::unpack(lds_a[c - kRegSpan], ea);
                S::unpack(lds_b[c - kRegSpan], eb);
#pragma unroll
                for (int j = 0; j < VEC; ++j) { ea[j] *= fa; eb[j] *= fb; }
                if constexpr (KEEP) { lds_a[c - kRegSpan] = S::pack(ea); lds_b[c - kRegSpan] = S::pack(eb); }
            }
        };
        auto moved = [&](float ra, float rb, float &fa, float &fb) {
            if (s.rho_a == ra && s.rho_b == rb) return false;
            fa = fast_exp2(ra - s.rho_a);          // ra = -inf (nothing kept yet) gives 0: harmless
            fb = fast_exp2(rb - s.rho_b);
            return true;
        };
#pragma unroll
        for (int k = 0; k < kRegChunks; ++k) {
            const int cr = tid + k * kThreads;
            if (cr < n) {
                float a[VEC], b[VEC];
                S::unpack(ka[k], a);
                S::unpack(kb[k], b);
                if constexpr (KEEP) {
                    const float ra = s.rho_a, rb = s.rho_b;
                    float ea[VEC], eb[VEC], fa, fb;
                    fold_chunk_keep<ClusterFold, VEC, REV>(s, a, b, cr, first_elem, ea, eb);
                    if (k > 0 && moved(ra, rb, fa, fb)) rescale_kept(k, 0, fa, fb);
                    ka[k] = S::pack(ea);
                    kb[k] = S::pack(eb);
                } else {
                    fold_chunk<ClusterFold, VEC, REV>(s, a, b, cr);
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(0);              // the direct loads have landed in LDS
        for (int c = tid + kRegSpan; c < n; c += kThreads) {
            float a[VEC], b[VEC];
            S::unpack(lds_a[c - kRegSpan], a);
            S::unpack(lds_b[c - kRegSpan], b);
            if constexpr (KEEP) {
                const float ra = s.rho_a, rb = s.rho_b;
                float ea[VEC], eb[VEC], fa, fb;
                fold_chunk_keep<ClusterFold, VEC, REV>(s, a, b, c, first_elem, ea, eb);
                if (moved(ra, rb, fa, fb)) rescale_kept(kRegChunks, c, fa, fb);
                lds_a[c - kRegSpan] = S::pack(ea);
                lds_b[c - kRegSpan] = S::pack(eb);
            } else {
                fold_chunk<ClusterFold, VEC, REV>(s, a, b, c);
            }
        }

        PPOW_TICK(0);                                   // load + fold
        // From here to the hand-over of the row totals the workgroup does little arithmetic but
        // sits on the critical path of its whole cluster (combine, publish, collect): its waves
        // go ahead of the other workgroup's bulk arithmetic on this CU.
        __builtin_amdgcn_s_setprio(1);
        // ragged ends of the row belong to member 0
        const int ragged = (member == 0) ? head + (V - tail_begin) : 0;
        float rag_v = PPOW_NEG_INF;
        int rag_i = INT_MAX;
        if (tid < ragged) {
            rag_i = (tid < head) ? tid : tail_begin + (tid - head);
            const float a1[1] = {S::load1(row_a + rag_i)};
            const float b1[1] = {S::load1(row_b + rag_i)};
            const float ra = s.rho_a, rb = s.rho_b;
            fold<ClusterFold, 1, REV>(s, a1, b1, a1[0], b1[0]);
            rag_v = a1[0];
            if constexpr (KEEP) {
                float fa, fb;
                if (moved(ra, rb, fa, fb)) rescale_kept(kRegChunks, n, fa, fb);
            }
        }

        // ---- workgroup combine of the slice ------------------------------------------------
        RowTotals t;
        t.ref_a = wave_max(s.rho_a);
        t.ref_b = wave_max(s.rho_b);
        t.row_max = wave_max(fmaxf(s.m_a, rag_v));
        if (lane == 0) { sh_m[wave][0] = t.ref_a; sh_m[wave][1] = t.ref_b; sh_m[wave][2] = t.row_max; }
        __syncthreads();
        t.ref_a = sh_m[0][0]; t.ref_b = sh_m[0][1]; t.row_max = sh_m[0][2];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) {
            t.ref_a = fmaxf(t.ref_a, sh_m[w][0]);
            t.ref_b = fmaxf(t.ref_b, sh_m[w][1]);
            t.row_max = fmaxf(t.row_max, sh_m[w][2]);
        }
        // (the sums below go to sh_f, not over sh_m: no barrier needed before they are written)

        // First index of the slice maximum: a lane that holds it knows the element (fp32) or
        // scans its own chunks (registers, then LDS) in index order (bf16).
        int arg_i = (rag_v == t.row_max) ? rag_i : INT_MAX;
        if (s.m_a == t.row_max && s.best >= 0) {
            int found = INT_MAX;
            if constexpr (KEEP) {
                found = head + c0 * VEC + first_elem;
            } else {
#pragma unroll
                for (int k = kRegChunks - 1; k >= 0; --k) {
                    const int cr = tid + k * kThreads;
                    if (cr < n) {
                        float a[VEC];
                        S::unpack(ka[k], a);
#pragma unroll
                        for (int j = VEC - 1; j >= 0; --j)
                            found = (a[j] == t.row_max) ? head + (c0 + cr) * VEC + j : found;
                    }
                }
                if (found == INT_MAX) {               // not in the register part: the LDS chunk
                    float a[VEC];
                    S::unpack(lds_a[s.best - kRegSpan], a);
#pragma unroll
                    for (int j = VEC - 1; j >= 0; --j)
                        found = (a[j] == t.row_max) ? head + (c0 + s.best) * VEC + j : found;
                }
            }
            arg_i = found < arg_i ? found : arg_i;
        }

        to_common_reference(s.rho_a, s.rho_b, t.ref_a, t.ref_b, s.z_a, s.s1, s.s2, s.z_b, s.s2r);
        t.z_a = wave_sum(s.z_a); t.s1 = wave_sum(s.s1); t.s2 = wave_sum(s.s2);
        t.z_b = wave_sum(s.z_b);
        t.s2r = REV ? wave_sum(s.s2r) : 0.f;
        arg_i = wave_min(arg_i);
        if (lane == 0) {
            sh_f[wave][0] = t.z_a; sh_f[wave][1] = t.s1; sh_f[wave][2] = t.s2; sh_f[wave][3] = t.z_b;
            sh_f[wave][4] = t.s2r; sh_i[wave] = arg_i;
        }
        __syncthreads();

        PPOW_TICK(1);                                   // workgroup combine
        // ---- publish the slice's partial sums ------------------------------------------------
        const uint32_t tag = epoch + 1u;
        uint64_t *slot_base = ca.slots + (static_cast<size_t>(cluster) * 2 + (epoch & 1u)) *
                                             kExchanged * ca.stride;
        uint64_t *my_slot = slot_base + member;
        if (tid < 9) {
            // lane i publishes word i: the two references, the five sums (added over the waves
            // in wave order), the slice maximum and its first index; an empty slice publishes
            // the neutral element (references at -inf)
            uint32_t bits;
            if (tid >= 2 && tid <= 6) {
                float v = sh_f[0][tid - 2];
#pragma unroll
                for (int w = 1; w < kWaves; ++w) v += sh_f[w][tid - 2];
                bits = __builtin_bit_cast(uint32_t, v);
            } else if (tid == 8) {
                int best = sh_i[0];
#pragma unroll
                for (int w = 1; w < kWaves; ++w) best = sh_i[w] < best ? sh_i[w] : best;
                bits = static_cast<uint32_t>(best);
            } else {
                bits = __builtin_bit_cast(uint32_t, tid == 0 ? t.ref_a : tid == 1 ? t.ref_b : t.row_max);
            }
            publish(my_slot + tid * ca.stride, tag, bits);
        }

        // A row this member still has to close is closed here, off the critical path: its
        // min-sums were published a whole row ago, and the other members are now busy
        // reaching the exchange this member has just joined.
        PPOW_TICK(2);                                   // publish
        if (pending_open && wave == 0) close_row<DTYPE>(ca, pending, lane);
        pending_open = false;
        PPOW_TICK(3);                                   // deferred close

        // ---- wave 0 collects the S partials (member l on lane l) and combines them ----------
        if (wave == 0) {
            const bool has = lane < members;
            const uint64_t *slot = slot_base + (has ? lane : 0);
            uint64_t w[9];
            unsigned spins = 0;
            int abort = 0;
            for (;;) {
                bool ok = true;
#pragma unroll
                for (int i = 0; i < 9; ++i) {
                    w[i] = observe(slot + i * ca.stride);
                    ok = ok && tagged(w[i], tag);
                }
                if (__all(ok || !has)) break;
                __builtin_amdgcn_s_sleep(1);
                // never expected: report and leave instead of hanging; a wait that expired
                // anywhere ends every other wait at its next look at the status word
                ++spins;
                if (spins > ca.max_spins ||
                    ((spins & 255u) == 0 &&
                     __hip_atomic_load(ca.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)) {
                    abort = 1;
                    break;
                }
            }
            if (abort && lane == 0)
                __hip_atomic_fetch_or(ca.status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            float rho_a = has ? value_of(w[0]) : PPOW_NEG_INF;
            float rho_b = has ? value_of(w[1]) : PPOW_NEG_INF;
            float z_a = has ? value_of(w[2]) : 0.f;
            float s1 = has ? value_of(w[3]) : 0.f;
            float s2 = has ? value_of(w[4]) : 0.f;
            float z_b = has ? value_of(w[5]) : 0.f;
            float s2r = has ? value_of(w[6]) : 0.f;
            const float mx = has ? value_of(w[7]) : PPOW_NEG_INF;
            const int idx = has ? static_cast<int>(static_cast<uint32_t>(w[8])) : INT_MAX;
            const float ref_a = wave_max(rho_a);
            const float ref_b = wave_max(rho_b);
            const float row_max = wave_max(mx);
            to_common_reference(rho_a, rho_b, ref_a, ref_b, z_a, s1, s2, z_b, s2r);
            z_a = wave_sum(z_a); s1 = wave_sum(s1); s2 = wave_sum(s2);
            z_b = wave_sum(z_b); s2r = wave_sum(s2r);
            const int arg = wave_min(mx == row_max ? idx : INT_MAX);
            if (lane == 0) {
                sh_g[0] = ref_a; sh_g[1] = ref_b; sh_g[2] = z_a; sh_g[3] = s1; sh_g[4] = s2;
                sh_g[5] = z_b; sh_g[6] = s2r; sh_g[7] = row_max; sh_g[8] = __int_as_float(arg);
                sh_abort = abort;
            }
        }
        PPOW_TICK(4);                                   // poll + combine of the partials
        __syncthreads();
        __builtin_amdgcn_s_setprio(0);
        if (sh_abort) return;                              // uniform: the whole workgroup leaves
        RowTotals g;
        g.ref_a = sh_g[0]; g.ref_b = sh_g[1]; g.z_a = sh_g[2]; g.s1 = sh_g[3]; g.s2 = sh_g[4];
        g.z_b = sh_g[5]; g.s2r = sh_g[6]; g.row_max = sh_g[7]; g.arg_i = __float_as_int(sh_g[8]);

        // ---- pass 2 from registers and LDS: this slice's share of sum_y min(P(y), Q(y)) -----
        const float lam_a = g.ref_a + fast_log2(g.z_a);
        const float lam_b = g.ref_b + fast_log2(g.z_b);
        float acc = 0.f;
        // kept exponentials are relative to this lane's references: one scale per side
        const float keep_a = (KEEP && s.rho_a != PPOW_NEG_INF) ? fast_exp2(s.rho_a - lam_a) : 0.f;
        const float keep_b = (KEEP && s.rho_b != PPOW_NEG_INF) ? fast_exp2(s.rho_b - lam_b) : 0.f;
#pragma unroll
        for (int k = 0; k < kRegChunks; ++k) {
            if (tid + k * kThreads < n) {
                float a[VEC], b[VEC];
                S::unpack(ka[k], a);
                S::unpack(kb[k], b);
                acc += KEEP ? min_prob_sum_kept<VEC>(a, b, keep_a, keep_b)
                            : min_prob_sum<VEC>(a, b, lam_a, lam_b);
            }
        }
        for (int cc = tid + kRegSpan; cc < n; cc += kThreads) {
            float a[VEC], b[VEC];
            S::unpack(lds_a[cc - kRegSpan], a);
            S::unpack(lds_b[cc - kRegSpan], b);
            acc += KEEP ? min_prob_sum_kept<VEC>(a, b, keep_a, keep_b)
                        : min_prob_sum<VEC>(a, b, lam_a, lam_b);
        }
        if (tid < ragged) {
            const float a1[1] = {S::load1(row_a + rag_i)};
            const float b1[1] = {S::load1(row_b + rag_i)};
            acc += min_prob_sum<1>(a1, b1, lam_a, lam_b);
        }
        acc = wave_sum(acc);
        PPOW_TICK(5);                                   // barrier after poll + pass 2
        if (lane == 0) sh_f[wave][5] = acc;
        __syncthreads();
        if (tid == 0) {
            float part = sh_f[0][5];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) part += sh_f[w][5];
            publish(my_slot + 9 * ca.stride, tag, part);
        }

        // ---- the closing member (it rotates with the epoch) finishes the row later, after it
        //      has joined the next row's exchange (or after the loop) ---------------------------
        if (closer) {
            pending_open = true;
            if (tid == 0) {         // read again by wave 0 only, after the barriers in between
                pending.row = row;
                pending.tag = tag;
                pending.slot_base = slot_base;
                pending.totals = g;
                pending.drafted = drafted;
            }
        }
        __syncthreads();        // sh_* and the LDS slice are reused by the next row
        PPOW_TICK(6);                                   // second publish + barriers
    }
    if (pending_open && wave == 0) close_row<DTYPE>(ca, pending, lane);
#if PPOW_CLUSTER_TIMING
    if (tid == 0) {
        long long *out = reinterpret_cast<long long *>(reinterpret_cast<char *>(ca.status) + kTimingOffset) +
                         static_cast<size_t>(blockIdx.x) * 8;
        for (int i = 0; i < 8; ++i) out[i] = phase_[i];
    }
#endif
}

// Compute units of the current device (0 when it cannot be queried), cached per device.
int compute_units() {
    static thread_local int cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (cached[dev] == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) {
            (void)hipGetLastError();
            return 0;
        }
        cached[dev] = cus;
    }
    return cached[dev];
}

// Two cluster kernels must never share the GPU: each assumes that all of its workgroups become
// resident, and two of them that are each half resident would wait for each other until the
// bounded waits expire.  Launches on different streams are therefore chained through an event
// per device: a launch waits for the previous cluster kernel on that device to finish.  The
// event is created by the first launch on a device (or by prepare_cluster_chain) and lives
// until release_cluster_chain() -- the library's ppow_release() -- destroys it; nothing in the
// library refers to it after that, and a later launch simply creates a new one.
struct ClusterChain {
    std::mutex lock;
    hipEvent_t done[64] = {};
    bool have[64] = {};
    bool recorded[64] = {};
};
ClusterChain &cluster_chain() {
    static ClusterChain chain;
    return chain;
}
std::atomic<uint32_t> g_max_spins{kDefaultMaxSpins};

template <int DTYPE, bool REV>
hipError_t launch_variant(ClusterArgs &ca, int lds_bytes, int cus, hipStream_t stream, bool *launched) {
    const void *fn = reinterpret_cast<const void *>(row_cluster_kernel<DTYPE, REV>);
    // resident workgroups per CU for this LDS size, queried once per variant and size
    static thread_local int cached_lds = -1, cached_per_cu = 0;
    hipError_t err;
    if (cached_lds != lds_bytes) {
        err = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (err != hipSuccess) { (void)hipGetLastError(); return hipSuccess; }      // fall back
        int q = 0;
        err = hipOccupancyMaxActiveBlocksPerMultiprocessor(&q, fn, kThreads, lds_bytes);
        if (err != hipSuccess || q < 1) { (void)hipGetLastError(); return hipSuccess; }
        cached_lds = lds_bytes;
        cached_per_cu = q;
    }
    // The grid never exceeds what the device holds at once: that is what lets every member of
    // a cluster count on the others being (or becoming) resident.
    const int per_cu = cached_per_cu;
    int64_t clusters = static_cast<int64_t>(per_cu) * cus / ca.members;
    if (clusters > ca.rows) clusters = ca.rows;
    if (clusters > kMaxClusters) clusters = kMaxClusters;
    // both parities of every cluster's exchange words have to fit the scratch
    const size_t per_cluster = static_cast<size_t>(2) * kExchanged * ca.stride * 8;
    const int64_t fit = static_cast<int64_t>((kSlotLimit - kSlotOffset) / per_cluster);
    if (clusters > fit) clusters = fit;
    if (clusters < 1) return hipSuccess;
    ca.clusters = static_cast<int32_t>(clusters);
    ca.max_spins = g_max_spins.load(std::memory_order_relaxed);

    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    ClusterChain &chain = cluster_chain();
    std::lock_guard<std::mutex> guard(chain.lock);
    if (!chain.have[dev]) {
        err = hipEventCreateWithFlags(&chain.done[dev], hipEventDisableTiming);
        if (err != hipSuccess) return err;
        chain.have[dev] = true;
        chain.recorded[dev] = false;
    }
    if (chain.recorded[dev]) {
        err = hipStreamWaitEvent(stream, chain.done[dev], 0);
        if (err != hipSuccess) return err;
    }

    // status, counters and every slot tag start from zero on every call (a fill kernel, not a
    // memset node): a tag left by an earlier call must never look like this call's
    const int words = static_cast<int>(kClusterScratchBytes / 4);
    hipLaunchKernelGGL(zero_words_kernel, dim3((words + 255) / 256), dim3(256), 0, stream,
                       ca.status, words);
    err = hipGetLastError();
    if (err != hipSuccess) return err;

    hipLaunchKernelGGL((row_cluster_kernel<DTYPE, REV>),
                       dim3(static_cast<unsigned>(clusters * ca.members)), dim3(kThreads),
                       lds_bytes, stream, ca);
    err = hipGetLastError();
    if (err != hipSuccess) return err;
    err = hipEventRecord(chain.done[dev], stream);
    if (err != hipSuccess) return err;
    chain.recorded[dev] = true;
    *launched = true;
    return hipSuccess;
}

}  // namespace

// One-time set-up of the current device for callers that must not create anything later:
// the event that chains cluster launches.
hipError_t prepare_cluster_chain() {
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    ClusterChain &chain = cluster_chain();
    std::lock_guard<std::mutex> guard(chain.lock);
    if (!chain.have[dev]) {
        err = hipEventCreateWithFlags(&chain.done[dev], hipEventDisableTiming);
        if (err != hipSuccess) return err;
        chain.have[dev] = true;
        chain.recorded[dev] = false;
    }
    return hipSuccess;
}

// Destroys the chaining events of every device.  Work already enqueued keeps its ordering (a
// stream that was told to wait for an event keeps waiting for what was recorded); the caller
// makes sure that no other thread is inside a scoring call.
hipError_t release_cluster_chain() {
    ClusterChain &chain = cluster_chain();
    std::lock_guard<std::mutex> guard(chain.lock);
    hipError_t first = hipSuccess;
    for (int dev = 0; dev < 64; ++dev) {
        if (!chain.have[dev]) continue;
        const hipError_t err = hipEventDestroy(chain.done[dev]);
        if (err != hipSuccess && first == hipSuccess) first = err;
        chain.have[dev] = false;
        chain.recorded[dev] = false;
    }
    return first;
}

void set_cluster_spin_limit(uint32_t spins) {
    g_max_spins.store(spins == 0 ? kDefaultMaxSpins : spins, std::memory_order_relaxed);
}

// Launches the cluster kernel if the device and the sizes allow it; *launched says whether it
// did (otherwise the caller uses the one-workgroup-per-row kernel).
hipError_t launch_row_cluster(const RowArgs &args, int64_t rows, int32_t dtype, void *scratch,
                              hipStream_t stream, bool *launched) {
    *launched = false;
    if (rows == 0) return hipSuccess;
    // The event that chains cluster launches must not be recorded into a graph (a replay on
    // another stream would escape the chain): while the stream is being captured the caller
    // gets the one-workgroup-per-row kernel (second pass from memory).
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &capture) != hipSuccess) {
        (void)hipGetLastError();        // e.g. the null stream while another stream captures
        capture = hipStreamCaptureStatusNone;
    }
    if (capture != hipStreamCaptureStatusNone) return hipSuccess;
    const int cus = compute_units();
    if (cus < 1) return hipSuccess;

    const int vec = dtype == PPOW_BF16 ? 8 : 4;
    const int64_t max_chunks = args.V / vec;                  // per row side, when head = 0
    const int64_t reg_chunks = static_cast<int64_t>(kRegChunks) * kThreads;   // per row side
    const int64_t lds_chunks = PPOW_CLUSTER_LDS_BYTES / 32;   // two sides, 16 bytes a chunk
    const int64_t cap_chunks = reg_chunks + lds_chunks;
    int64_t members = (max_chunks + cap_chunks - 1) / cap_chunks;
    if (members < 1) members = 1;
    if (members > kMaxMembers) return hipSuccess;             // row too long for one wavefront of slots
    const int64_t per = ((max_chunks + members - 1) / members + 7) & ~int64_t{7};   // as the kernel
    const int64_t in_lds = per > reg_chunks ? per - reg_chunks : 1;
    const int lds_bytes = static_cast<int>(in_lds * 32);

    ClusterArgs ca;
    ca.row = args;
    ca.rows = rows;
    ca.members = static_cast<int32_t>(members);
    ca.stride = static_cast<int32_t>((members + 7) & ~static_cast<int64_t>(7));
    ca.clusters = 0;
    ca.slice_chunks = static_cast<int32_t>(in_lds);
    ca.max_spins = kDefaultMaxSpins;
    char *base = static_cast<char *>(scratch);
    ca.status = reinterpret_cast<uint32_t *>(base);
    ca.slots = reinterpret_cast<uint64_t *>(base + kSlotOffset);

    if (dtype == PPOW_BF16) {
        if (args.want_policy_terms) return launch_variant<PPOW_BF16, true>(ca, lds_bytes, cus, stream, launched);
        return launch_variant<PPOW_BF16, false>(ca, lds_bytes, cus, stream, launched);
    }
    if (args.want_policy_terms) return launch_variant<PPOW_F32, true>(ca, lds_bytes, cus, stream, launched);
    return launch_variant<PPOW_F32, false>(ca, lds_bytes, cus, stream, launched);
}

}  // namespace ppow
