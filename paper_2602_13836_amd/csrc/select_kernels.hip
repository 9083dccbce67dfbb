// Candidate-vocabulary selection (Section 3.3): approximate logits s = W_vocab h' (Step 1) and
// k_t = top-k(s_t, k) (Step 2), exact, ids in ascending order, ties to the smaller id.
//
// Three launches after the down-projection (with more than eight hidden rows: a histogram pass over
// scores that a matrix-core kernel produced, then four).  Every step that needs a result of the whole
// row sits behind a kernel boundary: on this multi-die part a kernel boundary is the cheapest
// device-wide synchronisation (a device-scope release fence writes back a whole L2, and atomics on one
// address serialise at ~50 ns each), so there is no "last block" hand-over and no contended counter.
// Up to eight hidden rows the kernels are shaped for latency (few launches, redundant work per block);
// beyond that for throughput (small workgroups, 16-byte loads, the row-wide results computed once).
//   scores_hist   streams W_vocab once.  A selector row is short (d' = d/16 .. d/8: a few hundred
//                 bytes), so a wavefront is split into groups of G lanes, one row per group, and
//                 every load instruction still covers 1 KiB of consecutive memory.  Each score is
//                 stored and counted into a 4096-bin histogram of the top 12 bits of its
//                 order-preserving key: in LDS per block, then merged into one of several global
//                 replicas of the histogram (replicas keep same-address atomics apart).
//   collect       every block first sums the replicas and finds the bin B that holds the k-th
//                 largest score (redundantly: cheaper than one more launch -- with more than eight
//                 hidden rows a launch of one block per row does it once instead); it then counts
//                 its scores in bins above B (all selected) and appends (key, id) of its scores in
//                 bin B to the row's candidate list.
//   resolve       MSB-first radix selection among the candidates over the remaining 20 key bits
//                 and, only if scores tie exactly, the inverted id bits (digits of 11, 9, 11, 11 and
//                 10 bits; as soon as at most 64 candidates share the decided prefix, one wavefront
//                 ranks them by counting instead), which yields a 64-bit threshold T with
//                 selected(v) <=> (key(v) << 32 | ~v) >= T ; it also turns the per-block counts into
//                 output offsets (all of them, or just the one block's that asks).  With up to 8 hidden rows every emit block
//                 does this itself (redundant work, one launch less); with more rows it is one
//                 block per row in a launch of its own.
//   emit          every block re-evaluates the predicate on its entries in id order and writes the
//                 selected ids (and scores) at its offset: the output is ascending by construction.
#include "sv_device.h"
#include "sv_launch.h"

#include <math.h>

#include <type_traits>

namespace sv {

namespace {

typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kHistBits = 12;
constexpr int kHistBins = 1 << kHistBits;                // 4096
constexpr int kKeyLowBits = 32 - kHistBits;              // 20
constexpr int kScoreThreads = 1024;                      // scores_hist workgroup
constexpr int kScoreWaves = kScoreThreads / 64;
constexpr int kSelThreads = 1024;                        // collect / resolve / emit workgroup
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kMaxBlocksPerRow = 1024;                   // vocabulary blocks per row in collect / emit
constexpr int kEpt = 4;                                  // entries per thread in collect / emit
constexpr int kCandPerThread = 8;                        // candidates a resolve thread keeps in registers
constexpr int kRbThreads = 256;                         // workgroup of the bracketed selection's per-row kernels
constexpr int kRbWaves = kRbThreads / 64;
constexpr int kFewRows = 8;                              // up to here the latency-shaped tail (measured: 5 us
                                                         // faster at 5 to 8 rows, slower from 10)

// per-row state words (zeroed before every call together with the histogram replicas)
enum { ST_NCAND = 0, ST_T_HI = 1, ST_T_LO = 2, ST_WORDS = 4 };

struct SelLayout {
    int64_t V;
    int64_t chunk;      // vocabulary entries per collect / emit block
    int64_t nb;         // blocks per row (<= kMaxBlocksPerRow)
    int replicas;       // copies of the global histogram per row
    size_t zero_words;  // per row: state + histogram replicas
    size_t rest_words;  // per row: candidate list, per-block counts and offsets, bin info (even)
};
__host__ __device__ inline SelLayout sel_layout(int64_t V, int64_t rows) {
    SelLayout L;
    L.V = V;
    L.chunk = (int64_t)kEpt * kSelThreads;
    L.nb = (V + L.chunk - 1) / L.chunk;
    L.replicas = rows <= 2 ? 8 : (rows <= 16 ? 2 : 1);     // at most kMaxReplicas
    L.zero_words = ST_WORDS + (size_t)L.replicas * kHistBins;
    L.rest_words = 2 * (size_t)V + 2 * (size_t)L.nb + 2;
    return L;
}
struct SelPtrs {
    uint32_t* state;    // [ST_WORDS]
    uint32_t* hist;     // [replicas][kHistBins]
    uint64_t* cand;     // [V]   (key << 32 | ~id) of the entries in bin B
    uint32_t* sure;     // [nb]  entries in bins above B per block
    uint32_t* offset;   // [nb]  first output slot of each block
    uint32_t* binfo;    // [2]   B, entries above B (every collect block computes the same values)
};
// the zeroed words of all rows come first, so that one contiguous range is cleared
__host__ __device__ inline size_t sel_zero_total(int64_t rows, const SelLayout& L) {
    return ((size_t)rows * L.zero_words + 1) & ~(size_t)1;      // keeps the 64-bit lists 8-byte aligned
}
__host__ __device__ inline SelPtrs sel_ptrs(uint32_t* base, int64_t rows, int64_t r, const SelLayout& L) {
    SelPtrs p;
    p.state = base + (size_t)r * L.zero_words;
    p.hist = p.state + ST_WORDS;
    uint32_t* rest = base + sel_zero_total(rows, L) + (size_t)r * L.rest_words;
    p.cand = reinterpret_cast<uint64_t*>(rest);
    p.sure = rest + 2 * (size_t)L.V;
    p.offset = p.sure + L.nb;
    p.binfo = p.offset + L.nb;
    return p;
}

// c[0..4) += bins [4 * tid, 4 * tid + 4) of every replica of the histogram.  All loads leave at once: the
// replica count varies at run time, so indices past it repeat the last replica and are not added.
constexpr int kMaxReplicas = 8;
__device__ __forceinline__ void sum_replicas(const uint32_t* hist, int replicas, int tid, uint32_t (&c)[4]) {
    u32x4 q[kMaxReplicas];
#pragma unroll
    for (int rep = 0; rep < kMaxReplicas; ++rep)
        q[rep] = reinterpret_cast<const u32x4*>(hist + (size_t)(rep < replicas ? rep : replicas - 1) * kHistBins)[tid];
#pragma unroll
    for (int rep = 0; rep < kMaxReplicas; ++rep)
#pragma unroll
        for (int i = 0; i < 4; ++i) c[i] += rep < replicas ? q[rep][i] : 0u;
}

// Histogram held as PER consecutive bins per thread (thread t owns bins [t*PER, t*PER+PER)):
// finds the bin with  above(bin) < remain <= above(bin) + count(bin)  (above = entries in higher
// bins) and reports (bin, above, count) in s_out to every thread.  Exactly one bin qualifies
// whenever the histogram holds at least `remain` entries.
template <int PER>
__device__ __forceinline__ void locate_bin(const uint32_t (&c)[PER], uint32_t remain, uint32_t* s_w,
                                           uint32_t* s_out) {
    uint32_t local = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) local += c[i];
    uint32_t above = block_suffix_exclusive<kSelWaves>(local, s_w);
#pragma unroll
    for (int i = PER - 1; i >= 0; --i) {
        if (above < remain && remain <= above + c[i]) {
            s_out[0] = (uint32_t)(threadIdx.x * PER + i);
            s_out[1] = above;
            s_out[2] = c[i];
        }
        above += c[i];
    }
    __syncthreads();
}

// locate_bin for a workgroup of WAVES wavefronts (see locate_bin)
template <int PER, int WAVES>
__device__ __forceinline__ void locate_bin_w(const uint32_t (&c)[PER], uint32_t remain, uint32_t* s_w, uint32_t* s_out) {
    uint32_t local = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) local += c[i];
    uint32_t above = block_suffix_exclusive<WAVES>(local, s_w);
#pragma unroll
    for (int i = PER - 1; i >= 0; --i) {
        if (above < remain && remain <= above + c[i]) {
            s_out[0] = (uint32_t)(threadIdx.x * PER + i);
            s_out[1] = above;
            s_out[2] = c[i];
        }
        above += c[i];
    }
    __syncthreads();
}

// ------------------------------------------------------------------------------------------
// scores (+ histogram)
// ------------------------------------------------------------------------------------------
// FULL: a selector row is exactly G units, so the UNR loads of a wavefront sit at compile-time offsets
// from one base address.  Loads are branch-free and all leave before the first product: a window that
// would run past the last row is moved back to end at it (rows it re-computes are not stored or counted
// again); vocabularies shorter than one window clamp row by row instead.
// (leading plain arguments are preloaded into scalar registers with the wavefront; the struct is not)
template <int DT, int G, int UNR, bool FULL>
__global__ __launch_bounds__(kScoreThreads) void scores_hist_kernel(const char* __restrict__ hp_base,
                                                                    const char* __restrict__ wv_base, const int64_t V,
                                                                    float* __restrict__ s_base, const int chunks,
                                                                    const ScoresArgs a, uint32_t* scratch) {
    constexpr int RPW = 64 / G;                       // vocabulary rows per wave-wide load
    constexpr int64_t kWindow = (int64_t)RPW * UNR;   // rows per wavefront and iteration
    __shared__ uint32_t lh[kHistBins];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane % G;                           // 16-byte unit within the row
    const int sub = lane / G;                         // which of the RPW rows
    const int64_t r = blockIdx.y;
    const int C = FULL ? G : chunks;
    const int64_t row_bytes = (int64_t)C * 16;

    for (int b = tid; b < kHistBins; b += kScoreThreads) lh[b] = 0u;
    const int gc = (FULL || g < C) ? g : C - 1;
    const u32x4 xraw = reinterpret_cast<const u32x4*>(hp_base + r * row_bytes)[gc];
    const u32x4 xreg = (FULL || g < C) ? xraw : zero16();   // units past the end of a row meet zeros
    float* s = s_base + r * V;
    __syncthreads();

    const int64_t step = (int64_t)gridDim.x * kScoreWaves * kWindow;
    // two copies of the loop (a branch around the loads inside one loop makes the compiler wait for
    // everything in flight, the previous iteration's stores included)
    auto run = [&](auto tiny_tag) {
        constexpr bool TINY = decltype(tiny_tag)::value;
        for (int64_t base = ((int64_t)blockIdx.x * kScoreWaves + wave) * kWindow; base < V; base += step) {
            const int64_t b0 = (TINY || base + kWindow <= V) ? base : V - kWindow;
            u32x4 w[UNR];
            if constexpr (!TINY) {
                const char* p = wv_base + (b0 + sub) * row_bytes + (int64_t)gc * 16;
#pragma unroll
                for (int u = 0; u < UNR; ++u)
                    w[u] = load16<false>(reinterpret_cast<const u32x4*>(p + (int64_t)u * RPW * row_bytes));
            } else {
#pragma unroll
                for (int u = 0; u < UNR; ++u) {
                    const int64_t v = b0 + (int64_t)u * RPW + sub;
                    w[u] = load16<false>(reinterpret_cast<const u32x4*>(wv_base + (v < V ? v : V - 1) * row_bytes) + gc);
                }
            }
            __builtin_amdgcn_sched_barrier(0);        // every request leaves before anything waits
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                float acc = dot16<DT>(w[u], xreg, 0.0f);
                // sum over the G lanes of the group (G is a power of two, groups are lane-aligned)
                if constexpr (G >= 2) acc += dpp_f32<DPP_QUAD_1032>(acc);
                if constexpr (G >= 4) acc += dpp_f32<DPP_QUAD_2301>(acc);
                if constexpr (G >= 8) acc += dpp_f32<DPP_ROW_HALF_MIRROR>(acc);
                if constexpr (G >= 16) acc += dpp_f32<DPP_ROW_MIRROR>(acc);
                if constexpr (G >= 32) acc += __shfl_xor(acc, 16);
                if constexpr (G >= 64) acc += __shfl_xor(acc, 32);
                const int64_t v = b0 + (int64_t)u * RPW + sub;
                if (g == 0 && v >= base && v < V) {
                    s[v] = acc;
                    atomicAdd(&lh[f32_to_ord(acc) >> kKeyLowBits], 1u);
                }
            }
        }
    };
    if (V < kWindow) run(std::true_type{});
    else run(std::false_type{});
    __syncthreads();

    const SelLayout L = sel_layout(V, a.rows);
    const SelPtrs p = sel_ptrs(scratch, a.rows, r, L);
    uint32_t* hist = p.hist + (size_t)(blockIdx.x % L.replicas) * kHistBins;
    for (int b = tid; b < kHistBins; b += kScoreThreads) {
        const uint32_t c = lh[b];
        if (c) atomicAdd(&hist[b], c);
    }
}

// histogram only (scores produced by another kernel)
__global__ __launch_bounds__(kScoreThreads) void hist_kernel(const float* s_all, int64_t V, uint32_t* scratch,
                                                             int rows) {
    __shared__ uint32_t lh[kHistBins];
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.y;
    const float* s = s_all + r * V;
    for (int b = tid; b < kHistBins; b += kScoreThreads) lh[b] = 0u;
    __syncthreads();
    // 16-byte loads, four in flight per thread; the unaligned head and the tail go one by one
    const int64_t head = min<int64_t>(V, (int64_t)((16u - (reinterpret_cast<uintptr_t>(s) & 15u)) & 15u) / 4);
    const int64_t nvec = (V - head) / 4;
    const f32x4_t* sv4 = reinterpret_cast<const f32x4_t*>(s + head);
    const int64_t stride = (int64_t)gridDim.x * kScoreThreads;
    constexpr int UNR = 4;
    for (int64_t q0 = (int64_t)blockIdx.x * kScoreThreads + tid; q0 < nvec; q0 += stride * UNR) {
        f32x4_t v[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int64_t q = q0 + u * stride;
            v[u] = q < nvec ? sv4[q] : f32x4_t{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u)
            if (q0 + u * stride < nvec) {
#pragma unroll
                for (int e = 0; e < 4; ++e) atomicAdd(&lh[f32_to_ord(v[u][e]) >> kKeyLowBits], 1u);
            }
    }
    if (blockIdx.x == 0) {
        const int64_t rest = V - head - nvec * 4;        // < 4
        if (tid < head) atomicAdd(&lh[f32_to_ord(s[tid]) >> kKeyLowBits], 1u);
        else if (tid - head < rest) atomicAdd(&lh[f32_to_ord(s[head + nvec * 4 + (tid - head)]) >> kKeyLowBits], 1u);
    }
    __syncthreads();
    const SelLayout L = sel_layout(V, rows);
    const SelPtrs p = sel_ptrs(scratch, rows, r, L);
    uint32_t* hist = p.hist + (size_t)(blockIdx.x % L.replicas) * kHistBins;
    for (int b = tid; b < kHistBins; b += kScoreThreads) {
        const uint32_t c = lh[b];
        if (c) atomicAdd(&hist[b], c);
    }
}

template <int DT, int G>
hipError_t launch_scores_g(const ScoresArgs& a, uint32_t* scratch, int cus, hipStream_t stream) {
    constexpr int UNR = 8;
    const int64_t per_block = (int64_t)(64 / G) * UNR * kScoreWaves;
    int64_t bx = (a.V + per_block - 1) / per_block;
    int64_t cap = ((int64_t)cus + a.rows - 1) / a.rows;         // one long-lived block per CU
    if (cap < 1) cap = 1;
    if (bx > cap) bx = cap;
    if (a.chunks == G)
        hipLaunchKernelGGL((scores_hist_kernel<DT, G, UNR, true>), dim3((unsigned)bx, (unsigned)a.rows),
                           dim3(kScoreThreads), 0, stream, a.hp, a.Wv, a.V, a.s, a.chunks, a, scratch);
    else
        hipLaunchKernelGGL((scores_hist_kernel<DT, G, UNR, false>), dim3((unsigned)bx, (unsigned)a.rows),
                           dim3(kScoreThreads), 0, stream, a.hp, a.Wv, a.V, a.s, a.chunks, a, scratch);
    return hipGetLastError();
}

template <int DT>
hipError_t launch_scores_dt(const ScoresArgs& a, uint32_t* scratch, int cus, hipStream_t stream) {
    if (a.chunks <= 8) return launch_scores_g<DT, 8>(a, scratch, cus, stream);
    if (a.chunks <= 16) return launch_scores_g<DT, 16>(a, scratch, cus, stream);
    if (a.chunks <= 32) return launch_scores_g<DT, 32>(a, scratch, cus, stream);
    return launch_scores_g<DT, 64>(a, scratch, cus, stream);
}

// ------------------------------------------------------------------------------------------
// collect
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t key64(uint32_t key, uint32_t v) {
    return ((uint64_t)key << 32) | (uint32_t)(~v);      // larger score first, then smaller id
}

// the bin B of the k-th largest score of every row, once per row (many hidden rows: cheaper than having
// each of the row's collect blocks work it out again)
__global__ __launch_bounds__(kSelThreads) void locate_kernel(int64_t V, int64_t k, uint32_t* scratch, int rows) {
    __shared__ uint32_t s_w[kSelWaves];
    __shared__ uint32_t s_out[4];
    const int tid = threadIdx.x;
    const SelLayout L = sel_layout(V, rows);
    const SelPtrs p = sel_ptrs(scratch, rows, blockIdx.x, L);
    constexpr int PER = kHistBins / kSelThreads;
    uint32_t c[PER] = {0u, 0u, 0u, 0u};
    sum_replicas(p.hist, L.replicas, tid, c);
    locate_bin<PER>(c, (uint32_t)k, s_w, s_out);
    if (tid == 0) {
        p.binfo[0] = s_out[0];
        p.binfo[1] = s_out[1];
    }
}

// few hidden rows: every block finds the row's bin B itself (one launch less on the critical path)
__global__ __launch_bounds__(kSelThreads) void collect_kernel(const float* s_all, int64_t V, int64_t k,
                                                              uint32_t* scratch, int rows) {
    __shared__ uint64_t s_list[kSelThreads * kEpt];    // this block's bin-B entries
    __shared__ uint32_t s_w[kSelWaves];
    __shared__ uint32_t s_out[4];
    __shared__ uint32_t s_n, s_gbase;
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.y;
    const SelLayout L = sel_layout(V, rows);
    const SelPtrs p = sel_ptrs(scratch, rows, r, L);
    const float* s = s_all + r * V;

    // this block's scores first: their latency overlaps the histogram reduction below
    const int64_t base = (int64_t)blockIdx.x * L.chunk;
    uint32_t key[kEpt];
#pragma unroll
    for (int i = 0; i < kEpt; ++i) {
        const int64_t v = base + (int64_t)i * kSelThreads + tid;
        key[i] = (v < V) ? f32_to_ord(s[v]) : 0u;    // 0: below every finite score
    }

    // the bin B of the k-th largest score, from the sum of the histogram replicas
    constexpr int PER = kHistBins / kSelThreads;          // 4 consecutive bins per thread
    uint32_t c[PER] = {0u, 0u, 0u, 0u};
    sum_replicas(p.hist, L.replicas, tid, c);
    if (tid == 0) s_n = 0u;
    locate_bin<PER>(c, (uint32_t)k, s_w, s_out);
    const uint32_t B = s_out[0];
    if (blockIdx.x == 0 && tid == 0) {
        p.binfo[0] = B;
        p.binfo[1] = s_out[1];
    }

    uint32_t sure = 0u;
#pragma unroll
    for (int i = 0; i < kEpt; ++i) {
        const int64_t v = base + (int64_t)i * kSelThreads + tid;
        if (v < V) {
            const uint32_t bin = key[i] >> kKeyLowBits;
            sure += bin > B;
            if (bin == B) s_list[atomicAdd(&s_n, 1u)] = key64(key[i], (uint32_t)v);
        }
    }
    sure = wave_sum_u32(sure);
    __syncthreads();                                      // s_w free again, s_list complete
    if ((tid & 63) == 0) s_w[tid >> 6] = sure;
    __syncthreads();
    const uint32_t n_local = s_n;
    if (tid == 0) {
        uint32_t tot = 0u;
        for (int w = 0; w < kSelWaves; ++w) tot += s_w[w];
        p.sure[blockIdx.x] = tot;
        s_gbase = n_local ? atomicAdd(&p.state[ST_NCAND], n_local) : 0u;
    }
    __syncthreads();
    const uint32_t gbase = s_gbase;
    for (uint32_t i = tid; i < n_local; i += kSelThreads) p.cand[gbase + i] = s_list[i];
}

// Many hidden rows: thousands of vocabulary blocks, each a short chain of dependent memory round
// trips (scores, then one atomic to reserve space in the candidate list).  Small workgroups with
// many entries per thread keep eight such chains in flight per CU, and B comes from locate_kernel.
constexpr int kRowThreads = 256;
constexpr int kRowWaves = kRowThreads / 64;
constexpr int kRowEpt = kSelThreads * kEpt / kRowThreads;     // 16: the same vocabulary block as above
static_assert(kRowThreads * kRowEpt == kSelThreads * kEpt, "both forms must cut the vocabulary alike");
static_assert(kRowThreads * kRowEpt < 65536, "two 16-bit counts are packed into one word");

__global__ __launch_bounds__(kRowThreads) void collect_rows_kernel(const float* s_all, int64_t V,
                                                                   uint32_t* scratch, int rows) {
    __shared__ uint32_t s_w[kRowWaves];
    __shared__ uint32_t s_gbase;
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.y;
    const SelLayout L = sel_layout(V, rows);
    const SelPtrs p = sel_ptrs(scratch, rows, r, L);
    const float* s = s_all + r * V;
    const int64_t base = (int64_t)blockIdx.x * L.chunk;
    const uint32_t B = p.binfo[0];
    const bool aligned = (reinterpret_cast<uintptr_t>(s + base) & 15u) == 0;
    // thread t owns the four-id groups t, t + 256, t + 512, t + 768 of the block (16-byte loads)
    auto id_of = [&](int i) { return base + 4 * ((int64_t)(i >> 2) * kRowThreads + tid) + (i & 3); };
    uint32_t key[kRowEpt];
#pragma unroll
    for (int j = 0; j < kRowEpt / 4; ++j) {
        const int64_t v0 = id_of(4 * j);
        if (aligned && v0 + 3 < V) {
            const f32x4_t q = *reinterpret_cast<const f32x4_t*>(s + v0);
#pragma unroll
            for (int e = 0; e < 4; ++e) key[4 * j + e] = f32_to_ord(q[e]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) key[4 * j + e] = (v0 + e < V) ? f32_to_ord(s[v0 + e]) : 0u;
        }
    }
    uint32_t packed = 0u;                                 // candidates (bin B) | sure entries (above B) << 16
#pragma unroll
    for (int i = 0; i < kRowEpt; ++i) {
        const uint32_t bin = key[i] >> kKeyLowBits;
        if (id_of(i) < V) packed += (bin == B ? 1u : 0u) + (bin > B ? 0x10000u : 0u);
    }
    const uint32_t pre = block_prefix_exclusive<kRowWaves>(packed, s_w);
    if (tid == 0) {
        uint32_t tot = 0u;
        for (int w = 0; w < kRowWaves; ++w) tot += s_w[w];
        p.sure[blockIdx.x] = tot >> 16;
        const uint32_t n_local = tot & 0xffffu;
        s_gbase = n_local ? atomicAdd(&p.state[ST_NCAND], n_local) : 0u;
    }
    __syncthreads();
    uint32_t off = s_gbase + (pre & 0xffffu);
#pragma unroll
    for (int i = 0; i < kRowEpt; ++i) {
        const int64_t v = id_of(i);
        if (v < V && (key[i] >> kKeyLowBits) == B) p.cand[off++] = key64(key[i], (uint32_t)v);
    }
}

// ------------------------------------------------------------------------------------------
// resolve: one block per row
// ------------------------------------------------------------------------------------------
struct ResolveSmem {
    uint32_t hist[2048];
    uint32_t w[kSelWaves];
    uint32_t out[4];
    uint32_t cnt[kMaxBlocksPerRow];
    uint64_t few[64];       // the last candidates, ranked by one wavefront
    uint32_t nfew;
};

// Row-wide part of the selection, run by one whole workgroup: the 64-bit threshold T and the first
// output slots of the vocabulary blocks -- ONE < 0: of block t in thread t (an exclusive scan over all
// blocks); ONE >= 0: of that block alone, in every thread (one sum instead of a histogram and a scan).
template <bool ONE_BLOCK>
__device__ __forceinline__ void resolve_row(const SelPtrs& p, const SelLayout& L, int64_t k, ResolveSmem& sm,
                                            uint64_t& T, uint32_t& offset_out, const uint32_t one_block = 0u) {
    const int tid = threadIdx.x;
    const uint32_t B = p.binfo[0];
    const uint32_t above = p.binfo[1];
    const uint32_t sure_of_block_tid = tid < (int)L.nb ? p.sure[tid] : 0u;   // requested with everything else
    if (tid == 0) sm.nfew = 0u;

    // candidates: 52-bit sub-keys (20 low key bits, then the inverted id); the top 12 bits are all B
    constexpr uint64_t kSubMask = (1ull << 52) - 1ull;
    uint64_t sk[kCandPerThread];
    // the first kSpec slots of every thread are requested before the count is known (a typical row has
    // one to two thousand candidates): one memory round trip instead of two on the usual path
    constexpr int kSpec = 2;
    uint64_t spec[kSpec];
#pragma unroll
    for (int i = 0; i < kSpec; ++i) {
        const int64_t j = (int64_t)i * kSelThreads + tid;
        spec[i] = p.cand[j < L.V ? j : L.V - 1];
    }
    const uint32_t n = p.state[ST_NCAND];
    const bool in_regs = n <= (uint32_t)(kSelThreads * kCandPerThread);
#pragma unroll
    for (int i = 0; i < kCandPerThread; ++i) {
        const uint32_t j = (uint32_t)i * kSelThreads + tid;
        if (i < kSpec) sk[i] = (in_regs && j < n) ? (spec[i] & kSubMask) : 0ull;
        else sk[i] = (in_regs && j < n) ? (p.cand[j] & kSubMask) : 0ull;
    }
    auto for_each_candidate = [&](auto&& f) {
        if (in_regs) {
#pragma unroll
            for (int i = 0; i < kCandPerThread; ++i)
                if ((uint32_t)i * kSelThreads + tid < n) f(sk[i]);
        } else {
            for (uint32_t j = tid; j < n; j += kSelThreads) f(p.cand[j] & kSubMask);
        }
    };

    uint32_t remain = (uint32_t)k - above;              // 1 <= remain <= n
    uint64_t prefix = 0ull;                             // decided high bits of the threshold sub-key
    int decided = 0;                                    // how many of the 52 bits are decided
    bool all_of_prefix = false;
    // digit widths from the MSB: the 20 key bits as 11 + 9, then the 32 id bits as 11 + 11 + 10
    const int widths[5] = {11, 9, 11, 11, 10};
    for (int pass = 0; pass < 5 && !all_of_prefix; ++pass) {
        const int w = widths[pass];
        const int shift = 52 - decided - w;
        sm.hist[tid] = 0u;
        sm.hist[tid + kSelThreads] = 0u;
        __syncthreads();
        for_each_candidate([&](uint64_t x) {
            if (decided == 0 || (x >> (52 - decided)) == (prefix >> (52 - decided)))
                atomicAdd(&sm.hist[(uint32_t)(x >> shift) & ((1u << w) - 1u)], 1u);
        });
        __syncthreads();
        const uint32_t c[2] = {sm.hist[tid * 2], sm.hist[tid * 2 + 1]};
        locate_bin<2>(c, remain, sm.w, sm.out);
        prefix |= (uint64_t)sm.out[0] << shift;
        remain -= sm.out[1];
        decided += w;
        const uint32_t left = sm.out[2];                // candidates that share the decided prefix
        all_of_prefix = (remain == left);               // every one of them is selected
        __syncthreads();
        if (!all_of_prefix && left <= 64u) {
            // A handful left (the usual case after the first digit): one wavefront ranks them by counting
            // instead of more digit passes.  Sub-keys are unique (they end in the id), so exactly one has
            // remain - 1 larger ones: that one is the threshold.
            for_each_candidate([&](uint64_t x) {
                if ((x >> (52 - decided)) == (prefix >> (52 - decided))) sm.few[atomicAdd(&sm.nfew, 1u)] = x;
            });
            __syncthreads();
            const int lane = tid & 63;
            const uint64_t mine = (uint32_t)lane < left ? sm.few[lane] : 0ull;
            uint32_t larger = 0u;
            for (uint32_t j = 0; j < left; ++j) larger += readlane_u64(mine, (int)j) > mine;
            const uint64_t pick = __builtin_amdgcn_ballot_w64((uint32_t)lane < left && larger == remain - 1u);
            prefix = readlane_u64(mine, pick ? __ffsll((long long)pick) - 1 : 0);
            break;
        }
    }
    // threshold: selected(v) <=> (key << 32 | ~v) >= T, T = (B << 20 | prefix.hi) << 32 | prefix.lo
    T = ((uint64_t)((B << kKeyLowBits) | (uint32_t)(prefix >> 32)) << 32) | (uint32_t)prefix;

    // output offsets: selected entries per block = sure + selected candidates
    const int nb = (int)L.nb;
    constexpr int kChunkShift = 12;
    static_assert((1 << kChunkShift) == kEpt * kSelThreads, "a vocabulary block is 4096 ids");
    if constexpr (ONE_BLOCK) {
        // everything in front of one block: its sure entries and the selected candidates of lower blocks
        uint32_t before = tid < (int)one_block ? sure_of_block_tid : 0u;
        for_each_candidate([&](uint64_t x) {
            before += (x >= prefix && ((uint32_t)(~(uint32_t)x) >> kChunkShift) < one_block) ? 1u : 0u;
        });
        before = wave_sum_u32(before);
        __syncthreads();                                  // sm.w may still be read by the last locate
        if ((tid & 63) == 0) sm.w[tid >> 6] = before;
        __syncthreads();
        uint32_t tot = 0u;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) tot += sm.w[w];
        offset_out = tot;
        return;
    }
    sm.cnt[tid] = 0u;
    __syncthreads();
    // Candidates of one vocabulary block sit next to each other in the list, so the lanes of a wavefront
    // mostly count into the same word: one atomic per distinct block and wavefront, not one per candidate.
    auto count_selected = [&](bool valid, uint64_t x) {
        const bool sel = valid && x >= prefix;
        const uint32_t blk = (uint32_t)(~(uint32_t)x) >> kChunkShift;
        uint64_t todo = __builtin_amdgcn_ballot_w64(sel);
        while (todo) {
            const uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)blk, __ffsll((long long)todo) - 1);
            const uint64_t same = __builtin_amdgcn_ballot_w64(sel && blk == b);
            if ((tid & 63) == __ffsll((long long)same) - 1) atomicAdd(&sm.cnt[b], (uint32_t)__popcll(same));
            todo &= ~same;
        }
    };
    if (in_regs) {
#pragma unroll
        for (int i = 0; i < kCandPerThread; ++i) {
            if ((uint32_t)i * kSelThreads >= n) break;             // uniform: no candidate in this round
            count_selected((uint32_t)i * kSelThreads + tid < n, sk[i]);
        }
    } else {
        for (uint32_t j0 = 0; j0 < n; j0 += kSelThreads) {
            const uint32_t j = j0 + tid;
            count_selected(j < n, j < n ? (p.cand[j] & kSubMask) : 0ull);
        }
    }
    __syncthreads();
    const uint32_t mine = tid < nb ? sm.cnt[tid] + sure_of_block_tid : 0u;
    offset_out = block_prefix_exclusive<kSelWaves>(mine, sm.w);
}

// one block per row (many hidden rows: the result is shared by the row's emit blocks through memory)
__global__ __launch_bounds__(kSelThreads) void resolve_kernel(int64_t V, int64_t k, uint32_t* scratch, int rows) {
    __shared__ ResolveSmem sm;
    const int tid = threadIdx.x;
    const SelLayout L = sel_layout(V, rows);
    const SelPtrs p = sel_ptrs(scratch, rows, blockIdx.x, L);
    uint64_t T;
    uint32_t off;
    resolve_row<false>(p, L, k, sm, T, off);
    if (tid == 0) {
        p.state[ST_T_HI] = (uint32_t)(T >> 32);
        p.state[ST_T_LO] = (uint32_t)T;
    }
    if (tid < (int)L.nb) p.offset[tid] = off;
}

// ------------------------------------------------------------------------------------------
// emit
// ------------------------------------------------------------------------------------------
// few hidden rows: every emit block resolves the row itself instead of reading the result of a separate
// one-block launch -- redundant work, one launch less on the critical path
__global__ __launch_bounds__(kSelThreads) void emit_kernel(const float* s_all, int64_t V, int64_t k,
                                                           uint32_t* scratch, int rows, int32_t* idx_out,
                                                           float* scores_out, float tau) {
    __shared__ uint32_t s_w[kSelWaves];
    __shared__ ResolveSmem sm;
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.y;
    const SelLayout L = sel_layout(V, rows);
    const SelPtrs p = sel_ptrs(scratch, rows, r, L);
    const float* s = s_all + r * V;

    // thread t owns kEpt consecutive ids, so (thread, i) order is ascending id order
    const int64_t v0 = (int64_t)blockIdx.x * L.chunk + (int64_t)tid * kEpt;
    float val[kEpt];
#pragma unroll
    for (int i = 0; i < kEpt; ++i) val[i] = (v0 + i < V) ? s[v0 + i] : 0.0f;
    uint64_t T;
    uint32_t block_off;
    resolve_row<true>(p, L, k, sm, T, block_off, blockIdx.x);

    uint32_t mask = 0u;
#pragma unroll
    for (int i = 0; i < kEpt; ++i)
        if (v0 + i < V && key64(f32_to_ord(val[i]), (uint32_t)(v0 + i)) >= T) mask |= 1u << i;
    const uint32_t mine = (uint32_t)__popc(mask);
    uint32_t pos = block_off + block_prefix_exclusive<kSelWaves>(mine, s_w);

    int32_t* out = idx_out + r * k;
#pragma unroll
    for (int i = 0; i < kEpt; ++i) {
        if (mask & (1u << i)) {
            if (pos < (uint32_t)k) {                      // always true for a consistent threshold
                const bool keep = val[i] >= tau;          // below the threshold: a padding slot
                out[pos] = keep ? (int32_t)(v0 + i) : -1;
                if (scores_out) scores_out[r * k + pos] = keep ? val[i] : -INFINITY;
            }
            ++pos;
        }
    }
}

// Many hidden rows (threshold and block offsets come from resolve_kernel): small workgroups as in
// collect_rows_kernel.  Thread t owns the four-id groups t, t + 256, t + 512, t + 768 of the
// vocabulary block (16-byte loads, consecutive lanes on consecutive groups), so ascending id order
// is (group round j, thread, element): one packed prefix sum per two rounds places every id.
__global__ __launch_bounds__(kRowThreads) void emit_rows_kernel(const float* s_all, int64_t V, int64_t k,
                                                                uint32_t* scratch, int rows, int32_t* idx_out,
                                                                float* scores_out, float tau) {
    constexpr int kRounds = kRowEpt / 4;                  // 4
    static_assert(kRounds == 4, "two packed scans cover four rounds");
    __shared__ uint32_t s_w[kRowWaves];
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.y;
    const SelLayout L = sel_layout(V, rows);
    const SelPtrs p = sel_ptrs(scratch, rows, r, L);
    const float* s = s_all + r * V;
    const int64_t base = (int64_t)blockIdx.x * L.chunk;
    const bool aligned = (reinterpret_cast<uintptr_t>(s + base) & 15u) == 0;

    float val[kRounds][4];
#pragma unroll
    for (int j = 0; j < kRounds; ++j) {
        const int64_t v0 = base + 4 * ((int64_t)j * kRowThreads + tid);
        if (aligned && v0 + 3 < V) {
            const f32x4_t q = *reinterpret_cast<const f32x4_t*>(s + v0);
#pragma unroll
            for (int e = 0; e < 4; ++e) val[j][e] = q[e];
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) val[j][e] = (v0 + e < V) ? s[v0 + e] : 0.0f;
        }
    }
    const uint64_t T = ((uint64_t)p.state[ST_T_HI] << 32) | p.state[ST_T_LO];
    const uint32_t block_off = p.offset[blockIdx.x];

    uint32_t mask[kRounds];
#pragma unroll
    for (int j = 0; j < kRounds; ++j) {
        const int64_t v0 = base + 4 * ((int64_t)j * kRowThreads + tid);
        mask[j] = 0u;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (v0 + e < V && key64(f32_to_ord(val[j][e]), (uint32_t)(v0 + e)) >= T) mask[j] |= 1u << e;
    }
    const uint32_t c01 = (uint32_t)__popc(mask[0]) | ((uint32_t)__popc(mask[1]) << 16);
    const uint32_t c23 = (uint32_t)__popc(mask[2]) | ((uint32_t)__popc(mask[3]) << 16);
    const uint32_t pre01 = block_prefix_exclusive<kRowWaves>(c01, s_w);
    uint32_t tot01 = 0u;
    for (int w = 0; w < kRowWaves; ++w) tot01 += s_w[w];
    const uint32_t pre23 = block_prefix_exclusive<kRowWaves>(c23, s_w);      // its first barrier: all have read s_w
    uint32_t tot23 = 0u;
    for (int w = 0; w < kRowWaves; ++w) tot23 += s_w[w];
    uint32_t pos[kRounds];
    pos[0] = block_off + (pre01 & 0xffffu);
    pos[1] = block_off + (tot01 & 0xffffu) + (pre01 >> 16);
    pos[2] = block_off + (tot01 & 0xffffu) + (tot01 >> 16) + (pre23 & 0xffffu);
    pos[3] = block_off + (tot01 & 0xffffu) + (tot01 >> 16) + (tot23 & 0xffffu) + (pre23 >> 16);

    int32_t* out = idx_out + r * k;
#pragma unroll
    for (int j = 0; j < kRounds; ++j) {
        const int64_t v0 = base + 4 * ((int64_t)j * kRowThreads + tid);
        uint32_t q = pos[j];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (mask[j] & (1u << e)) {
                if (q < (uint32_t)k) {                    // always true for a consistent threshold
                    const bool keep = val[j][e] >= tau;   // below the threshold: a padding slot
                    out[q] = keep ? (int32_t)(v0 + e) : -1;
                    if (scores_out) scores_out[r * k + q] = keep ? val[j][e] : -INFINITY;
                }
                ++q;
            }
        }
    }
}


// ------------------------------------------------------------------------------------------
// Bracketed selection: a batch of hidden rows without the score matrix
// ------------------------------------------------------------------------------------------
// With hundreds of hidden rows the scores s [rows x V] are hundreds of megabytes: writing them and reading
// them back for the histogram, the collect and the emit passes costs several times the product that makes
// them.  Here they never reach memory:
//   sample    the scores of kSample evenly spaced tokens (a small matrix product);
//   bracket   per row, from the sample's order statistics, two values hi > lo that enclose the k-th largest
//             score of the whole row except with negligible probability (ranks k/V * m -/+ 6 standard
//             deviations of the hypergeometric count, -/+ 8);
//   classify  the full product on the matrix cores, whose epilogue keeps only: one bit per (row, token)
//             "score > hi" (all of these are selected), and (key, id) of the few per cent of scores inside
//             [lo, hi] (tile_mfma_kernels.hip);
//   resolve   per row, with the row's bits in LDS: popcount of the bits = n_above; the (k - n_above)-th largest
//             candidate by exact radix selection on (key, ~id) is the threshold; the selected candidates'
//             bits are set; the ids of the set bits are written in ascending order.  A row whose bracket
//             missed (k - n_above outside [0, candidates]) is only flagged;
//   redo      a flagged row is redone by ONE workgroup that recomputes the row's scores itself in three
//             passes (histogram, collect, emit): slow, exact, and only ever run for the one-in-a-billion row
//             (or for inputs built to defeat the sample); every other workgroup of the launch leaves at once.
// The result is exact with respect to the scores the classify pass computes: ties go to the smaller id.

struct BracketLayout {
    int64_t V;
    int rows;
    int tn;              // items per tile of the classify pass
    int64_t tiles;       // item tiles per row
    int64_t words;       // bit-mask words per row
    int64_t m;           // sample size
    int64_t nb;          // 4096-id vocabulary blocks (the redo path)
    // offsets in uint32 words from the scratch base (all multiples of 4: 16-byte aligned)
    size_t ids, samp, thr, flag, bits, cnt, sure, boff, state, first, cand, total;
};
__host__ __device__ inline size_t quad4(size_t n) { return (n + 3) & ~(size_t)3; }
__host__ __device__ inline BracketLayout bracket_layout(int64_t V, int rows, int tn, int64_t m) {
    BracketLayout L;
    L.V = V;
    L.rows = rows;
    L.tn = tn;
    L.tiles = (V + tn - 1) / tn;
    L.words = L.tiles * (tn / 32);
    L.m = m;
    L.nb = (V + (int64_t)kEpt * kSelThreads - 1) / ((int64_t)kEpt * kSelThreads);
    size_t o = 0;
    L.ids = o;    o += quad4((size_t)m);
    L.samp = o;   o += quad4((size_t)rows * m);
    L.thr = o;    o += quad4((size_t)rows * 2);
    L.flag = o;   o += quad4((size_t)rows);
    L.bits = o;   o += quad4((size_t)rows * L.words);
    L.cnt = o;    o += quad4((size_t)rows * L.tiles);
    L.sure = o;   o += quad4((size_t)rows * L.nb);
    L.boff = o;   o += quad4((size_t)rows * L.nb);
    L.state = o;  o += (size_t)rows * 8;
    L.first = o;  o += (size_t)rows * L.tiles * kCandFirst * 2;
    L.cand = o;   o += (size_t)rows * L.tiles * tn * 2;
    L.total = o;
    return L;
}

// thr[r] = {hi, lo} from the row's m sample scores: hi = the largest value of the 2^-23-wide key interval
// that holds the sample's rank_hi-th largest score (+inf if rank_hi < 1), lo = the smallest value of the
// interval that holds the rank_lo-th largest (-inf if rank_lo > m)
__global__ __launch_bounds__(kRbThreads) void bracket_kernel(const float* samp, int64_t m, int64_t rank_hi,
                                                             int64_t rank_lo, float* thr) {
    __shared__ uint32_t s_h1[kHistBins];
    __shared__ uint32_t s_h2[2][2048];
    __shared__ uint32_t s_w[kRbWaves];
    __shared__ uint32_t s_out[4];
    const int tid = threadIdx.x;
    const float* s = samp + (int64_t)blockIdx.x * m;
    // the first 32 sample scores of every thread stay in registers for both passes (all of them at the usual
    // sample size); all loads leave at once, entries past the end repeat the last one and are not counted
    constexpr int kHeld = 32;
    float held[kHeld];
#pragma unroll
    for (int u = 0; u < kHeld; ++u) {
        const int64_t j = (int64_t)u * kRbThreads + tid;
        held[u] = s[j < m ? j : m - 1];
    }
    for (int b = tid; b < kHistBins; b += kRbThreads) s_h1[b] = 0u;
    for (int b = tid; b < 2 * 2048; b += kRbThreads) (&s_h2[0][0])[b] = 0u;
    __syncthreads();
    auto for_each_key = [&](auto&& f) {
#pragma unroll
        for (int u = 0; u < kHeld; ++u)
            if ((int64_t)u * kRbThreads + tid < m) f(f32_to_ord(held[u]));
        for (int64_t j = (int64_t)kHeld * kRbThreads + tid; j < m; j += kRbThreads) f(f32_to_ord(s[j]));
    };
    for_each_key([&](uint32_t key) { atomicAdd(&s_h1[key >> kKeyLowBits], 1u); });
    __syncthreads();
    constexpr int PER = kHistBins / kRbThreads;
    uint32_t c[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) c[i] = s_h1[tid * PER + i];
    const bool has_hi = rank_hi >= 1, has_lo = rank_lo <= m;
    uint32_t bin_hi = 0u, rem_hi = 0u, bin_lo = 0u, rem_lo = 0u;
    if (has_hi) {                                             // uniform
        locate_bin_w<PER, kRbWaves>(c, (uint32_t)rank_hi, s_w, s_out);
        bin_hi = s_out[0];
        rem_hi = (uint32_t)rank_hi - s_out[1];
    }
    if (has_lo) {
        locate_bin_w<PER, kRbWaves>(c, (uint32_t)rank_lo, s_w, s_out);
        bin_lo = s_out[0];
        rem_lo = (uint32_t)rank_lo - s_out[1];
    }
    for_each_key([&](uint32_t key) {
        if (has_hi && (key >> kKeyLowBits) == bin_hi) atomicAdd(&s_h2[0][(key >> 9) & 2047u], 1u);
        if (has_lo && (key >> kKeyLowBits) == bin_lo) atomicAdd(&s_h2[1][(key >> 9) & 2047u], 1u);
    });
    __syncthreads();
    constexpr int PER2 = 2048 / kRbThreads;
    float hi = INFINITY, lo = -INFINITY;
    if (has_hi) {
        uint32_t c2[PER2];
#pragma unroll
        for (int i = 0; i < PER2; ++i) c2[i] = s_h2[0][tid * PER2 + i];
        locate_bin_w<PER2, kRbWaves>(c2, rem_hi, s_w, s_out);
        hi = ord_to_f32((bin_hi << kKeyLowBits) | (s_out[0] << 9) | 0x1FFu);
    }
    if (has_lo) {
        uint32_t c2[PER2];
#pragma unroll
        for (int i = 0; i < PER2; ++i) c2[i] = s_h2[1][tid * PER2 + i];
        locate_bin_w<PER2, kRbWaves>(c2, rem_lo, s_w, s_out);
        lo = ord_to_f32((bin_lo << kKeyLowBits) | (s_out[0] << 9));
    }
    if (tid == 0) {
        thr[2 * blockIdx.x] = hi;
        thr[2 * blockIdx.x + 1] = lo;
    }
}

// The redo of a row whose bracket missed, by one workgroup: the row's scores are recomputed three times
// (histogram of the key's top bits; count above the k-th score's bin and collect that bin; emit), each
// selector row by a group of 16 lanes.  Exact with respect to these scores; slow, and all but never run.
struct RedoSmem {
    uint32_t hist[kHistBins];
    float val[kEpt * kSelThreads];
    uint32_t w[kSelWaves];
    uint32_t out[4];
    uint32_t n;
    ResolveSmem resolve;
};
template <int DT>
__device__ __forceinline__ void redo_scores(const char* hp_row, const char* Wv, int chunks, int64_t V, int64_t base,
                                            float* val) {
    // 64 groups of 16 lanes; group q computes the scores of tokens base + q, base + q + 64, ...
    const int tid = threadIdx.x;
    const int g = tid & 15, q = tid >> 4;
    for (int i = q; i < kEpt * kSelThreads; i += kSelThreads / 16) {
        const int64_t v = base + i;
        float acc = 0.0f;
        if (v < V) {
            const u32x4* wp = reinterpret_cast<const u32x4*>(Wv + v * (int64_t)chunks * 16);
            const u32x4* xp = reinterpret_cast<const u32x4*>(hp_row);
            for (int c = g; c < chunks; c += 16) acc = dot16<DT>(wp[c], xp[c], acc);
        }
        acc = row16_sum(acc);
        if (g == 0) val[i] = acc;
    }
}
template <int DT>
__device__ __forceinline__ void redo_row(const char* hp_row, const char* Wv, int chunks, int64_t V, int64_t k,
                                         const SelPtrs& p, const SelLayout& SL, int32_t* out, RedoSmem& rs) {
    const int tid = threadIdx.x;
    const int64_t chunk = (int64_t)kEpt * kSelThreads;
    for (int b = tid; b < kHistBins; b += kSelThreads) rs.hist[b] = 0u;
    if (tid == 0) rs.n = 0u;
    __syncthreads();
    for (int64_t blk = 0; blk < SL.nb; ++blk) {
        redo_scores<DT>(hp_row, Wv, chunks, V, blk * chunk, rs.val);
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kEpt; ++i)
            if (blk * chunk + tid * kEpt + i < V) atomicAdd(&rs.hist[f32_to_ord(rs.val[tid * kEpt + i]) >> kKeyLowBits], 1u);
        __syncthreads();
    }
    constexpr int PER = kHistBins / kSelThreads;
    uint32_t c[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) c[i] = rs.hist[tid * PER + i];
    locate_bin<PER>(c, (uint32_t)k, rs.w, rs.out);
    const uint32_t B = rs.out[0], above = rs.out[1];
    for (int64_t blk = 0; blk < SL.nb; ++blk) {
        redo_scores<DT>(hp_row, Wv, chunks, V, blk * chunk, rs.val);
        __syncthreads();
        uint32_t sure = 0u;
#pragma unroll
        for (int i = 0; i < kEpt; ++i) {
            const int64_t v = blk * chunk + tid * kEpt + i;
            if (v < V) {
                const uint32_t key = f32_to_ord(rs.val[tid * kEpt + i]);
                sure += (key >> kKeyLowBits) > B;
                if ((key >> kKeyLowBits) == B) p.cand[atomicAdd(&rs.n, 1u)] = key64(key, (uint32_t)v);
            }
        }
        sure = wave_sum_u32(sure);
        if ((tid & 63) == 0) rs.w[tid >> 6] = sure;
        __syncthreads();
        if (tid == 0) {
            uint32_t tot = 0u;
            for (int w = 0; w < kSelWaves; ++w) tot += rs.w[w];
            p.sure[blk] = tot;
        }
        __syncthreads();
    }
    if (tid == 0) {
        p.state[ST_NCAND] = rs.n;
        p.binfo[0] = B;
        p.binfo[1] = above;
    }
    __threadfence_block();
    __syncthreads();
    uint64_t T;
    uint32_t off;
    resolve_row<false>(p, SL, k, rs.resolve, T, off);
    if (tid < (int)SL.nb) p.offset[tid] = off;
    __threadfence_block();
    __syncthreads();
    for (int64_t blk = 0; blk < SL.nb; ++blk) {
        redo_scores<DT>(hp_row, Wv, chunks, V, blk * chunk, rs.val);
        __syncthreads();
        const int64_t v0 = blk * chunk + (int64_t)tid * kEpt;
        uint32_t mask = 0u;
#pragma unroll
        for (int i = 0; i < kEpt; ++i)
            if (v0 + i < V && key64(f32_to_ord(rs.val[tid * kEpt + i]), (uint32_t)(v0 + i)) >= T) mask |= 1u << i;
        uint32_t pos = p.offset[blk] + block_prefix_exclusive<kSelWaves>((uint32_t)__popc(mask), rs.w);
#pragma unroll
        for (int i = 0; i < kEpt; ++i)
            if (mask & (1u << i)) {
                if (pos < (uint32_t)k) out[pos] = (int32_t)(v0 + i);
                ++pos;
            }
        __syncthreads();
    }
}

// One workgroup of 256 threads per row (small workgroups: several rows per CU overlap their memory round trips
// and barriers are cheap): see the overview above.  The row's bit mask lives in LDS from the first step to
// the last, so the selected candidates join it there and the ids are written from it.
// Dynamic LDS: [words] bit mask | [cand_cap] candidates (8 bytes each).
// A row with at most cand_cap candidates packs them into LDS once and every later walk reads that dense list
// (a few balanced iterations per thread); a row with more (ties by the thousand) walks the registers and the
// memory regions instead.
constexpr int kRbTiles = 4;                              // item tiles per thread whose candidates are held in registers
constexpr int kRbSpec = kCandFirst;                      // ... candidates per such tile: the compact array (mean 8, 99th
                                                         // percentile 16 at the usual shapes); the rest are re-read
constexpr int kRbBins = 2048;
constexpr int kRbBitBatch = 24;                          // words of the bit mask per thread requested at once
// dynamic LDS of a resolve workgroup: with its 9 KB of static LDS two of them share a CU's 160 KB (a launch
// of 512 rows is then one round of workgroups on 256 CUs)
constexpr size_t kResolveLdsBytes = 69 * 1024;
struct ResolveEmitSmem {
    uint32_t hist[kRbBins];
    uint32_t w[kRbWaves];
    uint32_t out[4];
    uint64_t few[64];
    uint32_t nfew;
    uint32_t tot[kRbWaves];
};

__global__ __launch_bounds__(kRbThreads) void resolve_emit_kernel(int64_t V, int rows, int tn, int64_t m, int64_t k,
                                                                  uint32_t* scratch, int32_t* idx_out,
                                                                  uint32_t cand_cap) {
    extern __shared__ __attribute__((aligned(16))) uint32_t s_bits[];         // [words], then the candidate list
    __shared__ ResolveEmitSmem sm;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int64_t r = blockIdx.x;
    const BracketLayout L = bracket_layout(V, rows, tn, m);
    uint64_t* s_cand = reinterpret_cast<uint64_t*>(s_bits + L.words);         // words is a multiple of 4
    const uint32_t* bits = scratch + L.bits + (size_t)r * L.words;
    const uint32_t* cnt = scratch + L.cnt + (size_t)r * L.tiles;
    const uint64_t* cand = reinterpret_cast<const uint64_t*>(scratch + L.cand) + (size_t)r * L.tiles * tn;
    const uint64_t* first = reinterpret_cast<const uint64_t*>(scratch + L.first) + (size_t)r * L.tiles * kCandFirst;
    // everything independent is requested up front, in the order of use: the bracket, the candidate counts of
    // this thread's tiles, the first words of the bit mask, the first candidates of each tile (before their
    // count is known)
    const float hi = reinterpret_cast<const float*>(scratch + L.thr)[2 * r];
    const float lo = reinterpret_cast<const float*>(scratch + L.thr)[2 * r + 1];
    uint32_t tc[kRbTiles];
#pragma unroll
    for (int j = 0; j < kRbTiles; ++j) {
        const int64_t t = tid + (int64_t)j * kRbThreads;
        tc[j] = t < L.tiles ? cnt[t] : 0u;
    }
    uint32_t wv[kRbBitBatch];
#pragma unroll
    for (int u = 0; u < kRbBitBatch; ++u) {
        const int64_t w = (int64_t)u * kRbThreads + tid;
        wv[u] = bits[w < L.words ? w : L.words - 1];
    }
    uint64_t reg[kRbTiles][kRbSpec];
#pragma unroll
    for (int j = 0; j < kRbTiles; ++j) {
        const int64_t t = tid + (int64_t)j * kRbThreads;
        const uint64_t* p = first + (t < L.tiles ? t : 0) * (int64_t)kCandFirst;
#pragma unroll
        for (int i = 0; i < kRbSpec; ++i) reg[j][i] = p[i];
    }
    if (tid == 0) sm.nfew = 0u;
    // the row's bits above hi: into LDS, counted on the way
    uint32_t mine = 0u;
#pragma unroll
    for (int u = 0; u < kRbBitBatch; ++u) {
        const int64_t w = (int64_t)u * kRbThreads + tid;
        if (w < L.words) {
            s_bits[w] = wv[u];
            mine += (uint32_t)__popc(wv[u]);
        }
    }
    for (int64_t w = (int64_t)kRbBitBatch * kRbThreads + tid; w < L.words; w += kRbThreads) {   // very large V
        const uint32_t x = bits[w];
        s_bits[w] = x;
        mine += (uint32_t)__popc(x);
    }
    uint32_t band_mine = 0u;
#pragma unroll
    for (int j = 0; j < kRbTiles; ++j) band_mine += tc[j];
    for (int64_t t = tid + (int64_t)kRbTiles * kRbThreads; t < L.tiles; t += kRbThreads) band_mine += cnt[t];
    mine = wave_sum_u32(mine);
    const uint32_t band_incl = wave_prefix_inclusive_u32(band_mine);
    if (lane == 0) sm.w[wave] = mine;
    if (lane == 63) sm.tot[wave] = band_incl;
    __syncthreads();
    uint32_t n_above = 0u, n_band = 0u, band_before = 0u;
#pragma unroll
    for (int w = 0; w < kRbWaves; ++w) {
        n_above += sm.w[w];
        n_band += sm.tot[w];
        band_before += w < wave ? sm.tot[w] : 0u;
    }
    const bool miss = n_above > (uint32_t)k || (uint32_t)k - n_above > n_band;
    if (tid == 0) scratch[L.flag + r] = miss ? 1u : 0u;
    if (miss) return;                                         // uniform: the redo launch handles this row
    uint32_t remain = (uint32_t)k - n_above;                  // candidates to select, 0 <= remain <= n_band

    // candidates of this thread's tiles, from the registers and (crowded or far tiles) from memory
    auto for_each_own = [&](auto&& f) {
#pragma unroll
        for (int j = 0; j < kRbTiles; ++j) {
#pragma unroll
            for (int i = 0; i < kRbSpec; ++i)
                if ((uint32_t)i < tc[j]) f(reg[j][i]);
            if (tc[j] > (uint32_t)kRbSpec) {                  // a crowded tile (ties): the rest from memory
                const uint64_t* p = cand + (tid + (int64_t)j * kRbThreads) * tn;
                for (uint32_t i = kRbSpec; i < tc[j]; ++i) f(p[i]);
            }
        }
        for (int64_t t = tid + (int64_t)kRbTiles * kRbThreads; t < L.tiles; t += kRbThreads) {   // very large V
            const uint32_t n = cnt[t];
            const uint64_t* p0 = first + t * kCandFirst;
            const uint64_t* p = cand + t * tn;
            for (uint32_t i = 0; i < n; ++i) f(i < (uint32_t)kCandFirst ? p0[i] : p[i]);
        }
    };
    const bool dense = remain > 0u && n_band <= cand_cap;     // uniform
    if (dense) {
        uint32_t pos = band_before + band_incl - band_mine;
        for_each_own([&](uint64_t x) { s_cand[pos++] = x; });
        __syncthreads();
    }
    auto for_each_candidate = [&](auto&& f) {
        if (dense) {
            for (uint32_t i = tid; i < n_band; i += kRbThreads) f(s_cand[i]);
        } else {
            for_each_own(f);
        }
    };
    if (remain > 0u) {                                        // uniform
        // MSB-first radix selection of the remain-th largest (key << 32 | ~id).  All candidate keys lie in
        // [key(lo), key(hi)]: the bits these two share are decided from the start.
        const uint32_t khi = f32_to_ord(hi), klo = f32_to_ord(lo);
        int decided = khi == klo ? 32 : __clz((int)(khi ^ klo));
        uint64_t prefix = decided ? ((uint64_t)(khi >> (32 - decided)) << (64 - decided)) : 0ull;
        constexpr int PER = kRbBins / kRbThreads;
        auto set_bit = [&](uint64_t x) {
            const uint32_t id = ~(uint32_t)x;
            atomicOr(&s_bits[id >> 5], 1u << (id & 31u));
        };
        // One wavefront's worth of candidates that share the decided prefix, in sm.few: rank them by counting
        // (keys are unique: they end in the id) and select the `remain` largest.  Called by every thread.
        auto finish_few = [&](uint32_t left, uint32_t remain_now) {
            __syncthreads();
            if (wave == 0) {
                const uint64_t cur = (uint32_t)lane < left ? sm.few[lane] : 0ull;
                uint32_t larger = 0u;
                for (uint32_t j = 0; j < left; ++j) larger += readlane_u64(cur, (int)j) > cur;
                if ((uint32_t)lane < left && larger < remain_now) set_bit(cur);
            }
        };
        // first digit: every candidate shares the bracket's common prefix, so nothing is filtered
        int w = 64 - decided < 11 ? 64 - decided : 11;
        int shift = 64 - decided - w;
#pragma unroll
        for (int i = 0; i < PER; ++i) sm.hist[tid + i * kRbThreads] = 0u;
        __syncthreads();
        for_each_candidate([&](uint64_t x) { atomicAdd(&sm.hist[(uint32_t)(x >> shift) & ((1u << w) - 1u)], 1u); });
        __syncthreads();
        uint32_t c[PER];
#pragma unroll
        for (int i = 0; i < PER; ++i) c[i] = sm.hist[tid * PER + i];
        locate_bin_w<PER, kRbWaves>(c, remain, sm.w, sm.out);
        const uint32_t digit = sm.out[0];
        uint32_t left = sm.out[2];                            // candidates in the digit's bin
        remain -= sm.out[1];                                  // ... of which this many are selected
        prefix |= (uint64_t)digit << shift;
        decided += w;
        if (remain == left || left <= 64u || decided == 64) {
            // the usual case, one more walk: bins above the digit's are selected, the digit's bin is selected
            // as a whole or -- a handful -- ranked
            const bool whole = remain == left || decided == 64;
            for_each_candidate([&](uint64_t x) {
                const uint32_t dg = (uint32_t)(x >> shift) & ((1u << w) - 1u);
                if (dg > digit || (whole && dg == digit)) set_bit(x);
                else if (dg == digit) sm.few[atomicAdd(&sm.nfew, 1u)] = x;
            });
            if (!whole) finish_few(left, remain);
        } else {
            // many candidates share the digit (tied scores): further digits, down to the inverted id
            bool done = false;
            uint64_t T = 0ull;
            while (!done) {
                w = 64 - decided < 11 ? 64 - decided : 11;
                shift = 64 - decided - w;
                __syncthreads();                              // the histogram may still be read by the last locate
#pragma unroll
                for (int i = 0; i < PER; ++i) sm.hist[tid + i * kRbThreads] = 0u;
                __syncthreads();
                for_each_candidate([&](uint64_t x) {
                    if ((x >> (64 - decided)) == (prefix >> (64 - decided)))
                        atomicAdd(&sm.hist[(uint32_t)(x >> shift) & ((1u << w) - 1u)], 1u);
                });
                __syncthreads();
#pragma unroll
                for (int i = 0; i < PER; ++i) c[i] = sm.hist[tid * PER + i];
                locate_bin_w<PER, kRbWaves>(c, remain, sm.w, sm.out);
                prefix |= (uint64_t)sm.out[0] << shift;
                remain -= sm.out[1];
                decided += w;
                left = sm.out[2];
                if (remain == left || decided == 64) {
                    T = prefix;                               // every candidate with the prefix is selected
                    done = true;
                } else if (left <= 64u) {
                    for_each_candidate([&](uint64_t x) {
                        if ((x >> (64 - decided)) == (prefix >> (64 - decided))) sm.few[atomicAdd(&sm.nfew, 1u)] = x;
                    });
                    T = prefix | ((decided < 64 ? (1ull << (64 - decided)) : 0ull) - 1ull);   // above every key with the prefix
                    T += 1ull;                                // (never wraps: the prefix is not all ones below an id)
                    finish_few(left, remain);
                    done = true;
                }
            }
            for_each_candidate([&](uint64_t x) {
                if (x >= T) set_bit(x);
            });
        }
    }
    __syncthreads();                                          // the mask is final
    // ids of the set bits, ascending: wavefront w owns the word pairs [w * ppw, w * ppw + ppw) and walks them 64 at
    // a time with a running output position (no workgroup barrier inside the walk).  The ids go straight to
    // memory: gathering them in LDS first and writing whole lines afterwards was measured slower -- all rows
    // reach that point together, and the stores of the walk overlap its arithmetic instead
    const uint64_t* s_pairs = reinterpret_cast<const uint64_t*>(s_bits);      // words is a multiple of 4
    const int64_t pairs = L.words / 2;
    const int64_t ppw = (pairs + kRbWaves - 1) / kRbWaves;
    const int64_t pbeg = wave * ppw, pend = pbeg + ppw < pairs ? pbeg + ppw : pairs;
    uint32_t total = 0u;
    for (int64_t p = pbeg + lane; p < pend; p += 64) total += (uint32_t)__popcll(s_pairs[p]);
    total = wave_sum_u32(total);
    if (lane == 0) sm.tot[wave] = total;
    __syncthreads();
    uint32_t base = 0u;
#pragma unroll
    for (int w = 0; w < kRbWaves; ++w) base += w < wave ? sm.tot[w] : 0u;
    int32_t* out = idx_out + r * k;
    for (int64_t p0 = pbeg; p0 < pend; p0 += 64) {
        const int64_t p = p0 + lane;
        uint64_t word = p < pend ? s_pairs[p] : 0ull;
        const uint32_t c = (uint32_t)__popcll(word);
        const uint32_t incl = wave_prefix_inclusive_u32(c);
        uint32_t pos = base + incl - c;
        base += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
        while (word) {
            const int b = __ffsll((long long)word) - 1;
            if (pos < (uint32_t)k) out[pos] = (int32_t)(p * 64 + b);          // always true for consistent bits
            ++pos;
            word &= word - 1ull;
        }
    }
}

// Rows flagged by resolve_emit_kernel, redone one after the other by a few workgroups of 1024 threads that walk
// the flags (a launch of one workgroup per row costs microseconds even when every workgroup leaves at once,
// which is the normal case)
constexpr int kRedoBlocks = 32;
template <int DT>
__global__ __launch_bounds__(kSelThreads) void redo_bracket_kernel(int64_t V, int rows, int tn, int64_t m, int64_t k,
                                                                   uint32_t* scratch, int32_t* idx_out, const char* hp,
                                                                   const char* Wv, int chunks) {
    __shared__ RedoSmem rs;
    __shared__ int s_todo[kSelThreads];
    __shared__ uint32_t s_ntodo;
    const BracketLayout L = bracket_layout(V, rows, tn, m);
    const int tid = threadIdx.x;
    // all flags are read at once (one round trip); this workgroup's share of the flagged rows goes to a list
    for (int64_t base = 0; base < rows; base += kSelThreads) {
        const int64_t cand_row = base + tid;
        const bool mine = cand_row < rows && scratch[L.flag + cand_row] != 0u && cand_row % gridDim.x == blockIdx.x;
        if (tid == 0) s_ntodo = 0u;
        __syncthreads();
        if (mine) s_todo[atomicAdd(&s_ntodo, 1u)] = (int)cand_row;
        __syncthreads();
        const uint32_t ntodo = s_ntodo;
        for (uint32_t i = 0; i < ntodo; ++i) {
            const int64_t r = s_todo[i];
            SelLayout SL;
            SL.V = V;
            SL.chunk = (int64_t)kEpt * kSelThreads;
            SL.nb = L.nb;
            SL.replicas = 1;
            SL.zero_words = 0;
            SL.rest_words = 0;
            SelPtrs p;
            p.state = scratch + L.state + (size_t)r * 8;
            p.hist = nullptr;
            p.binfo = p.state + 4;
            p.cand = reinterpret_cast<uint64_t*>(scratch + L.cand) + (size_t)r * L.tiles * tn;   // >= V entries
            p.sure = scratch + L.sure + (size_t)r * L.nb;
            p.offset = scratch + L.boff + (size_t)r * L.nb;
            __syncthreads();                                      // the LDS of the previous row's redo is free again
            redo_row<DT>(hp + r * (int64_t)chunks * 16, Wv, chunks, V, k, p, SL, idx_out + r * k, rs);
        }
        __syncthreads();                                      // the list is rewritten by the next batch of flags
    }
}

}  // namespace

bool scores_supported(int chunks) { return chunks >= 1 && chunks <= 64; }

// more than 64 KiB of dynamic LDS needs an explicit opt-in per kernel and device (called once per device,
// outside any stream capture, by the library's device set-up)
hipError_t configure_select_lds() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&resolve_emit_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kResolveLdsBytes);
}

int64_t select_max_vocab() { return (int64_t)kSelThreads * kMaxBlocksPerRow * kEpt; }

size_t select_scratch_words(int64_t rows, int64_t V) {
    const SelLayout L = sel_layout(V, rows);
    return sel_zero_total(rows, L) + (size_t)rows * L.rest_words;
}

void select_zero_range(int64_t rows, int64_t V, size_t* words) {
    *words = (size_t)rows * sel_layout(V, rows).zero_words;
}

// ---- bracketed selection (many hidden rows, bf16): host side
constexpr int64_t kSample = 8192;                        // sampled tokens per call
constexpr int64_t kBracketMaxVocab = 393216;             // the row's bit mask (V / 8 bytes) lives in LDS: 48 KiB here

// From 65 hidden rows on (measured: at 60 rows the path that materialises the 30 MB of scores, which then stay
// in the last-level cache, takes 71 us against 80 us; at 512 rows 335 us against 160 us)
constexpr int64_t kBracketMinRows = 65;
bool bracket_select_supported(int dt, int64_t rows, int64_t V, int64_t k) {
    (void)k;
    return dt == DT_BF16 && rows >= kBracketMinRows && V >= 4 * kSample && V <= kBracketMaxVocab;
}

size_t bracket_scratch_words(int64_t rows, int64_t V) {
    return bracket_layout(V, (int)rows, bracket_tile_items((int)rows), kSample).total;
}

void bracket_sample(int64_t rows, int64_t V, uint32_t* scratch, int32_t** ids, int64_t* m, float** samp) {
    const BracketLayout L = bracket_layout(V, (int)rows, bracket_tile_items((int)rows), kSample);
    *ids = reinterpret_cast<int32_t*>(scratch + L.ids);
    *m = L.m;
    *samp = reinterpret_cast<float*>(scratch + L.samp);
}

hipError_t launch_bracket_select(const BracketArgs& a, hipStream_t stream) {
    const int tn = bracket_tile_items(a.rows);
    const BracketLayout L = bracket_layout(a.V, a.rows, tn, kSample);
    // ranks of the bracket in the sample: the number of sampled tokens among the row's k best is
    // hypergeometric with mean m k / V; 6 standard deviations and 8 more on either side
    const double q = (double)a.k / (double)a.V, mean = (double)L.m * q;
    const double sd = sqrt((double)L.m * q * (1.0 - q));
    const int64_t rank_hi = (int64_t)floor(mean - 6.0 * sd - 8.0), rank_lo = (int64_t)ceil(mean + 6.0 * sd + 8.0);
    float* thr = reinterpret_cast<float*>(a.scratch + L.thr);
    hipLaunchKernelGGL(bracket_kernel, dim3((unsigned)a.rows), dim3(kRbThreads), 0, stream,
                       reinterpret_cast<const float*>(a.scratch + L.samp), L.m, rank_hi, rank_lo, thr);
    // classify: the full product, nothing stored but bits and candidates
    GemvArgs g{};
    g.x = a.hp;
    g.x_row_bytes = (int64_t)a.chunks * 16;
    g.M = a.Wv;
    g.m_row_bytes = (int64_t)a.chunks * 16;
    g.n_items = a.V;
    g.chunks = a.chunks;
    g.rows = a.rows;
    BracketEpi ep{};
    ep.thr = thr;
    ep.bits = a.scratch + L.bits;
    ep.words_per_row = L.words;
    ep.cand_first = reinterpret_cast<uint64_t*>(a.scratch + L.first);
    ep.cand = reinterpret_cast<uint64_t*>(a.scratch + L.cand);
    ep.cnt = a.scratch + L.cnt;
    ep.item_tiles = L.tiles;
    hipError_t e = launch_tile_mfma_bracket(g, ep, stream);
    if (e != hipSuccess) return e;
    // LDS of a resolve workgroup: the bit mask, then as many candidate slots as keep two workgroups on a CU
    const size_t bits_bytes = (size_t)L.words * 4;
    const size_t room = kResolveLdsBytes > bits_bytes ? kResolveLdsBytes - bits_bytes : 0;
    uint32_t cand_cap = (uint32_t)(room / 8);
    if (cand_cap < 1024u) cand_cap = 0u;                      // not worth a packing pass
    const size_t lds = bits_bytes + (size_t)cand_cap * 8;
    hipLaunchKernelGGL(resolve_emit_kernel, dim3((unsigned)a.rows), dim3(kRbThreads), lds, stream, a.V, a.rows, tn, L.m,
                       a.k, a.scratch, a.idx_out, cand_cap);
    hipLaunchKernelGGL(redo_bracket_kernel<DT_BF16>, dim3((unsigned)(a.rows < kRedoBlocks ? a.rows : kRedoBlocks)),
                       dim3(kSelThreads), 0, stream, a.V, a.rows, tn, L.m, a.k, a.scratch, a.idx_out, a.hp, a.Wv, a.chunks);
    return hipGetLastError();
}

hipError_t launch_scores_hist(int dt, const ScoresArgs& a, uint32_t* scratch, hipStream_t stream) {
    DeviceInfo di;
    hipError_t e = device_info(&di);
    if (e != hipSuccess) return e;
    if (dt == DT_BF16) return launch_scores_dt<DT_BF16>(a, scratch, di.cus, stream);
    return launch_scores_dt<DT_F32>(a, scratch, di.cus, stream);
}

hipError_t launch_hist(const float* s, int64_t V, int64_t k, int rows, uint32_t* scratch, hipStream_t stream) {
    (void)k;
    DeviceInfo di;
    hipError_t e = device_info(&di);
    if (e != hipSuccess) return e;
    int64_t bx = (V + kScoreThreads * 16 - 1) / (kScoreThreads * 16);
    int64_t cap = ((int64_t)di.cus * 2 + rows - 1) / rows;
    if (cap < 1) cap = 1;
    if (bx > cap) bx = cap;
    hipLaunchKernelGGL(hist_kernel, dim3((unsigned)bx, (unsigned)rows), dim3(kScoreThreads), 0, stream, s, V,
                       scratch, rows);
    return hipGetLastError();
}

hipError_t launch_topk_of_scores(const RadixArgs& a, hipStream_t stream) {
    const SelLayout L = sel_layout(a.V, a.rows);
    const dim3 grid((unsigned)L.nb, (unsigned)a.rows);
    if (a.rows <= kFewRows) {
        hipLaunchKernelGGL(collect_kernel, grid, dim3(kSelThreads), 0, stream, a.s, a.V, a.k, a.scratch, a.rows);
        hipLaunchKernelGGL(emit_kernel, grid, dim3(kSelThreads), 0, stream, a.s, a.V, a.k, a.scratch, a.rows,
                           a.idx_out, a.scores_out, a.tau);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(locate_kernel, dim3((unsigned)a.rows), dim3(kSelThreads), 0, stream, a.V, a.k, a.scratch,
                       a.rows);
    hipLaunchKernelGGL(collect_rows_kernel, grid, dim3(kRowThreads), 0, stream, a.s, a.V, a.scratch, a.rows);
    hipLaunchKernelGGL(resolve_kernel, dim3((unsigned)a.rows), dim3(kSelThreads), 0, stream, a.V, a.k, a.scratch,
                       a.rows);
    hipLaunchKernelGGL(emit_rows_kernel, grid, dim3(kRowThreads), 0, stream, a.s, a.V, a.k, a.scratch, a.rows,
                       a.idx_out, a.scores_out, a.tau);
    return hipGetLastError();
}

}  // namespace sv
