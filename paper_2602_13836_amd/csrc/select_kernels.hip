// Candidate-vocabulary selection (Section 3.3): approximate logits s = W_vocab h' (Step 1) and
// k_t = top-k(s_t, k) (Step 2).
//
// scores_kernel   streams W_vocab once.  A selector row is short (d' = d/16 .. d/8, i.e. a few
//                 hundred bytes), so a wavefront is split into groups of G lanes, one row per
//                 group, and each load instruction still covers 1 KiB of consecutive memory.
// radix select    exact top-k without sorting: three MSB-first passes over the order-preserving
//                 32-bit keys (11 + 11 + 10 bits) find the key T of the k-th largest score and
//                 how many scores equal to T still belong to the set; a counting pass and an
//                 ordered emission pass then write the selected ids in ascending order (ties on T
//                 go to the smaller ids).  Each pass is one grid over (blocks of the vocabulary,
//                 rows); the last block of a row to finish a histogram pass scans the histogram
//                 ("last block done" ticket), so no pass needs a host round trip.
#include "sv_device.h"
#include "sv_launch.h"

namespace sv {

namespace {

// ------------------------------------------------------------------------------------------
// scores
// ------------------------------------------------------------------------------------------
template <int DT, int G, int UNR>
__global__ __launch_bounds__(256) void scores_kernel(const ScoresArgs a) {
    constexpr int RPW = 64 / G;                       // vocabulary rows per wave-wide load
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane % G;                           // 16-byte unit within the row
    const int sub = lane / G;                         // which of the RPW rows
    const int64_t r = blockIdx.y;
    const int C = a.chunks;
    const int64_t V = a.V;
    const int64_t row_bytes = (int64_t)C * 16;

    const u32x4 xreg = g < C ? reinterpret_cast<const u32x4*>(a.hp + r * row_bytes)[g] : zero16();
    float* s = a.s + r * V;

    const int64_t per_iter = (int64_t)RPW * UNR;
    const int64_t step = (int64_t)gridDim.x * 4 * per_iter;
    for (int64_t base = ((int64_t)blockIdx.x * 4 + wave) * per_iter; base < V; base += step) {
        u32x4 w[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int64_t v = base + (int64_t)u * RPW + sub;
            w[u] = (v < V && g < C)
                       ? load16<false>(reinterpret_cast<const u32x4*>(a.Wv + v * row_bytes) + g)
                       : zero16();
        }
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
            const int64_t v = base + (int64_t)u * RPW + sub;
            if (g == 0 && v < V) s[v] = acc;
        }
    }
}

template <int DT, int G>
hipError_t launch_scores_g(const ScoresArgs& a, int cus, hipStream_t stream) {
    constexpr int UNR = 8;
    const int64_t per_wave = (int64_t)(64 / G) * UNR;
    int64_t bx = ((a.V + per_wave - 1) / per_wave + 3) / 4;
    const int64_t cap = ((int64_t)cus * 8 + a.rows - 1) / a.rows;
    if (bx > cap) bx = cap;
    if (bx < 1) bx = 1;
    hipLaunchKernelGGL((scores_kernel<DT, G, UNR>), dim3((unsigned)bx, (unsigned)a.rows), dim3(256), 0,
                       stream, a);
    return hipGetLastError();
}

template <int DT>
hipError_t launch_scores_dt(const ScoresArgs& a, int cus, hipStream_t stream) {
    if (a.chunks <= 8) return launch_scores_g<DT, 8>(a, cus, stream);
    if (a.chunks <= 16) return launch_scores_g<DT, 16>(a, cus, stream);
    if (a.chunks <= 32) return launch_scores_g<DT, 32>(a, cus, stream);
    return launch_scores_g<DT, 64>(a, cus, stream);
}

// ------------------------------------------------------------------------------------------
// radix select
// ------------------------------------------------------------------------------------------
constexpr int kBins = 2048;
constexpr int kSelThreads = 256;
constexpr int kSelPerThread = 16;
constexpr int kSelChunk = kSelThreads * kSelPerThread;   // vocabulary entries per block

// per-row state words
enum { ST_PREFIX = 0, ST_REMAIN = 1, ST_TICKET0 = 2, ST_T = 6, ST_NEED_EQ = 7, ST_WORDS = 8 };

__host__ __device__ inline int64_t sel_blocks(int64_t V) { return (V + kSelChunk - 1) / kSelChunk; }

struct Scratch {
    uint32_t* state;    // [rows][ST_WORDS]
    uint32_t* hist;     // [rows][3][kBins]
    uint32_t* counts;   // [rows][nb][2]   (greater-than-T, equal-to-T) per block
};
__host__ __device__ inline size_t zeroed_words(int64_t rows) {
    return (size_t)rows * (ST_WORDS + 3 * kBins);
}
__host__ __device__ inline Scratch carve(uint32_t* base, int64_t rows) {
    Scratch s;
    s.state = base;
    s.hist = base + (size_t)rows * ST_WORDS;
    s.counts = base + zeroed_words(rows);
    return s;
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t* p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0u;
}

__device__ __forceinline__ uint32_t coherent_load(const uint32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Histogram pass P (0: key bits 31..21, 1: bits 20..10, 2: bits 9..0) over the keys that share
// the prefix fixed by the earlier passes; the row's last block locates the bin holding the
// remaining-th largest key and extends the prefix.
template <int P>
__global__ __launch_bounds__(kSelThreads) void radix_hist_kernel(const float* s_all, int64_t V, int64_t k,
                                                                 uint32_t* scratch, int rows) {
    __shared__ uint32_t lh[kBins];
    __shared__ uint32_t s_sum[kSelThreads];
    __shared__ int s_last;
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.y;
    const Scratch sc = carve(scratch, rows);
    uint32_t* state = sc.state + r * ST_WORDS;
    uint32_t* hist = sc.hist + (r * 3 + P) * kBins;
    const float* s = s_all + r * V;
    constexpr int nbins = (P == 2) ? 1024 : kBins;
    constexpr int shift = (P == 0) ? 21 : (P == 1 ? 10 : 0);

    for (int b = tid; b < nbins; b += kSelThreads) lh[b] = 0u;
    __syncthreads();
    const uint32_t prefix = (P == 0) ? 0u : state[ST_PREFIX];
    const int64_t base = (int64_t)blockIdx.x * kSelChunk;
#pragma unroll 4
    for (int i = 0; i < kSelPerThread; ++i) {
        const int64_t v = base + (int64_t)i * kSelThreads + tid;
        if (v < V) {
            const uint32_t key = f32_to_ord(s[v]);
            bool match = true;
            if (P == 1) match = (key >> 21) == (prefix >> 21);
            if (P == 2) match = (key >> 10) == (prefix >> 10);
            if (match) atomicAdd(&lh[(key >> shift) & (nbins - 1)], 1u);
        }
    }
    __syncthreads();
    for (int b = tid; b < nbins; b += kSelThreads) {
        const uint32_t c = lh[b];
        if (c) atomicAdd(&hist[b], c);
    }
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const uint32_t t = atomicAdd(&state[ST_TICKET0 + P], 1u);
        s_last = (t == gridDim.x - 1);
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();

    // the last block of this row: find bin b with  above(b) < remain <= above(b) + count(b)
    constexpr int per = nbins / kSelThreads;             // bins per thread (8 or 4)
    const uint32_t remain = (P == 0) ? (uint32_t)k : state[ST_REMAIN];
    uint32_t c[per];
    uint32_t local = 0;
#pragma unroll
    for (int i = 0; i < per; ++i) {
        c[i] = coherent_load(&hist[tid * per + i]);
        local += c[i];
    }
    s_sum[tid] = local;
    __syncthreads();
    uint32_t above = 0;                                   // keys in bins owned by higher threads
    for (int t = tid + 1; t < kSelThreads; ++t) above += s_sum[t];
#pragma unroll
    for (int i = per - 1; i >= 0; --i) {
        if (above < remain && remain <= above + c[i]) {
            const uint32_t bin = (uint32_t)(tid * per + i);
            const uint32_t np = prefix | (bin << shift);
            state[ST_PREFIX] = np;
            state[ST_REMAIN] = remain - above;
            if (P == 2) {
                state[ST_T] = np;
                state[ST_NEED_EQ] = remain - above;
            }
        }
        above += c[i];
    }
}

// per-block counts of keys above T and equal to T
__global__ __launch_bounds__(kSelThreads) void radix_count_kernel(const float* s_all, int64_t V,
                                                                  uint32_t* scratch, int rows) {
    __shared__ uint32_t s_gt[4], s_eq[4];
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.y;
    const Scratch sc = carve(scratch, rows);
    const uint32_t T = sc.state[r * ST_WORDS + ST_T];
    const float* s = s_all + r * V;
    const int64_t base = (int64_t)blockIdx.x * kSelChunk;
    uint32_t gt = 0, eq = 0;
#pragma unroll 4
    for (int i = 0; i < kSelPerThread; ++i) {
        const int64_t v = base + (int64_t)i * kSelThreads + tid;
        if (v < V) {
            const uint32_t key = f32_to_ord(s[v]);
            gt += key > T;
            eq += key == T;
        }
    }
    gt = wave_sum_u32(gt);
    eq = wave_sum_u32(eq);
    if ((tid & 63) == 0) {
        s_gt[tid >> 6] = gt;
        s_eq[tid >> 6] = eq;
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t* cnt = sc.counts + (r * gridDim.x + blockIdx.x) * 2;
        cnt[0] = s_gt[0] + s_gt[1] + s_gt[2] + s_gt[3];
        cnt[1] = s_eq[0] + s_eq[1] + s_eq[2] + s_eq[3];
    }
}

// ordered emission: thread t of a block owns kSelPerThread consecutive vocabulary entries, so
// (block, thread, i) order is ascending token id and a prefix count gives each selected id its slot
__global__ __launch_bounds__(kSelThreads) void radix_emit_kernel(const float* s_all, int64_t V, int64_t k,
                                                                 uint32_t* scratch, int rows,
                                                                 int32_t* idx_out, float* scores_out) {
    __shared__ uint32_t s_gt[kSelThreads], s_eq[kSelThreads];
    __shared__ uint32_t s_base[2];
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.y;
    const Scratch sc = carve(scratch, rows);
    const uint32_t T = sc.state[r * ST_WORDS + ST_T];
    const uint32_t need_eq = sc.state[r * ST_WORDS + ST_NEED_EQ];
    const float* s = s_all + r * V;

    // selected entries in the blocks before this one
    uint32_t pg = 0, pe = 0;
    const uint32_t* cnt = sc.counts + r * gridDim.x * 2;
    for (int b = tid; b < (int)blockIdx.x; b += kSelThreads) {
        pg += cnt[b * 2];
        pe += cnt[b * 2 + 1];
    }
    s_gt[tid] = pg;
    s_eq[tid] = pe;
    __syncthreads();
    if (tid == 0) {
        uint32_t g = 0, e = 0;
        for (int t = 0; t < kSelThreads; ++t) {
            g += s_gt[t];
            e += s_eq[t];
        }
        s_base[0] = g;
        s_base[1] = e;
    }
    __syncthreads();
    const uint32_t base_gt = s_base[0], base_eq = s_base[1];
    __syncthreads();

    const int64_t v0 = (int64_t)blockIdx.x * kSelChunk + (int64_t)tid * kSelPerThread;
    uint32_t key[kSelPerThread];
    uint32_t gt = 0, eq = 0;
#pragma unroll
    for (int i = 0; i < kSelPerThread; ++i) {
        const int64_t v = v0 + i;
        key[i] = v < V ? f32_to_ord(s[v]) : 0u;          // key 0 is below every finite score
        gt += (v < V) && key[i] > T;
        eq += (v < V) && key[i] == T;
    }
    s_gt[tid] = gt;
    s_eq[tid] = eq;
    __syncthreads();
    if (tid == 0) {                                       // exclusive scan over the block's threads
        uint32_t g = 0, e = 0;
        for (int t = 0; t < kSelThreads; ++t) {
            const uint32_t tg = s_gt[t], te = s_eq[t];
            s_gt[t] = g;
            s_eq[t] = e;
            g += tg;
            e += te;
        }
    }
    __syncthreads();
    uint32_t ng = base_gt + s_gt[tid];
    uint32_t ne = base_eq + s_eq[tid];
    int32_t* out = idx_out + r * k;
#pragma unroll
    for (int i = 0; i < kSelPerThread; ++i) {
        const int64_t v = v0 + i;
        if (v < V) {
            const bool is_gt = key[i] > T, is_eq = key[i] == T;
            if (is_gt || (is_eq && ne < need_eq)) {
                const uint32_t pos = ng + (ne < need_eq ? ne : need_eq);
                if (pos < (uint32_t)k) {                  // always true for a consistent (T, need_eq)
                    out[pos] = (int32_t)v;
                    if (scores_out) scores_out[r * k + pos] = s[v];
                }
            }
            ng += is_gt;
            ne += is_eq;
        }
    }
}

}  // namespace

bool scores_supported(int chunks) { return chunks >= 1 && chunks <= 64; }

hipError_t launch_scores(int dt, const ScoresArgs& a, hipStream_t stream) {
    DeviceInfo di;
    hipError_t e = device_info(&di);
    if (e != hipSuccess) return e;
    if (dt == DT_BF16) return launch_scores_dt<DT_BF16>(a, di.cus, stream);
    return launch_scores_dt<DT_F32>(a, di.cus, stream);
}

size_t radix_scratch_words(int64_t rows, int64_t V) {
    return zeroed_words(rows) + (size_t)rows * (size_t)sel_blocks(V) * 2;
}

hipError_t launch_radix_select(const RadixArgs& a, hipStream_t stream) {
    const size_t nz = zeroed_words(a.rows);
    unsigned zb = (unsigned)((nz + 255) / 256);
    if (zb > 1024) zb = 1024;
    hipLaunchKernelGGL(fill_zero_kernel, dim3(zb), dim3(256), 0, stream, a.scratch, nz);
    const dim3 grid((unsigned)sel_blocks(a.V), (unsigned)a.rows), block(kSelThreads);
    hipLaunchKernelGGL((radix_hist_kernel<0>), grid, block, 0, stream, a.s, a.V, a.k, a.scratch, a.rows);
    hipLaunchKernelGGL((radix_hist_kernel<1>), grid, block, 0, stream, a.s, a.V, a.k, a.scratch, a.rows);
    hipLaunchKernelGGL((radix_hist_kernel<2>), grid, block, 0, stream, a.s, a.V, a.k, a.scratch, a.rows);
    hipLaunchKernelGGL(radix_count_kernel, grid, block, 0, stream, a.s, a.V, a.scratch, a.rows);
    hipLaunchKernelGGL(radix_emit_kernel, grid, block, 0, stream, a.s, a.V, a.k, a.scratch, a.rows,
                       a.idx_out, a.scores_out);
    return hipGetLastError();
}

}  // namespace sv
