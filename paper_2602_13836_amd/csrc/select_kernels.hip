// Candidate-vocabulary selection (Section 3.3): approximate logits s = W_vocab h' (Step 1) and
// k_t = top-k(s_t, k) (Step 2), exact, ids in ascending order, ties to the smaller id.
//
// Five launches after the down-projection.  Steps that need a result of the whole row sit behind a
// kernel boundary rather than behind a device-scope fence inside a kernel: on this multi-die part a
// release fence writes back a whole L2, which costs more than a launch.
//   scores_hist   streams W_vocab once.  A selector row is short (d' = d/16 .. d/8: a few hundred
//                 bytes), so a wavefront is split into groups of G lanes, one row per group, and
//                 every load instruction still covers 1 KiB of consecutive memory.  Each score is
//                 stored and counted into a 4096-bin histogram of the top 12 bits of its
//                 order-preserving key (LDS per block, merged with global atomics).
//   locate        one block per row finds the bin B that holds the k-th largest score.
//   collect       counts, per vocabulary block, the scores in bins above B (all selected) and
//                 appends the ids of the scores in bin B to a candidate list.
//   resolve       one block per row: MSB-first radix selection among the candidates over the
//                 remaining 20 key bits and, only if scores tie exactly, the inverted id bits, which
//                 yields a 64-bit threshold T with  selected(v) <=> (key(v) << 32 | ~v) >= T ; it
//                 also turns the per-block counts into output offsets.
//   emit          every block re-evaluates the predicate on its entries in id order and writes the
//                 selected ids (and scores) at its offset: the output is ascending by construction.
#include "sv_device.h"
#include "sv_launch.h"

namespace sv {

namespace {

constexpr int kHistBits = 12;
constexpr int kHistBins = 1 << kHistBits;                // 4096
constexpr int kKeyLowBits = 32 - kHistBits;              // 20
constexpr int kSelThreads = 256;
constexpr int kMaxBlocksPerRow = 1024;                   // vocabulary blocks per row in collect / emit
constexpr int kMaxEpt = 32;                              // entries per thread in collect / emit

// per-row state words (zeroed before every call together with the histogram)
enum { ST_BIN = 2, ST_ABOVE = 3, ST_NCAND = 4, ST_T_HI = 5, ST_T_LO = 6,
       ST_WORDS = 8 };

struct SelLayout {
    int64_t ept;        // vocabulary entries per thread of a collect / emit block
    int64_t chunk;      // entries per block
    int64_t nb;         // blocks per row
    size_t zero_words;  // per row: state + histogram
    size_t row_words;   // per row: everything
};
__host__ __device__ inline SelLayout sel_layout(int64_t V) {
    SelLayout L;
    L.ept = (V + (int64_t)kSelThreads * kMaxBlocksPerRow - 1) / ((int64_t)kSelThreads * kMaxBlocksPerRow);
    if (L.ept < 4) L.ept = 4;
    L.chunk = L.ept * kSelThreads;
    L.nb = (V + L.chunk - 1) / L.chunk;
    L.zero_words = ST_WORDS + kHistBins;
    L.row_words = L.zero_words + 2 * (size_t)L.nb + (size_t)V;
    return L;
}
struct SelPtrs {
    uint32_t* state;    // [ST_WORDS]
    uint32_t* hist;     // [kHistBins]
    uint32_t* sure;     // [nb]  entries in bins above B per block
    uint32_t* offset;   // [nb]  first output slot of each block
    uint32_t* cand;     // [V]   ids of the entries in bin B
};
// zeroed words of all rows come first so that one contiguous range is cleared
__host__ __device__ inline SelPtrs sel_ptrs(uint32_t* base, int64_t rows, int64_t r, const SelLayout& L) {
    SelPtrs p;
    p.state = base + (size_t)r * L.zero_words;
    p.hist = p.state + ST_WORDS;
    uint32_t* rest = base + (size_t)rows * L.zero_words + (size_t)r * (L.row_words - L.zero_words);
    p.sure = rest;
    p.offset = rest + L.nb;
    p.cand = rest + 2 * L.nb;
    return p;
}

// Suffix scan of a histogram held as `per` bins per thread: finds the bin with
//   above(bin) < remain <= above(bin) + count(bin)   (above = entries in higher bins)
// and reports (bin, above, count) through LDS to every thread.  Exactly one bin qualifies whenever
// the histogram holds at least `remain` entries.
template <int PER>
__device__ __forceinline__ void locate_bin(const uint32_t (&c)[PER], uint32_t remain, uint32_t* s_sum,
                                           uint32_t* s_out) {
    const int tid = threadIdx.x;
    uint32_t local = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) local += c[i];
    s_sum[tid] = local;
    __syncthreads();
    uint32_t above = 0;
    for (int t = tid + 1; t < kSelThreads; ++t) above += s_sum[t];
#pragma unroll
    for (int i = PER - 1; i >= 0; --i) {
        if (above < remain && remain <= above + c[i]) {
            s_out[0] = (uint32_t)(tid * PER + i);
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
template <int DT, int G, int UNR>
__global__ __launch_bounds__(kSelThreads) void scores_hist_kernel(const ScoresArgs a, uint32_t* scratch) {
    constexpr int RPW = 64 / G;                       // vocabulary rows per wave-wide load
    __shared__ uint32_t lh[kHistBins];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane % G;                           // 16-byte unit within the row
    const int sub = lane / G;                         // which of the RPW rows
    const int64_t r = blockIdx.y;
    const int C = a.chunks;
    const int64_t V = a.V;
    const int64_t row_bytes = (int64_t)C * 16;

    for (int b = tid; b < kHistBins; b += kSelThreads) lh[b] = 0u;
    const u32x4 xreg = g < C ? reinterpret_cast<const u32x4*>(a.hp + r * row_bytes)[g] : zero16();
    float* s = a.s + r * V;
    __syncthreads();

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
            if (g == 0 && v < V) {
                s[v] = acc;
                atomicAdd(&lh[f32_to_ord(acc) >> kKeyLowBits], 1u);
            }
        }
    }
    __syncthreads();

    const SelLayout L = sel_layout(V);
    const SelPtrs p = sel_ptrs(scratch, a.rows, r, L);
    for (int b = tid; b < kHistBins; b += kSelThreads) {
        const uint32_t c = lh[b];
        if (c) atomicAdd(&p.hist[b], c);
    }
}

// histogram only (scores produced by another kernel)
__global__ __launch_bounds__(kSelThreads) void hist_kernel(const float* s_all, int64_t V, int64_t k,
                                                           uint32_t* scratch, int rows) {
    __shared__ uint32_t lh[kHistBins];
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.y;
    const float* s = s_all + r * V;
    for (int b = tid; b < kHistBins; b += kSelThreads) lh[b] = 0u;
    __syncthreads();
    for (int64_t v = (int64_t)blockIdx.x * kSelThreads + tid; v < V; v += (int64_t)gridDim.x * kSelThreads)
        atomicAdd(&lh[f32_to_ord(s[v]) >> kKeyLowBits], 1u);
    __syncthreads();
    const SelLayout L = sel_layout(V);
    const SelPtrs p = sel_ptrs(scratch, rows, r, L);
    for (int b = tid; b < kHistBins; b += kSelThreads) {
        const uint32_t c = lh[b];
        if (c) atomicAdd(&p.hist[b], c);
    }
}

// the bin that holds the k-th largest score of each row
__global__ __launch_bounds__(kSelThreads) void locate_kernel(int64_t V, int64_t k, uint32_t* scratch, int rows) {
    __shared__ uint32_t s_sum[kSelThreads];
    __shared__ uint32_t s_out[4];
    const int tid = threadIdx.x;
    const SelLayout L = sel_layout(V);
    const SelPtrs p = sel_ptrs(scratch, rows, blockIdx.x, L);
    constexpr int PER = kHistBins / kSelThreads;      // 16
    uint32_t c[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) c[i] = p.hist[tid * PER + i];
    locate_bin<PER>(c, (uint32_t)k, s_sum, s_out);
    if (tid == 0) {
        p.state[ST_BIN] = s_out[0];
        p.state[ST_ABOVE] = s_out[1];
    }
}

template <int DT, int G>
hipError_t launch_scores_g(const ScoresArgs& a, uint32_t* scratch, int cus, hipStream_t stream) {
    constexpr int UNR = 8;
    const int64_t per_block = (int64_t)(64 / G) * UNR * 4;
    int64_t bx = (a.V + per_block - 1) / per_block;
    int64_t cap = ((int64_t)cus * 2 + a.rows - 1) / a.rows;     // a few long-lived blocks per CU
    if (cap < 1) cap = 1;
    if (bx > cap) bx = cap;
    hipLaunchKernelGGL((scores_hist_kernel<DT, G, UNR>), dim3((unsigned)bx, (unsigned)a.rows),
                       dim3(kSelThreads), 0, stream, a, scratch);
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
// collect + resolve
// ------------------------------------------------------------------------------------------
// 52-bit sub-key of a candidate: the 20 low key bits, then the inverted id (smaller id = larger)
__device__ __forceinline__ uint64_t sub_key(uint32_t key, uint32_t v) {
    return ((uint64_t)(key & ((1u << kKeyLowBits) - 1u)) << 32) | (uint32_t)(~v);
}

__global__ __launch_bounds__(kSelThreads) void collect_kernel(const float* s_all, int64_t V, uint32_t* scratch,
                                                              int rows) {
    __shared__ uint32_t s_list[kSelThreads * kMaxEpt];    // ids of this block's bin-B entries
    __shared__ uint32_t s_n, s_gbase, s_sure[4];
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.y;
    const SelLayout L = sel_layout(V);
    const SelPtrs p = sel_ptrs(scratch, rows, r, L);
    const float* s = s_all + r * V;
    const uint32_t B = p.state[ST_BIN];

    if (tid == 0) s_n = 0u;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * L.chunk;
    uint32_t sure = 0u;
    for (int64_t i = 0; i < L.ept; ++i) {
        const int64_t v = base + i * kSelThreads + tid;
        if (v < V) {
            const uint32_t bin = f32_to_ord(s[v]) >> kKeyLowBits;
            sure += bin > B;
            if (bin == B) s_list[atomicAdd(&s_n, 1u)] = (uint32_t)v;
        }
    }
    sure = wave_sum_u32(sure);
    if ((tid & 63) == 0) s_sure[tid >> 6] = sure;
    __syncthreads();
    const uint32_t n_local = s_n;
    if (tid == 0) {
        p.sure[blockIdx.x] = s_sure[0] + s_sure[1] + s_sure[2] + s_sure[3];
        s_gbase = n_local ? atomicAdd(&p.state[ST_NCAND], n_local) : 0u;
    }
    __syncthreads();
    const uint32_t gbase = s_gbase;
    for (uint32_t i = tid; i < n_local; i += kSelThreads) p.cand[gbase + i] = s_list[i];
}

// one block per row: threshold among the candidates of bin B, then the output offset of every block
__global__ __launch_bounds__(kSelThreads) void resolve_kernel(const float* s_all, int64_t V, int64_t k,
                                                              uint32_t* scratch, int rows) {
    __shared__ uint32_t s_hist[2048];
    __shared__ uint32_t s_sum[kSelThreads];
    __shared__ uint32_t s_out[4];
    __shared__ uint32_t s_cnt[kMaxBlocksPerRow];
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.x;
    const SelLayout L = sel_layout(V);
    const SelPtrs p = sel_ptrs(scratch, rows, r, L);
    const float* s = s_all + r * V;
    const uint32_t B = p.state[ST_BIN];
    const uint32_t above = p.state[ST_ABOVE];

    // ---- resolver: the m-th largest sub-key among the n candidates of bin B
    const uint32_t n = p.state[ST_NCAND];
    uint32_t remain = (uint32_t)k - above;              // 1 <= remain <= n
    uint64_t prefix = 0ull;                             // decided high bits of the threshold sub-key
    int decided = 0;                                    // how many of the 52 bits are decided
    bool all_of_prefix = false;
    // digit widths from the MSB: the 20 key bits as 11 + 9, then the 32 id bits as 11 + 11 + 10
    const int widths[5] = {11, 9, 11, 11, 10};
    for (int pass = 0; pass < 5 && !all_of_prefix; ++pass) {
        const int w = widths[pass];
        const int shift = 52 - decided - w;
        for (int b = tid; b < 2048; b += kSelThreads) s_hist[b] = 0u;
        __syncthreads();
        for (uint32_t i = tid; i < n; i += kSelThreads) {
            const uint32_t v = p.cand[i];
            const uint64_t sk = sub_key(f32_to_ord(s[v]), v);
            if (decided == 0 || (sk >> (52 - decided)) == (prefix >> (52 - decided)))
                atomicAdd(&s_hist[(uint32_t)(sk >> shift) & ((1u << w) - 1u)], 1u);
        }
        __syncthreads();
        uint32_t c[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) c[i] = s_hist[tid * 8 + i];
        locate_bin<8>(c, remain, s_sum, s_out);
        prefix |= (uint64_t)s_out[0] << shift;
        remain -= s_out[1];
        decided += w;
        all_of_prefix = (remain == s_out[2]);           // every candidate with this prefix is selected
        __syncthreads();
    }
    // threshold: selected(v) <=> (key << 32 | ~v) >= T, T = (B << 20 | prefix.hi) << 32 | prefix.lo
    const uint32_t t_hi = (B << kKeyLowBits) | (uint32_t)(prefix >> 32);
    const uint32_t t_lo = (uint32_t)prefix;
    if (tid == 0) {
        p.state[ST_T_HI] = t_hi;
        p.state[ST_T_LO] = t_lo;
    }
    // ---- output offsets: selected entries per block = sure + selected candidates, exclusive scan
    const int nb = (int)L.nb;
    for (int b = tid; b < nb; b += kSelThreads) s_cnt[b] = 0u;
    __syncthreads();
    for (uint32_t i = tid; i < n; i += kSelThreads) {
        const uint32_t v = p.cand[i];
        if (sub_key(f32_to_ord(s[v]), v) >= prefix) atomicAdd(&s_cnt[v / (uint32_t)L.chunk], 1u);
    }
    __syncthreads();
    constexpr int PERB = kMaxBlocksPerRow / kSelThreads;   // 4 consecutive blocks per thread
    uint32_t tot[PERB];
    uint32_t local = 0u;
#pragma unroll
    for (int i = 0; i < PERB; ++i) {
        const int b = tid * PERB + i;
        tot[i] = b < nb ? s_cnt[b] + p.sure[b] : 0u;
        local += tot[i];
    }
    s_sum[tid] = local;
    __syncthreads();
    uint32_t run = 0u;
    for (int t = 0; t < tid; ++t) run += s_sum[t];
#pragma unroll
    for (int i = 0; i < PERB; ++i) {
        const int b = tid * PERB + i;
        if (b < nb) p.offset[b] = run;
        run += tot[i];
    }
}

// ------------------------------------------------------------------------------------------
// emit
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelThreads) void emit_kernel(const float* s_all, int64_t V, int64_t k,
                                                           uint32_t* scratch, int rows, int32_t* idx_out,
                                                           float* scores_out) {
    __shared__ uint32_t s_wave[4];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int64_t r = blockIdx.y;
    const SelLayout L = sel_layout(V);
    const SelPtrs p = sel_ptrs(scratch, rows, r, L);
    const float* s = s_all + r * V;
    const uint64_t T = ((uint64_t)p.state[ST_T_HI] << 32) | p.state[ST_T_LO];
    const uint32_t block_off = p.offset[blockIdx.x];

    // thread t owns ept consecutive ids, so (thread, i) order is ascending id order
    const int64_t v0 = (int64_t)blockIdx.x * L.chunk + (int64_t)tid * L.ept;
    uint32_t mask = 0u;
    for (int64_t i = 0; i < L.ept; ++i) {
        const int64_t v = v0 + i;
        if (v < V) {
            const uint64_t key64 = ((uint64_t)f32_to_ord(s[v]) << 32) | (uint32_t)(~(uint32_t)v);
            if (key64 >= T) mask |= 1u << i;
        }
    }
    const uint32_t mine = (uint32_t)__popc(mask);
    // exclusive prefix over the block: wave scan, then the four wave totals
    uint32_t incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t o = __shfl_up(incl, off);
        if (lane >= off) incl += o;
    }
    if (lane == 63) s_wave[tid >> 6] = incl;
    __syncthreads();
    uint32_t pos = block_off + incl - mine;
    for (int w = 0; w < (tid >> 6); ++w) pos += s_wave[w];

    int32_t* out = idx_out + r * k;
    for (int64_t i = 0; i < L.ept; ++i) {
        if (mask & (1u << i)) {
            if (pos < (uint32_t)k) {                      // always true for a consistent threshold
                out[pos] = (int32_t)(v0 + i);
                if (scores_out) scores_out[r * k + pos] = s[v0 + i];
            }
            ++pos;
        }
    }
}

}  // namespace

bool scores_supported(int chunks) { return chunks >= 1 && chunks <= 64; }

int64_t select_max_vocab() { return (int64_t)kSelThreads * kMaxBlocksPerRow * kMaxEpt; }

size_t select_scratch_words(int64_t rows, int64_t V) { return (size_t)rows * sel_layout(V).row_words; }

void select_zero_range(int64_t rows, int64_t V, size_t* words) { *words = (size_t)rows * sel_layout(V).zero_words; }

hipError_t launch_scores_hist(int dt, const ScoresArgs& a, uint32_t* scratch, hipStream_t stream) {
    DeviceInfo di;
    hipError_t e = device_info(&di);
    if (e != hipSuccess) return e;
    if (dt == DT_BF16) return launch_scores_dt<DT_BF16>(a, scratch, di.cus, stream);
    return launch_scores_dt<DT_F32>(a, scratch, di.cus, stream);
}

hipError_t launch_hist(const float* s, int64_t V, int64_t k, int rows, uint32_t* scratch, hipStream_t stream) {
    DeviceInfo di;
    hipError_t e = device_info(&di);
    if (e != hipSuccess) return e;
    int64_t bx = (V + kSelThreads * 4 - 1) / (kSelThreads * 4);
    int64_t cap = ((int64_t)di.cus * 4 + rows - 1) / rows;
    if (cap < 1) cap = 1;
    if (bx > cap) bx = cap;
    hipLaunchKernelGGL(hist_kernel, dim3((unsigned)bx, (unsigned)rows), dim3(kSelThreads), 0, stream, s, V, k,
                       scratch, rows);
    return hipGetLastError();
}

hipError_t launch_topk_of_scores(const RadixArgs& a, hipStream_t stream) {
    const SelLayout L = sel_layout(a.V);
    const dim3 grid((unsigned)L.nb, (unsigned)a.rows), block(kSelThreads);
    hipLaunchKernelGGL(locate_kernel, dim3((unsigned)a.rows), block, 0, stream, a.V, a.k, a.scratch, a.rows);
    hipLaunchKernelGGL(collect_kernel, grid, block, 0, stream, a.s, a.V, a.scratch, a.rows);
    hipLaunchKernelGGL(resolve_kernel, dim3((unsigned)a.rows), block, 0, stream, a.s, a.V, a.k, a.scratch, a.rows);
    hipLaunchKernelGGL(emit_kernel, grid, block, 0, stream, a.s, a.V, a.k, a.scratch, a.rows, a.idx_out,
                       a.scores_out);
    return hipGetLastError();
}

}  // namespace sv
