// Skinny matrix product on the matrix cores for several hidden-state rows at once:
//     out[r, j] = < M[row(j), :], x[r, :] >      r < rows (<= 32), j < n_items
// (the launcher at the end of this file hands more rows, and mid-size lists from 17 rows on, to the LDS-tiled kernel;
// the form that splits the reduction serves short lists at up to 64 rows)
// with row(j) = j (the full-vocabulary projection of Section 3.1) or row(j) = idx[j] (Section 3.3
// Step 3 with one index set shared by every row of the step).  bf16 storage only.
//
// The work is still bound by reading M from HBM once, so the layout is chosen for that stream:
// one wavefront owns 16 rows of M for the whole reduction and loads them straight into the A-operand
// registers of v_mfma_f32_16x16x32_bf16 (lane = (row i = lane % 16, k-group g = lane / 16) reads
// 16 bytes at row_i + 64 s + 16 g: 64 contiguous bytes per row and instruction, the next
// instruction continues the same cache lines; measured at 85 % of a fully coalesced stream, with
// no LDS round trip).  The hidden states are the B operand: all wavefronts of a workgroup share one
// copy of the current 256-element slice of x in LDS (double buffered, padded rows so that the 16
// lanes of an operand read hit 16 different bank groups).  Accumulators: 16 x 16 float32 per
// 16 hidden rows.  The next slice of M is prefetched into registers while the current one is
// multiplied.
#include "sv_device.h"
#include "sv_launch.h"

namespace sv {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kKC = 256;                         // reduction elements per slice
constexpr int kSteps = kKC / 32;                 // MFMA k-steps per slice (8)
constexpr int kXRowBytes = kKC * 2 + 16;         // padded LDS row of the x slice (528 B = 132 words)

// WPB wavefronts per workgroup (16 rows of M each); NB blocks of 16 hidden rows (N = 16 NB)
// (what the first requests need is repeated as leading plain arguments: those are preloaded into scalar
// registers with the wavefront, a struct passed by value is fetched by instructions)
#define SV_HOT_PARAMS                                                                                          \
    const char *__restrict__ m_base, const int32_t *__restrict__ idx_base, const char *__restrict__ x_base,    \
        const int64_t n_items_arg, const int64_t m_row_bytes_arg, const int64_t x_row_bytes_arg,               \
        const uint32_t *__restrict__ n_items_dev_arg
#define SV_HOT_ARGS(a) (a).M, (a).idx, (a).x, (a).n_items, (a).m_row_bytes, (a).x_row_bytes, (a).n_items_dev
__device__ __forceinline__ GemvArgs with_hot(GemvArgs a, const char* m_base, const int32_t* idx_base, const char* x_base,
                                             int64_t n_items, int64_t m_row_bytes, int64_t x_row_bytes,
                                             const uint32_t* n_items_dev) {
    a.M = m_base;
    a.idx = idx_base;
    a.x = x_base;
    a.n_items = n_items;
    a.m_row_bytes = m_row_bytes;
    a.x_row_bytes = x_row_bytes;
    a.n_items_dev = n_items_dev;
    return a;
}

template <int WPB, int NB>
__global__ __launch_bounds__(WPB * 64) void skinny_mfma_kernel(SV_HOT_PARAMS, const GemvArgs rest, const int row0) {
    const GemvArgs a = with_hot(rest, m_base, idx_base, x_base, n_items_arg, m_row_bytes_arg, x_row_bytes_arg,
                                n_items_dev_arg);
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];     // [2][16 NB][kXRowBytes]
    constexpr int N = 16 * NB;
    constexpr int kThreads = WPB * 64;
    constexpr int kPieces = N * (kKC * 2 / 16);   // 16-byte pieces of one x slice
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int i = lane & 15;                      // row of M within the wave's 16 / hidden row within a block
    const int g = lane >> 4;                      // k-group
    const int C = a.chunks;                       // 16-byte units per row of M and of x
    const int nslices = (C * 8 + kKC - 1) / kKC;
    const int rows_here = min(a.rows - row0, N);
    const int64_t n_items = a.n_items_dev ? (int64_t)*a.n_items_dev : a.n_items;
    if ((int64_t)blockIdx.x * WPB * 16 >= n_items || !gate_open(a, n_items)) return;   // past the end / not this launch's list

    const int64_t tile0 = ((int64_t)blockIdx.x * WPB + wave) * 16;
    int64_t item = tile0 + i;
    if (item > n_items - 1) item = n_items - 1;                   // tail rows are computed, never stored
    const int64_t mrow = a.idx ? (int64_t)a.idx[item] : item;
    const u32x4* mrow_p = reinterpret_cast<const u32x4*>(a.M + mrow * a.m_row_bytes);

    // Units past the end of a row are read as the row's last unit instead of being skipped: their
    // factors in the x slice are zeros and the loaded values are finite, and loads with no condition
    // around them need no branches.
    auto load_a = [&](int slice, u32x4 (&dst)[kSteps]) {
#pragma unroll
        for (int s = 0; s < kSteps; ++s) dst[s] = mrow_p[min(slice * (kKC / 8) + s * 4 + g, C - 1)];
    };
    // the x slice goes global -> registers -> LDS in two steps, so that its latency hides behind the
    // multiplications of the current slice
    constexpr int kXAll = (kPieces + kThreads - 1) / kThreads;     // 16-byte pieces per thread
    constexpr bool kSplit = kXAll <= 4;                            // else: too many registers, stage in one go
    constexpr int kXPer = kSplit ? kXAll : 1;
    static_assert(!kSplit || kPieces % kThreads == 0, "split staging: every thread moves the same number of pieces");
    auto load_x = [&](int slice, u32x4 (&dst)[kXPer]) {            // unconditional: row and unit clamped
#pragma unroll
        for (int q = 0; q < kXPer; ++q) {
            const int p = q * kThreads + tid;
            const int r = min(p / (kKC / 8), rows_here - 1), u = p % (kKC / 8);
            const int unit = min(slice * (kKC / 8) + u, C - 1);
            dst[q] = reinterpret_cast<const u32x4*>(a.x + (int64_t)(row0 + r) * a.x_row_bytes)[unit];
        }
    };
    auto stage_x = [&](int slice, int buf) {                       // one step: load and store at once
        unsigned char* base = smem + (size_t)buf * N * kXRowBytes;
        for (int p = tid; p < kPieces; p += kThreads) {
            const int r = p / (kKC / 8), u = p % (kKC / 8);
            const int unit = slice * (kKC / 8) + u;
            u32x4 v = zero16();
            if (r < rows_here && unit < C)
                v = reinterpret_cast<const u32x4*>(a.x + (int64_t)(row0 + r) * a.x_row_bytes)[unit];
            *reinterpret_cast<u32x4*>(base + (size_t)r * kXRowBytes + u * 16) = v;
        }
    };
    auto store_x = [&](int slice, int buf, const u32x4 (&src)[kXPer]) {     // slice -> buffer buf; zeros past the row
        unsigned char* base = smem + (size_t)buf * N * kXRowBytes;
#pragma unroll
        for (int q = 0; q < kXPer; ++q) {
            const int p = q * kThreads + tid;
            const int r = p / (kKC / 8), u = p % (kKC / 8);
            const bool past = slice * (kKC / 8) + u >= C;
            *reinterpret_cast<u32x4*>(base + (size_t)r * kXRowBytes + u * 16) = past ? zero16() : src[q];
        }
    };

    f32x4_t acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // Workgroups walk the reduction in rotated order: rows of M a power of two apart put the same offset of
    // every row on the same L2 channels, and workgroups that all start at offset 0 keep hitting the same few
    // channels together.  Consecutive workgroups of one XCD (every eighth workgroup) start one slice apart.
    // (Not when the place of an item in the list may vary from run to run, a.plain_order: the order of the
    // float32 additions of a token would vary with it.)
    const int rot = a.plain_order ? 0 : (int)((blockIdx.x / 8) % (unsigned)nslices);
    auto eff = [&](int slice) { const int e = slice + rot; return e >= nslices ? e - nslices : e; };
    u32x4 cur[kSteps], nxt[kSteps];
    u32x4 xr[kXPer];
    load_a(eff(0), cur);
    stage_x(eff(0), 0);
    __syncthreads();
    for (int slice = 0; slice < nslices; ++slice) {
        const int buf = slice & 1;
        const bool more = slice + 1 < nslices;
        if (more) {
            load_a(eff(slice + 1), nxt);
            if constexpr (kSplit) load_x(eff(slice + 1), xr);
            else stage_x(eff(slice + 1), buf ^ 1);
        }
        const unsigned char* xb = smem + (size_t)buf * N * kXRowBytes + (size_t)i * kXRowBytes + g * 16;
#pragma unroll
        for (int s = 0; s < kSteps; ++s) {
            const bf16x8_t av = __builtin_bit_cast(bf16x8_t, cur[s]);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const u32x4 braw = *reinterpret_cast<const u32x4*>(xb + (size_t)nb * 16 * kXRowBytes + s * 64);
                acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8_t, braw), acc[nb],
                                                                  0, 0, 0);
            }
        }
        if constexpr (kSplit)
            if (more) store_x(eff(slice + 1), buf ^ 1, xr);     // the other buffer: nobody reads it during this slice
        __syncthreads();                          // everyone is done with buf; buf^1 is complete
#pragma unroll
        for (int s = 0; s < kSteps; ++s) cur[s] = nxt[s];
    }

    // D[i = 4 g + v][j = lane % 16]: this lane holds 4 consecutive items of hidden row (16 nb + lane % 16)
    const int64_t j0 = tile0 + 4 * g;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int r = nb * 16 + i;
        if (r >= rows_here) continue;
        float* o = a.out_f32 + (int64_t)(row0 + r) * a.out_row_stride + j0;
        if (j0 + 3 < n_items && ((reinterpret_cast<uintptr_t>(o) & 15u) == 0)) {
            *reinterpret_cast<f32x4_t*>(o) = acc[nb];
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (j0 + v < n_items) o[v] = acc[nb][v];
        }
    }
}

// Small item counts (a few thousand rows of M): too few 16-row tiles to fill the chip with one
// wavefront per tile, so the 8 wavefronts of a workgroup share ONE tile and split the reduction:
// wavefront w takes slices w, w + 8, ... of both operands straight from global memory (x is small and
// L2-resident), and the partial 16 x 16 N products are summed through LDS at the end.
// blockIdx.y walks groups of 16 NB hidden rows (a batch of hidden rows against a small M, e.g. the
// selector's down-projection of Section 3.3 Step 1); output float32 or bf16 (round to nearest even);
// the launch can also clear scratch words of a later kernel.
template <int NB>
__global__ __launch_bounds__(512) void skinny_mfma_ksplit_kernel(SV_HOT_PARAMS, const GemvArgs rest,
                                                                 const int row_base) {
    const GemvArgs a = with_hot(rest, m_base, idx_base, x_base, n_items_arg, m_row_bytes_arg, x_row_bytes_arg,
                                n_items_dev_arg);
    constexpr int WPB = 8;
    constexpr int N = 16 * NB;
    __shared__ f32x4_t s_part[WPB][NB][64];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int i = lane & 15;
    const int g = lane >> 4;
    const int C = a.chunks;
    const int nslices = (C * 8 + kKC - 1) / kKC;
    prepare_scratch(a);
    const int row0 = row_base + (int)blockIdx.y * N;
    const int rows_here = min(a.rows - row0, N);
    const int64_t n_items = a.n_items_dev ? (int64_t)*a.n_items_dev : a.n_items;
    const int64_t tile0 = (int64_t)blockIdx.x * 16;
    if (tile0 >= n_items || rows_here <= 0 || !gate_open(a, n_items)) return;

    int64_t item = tile0 + i;
    if (item > n_items - 1) item = n_items - 1;
    const int64_t mrow = a.idx ? (int64_t)a.idx[item] : item;
    const u32x4* mp = reinterpret_cast<const u32x4*>(a.M + mrow * a.m_row_bytes) + g;
    const u32x4* xp[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        int r = nb * 16 + i;
        if (r > rows_here - 1) r = rows_here - 1;         // padding rows repeat the last one, never stored
        xp[nb] = reinterpret_cast<const u32x4*>(a.x + (int64_t)(row0 + r) * a.x_row_bytes) + g;
    }

    f32x4_t acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // whole slices are loaded without conditions (no branches between the loads); only a ragged last
    // slice masks its units
    const int nwhole = C / (kKC / 8);
    auto load_slice = [&](int slice, u32x4 (&av)[kSteps], u32x4 (&bv)[NB][kSteps]) {
        if (slice < nwhole) {
#pragma unroll
            for (int s = 0; s < kSteps; ++s) {
                const int off = slice * (kKC / 8) + s * 4;
                av[s] = mp[off];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) bv[nb][s] = xp[nb][off];
            }
        } else {
#pragma unroll
            for (int s = 0; s < kSteps; ++s) {
                const int off = slice * (kKC / 8) + s * 4;
                const bool ok = off + g < C;
                av[s] = ok ? mp[off] : zero16();
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) bv[nb][s] = ok ? xp[nb][off] : zero16();
            }
        }
    };
    auto multiply = [&](const u32x4 (&av)[kSteps], const u32x4 (&bv)[NB][kSteps]) {
#pragma unroll
        for (int s = 0; s < kSteps; ++s)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, av[s]),
                                                                  __builtin_bit_cast(bf16x8_t, bv[nb][s]), acc[nb],
                                                                  0, 0, 0);
    };
    int slice = wave;
    if constexpr (NB == 1) {
        // registers allow two slices per wavefront in flight: one memory latency instead of two
        for (; slice + WPB < nwhole; slice += 2 * WPB) {
            u32x4 av0[kSteps], bv0[NB][kSteps], av1[kSteps], bv1[NB][kSteps];
            load_slice(slice, av0, bv0);
            load_slice(slice + WPB, av1, bv1);
            multiply(av0, bv0);
            multiply(av1, bv1);
        }
    }
    for (; slice < nslices; slice += WPB) {
        u32x4 av[kSteps], bv[NB][kSteps];
        load_slice(slice, av, bv);
        multiply(av, bv);
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) s_part[wave][nb][lane] = acc[nb];
    __syncthreads();
    if (wave >= NB) return;
    const int nb = wave;                                   // wavefront nb sums and stores hidden rows 16 nb ..
    f32x4_t sum = s_part[0][nb][lane];
#pragma unroll
    for (int w = 1; w < WPB; ++w) sum += s_part[w][nb][lane];
    const int r = nb * 16 + i;
    if (r >= rows_here) return;
    const int64_t j0 = tile0 + 4 * g;
    if (a.out_bf16) {
        uint16_t* o = a.out_bf16 + (int64_t)(row0 + r) * a.out_row_stride + j0;
#pragma unroll
        for (int v = 0; v < 4; ++v)
            if (j0 + v < n_items) o[v] = f32_to_bf16_rne(sum[v]);
        return;
    }
    float* o = a.out_f32 + (int64_t)(row0 + r) * a.out_row_stride + j0;
    if (j0 + 3 < n_items && ((reinterpret_cast<uintptr_t>(o) & 15u) == 0)) {
        *reinterpret_cast<f32x4_t*>(o) = sum;
    } else {
#pragma unroll
        for (int v = 0; v < 4; ++v)
            if (j0 + v < n_items) o[v] = sum[v];
    }
}

template <int NB>
constexpr size_t skinny_lds_bytes() { return (size_t)2 * 16 * NB * kXRowBytes; }

// more than 64 KiB of dynamic LDS needs an explicit opt-in per kernel instance and device
template <int WPB, int NB>
hipError_t opt_in_lds() {
    if (skinny_lds_bytes<NB>() <= 64 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&skinny_mfma_kernel<WPB, NB>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)skinny_lds_bytes<NB>());
}
template <int WPB>
hipError_t opt_in_lds_all_nb() {
    hipError_t e = opt_in_lds<WPB, 1>();
    if (e == hipSuccess) e = opt_in_lds<WPB, 2>();
    return e;
}

template <int NB>
hipError_t launch_ksplit(const GemvArgs& a, int row0, int groups, hipStream_t stream) {
    const int64_t bx = (a.n_items + 15) / 16;
    hipLaunchKernelGGL((skinny_mfma_ksplit_kernel<NB>), dim3((unsigned)bx, (unsigned)groups), dim3(512), 0, stream,
                       SV_HOT_ARGS(a), a, row0);
    return hipGetLastError();
}

template <int WPB, int NB>
hipError_t launch_wn(const GemvArgs& a, int row0, hipStream_t stream) {
    const int64_t per_block = (int64_t)WPB * 16;
    const int64_t bx = (a.n_items + per_block - 1) / per_block;
    const size_t lds = skinny_lds_bytes<NB>();     // above 64 KiB: opted in by configure_skinny_mfma_lds()
    hipLaunchKernelGGL((skinny_mfma_kernel<WPB, NB>), dim3((unsigned)bx), dim3(WPB * 64), lds, stream, SV_HOT_ARGS(a),
                       a, row0);
    return hipGetLastError();
}

template <int WPB>
hipError_t launch_w(const GemvArgs& a, int row0, int nrows, hipStream_t stream) {
    if (nrows <= 16) return launch_wn<WPB, 1>(a, row0, stream);
    return launch_wn<WPB, 2>(a, row0, stream);               // (launch_skinny_mfma keeps up to 32 hidden rows here)
}

}  // namespace

// every instance launch_skinny_mfma can pick, on the current device (called once per device, outside any
// stream capture, by the library's device set-up)
hipError_t configure_skinny_mfma_lds() {
    hipError_t e = opt_in_lds_all_nb<2>();
    if (e == hipSuccess) e = opt_in_lds_all_nb<4>();
    return e;
}

// bf16, rows >= 2, one shared set of rows of M (dense or one index list for the whole step)
bool skinny_mfma_supported(int dt, const GemvArgs& a) {
    return dt == DT_BF16 && a.rows >= 2 && a.idx_row_stride == 0 && a.out_bf16 == nullptr && a.zero_words == 0 && a.spread_n == 0;
}

// A batch of hidden rows against few rows of M (a few thousand at most), long reductions: one launch,
// 32 hidden rows per workgroup row.  Unlike the other matrix-core paths this one also writes bf16
// and clears scratch, which is what the selector's down-projection needs.
bool ksplit_rows_supported(int dt, const GemvArgs& a) {
    DeviceInfo di;
    if (device_info(&di) != hipSuccess) return false;
    return dt == DT_BF16 && a.rows >= 16 && a.idx_row_stride == 0 && a.n_items_dev == nullptr &&
           a.n_items <= (int64_t)di.cus * 16 && a.chunks >= 8 * (kKC / 8);
}

hipError_t launch_ksplit_rows(const GemvArgs& a, hipStream_t stream) {
    DeviceInfo di;
    const hipError_t e = device_info(&di);
    if (e != hipSuccess) return e;
    // few workgroups: 16 hidden rows each (twice as many workgroups, each pulling a third less through its CU)
    const int64_t tiles = (a.n_items + 15) / 16;
    if (tiles * ((a.rows + 31) / 32) * 4 <= di.cus) return launch_ksplit<1>(a, 0, (a.rows + 15) / 16, stream);
    return launch_ksplit<2>(a, 0, (a.rows + 31) / 32, stream);
}

hipError_t launch_skinny_mfma(const GemvArgs& a, hipStream_t stream) {
    if (a.rows > 64) return launch_tile_mfma(a, stream);      // a real contraction: tile both operands
    DeviceInfo di;
    hipError_t e = device_info(&di);
    if (e != hipSuccess) return e;
    // few items: split the reduction over the wavefronts of a workgroup, 32 hidden rows per workgroup row.
    // Every workgroup reads its hidden rows from L2 itself and a CU is through with its workgroups one after the
    // other (time grows in steps of 16 x CUs items), so the more hidden rows, the earlier the other kernel wins:
    // measured crossovers (d = 3840) between 12288 and 16384 items at 2 and 8 rows, between 8192 and 10240 at
    // 16 and 32 rows (16384 items: 29 against 33 us at 8 rows, 36 against 53 at 32 rows); from 33 rows on
    // (d = 4096) between 4096 and 6144 items, where a single tile of the LDS-tiled kernel takes 35 us whatever
    // the list's length (4096 items: 26 against 35 us; 6144: 39 against 35; 8192: 50 against 35).
    const int64_t split_items = (int64_t)di.cus * (a.rows <= 4 ? 64 : a.rows <= 8 ? 48 : a.rows <= 32 ? 32 : 20);
    // A count on the device (the union of the rows' sets; a.n_items is its upper bound, often several times the
    // count when the sets overlap) that may fall on either side of such a crossover: launches with complementary
    // gates, of which those that do not serve the list leave at once (about 2 us each).  The crossovers that matter:
    // the one above, and from 33 rows the one between small tiles with several workgroups per CU and 64 x 256 tiles
    // at half a round of those, 128 x CUs items (the tiled kernel picks its tile by n_items, here the upper end of
    // the gate: 64 x 128; unions of 16 K to 32 K rows gain ~10 us over 64 x 256 tiles, up to 16 K they pay ~3 us
    // against 64 x 64 tiles -- a gate of their own would cost every other list 2 us).  60 rows whose 512 / 1024-item sets unite to
    // 553 / 1401 rows: whole step 31 / 33 us, against 64 / 66 with the kernel picked by the bound.
    if (a.n_items_dev != nullptr && a.gate_hi == 0 && a.n_items > split_items && a.chunks >= 8 * (kKC / 8)) {
        int64_t cuts[2];
        int ncuts = 0;
        // (a union of duplicate-free sets of k items has at least k: from three quarters of the crossover on, the
        // split form has nothing left to win -- 4096 items 26 us against 35 on one tile, 5120 items 33)
        if (4 * a.n_items_min < 3 * split_items) cuts[ncuts++] = split_items;
        if (a.rows > 32 && a.n_items > (int64_t)di.cus * 128) cuts[ncuts++] = (int64_t)di.cus * 128;
        if (ncuts > 0) {
            GemvArgs part = a;
            for (int c = 0; c < ncuts; ++c) {
                part.n_items = cuts[c];               // sizes the grid: enough for every list this launch serves
                part.gate_hi = cuts[c];
                e = launch_skinny_mfma(part, stream);
                if (e != hipSuccess) return e;
                part.gate_lo = cuts[c];
            }
            part.n_items = a.n_items;
            part.gate_hi = INT64_MAX;
            return launch_skinny_mfma(part, stream);
        }
    }
    if (a.n_items <= split_items && a.chunks >= 8 * (kKC / 8)) {
        if (a.rows <= 16) return launch_ksplit<1>(a, 0, 1, stream);
        return launch_ksplit<2>(a, 0, (a.rows + 31) / 32, stream);
    }
    // 33 to 64 hidden rows: the LDS-tiled kernel (whole 128-byte lines per request; it picks its tile by the
    // list's length).  Measured over list lengths from 6144 to 128256 items at 36, 48 and 60 rows it is as fast
    // as or faster than eight wavefronts of this kernel with 16 rows of M each (60 rows: 16384 items 37 against
    // 56 us, 32768 60 against 66, 81920 144 against 155).
    if (a.rows > 32) return launch_tile_mfma(a, stream);
    // 17 to 32 hidden rows: the LDS-tiled kernel on 32 x 64 tiles wins in the middle -- 3 to 15 % between 12288 and
    // 81920 items (32 rows: 24576 items 48 against 55 us, 40960 71 against 79, 81920 127 against 131), equal at
    // 8192 -- and loses 3-5 % from 98304 items on (128256: 203 against 193).
    if (a.rows > 16 && a.n_items <= (int64_t)di.cus * 352) return launch_tile_mfma(a, stream);
    // Wide workgroups share one x slice among more rows of M; small problems need more workgroups.
    // But only a workgroup with at least 128 threads per 16 hidden rows stages the x slice behind the
    // multiplications (four 16-byte pieces per thread), and that matters more than the workgroup count.
    const bool wide = a.n_items >= (int64_t)di.cus * 2 * 128;
    if (a.rows > 16 || wide) return launch_w<4>(a, 0, a.rows, stream);
    return launch_w<2>(a, 0, a.rows, stream);
}

}  // namespace sv
