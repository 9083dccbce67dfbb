// Tiled matrix product on the matrix cores for MANY hidden-state rows (more than 64):
//     out[r, j] = < M[row(j), :], x[r, :] >      r < rows, j < n_items
// with row(j) = j (the full-vocabulary projection of Section 3.1, or the selector's score matrix of
// Section 3.3 Step 1 for a whole batch) or row(j) = idx[j] (Section 3.3 Step 3 over one set of rows
// shared by every hidden row).  bf16 storage only.
//
// With hundreds of hidden rows the product is a real contraction (Section 3.4 counts V d
// multiply-adds per hidden row): reading M once per 64 hidden rows, as the skinny kernel does, turns
// into many passes over M.  Here a workgroup owns a TM x TN tile of the output (TM hidden rows, TN
// rows of M) and walks the reduction in slices of 64 elements: both operand slices go
// global -> registers -> LDS (double buffered, one barrier per slice) and every wavefront multiplies
// its part of the tile with v_mfma_f32_32x32x16_bf16 from LDS.  LDS rows are padded to 144 bytes so
// that the 16-byte operand reads of consecutive lanes fall into distinct banks (measured: full LDS
// read rate, no bank conflicts).  Workgroups that share rows of M (the different hidden-row tiles of
// one TN block) are given consecutive slots on the same XCD, so that M comes from HBM once and from
// that die's L2 afterwards (measured: HBM traffic 1.27 x the size of M at 512 hidden rows).
//
// Two forms of the main loop.  The plain one leaves the order of loads, LDS traffic and MFMAs to the
// compiler and relies on two workgroups per CU to overlap them: best while the kernel is bound by
// the one pass over M (up to 128 hidden rows).  The pipelined one is for 256 x 256 tiles, where a
// SIMD holds one or two wavefronts and nothing else hides their waits: operand fragments are read
// one 16-element step ahead, the LDS copy of the next slice is spread over the four steps of the
// current one (LDS writes run at a third of the read rate; a burst of them stalls the fragment
// reads), and scheduling-group fences pin that order against the compiler's own scheduler.
#include "sv_device.h"
#include "sv_launch.h"

namespace sv {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kTK = 64;                  // reduction elements per slice (128 bytes of a row)
constexpr int kRowB = kTK * 2 + 16;      // padded LDS row (144 B = 36 words)
constexpr int kXcds = 8;

// Wanted instruction order of one 16-element step: M MFMAs with R LDS reads, W LDS writes and W global
// loads spread evenly between them (the sizes of a scheduling group must be compile-time constants).
template <int M, int R, int W, int I>
__device__ __forceinline__ void sched_pattern() {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                       // one MFMA
    constexpr int r = (I + 1) * R / M - I * R / M;
    if constexpr (r > 0) __builtin_amdgcn_sched_group_barrier(0x100, r, 0);  // LDS reads
    constexpr int w = (I + 1) * W / M - I * W / M;
    if constexpr (w > 0) {
        __builtin_amdgcn_sched_group_barrier(0x200, w, 0);                   // LDS writes
        __builtin_amdgcn_sched_group_barrier(0x020, w, 0);                   // global loads
    }
    if constexpr (I + 1 < M) sched_pattern<M, R, W, I + 1>();
}

// GM x GN wavefronts; each owns WM x WN MFMA tiles of 32 x 32: TM = 32 GM WM hidden rows, TN = 32 GN WN items.
// PIPE selects the hand-ordered main loop.
template <int GM, int GN, int WM, int WN, bool PIPE>
__global__ __launch_bounds__(64 * GM * GN) void tile_mfma_kernel(const GemvArgs a) {
    constexpr int kThreads = 64 * GM * GN;
    constexpr int kRowsPerPass = kThreads / 8;           // loader: 8 threads per 128-byte row slice
    constexpr int TM = 32 * GM * WM, TN = 32 * GN * WN;
    constexpr int QA = TM / kRowsPerPass, QB = TN / kRowsPerPass;   // 16-byte loads per thread and slice
    static_assert(TM % kRowsPerPass == 0 && TN % kRowsPerPass == 0, "tile rows must fill whole loader passes");
    constexpr int kStage = (TM + TN) * kRowB;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // [2][TM + TN][kRowB]
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wr = wave / GN, wc = wave % GN;
    const int C = a.chunks;
    const int nk = (C + 7) / 8;
    const int64_t n_items = a.n_items_dev ? (int64_t)*a.n_items_dev : a.n_items;
    const int RT = (a.rows + TM - 1) / TM;
    const int64_t IT = (n_items + TN - 1) / TN;
    // block id -> (XCD, slot on that XCD); consecutive slots of one XCD: the RT hidden-row tiles of one item tile
    const int64_t slot = blockIdx.x / kXcds;
    const int rt = (int)(slot % RT);
    const int64_t it = (slot / RT) * kXcds + (blockIdx.x % kXcds);
    if (it >= IT) return;

    // loader role: 8 threads cover the 128-byte slice of one row, 32 rows per pass
    const int piece = tid & 7, r0 = tid >> 3;
    const u32x4* pa[QA];
    const u32x4* pb[QB];
#pragma unroll
    for (int q = 0; q < QA; ++q) {
        int row = rt * TM + r0 + kRowsPerPass * q;
        if (row > a.rows - 1) row = a.rows - 1;                       // padding rows: computed, never stored
        pa[q] = reinterpret_cast<const u32x4*>(a.x + (int64_t)row * a.x_row_bytes);
    }
#pragma unroll
    for (int q = 0; q < QB; ++q) {
        int64_t item = it * TN + r0 + kRowsPerPass * q;
        if (item > n_items - 1) item = n_items - 1;
        const int64_t mrow = a.idx ? (int64_t)a.idx[item] : item;
        pb[q] = reinterpret_cast<const u32x4*>(a.M + mrow * a.m_row_bytes);
    }
    // Loads and stores of the pipeline are unconditional (slice and unit indices are clamped; the
    // units of a ragged last slice that lie past the row are zeroed on their way into LDS, when the
    // data has arrived anyway): without branches between them the compiler can count the loads in
    // flight and wait for exactly the oldest slice.
    auto load = [&](int ks, u32x4 (&ga)[QA], u32x4 (&gb)[QB]) {
        const int u = min(min(ks, nk - 1) * 8 + piece, C - 1);
#pragma unroll
        for (int q = 0; q < QB; ++q) gb[q] = pb[q][u];
#pragma unroll
        for (int q = 0; q < QA; ++q) ga[q] = pa[q][u];
    };
    auto store = [&](int ks, const u32x4 (&ga)[QA], const u32x4 (&gb)[QB]) {      // slice ks -> buffer ks % 2
        unsigned char* base = smem + (size_t)(ks & 1) * kStage + (size_t)r0 * kRowB + piece * 16;
        const bool past = ks * 8 + piece >= C;
#pragma unroll
        for (int q = 0; q < QA; ++q)
            *reinterpret_cast<u32x4*>(base + (size_t)(kRowsPerPass * q) * kRowB) = past ? zero16() : ga[q];
#pragma unroll
        for (int q = 0; q < QB; ++q)
            *reinterpret_cast<u32x4*>(base + (size_t)(TM + kRowsPerPass * q) * kRowB) = past ? zero16() : gb[q];
    };

    f32x16_t acc[WM][WN];
#pragma unroll
    for (int m = 0; m < WM; ++m)
#pragma unroll
        for (int n = 0; n < WN; ++n)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[m][n][e] = 0.f;

    // operand role: lane = (row within the 32 x 32 tile = lane % 32, k-group = lane / 32)
    const size_t a_off = (size_t)(wr * 32 * WM + (lane & 31)) * kRowB + (lane >> 5) * 16;
    const size_t b_off = (size_t)(TM + wc * 32 * WN + (lane & 31)) * kRowB + (lane >> 5) * 16;
    auto multiply = [&](int buf) {
        const unsigned char* sa = smem + (size_t)buf * kStage + a_off;
        const unsigned char* sb = smem + (size_t)buf * kStage + b_off;
#pragma unroll
        for (int kk = 0; kk < kTK / 16; ++kk) {
            bf16x8_t af[WM], bf[WN];
#pragma unroll
            for (int m = 0; m < WM; ++m)
                af[m] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4*>(sa + (size_t)(32 * m) * kRowB + kk * 32));
#pragma unroll
            for (int n = 0; n < WN; ++n)
                bf[n] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4*>(sb + (size_t)(32 * n) * kRowB + kk * 32));
#pragma unroll
            for (int m = 0; m < WM; ++m)
#pragma unroll
                for (int n = 0; n < WN; ++n)
                    acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[m], bf[n], acc[m][n], 0, 0, 0);
        }
    };
    if constexpr (PIPE) {
        // the slice is walked in four 16-element steps with the operand fragments of the next step
        // already on their way from LDS while the current step multiplies
        u32x4 ga[QA], gb[QB];
        bf16x8_t fa[2][WM], fb[2][WN];
        auto read_frags = [&](int buf, int kk, bf16x8_t (&A)[WM], bf16x8_t (&B)[WN]) {
            const unsigned char* sa = smem + (size_t)buf * kStage + a_off + kk * 32;
            const unsigned char* sb = smem + (size_t)buf * kStage + b_off + kk * 32;
#pragma unroll
            for (int m = 0; m < WM; ++m)
                A[m] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4*>(sa + (size_t)(32 * m) * kRowB));
#pragma unroll
            for (int n = 0; n < WN; ++n)
                B[n] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4*>(sb + (size_t)(32 * n) * kRowB));
        };
        auto mfmas = [&](const bf16x8_t (&A)[WM], const bf16x8_t (&B)[WN]) {
#pragma unroll
            for (int m = 0; m < WM; ++m)
#pragma unroll
                for (int n = 0; n < WN; ++n)
                    acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[m], B[n], acc[m][n], 0, 0, 0);
        };
        // The copy of the next slice into LDS is cut into four parts, one per step; each part's
        // registers are reloaded with the slice after next at once.  Part 0 goes right after the
        // barrier (the buffer just read is free then), parts 1..3 in the first three steps.
        static_assert(QA % 4 == 0 && QB % 4 == 0, "the staged slice is copied in four parts");
        constexpr int PA = QA / 4, PB = QB / 4;
        auto load_part = [&](int j, int ks) {
            const int u = min(min(ks, nk - 1) * 8 + piece, C - 1);
#pragma unroll
            for (int q = 0; q < PB; ++q) gb[j * PB + q] = pb[j * PB + q][u];
#pragma unroll
            for (int q = 0; q < PA; ++q) ga[j * PA + q] = pa[j * PA + q][u];
        };
        auto store_part = [&](int j, int ks) {
            unsigned char* base = smem + (size_t)(ks & 1) * kStage + (size_t)r0 * kRowB + piece * 16;
            const bool past = ks * 8 + piece >= C;
#pragma unroll
            for (int q = 0; q < PA; ++q)
                *reinterpret_cast<u32x4*>(base + (size_t)(kRowsPerPass * (j * PA + q)) * kRowB) = past ? zero16() : ga[j * PA + q];
#pragma unroll
            for (int q = 0; q < PB; ++q)
                *reinterpret_cast<u32x4*>(base + (size_t)(TM + kRowsPerPass * (j * PB + q)) * kRowB) = past ? zero16() : gb[j * PB + q];
        };
        // one step: fragment reads of the next step, a quarter of the slice copy, and this step's MFMAs,
        // interleaved so that every memory instruction issues in the shadow of a running MFMA
        auto interleave = [&]() {
            sched_pattern<WM * WN, WM + WN, PA + PB, 0>();
            __builtin_amdgcn_sched_barrier(0);
        };
        load(0, ga, gb);
        store(0, ga, gb);
        load(1, ga, gb);
        __syncthreads();
        store_part(0, 1);
        load_part(0, 2);
        read_frags(0, 0, fa[0], fb[0]);
        for (int ks = 0; ks < nk; ++ks) {
            const int buf = ks & 1;
            read_frags(buf, 1, fa[1], fb[1]);
            store_part(1, ks + 1);
            load_part(1, ks + 2);
            mfmas(fa[0], fb[0]);
            interleave();
            read_frags(buf, 2, fa[0], fb[0]);
            store_part(2, ks + 1);
            load_part(2, ks + 2);
            mfmas(fa[1], fb[1]);
            interleave();
            read_frags(buf, 3, fa[1], fb[1]);
            store_part(3, ks + 1);
            load_part(3, ks + 2);
            mfmas(fa[0], fb[0]);
            interleave();
            __syncthreads();     // slice ks + 1 is complete in the other buffer; this one is free again
            read_frags(buf ^ 1, 0, fa[0], fb[0]);
            store_part(0, ks + 2);
            load_part(0, ks + 3);
            mfmas(fa[1], fb[1]);
            interleave();
        }
    } else {
        // Two register sets keep two slices in flight from global memory while a third is multiplied
        // out of LDS: on entry to step(ks, set) the set holds slice ks + 1 (the other set slice ks + 2).
        u32x4 ga0[QA], gb0[QB], ga1[QA], gb1[QB];
        auto step = [&](int ks, u32x4 (&ga)[QA], u32x4 (&gb)[QB]) {
            multiply(ks & 1);
            store(ks + 1, ga, gb);            // the other buffer: nobody reads it during this slice
            __syncthreads();                  // everyone is done with this buffer; the other is complete
            load(ks + 3, ga, gb);
        };
        load(0, ga0, gb0);
        store(0, ga0, gb0);
        load(1, ga0, gb0);
        load(2, ga1, gb1);
        __syncthreads();
        for (int ks = 0; ks < nk; ks += 2) {  // an odd slice count runs one more step, on a slice of zeros
            step(ks, ga0, gb0);
            step(ks + 1, ga1, gb1);
        }
    }

    // D[i][j]: j = lane % 32 (item), i = 8 (e / 4) + 4 (lane / 32) + e % 4 (hidden row) for element e
    const int64_t item0 = it * TN + wc * 32 * WN + (lane & 31);
    const int row0 = rt * TM + wr * 32 * WM + 4 * (lane >> 5);
#pragma unroll
    for (int m = 0; m < WM; ++m)
#pragma unroll
        for (int n = 0; n < WN; ++n) {
            const int64_t item = item0 + 32 * n;
            if (item >= n_items) continue;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int r = row0 + 32 * m + 8 * (e >> 2) + (e & 3);
                if (r < a.rows) a.out_f32[(int64_t)r * a.out_row_stride + item] = acc[m][n][e];
            }
        }
}

template <int GM, int GN, int WM, int WN>
constexpr size_t tile_lds_bytes() { return (size_t)2 * (32 * GM * WM + 32 * GN * WN) * kRowB; }

// more than 64 KiB of dynamic LDS needs an explicit opt-in per kernel instance and device
template <int GM, int GN, int WM, int WN, bool PIPE>
hipError_t opt_in_lds() {
    if (tile_lds_bytes<GM, GN, WM, WN>() <= 64 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&tile_mfma_kernel<GM, GN, WM, WN, PIPE>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)tile_lds_bytes<GM, GN, WM, WN>());
}

template <int GM, int GN, int WM, int WN, bool PIPE>
hipError_t launch_tile(const GemvArgs& a, hipStream_t stream) {
    constexpr int TM = 32 * GM * WM, TN = 32 * GN * WN;
    const int64_t RT = (a.rows + TM - 1) / TM;
    const int64_t IT = (a.n_items + TN - 1) / TN;
    const int64_t groups = (IT + kXcds - 1) / kXcds;            // item tiles per XCD, rounded up
    const int64_t bx = groups * RT * kXcds;
    if (bx > 0x7fffffffLL) return hipErrorInvalidValue;         // more tiles than a grid dimension holds
    const size_t lds = tile_lds_bytes<GM, GN, WM, WN>();     // above 64 KiB: opted in by configure_tile_mfma_lds()
    hipLaunchKernelGGL((tile_mfma_kernel<GM, GN, WM, WN, PIPE>), dim3((unsigned)bx), dim3(64 * GM * GN), lds, stream, a);
    return hipGetLastError();
}

}  // namespace

// every instance launch_tile_mfma can pick, on the current device (called once per device, outside any
// stream capture, by the library's device set-up)
hipError_t configure_tile_mfma_lds() {
    hipError_t e = opt_in_lds<2, 2, 2, 2, false>();
    if (e == hipSuccess) e = opt_in_lds<2, 4, 4, 2, true>();
    if (e == hipSuccess) e = opt_in_lds<2, 2, 2, 2, true>();
    return e;
}

hipError_t launch_tile_mfma(const GemvArgs& a, hipStream_t stream) {
    if (a.n_items <= 0 || a.rows <= 0) return hipSuccess;
    // Up to 128 hidden rows the work is bound by streaming M once: small tiles, two workgroups per
    // CU.  Beyond that the 256 x 256 tile halves the operand traffic per multiply-add -- unless rounding
    // the row count up to 256s would add a whole idle half-tile that 128-row tiles avoid.
    if (a.rows <= 128) return launch_tile<2, 2, 2, 2, false>(a, stream);
    const int pad256 = (a.rows + 255) / 256 * 256, pad128 = (a.rows + 127) / 128 * 128;
    if (pad256 == pad128) return launch_tile<2, 4, 4, 2, true>(a, stream);
    return launch_tile<2, 2, 2, 2, true>(a, stream);
}

}  // namespace sv
