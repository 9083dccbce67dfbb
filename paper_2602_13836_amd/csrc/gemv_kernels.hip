// Row-gather matrix-vector kernels (Section 3.3 Step 3 and, with no index list, Section 3.1).
//
// One wavefront owns one (or RPI) whole rows of the matrix at a time: the 64 lanes read the row
// as consecutive 16-byte units (one global_load_dwordx4 per 1 KiB), so every byte of a gathered
// row is fetched exactly once and in full cache lines.  Products are accumulated per lane in
// float32 and reduced across the wave with DPP row operations.
//   gemv_rows_once_kernel   rows of 3 to 16 KiB: one row per wavefront, the hidden-state row in LDS
//   gemv_rows_kernel        shorter rows: several rows per wavefront and a loop, the hidden-state row
//                           in registers in the same lane layout for the whole life of the wave
//   gemv_long_rows_kernel   longer rows, walked in 1 KiB pieces
// An index of -1 (a padding slot of a padded list) reads row 0 and stores -inf: negative indices cost a
// scalar maximum and a select, so all three kernels accept them whether the list is padded or not.
#include <stddef.h>
#include "sv_device.h"
#include "sv_launch.h"

namespace sv {

namespace {

// FULL: every row is exactly NL * 64 16-byte units, so no load needs a bounds check
template <int DT, int NL, int RPI, bool OUT_BF16, bool FULL>
__global__ __launch_bounds__(256) void gemv_rows_kernel(const GemvArgs a) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t r = blockIdx.y;
    const int C = a.chunks;

    const int32_t* idx = a.idx ? a.idx + r * a.idx_row_stride : nullptr;
    const int64_t n = a.n_items;
    const int64_t step = (int64_t)gridDim.x * 4 * RPI;
    int64_t it = ((int64_t)blockIdx.x * 4 + wave) * RPI;

    // Order of the first requests matters for a launch that lasts only microseconds: the hidden-state
    // row is requested first (vector loads, nothing waits for them yet), then the scalar index loads, and
    // the rows of the matrix as soon as the indices arrive -- one dependent round trip, not three.
    const u32x4* xp = reinterpret_cast<const u32x4*>(a.x + r * a.x_row_bytes);
    u32x4 xreg[NL];
#pragma unroll
    for (int c = 0; c < NL; ++c) {
        const int ch = c * 64 + lane;
        xreg[c] = (FULL || ch < C) ? xp[ch] : zero16();
    }
    auto row_of = [&](int64_t item) -> int64_t {          // -1 (a padding slot of a padded list) stays -1
        if (item > n - 1) item = n - 1;               // tail: recompute the last item, never stored
        return idx ? (int64_t)idx[item] : item;
    };
    int64_t row[RPI];
#pragma unroll
    for (int q = 0; q < RPI; ++q) row[q] = row_of(it + q);

    auto load_rows = [&](u32x4 (&w)[RPI][NL]) {
#pragma unroll
        for (int q = 0; q < RPI; ++q) {
            const u32x4* mp = reinterpret_cast<const u32x4*>(a.M + (row[q] < 0 ? 0 : row[q]) * a.m_row_bytes);
#pragma unroll
            for (int c = 0; c < NL; ++c) {
                const int ch = c * 64 + lane;
                w[q][c] = (FULL || ch < C) ? load16<true>(mp + ch) : zero16();
            }
        }
    };
    auto finish = [&](const u32x4 (&w)[RPI][NL]) {
        float acc[RPI];
#pragma unroll
        for (int q = 0; q < RPI; ++q) {
            // four independent partial sums: the 8 NL multiply-adds of a lane do not form one long
            // dependent chain (it would sit in the tail of a launch that lasts only microseconds)
            float part[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int c = 0; c < NL; ++c) part[c & 3] = dot16<DT>(w[q][c], xreg[c], part[c & 3]);
            acc[q] = wave_sum((part[0] + part[1]) + (part[2] + part[3]));
        }
        if (lane == 0) {
#pragma unroll
            for (int q = 0; q < RPI; ++q) {
                if (it + q < n) {
                    if constexpr (OUT_BF16) a.out_bf16[r * a.out_row_stride + it + q] = f32_to_bf16_rne(acc[q]);
                    else a.out_f32[r * a.out_row_stride + it + q] = row[q] < 0 ? -INFINITY : acc[q];
                }
            }
        }
    };

    {   // first items: peeled, so that nothing loop-invariant is computed (and waited for) up front
        u32x4 w[RPI][NL];
        load_rows(w);
        finish(w);
    }
    for (it += step; it < n; it += step) {
#pragma unroll
        for (int q = 0; q < RPI; ++q) row[q] = row_of(it + q);
        u32x4 w[RPI][NL];
        load_rows(w);
        finish(w);
    }

    prepare_scratch(a);     // clear / fill a later kernel's scratch with this launch
}

// One row per wavefront and one wavefront per item, rows of up to NL * 64 units (NL = 4 .. 16).  The
// hidden-state row waits in LDS instead of registers, which halves the registers of a wavefront: all
// wavefronts of a short gather are resident at once, so the index -> row round trip is paid once, and a
// long product simply streams workgroup after workgroup.  Loads are branch-free: units past the end of
// a row are clamped to its last unit and meet zeros in the staged hidden row (FULL: rows of exactly
// NL * 64 units, nothing to clamp -- the address arithmetic in front of the first requests is worth 1 %).
// Wavefronts per workgroup (WAVES): four, or eight for gathers of a few thousand to 16 K rows, where staging the
// hidden row half as often is worth 0.5-1 % (k = 8192: 12.08 -> 11.99 us cold); with fewer rows eight leave
// compute units idle (k = 512: 2.65 -> 3.04 us), with more they lose 1 %; two and sixteen lose everywhere.
// The arguments the first requests need come first and one by one: plain leading arguments are preloaded
// into scalar registers with the wavefront (a struct passed by value is fetched by the first instructions).
// the kernel's argument segment as bytes (the host pass of the compiler only parses this)
__device__ __forceinline__ const char* kernarg_bytes() {
#if defined(__HIP_DEVICE_COMPILE__)
    return (const char*)__builtin_amdgcn_kernarg_segment_ptr();
#else
    return nullptr;
#endif
}
// offset of the argument struct in the kernel's argument segment: three pointers and four 64-bit integers lie
// in front of it (the segment is laid out like a struct of the arguments)
struct OnceArgsLayout {
    const char* x_base;
    const char* m_base;
    const int32_t* idx_base;
    int64_t n, x_row_bytes, m_row_bytes, idx_row_stride;
    GemvArgs a;
};
constexpr int kOnceStructOffset = (int)offsetof(OnceArgsLayout, a);
static_assert(kOnceStructOffset == 56, "gemv_rows_once_kernel reads its last argument at this offset by hand");
template <int DT, int NL, bool OUT_BF16, bool FULL, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void gemv_rows_once_kernel(
    const char* __restrict__ x_base, const char* __restrict__ m_base, const int32_t* __restrict__ idx_base,
    const int64_t n, const int64_t x_row_bytes, const int64_t m_row_bytes, const int64_t idx_row_stride,
    const GemvArgs a) {
    constexpr int kT = WAVES * 64;
    constexpr int kUnits = NL * 64;
    constexpr int kRounds = (kUnits + kT - 1) / kT;
    __shared__ u32x4 s_x[kUnits];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t r = blockIdx.y;
    const int last = FULL ? kUnits - 1 : a.chunks - 1;
    const int64_t it = (int64_t)blockIdx.x * WAVES + wave;

    // request order as in gemv_rows_kernel: hidden row, scalar index, row of the matrix
    const u32x4* xp = reinterpret_cast<const u32x4*>(x_base + r * x_row_bytes);
    u32x4 xs[kRounds];
    int unit[kRounds];
#pragma unroll
    for (int q = 0; q < kRounds; ++q) {
        unit[q] = q * kT + tid < kUnits ? q * kT + tid : kUnits - 1;   // spare threads: the last unit once more
        xs[q] = xp[FULL || unit[q] < last ? unit[q] : last];
    }
    const int64_t item = it < n ? it : n - 1;          // tail: recompute the last item, never stored
    const int64_t row = idx_base ? (int64_t)idx_base[r * idx_row_stride + item] : item;   // -1: a padding slot
    const u32x4* mp = reinterpret_cast<const u32x4*>(m_base + (row < 0 ? 0 : row) * m_row_bytes);
    u32x4 w[NL];
#pragma unroll
    for (int c = 0; c < NL; ++c) {
        const int ch = c * 64 + lane;
        w[c] = load16<true>(mp + (FULL || ch < last ? ch : last));
    }
    __builtin_amdgcn_sched_barrier(0);                 // every row request leaves before anything waits
    // What the end of the kernel needs of the argument struct is fetched only now, by hand: argument loads
    // that the compiler places at the kernel's entry are scalar loads like the one of the index, scalar loads
    // return in any order, so the wait for the index would wait for that cold fetch as well (0.07 us of a
    // 12 us launch).
    const GemvArgs& late = *reinterpret_cast<const GemvArgs*>(kernarg_bytes() + kOnceStructOffset);
    float* late_out_f32 = late.out_f32;
    uint16_t* late_out_bf16 = late.out_bf16;
    int64_t late_out_stride = late.out_row_stride;
    size_t late_zero_words = late.zero_words;
    int64_t late_spread_n = late.spread_n;
    // (pinned to scalar registers here, or the compiler moves each load down to its first use)
    asm volatile("" : "+s"(late_out_f32), "+s"(late_out_bf16), "+s"(late_out_stride), "+s"(late_zero_words), "+s"(late_spread_n));
    __builtin_amdgcn_sched_barrier(0);                 // ... and these requests leave before the first wait too
#pragma unroll
    for (int q = 0; q < kRounds; ++q) s_x[unit[q]] = FULL || unit[q] <= last ? xs[q] : zero16();
    __syncthreads();
    float part[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int c = 0; c < NL; ++c) part[c & 3] = dot16<DT>(w[c], s_x[c * 64 + lane], part[c & 3]);
    const float acc = wave_sum((part[0] + part[1]) + (part[2] + part[3]));
    if (lane == 0 && it < n) {
        if constexpr (OUT_BF16) late_out_bf16[r * late_out_stride + it] = f32_to_bf16_rne(acc);
        else late_out_f32[r * late_out_stride + it] = row < 0 ? -INFINITY : acc;
    }
    if (late_zero_words != 0 || late_spread_n != 0) prepare_scratch(late);   // clear / fill a later kernel's scratch
}

// any row length: the row is walked in 1 KiB pieces, x is re-read (from L2) for every item
template <int DT, bool OUT_BF16>
__global__ __launch_bounds__(256) void gemv_long_rows_kernel(const GemvArgs a) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t r = blockIdx.y;
    const int C = a.chunks;
    prepare_scratch(a);     // clear / fill a later kernel's scratch with this launch
    const u32x4* xp = reinterpret_cast<const u32x4*>(a.x + r * a.x_row_bytes);
    const int32_t* idx = a.idx ? a.idx + r * a.idx_row_stride : nullptr;
    const int64_t n = a.n_items;
    const int64_t step = (int64_t)gridDim.x * 4;
    for (int64_t it = (int64_t)blockIdx.x * 4 + wave; it < n; it += step) {
        const int64_t row = idx ? (int64_t)idx[it] : it;                      // -1: a padding slot
        const u32x4* mp = reinterpret_cast<const u32x4*>(a.M + (row < 0 ? 0 : row) * a.m_row_bytes);
        float acc = 0.0f;
        for (int ch = lane; ch < C; ch += 64) acc = dot16<DT>(load16<true>(mp + ch), xp[ch], acc);
        acc = wave_sum(acc);
        if (lane == 0) {
            if constexpr (OUT_BF16) a.out_bf16[r * a.out_row_stride + it] = f32_to_bf16_rne(acc);
            else a.out_f32[r * a.out_row_stride + it] = row < 0 ? -INFINITY : acc;
        }
    }
}

// debug aid: counts the entries of idx outside [0, V)
__device__ unsigned int g_bad_indices;

__global__ __launch_bounds__(256) void check_indices_kernel(const int32_t* idx, int64_t n, int64_t V,
                                                            int64_t lowest, int64_t sorted_row_len) {
    unsigned bad = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t v = idx[i];
        bad += (v < lowest) || (v >= V);
        if (sorted_row_len > 0 && i % sorted_row_len != 0) bad += v < (int64_t)idx[i - 1];   // a declared order
    }
    if (bad) atomicAdd(&g_bad_indices, bad);
}

// index lists with padding slots (-1 = no token): a clean copy for the kernels that follow addresses ...
__global__ __launch_bounds__(256) void pad_clean_kernel(const int32_t* idx, int64_t n, int32_t* clean) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int32_t v = idx[i];
        clean[i] = v < 0 ? 0 : v;
    }
}
// ... and -inf for the logits of the padding slots afterwards
__global__ __launch_bounds__(256) void pad_mask_kernel(const int32_t* idx, int64_t idx_row_stride, int64_t k,
                                                       float* logits) {
    const int64_t r = blockIdx.y;                         // (no division of a pair number by k per entry)
    const int32_t* list = idx + r * idx_row_stride;
    float* z = logits + r * k;
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < k; j += (int64_t)gridDim.x * blockDim.x)
        if (list[j] < 0) z[j] = -INFINITY;
}

// dst[j, :] = M[idx[j], :]: one wavefront per row, 16 bytes per lane and step
__global__ __launch_bounds__(256) void materialize_rows_kernel(const char* M, int64_t m_row_bytes,
                                                               const int32_t* idx, int64_t n_rows, int chunks,
                                                               char* dst) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t step = (int64_t)gridDim.x * 4;
    for (int64_t j = (int64_t)blockIdx.x * 4 + wave; j < n_rows; j += step) {
        const u32x4* src = reinterpret_cast<const u32x4*>(M + (int64_t)idx[j] * m_row_bytes);
        u32x4* out = reinterpret_cast<u32x4*>(dst + j * (int64_t)chunks * 16);
        for (int ch = lane; ch < chunks; ch += 64) out[ch] = src[ch];
    }
}

template <int DT, int NL, int RPI>
hipError_t launch_rows(const GemvArgs& a, int cus, hipStream_t stream) {
    const int64_t waves = (a.n_items + RPI - 1) / RPI;
    int64_t bx = (waves + 3) / 4;
    const int64_t cap = ((int64_t)cus * 8 + a.rows - 1) / a.rows;
    if (bx > cap) bx = cap;
    if (bx < 1) bx = 1;
    dim3 grid((unsigned)bx, (unsigned)a.rows, 1), block(256, 1, 1);
    const bool full = a.chunks == NL * 64;
    if (a.out_bf16) {
        if (full) hipLaunchKernelGGL((gemv_rows_kernel<DT, NL, RPI, true, true>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((gemv_rows_kernel<DT, NL, RPI, true, false>), grid, block, 0, stream, a);
    } else {
        if (full) hipLaunchKernelGGL((gemv_rows_kernel<DT, NL, RPI, false, true>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((gemv_rows_kernel<DT, NL, RPI, false, false>), grid, block, 0, stream, a);
    }
    return hipGetLastError();
}

template <int DT, int NL, int WAVES>
hipError_t launch_once_w(const GemvArgs& a, hipStream_t stream) {
    dim3 grid((unsigned)((a.n_items + WAVES - 1) / WAVES), (unsigned)a.rows, 1), block(WAVES * 64, 1, 1);
    const bool full = a.chunks == NL * 64;
#define SV_ONCE(OUT, FULLROW)                                                                                       \
    hipLaunchKernelGGL((gemv_rows_once_kernel<DT, NL, OUT, FULLROW, WAVES>), grid, block, 0, stream, a.x, a.M, a.idx, \
                       a.n_items, a.x_row_bytes, a.m_row_bytes, a.idx_row_stride, a)
    if (a.out_bf16) {
        if (full) SV_ONCE(true, true);
        else SV_ONCE(true, false);
    } else {
        if (full) SV_ONCE(false, true);
        else SV_ONCE(false, false);
    }
#undef SV_ONCE
    return hipGetLastError();
}
template <int DT, int NL>
hipError_t launch_once(const GemvArgs& a, hipStream_t stream) {
    if (a.rows == 1 && a.n_items > 2048 && a.n_items <= 16384) return launch_once_w<DT, NL, 8>(a, stream);   // (measured at one row)
    return launch_once_w<DT, NL, 4>(a, stream);
}

template <int DT>
hipError_t launch_dt(const GemvArgs& a, int cus, hipStream_t stream) {
    const int nl = (a.chunks + 63) / 64;
    switch (nl) {
        case 4: return launch_once<DT, 4>(a, stream);
        case 5: return launch_once<DT, 5>(a, stream);
        case 6: return launch_once<DT, 6>(a, stream);
        case 7: return launch_once<DT, 7>(a, stream);
        case 8: return launch_once<DT, 8>(a, stream);
        case 9: return launch_once<DT, 9>(a, stream);
        case 10: return launch_once<DT, 10>(a, stream);
        case 11: return launch_once<DT, 11>(a, stream);
        case 12: return launch_once<DT, 12>(a, stream);
        case 13: return launch_once<DT, 13>(a, stream);
        case 14: return launch_once<DT, 14>(a, stream);
        case 15: return launch_once<DT, 15>(a, stream);
        case 16: return launch_once<DT, 16>(a, stream);
        default: break;
    }
    if (nl <= 1) return launch_rows<DT, 1, 4>(a, cus, stream);
    if (nl <= 2) return launch_rows<DT, 2, 4>(a, cus, stream);
    if (nl <= 3) return launch_rows<DT, 4, 2>(a, cus, stream);
    int64_t bx = (a.n_items + 3) / 4;
    const int64_t cap = ((int64_t)cus * 8 + a.rows - 1) / a.rows;
    if (bx > cap) bx = cap;
    if (bx < 1) bx = 1;
    dim3 grid((unsigned)bx, (unsigned)a.rows, 1), block(256, 1, 1);
    if (a.out_bf16) hipLaunchKernelGGL((gemv_long_rows_kernel<DT, true>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((gemv_long_rows_kernel<DT, false>), grid, block, 0, stream, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_pad_clean(const int32_t* idx, int64_t n, int32_t* clean, hipStream_t stream) {
    int64_t bx = (n + 1023) / 1024;
    if (bx > 2048) bx = 2048;
    if (bx < 1) bx = 1;
    hipLaunchKernelGGL(pad_clean_kernel, dim3((unsigned)bx), dim3(256), 0, stream, idx, n, clean);
    return hipGetLastError();
}

hipError_t launch_pad_mask(const int32_t* idx, int64_t idx_row_stride, int rows, int64_t k, float* logits,
                           hipStream_t stream) {
    int64_t bx = (k + 1023) / 1024;
    if (bx * rows > 4096) bx = (4096 + rows - 1) / rows;
    if (bx < 1) bx = 1;
    hipLaunchKernelGGL(pad_mask_kernel, dim3((unsigned)bx, (unsigned)rows), dim3(256), 0, stream, idx, idx_row_stride, k,
                       logits);
    return hipGetLastError();
}

hipError_t count_bad_indices(const int32_t* idx, int64_t n, int64_t V, bool padded, int64_t sorted_row_len,
                             hipStream_t stream, unsigned* bad_out) {
    const unsigned zero = 0;
    hipError_t e = hipMemcpyToSymbolAsync(HIP_SYMBOL(g_bad_indices), &zero, sizeof zero, 0, hipMemcpyHostToDevice,
                                          stream);
    if (e != hipSuccess) return e;
    int64_t bx = (n + 255) / 256;
    if (bx > 1024) bx = 1024;
    if (bx < 1) bx = 1;
    hipLaunchKernelGGL(check_indices_kernel, dim3((unsigned)bx), dim3(256), 0, stream, idx, n, V,
                       (int64_t)(padded ? -1 : 0), sorted_row_len);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = hipMemcpyFromSymbolAsync(bad_out, HIP_SYMBOL(g_bad_indices), sizeof(unsigned), 0, hipMemcpyDeviceToHost,
                                 stream);
    if (e != hipSuccess) return e;
    return hipStreamSynchronize(stream);
}

hipError_t launch_materialize_rows(const char* M, int64_t m_row_bytes, const int32_t* idx, int64_t n_rows,
                                   int chunks, char* dst, hipStream_t stream) {
    DeviceInfo di;
    hipError_t e = device_info(&di);
    if (e != hipSuccess) return e;
    int64_t bx = (n_rows + 3) / 4;
    if (bx > (int64_t)di.cus * 8) bx = (int64_t)di.cus * 8;
    if (bx < 1) bx = 1;
    hipLaunchKernelGGL(materialize_rows_kernel, dim3((unsigned)bx), dim3(256), 0, stream, M, m_row_bytes, idx, n_rows,
                       chunks, dst);
    return hipGetLastError();
}

hipError_t launch_gemv(int dt, const GemvArgs& a, hipStream_t stream) {
    DeviceInfo di;
    hipError_t e = device_info(&di);
    if (e != hipSuccess) return e;
    if (dt == DT_BF16) return launch_dt<DT_BF16>(a, di.cus, stream);
    return launch_dt<DT_F32>(a, di.cus, stream);
}

}  // namespace sv
