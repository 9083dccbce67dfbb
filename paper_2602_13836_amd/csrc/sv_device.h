// Device-side helpers shared by the gfx950 kernels: storage formats, 16-byte dot products,
// DPP wave reductions and the order-preserving float key used by every top-k.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sv {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

enum { DT_F32 = 0, DT_BF16 = 1 };

__device__ __forceinline__ u32x4 zero16() { return u32x4{0u, 0u, 0u, 0u}; }

// streaming 16-byte load: the gathered rows are read once per step and need not stay in L2
template <bool NT>
__device__ __forceinline__ u32x4 load16(const u32x4* p) {
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

// acc + <w, x> over the 16 bytes held in w and x (8 bf16 pairs or 4 float32 pairs), fp32 accumulate.
template <int DT>
__device__ __forceinline__ float dot16(const u32x4 w, const u32x4 x, float acc) {
    if constexpr (DT == DT_BF16) {
        // v_dot2_f32_bf16: both products of a 32-bit word and the sum in one instruction instead of two shifts, two
        // masks and two fused multiply-adds (products of bf16 are exact in float32; the sum rounds to within an
        // ulp of the fused chain: 12 of 32768 random words differed, by one ulp, none on integers).
        // The words go through scalars first: a bit cast applied to an element of the vector types made the
        // compiler use element 0 four times.
        typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t wi = w[i], xi = x[i];
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, wi), __builtin_bit_cast(bf16x2_t, xi), acc,
                                                  false);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) acc = fmaf(__uint_as_float(w[i]), __uint_as_float(x[i]), acc);
    }
    return acc;
}

// float32 -> bfloat16 bits, round-to-nearest-even (finite inputs)
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) {
    uint32_t u = __float_as_uint(x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// ---- DPP lane exchange ------------------------------------------------------------------
// dpp_ctrl encodings of the CDNA ISA
constexpr int DPP_QUAD_1032 = 0xB1;        // quad_perm:[1,0,3,2]
constexpr int DPP_QUAD_2301 = 0x4E;        // quad_perm:[2,3,0,1]
constexpr int DPP_ROW_HALF_MIRROR = 0x141;
constexpr int DPP_ROW_MIRROR = 0x140;

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, true);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
    return __uint_as_float(dpp_u32<CTRL>(__float_as_uint(x)));
}
template <int CTRL>
__device__ __forceinline__ uint64_t dpp_u64(uint64_t x) {
    uint32_t lo = dpp_u32<CTRL>((uint32_t)x), hi = dpp_u32<CTRL>((uint32_t)(x >> 32));
    return ((uint64_t)hi << 32) | lo;
}

// sum over the 16 lanes of a DPP row; every lane of the row ends with the row's sum
__device__ __forceinline__ float row16_sum(float x) {
    x += dpp_f32<DPP_QUAD_1032>(x);
    x += dpp_f32<DPP_QUAD_2301>(x);
    x += dpp_f32<DPP_ROW_HALF_MIRROR>(x);
    x += dpp_f32<DPP_ROW_MIRROR>(x);
    return x;
}

__device__ __forceinline__ float readlane_f32(float x, int lane) {
    return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(x), lane));
}

// sum over all 64 lanes, result uniform across the wave. All lanes must be active.
__device__ __forceinline__ float wave_sum(float x) {
    x = row16_sum(x);
    return (readlane_f32(x, 0) + readlane_f32(x, 16)) + (readlane_f32(x, 32) + readlane_f32(x, 48));
}

// max over all 64 lanes, result uniform across the wave. All lanes must be active.
__device__ __forceinline__ float wave_max_f32(float x) {
    x = fmaxf(x, dpp_f32<DPP_QUAD_1032>(x));
    x = fmaxf(x, dpp_f32<DPP_QUAD_2301>(x));
    x = fmaxf(x, dpp_f32<DPP_ROW_HALF_MIRROR>(x));
    x = fmaxf(x, dpp_f32<DPP_ROW_MIRROR>(x));
    return fmaxf(fmaxf(readlane_f32(x, 0), readlane_f32(x, 16)), fmaxf(readlane_f32(x, 32), readlane_f32(x, 48)));
}

__device__ __forceinline__ uint64_t umax64(uint64_t a, uint64_t b) { return a > b ? a : b; }

__device__ __forceinline__ uint64_t readlane_u64(uint64_t x, int lane) {
    uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, lane);
    uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), lane);
    return ((uint64_t)hi << 32) | lo;
}

// max over all 64 lanes, result uniform across the wave. All lanes must be active.
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t x) {
    x = umax64(x, dpp_u64<DPP_QUAD_1032>(x));
    x = umax64(x, dpp_u64<DPP_QUAD_2301>(x));
    x = umax64(x, dpp_u64<DPP_ROW_HALF_MIRROR>(x));
    x = umax64(x, dpp_u64<DPP_ROW_MIRROR>(x));
    return umax64(umax64(readlane_u64(x, 0), readlane_u64(x, 16)),
                  umax64(readlane_u64(x, 32), readlane_u64(x, 48)));
}

__device__ __forceinline__ uint32_t umax32(uint32_t a, uint32_t b) { return a > b ? a : b; }

// max over all 64 lanes, result uniform across the wave. All lanes must be active.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x) {
    x = umax32(x, dpp_u32<DPP_QUAD_1032>(x));
    x = umax32(x, dpp_u32<DPP_QUAD_2301>(x));
    x = umax32(x, dpp_u32<DPP_ROW_HALF_MIRROR>(x));
    x = umax32(x, dpp_u32<DPP_ROW_MIRROR>(x));
    const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)x, 0), b = (uint32_t)__builtin_amdgcn_readlane((int)x, 16);
    const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)x, 32), d = (uint32_t)__builtin_amdgcn_readlane((int)x, 48);
    return umax32(umax32(a, b), umax32(c, d));
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t x) {
    x += dpp_u32<DPP_QUAD_1032>(x);
    x += dpp_u32<DPP_QUAD_2301>(x);
    x += dpp_u32<DPP_ROW_HALF_MIRROR>(x);
    x += dpp_u32<DPP_ROW_MIRROR>(x);
    return (uint32_t)__builtin_amdgcn_readlane((int)x, 0) + (uint32_t)__builtin_amdgcn_readlane((int)x, 16) +
           (uint32_t)__builtin_amdgcn_readlane((int)x, 32) + (uint32_t)__builtin_amdgcn_readlane((int)x, 48);
}

// ---- wave-wide inclusive scans on DPP row shifts (a shuffle-based scan costs six LDS-path round trips)
constexpr int DPP_ROW_SHR1 = 0x111, DPP_ROW_SHR2 = 0x112, DPP_ROW_SHR4 = 0x114, DPP_ROW_SHR8 = 0x118;
constexpr int DPP_ROW_SHL1 = 0x101, DPP_ROW_SHL2 = 0x102, DPP_ROW_SHL4 = 0x104, DPP_ROW_SHL8 = 0x108;

// sum over the lanes with a lower or equal index.  All lanes must be active.
__device__ __forceinline__ uint32_t wave_prefix_inclusive_u32(uint32_t x) {
    x += dpp_u32<DPP_ROW_SHR1>(x);            // lanes shifted in from outside a 16-lane row read 0
    x += dpp_u32<DPP_ROW_SHR2>(x);
    x += dpp_u32<DPP_ROW_SHR4>(x);
    x += dpp_u32<DPP_ROW_SHR8>(x);            // inclusive within each row of 16
    const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)x, 15);
    const uint32_t r1 = (uint32_t)__builtin_amdgcn_readlane((int)x, 31);
    const uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)x, 47);
    const int row = (threadIdx.x & 63) >> 4;
    return x + (row >= 1 ? r0 : 0u) + (row >= 2 ? r1 : 0u) + (row >= 3 ? r2 : 0u);
}
// sum over the lanes with a higher or equal index.  All lanes must be active.
__device__ __forceinline__ uint32_t wave_suffix_inclusive_u32(uint32_t x) {
    x += dpp_u32<DPP_ROW_SHL1>(x);
    x += dpp_u32<DPP_ROW_SHL2>(x);
    x += dpp_u32<DPP_ROW_SHL4>(x);
    x += dpp_u32<DPP_ROW_SHL8>(x);
    const uint32_t r1 = (uint32_t)__builtin_amdgcn_readlane((int)x, 16);
    const uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)x, 32);
    const uint32_t r3 = (uint32_t)__builtin_amdgcn_readlane((int)x, 48);
    const int row = (threadIdx.x & 63) >> 4;
    return x + (row <= 0 ? r1 : 0u) + (row <= 1 ? r2 : 0u) + (row <= 2 ? r3 : 0u);
}

// ---- block-wide exclusive scans, one value per thread, WAVES wavefronts per workgroup -------
// s_w: WAVES words of LDS.  Every thread of the workgroup must call.
// sum over the threads with a LOWER index
template <int WAVES>
__device__ __forceinline__ uint32_t block_prefix_exclusive(uint32_t x, uint32_t* s_w) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t incl = wave_prefix_inclusive_u32(x);
    __syncthreads();                                   // s_w may still be read from an earlier scan
    if (lane == 63) s_w[wave] = incl;
    __syncthreads();
    // all WAVES partial sums are read at once (a loop up to `wave` would wait for one LDS read after the other)
    uint32_t lower = 0;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
        const uint32_t v = s_w[w];
        lower += w < wave ? v : 0u;
    }
    return incl - x + lower;
}
// sum over the threads with a HIGHER index
template <int WAVES>
__device__ __forceinline__ uint32_t block_suffix_exclusive(uint32_t x, uint32_t* s_w) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t incl = wave_suffix_inclusive_u32(x);
    __syncthreads();
    if (lane == 0) s_w[wave] = incl;
    __syncthreads();
    uint32_t higher = 0;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
        const uint32_t v = s_w[w];
        higher += w > wave ? v : 0u;
    }
    return incl - x + higher;
}

// ---- order-preserving keys ----------------------------------------------------------------
// a > b (floats, -0 == +0)  <=>  ord(a) > ord(b) (unsigned); finite inputs map to keys >= 0x00800000
__device__ __forceinline__ uint32_t f32_to_ord(float f) {
    uint32_t u = __float_as_uint(f + 0.0f);   // -0.0 + 0.0 = +0.0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float ord_to_f32(uint32_t k) {
    uint32_t u = (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k;
    return __uint_as_float(u);
}
// (value, token) -> 64-bit key: larger value first, equal values -> smaller token id first
__device__ __forceinline__ uint64_t make_key(float z, int32_t tok) {
    return ((uint64_t)f32_to_ord(z) << 32) | (uint32_t)(~(uint32_t)tok);
}
__device__ __forceinline__ int32_t key_token(uint64_t k) { return (int32_t)(~(uint32_t)k); }
__device__ __forceinline__ float key_value(uint64_t k) { return ord_to_f32((uint32_t)(k >> 32)); }

}  // namespace sv
