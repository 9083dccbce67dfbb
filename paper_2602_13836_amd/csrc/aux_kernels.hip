// The vocabulary speculator's own distribution over the ENTIRE vocabulary (Section 3.4, training):
//     q_aux = softmax(s),  s = W_vocab (W_down h)
// as natural-log probabilities, in place over the float32 scores:
//     out[r, v] = s[r, v] - ( m_r + log sum_u exp(s[r, u] - m_r) )
// Two launches, because the normaliser is a property of the whole row and a kernel boundary is the
// cheap device-wide synchronisation here:
//   partial   every workgroup reduces its block of the row to (maximum, sum of exp relative to it);
//   apply     every workgroup folds the row's partial pairs into the normaliser itself (at most 1024
//             pairs: cheaper than a launch of its own) and rewrites its block.
// Bandwidth-bound: the scores are read twice and written once.
#include "sv_device.h"
#include "sv_launch.h"

namespace sv {

namespace {

typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kLsThreads = 256;
constexpr int kLsWaves = kLsThreads / 64;
constexpr int kLsMaxBlocks = 1024;              // vocabulary blocks per row

// entries per block: a multiple of 4 * kLsThreads, at most kLsMaxBlocks blocks per row
__host__ __device__ inline int64_t ls_chunk(int64_t V) {
    const int64_t unit = 4 * kLsThreads;
    int64_t rounds = (V + unit * kLsMaxBlocks - 1) / (unit * kLsMaxBlocks);
    if (rounds < 4) rounds = 4;                 // 4096 entries per block at least
    return rounds * unit;
}

// visits this block's entries: thread t owns the four-entry groups t, t + 256, ... of the block
template <typename F>
__device__ __forceinline__ void for_each_group(const float* s, int64_t V, int64_t base, int64_t chunk, F&& f) {
    const bool aligned = (reinterpret_cast<uintptr_t>(s + base) & 15u) == 0;
    for (int64_t g0 = 4 * (int64_t)threadIdx.x; g0 < chunk; g0 += 4 * kLsThreads) {
        const int64_t v0 = base + g0;
        if (v0 >= V) break;
        f32x4_t q;
        int n = 4;
        if (aligned && v0 + 3 < V) {
            q = *reinterpret_cast<const f32x4_t*>(s + v0);
        } else {
            n = (int)(V - v0 < 4 ? V - v0 : 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) q[e] = e < n ? s[v0 + e] : 0.0f;
        }
        f(v0, q, n, aligned && n == 4);
    }
}

__device__ __forceinline__ float block_max(float x, float* s_w) {
    x = wave_max_f32(x);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_w[threadIdx.x >> 6] = x;
    __syncthreads();
    float m = s_w[0];
#pragma unroll
    for (int w = 1; w < kLsWaves; ++w) m = fmaxf(m, s_w[w]);
    return m;
}
__device__ __forceinline__ float block_sum(float x, float* s_w) {
    x = wave_sum(x);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_w[threadIdx.x >> 6] = x;
    __syncthreads();
    float t = 0.0f;
#pragma unroll
    for (int w = 0; w < kLsWaves; ++w) t += s_w[w];
    return t;
}

__global__ __launch_bounds__(kLsThreads) void lse_partial_kernel(const float* s_all, int64_t V, int64_t chunk,
                                                                 float* partial) {
    __shared__ float s_w[kLsWaves];
    const int64_t r = blockIdx.y;
    const float* s = s_all + r * V;
    const int64_t base = (int64_t)blockIdx.x * chunk;
    float m = -INFINITY;
    for_each_group(s, V, base, chunk, [&](int64_t, f32x4_t q, int n, bool) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (e < n) m = fmaxf(m, q[e]);
    });
    m = block_max(m, s_w);
    float acc = 0.0f;
    for_each_group(s, V, base, chunk, [&](int64_t, f32x4_t q, int n, bool) {     // second read: L1 / L2
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (e < n) acc += __expf(q[e] - m);
    });
    acc = block_sum(acc, s_w);
    if (threadIdx.x == 0) {
        float* p = partial + 2 * (r * gridDim.x + blockIdx.x);
        p[0] = m;
        p[1] = acc;
    }
}

__global__ __launch_bounds__(kLsThreads) void lse_apply_kernel(float* s_all, int64_t V, int64_t chunk,
                                                               const float* partial) {
    __shared__ float s_w[kLsWaves];
    const int64_t r = blockIdx.y;
    float* s = s_all + r * V;
    const int nb = (int)gridDim.x;
    const float* p = partial + 2 * r * nb;
    // the row's normaliser from its (max, sum) pairs
    float m = -INFINITY;
    for (int b = threadIdx.x; b < nb; b += kLsThreads) m = fmaxf(m, p[2 * b]);
    m = block_max(m, s_w);
    float acc = 0.0f;
    for (int b = threadIdx.x; b < nb; b += kLsThreads) acc += p[2 * b + 1] * __expf(p[2 * b] - m);
    acc = block_sum(acc, s_w);
    const float lse = m + logf(acc);

    const int64_t base = (int64_t)blockIdx.x * chunk;
    for_each_group(s, V, base, chunk, [&](int64_t v0, f32x4_t q, int n, bool vec) {
        if (vec) {
#pragma unroll
            for (int e = 0; e < 4; ++e) q[e] -= lse;
            *reinterpret_cast<f32x4_t*>(s + v0) = q;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (e < n) s[v0 + e] = q[e] - lse;
        }
    });
}

}  // namespace

size_t log_softmax_ws_floats(int64_t rows, int64_t V) {
    const int64_t chunk = ls_chunk(V);
    return (size_t)rows * (size_t)((V + chunk - 1) / chunk) * 2;
}

hipError_t launch_log_softmax_rows(float* s, int64_t V, int rows, float* partial, hipStream_t stream) {
    const int64_t chunk = ls_chunk(V);
    const dim3 grid((unsigned)((V + chunk - 1) / chunk), (unsigned)rows);
    hipLaunchKernelGGL(lse_partial_kernel, grid, dim3(kLsThreads), 0, stream, s, V, chunk, partial);
    hipLaunchKernelGGL(lse_apply_kernel, grid, dim3(kLsThreads), 0, stream, s, V, chunk, partial);
    return hipGetLastError();
}

}  // namespace sv
