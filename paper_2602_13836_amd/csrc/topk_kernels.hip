// Subset softmax and draft top-kd (Section 3.3, q_K = softmax(z'); inference "Top-k" draft tokens).
//
// One workgroup per row.  Every (logit, token id) pair becomes one 64-bit key whose unsigned order
// is "larger logit first, then smaller token id", so a top-kd is kd rounds of "largest key below
// the previous winner": no element is ever marked or moved.  Each wavefront extracts the top-kd
// of its own share with DPP reductions only (no barrier), the wave lists meet in LDS, and the
// first wavefront extracts the row's top-kd from them.  The row maximum is the first winner; the
// softmax denominator is one more pass over the keys held in registers.
#include "sv_device.h"
#include "sv_launch.h"

namespace sv {

namespace {

constexpr int kMaxKd = 64;

// M > 0: each thread keeps M keys in registers (k <= M * blockDim.x).  M == 0: keys are rebuilt
// from global memory on every pass (any k).
template <int M>
__global__ __launch_bounds__(1024) void softmax_topk_kernel(const TopkArgs a) {
    __shared__ uint64_t s_cand[16 * kMaxKd];
    __shared__ float s_part[16];
    __shared__ float s_bcast[2];

    const int tid = threadIdx.x;
    const int T = blockDim.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int nw = T >> 6;
    const int64_t r = blockIdx.x;
    const int64_t k = a.k;
    const int kd = a.kd;
    const float* z = a.logits + r * k;
    const int32_t* idx = a.idx + r * a.idx_row_stride;

    uint64_t key[M > 0 ? M : 1];
    if constexpr (M > 0) {
#pragma unroll
        for (int i = 0; i < M; ++i) {
            const int64_t j = (int64_t)i * T + tid;
            key[i] = j < k ? make_key(z[j], idx[j]) : 0ull;
        }
    }

    // ---- per-wave top-kd: lane t ends up holding the wave's t-th best key
    uint64_t prev = ~0ull, mine = 0ull;
    for (int t = 0; t < kd; ++t) {
        uint64_t cand = 0ull;
        if constexpr (M > 0) {
#pragma unroll
            for (int i = 0; i < M; ++i) {
                const uint64_t kk = key[i];
                if (kk < prev && kk > cand) cand = kk;
            }
        } else {
            for (int64_t j = tid; j < k; j += T) {
                const uint64_t kk = make_key(z[j], idx[j]);
                if (kk < prev && kk > cand) cand = kk;
            }
        }
        const uint64_t wm = wave_max_u64(cand);
        if (lane == t) mine = wm;
        prev = wm;
    }
    if (lane < kd) s_cand[wave * kd + lane] = mine;
    __syncthreads();

    // ---- merge: the first wave extracts the row's top-kd from the nw * kd candidates
    uint64_t best = 0ull;
    if (wave == 0) {
        const int n = nw * kd;
        prev = ~0ull;
        for (int t = 0; t < kd; ++t) {
            uint64_t cand = 0ull;
            for (int i = lane; i < n; i += 64) {
                const uint64_t kk = s_cand[i];
                if (kk < prev && kk > cand) cand = kk;
            }
            const uint64_t wm = wave_max_u64(cand);
            if (lane == t) best = wm;
            prev = wm;
        }
        if (lane == 0) s_bcast[0] = key_value(best);
    }
    __syncthreads();
    const float zmax = s_bcast[0];

    // ---- softmax denominator
    float part = 0.0f;
    if constexpr (M > 0) {
#pragma unroll
        for (int i = 0; i < M; ++i)
            if (key[i] != 0ull) part += expf(key_value(key[i]) - zmax);
    } else {
        for (int64_t j = tid; j < k; j += T) part += expf((z[j] + 0.0f) - zmax);
    }
    part = wave_sum(part);
    if (lane == 0) s_part[wave] = part;
    __syncthreads();
    if (tid == 0) {
        float tot = 0.0f;
        for (int w = 0; w < nw; ++w) tot += s_part[w];
        s_bcast[1] = tot;
    }
    __syncthreads();
    const float inv = 1.0f / s_bcast[1];

    if (wave == 0 && lane < kd) {
        a.tok_out[r * kd + lane] = key_token(best);
        a.prob_out[r * kd + lane] = expf(key_value(best) - zmax) * inv;
    }
    if (a.probs_full_out) {
        float* q = a.probs_full_out + r * k;
        if constexpr (M > 0) {
#pragma unroll
            for (int i = 0; i < M; ++i) {
                const int64_t j = (int64_t)i * T + tid;
                if (j < k) q[j] = expf(key_value(key[i]) - zmax) * inv;
            }
        } else {
            for (int64_t j = tid; j < k; j += T) q[j] = expf((z[j] + 0.0f) - zmax) * inv;
        }
    }
}

template <int M>
hipError_t launch_m(const TopkArgs& a, int threads, hipStream_t stream) {
    hipLaunchKernelGGL((softmax_topk_kernel<M>), dim3((unsigned)a.rows), dim3(threads), 0, stream, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_softmax_topk(const TopkArgs& a, hipStream_t stream) {
    const int threads = a.k > 2048 ? 1024 : 256;
    const int64_t m = (a.k + threads - 1) / threads;
    if (m <= 1) return launch_m<1>(a, threads, stream);
    if (m <= 2) return launch_m<2>(a, threads, stream);
    if (m <= 4) return launch_m<4>(a, threads, stream);
    if (m <= 8) return launch_m<8>(a, threads, stream);
    if (m <= 16) return launch_m<16>(a, threads, stream);
    if (m <= 32) return launch_m<32>(a, threads, stream);
    return launch_m<0>(a, 1024, stream);
}

}  // namespace sv
