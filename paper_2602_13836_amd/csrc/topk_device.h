// Subset softmax and draft top-kd of one row by one workgroup of 1024 threads
// (Section 3.3, q_K = softmax(z'); inference "Top-k" draft tokens).
//
// kd is tiny next to k, so nothing is sorted:
//   1. every thread turns its logits into order-preserving 32-bit keys and takes their maximum;
//      a 16-lane DPP row reduction gives 64 "row maxima" per workgroup;
//   2. the kd-th largest of those 64 maxima is a lower bound L of the kd-th largest logit of the
//      whole row (at least kd different rows hold an element >= L), found by rank counting;
//   3. only the few elements >= L (about kd of them on untied data) are appended to an LDS list
//      as 64-bit keys (logit order, then smaller token id), while the softmax denominator is
//      summed over everything in the same pass;
//   4. the first wavefront ranks the list by counting and writes rank t < kd to output slot t.
// If ties push more than CAP elements over L, a slower exact path extracts the winners one by
// one ("largest key below the previous winner"), so the result is exact for any input.
#pragma once
#include "sv_device.h"
#include "sv_launch.h"

namespace sv {
namespace topk {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kRows16 = kThreads / 16;       // DPP rows per workgroup = 64 = SPECVOCAB_MAX_KD
constexpr int kCap = 512;                    // candidate list capacity

// M > 0: each thread keeps M (key, token) pairs in registers (k <= M * 1024).
// M == 0: the row is streamed from global memory (L2) in every pass (any k).
// VEC (M % 4 == 0, k % 4 == 0, 16-byte aligned rows): a thread owns groups of 4 consecutive
// elements and moves them with 128-bit loads and stores.
// Long rows (M >= kDeferFrom): one compute unit pulls a long row slowly, so the token ids -- half the
// bytes -- are not read up front: candidates carry their position and only the few of them fetch
// their token (one more round trip, a quarter of a megabyte less at k = 32768).
constexpr int kDeferFrom = 16;
// PICK (registers, tokens read up front): the row's logits are picked from the product over the union of the rows' sets -- entry j is
// a.pick_zu[r, a.pick_pos[idx[j]]] -- and written out as the logits row on the way.
template <int M, bool VEC, bool PICK = false>
__device__ __forceinline__ void softmax_topk_block(const TopkArgs& a, const int64_t r) {
    static_assert(!PICK || (M > 0 && M < kDeferFrom), "the picking form keeps logits and tokens in registers");
    __shared__ __attribute__((aligned(16))) uint32_t s_rowmax[kRows16];   // exact row maxima
    __shared__ __attribute__((aligned(16))) uint32_t s_rowtag[kRows16];   // made unique: low 6 bits = 63 - row
    __shared__ uint64_t s_cand[kCap];
    __shared__ uint64_t s_round[kWaves];
    __shared__ float s_part[kWaves];
    __shared__ uint32_t s_count;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int64_t k = a.k;
    const int kd = a.kd;
    const float* z = a.logits + r * k;
    const int32_t* idx = a.idx + r * a.idx_row_stride;

    if (tid == 0) s_count = 0u;

    // ---- 1. keys and row maxima
    constexpr bool DEFER = M >= kDeferFrom;
    uint32_t key[M > 0 ? M : 1];
    int32_t tk[M > 0 && !DEFER ? M : 1];
    uint32_t lmax = 0u;
    // position of the thread's i-th element in the row
    auto pos_of = [&](int i) -> int32_t {                 // < M * 1024
        if constexpr (VEC) return (i / 4) * (4 * kThreads) + 4 * tid + (i & 3);
        else return i * kThreads + tid;
    };
    if constexpr (M > 0 && VEC) {
#pragma unroll
        for (int q = 0; q < M / 4; ++q) {
            const int64_t j0 = (int64_t)q * (4 * kThreads) + 4 * tid;
            u32x4 zz = zero16(), tt = zero16();
            if (j0 < k) {
                if constexpr (PICK) {
                    tt = *reinterpret_cast<const u32x4*>(idx + j0);
                    const float* zu = a.pick_zu + r * a.pick_zu_stride;
                    uint32_t at[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) at[e] = a.pick_pos[tt[e]];
#pragma unroll
                    for (int e = 0; e < 4; ++e) zz[e] = __float_as_uint(zu[at[e]]);
                    *reinterpret_cast<u32x4*>(a.pick_logits_out + r * k + j0) = zz;
                } else {
                    zz = *reinterpret_cast<const u32x4*>(z + j0);
                    if constexpr (!DEFER) tt = *reinterpret_cast<const u32x4*>(idx + j0);
                }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                key[q * 4 + e] = j0 < k ? f32_to_ord(__uint_as_float(zz[e])) : 0u;
                if constexpr (!DEFER) tk[q * 4 + e] = (int32_t)tt[e];
                lmax = key[q * 4 + e] > lmax ? key[q * 4 + e] : lmax;
            }
        }
    } else if constexpr (M > 0) {
#pragma unroll
        for (int i = 0; i < M; ++i) {
            const int64_t j = (int64_t)i * kThreads + tid;
            if constexpr (PICK) {
                tk[i] = j < k ? idx[j] : 0;
                if (j < k) {
                    const float f = a.pick_zu[r * a.pick_zu_stride + a.pick_pos[tk[i]]];
                    a.pick_logits_out[r * k + j] = f;
                    key[i] = f32_to_ord(f);
                } else {
                    key[i] = 0u;
                }
            } else {
                key[i] = j < k ? f32_to_ord(z[j]) : 0u;      // 0 = no element (finite keys are larger)
                if constexpr (!DEFER) tk[i] = j < k ? idx[j] : 0;
            }
            lmax = key[i] > lmax ? key[i] : lmax;
        }
    } else {
        for (int64_t j = tid; j < k; j += kThreads) {
            const uint32_t kk = f32_to_ord(z[j]);
            lmax = kk > lmax ? kk : lmax;
        }
    }
    {
        uint32_t o;
        o = dpp_u32<DPP_QUAD_1032>(lmax); lmax = o > lmax ? o : lmax;
        o = dpp_u32<DPP_QUAD_2301>(lmax); lmax = o > lmax ? o : lmax;
        o = dpp_u32<DPP_ROW_HALF_MIRROR>(lmax); lmax = o > lmax ? o : lmax;
        o = dpp_u32<DPP_ROW_MIRROR>(lmax); lmax = o > lmax ? o : lmax;
    }
    if ((lane & 15) == 0) {
        const int row = tid >> 4;
        s_rowmax[row] = lmax;
        s_rowtag[row] = (lmax & ~63u) | (uint32_t)(63 - row);
    }
    __syncthreads();

    // ---- 2. threshold L (kd-th largest row maximum, low bits cleared) and the row maximum.
    // Every wavefront computes them redundantly from LDS: no second barrier.
    const uint32_t zmaxkey = wave_max_u32(s_rowmax[lane]);
    const uint32_t mytag = s_rowtag[lane];
    uint32_t cnt = 0u;
#pragma unroll
    for (int q = 0; q < kRows16 / 4; ++q) {
        const u32x4 v = reinterpret_cast<const u32x4*>(s_rowtag)[q];
#pragma unroll
        for (int e = 0; e < 4; ++e) cnt += v[e] > mytag;
    }
    const uint64_t pick = __builtin_amdgcn_ballot_w64(cnt == (uint32_t)(kd - 1));   // exactly one lane
    const int src = __ffsll((long long)pick) - 1;
    uint32_t L = (uint32_t)__builtin_amdgcn_readlane((int)mytag, src) & ~63u;
    if (L == 0u) L = 1u;                                      // never admit the "no element" key
    // padding slots carry -inf (probability 0); a row of nothing else has all probabilities 0
    constexpr uint32_t kNegInfKey = 0x007FFFFFu;              // f32_to_ord(-inf)
    const bool empty = zmaxkey <= kNegInfKey;
    const float zmax = empty ? 0.0f : ord_to_f32(zmaxkey);

    // ---- 3. candidates >= L into LDS; softmax denominator over everything
    float part = 0.0f;
    auto visit = [&](uint32_t kk, int32_t tok) {
        part += __expf(ord_to_f32(kk) - zmax);
        if (kk >= L) {
            const uint32_t pos = atomicAdd(&s_count, 1u);
            if (pos < (uint32_t)kCap) s_cand[pos] = ((uint64_t)kk << 32) | (uint32_t)(~(uint32_t)tok);
        }
    };
    if constexpr (M > 0) {
#pragma unroll
        for (int i = 0; i < M; ++i) {
            if (key[i] != 0u) {
                if constexpr (DEFER) visit(key[i], pos_of(i));              // the token follows below
                else visit(key[i], tk[i]);
            }
        }
    } else {
        for (int64_t j = tid; j < k; j += kThreads) visit(f32_to_ord(z[j]), idx[j]);
    }
    part = wave_sum(part);
    if (lane == 0) s_part[wave] = part;
    __syncthreads();

    float tot = 0.0f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) tot += s_part[w];
    const float inv = empty ? 0.0f : 1.0f / tot;
    const uint32_t n = s_count;
    auto prob_of = [&](uint64_t k64) {                        // keys at or below -inf: padding or no entry at all
        return (uint32_t)(k64 >> 32) <= kNegInfKey ? 0.0f : __expf(key_value(k64) - zmax) * inv;
    };

    if (n <= (uint32_t)kCap) {
        if constexpr (DEFER) {
            // the candidates' tokens: only the first wavefront goes on from here, and it sees its own LDS writes
            if (wave == 0) {
                for (uint32_t c = lane; c < n; c += 64) {
                    const uint64_t e = s_cand[c];
                    const int32_t tok = idx[(uint32_t)(~(uint32_t)e)];
                    s_cand[c] = (e & 0xFFFFFFFF00000000ull) | (uint32_t)(~(uint32_t)tok);
                }
            }
        }
        // ---- 4. rank the candidates by counting; ranks are unique (position breaks exact ties)
        if (wave == 0 && n <= 64u) {
            // the usual case: one candidate per lane, the others arrive by lane broadcast (no LDS latency)
            const uint64_t mine = (uint32_t)lane < n ? s_cand[lane] : 0ull;
            uint32_t rank = 0u;
            for (uint32_t j = 0; j < n; ++j) {
                const uint64_t o = readlane_u64(mine, (int)j);
                rank += (o > mine) || (o == mine && j < (uint32_t)lane);
            }
            if ((uint32_t)lane < n && rank < (uint32_t)kd) {
                a.tok_out[r * kd + rank] = key_token(mine);
                a.prob_out[r * kd + rank] = prob_of(mine);
            }
        } else if (wave == 0) {
            for (uint32_t i = lane; i < n; i += 64) {
                const uint64_t mine = s_cand[i];
                uint32_t rank = 0u;
                for (uint32_t j = 0; j < n; ++j) {
                    const uint64_t o = s_cand[j];
                    rank += (o > mine) || (o == mine && j < i);
                }
                if (rank < (uint32_t)kd) {
                    a.tok_out[r * kd + rank] = key_token(mine);
                    a.prob_out[r * kd + rank] = prob_of(mine);
                }
            }
        }
    } else {
        // ---- slow exact path: kd rounds of "largest 64-bit key below the previous winner"
        uint64_t prev = ~0ull;
        for (int t = 0; t < kd; ++t) {
            uint64_t cand = 0ull;
            auto consider = [&](uint32_t kk, int32_t tok) {
                const uint64_t k64 = ((uint64_t)kk << 32) | (uint32_t)(~(uint32_t)tok);
                if (k64 < prev && k64 > cand) cand = k64;
            };
            if constexpr (M > 0 && !DEFER) {
#pragma unroll
                for (int i = 0; i < M; ++i)
                    if (key[i] != 0u) consider(key[i], tk[i]);
            } else {
                for (int64_t j = tid; j < k; j += kThreads) consider(f32_to_ord(z[j]), idx[j]);
            }
            cand = wave_max_u64(cand);
            if (lane == 0) s_round[wave] = cand;
            __syncthreads();
            uint64_t best = 0ull;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) best = umax64(best, s_round[w]);
            __syncthreads();
            if (tid == 0) {
                a.tok_out[r * kd + t] = key_token(best);
                a.prob_out[r * kd + t] = prob_of(best);
            }
            prev = best;
        }
    }

    if (a.probs_full_out) {
        float* q = a.probs_full_out + r * k;
        if constexpr (M > 0 && VEC) {
#pragma unroll
            for (int g = 0; g < M / 4; ++g) {
                const int64_t j0 = (int64_t)g * (4 * kThreads) + 4 * tid;
                if (j0 < k) {
                    u32x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        o[e] = __float_as_uint(__expf(ord_to_f32(key[g * 4 + e]) - zmax) * inv);
                    *reinterpret_cast<u32x4*>(q + j0) = o;
                }
            }
        } else if constexpr (M > 0) {
#pragma unroll
            for (int i = 0; i < M; ++i) {
                const int64_t j = (int64_t)i * kThreads + tid;
                if (j < k) q[j] = __expf(ord_to_f32(key[i]) - zmax) * inv;
            }
        } else {
            for (int64_t j = tid; j < k; j += kThreads) q[j] = __expf(ord_to_f32(f32_to_ord(z[j])) - zmax) * inv;
        }
    }
}

}  // namespace topk
}  // namespace sv
