// Stand-alone launch of the subset softmax + draft top-kd: one workgroup per row.
#include "topk_device.h"

namespace sv {

namespace {

using topk::kThreads;

// what the first loads need comes first and as plain arguments: those are preloaded into scalar registers
// with the wavefront, the struct is fetched by instructions
template <int M, bool VEC, bool PICK = false>
__global__ __launch_bounds__(kThreads) void softmax_topk_kernel(const float* logits, const int32_t* idx,
                                                                const int64_t idx_row_stride, const int64_t k,
                                                                const TopkArgs rest) {
    TopkArgs a = rest;
    a.logits = logits;
    a.idx = idx;
    a.idx_row_stride = idx_row_stride;
    a.k = k;
    topk::softmax_topk_block<M, VEC, PICK>(a, blockIdx.x);
}

// the form that picks its logits from the union's product keeps a row in registers
constexpr int kPickMaxM = 8;
bool vec_ok(const TopkArgs& a) {
    return ((reinterpret_cast<uintptr_t>(a.logits) | reinterpret_cast<uintptr_t>(a.idx) |
             reinterpret_cast<uintptr_t>(a.probs_full_out)) & 15u) == 0 && a.k % 4 == 0;
}

template <int M>
hipError_t launch_m(const TopkArgs& a, hipStream_t stream) {
    constexpr bool can_vec = M >= 4 && M % 4 == 0;
    const bool aligned = vec_ok(a);
    if (a.pick_pos != nullptr) {
        if constexpr (M > 0 && M <= kPickMaxM) {
            if ((can_vec && !aligned) || a.pick_logits_out != a.logits) return hipErrorInvalidValue;
            hipLaunchKernelGGL((softmax_topk_kernel<M, can_vec, true>), dim3((unsigned)a.rows), dim3(kThreads), 0, stream,
                               a.logits, a.idx, a.idx_row_stride, a.k, a);
            return hipGetLastError();
        } else {
            return hipErrorInvalidValue;                      // the caller asks softmax_topk_can_pick first
        }
    }
    if (can_vec && aligned)
        hipLaunchKernelGGL((softmax_topk_kernel<M, can_vec>), dim3((unsigned)a.rows), dim3(kThreads), 0, stream,
                           a.logits, a.idx, a.idx_row_stride, a.k, a);
    else
        hipLaunchKernelGGL((softmax_topk_kernel<M, false>), dim3((unsigned)a.rows), dim3(kThreads), 0, stream,
                           a.logits, a.idx, a.idx_row_stride, a.k, a);
    return hipGetLastError();
}

}  // namespace

bool softmax_topk_can_pick(const TopkArgs& a) {
    const int64_t m = (a.k + kThreads - 1) / kThreads;
    // (the instances launch_softmax_topk picks for rows of up to 8192 entries: one or two entries per thread, or
    // whole groups of four, which need the alignment)
    return m <= kPickMaxM && (m <= 2 || vec_ok(a)) && a.idx_row_stride == a.k;
}

hipError_t launch_softmax_topk(const TopkArgs& a, hipStream_t stream) {
    static_assert(topk::kRows16 == 64, "the threshold step ranks exactly 64 row maxima, one per lane");
    const int64_t m = (a.k + kThreads - 1) / kThreads;
    if (m <= 1) return launch_m<1>(a, stream);
    if (m <= 2) return launch_m<2>(a, stream);
    if (m <= 4) return launch_m<4>(a, stream);
    if (m <= 8) return launch_m<8>(a, stream);
    if (m <= 16) return launch_m<16>(a, stream);
    if (m <= 32) return launch_m<32>(a, stream);
    return launch_m<0>(a, stream);
}

}  // namespace sv
