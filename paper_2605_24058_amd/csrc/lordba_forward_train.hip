// C entry point of the training forward of the one-envelope adapter branch: lordba_forward that also keeps the rank-r
// intermediate t for the backward pass.  This unit holds the training instantiations of the kernels in lordba_fwd_impl.h.
#define LORDBA_FWD_TRAINING 1
#include "lordba_fwd_impl.h"

extern "C" lordba_status lordba_forward_save_t(const void* x, const uint32_t* packedA, const uint32_t* packedB,
                                               const void* s_in, const void* s_rank, const void* s_out,
                                               const void* y_base, void* y_out, float* t_out, int64_t t_stride,
                                               int64_t T, int64_t d_in, int64_t d_out, int64_t r, void* stream) {
    if (t_out == nullptr && T != 0) return LORDBA_ERR_NULL;   // (an empty batch has nothing to keep)
    return forward_impl<1>(x, packedA, packedB, s_in, s_rank, s_out, y_base, y_out, T, d_in, d_out, r, stream,
                           LORDBA_ALGO_AUTO, nullptr, 1, false, t_out, t_stride);
}
