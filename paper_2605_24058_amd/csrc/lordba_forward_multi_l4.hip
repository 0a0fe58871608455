// The multi-envelope adapter forward branch with 4 envelopes (Eq. (lordba), l = 4): inference instantiations.
#include "lordba_fwd_impl.h"
#include "lordba_forward_multi_units.h"

lordba_status lordba_forward_multi_l4(const void* x, const uint32_t* packedA, const uint32_t* packedB, const void* s_in,
                                      const void* s_rank, const void* s_out, const void* y_base, void* y_out, int64_t T,
                                      int64_t d_in, int64_t d_out, int64_t r, void* stream, int algo, float* t_out, int64_t t_stride,
                                      const int32_t* ids, int64_t n_adapters, int batched) {
    return forward_impl<4>(x, packedA, packedB, s_in, s_rank, s_out, y_base, y_out, T, d_in, d_out, r, stream, algo, ids, n_adapters, batched != 0,
                           t_out, t_stride);
}
