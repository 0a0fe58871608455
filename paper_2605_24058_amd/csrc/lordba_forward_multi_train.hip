// The multi-envelope adapter forward branch as training runs it (t of every envelope is kept): the training instantiations
// for 2, 3 and 4 envelopes (one variant family each, see launch_mfma_gm).
#define LORDBA_FWD_TRAINING 1
#include "lordba_fwd_impl.h"
#include "lordba_forward_multi_units.h"

#define LORDBA_DEFINE_MULTI_T(L)                                                                                               \
    lordba_status lordba_forward_multi_l##L##t(const void* x, const uint32_t* packedA, const uint32_t* packedB, const void* s_in, \
                                               const void* s_rank, const void* s_out, const void* y_base, void* y_out, int64_t T, \
                                               int64_t d_in, int64_t d_out, int64_t r, void* stream, int algo, float* t_out,    \
                                               int64_t t_stride, const int32_t*, int64_t, int) {                              \
        return forward_impl<L>(x, packedA, packedB, s_in, s_rank, s_out, y_base, y_out, T, d_in, d_out, r, stream, algo, nullptr, 1, \
                               false, t_out, t_stride);                                                                       \
    }
LORDBA_DEFINE_MULTI_T(2)
LORDBA_DEFINE_MULTI_T(3)
LORDBA_DEFINE_MULTI_T(4)
#undef LORDBA_DEFINE_MULTI_T
