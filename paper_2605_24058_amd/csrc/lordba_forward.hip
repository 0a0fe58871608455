// C entry points of the one-envelope adapter forward branch (the kernels and the dispatch live in lordba_fwd_impl.h).
#include "lordba_fwd_impl.h"

extern "C" lordba_status lordba_forward_algo(const void* x, const uint32_t* packedA, const uint32_t* packedB,
                                             const void* s_in, const void* s_rank, const void* s_out,
                                             const void* y_base, void* y_out,
                                             int64_t T, int64_t d_in, int64_t d_out, int64_t r, void* stream,
                                             int algo) {
    return forward_impl<1>(x, packedA, packedB, s_in, s_rank, s_out, y_base, y_out, T, d_in, d_out, r, stream, algo);
}

extern "C" lordba_status lordba_forward(const void* x, const uint32_t* packedA, const uint32_t* packedB,
                                        const void* s_in, const void* s_rank, const void* s_out,
                                        const void* y_base, void* y_out,
                                        int64_t T, int64_t d_in, int64_t d_out, int64_t r, void* stream) {
    return forward_impl<1>(x, packedA, packedB, s_in, s_rank, s_out, y_base, y_out, T, d_in, d_out, r, stream,
                           LORDBA_ALGO_AUTO);
}
