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

extern "C" lordba_status lordba_forward_batched_algo(const void* x, const uint32_t* packedA_pool, const uint32_t* packedB_pool,
                                                     const void* s_in_pool, const void* s_rank_pool, const void* s_out_pool,
                                                     const int32_t* adapter_of_row, const void* y_base, void* y_out,
                                                     int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t n_adapters,
                                                     void* stream, int algo) {
    return forward_impl<1>(x, packedA_pool, packedB_pool, s_in_pool, s_rank_pool, s_out_pool, y_base, y_out, T, d_in, d_out, r,
                           stream, algo, adapter_of_row, n_adapters, true);
}

extern "C" lordba_status lordba_forward_batched(const void* x, const uint32_t* packedA_pool, const uint32_t* packedB_pool,
                                                const void* s_in_pool, const void* s_rank_pool, const void* s_out_pool,
                                                const int32_t* adapter_of_row, const void* y_base, void* y_out,
                                                int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t n_adapters,
                                                void* stream) {
    return forward_impl<1>(x, packedA_pool, packedB_pool, s_in_pool, s_rank_pool, s_out_pool, y_base, y_out, T, d_in, d_out, r,
                           stream, LORDBA_ALGO_AUTO, adapter_of_row, n_adapters, true);
}
