// C entry points of the multi-envelope adapter forward branch (Eq. (lordba) with envelope rank l >= 2).  The kernels are
// instantiated in one translation unit per envelope count (lordba_forward_multi_l2/3/4.hip, and lordba_forward_multi_train.hip
// for the calls that keep t); this file only dispatches on the envelope count.
#include "lordba_forward_multi_units.h"

extern "C" lordba_status lordba_forward_multi_algo(const void* x, const uint32_t* packedA, const uint32_t* packedB,
                                                   const void* s_in, const void* s_rank, const void* s_out,
                                                   const void* y_base, void* y_out,
                                                   int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t ell,
                                                   void* stream, int algo) {
    switch (ell) {
        case 1: return lordba_forward_algo(x, packedA, packedB, s_in, s_rank, s_out, y_base, y_out, T, d_in, d_out, r, stream, algo);
        case 2: return lordba_forward_multi_l2(x, packedA, packedB, s_in, s_rank, s_out, y_base, y_out, T, d_in, d_out, r, stream, algo, nullptr, 0, nullptr, 1, 0);
        case 3: return lordba_forward_multi_l3(x, packedA, packedB, s_in, s_rank, s_out, y_base, y_out, T, d_in, d_out, r, stream, algo, nullptr, 0, nullptr, 1, 0);
        case 4: return lordba_forward_multi_l4(x, packedA, packedB, s_in, s_rank, s_out, y_base, y_out, T, d_in, d_out, r, stream, algo, nullptr, 0, nullptr, 1, 0);
        default: return LORDBA_ERR_DIM;
    }
}

extern "C" lordba_status lordba_forward_multi(const void* x, const uint32_t* packedA, const uint32_t* packedB,
                                              const void* s_in, const void* s_rank, const void* s_out,
                                              const void* y_base, void* y_out,
                                              int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t ell,
                                              void* stream) {
    return lordba_forward_multi_algo(x, packedA, packedB, s_in, s_rank, s_out, y_base, y_out, T, d_in, d_out, r, ell, stream,
                                     LORDBA_ALGO_AUTO);
}

extern "C" lordba_status lordba_forward_multi_save_t(const void* x, const uint32_t* packedA, const uint32_t* packedB,
                                                     const void* s_in, const void* s_rank, const void* s_out,
                                                     const void* y_base, void* y_out, float* t_out, int64_t t_stride,
                                                     int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t ell, void* stream) {
    if (t_out == nullptr && T != 0) return LORDBA_ERR_NULL;   // (an empty batch has nothing to keep)
    const int algo = LORDBA_ALGO_AUTO;
    switch (ell) {
        case 1: return lordba_forward_save_t(x, packedA, packedB, s_in, s_rank, s_out, y_base, y_out, t_out, t_stride, T, d_in, d_out, r, stream);
        case 2: return lordba_forward_multi_l2t(x, packedA, packedB, s_in, s_rank, s_out, y_base, y_out, T, d_in, d_out, r, stream, algo, t_out, t_stride, nullptr, 1, 0);
        case 3: return lordba_forward_multi_l3t(x, packedA, packedB, s_in, s_rank, s_out, y_base, y_out, T, d_in, d_out, r, stream, algo, t_out, t_stride, nullptr, 1, 0);
        case 4: return lordba_forward_multi_l4t(x, packedA, packedB, s_in, s_rank, s_out, y_base, y_out, T, d_in, d_out, r, stream, algo, t_out, t_stride, nullptr, 1, 0);
        default: return LORDBA_ERR_DIM;
    }
}

extern "C" lordba_status lordba_forward_batched_multi_algo(const void* x, const uint32_t* packedA_pool, const uint32_t* packedB_pool,
                                                           const void* s_in_pool, const void* s_rank_pool, const void* s_out_pool,
                                                           const int32_t* adapter_of_row, const void* y_base, void* y_out,
                                                           int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t ell,
                                                           int64_t n_adapters, void* stream, int algo) {
    switch (ell) {
        case 1: return lordba_forward_batched_algo(x, packedA_pool, packedB_pool, s_in_pool, s_rank_pool, s_out_pool, adapter_of_row, y_base,
                                                   y_out, T, d_in, d_out, r, n_adapters, stream, algo);
        case 2: return lordba_forward_multi_l2(x, packedA_pool, packedB_pool, s_in_pool, s_rank_pool, s_out_pool, y_base, y_out, T, d_in, d_out, r,
                                               stream, algo, nullptr, 0, adapter_of_row, n_adapters, 1);
        case 3: return lordba_forward_multi_l3(x, packedA_pool, packedB_pool, s_in_pool, s_rank_pool, s_out_pool, y_base, y_out, T, d_in, d_out, r,
                                               stream, algo, nullptr, 0, adapter_of_row, n_adapters, 1);
        case 4: return lordba_forward_multi_l4(x, packedA_pool, packedB_pool, s_in_pool, s_rank_pool, s_out_pool, y_base, y_out, T, d_in, d_out, r,
                                               stream, algo, nullptr, 0, adapter_of_row, n_adapters, 1);
        default: return LORDBA_ERR_DIM;
    }
}

extern "C" lordba_status lordba_forward_batched_multi(const void* x, const uint32_t* packedA_pool, const uint32_t* packedB_pool,
                                                      const void* s_in_pool, const void* s_rank_pool, const void* s_out_pool,
                                                      const int32_t* adapter_of_row, const void* y_base, void* y_out,
                                                      int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t ell,
                                                      int64_t n_adapters, void* stream) {
    return lordba_forward_batched_multi_algo(x, packedA_pool, packedB_pool, s_in_pool, s_rank_pool, s_out_pool, adapter_of_row, y_base, y_out,
                                             T, d_in, d_out, r, ell, n_adapters, stream, LORDBA_ALGO_AUTO);
}
