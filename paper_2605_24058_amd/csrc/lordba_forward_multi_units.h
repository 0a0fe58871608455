// Internal: one function per envelope count, each in its own translation unit (lordba_forward_multi_l.h instantiates the
// kernels of lordba_fwd_impl.h for one L), so that the units compile side by side.
#pragma once
#include <stdint.h>

#include "lordba.h"

#define LORDBA_DECLARE_MULTI(L)                                                                                              \
    lordba_status lordba_forward_multi_l##L(const void* x, const uint32_t* packedA, const uint32_t* packedB, const void* s_in, \
                                            const void* s_rank, const void* s_out, const void* y_base, void* y_out, int64_t T, \
                                            int64_t d_in, int64_t d_out, int64_t r, void* stream, int algo, float* t_out,      \
                                            int64_t t_stride, const int32_t* ids, int64_t n_adapters, int batched);
LORDBA_DECLARE_MULTI(2)
LORDBA_DECLARE_MULTI(3)
LORDBA_DECLARE_MULTI(4)
LORDBA_DECLARE_MULTI(2t)
LORDBA_DECLARE_MULTI(3t)
LORDBA_DECLARE_MULTI(4t)
#undef LORDBA_DECLARE_MULTI
