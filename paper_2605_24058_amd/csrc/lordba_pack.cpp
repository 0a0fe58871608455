// Host side of the LoRDBA library: canonical carrier packing (Sec. 3.3 "bit-packed {B1, B2}",
// R(N+M) bits by Eq. (lordba-bits)) and the status strings.  No device code here.
//
// Format: a [rows, cols] sign matrix is the row-major bit stream n = row*cols + col, bit n in bit
// (n & 31) of word (n >> 5), bit 1 = -1, bit 0 = +1, pad bits zero.
#include "lordba.h"

#include <cmath>
#include <cstring>

namespace {

// Packs 32 entries at a time; `neg(i)` says whether stream entry i is -1, `ok(i)` whether it is legal.
template <typename Neg, typename Ok>
lordba_status pack_stream(int64_t nbits, uint32_t* words, Neg neg, Ok ok) {
    const int64_t nwords = (nbits + 31) >> 5;
    for (int64_t w = 0; w < nwords; ++w) {
        const int64_t base = w << 5;
        const int64_t left = nbits - base;
        const int lim = left < 32 ? static_cast<int>(left) : 32;
        uint32_t word = 0;
        for (int b = 0; b < lim; ++b) {
            if (!ok(base + b)) return LORDBA_ERR_VALUE;
            word |= static_cast<uint32_t>(neg(base + b)) << b;
        }
        words[w] = word;
    }
    return LORDBA_OK;
}

lordba_status check_pack_dims(const void* a, const void* b, const void* pa, const void* pb,
                              int64_t d_in, int64_t d_out, int64_t r) {
    if (!a || !b || !pa || !pb) return LORDBA_ERR_NULL;
    if (d_in < 1 || d_out < 1 || r < 1 || r > LORDBA_MAX_RANK) return LORDBA_ERR_DIM;
    if (d_in > (INT64_C(1) << 40) || d_out > (INT64_C(1) << 40)) return LORDBA_ERR_DIM;
    return LORDBA_OK;
}

}  // namespace

extern "C" size_t lordba_packed_words(int64_t rows, int64_t cols) {
    if (rows < 0 || cols < 0) return 0;
    return static_cast<size_t>((rows * cols + 31) >> 5);
}

extern "C" lordba_status lordba_pack_signs(const int8_t* signsA, const int8_t* signsB,
                                           uint32_t* packedA, uint32_t* packedB,
                                           int64_t d_in, int64_t d_out, int64_t r) {
    lordba_status st = check_pack_dims(signsA, signsB, packedA, packedB, d_in, d_out, r);
    if (st != LORDBA_OK) return st;
    auto pack_i8 = [](const int8_t* s, int64_t n, uint32_t* out) {
        return pack_stream(n, out,
                           [s](int64_t i) { return s[i] < 0; },
                           [s](int64_t i) { return s[i] == 1 || s[i] == -1; });
    };
    st = pack_i8(signsA, r * d_in, packedA);
    if (st != LORDBA_OK) return st;
    return pack_i8(signsB, d_out * r, packedB);
}

extern "C" lordba_status lordba_pack_signs_f32(const float* latentA, const float* latentB,
                                               uint32_t* packedA, uint32_t* packedB,
                                               int64_t d_in, int64_t d_out, int64_t r) {
    lordba_status st = check_pack_dims(latentA, latentB, packedA, packedB, d_in, d_out, r);
    if (st != LORDBA_OK) return st;
    // sign(0) = +1 (Sec. 2, Notation): an entry is -1 only if its value is below zero, so -0.0 is +1.
    auto pack_f32 = [](const float* u, int64_t n, uint32_t* out) {
        return pack_stream(n, out,
                           [u](int64_t i) { return u[i] < 0.0f; },
                           [u](int64_t i) { return !std::isnan(u[i]); });
    };
    st = pack_f32(latentA, r * d_in, packedA);
    if (st != LORDBA_OK) return st;
    return pack_f32(latentB, d_out * r, packedB);
}

extern "C" lordba_status lordba_unpack_signs(const uint32_t* packedA, const uint32_t* packedB,
                                             int8_t* signsA, int8_t* signsB,
                                             int64_t d_in, int64_t d_out, int64_t r) {
    lordba_status st = check_pack_dims(packedA, packedB, signsA, signsB, d_in, d_out, r);
    if (st != LORDBA_OK) return st;
    auto unpack = [](const uint32_t* w, int64_t n, int8_t* out) {
        for (int64_t i = 0; i < n; ++i) out[i] = ((w[i >> 5] >> (i & 31)) & 1u) ? -1 : 1;
    };
    unpack(packedA, r * d_in, signsA);
    unpack(packedB, d_out * r, signsB);
    return LORDBA_OK;
}

extern "C" const char* lordba_status_string(lordba_status status) {
    switch (status) {
        case LORDBA_OK: return "ok";
        case LORDBA_ERR_NULL: return "null pointer argument";
        case LORDBA_ERR_DIM: return "dimension out of range (need T >= 0, d_in, d_out >= 1, 1 <= r <= 64)";
        case LORDBA_ERR_VALUE: return "carrier entry is not +1/-1 (or is NaN)";
        case LORDBA_ERR_ALIAS: return "y_out overlaps an input (only y_out == y_base is allowed)";
        case LORDBA_ERR_ALIGN: return "pointer not aligned to its element size";
        case LORDBA_ERR_NO_DEVICE: return "no usable gfx950 HIP device";
        case LORDBA_ERR_LAUNCH: return "HIP runtime rejected the kernel launch";
        case LORDBA_ERR_ALGO: return "requested kernel cannot run this shape or alignment";
        case LORDBA_ERR_WORKSPACE: return "workspace smaller than lordba_backward_workspace_bytes";
        default: return "unknown status";
    }
}
