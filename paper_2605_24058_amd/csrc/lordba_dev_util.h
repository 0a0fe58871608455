// Device helpers shared by the forward and backward kernels of the LoRDBA library (gfx950, wave64): 16-byte accesses,
// sign application by XOR into fp16 sign bits from packed carrier bits, DPP row reductions, MFMA row mapping.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ u4 load16(const void* p) { return *reinterpret_cast<const u4*>(p); }
__device__ __forceinline__ void store16(void* p, u4 v) { *reinterpret_cast<u4*>(p) = v; }
// Streaming accesses for x, y_base and y_out: each byte is touched once, so it should not displace the adapter
// (carrier bits, scales) from the caches.
__device__ __forceinline__ u4 load16_stream(const void* p) { return __builtin_nontemporal_load(reinterpret_cast<const u4*>(p)); }
__device__ __forceinline__ void store16_stream(void* p, u4 v) { __builtin_nontemporal_store(v, reinterpret_cast<u4*>(p)); }
// Address = uniform base (kept in scalar registers) + unsigned 32-bit byte offset per lane: one add-free addressing
// mode, no 64-bit vector arithmetic.
__device__ __forceinline__ const void* at(const void* base, uint32_t byte_off) { return static_cast<const char*>(base) + byte_off; }
__device__ __forceinline__ void* at(void* base, uint32_t byte_off) { return static_cast<char*>(base) + byte_off; }
__device__ __forceinline__ h8 as_h8(u4 v) { return __builtin_bit_cast(h8, v); }
// Value of the lane N places further along its row of 16 lanes (rotation inside the row, a DPP move: no LDS traffic).
template <int N>
__device__ __forceinline__ float row_rotate(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x120 + N, 0xf, 0xf, false));
}
__device__ __forceinline__ float row_max16(float v) {
    v = fmaxf(v, row_rotate<8>(v));
    v = fmaxf(v, row_rotate<4>(v));
    v = fmaxf(v, row_rotate<2>(v));
    return fmaxf(v, row_rotate<1>(v));
}
__device__ __forceinline__ float flip(float v, uint32_t bit) { return __uint_as_float(__float_as_uint(v) ^ (bit << 31)); }

// Row of the MFMA token operand -> token row of the tile.  With 16 token rows it is the identity.  With 8, MFMA
// rows 4q+0 and 4q+1 carry token rows 2q and 2q+1 and rows 4q+2, 4q+3 repeat them (their results are ignored), so
// that in the accumulator layout (lane = column, registers = rows 4q..4q+3) every lane owns two live token rows.
template <int TMV>
__device__ __forceinline__ int tile_row_of_mfma_row(int m) { return TMV == 16 ? m : ((m >> 2) * 2 + (m & 1)); }

constexpr int kXRow = 136;  // halves per row of the x transpose tile: 128 columns + 8 pad -> conflict-free b128 reads

typedef uint16_t us2 __attribute__((ext_vector_type(2)));

// Sign masks of one operand dword from a word whose two 16-bit halves both hold the 8 carrier bits of the lane in
// their low byte: bit 2i goes to the sign of the low fp16, bit 2i+1 to the sign of the high fp16.  The packed 16-bit
// shift drops everything above the wanted bit; the bits below it are removed by the caller's mask.
template <int I>
__device__ __forceinline__ uint32_t spread_pair(uint32_t both) {
    const us2 sh = {static_cast<uint16_t>(15 - 2 * I), static_cast<uint16_t>(14 - 2 * I)};
    return __builtin_bit_cast(uint32_t, static_cast<us2>(__builtin_bit_cast(us2, both) << sh));
}
// 8 carrier bits -> 8 fp16 values +-1.0 (bit set = -1.0), with vector ALU only.
__device__ __forceinline__ u4 pm_one_from_bits(uint32_t both) {
    // (shifted & sign bits) | 1.0 in one three-input bit operation (truth table 0xEA = (a & b) | c)
    u4 f;
    f[0] = __builtin_amdgcn_bitop3_b32(spread_pair<0>(both), 0x80008000u, 0x3C003C00u, 0xEA);
    f[1] = __builtin_amdgcn_bitop3_b32(spread_pair<1>(both), 0x80008000u, 0x3C003C00u, 0xEA);
    f[2] = __builtin_amdgcn_bitop3_b32(spread_pair<2>(both), 0x80008000u, 0x3C003C00u, 0xEA);
    f[3] = __builtin_amdgcn_bitop3_b32(spread_pair<3>(both), 0x80008000u, 0x3C003C00u, 0xEA);
    return f;
}
// 8 fp16 values with the sign of element e flipped where carrier bit e is set.
__device__ __forceinline__ u4 flip_by_bits(u4 v, uint32_t both) {
    v[0] ^= spread_pair<0>(both) & 0x80008000u;
    v[1] ^= spread_pair<1>(both) & 0x80008000u;
    v[2] ^= spread_pair<2>(both) & 0x80008000u;
    v[3] ^= spread_pair<3>(both) & 0x80008000u;
    return v;
}

// The epilogue y = fp16(v * s + b) is written in plain C++ on fp16 operands converted to float, so that the compiler
// selects the mixed-precision FMA (v_fma_mixlo/mixhi_f16: fp16 operands read directly, fp32 arithmetic, one rounding to
// fp16).  Deliberately not inline assembly: the compiler reuses dead accumulator registers of an MFMA that is still in
// flight, and it inserts the wait states such a write needs only for instructions it can see.
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
// Raw buffer access (stride 0) to `bytes` bytes behind p, with the range check of the buffer instructions: a load whose
// offset is not below `bytes` returns zeros and a store there is dropped, without a memory request.  An access that is to
// be left out is given the offset kBufferSkip instead of being put under a branch: the number of outstanding vector
// memory operations at any point of the code then does not depend on the data, and the compiler's wait counts can be exact
// (bytes <= 2^30 here).
constexpr uint32_t kBufferSkip = 0x80000000u;
__device__ __forceinline__ __amdgpu_buffer_rsrc_t buffer_over(const void* p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, static_cast<int>(bytes), 0x00020000);
}
__device__ __forceinline__ u4 buffer_load16_stream(__amdgpu_buffer_rsrc_t rs, uint32_t byte_off) {
    return __builtin_bit_cast(u4, __builtin_amdgcn_raw_buffer_load_b128(rs, static_cast<int>(byte_off), 0, 2));  // 2: nontemporal
}
__device__ __forceinline__ void buffer_store16_stream(__amdgpu_buffer_rsrc_t rs, uint32_t byte_off, u4 v) {
    typedef unsigned raw4 __attribute__((vector_size(16)));
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(raw4, v), rs, static_cast<int>(byte_off), 0, 2);
}

// The four lane groups of 16 (lanes 16 g .. 16 g + 15) each hold four dwords v[0..3]; afterwards group g holds in v[n] what
// group n held in v[g] (a 4 x 4 transpose between the groups, lane by lane).  Two rounds of the row swaps of gfx950:
// v_permlane32_swap exchanges lanes 32..63 of its first operand with lanes 0..31 of its second, v_permlane16_swap lanes
// 16..31 and 48..63 of the first with lanes 0..15 and 32..47 of the second.
__device__ __forceinline__ void transpose_lane_groups(u4& v) {
    const auto a = __builtin_amdgcn_permlane32_swap(v[0], v[2], false, false);
    const auto b = __builtin_amdgcn_permlane32_swap(v[1], v[3], false, false);
    const auto c = __builtin_amdgcn_permlane16_swap(a[0], b[0], false, false);
    const auto d = __builtin_amdgcn_permlane16_swap(a[1], b[1], false, false);
    v = u4{c[0], c[1], d[0], d[1]};
}

__device__ __forceinline__ h2 as_h2(uint32_t v) { return __builtin_bit_cast(h2, v); }

}  // namespace
