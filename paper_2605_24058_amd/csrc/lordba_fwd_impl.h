// LoRDBA adapter forward branch for MI355X (gfx950, wave64, MFMA):
//
//   y_out[t,j] = y_base[t,j] + s_out[j] * sum_k S_B[j,k] * s_rank[k] * sum_i S_A[k,i] * s_in[i] * x[t,i]
//
// (Def. 1 / Eq. (lordba) with l = 1, Eq. (adapter-mode-fwd), evaluation order of Eq. (lordba-fwd).)
//
// Token rows are independent, so one workgroup owns a tile of token rows from the first load of x to
// the last store of y_out and no workgroup ever waits for another: there is no split over d_in across
// workgroups, no partial-sum workspace and no second launch.
//
// Matrix-core kernel (lordba_fwd_mfma_kernel), per workgroup of NW waves and TMV token rows:
//   stage 1  t[tok, k] = sum_i x[tok,i] * (+-s_in[i]).  The 128-column chunks of d_in are dealt round-robin
//            to the waves.  A wave reads its chunk of x with row-contiguous 16-byte loads, transposes it
//            through a wave-private LDS tile into the MFMA operand layout, builds the other operand
//            (+-s_in as fp16: s_in with its sign bit XORed with the carrier bit, so the product with x is
//            exact in fp32) with a few vector-ALU bit operations from one dword of carrier bits per lane, and
//            issues v_mfma_f32_16x16x32_f16.  No workgroup barrier is involved: a wave starts as soon as its
//            own data is there.  The partial tiles of the waves are summed through LDS in a fixed order.
//   stage 2  u = s_rank * t in fp32; each token row of u is scaled by a power of two so that its largest
//            entry is in [2^13, 2^14) and split into fp16 hi + fp16 lo (22 significant bits, no overflow or
//            underflow whatever the magnitude of the scales); hi and lo fill the K = 32 slots of one MFMA
//            per 16 ranks.
//   stage 3  v[tok, j] = sum_k u[tok,k] * (+-1), 8 MFMAs per 128 output columns, arranged so that each lane
//            ends up with 8 consecutive output columns of its token rows: y_base is read and y_out written
//            with row-contiguous 16-byte accesses, y_out = fp16_rne(y_base + s_out * v * 2^-scale).  The +-1
//            operands come from a 256-entry LDS table (8 carrier bits -> 8 fp16); those of a wave's first
//            block are built with the vector ALU while the wave waits for the others to finish stage 1.
//
// General kernel (lordba_fwd_general_kernel): plain vector-ALU code, one workgroup per token row, any
// shape and alignment; also the fallback when the LDS need of the matrix-core kernel exceeds the CU.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "lordba.h"
#include "lordba_dev_util.h"
#include "lordba_host_util.h"

namespace {

constexpr unsigned kSplitBlocks = 4;  // output blocks per workgroup when a tile's blocks are split (one per SIMD)
constexpr int kURow = 40;   // halves per row of the u tile: 32 slots + 8 pad
constexpr int kLutBytes = 256 * 16;

struct FwdArgs {
    const _Float16* x;
    const uint32_t* pA;
    const uint32_t* pB;
    const _Float16* s_in;
    const _Float16* s_rank;
    const _Float16* s_out;
    const _Float16* y_base;
    _Float16* y_out;
    int T, d_in, d_out, r;
    int ell;  // envelopes: s_in, s_rank, s_out are [ell, d_in], [ell, r], [ell, d_out]
    int blocks_per_wg;  // matrix-core kernel: 128-column output blocks per workgroup (the grid's y extent covers d_out)
    // Multi-adapter batch (ids != nullptr): pA, pB, s_in, s_rank, s_out are pools of n_adapters adapters laid out one
    // after the other, and token row t uses adapter ids[t]; an id outside [0, n_adapters) means "no adapter".
    const int32_t* ids;
    int n_adapters;
    // Training: if t_out != nullptr the rank-r intermediate t = (x D_alpha) B1 (before the rank scaling) is also written,
    // fp32, rank-major, one [r, t_stride] block per envelope: t_out[(e * r + k) * t_stride + token].  With
    // y_out == nullptr nothing else is computed (no stage 3).
    float* t_out;
    int t_stride;
};

// The arguments of one adapter of a pool.
__device__ __forceinline__ FwdArgs select_adapter(const FwdArgs& a, int id) {
    FwdArgs b = a;
    b.pA += static_cast<int64_t>(id) * ((static_cast<int64_t>(a.r) * a.d_in + 31) >> 5);
    b.pB += static_cast<int64_t>(id) * ((static_cast<int64_t>(a.d_out) * a.r + 31) >> 5);
    b.s_in += static_cast<int64_t>(id) * a.ell * a.d_in;   // each adapter of the pool has its ell rows of scales
    b.s_rank += static_cast<int64_t>(id) * a.ell * a.r;
    b.s_out += static_cast<int64_t>(id) * a.ell * a.d_out;
    return b;
}

// 8 carrier bits starting at bit `bit0` of a packed stream of `nwords` words.  Both words are always read from a
// clamped, valid index (no branch, no access past the end); bits past the end of the stream are not meaningful and
// the callers only use them for padded ranks, whose other operand is zero.
__device__ __forceinline__ uint32_t fetch8(const uint32_t* __restrict__ words, int64_t bit0, int64_t nwords) {
    int64_t w = bit0 >> 5;
    w = w < nwords ? w : nwords - 1;
    const int64_t w1 = (w + 1) < nwords ? w + 1 : nwords - 1;
    const uint32_t lo = words[w], hi = words[w1];
    return static_cast<uint32_t>(((static_cast<uint64_t>(hi) << 32) | lo) >> (bit0 & 31)) & 0xffu;
}

constexpr int kUBytes = 16 * kURow * 2;  // one rank block of the u tile

// LDS bytes of the matrix-core kernel (host and device use the same formula).
__host__ __device__ constexpr size_t mfma_lds_bytes(int RB, int TMV, int NW, int D1, int L) {
    return kLutBytes + static_cast<size_t>(NW) * D1 * L * 256 + static_cast<size_t>(NW) * TMV * kXRow * 2 +
           static_cast<size_t>(NW) * RB * L * 1024 + static_cast<size_t>(RB) * L * kUBytes + 64 * static_cast<size_t>(L);
}

// RB   rank blocks of 16 (r <= 16 * RB)
// TMV  token rows per workgroup (8 or 16)
// NW   waves per workgroup (>= 4)
// D1   128-column chunks of x a wave keeps in flight
// OS   "one shot": every wave's chunks fit in D1, so stage 1 is straight-line code; otherwise stage 1 loops over
//      groups of D1 chunks
// BM   how a lane fetches the sign(B) bits of its 8 output columns: 1 = r is a multiple of 16 (RB aligned 16-byte
//      loads), 2 = r is 8 (one aligned 8-byte load, one byte per column), 0 = any r (two dwords per operand)
// GM   grid mode.  1 (grids that fill the chip): the waves that do not run stage 2 build their first block's sign
//      operands during stage 2 instead of before it.  2 (a handful of tiles): gridDim.y workgroups share a token tile
//      and split its output blocks; the x extent of the grid is padded to a multiple of 8 and padding workgroups exit.
//      3 (fewer token rows than a tile): as 2, and rows past T are not requested at all.  4: multi-adapter batch,
//      the gridDim.y workgroups of a tile share its runs of rows that use the same adapter (rows outside a run are not
//      requested).  0: none of these.
// L    scale envelopes over the same carriers (Eq. (lordba)): s_in, s_rank, s_out hold L rows; everything that depends
//      on a scale is done L times, everything that depends only on x or on the carrier bits once
//
// fwd_tile: rows first..last (inclusive, relative to token row t0) of one tile through one adapter, by the whole
// workgroup.  Rows of the tile outside that range are neither requested as such (loads are clamped into the range) nor
// stored.  The function may be called several times in a row by a workgroup (its barriers order the reuse of LDS).
template <int RB, int TMV, int NW, int D1, bool OS, int BM, int GM, int L, bool TR>
__device__ __forceinline__ void fwd_tile(const FwdArgs& a, unsigned char* smem, const int64_t t0, const int first, const int last) {
    static_assert(NW >= 4, "stage 2 is spread over the first four waves");
    constexpr bool LP = GM == 1, SPLIT = GM == 2 || GM == 3, MASK = GM == 3 || GM == 4;
    constexpr int NI = TMV / 4;           // 16-byte row accesses per lane per 128-column block of a tile
    // y_base column blocks in flight per wave.  Three and four envelopes run on 8 waves (their registers do not fit 16
    // waves): on 8-row tiles four blocks in flight per wave keep as many bytes of y_base under way per compute unit as 16
    // waves with two.  The multi-adapter batch on 8 waves holds three (two of its workgroups share a compute unit, so a
    // lane has 128 registers).  Four envelopes on 16-row tiles (grids of at least 256 tiles, two workgroups per compute
    // unit) hold one.
    constexpr int D2 = (TMV == 16 && L == 4) ? 1 : (GM == 4 && NW == 8 && RB == 1 && L == 1) ? 3 : (NW == 8 && TMV == 8 && GM != 4 && ((L >= 3 && RB == 1) || (L == 3 && RB == 2))) ? 4 : 2;
    constexpr bool R16 = BM == 1, R8 = BM == 2;
    static_assert(!R8 || RB == 1, "r = 8 is one rank block");
    // Four envelopes on 16-row tiles: to stay inside the registers, no sign operands are built ahead and the row scalings
    // are read from LDS where they are used.
    constexpr bool LEAN = TMV == 16 && L == 4;
    // (not in the multi-adapter batch on 8 waves either: two of its workgroups must fit a compute unit, 128 registers per lane)
    constexpr bool PRE = (R16 || R8) && RB == 1 && !LEAN && !(GM == 4 && NW == 8);  // sign operands of the first block are built before u is known

    // The wave index is read into a scalar register: what depends on it (which chunks and blocks a wave owns, which waves
    // run stage 2) then branches on scalar conditions.  MFMA instructions ignore the EXEC mask, so they must never end up
    // under a vector-predicated branch, which is what a condition on a value derived from threadIdx may compile to.
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, q = lane >> 4;
    const int li_ = li, q_ = q;  // (issue_x shadows li and q, see there)
    const int d_in = a.d_in, d_out = a.d_out, r = a.r;
    const int nchunks = (d_in + 127) >> 7;

    u4* lutp = reinterpret_cast<u4*>(smem);  // 8 bits -> 8 fp16 values +-1.0
    unsigned char* p = smem + kLutBytes;
    _Float16* sinw = reinterpret_cast<_Float16*>(p) + wave * D1 * L * 128;  // wave-private s_in slices, one per chunk slot and envelope
    p += NW * D1 * L * 256;
    _Float16* xs = reinterpret_cast<_Float16*>(p) + wave * TMV * kXRow;  // wave-private x transpose tile
    p += NW * TMV * kXRow * 2;
    float* red = reinterpret_cast<float*>(p);
    p += NW * RB * L * 1024;
    _Float16* us = reinterpret_cast<_Float16*>(p);
    p += RB * L * kUBytes;
    float* invs = reinterpret_cast<float*>(p);

    // The CU's vector memory pipeline takes a bounded number of outstanding requests and returns data in request
    // order, so loads are issued in the order their data is needed: s_rank, then per chunk s_in and x, and y_base only
    // after the wave has consumed its x (an earlier request would sit in front of other waves' x).
    // A tile never spans more than 16 rows of at most 2^24 columns, so offsets inside it fit 32 bits.
    const _Float16* xt = a.x + t0 * d_in;
    const _Float16* ybt = a.y_base + t0 * d_out;
    _Float16* yot = a.y_out + t0 * d_out;
    // Multi-adapter batch: y_base and y_out of the tile as buffers of rows 0..last; rows of stage 3 that are not live get an
    // offset outside instead of a branch around the access (the runs of a tile make most accesses partial there).
    constexpr bool BUFY = GM == 4 || (L == 1 && (GM == 0 || GM == 1) && TMV == 8 && NW == 8);
    const uint32_t ytile_bytes = static_cast<uint32_t>(last + 1) * static_cast<uint32_t>(d_out) * 2u;
    const __amdgpu_buffer_rsrc_t yb_rs = buffer_over(ybt, BUFY ? ytile_bytes : 0u), yo_rs = buffer_over(yot, BUFY ? ytile_bytes : 0u);

    // ---------------------------------------------------------------- stage 1 loads -----------------
    // Chunk c = 128 columns of d_in; wave w owns chunks w, w + NW, ...  x: lane (row q + 4m, 16-byte column group li)
    // -> 256 contiguous bytes per row and quarter-wave.  s_in: the chunk's 256 bytes, one dword per lane.  Carrier
    // bits: lane (rank li, dword q of the chunk) holds the 32 bits of its rank for columns 32q..32q+31 of the chunk;
    // byte s of that dword belongs to MFMA step s.
    // One-shot variants (every chunk of a wave in flight at once): a wave owns CONSECUTIVE chunks, so that the carrier bits
    // of its chunks are 16 contiguous bytes per rank and group of four slots; one 16-byte load per lane (lane group q
    // fetches the four words of the wave's q-th chunk) and a transpose between the lane groups replace four gathering
    // dword loads, each of which has the memory pipeline look up 16 cache lines for 256 bytes.  At decode sizes, where a
    // few workgroups run alone and the time to issue the loads is latency of the call, that is 2.4 us of 9.6 at r = 64;
    // grids that fill the chip gain 1 to 5 %.  (The multi-adapter batch keeps the round-robin deal: 128 registers.)
    constexpr bool CA = OS && GM != 4;
    const int words_per_row = d_in >> 5;  // d_in % 32 == 0 on this path
    // (the first nchunks mod NW waves own one chunk more than the others: at most ceil(nchunks / NW), <= D1 where OS)
    const int c_each = nchunks / NW, c_more = nchunks - c_each * NW;
    const int c_first = wave * c_each + (wave < c_more ? wave : c_more);   // first chunk of the wave's run
    const int my_n = CA ? c_each + (wave < c_more ? 1 : 0) : (wave < nchunks ? (nchunks - wave + NW - 1) / NW : 0);
    // (16-byte loads need whole chunks and rows that start on 16-byte boundaries)
    const bool wide_a = CA && (d_in & 127) == 0 && (reinterpret_cast<uintptr_t>(a.pA) & 15) == 0;
    u4 xbuf[D1][NI];
    uint32_t sinbuf[D1][L];
    uint32_t abits[D1][RB];

    auto issue_x = [&](int slot, int n) {
        int c = CA ? c_first + n : wave + NW * n;
        c = c < nchunks ? c : nchunks - 1;  // past the end: re-read a valid chunk, the result is not used
        // 16 waves leave 128 registers per lane.  In the looped pipeline the compiler would keep every lane's row and rank
        // offsets in registers across the loop (the chunk index is scalar, so they are loop invariants) and spill; hiding
        // the lane coordinates behind an empty asm makes it recompute them per chunk, a few vector-ALU instructions.
        int q = q_, li = li_;
        if constexpr (NW == 16 && !OS) {
            asm volatile("" : "+v"(q));
            asm volatile("" : "+v"(li));
        }
#pragma unroll
        for (int en = 0; en < L; ++en) {
            const int pair = c * 64 + lane;  // fp16 pair index; d_in is even, so a pair is inside or outside as a whole
            const uint32_t v = *static_cast<const uint32_t*>(
                at(a.s_in, static_cast<uint32_t>(en * d_in) * 2u + static_cast<uint32_t>(pair * 2 < d_in ? pair : 0) * 4u));
            sinbuf[slot][en] = pair * 2 < d_in ? v : 0u;  // columns past d_in get scale 0
        }
#pragma unroll
        for (int m = 0; m < NI; ++m) {
            int row = m * 4 + q;
            const bool live = row >= first && row <= last;
            row = row < last ? row : last;
            row = row > first ? row : first;
            int col = c * 128 + li * 8;
            col = col < d_in ? col : d_in - 8;
            if (MASK) {
                // fewer than 8 token rows: rows past T are not requested at all (a tile with one live row moves an eighth)
                xbuf[slot][m] = u4{0u, 0u, 0u, 0u};
                if (live) xbuf[slot][m] = load16_stream(at(xt, static_cast<uint32_t>(row * d_in + col) * 2u));
            } else {
                xbuf[slot][m] = load16_stream(at(xt, static_cast<uint32_t>(row * d_in + col) * 2u));
            }
        }
        if (!wide_a) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                int rk = rb * 16 + li;
                rk = rk < r ? rk : r - 1;
                int w = c * 4 + q;
                w = w < words_per_row ? w : words_per_row - 1;  // columns past d_in meet s_in = 0
                abits[slot][rb] = *static_cast<const uint32_t*>(at(a.pA, static_cast<uint32_t>(rk * words_per_row + w) * 4u));
            }
        }
    };
    constexpr int AG = CA ? (D1 + 3) / 4 : 1;  // groups of four chunk slots
    u4 awide[AG][CA ? RB : 1];
    if constexpr (CA) {
        if (wide_a) {  // needed first, so requested first
#pragma unroll
            for (int g = 0; g < AG; ++g) {
                int c = c_first + g * 4 + q;
                c = c < nchunks ? c : nchunks - 1;
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    int rk = rb * 16 + li;
                    rk = rk < r ? rk : r - 1;
                    awide[g][rb] = load16(at(a.pA, static_cast<uint32_t>(rk * words_per_row + c * 4) * 4u));
                }
            }
        }
    }
#pragma unroll
    for (int slot = 0; slot < D1; ++slot) issue_x(slot, slot);
    __builtin_amdgcn_sched_barrier(0);  // keep the issue order: nothing below may be hoisted above these requests
    float sr[RB][L];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
        for (int en = 0; en < L; ++en) {
            const int rk = rb * 16 + li;
            const _Float16 h = *static_cast<const _Float16*>(at(a.s_rank, static_cast<uint32_t>(en * r + (rk < r ? rk : r - 1)) * 2u));
            sr[rb][en] = rk < r ? static_cast<float>(h) : 0.f;
        }
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---------------------------------------------------------------- stage 3 loads (issued later) ---
    // Block b = 128 output columns; a wave owns a run of consecutive blocks (or blocks w, w + NW, ...); lane (li, q) owns columns 8 li .. 8 li + 7 of
    // the block for its token rows.
    // gridDim.y workgroups may share a token tile (small T: most of the chip would idle otherwise): each repeats stages 1
    // and 2, which costs no extra HBM traffic worth naming at such T, and takes its own contiguous range of blocks.
    const int nblk_all = (d_out + 127) >> 7;
    const int per_wg = SPLIT ? a.blocks_per_wg : nblk_all;
    const int b_first = SPLIT ? static_cast<int>(blockIdx.y) * per_wg : 0;
    const int nblk = nblk_all - b_first < per_wg ? (nblk_all - b_first > 0 ? nblk_all - b_first : 0) : per_wg;
    // A wave owns CONSECUTIVE blocks (its blocks in flight are then one contiguous piece of each row: 512 bytes per row at
    // the headline shape instead of two pieces 4 KiB apart: C2 9.99 -> 9.61 us, 4096 -> 11008 at T = 4096 42.1 -> 39.7),
    // The multi-adapter batch keeps the round-robin deal, which measured faster there.
    constexpr bool CB = GM != 4;
    // Runs of ceil(nblk / NW) blocks while that leaves the last wave at least half a run (108 blocks over 8 waves: 14 .. 14 10,
    // measured 1.5 % faster than 14 14 14 14 13 13 13 13); otherwise the first nblk mod NW waves own one block more than
    // the others (40 blocks over 16 waves: 3 .. 3 2 .. 2; runs of 3 would leave two waves without a block and cost 8 %).
    const int b_run = (nblk + NW - 1) / NW;
    const bool even_runs = 2 * (nblk - (NW - 1) * b_run) >= b_run;
    const int b_each = nblk / NW, b_more = nblk - b_each * NW;
    const int b_start = even_runs ? wave * b_run : wave * b_each + (wave < b_more ? wave : b_more);
    const int b_mine = even_runs ? (nblk - wave * b_run < b_run ? nblk - wave * b_run : b_run) : b_each + (wave < b_more ? 1 : 0);
    const int my_b = CB ? (b_mine > 0 ? b_mine : 0) : (wave < nblk ? (nblk - wave + NW - 1) / NW : 0);
    auto block_of = [&](int n) { return CB ? b_start + n : wave + NW * n; };  // the wave's n-th block (relative to b_first)
    const int64_t nwordsB = (static_cast<int64_t>(d_out) * r + 31) >> 5;
    u4 ybuf[D2][NI];
    u4 sobuf[D2][L];
    u4 bbuf[D2][R16 ? RB : 1];

    auto issue_y = [&](int slot, int n) {
        int b = b_first + block_of(n);
        const bool mine = n < my_b;  // (past the wave's share: with buffer accesses the rows of y_base are not requested)
        b = b < nblk_all ? b : nblk_all - 1;  // past the end: re-read a valid block, the result is not used
        int j0 = b * 128 + li * 8;
        j0 = j0 < d_out ? j0 : d_out - 8;
        if (R16) {  // 8 rows of r bits = RB * 16 contiguous, 16-byte aligned bytes
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) bbuf[slot][rb] = load16(at(a.pB, static_cast<uint32_t>(j0 * (r >> 3) + rb * 16)));
        }
        if (R8) {  // 8 rows of 8 bits: one aligned 8-byte load, byte e is column e
            const uint2 w = *static_cast<const uint2*>(at(a.pB, static_cast<uint32_t>(j0)));
            bbuf[slot][0] = u4{w.x, w.y, 0u, 0u};
        }
#pragma unroll
        for (int en = 0; en < L; ++en) sobuf[slot][en] = load16(at(a.s_out, static_cast<uint32_t>(en * d_out + j0) * 2u));
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            int row = TMV == 16 ? q * 4 + i : q * 2 + i;
            const bool live = row >= first && row <= last;
            row = row < last ? row : last;
            row = row > first ? row : first;
            if (BUFY) {
                ybuf[slot][i] = buffer_load16_stream(yb_rs, (mine && (!MASK || live)) ? static_cast<uint32_t>(row * d_out + j0) * 2u : kBufferSkip);
            } else if (MASK) {
                ybuf[slot][i] = u4{0u, 0u, 0u, 0u};
                if (live) ybuf[slot][i] = load16_stream(at(ybt, static_cast<uint32_t>(row * d_out + j0) * 2u));
            } else {
                ybuf[slot][i] = load16_stream(at(ybt, static_cast<uint32_t>(row * d_out + j0) * 2u));
            }
        }
    };

    // ---------------------------------------------------------------- stage 0: +-1 table -------------
    // Only used after the barriers of stage 2, which also make it visible.
    for (int e = tid; e < 256; e += NW * 64) lutp[e] = pm_one_from_bits(static_cast<uint32_t>(e) * 0x10001u);

    // ---------------------------------------------------------------- stage 1: sign(A) reduction ---
    // Every wave works on wave-private LDS as soon as its own data has arrived.  The barrier waits for no data: it only
    // keeps the fast waves from requesting y_base before the slow ones (held back by the bounded request queue) have
    // requested their x.
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    f4 acc[RB][L];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
        for (int en = 0; en < L; ++en) acc[rb][en] = f4{0.f, 0.f, 0.f, 0.f};
    }

    auto consume_x = [&](int slot) {
        _Float16* sw = sinw + slot * L * 128;
#pragma unroll
        for (int en = 0; en < L; ++en) reinterpret_cast<uint32_t*>(sw + en * 128)[lane] = sinbuf[slot][en];
#pragma unroll
        for (int m = 0; m < NI; ++m) store16(xs + (m * 4 + q) * kXRow + li * 8, xbuf[slot][m]);
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const h8 xf = as_h8(load16(xs + tile_row_of_mfma_row<TMV>(li) * kXRow + q * 32 + s * 8));
            u4 sv[L];
#pragma unroll
            for (int en = 0; en < L; ++en) sv[en] = load16(sw + en * 128 + q * 32 + s * 8);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                // byte s of the lane's carrier dword into the low byte of both halves (the other bytes are shifted out)
                const uint32_t both = __builtin_amdgcn_perm(abits[slot][rb], abits[slot][rb], 0x00010001u * s);
#pragma unroll
                for (int en = 0; en < L; ++en)
                    acc[rb][en] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xf, as_h8(flip_by_bits(sv[en], both)), acc[rb][en], 0, 0, 0);
            }
        }
        __builtin_amdgcn_wave_barrier();
    };

    if constexpr (CA) {
        if (wide_a) {  // lane group q now gets word q of every slot's chunk
#pragma unroll
            for (int g = 0; g < AG; ++g) {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    transpose_lane_groups(awide[g][rb]);
#pragma unroll
                    for (int n = 0; n < 4; ++n)
                        if (g * 4 + n < D1) abits[g * 4 + n][rb] = awide[g][rb][n];
                }
            }
        }
    }
    if (OS) {
#pragma unroll
        for (int slot = 0; slot < D1; ++slot)
            if (slot < my_n) consume_x(slot);
    } else {
        const int ngroups = (my_n + D1 - 1) / D1;
        for (int g = 0; g + 1 < ngroups; ++g) {
#pragma unroll
            for (int slot = 0; slot < D1; ++slot) {
                consume_x(slot);
                issue_x(slot, (g + 1) * D1 + slot);
            }
        }
#pragma unroll
        for (int slot = 0; slot < D1; ++slot)
            if ((ngroups - 1) * D1 + slot < my_n) consume_x(slot);
    }
    // TR (training instantiation): t is also written, and with y_out == nullptr nothing else is computed.  The inference
    // instantiation carries none of this.
    const bool with_y = !TR || a.y_out != nullptr;  // uniform: a kernel argument
    if (with_y) {
#pragma unroll
        for (int slot = 0; slot < D2; ++slot) issue_y(slot, slot);
    }

    // ---------------------------------------------------------------- stage 2: reduce, scale, split -
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
        for (int en = 0; en < L; ++en)
            *reinterpret_cast<f4*>(red + (((wave * RB + rb) * L + en) * 64 + lane) * 4) = acc[rb][en];
    }

    // While the slower waves finish stage 1, build the sign operands of the first block (they do not depend on u).
    // K slots of one stage-3 MFMA: hi(u) of ranks 0..15, then lo(u) of ranks 0..15; lane group q supplies ranks
    // 8 (q & 1) .. 8 (q & 1) + 7 for both halves, i.e. byte (q & 1) of the 16-bit row of its column.
    const uint32_t sel_even = 0x00010001u * static_cast<uint32_t>(q & 1);        // row in the low half-word of a dword
    const uint32_t sel_odd = 0x00010001u * static_cast<uint32_t>(2 + (q & 1));   // row in the high half-word
    u4 pre[PRE ? 8 : 1];
    auto build_pre = [&]() {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (R8) {  // ranks 8..15 (odd q) are padding and meet u = 0: any sign will do there
                const uint32_t word = bbuf[0][0][e >> 2];
                pre[e] = pm_one_from_bits(__builtin_amdgcn_perm(word, word, 0x00010001u * static_cast<uint32_t>(e & 3)));
            } else {
                const uint32_t word = bbuf[0][0][e >> 1];
                pre[e] = pm_one_from_bits(__builtin_amdgcn_perm(word, word, (e & 1) ? sel_odd : sel_even));
            }
        }
    };
    // The waves that run stage 2 build theirs while they wait for the slower waves to finish stage 1.  The others idle
    // during stage 2 anyway: with LP they build theirs there, which takes the work off the slowest wave's way to the
    // first barrier; without LP (a few workgroups, latency-bound) everything is built as early as possible.
    if (PRE && (!LP || wave < 4) && with_y) build_pre();
    __syncthreads();

    // Training: the rank-r intermediate t (before the rank scaling) is kept for the backward pass.  The stores are issued
    // after everything else: vector memory stores count in the same counter as the loads and may complete out of order
    // with them, so that a wait for y_base issued after such a store could also have to wait for the store.
    constexpr int SG = (L >= 3 && NW >= 8) ? 2 : 1;  // groups of four waves that share the envelopes of stage 2
    float tkeep[TR ? RB * L : 1];
    auto export_t = [&]() {
        if constexpr (TR) {
            if (wave < 4 * SG && a.t_out != nullptr) {
                const int i = wave & 3, grp = wave >> 2;
                const int row = TMV == 16 ? q * 4 + i : q * 2 + (i & 1);
                if ((TMV == 16 || i < 2) && row >= first && row <= last) {
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
                        for (int en = 0; en < L; ++en)
                            if (en % SG == grp && rb * 16 + li < r)
                                a.t_out[(static_cast<int64_t>(en) * r + rb * 16 + li) * a.t_stride + t0 + row] = tkeep[rb * L + en];
                    }
                }
            }
        }
    };
    if (wave < 4 * SG) {
        // Accumulator layout: lane (li, q) holds rank li of the block for MFMA rows 4q .. 4q+3; wave i takes row 4q+i.
        // With several envelopes and at least 8 waves, waves 0..3 take the even envelopes and waves 4..7 the odd ones.
        const int i = wave & 3, grp = wave >> 2;
#pragma unroll
        for (int en = 0; en < L; ++en) {
            if (SG > 1 && en % SG != grp) continue;
            float u[RB];
            float amax = 0.f;
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                float part[NW];  // all partial sums are requested before the first add; fixed order: deterministic
#pragma unroll
                for (int w = 0; w < NW; ++w) part[w] = red[(((w * RB + rb) * L + en) * 64 + lane) * 4 + i];
#pragma unroll
                for (int st = 1; st < NW; st <<= 1) {
#pragma unroll
                    for (int w = 0; w + st < NW; w += 2 * st) part[w] += part[w + st];
                }
                if constexpr (TR) tkeep[rb * L + en] = part[0];  // training: t is written out at the very end (see export_t)
                u[rb] = part[0] * sr[rb][en];
                amax = fmaxf(amax, fabsf(u[rb]));
            }
            const float rowmax = row_max16(amax);  // over the 16 ranks of a block; amax already spans the blocks
            int e = static_cast<int>((__float_as_uint(rowmax) >> 23) & 0xffu);
            e = e < 14 ? 14 : (e > 254 ? 254 : e);
            const float mul = __uint_as_float(static_cast<uint32_t>(267 - e) << 23);  // 2^(13 - (e - 127))
            if (li == 0) invs[en * 16 + q * 4 + i] = __uint_as_float(static_cast<uint32_t>(e - 13) << 23);  // its reciprocal
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                const float up = u[rb] * mul;
                const _Float16 hi = static_cast<_Float16>(up);
                const _Float16 lo = static_cast<_Float16>(up - static_cast<float>(hi));
                us[((rb * L + en) * 16 + q * 4 + i) * kURow + li] = hi;
                us[((rb * L + en) * 16 + q * 4 + i) * kURow + 16 + li] = lo;
            }
        }
    } else if (PRE && LP && with_y) {
        build_pre();
    }
    __syncthreads();
    if (!with_y) {  // every wave has passed the last barrier
        export_t();
        return;
    }
    // With 8 token rows, MFMA rows 4a+2 and 4a+3 only repeat rows 4a and 4a+1: in stage 3 they carry the SECOND envelope of
    // a pair instead, so that two envelopes cost the matrix-core work and the accumulator registers of one.
    constexpr int VS = TMV == 8 ? (L + 1) / 2 : L;  // accumulator sets per output column
    h8 ufrag[RB][VS];
    float inv[LEAN ? 1 : NI][LEAN ? 1 : L];
#pragma unroll
    for (int vs = 0; vs < VS; ++vs) {
        int en = vs;
        if (TMV == 8 && L > 1) {
            en = 2 * vs + ((li >> 1) & 1);
            en = en < L ? en : L - 1;  // odd L: the spare rows repeat the last envelope and are ignored
        }
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) ufrag[rb][vs] = as_h8(load16(us + ((rb * L + en) * 16 + li) * kURow + q * 8));
    }
    if constexpr (!LEAN) {
#pragma unroll
        for (int en = 0; en < L; ++en) {
#pragma unroll
            for (int i = 0; i < NI; ++i) inv[i][en] = invs[en * 16 + q * 4 + i];
        }
    }

    // ---------------------------------------------------------------- stage 3: expand + epilogue ----
    // MFMA e of a block produces column 8 li + e of the block for lane group li, so after the 8 MFMAs a lane holds 8
    // consecutive columns of its token rows.
    auto store_y = [&](int row, int j0, bool j_ok, u4 out) {
        const bool wanted = j_ok && row >= first && row <= last;
        const uint32_t off = static_cast<uint32_t>(row * d_out + j0) * 2u;
        if (BUFY) buffer_store16_stream(yo_rs, wanted ? off : kBufferSkip, out);
        else if (wanted) store16_stream(at(yot, off), out);
    };
    // (`run` false, only with buffer accesses: nothing is computed or stored, but the same vector memory instructions are issued)
    auto consume_y = [&](int slot, int n, bool use_pre, bool run) {
        const int b = b_first + block_of(n);
        const int j0 = b * 128 + li * 8;
        const bool j_ok = j0 < d_out;
        const int jc = j_ok ? j0 : d_out - 8;
        if (!run) {
#pragma unroll
            for (int i = 0; i < NI; ++i) store_y(0, 0, false, u4{0u, 0u, 0u, 0u});
            return;
        }
        // Table offsets of all 8 * RB sign operands first (for a general r these are global loads: one wait for all).
        uint32_t off[8][RB];
        if (!(PRE && use_pre)) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    if (R16) {
                        const int hw = e * RB + rb;  // half-word index inside the lane's RB * 8 half-words
                        const uint32_t word = bbuf[slot][hw >> 3][(hw >> 1) & 3] >> ((q & 1) * 8);
                        off[e][rb] = (hw & 1) ? (word >> 12) & 0xff0u : (word << 4) & 0xff0u;
                    } else if (R8) {
                        off[e][rb] = ((bbuf[slot][0][e >> 2] >> ((e & 3) * 8)) << 4) & 0xff0u;
                    } else {
                        off[e][rb] = fetch8(a.pB, static_cast<int64_t>(jc + e) * r + rb * 16 + (q & 1) * 8, nwordsB) << 4;
                    }
                }
            }
        }
        // The sign operand of (column e, rank block rb): built ahead for the first block; otherwise from the table (measured
        // faster than building it here with the vector ALU, which stage 3 needs for the epilogue).
        auto sign_operand = [&](int e, int rb) -> u4 {
            return (PRE && use_pre) ? pre[e] : *reinterpret_cast<const u4*>(reinterpret_cast<const unsigned char*>(lutp) + off[e][rb]);
        };
        if constexpr (L == 1) {
            f4 v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                v[e] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
                    v[e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ufrag[rb][0], as_h8(sign_operand(e, rb)), v[e], 0, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int row = TMV == 16 ? q * 4 + i : q * 2 + i;
                u4 out;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const h2 b = as_h2(ybuf[slot][i][d]);
                    const h2 so = as_h2(sobuf[slot][0][d]);
                    // y_out = fp16(fp32 fma): the fp32 result is made opaque so that every variant rounds twice (to fp32, then
                    // to fp16); left alone, the compiler fuses some of these pairs into one instruction that rounds once.
                    float f0 = __builtin_fmaf(v[2 * d][i] * inv[i][0], static_cast<float>(so[0]), static_cast<float>(b[0]));
                    float f1 = __builtin_fmaf(v[2 * d + 1][i] * inv[i][0], static_cast<float>(so[1]), static_cast<float>(b[1]));
                    asm("" : "+v"(f0));
                    asm("" : "+v"(f1));
                    h2 o;
                    o[0] = static_cast<_Float16>(f0);
                    o[1] = static_cast<_Float16>(f1);
                    out[d] = __builtin_bit_cast(uint32_t, o);
                }
                store_y(row, j0, j_ok, out);
            }
        } else {
            // Several envelopes: the accumulator sets are run one after the other into the same registers, and each set is
            // folded at once into the fp32 outputs of the lane's 8 columns (which start from y_base), so the register cost
            // is one accumulator set plus 8 NI floats whatever L is.  The sign operands are read again per set (LDS).
            // Envelopes are added in their order, in fp32; one rounding at the end.
            float o[NI][8];
#pragma unroll
            for (int i = 0; i < NI; ++i) {
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const h2 b = as_h2(ybuf[slot][i][d]);
                    o[i][2 * d] = static_cast<float>(b[0]);
                    o[i][2 * d + 1] = static_cast<float>(b[1]);
                }
            }
            constexpr int EH = (D2 > 2 || (TMV == 16 && L >= 3)) ? 4 : 8;   // columns per pass: half a set at a time where more blocks are in flight
#pragma unroll
            for (int vs = 0; vs < VS; ++vs) {
                // With three or four rank blocks the compiler would keep the 8 RB sign operands of the first set in
                // registers for the next one (same LDS addresses) and spill; this makes it read them again.
                if constexpr (RB >= 3) asm volatile("" ::: "memory");
#pragma unroll
                for (int e0 = 0; e0 < 8; e0 += EH) {
                    f4 v[EH];
#pragma unroll
                    for (int e = 0; e < EH; ++e) {
                        v[e] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int rb = 0; rb < RB; ++rb)
                            v[e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ufrag[rb][vs], as_h8(sign_operand(e0 + e, rb)), v[e], 0, 0, 0);
                    }
#pragma unroll
                    for (int sub = 0; sub < (TMV == 8 ? 2 : 1); ++sub) {
                        const int en = TMV == 8 ? 2 * vs + sub : vs;   // 8-row tiles: the set carries a pair of envelopes
                        if (en < L) {
#pragma unroll
                            for (int i = 0; i < NI; ++i) {
                                const int vi = TMV == 8 ? i + 2 * sub : i;   // the envelope's register inside the set
                                float iv;
                                if constexpr (LEAN) iv = invs[en * 16 + q * 4 + i];
                                else iv = inv[i][en];
#pragma unroll
                                for (int d = e0 / 2; d < (e0 + EH) / 2; ++d) {
                                    const h2 so = as_h2(sobuf[slot][en][d]);
                                    o[i][2 * d] = __builtin_fmaf(v[2 * d - e0][vi] * iv, static_cast<float>(so[0]), o[i][2 * d]);
                                    o[i][2 * d + 1] = __builtin_fmaf(v[2 * d + 1 - e0][vi] * iv, static_cast<float>(so[1]), o[i][2 * d + 1]);
                                }
                            }
                        }
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int row = TMV == 16 ? q * 4 + i : q * 2 + i;
                u4 out;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    h2 oh;
                    asm("" : "+v"(o[i][2 * d]));      // (round to fp32, then to fp16, in every variant: see the one-envelope epilogue)
                    asm("" : "+v"(o[i][2 * d + 1]));
                    oh[0] = static_cast<_Float16>(o[i][2 * d]);
                    oh[1] = static_cast<_Float16>(o[i][2 * d + 1]);
                    out[d] = __builtin_bit_cast(uint32_t, oh);
                }
                store_y(row, j0, j_ok, out);
            }
        }
    };

    // 8-row tiles on 8 waves with more blocks than the waves hold in flight: every pass of the loop issues the same vector
    // memory instructions whatever the wave's number of blocks is (what is not wanted is skipped by its offset), so that
    // the wait for a slot's y_base leaves the later requests and the stores in flight; with requests under branches the
    // compiler has to wait for all of them.
    constexpr bool kSteadyLoop = BUFY && GM != 4;
    if constexpr (kSteadyLoop) {
        if (my_b > 0) consume_y(0, 0, true, true);
        if (nblk > NW * D2) {
            for (int n0 = 0; n0 < my_b; n0 += D2) {
#pragma unroll
                for (int slot = 0; slot < D2; ++slot) {
                    const int n = n0 + slot;
                    consume_y(slot, n, false, n != 0 && n < my_b);
                    issue_y(slot, n + D2);
                }
            }
        } else {
            if (my_b > D2) issue_y(0, D2);
            for (int n0 = 0; n0 < my_b; n0 += D2) {
#pragma unroll
                for (int slot = 0; slot < D2; ++slot) {
                    const int n = n0 + slot;
                    if (n == 0) continue;
                    if (n < my_b) consume_y(slot, n, false, true);
                    if (n + D2 < my_b) issue_y(slot, n + D2);
                }
            }
        }
    } else {
        // (kept in exactly this shape: with the first block's request for its successor outside the branch, the
        // three-envelope variants with four rank blocks spill)
        if (my_b > 0) {
            consume_y(0, 0, true, true);
            if (D2 < my_b) issue_y(0, D2);
        }
        for (int n0 = 0; n0 < my_b; n0 += D2) {
#pragma unroll
            for (int slot = 0; slot < D2; ++slot) {
                const int n = n0 + slot;
                if (n == 0) continue;
                if (n < my_b) consume_y(slot, n, false, true);
                if (n + D2 < my_b) issue_y(slot, n + D2);
            }
        }
    }
    export_t();
}

// The second launch bound is the number of waves per SIMD the registers must leave room for: what the workgroup size
// implies, except in the multi-adapter batch on 8 waves (one envelope; one rank block, or two with whole-word carrier rows),
// where two workgroups have to share a compute unit.
template <int RB, int TMV, int NW, int D1, bool OS, int BM, int GM, int L, bool TR>
__global__ __launch_bounds__(NW * 64, (GM == 4 && NW == 8 && L == 1 && (RB == 1 || (RB == 2 && BM == 1))) ? 4 : NW / 4) void lordba_fwd_mfma_kernel(FwdArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    if constexpr (GM != 4) {
        const int64_t t0 = static_cast<int64_t>(blockIdx.x) * TMV;
        if ((GM == 2 || GM == 3) && t0 >= a.T) return;  // padding workgroup (the whole workgroup leaves, before any barrier)
        const int last = static_cast<int>(a.T - 1 - t0 < TMV - 1 ? a.T - 1 - t0 : TMV - 1);  // last live row of the tile
        fwd_tile<RB, TMV, NW, D1, OS, BM, GM, L, TR>(a, smem, t0, 0, last);
    } else {
        // Multi-adapter batch: the rows of a tile are taken in runs of equal adapter index.  A tile of a sorted batch has
        // one run (two where requests meet), a decode batch has one per row.  The gridDim.y workgroups of a tile share its
        // runs: workgroup y takes runs y, y + gridDim.y, ... and leaves if it has none.  The host launches 8 per tile while
        // the tiles are few (every run of a decode batch in parallel; the compute units would idle otherwise) and 2 on
        // grids that fill the chip: there the first workgroup of a tile of a sorted batch does all the work and the second
        // only finds out that it has none, which still holds a slot of a compute unit for most of a microsecond - the
        // workgroups have 8 waves, two fit a compute unit, so these pass through the second slot while the first works.
        // A workgroup's first run is straight-line code; further runs of the same workgroup go through a loop around a
        // second copy of the tile code, which compiles to about twice the time per run (spills, conservative waits) but
        // is only met by tiles with more runs than workgroups.
        // Consecutive tiles go to the same XCD (workgroups are dealt to the 8 XCDs round-robin in launch order): the tiles
        // of one request then read their adapter through one L2 instead of pulling it into several.
        static_assert(TMV == 8, "runs are found among 8 rows");
        const int64_t tiles = (static_cast<int64_t>(a.T) + TMV - 1) / TMV, per_xcd = (tiles + 7) >> 3;
        const bool by_xcd = a.blocks_per_wg != 0;  // (set by the host on grids that fill the chip; the x extent is then padded)
        const int64_t tile = by_xcd ? static_cast<int64_t>(blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3) : static_cast<int64_t>(blockIdx.x);
        if (tile >= tiles) return;  // padding workgroup
        const int64_t t0 = tile * TMV;
        const int last = static_cast<int>(a.T - 1 - t0 < TMV - 1 ? a.T - 1 - t0 : TMV - 1);
        const int lane = threadIdx.x & 63;
        int my_id = -1;
        if ((lane & 7) <= last) my_id = a.ids[t0 + (lane & 7)];
        if (my_id >= a.n_adapters) my_id = -1;
        auto run_end = [&](int first) {  // last row of the run that starts at `first` (scalar walk, same in every wave)
            const int id = __builtin_amdgcn_readlane(my_id, first);
            int end = first;
            while (end < last && __builtin_amdgcn_readlane(my_id, end + 1) == id) ++end;
            return end;
        };
        auto pass_through = [&](int first, int end) {  // no adapter: the rows pass through
            if (a.y_out == a.y_base) return;
            for (int row = first; row <= end; ++row) {
                const _Float16* src = a.y_base + (t0 + row) * a.d_out;
                _Float16* dst = a.y_out + (t0 + row) * a.d_out;
                for (int c = static_cast<int>(threadIdx.x) * 8; c < a.d_out; c += NW * 64 * 8)
                    store16_stream(dst + c, load16_stream(src + c));
            }
        };
        auto skip_runs = [&](int first, int n) {  // start of the run n runs after the one that starts at `first` (> last: none)
            for (int k = 0; k < n && first <= last; ++k) first = run_end(first) + 1;
            return first;
        };
        const int stride = static_cast<int>(gridDim.y);
        int first = skip_runs(0, static_cast<int>(blockIdx.y));
        if (first > last) return;  // no run for this workgroup: it leaves, before any barrier
        {
            const int end = run_end(first), id = __builtin_amdgcn_readlane(my_id, first);
            if (id >= 0) fwd_tile<RB, TMV, NW, D1, OS, BM, GM, L, TR>(select_adapter(a, id), smem, t0, first, end);
            else pass_through(first, end);
            first = skip_runs(end + 1, stride - 1);
        }
        while (first <= last) {
            const int end = run_end(first), id = __builtin_amdgcn_readlane(my_id, first);
            __syncthreads();  // the previous run's last LDS reads are over
            if (id >= 0) fwd_tile<RB, TMV, NW, D1, OS, BM, GM, L, TR>(select_adapter(a, id), smem, t0, first, end);
            else pass_through(first, end);
            first = skip_runs(end + 1, stride - 1);
        }
    }
}

// ------------------------------------------------------------------------------------ general kernel ----
// PLAIN: one envelope, no adapter pool (known at compile time: the envelope loop and the index lookup disappear).
template <int RP, bool PLAIN>
__global__ __launch_bounds__(256) void lordba_fwd_general_kernel(FwdArgs a0, int vec_x) {
    __shared__ float red[4][RP];
    __shared__ float u_s[LORDBA_MAX_ENVELOPES][RP];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t t = blockIdx.x;
    FwdArgs a = a0;
    if (!PLAIN && a0.ids != nullptr) {  // multi-adapter batch: this row's adapter, or none
        const int id = a0.ids[t];
        if (id < 0 || id >= a0.n_adapters) {
            if (a0.y_out != a0.y_base)
                for (int j = tid; j < a0.d_out; j += 256) a0.y_out[t * a0.d_out + j] = a0.y_base[t * a0.d_out + j];
            return;
        }
        a = select_adapter(a0, id);
    }
    const int d_in = a.d_in, d_out = a.d_out, r = a.r, ell = PLAIN ? 1 : a.ell;
    const _Float16* xr = a.x + t * d_in;

    for (int en = 0; en < ell; ++en) {  // u of every envelope (Eq. (lordba): the carriers are shared, the scales are not)
        const _Float16* s_in = a.s_in + static_cast<int64_t>(en) * d_in;
        float acc[RP];
#pragma unroll
        for (int k = 0; k < RP; ++k) acc[k] = 0.f;

        if (vec_x) {  // d_in % 8 == 0, x and s_in 16-byte aligned: 8 columns per lane per step, one carrier byte per rank
            const uint8_t* bytesA = reinterpret_cast<const uint8_t*>(a.pA);
            for (int i0 = tid * 8; i0 < d_in; i0 += 256 * 8) {
                const h8 xv = as_h8(load16(xr + i0));
                const h8 sv = as_h8(load16(s_in + i0));
                float w[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) w[e] = static_cast<float>(xv[e]) * static_cast<float>(sv[e]);
                // one carrier byte per rank, a row of sign(A) apart: a running per-lane pointer instead of RP row bases
                const uint8_t* pk = bytesA + (i0 >> 3);
                const int row_bytes = d_in >> 3;
#pragma unroll
                for (int k = 0; k < RP; ++k) {
                    if (k < r) {
                        const uint32_t byte = *pk;
                        pk += row_bytes;
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[k] += flip(w[e], (byte >> e) & 1u);
                    }
                }
            }
        } else {
            for (int i = tid; i < d_in; i += 256) {
                const float w = static_cast<float>(xr[i]) * static_cast<float>(s_in[i]);
#pragma unroll
                for (int k = 0; k < RP; ++k) {
                    if (k < r) {
                        const int64_t n = static_cast<int64_t>(k) * d_in + i;
                        acc[k] += flip(w, (a.pA[n >> 5] >> (n & 31)) & 1u);
                    }
                }
            }
        }
#pragma unroll
        for (int k = 0; k < RP; ++k) {
            float v = acc[k];
#pragma unroll
            for (int sh = 32; sh >= 1; sh >>= 1) v += __shfl_xor(v, sh, 64);
            if (lane == 0) red[wave][k] = v;
        }
        __syncthreads();
        if (tid < RP) {
            const float tk = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
            u_s[en][tid] = tid < r ? static_cast<float>(a.s_rank[en * r + tid]) * tk : 0.f;
            if (a.t_out != nullptr && a0.ids == nullptr && tid < r) a.t_out[(static_cast<int64_t>(en) * r + tid) * a.t_stride + t] = tk;
        }
        __syncthreads();
    }
    if (a.y_out == nullptr) return;  // only t was wanted
    const _Float16* ybr = a.y_base + t * d_out;
    _Float16* yor = a.y_out + t * d_out;
    for (int j = tid; j < d_out; j += 256) {
        float o = static_cast<float>(ybr[j]);
        const int64_t n0 = static_cast<int64_t>(j) * r;
        for (int en = 0; en < ell; ++en) {
            float v = 0.f;
            for (int k = 0; k < r; ++k) {
                const int64_t n = n0 + k;
                v += flip(u_s[en][k], (a.pB[n >> 5] >> (n & 31)) & 1u);
            }
            o = o + static_cast<float>(a.s_out[static_cast<int64_t>(en) * d_out + j]) * v;
        }
        yor[j] = static_cast<_Float16>(o);
    }
}

// ------------------------------------------------------------------------------------------ host side ----

constexpr size_t kMaxLds = 160 * 1024;  // LDS per CU on gfx950

// A translation unit holds either the inference instantiations of the matrix-core kernel (LORDBA_FWD_TRAINING 0, the
// default) or the training ones, which also keep t (LORDBA_FWD_TRAINING 1); every entry point lives in a unit of the
// matching kind, so that the units compile side by side and none carries both sets.
#ifndef LORDBA_FWD_TRAINING
#define LORDBA_FWD_TRAINING 0
#endif
constexpr bool kTraining = LORDBA_FWD_TRAINING != 0;

template <int RB, int TMV, int NW, int D1, bool OS, int BM, int GM, int L>
lordba_status launch_mfma_gm(const FwdArgs& a, hipStream_t stream) {
    constexpr bool TR = kTraining;
    if ((a.t_out != nullptr) != TR) return LORDBA_ERR_ALGO;  // (an entry point of the other kind of unit)
    // With several envelopes only the plain grid mode of the 8-row, 8-wave variants has a training instantiation (the
    // dispatch sends such calls there); the multi-adapter batch has none.
    if constexpr (TR && !((L == 1 && GM != 4) || (L > 1 && GM == 0 && TMV == 8 && NW == 8))) {
        return LORDBA_ERR_ALGO;
    } else {
    const size_t lds = mfma_lds_bytes(RB, TMV, NW, D1, L);
    if (lds > kMaxLds) return LORDBA_ERR_ALGO;
    auto kern = lordba_fwd_mfma_kernel<RB, TMV, NW, D1, OS, BM, GM, L, TR>;
    if (lds > 64 * 1024) {
        // Opt in to more than 64 KiB of dynamic LDS once per device and kernel; raising the limit is idempotent.
        static std::mutex mu;
        static bool granted[64] = {false};
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return LORDBA_ERR_NO_DEVICE;
        std::lock_guard<std::mutex> g(mu);
        if (!granted[dev]) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    static_cast<int>(kMaxLds)) != hipSuccess) {
                (void)hipGetLastError();
                return LORDBA_ERR_LAUNCH;
            }
            granted[dev] = true;
        }
    }
    const unsigned tiles = static_cast<unsigned>((static_cast<int64_t>(a.T) + TMV - 1) / TMV);
    FwdArgs b = a;
    dim3 grid(tiles);
    if constexpr (GM == 2 || GM == 3) {
        // A handful of tiles leaves most CUs idle and each workgroup with a long serial stage 3: the output blocks of a
        // tile are split over several workgroups (each repeats the cheap stages 1 and 2; nothing is exchanged).
        const unsigned nblk = static_cast<unsigned>((a.d_out + 127) / 128);
        unsigned split = (nblk + kSplitBlocks - 1) / kSplitBlocks;
        const unsigned cap = 256 / tiles;
        split = split < cap ? split : cap;
        split = split < 1 ? 1 : split;
        b.blocks_per_wg = static_cast<int>((nblk + split - 1) / split);
        split = (nblk + b.blocks_per_wg - 1) / b.blocks_per_wg;  // no workgroup without a block
        // Workgroups are dealt to the 8 XCDs round-robin in launch order (x fastest).  With an x extent that is a
        // multiple of 8, the workgroups that share a tile (same x) land on one XCD and read x, s_in and the carriers
        // through one L2 instead of fetching them into eight; the padding workgroups exit at once.
        grid = dim3((tiles + 7u) & ~7u, split);
    }
    if constexpr (GM == 4) {  // see the kernel
        const bool big = tiles > 32;
        b.blocks_per_wg = big ? 1 : 0;  // (read by the kernel as "tiles are dealt to the XCDs in contiguous ranges")
        grid = big ? dim3((tiles + 7u) & ~7u, 2) : dim3(tiles, TMV);
    }
    hipLaunchKernelGGL(kern, grid, dim3(NW * 64), lds, stream, b);
    return hipGetLastError() == hipSuccess ? LORDBA_OK : LORDBA_ERR_LAUNCH;
    }
}

// Grid mode 1 only exists where sign operands are built ahead (one rank block, byte-aligned carrier rows); it pays once
// the grid covers the chip, where the slowest wave at the first barrier sets the pace of the workgroup.  Grid mode 2
// is for 8-row tiles when there are at most 32 of them, grid mode 3 for a single partial tile (decode).
template <int RB, int TMV, int NW, int D1, bool OS, int BM, int L>
lordba_status launch_mfma(const FwdArgs& a, hipStream_t stream) {
    const int64_t tiles = (static_cast<int64_t>(a.T) + TMV - 1) / TMV;
    if (a.ids != nullptr) {
        // (two rank blocks on 16 waves would spill a few registers in the batch mode's second copy of the tile code: 8 waves)
        // Pools of adapters with several envelopes run the 8-wave variants (one workgroup per compute unit) up to r = 32 (r = 16 with four envelopes); beyond
        // that the registers do not hold the batch mode's two copies of the tile code, and the general kernel runs.
        if constexpr (TMV == 8 && D1 <= 4 && ((L == 1 && (NW == 8 || (NW == 16 && RB == 1))) || (L > 1 && NW == 8 && (RB == 1 || (RB == 2 && L <= 3))))) {
            return launch_mfma_gm<RB, TMV, NW, D1, OS, BM, 4, L>(a, stream);
        }
        return LORDBA_ERR_ALGO;
    }
    if constexpr (L > 1) {
        if (a.t_out != nullptr) return launch_mfma_gm<RB, TMV, NW, D1, OS, BM, 0, L>(a, stream);  // see launch_mfma_gm
    }
    if constexpr (RB == 1 && BM != 0 && L == 1) {
        if (tiles >= 128) return launch_mfma_gm<RB, TMV, NW, D1, OS, BM, 1, L>(a, stream);
    }
    if constexpr (TMV == 8 && NW >= 8) {
        if (a.T < TMV) return launch_mfma_gm<RB, TMV, NW, D1, OS, BM, 3, L>(a, stream);
        if (tiles <= 32 && a.d_out > static_cast<int>(kSplitBlocks) * 128) return launch_mfma_gm<RB, TMV, NW, D1, OS, BM, 2, L>(a, stream);
    }
    return launch_mfma_gm<RB, TMV, NW, D1, OS, BM, 0, L>(a, stream);
}

// Picks the x pipeline: one-shot when every wave's chunks fit the deepest pipeline that the register budget of the
// workgroup size allows, otherwise the looped variant.
template <int RB, int TMV, int NW, int BM, int L>
lordba_status launch_mfma_depth(const FwdArgs& a, hipStream_t stream) {
    constexpr bool kDeep = TMV == 8 && NW <= 8 && RB == 1 && L == 1;  // 8 chunks in flight only where the registers allow it
    const int nchunks = (a.d_in + 127) / 128;
    const int per_wave = (nchunks + NW - 1) / NW;
    if (per_wave <= 2) return launch_mfma<RB, TMV, NW, 2, true, BM, L>(a, stream);
    if (per_wave <= 4) return launch_mfma<RB, TMV, NW, 4, true, BM, L>(a, stream);
    if (kDeep && per_wave <= 8 && a.ids == nullptr) return launch_mfma<RB, TMV, NW, (kDeep ? 8 : 4), true, BM, L>(a, stream);  // (the batch mode has 128 registers)
    return launch_mfma<RB, TMV, NW, (TMV == 8 ? 4 : 2), false, BM, L>(a, stream);
}

template <int TMV, int NW, int L>
lordba_status launch_mfma_rb(const FwdArgs& a, hipStream_t stream) {
    // Rank blocks a variant holds in registers without spilling.  16 waves: 128 registers per lane.  Several envelopes
    // keep L accumulator sets per block: 16-row tiles then only fit two envelopes of at most two rank blocks.
    constexpr int kMaxRb = NW == 16 ? (L == 1 ? (TMV == 8 ? 2 : 1) : (L == 2 && TMV == 8 ? 1 : 0))
                           : L == 1 ? 4
                           : TMV == 16 ? (L == 2 ? 2 : 1)
                           : (L == 4 ? 3 : 4);
    const int rb = (a.r + 15) / 16;
    if (rb > kMaxRb) return LORDBA_ERR_ALGO;
    if constexpr (L == 1) {
        if (a.r == 8) return launch_mfma_depth<1, TMV, NW, 2, L>(a, stream);
    }
    const bool r16 = a.r % 16 == 0;
    if constexpr (kMaxRb >= 1) {
        if (rb == 1) return r16 ? launch_mfma_depth<1, TMV, NW, 1, L>(a, stream) : launch_mfma_depth<1, TMV, NW, 0, L>(a, stream);
    }
    if constexpr (kMaxRb >= 2) {
        if (rb == 2) return r16 ? launch_mfma_depth<2, TMV, NW, 1, L>(a, stream) : launch_mfma_depth<2, TMV, NW, 0, L>(a, stream);
    }
    if constexpr (kMaxRb >= 3) {
        if (rb == 3) return r16 ? launch_mfma_depth<3, TMV, NW, 1, L>(a, stream) : launch_mfma_depth<3, TMV, NW, 0, L>(a, stream);
    }
    if constexpr (kMaxRb >= 4) {
        if (rb == 4) return r16 ? launch_mfma_depth<4, TMV, NW, 1, L>(a, stream) : launch_mfma_depth<4, TMV, NW, 0, L>(a, stream);
    }
    return LORDBA_ERR_DIM;
}

template <bool PLAIN>
void launch_general_rp(const FwdArgs& a, hipStream_t stream, bool vec_x) {
    const dim3 grid(static_cast<unsigned>(a.T)), block(256);
    if (a.r <= 8) hipLaunchKernelGGL((lordba_fwd_general_kernel<8, PLAIN>), grid, block, 0, stream, a, vec_x ? 1 : 0);
    else if (a.r <= 16) hipLaunchKernelGGL((lordba_fwd_general_kernel<16, PLAIN>), grid, block, 0, stream, a, vec_x ? 1 : 0);
    else if (a.r <= 32) hipLaunchKernelGGL((lordba_fwd_general_kernel<32, PLAIN>), grid, block, 0, stream, a, vec_x ? 1 : 0);
    else hipLaunchKernelGGL((lordba_fwd_general_kernel<64, PLAIN>), grid, block, 0, stream, a, vec_x ? 1 : 0);
}

lordba_status launch_general(const FwdArgs& a, hipStream_t stream, bool vec_x) {
    if (a.ell == 1 && a.ids == nullptr) launch_general_rp<true>(a, stream, vec_x);
    else launch_general_rp<false>(a, stream, vec_x);
    return hipGetLastError() == hipSuccess ? LORDBA_OK : LORDBA_ERR_LAUNCH;
}

bool overlaps(const void* p, size_t pn, const void* q, size_t qn) {
    const uintptr_t a = reinterpret_cast<uintptr_t>(p), b = reinterpret_cast<uintptr_t>(q);
    return pn != 0 && qn != 0 && a < b + qn && b < a + pn;
}
bool aligned(const void* p, size_t n) { return (reinterpret_cast<uintptr_t>(p) & (n - 1)) == 0; }

// Validation and dispatch shared by the entry points; L = number of scale envelopes (compile-time in the kernels).
template <int L>
lordba_status forward_impl(const void* x, const uint32_t* packedA, const uint32_t* packedB,
                           const void* s_in, const void* s_rank, const void* s_out,
                           const void* y_base, void* y_out,
                           int64_t T, int64_t d_in, int64_t d_out, int64_t r, void* stream, int algo,
                           const int32_t* ids = nullptr, int64_t n_adapters = 1, bool batched = false,
                           float* t_out = nullptr, int64_t t_stride = 0) {
    if (T < 0 || d_in < 1 || d_out < 1 || r < 1 || r > LORDBA_MAX_RANK) return LORDBA_ERR_DIM;
    if (batched && (n_adapters < 1 || n_adapters > (1 << 20))) return LORDBA_ERR_DIM;
    if (T > INT32_MAX - 64 || d_in > (1 << 24) || d_out > (1 << 24)) return LORDBA_ERR_DIM;
    if (algo < 0 || algo > 7 || (L > 1 && (algo == 4 || algo == 5))) return LORDBA_ERR_ALGO;
    // With no token rows the activation pointers may legitimately be NULL (empty allocations).
    if (T == 0) return (packedA && packedB && s_in && s_rank && s_out) ? LORDBA_OK : LORDBA_ERR_NULL;
    const bool t_only = t_out != nullptr && y_base == nullptr && y_out == nullptr;  // training: only the rank-r intermediate
    if (!x || !packedA || !packedB || !s_in || !s_rank || !s_out) return LORDBA_ERR_NULL;
    if (!t_only && (!y_base || !y_out)) return LORDBA_ERR_NULL;
    if (t_out != nullptr && (batched || t_stride < T || t_stride > INT32_MAX || !aligned(t_out, 4))) return LORDBA_ERR_DIM;
    if (batched && !ids) return LORDBA_ERR_NULL;
    if (batched && !aligned(ids, 4)) return LORDBA_ERR_ALIGN;
    if (!aligned(x, 2) || !aligned(s_in, 2) || !aligned(s_rank, 2) || !aligned(s_out, 2) || !aligned(y_base, 2) ||
        !aligned(y_out, 2) || !aligned(packedA, 4) || !aligned(packedB, 4))
        return LORDBA_ERR_ALIGN;
    const size_t ny = t_only ? 0 : static_cast<size_t>(T) * d_out * 2, nx = static_cast<size_t>(T) * d_in * 2;
    const size_t np = static_cast<size_t>(batched ? n_adapters : 1);  // adapters behind the pool pointers
    const size_t nA = lordba_packed_words(r, d_in) * 4 * np, nB = lordba_packed_words(d_out, r) * 4 * np;
    if (overlaps(y_out, ny, x, nx) || overlaps(y_out, ny, packedA, nA) || overlaps(y_out, ny, packedB, nB) ||
        overlaps(y_out, ny, s_in, np * L * d_in * 2) || overlaps(y_out, ny, s_rank, np * L * r * 2) ||
        overlaps(y_out, ny, s_out, np * L * d_out * 2) || (batched && overlaps(y_out, ny, ids, static_cast<size_t>(T) * 4)))
        return LORDBA_ERR_ALIAS;
    if (y_out != y_base && overlaps(y_out, ny, y_base, ny)) return LORDBA_ERR_ALIAS;
    if (t_out != nullptr) {
        const size_t nt = (static_cast<size_t>(L * r - 1) * t_stride + T) * 4;
        if (overlaps(t_out, nt, x, nx) || overlaps(t_out, nt, y_out, ny) || overlaps(t_out, nt, y_base, ny))
            return LORDBA_ERR_ALIAS;
    }
    const lordba_status dev = check_device();
    if (dev != LORDBA_OK) return dev;

    FwdArgs a;
    a.x = static_cast<const _Float16*>(x);
    a.pA = packedA;
    a.pB = packedB;
    a.s_in = static_cast<const _Float16*>(s_in);
    a.s_rank = static_cast<const _Float16*>(s_rank);
    a.s_out = static_cast<const _Float16*>(s_out);
    a.y_base = static_cast<const _Float16*>(y_base);
    a.y_out = static_cast<_Float16*>(y_out);
    a.T = static_cast<int>(T);
    a.d_in = static_cast<int>(d_in);
    a.d_out = static_cast<int>(d_out);
    a.r = static_cast<int>(r);
    a.ell = L;
    a.blocks_per_wg = 0;  // set per launch in grid mode 2
    a.ids = batched ? ids : nullptr;
    a.n_adapters = static_cast<int>(n_adapters);
    a.t_out = t_out;
    a.t_stride = static_cast<int>(t_stride);
    hipStream_t st = static_cast<hipStream_t>(stream);

    // Rows of the scale arrays start at multiples of d_in / d_out elements: the conditions below also align them.
    const bool al16 = aligned(x, 16) && aligned(s_in, 16) && aligned(s_out, 16) && aligned(y_base, 16) &&
                      aligned(y_out, 16) && aligned(packedB, 16);
    // In a pool every adapter starts a whole number of words / elements after the previous one: the fast path needs the
    // packed sign(B) of each adapter 16-byte aligned, i.e. d_out * r a multiple of 128.
    const bool pool_ok = !batched || (d_out * r) % 128 == 0;
    const bool mfma_ok = al16 && (d_in % 32 == 0) && (d_out % 8 == 0) && pool_ok;
    const bool vec_x = aligned(x, 16) && aligned(s_in, 16) && (d_in % 8 == 0);

    if (algo == LORDBA_ALGO_GENERAL) return launch_general(a, st, vec_x);
    if (algo != LORDBA_ALGO_AUTO && !mfma_ok) return LORDBA_ERR_ALGO;
    if (algo == LORDBA_ALGO_AUTO && !mfma_ok) return launch_general(a, st, vec_x);

    // Tile and workgroup shape.  16-row tiles halve the per-row cost of building sign operands and are taken once
    // T / 16 tiles still fill the 256 CUs; below that, 8-row tiles keep every CU busy.  16 waves per workgroup hide
    // the most latency but leave 128 registers per lane, which is enough up to r = 32 (8 rows) or r = 16 (16 rows)
    // with one envelope; several envelopes keep L accumulator sets and run on 8 waves.
    const int rb = static_cast<int>((r + 15) / 16);
    const bool tall = batched ? false
                              : algo == LORDBA_ALGO_AUTO ? T >= 4096 : (algo == LORDBA_ALGO_MFMA_T16 || algo == 5 || algo == 7);
    if (batched && algo != LORDBA_ALGO_AUTO && algo != LORDBA_ALGO_MFMA_T8) return LORDBA_ERR_ALGO;
    auto far_apart = [](int64_t d) { return d >= 8192 && d % 4096 == 0; };
    lordba_status s;
    if constexpr (L == 1) {
        if (algo == 4 || algo == 5) {          // tuning variants: 4 waves
            s = tall ? launch_mfma_rb<16, 4, 1>(a, st) : launch_mfma_rb<8, 4, 1>(a, st);
        } else if (algo == 6 || algo == 7) {   // tuning variants: 8 waves
            s = tall ? launch_mfma_rb<16, 8, 1>(a, st) : launch_mfma_rb<8, 8, 1>(a, st);
        } else if (algo == LORDBA_ALGO_AUTO && !batched && T >= 4096 && (far_apart(d_in) || far_apart(d_out))) {
            // Rows of x or of y that lie a multiple of 8 KiB apart (16 KiB or more): the rows of a tile then meet in the
            // same memory channels, and 8-row tiles on 8 waves stream them faster than 16-row tiles do (up to 14 % on
            // eighteen shapes with d_in or d_out = 8192, 16384, 20480, 28672, never slower; no such gain at 11008, 13824,
            // 14336).  L2 counters at d_out = 8192: with 16-row tiles the requests to DRAM wait for credits 1.5 to 3 times
            // as often and the mean read latency at the L2 is 20 % longer (6 % at d_out = 11008).
            s = launch_mfma_rb<8, 8, 1>(a, st);
        } else if (tall) {
            // With more 16-row tiles than the 256 compute units, 8-wave workgroups win: two of them share a compute
            // unit, and one streams its y rows while the other is in its sign stages (0.5 to 9 % on nine shapes with
            // 384 to 1024 tiles).  With one tile per compute unit the 16 waves hide more latency.
            const bool two_per_cu = algo == LORDBA_ALGO_AUTO && (T + 15) / 16 > 256;
            // One 16-row tile per compute unit and at least three output blocks per wave of the 16: the call is mostly stage
            // 3, and 8-row tiles on 8 waves, two workgroups per compute unit that overlap each other's stages, stream it
            // faster (4096 -> 11008: 39.9 against 42.6 us; at 4096 -> 5120 the 16-row tiles still win, 19.4 against 21.2).
            // Beyond one tile per compute unit the same holds while the x pipeline of the 8 waves is one-shot (d_in <= 4096):
            // 4096 -> 11008 at T = 8192 77.3 against 85.9 us, at T = 16384 150.7 against 167.9; 4096 -> 14336 3 to 4 %.
            const bool mostly_stage3 = d_out >= 6144 && (!two_per_cu || d_in <= 4096);
            // Tiles are dealt to 256 compute units: 16-row tiles that leave the last round of a compute unit half empty
            // (T = 6144: 384 tiles, two on half of the units and one on the others) lose more than 8-row tiles cost
            // (768 tiles, three per unit): nine shapes at T = 6144, 8-row tiles 2.6 to 11 % faster on every one.
            auto fill = [](int64_t tiles) { return static_cast<double>(tiles) / static_cast<double>((tiles + 255) / 256 * 256); };
            const bool ragged_rounds = two_per_cu && fill((T + 7) / 8) >= 1.15 * fill((T + 15) / 16);
            if (algo == LORDBA_ALGO_AUTO && rb == 1 && (mostly_stage3 || ragged_rounds)) s = launch_mfma_rb<8, 8, 1>(a, st);
            else s = rb == 1 && !two_per_cu ? launch_mfma_rb<16, 16, 1>(a, st) : launch_mfma_rb<16, 8, 1>(a, st);
        } else if (batched && (T + 7) / 8 > 32) {
            s = launch_mfma_rb<8, 8, 1>(a, st);  // two workgroups per CU: see the batch mode of the kernel
        } else {
            // More 8-row tiles than compute units (2048 < T < 4096): 8 waves again, for the same reason (1 to 10 % on
            // twelve of thirteen shapes at T = 2304 ... 3584, 1 % slower on one).
            const bool two_per_cu = algo == LORDBA_ALGO_AUTO && (T + 7) / 8 > 256;
            s = rb <= 2 && !two_per_cu ? launch_mfma_rb<8, 16, 1>(a, st) : launch_mfma_rb<8, 8, 1>(a, st);
            if (batched && s == LORDBA_ERR_ALGO) s = launch_mfma_rb<8, 8, 1>(a, st);
        }
    } else {
        if (t_out != nullptr) {
            s = launch_mfma_rb<8, 8, L>(a, st);  // the variant family that has a training instantiation
        } else if (tall) {
            s = launch_mfma_rb<16, 8, L>(a, st);
            if (s == LORDBA_ERR_ALGO && algo == LORDBA_ALGO_AUTO) s = launch_mfma_rb<8, 8, L>(a, st);
        } else {
            // a pair of envelopes with one rank block fits the registers of 16 waves (the pair shares an accumulator set);
            // anything more, or the tuning value 6, runs 8 waves
            s = algo == 6 ? LORDBA_ERR_ALGO : launch_mfma_rb<8, 16, L>(a, st);
            if (s == LORDBA_ERR_ALGO) s = launch_mfma_rb<8, 8, L>(a, st);
        }
    }
    if (s == LORDBA_ERR_ALGO && algo == LORDBA_ALGO_AUTO) return launch_general(a, st, vec_x);
    return s;
}

}  // namespace
