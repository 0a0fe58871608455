// Backward pass of the LoRDBA adapter branch for MI355X (gfx950, wave64, MFMA), as training needs it (Sec. 3.2 "Forward
// and backward pass"; smooth-sign straight-through factor of Eq. (smoothsign); Alg. QAT-LoRDBA).
//
// Forward (Eq. (lordba-fwd)):  w = x D_alpha, t = w B1, u = t D_beta, v = u B2, y = y_base + v D_gamma, with S_A = B1^T
// [r, d_in], S_B = B2^T [d_out, r].  For an upstream gradient g = dL/dy:
//
//   du = (g D_gamma) B2^T          dt = du D_beta           dx = dx_base + (dt B1^T) D_alpha
//   Q  = dt^T x   [r, d_in]        P  = u^T g   [r, d_out]  (contractions over the token rows)
//   d_alpha_i = sum_k S_A[k,i] Q[k,i]       dS_A[k,i] = alpha_i Q[k,i]
//   d_gamma_j = sum_k S_B[j,k] P[k,j]       dS_B[j,k] = gamma_j P[k,j]
//   d_beta_k  = sum_t du[t,k] t[t,k]
//   d_latent  = dS * kappa (1 - tanh^2(kappa latent))                                    (Eq. (smoothsign))
//
// Four kernels on the caller's stream, no host synchronisation, every buffer beyond inputs and outputs in the caller's
// workspace:
//   rank    one workgroup per tile of token rows: the two sign reductions t (over d_in, from x) and du (over d_out,
//           from g) with the same MFMA scheme as stage 1 of the forward kernel; writes u and dt (fp32, rank-major),
//           the tile's share of d_beta, and the largest |u|, |dt| per rank (atomic max: order-independent).
//   dx      the forward kernel itself on the transposed adapter: DeltaW^T has the form of Eq. (lordba) with the
//           carriers transposed and alpha, gamma exchanged.
//   wgrad   Q and P: MFMA with the token rows as contraction index.  A lane reads 8 token rows x 8 columns of x (or g)
//           with row-contiguous 16-byte loads and transposes its 8 x 8 block in registers (v_perm_b32), MFMA e of a step
//           takes column 8 m + e from lane group m; dt (or u) enters as fp16 hi + lo after a power-of-two scaling per
//           rank.  Token ranges are split over waves and workgroups; partial sums are reduced in a fixed order.
//   finish  sums the partials, applies the carrier signs, the scales and the smooth-sign factor.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "lordba.h"
#include "lordba_dev_util.h"

namespace {

constexpr int kWgradWaves = 4;        // waves per workgroup of the wgrad kernel, each with its own token range
constexpr int kWgradTargetWgs = 256;  // workgroups the wgrad grid aims at (one per CU; more only adds partial sums)
constexpr int kWgradGroup = 4;        // 32-row steps a wave of the wgrad kernel keeps in flight (2 from three rank blocks on)

struct BwdPlan {
    int rp;          // ranks padded to a multiple of 16
    int t_pad;       // token rows padded to a multiple of 128 (a group of the wgrad kernel)
    int tmv;         // token rows per tile of the rank kernel
    int tiles;       // tiles of the rank kernel
    int nbx, nbg;    // 128-column blocks of d_in and of d_out
    int dcols;       // columns of one partial-sum plane: (nbx + nbg) * 128
    int tw;          // token rows per wave of the wgrad kernel (multiple of 128)
    int splits;      // workgroups along the token axis of the wgrad kernel
    // workspace layout, in 4-byte words
    size_t off_max, off_u, off_dt, off_dbeta, off_part, words;
};

BwdPlan make_plan(int64_t T, int64_t d_in, int64_t d_out, int64_t r) {
    BwdPlan p;
    p.rp = static_cast<int>((r + 15) / 16 * 16);
    p.t_pad = static_cast<int>((T + 127) / 128 * 128);
    p.tmv = T >= 4096 ? 16 : 8;
    p.tiles = static_cast<int>((T + p.tmv - 1) / p.tmv);
    p.nbx = static_cast<int>((d_in + 127) / 128);
    p.nbg = static_cast<int>((d_out + 127) / 128);
    p.dcols = (p.nbx + p.nbg) * 128;
    const int steps = p.t_pad / (32 * kWgradGroup);  // groups of steps: a wave takes whole groups
    int splits = (kWgradTargetWgs + p.nbx + p.nbg - 1) / (p.nbx + p.nbg);
    const int max_splits = (steps + kWgradWaves - 1) / kWgradWaves;  // at least one step per wave
    splits = splits > max_splits ? max_splits : splits;
    splits = splits < 1 ? 1 : splits;
    const int steps_per_wave = (steps + splits * kWgradWaves - 1) / (splits * kWgradWaves);
    p.tw = steps_per_wave * 32 * kWgradGroup;
    p.splits = (steps + steps_per_wave * kWgradWaves - 1) / (steps_per_wave * kWgradWaves);
    p.off_max = 0;
    p.off_u = 128;
    p.off_dt = p.off_u + static_cast<size_t>(p.rp) * p.t_pad;
    p.off_dbeta = p.off_dt + static_cast<size_t>(p.rp) * p.t_pad;
    p.off_part = p.off_dbeta + static_cast<size_t>(p.tiles) * p.rp;
    p.off_part = (p.off_part + 3) & ~static_cast<size_t>(3);
    p.words = p.off_part + static_cast<size_t>(p.splits) * p.rp * p.dcols;
    return p;
}

struct BwdArgs {
    const _Float16* x;
    const _Float16* g;
    const uint32_t* pA;    // S_A   [r, d_in]
    const uint32_t* pBt;   // S_B^T [r, d_out]
    const _Float16* s_in;
    const _Float16* s_rank;
    const _Float16* s_out;
    const float* latA;     // [r, d_in]
    const float* latB;     // [d_out, r]
    float kappa;
    float* d_s_in;
    float* d_s_rank;
    float* d_s_out;
    float* d_latA;
    float* d_latB;
    uint32_t* maxbits;     // [0..63] largest |u| per rank, [64..127] largest |dt| per rank (bit patterns)
    float* uT;             // [rp, t_pad]
    float* dtT;            // [rp, t_pad]
    float* dbeta_part;     // [tiles, rp]
    float* part;           // [splits, rp, dcols]
    int T, d_in, d_out, r;
    int rp, t_pad, tiles, nbx, nbg, dcols, tw, splits;
};

__global__ void bwd_clear_kernel(uint32_t* maxbits) { maxbits[threadIdx.x] = 0u; }
__global__ void bwd_zero_kernel(float* p, int64_t n) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.f;
}

// ------------------------------------------------------------------------------------------ rank kernel ----
// RB rank blocks of 16, TMV token rows per tile (8 or 16), NW waves, DEPTH chunks in flight per wave.  The 128-column
// chunks of x (d_in) and of g (d_out) form one list that is dealt round-robin to the waves; a chunk of x meets +-s_in
// built from S_A, a chunk of g meets +-s_out built from S_B^T, and they accumulate into two separate tiles.
template <int RB, int TMV, int NW, int DEPTH>
__global__ __launch_bounds__(NW * 64) void lordba_bwd_rank_kernel(BwdArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int NI = TMV / 4;
    // The wave index as a scalar: everything that depends on it (which chunks, how many steps) then branches on scalar
    // conditions.  MFMA instructions ignore the EXEC mask, so they must never sit under a vector-predicated branch.
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, q = lane >> 4;
    const int64_t t0 = static_cast<int64_t>(blockIdx.x) * TMV;
    const int last = static_cast<int>(a.T - 1 - t0 < TMV - 1 ? a.T - 1 - t0 : TMV - 1);  // last live row of the tile

    _Float16* sw = reinterpret_cast<_Float16*>(smem) + wave * 128;                       // wave-private scale slice
    _Float16* xs = reinterpret_cast<_Float16*>(smem + NW * 256) + wave * TMV * kXRow;    // wave-private transpose tile
    float* red = reinterpret_cast<float*>(smem + NW * 256 + NW * TMV * kXRow * 2);       // [wave][set][rb][lane][4]

    const int nchunks = a.nbx + a.nbg;
    const int my_n = wave < nchunks ? (nchunks - wave + NW - 1) / NW : 0;

    u4 xbuf[DEPTH][NI];
    uint32_t sbuf[DEPTH];
    uint32_t bits[DEPTH][RB];
    auto issue = [&](int slot, int n) {
        int c = wave + NW * n;
        c = c < nchunks ? c : nchunks - 1;  // past the end: re-read a valid chunk, the result is not used
        const bool is_x = c < a.nbx;
        const int cc = is_x ? c : c - a.nbx;
        const int d = is_x ? a.d_in : a.d_out;
        const _Float16* src = (is_x ? a.x : a.g) + t0 * d;
        const _Float16* sc = is_x ? a.s_in : a.s_out;
        const uint32_t* pk = is_x ? a.pA : a.pBt;
        const int words_per_row = d >> 5;  // d % 32 == 0 on this path
        const int pair = cc * 64 + lane;   // fp16 pair index of the scale slice
        // (columns past d get scale 0 when the chunk is consumed: nothing here may wait for a load)
        sbuf[slot] = *reinterpret_cast<const uint32_t*>(sc + (pair * 2 < d ? pair * 2 : 0));
#pragma unroll
        for (int m = 0; m < NI; ++m) {
            int row = m * 4 + q;
            row = row < last ? row : last;
            int col = cc * 128 + li * 8;
            col = col < d ? col : d - 8;
            xbuf[slot][m] = load16_stream(at(src, static_cast<uint32_t>(row * d + col) * 2u));
        }
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            int rk = rb * 16 + li;
            rk = rk < a.r ? rk : a.r - 1;
            int w = cc * 4 + q;
            w = w < words_per_row ? w : words_per_row - 1;  // columns past d meet scale 0
            bits[slot][rb] = pk[rk * words_per_row + w];
        }
    };

    f4 acc[2][RB];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) acc[s][rb] = f4{0.f, 0.f, 0.f, 0.f};
    }
    auto consume = [&](int slot, int n) {
        const int c = wave + NW * n;
        const bool is_x = c < a.nbx;
        const bool in_range = ((is_x ? c : c - a.nbx) * 64 + lane) * 2 < (is_x ? a.d_in : a.d_out);
        reinterpret_cast<uint32_t*>(sw)[lane] = in_range ? sbuf[slot] : 0u;
#pragma unroll
        for (int m = 0; m < NI; ++m) store16(xs + (m * 4 + q) * kXRow + li * 8, xbuf[slot][m]);
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const h8 xf = as_h8(load16(xs + tile_row_of_mfma_row<TMV>(li) * kXRow + q * 32 + s * 8));
            const u4 sv = load16(sw + q * 32 + s * 8);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                const uint32_t both = __builtin_amdgcn_perm(bits[slot][rb], bits[slot][rb], 0x00010001u * s);
                const h8 op = as_h8(flip_by_bits(sv, both));
                if (is_x) acc[0][rb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xf, op, acc[0][rb], 0, 0, 0);
                else acc[1][rb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xf, op, acc[1][rb], 0, 0, 0);
            }
        }
        __builtin_amdgcn_wave_barrier();
    };

    // The first DEPTH chunks are requested without any condition (past the end a valid chunk is re-read and not used), and
    // so is the next group's chunk after each consumed one: every wait then counts exactly the loads issued after the one
    // it needs.  The last group is consumed without issuing anything.
#pragma unroll
    for (int slot = 0; slot < DEPTH; ++slot) issue(slot, slot);
    int n0 = 0;
    for (; n0 + DEPTH < my_n; n0 += DEPTH) {
#pragma unroll
        for (int slot = 0; slot < DEPTH; ++slot) {
            consume(slot, n0 + slot);
            issue(slot, n0 + DEPTH + slot);
        }
    }
#pragma unroll
    for (int slot = 0; slot < DEPTH; ++slot)
        if (n0 + slot < my_n) consume(slot, n0 + slot);
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) *reinterpret_cast<f4*>(red + (((wave * 2 + s) * RB + rb) * 64 + lane) * 4) = acc[s][rb];
    }
    __syncthreads();
    if (wave != 0) return;

    // Accumulator layout: lane (li, q) holds rank rb*16 + li for MFMA rows 4q .. 4q+3.
    constexpr int LIVE = TMV == 16 ? 4 : 2;  // live rows per lane: token rows 4q + i, or 2q + i
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        f4 ts = f4{0.f, 0.f, 0.f, 0.f}, gs = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < NW; ++w) {  // fixed order: deterministic
            ts += *reinterpret_cast<const f4*>(red + (((w * 2 + 0) * RB + rb) * 64 + lane) * 4);
            gs += *reinterpret_cast<const f4*>(red + (((w * 2 + 1) * RB + rb) * 64 + lane) * 4);
        }
        const int rk = rb * 16 + li;
        const float beta = rk < a.r ? static_cast<float>(a.s_rank[rk]) : 0.f;
        float uv[LIVE], dv[LIVE];
        float db = 0.f, umax = 0.f, dmax = 0.f;
#pragma unroll
        for (int i = 0; i < LIVE; ++i) {
            const int row = (TMV == 16 ? 4 * q : 2 * q) + i;
            const bool live = row <= last && rk < a.r;
            uv[i] = live ? beta * ts[i] : 0.f;
            dv[i] = live ? beta * gs[i] : 0.f;
            db += live ? gs[i] * ts[i] : 0.f;
            umax = fmaxf(umax, fabsf(uv[i]));
            dmax = fmaxf(dmax, fabsf(dv[i]));
        }
        // over the four lane groups (token rows) of the same rank, fixed order
        db += __shfl_xor(db, 16, 64);
        db += __shfl_xor(db, 32, 64);
        umax = fmaxf(umax, __shfl_xor(umax, 16, 64));
        umax = fmaxf(umax, __shfl_xor(umax, 32, 64));
        dmax = fmaxf(dmax, __shfl_xor(dmax, 16, 64));
        dmax = fmaxf(dmax, __shfl_xor(dmax, 32, 64));
        float* up = a.uT + static_cast<size_t>(rk) * a.t_pad + t0 + (TMV == 16 ? 4 * q : 2 * q);
        float* dp = a.dtT + static_cast<size_t>(rk) * a.t_pad + t0 + (TMV == 16 ? 4 * q : 2 * q);
        if (TMV == 16) {
            *reinterpret_cast<f4*>(up) = f4{uv[0], uv[1], uv[LIVE - 2], uv[LIVE - 1]};
            *reinterpret_cast<f4*>(dp) = f4{dv[0], dv[1], dv[LIVE - 2], dv[LIVE - 1]};
        } else {
            *reinterpret_cast<float2*>(up) = float2{uv[0], uv[1]};
            *reinterpret_cast<float2*>(dp) = float2{dv[0], dv[1]};
        }
        if (q == 0) {
            a.dbeta_part[static_cast<size_t>(blockIdx.x) * a.rp + rk] = db;
            // bit patterns of non-negative floats order like unsigned integers
            __hip_atomic_fetch_max(a.maxbits + rk, __float_as_uint(umax), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_fetch_max(a.maxbits + 64 + rk, __float_as_uint(dmax), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    // The last tile also clears the padding rows up to t_pad, which the wgrad kernel reads as whole groups of steps.
    if (blockIdx.x == gridDim.x - 1) {
        const int from = static_cast<int>(t0) + TMV, n = a.t_pad - from;
        for (int e = lane; e < a.rp * n; e += 64) {
            const int rk = e / n, t = from + e % n;
            a.uT[static_cast<size_t>(rk) * a.t_pad + t] = 0.f;
            a.dtT[static_cast<size_t>(rk) * a.t_pad + t] = 0.f;
        }
    }
}

constexpr size_t rank_lds_bytes(int RB, int TMV, int NW) {
    return static_cast<size_t>(NW) * 256 + static_cast<size_t>(NW) * TMV * kXRow * 2 + static_cast<size_t>(NW) * 2 * RB * 1024;
}

// ----------------------------------------------------------------------------------------- wgrad kernel ----
// Workgroup (cb, s): column block cb of x (cb < nbx: Q, with dt) or of g (P, with u), token rows [s * 4 tw, (s+1) * 4 tw),
// a quarter per wave.  One step = 32 token rows x 128 columns.
// G steps are in flight per wave: the loads of a group are issued without any condition (past the end of the wave's range
// they re-read valid addresses and are not used), so that every wait counts exactly the loads issued after the one it
// needs; the last group is consumed without issuing anything.
template <int RB, int G>
__global__ __launch_bounds__(kWgradWaves * 64) void lordba_bwd_wgrad_kernel(BwdArgs a) {
    __shared__ __align__(16) float red[kWgradWaves][8][64][4];
    // The wave index as a scalar: everything that depends on it (which chunks, how many steps) then branches on scalar
    // conditions.  MFMA instructions ignore the EXEC mask, so they must never sit under a vector-predicated branch.
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, q = lane >> 4;
    const int cb = blockIdx.x;
    const bool is_x = cb < a.nbx;
    const int cc = is_x ? cb : cb - a.nbx;
    const int d = is_x ? a.d_in : a.d_out;
    const _Float16* src = is_x ? a.x : a.g;
    const float* small = is_x ? a.dtT : a.uT;
    const uint32_t* mb = a.maxbits + (is_x ? 64 : 0);

    // Power-of-two scaling per rank: the largest entry of the rank's column lands in [2^13, 2^14), so that hi + lo (two
    // fp16) keep 22 bits of every entry that matters to the sum, whatever the magnitude of the gradients.
    float mul[RB], inv[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        int e = static_cast<int>((mb[rb * 16 + li] >> 23) & 0xffu);
        e = e < 14 ? 14 : (e > 254 ? 254 : e);
        mul[rb] = __uint_as_float(static_cast<uint32_t>(267 - e) << 23);
        inv[rb] = __uint_as_float(static_cast<uint32_t>(e - 13) << 23);
    }

    const int tk_begin = (static_cast<int>(blockIdx.y) * kWgradWaves + wave) * a.tw;
    int tk_end = tk_begin + a.tw;
    tk_end = tk_end < a.t_pad ? tk_end : a.t_pad;
    int col = cc * 128 + li * 8;
    col = col < d ? col : d - 8;  // past the end: a valid column group is re-read, its sums are never used

    f4 acc[RB][8];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[rb][e] = f4{0.f, 0.f, 0.f, 0.f};
    }
    u4 xb[G][8];
    u4 sb[G][RB][2];
    auto issue = [&](int slot, int tk) {
        tk = tk < a.t_pad - 32 ? tk : a.t_pad - 32;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int row = tk + 8 * q + e;
            row = row < a.T ? row : a.T - 1;  // padding rows meet dt = u = 0
            xb[slot][e] = load16_stream(src + static_cast<size_t>(row) * d + col);
        }
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const float* p = small + static_cast<size_t>(rb * 16 + li) * a.t_pad + tk + 8 * q;
            sb[slot][rb][0] = load16(p);
            sb[slot][rb][1] = load16(p + 4);
        }
    };
    auto consume = [&](int slot) {
        u4 hi[RB], lo[RB];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float v0 = __uint_as_float(sb[slot][rb][w >> 1][(w & 1) * 2]) * mul[rb];
                const float v1 = __uint_as_float(sb[slot][rb][w >> 1][(w & 1) * 2 + 1]) * mul[rb];
                h2 h, l;
                h[0] = static_cast<_Float16>(v0);
                h[1] = static_cast<_Float16>(v1);
                l[0] = static_cast<_Float16>(v0 - static_cast<float>(h[0]));
                l[1] = static_cast<_Float16>(v1 - static_cast<float>(h[1]));
                hi[rb][w] = __builtin_bit_cast(uint32_t, h);
                lo[rb][w] = __builtin_bit_cast(uint32_t, l);
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            // column e of the lane's 8 x 8 block: token pairs (0,1), (2,3), (4,5), (6,7)
            const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
            u4 col8;
#pragma unroll
            for (int pr = 0; pr < 4; ++pr)
                col8[pr] = __builtin_amdgcn_perm(xb[slot][2 * pr + 1][e >> 1], xb[slot][2 * pr][e >> 1], sel);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                acc[rb][e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(col8), as_h8(hi[rb]), acc[rb][e], 0, 0, 0);
                acc[rb][e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(col8), as_h8(lo[rb]), acc[rb][e], 0, 0, 0);
            }
        }
    };
    // t_pad and tw are multiples of 32 G: a wave's range is a whole number of groups (possibly none)
    if (tk_begin < tk_end) {
#pragma unroll
        for (int i = 0; i < G; ++i) issue(i, tk_begin + 32 * i);
        int tk = tk_begin;
        for (; tk + 32 * G < tk_end; tk += 32 * G) {
#pragma unroll
            for (int i = 0; i < G; ++i) {
                consume(i);
                issue(i, tk + 32 * (G + i));
            }
        }
#pragma unroll
        for (int i = 0; i < G; ++i) consume(i);
    }

    // Accumulator e, register i of lane (li, q): rank rb*16 + li, column 8 (4q + i) + e of the block.  The four waves'
    // tiles are summed in wave order; wave w sums register i = w and so ends up with 8 consecutive columns.
    float* out = a.part + static_cast<size_t>(blockIdx.y) * a.rp * a.dcols + static_cast<size_t>(cb) * 128;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        if (rb > 0) __syncthreads();
#pragma unroll
        for (int e = 0; e < 8; ++e) *reinterpret_cast<f4*>(&red[wave][e][lane][0]) = acc[rb][e];
        __syncthreads();
        float sum[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float s = red[0][e][lane][wave];
#pragma unroll
            for (int w = 1; w < kWgradWaves; ++w) s += red[w][e][lane][wave];
            sum[e] = s * inv[rb];
        }
        float* dst = out + static_cast<size_t>(rb * 16 + li) * a.dcols + 8 * (4 * q + wave);
        *reinterpret_cast<f4*>(dst) = f4{sum[0], sum[1], sum[2], sum[3]};
        *reinterpret_cast<f4*>(dst + 4) = f4{sum[4], sum[5], sum[6], sum[7]};
    }
}

// ---------------------------------------------------------------------------------------- finish kernel ----
// kappa (1 - tanh^2(z)) = 4 kappa e / (1 + e)^2 with e = exp(-2 |z|): no cancellation at large |z|.
__device__ __forceinline__ float smooth_sign_factor(float latent, float kappa) {
    const float e = expf(-2.f * fabsf(kappa * latent));
    const float s = 1.f + e;
    return 4.f * kappa * e / (s * s);
}

// One workgroup per group of 32 columns of d_in (Q, d_s_in, d_latentA) or of d_out (P, d_s_out, d_latentB), plus one for
// d_s_rank.  Thread (c, kq) takes column c of the group and ranks kq, kq + 8, ...; every sum has a fixed order.
__global__ __launch_bounds__(256) void lordba_bwd_finish_kernel(BwdArgs a) {
    __shared__ float sh[256];
    __shared__ float lat[32 * LORDBA_MAX_RANK];
    const int gx = a.d_in >> 5, gg = a.d_out >> 5;
    const int tid = threadIdx.x;
    if (static_cast<int>(blockIdx.x) == gx + gg) {
        // d_beta: the tiles' shares (thread (k, c) takes tiles c, c + nc, ...; then the nc partial sums in order)
        const int nc = 256 / a.rp, k = tid % a.rp, c = tid / a.rp;
        float s = 0.f;
        if (c < nc)
            for (int t = c; t < a.tiles; t += nc) s += a.dbeta_part[static_cast<size_t>(t) * a.rp + k];
        sh[tid] = s;
        __syncthreads();
        if (tid < a.r) {
            float tot = 0.f;
            for (int cc = 0; cc < nc; ++cc) tot += sh[cc * a.rp + tid];
            a.d_s_rank[tid] = tot;
        }
        return;
    }
    const bool is_x = static_cast<int>(blockIdx.x) < gx;
    const int grp = is_x ? blockIdx.x : blockIdx.x - gx;
    const int d = is_x ? a.d_in : a.d_out;
    const int c = tid & 31, kq = tid >> 5;
    const int col = grp * 32 + c;
    const float* plane = a.part + (is_x ? col : a.nbx * 128 + col);
    const uint32_t* pk = is_x ? a.pA : a.pBt;   // both [r, d]: the group's 32 bits of rank k are one word
    const float scale = static_cast<float>(is_x ? a.s_in[col] : a.s_out[col]);
    const int r = a.r;
    if (!is_x) {  // latentB [d_out, r]: the group's 32 rows are 32 r contiguous floats; through LDS for coalesced accesses
        for (int e = tid; e < 32 * r; e += 256) lat[e] = a.latB[static_cast<size_t>(grp) * 32 * r + e];
        __syncthreads();
    }
    float dscale = 0.f;
    for (int k = kq; k < r; k += 8) {
        float s = 0.f;
        for (int sp = 0; sp < a.splits; ++sp) s += plane[(static_cast<size_t>(sp) * a.rp + k) * a.dcols];
        const uint32_t bit = (pk[k * (d >> 5) + grp] >> c) & 1u;
        dscale += flip(s, bit);
        if (is_x) {
            const size_t n = static_cast<size_t>(k) * d + col;
            a.d_latA[n] = scale * s * smooth_sign_factor(a.latA[n], a.kappa);
        } else {
            lat[c * r + k] = scale * s * smooth_sign_factor(lat[c * r + k], a.kappa);
        }
    }
    sh[tid] = dscale;
    __syncthreads();
    if (!is_x)
        for (int e = tid; e < 32 * r; e += 256) a.d_latB[static_cast<size_t>(grp) * 32 * r + e] = lat[e];
    if (kq == 0) {
        float tot = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) tot += sh[j * 32 + c];
        (is_x ? a.d_s_in : a.d_s_out)[col] = tot;
    }
}

// ------------------------------------------------------------------------------------------ host side ----
bool aligned_to(const void* p, size_t n) { return (reinterpret_cast<uintptr_t>(p) & (n - 1)) == 0; }

template <int RB, int TMV>
lordba_status launch_rank(const BwdArgs& a, hipStream_t st) {
    // 16 waves (128 registers per lane) where the accumulators leave room for four chunks in flight, else 8 waves
    constexpr int NW = (TMV == 8 && RB <= 2) ? 16 : 8;
    constexpr int DEPTH = 4;
    constexpr size_t lds = rank_lds_bytes(RB, TMV, NW);
    static_assert(lds <= 160 * 1024, "LDS of a gfx950 CU");
    if (lds > 64 * 1024) {
        // Opt in to more than 64 KiB of dynamic LDS once per device and kernel; raising the limit is idempotent.
        static std::mutex mu;
        static bool granted[64] = {false};
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return LORDBA_ERR_NO_DEVICE;
        std::lock_guard<std::mutex> lk(mu);
        if (!granted[dev]) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(lordba_bwd_rank_kernel<RB, TMV, NW, DEPTH>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) {
                (void)hipGetLastError();
                return LORDBA_ERR_LAUNCH;
            }
            granted[dev] = true;
        }
    }
    hipLaunchKernelGGL((lordba_bwd_rank_kernel<RB, TMV, NW, DEPTH>), dim3(a.tiles), dim3(NW * 64), lds, st, a);
    return hipGetLastError() == hipSuccess ? LORDBA_OK : LORDBA_ERR_LAUNCH;
}

template <int RB>
lordba_status launch_all(const BwdArgs& a, int tmv, hipStream_t st) {
    const lordba_status s = tmv == 16 ? launch_rank<RB, 16>(a, st) : launch_rank<RB, 8>(a, st);
    if (s != LORDBA_OK) return s;
    // kWgradGroup steps in flight where the registers allow two waves per SIMD or nearly so, else half of it
    hipLaunchKernelGGL((lordba_bwd_wgrad_kernel<RB, (RB <= 2 ? kWgradGroup : kWgradGroup / 2)>), dim3(a.nbx + a.nbg, a.splits),
                       dim3(kWgradWaves * 64), 0, st, a);
    if (hipGetLastError() != hipSuccess) return LORDBA_ERR_LAUNCH;
    hipLaunchKernelGGL(lordba_bwd_finish_kernel, dim3((a.d_in >> 5) + (a.d_out >> 5) + 1), dim3(256), 0, st, a);
    return hipGetLastError() == hipSuccess ? LORDBA_OK : LORDBA_ERR_LAUNCH;
}

bool supported(int64_t T, int64_t d_in, int64_t d_out, int64_t r) {
    return T >= 0 && d_in >= 32 && d_out >= 32 && d_in % 32 == 0 && d_out % 32 == 0 && r >= 1 && r <= LORDBA_MAX_RANK &&
           T <= INT32_MAX - 64 && d_in <= (1 << 24) && d_out <= (1 << 24);
}

}  // namespace

extern "C" size_t lordba_backward_workspace_bytes(int64_t T, int64_t d_in, int64_t d_out, int64_t r) {
    if (!supported(T, d_in, d_out, r)) return 0;
    return make_plan(T, d_in, d_out, r).words * 4;
}

extern "C" lordba_status lordba_backward(const void* x, const void* g,
                                         const uint32_t* packedA, const uint32_t* packedAt, const uint32_t* packedBt,
                                         const void* s_in, const void* s_rank, const void* s_out,
                                         const float* latentA, const float* latentB, float kappa,
                                         const void* dx_base, void* dx,
                                         float* d_s_in, float* d_s_rank, float* d_s_out,
                                         float* d_latentA, float* d_latentB,
                                         void* workspace, size_t workspace_bytes,
                                         int64_t T, int64_t d_in, int64_t d_out, int64_t r, void* stream) {
    if (!supported(T, d_in, d_out, r)) return LORDBA_ERR_DIM;
    if (!packedA || !packedAt || !packedBt || !s_in || !s_rank || !s_out || !latentA || !latentB || !d_s_in || !d_s_rank ||
        !d_s_out || !d_latentA || !d_latentB || !workspace)
        return LORDBA_ERR_NULL;
    if (T > 0 && (!x || !g)) return LORDBA_ERR_NULL;
    if ((dx == nullptr) != (dx_base == nullptr)) return LORDBA_ERR_NULL;
    if (!aligned_to(x, 16) || !aligned_to(g, 16) || !aligned_to(s_in, 16) || !aligned_to(s_out, 16) || !aligned_to(s_rank, 2) ||
        !aligned_to(packedA, 4) || !aligned_to(packedBt, 4) || !aligned_to(latentA, 4) || !aligned_to(latentB, 4) ||
        !aligned_to(d_s_in, 4) || !aligned_to(d_s_rank, 4) || !aligned_to(d_s_out, 4) || !aligned_to(d_latentA, 4) ||
        !aligned_to(d_latentB, 4) || !aligned_to(workspace, 16))
        return LORDBA_ERR_ALIGN;
    const BwdPlan p = make_plan(T, d_in, d_out, r);
    if (workspace_bytes < p.words * 4) return LORDBA_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);

    if (T == 0) {  // no token rows: every parameter gradient is zero
        float* outs[5] = {d_s_in, d_s_rank, d_s_out, d_latentA, d_latentB};
        const int64_t ns[5] = {d_in, r, d_out, r * d_in, d_out * r};
        for (int i = 0; i < 5; ++i) {
            hipLaunchKernelGGL(bwd_zero_kernel, dim3(static_cast<unsigned>((ns[i] + 255) / 256)), dim3(256), 0, st, outs[i], ns[i]);
            if (hipGetLastError() != hipSuccess) return LORDBA_ERR_LAUNCH;
        }
        return LORDBA_OK;
    }
    if (dx != nullptr) {
        // dx = dx_base + g DeltaW^T: the forward branch of the transposed adapter (validates its own arguments)
        const lordba_status s = lordba_forward(g, packedBt, packedAt, s_out, s_rank, s_in, dx_base, dx, T, d_out, d_in, r, stream);
        if (s != LORDBA_OK) return s;
    } else {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return LORDBA_ERR_NO_DEVICE; }
    }

    BwdArgs a;
    a.x = static_cast<const _Float16*>(x);
    a.g = static_cast<const _Float16*>(g);
    a.pA = packedA;
    a.pBt = packedBt;
    a.s_in = static_cast<const _Float16*>(s_in);
    a.s_rank = static_cast<const _Float16*>(s_rank);
    a.s_out = static_cast<const _Float16*>(s_out);
    a.latA = latentA;
    a.latB = latentB;
    a.kappa = kappa;
    a.d_s_in = d_s_in;
    a.d_s_rank = d_s_rank;
    a.d_s_out = d_s_out;
    a.d_latA = d_latentA;
    a.d_latB = d_latentB;
    uint32_t* ws = static_cast<uint32_t*>(workspace);
    a.maxbits = ws + p.off_max;
    a.uT = reinterpret_cast<float*>(ws + p.off_u);
    a.dtT = reinterpret_cast<float*>(ws + p.off_dt);
    a.dbeta_part = reinterpret_cast<float*>(ws + p.off_dbeta);
    a.part = reinterpret_cast<float*>(ws + p.off_part);
    a.T = static_cast<int>(T);
    a.d_in = static_cast<int>(d_in);
    a.d_out = static_cast<int>(d_out);
    a.r = static_cast<int>(r);
    a.rp = p.rp;
    a.t_pad = p.t_pad;
    a.tiles = p.tiles;
    a.nbx = p.nbx;
    a.nbg = p.nbg;
    a.dcols = p.dcols;
    a.tw = p.tw;
    a.splits = p.splits;

    hipLaunchKernelGGL(bwd_clear_kernel, dim3(1), dim3(128), 0, st, a.maxbits);
    if (hipGetLastError() != hipSuccess) return LORDBA_ERR_LAUNCH;
    switch (p.rp / 16) {
        case 1: return launch_all<1>(a, p.tmv, st);
        case 2: return launch_all<2>(a, p.tmv, st);
        case 3: return launch_all<3>(a, p.tmv, st);
        default: return launch_all<4>(a, p.tmv, st);
    }
}
