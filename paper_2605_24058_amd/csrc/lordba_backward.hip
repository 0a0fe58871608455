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
// Kernels, all on the caller's stream, no host synchronisation, every buffer beyond inputs and outputs in the caller's
// workspace:
//   dx      The forward kernel itself on the transposed adapter: DeltaW^T has the form of Eq. (lordba) with the carriers
//           transposed and alpha, gamma exchanged.  Its rank-r intermediate is du, which it also writes out.
//   t       The forward kernel on x, stopped after its rank-r intermediate t (skipped when the caller kept t from the
//           training forward pass, lordba_forward_save_t).  With several envelopes both calls produce the intermediates of
//           all envelopes at once; wgrad and finish then run once per envelope.
//   wgrad   Q and P: MFMA with the token rows as contraction index.  A lane reads 8 token rows x 8 columns of x (or g)
//           with row-contiguous 16-byte loads and transposes its 8 x 8 block in registers (v_perm_b32); MFMA e of a step
//           takes column 8 m + e from lane group m.  dt = beta du (or u = beta t) enters as fp16 hi + lo after a
//           power-of-two scaling per rank that follows the largest entry seen so far.  Token ranges are split over waves
//           and workgroups; partial sums are reduced in a fixed order.  One extra workgroup column does d_beta.
//   finish  sums the partials, applies the carrier signs, the scales and the smooth-sign factor.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "lordba.h"
#include "lordba_dev_util.h"

namespace {

constexpr int kWgradWaves = 4;        // waves per workgroup of the wgrad kernel, each with its own token range (8 on short batches)
// Workgroups the wgrad grid aims at: two per CU once the token ranges are long (measured 3-4 % faster from T = 4096 on),
// one per CU below that, where a second one only doubles the partial sums the finish kernel has to read.
constexpr int kWgradTargetWgsLong = 512, kWgradTargetWgsShort = 256;
// 32-row steps a wave of the wgrad kernel keeps in flight: one (two from three rank blocks on).  Deeper requests per wave
// were slower wherever they were tried (four steps against one: 4 to 5 % of the whole call at T = 8192, 1 to 6 % below 4096);
// a kernel that only reads the same column stripes shows the same (5120 columns, 8192 rows, 240 workgroups: 4.4 TB/s with
// four steps in flight per wave, 5.9 with one or two): a wave that requests 128 rows at a time spreads its requests over
// more DRAM pages than one that walks 32 rows at a time.
constexpr int kWgradGroup = 1, kWgradGroupWide = 2;

struct BwdPlan {
    int rp;          // ranks padded to a multiple of 16
    int t_pad;       // token rows padded to a multiple of 128 (whole groups of steps of the wgrad kernel, whole 16-byte pieces of t and du)
    int nbx, nbg;    // 128-column blocks of d_in and of d_out
    int dcols;       // columns of one partial-sum plane: (nbx + nbg) * 128
    int tw;          // token rows per wave of the wgrad kernel (multiple of 128)
    int splits;      // workgroups along the token axis of the wgrad kernel
    int waves;       // waves per workgroup of the wgrad kernel: 4, or 8 on short batches (see make_plan)
    // workspace layout, in 4-byte words
    size_t off_t, off_du, off_dbeta, off_part, words;
};

// ell_fused: envelopes whose partial sums the wgrad kernel holds at once (1: one envelope per wgrad / finish pass).
BwdPlan make_plan(int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t ell_fused = 1) {
    BwdPlan p;
    p.rp = static_cast<int>((r + 15) / 16 * 16);
    p.t_pad = static_cast<int>((T + 127) / 128 * 128);
    p.t_pad = p.t_pad < 128 ? 128 : p.t_pad;  // T == 0 still yields a well-formed (unused) plan
    p.nbx = static_cast<int>((d_in + 127) / 128);
    p.nbg = static_cast<int>((d_out + 127) / 128);
    p.dcols = (p.nbx + p.nbg) * 128;
    // Below 4096 token rows a wave of a 4-wave workgroup would have little to overlap with: such batches run 8 waves (two
    // per SIMD), up to two rank blocks (registers).
    const bool narrow = p.rp * ell_fused <= 32;
    const bool short_batch = T < 4096 && narrow;
    p.waves = short_batch ? 2 * kWgradWaves : kWgradWaves;
    const int group_rows = 32 * (narrow ? kWgradGroup : kWgradGroupWide);
    const int groups = p.t_pad / group_rows;  // a wave takes whole groups of steps (t_pad is a multiple of 128)
    const int target = T >= 4096 ? kWgradTargetWgsLong : kWgradTargetWgsShort;
    int splits = target / (p.nbx + p.nbg);   // rounded down: a grid just above the target would start another round
    const int max_splits = (groups + p.waves - 1) / p.waves;  // at least one group per wave
    splits = splits > max_splits ? max_splits : splits;
    splits = splits < 1 ? 1 : splits;
    const int groups_per_wave = (groups + splits * p.waves - 1) / (splits * p.waves);
    p.tw = groups_per_wave * group_rows;
    p.splits = (groups + groups_per_wave * p.waves - 1) / (groups_per_wave * p.waves);
    // t and du: one [r, t_pad] block per envelope, room for the largest envelope count
    p.off_t = 0;
    p.off_du = p.off_t + static_cast<size_t>(LORDBA_MAX_ENVELOPES) * p.rp * p.t_pad;
    p.off_dbeta = p.off_du + static_cast<size_t>(LORDBA_MAX_ENVELOPES) * p.rp * p.t_pad;
    p.off_part = p.off_dbeta + static_cast<size_t>(p.splits) * p.rp * ell_fused;
    p.off_part = (p.off_part + 3) & ~static_cast<size_t>(3);
    p.words = p.off_part + static_cast<size_t>(p.splits) * p.rp * ell_fused * p.dcols;
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
    const float* tT;       // t,  rank-major: tT[k * t_stride + token], defined for k < r, token < T
    const float* duT;      // du, rank-major: duT[k * du_stride + token]
    float* dbeta_part;     // [splits, ell, rp]
    float* part;           // [splits, ell, rp, dcols]
    int T, d_in, d_out, r;
    int rp, t_pad, t_stride, du_stride, nbx, nbg, dcols, tw, splits, waves;
    int accumulate;        // latent gradients are added to what the arrays hold (second and later envelopes, one pass each)
    // Envelopes held at once (Eq. (lordba): the carriers are shared, so Q and P of all envelopes contract the same x and g
    // with different small operands).  s_in, s_rank, s_out and the scale gradients then have ell rows, tT and duT one
    // [r, stride] block per envelope, and the wgrad kernel's rank blocks are the ell * rp / 16 blocks of all envelopes.
    int ell;
};

__global__ void bwd_zero_kernel(float* p, int64_t n) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.f;
}

// ----------------------------------------------------------------------------------------- wgrad kernel ----
// Workgroup (cb, s): column block cb of x (cb < nbx: Q, with dt) or of g (P, with u), token rows [s * W tw, (s+1) * W tw),
// one range of tw rows per wave; the workgroups with cb == 0 also take the share of d_beta of those token rows.  One step = 32 token rows x 128 columns.
// G steps are in flight per wave: the loads of a group are issued without any condition (past the end of the wave's range
// they re-read valid addresses and are not used), so that every wait counts exactly the loads issued after the one it
// needs; the last group is consumed without issuing anything.
template <int RB, int G, int W>
__global__ __launch_bounds__(W * 64) void lordba_bwd_wgrad_kernel(BwdArgs a) {
    static_assert(W == 4 || W == 8, "the final sums are dealt to 4 or 8 waves");
    __shared__ __align__(16) float red[W][8][64][4];
    // The wave index as a scalar: everything that depends on it (how many steps) then branches on scalar conditions.
    // MFMA instructions ignore the EXEC mask, so they must never sit under a vector-predicated branch.
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, q = lane >> 4;
    const int cb = blockIdx.x;
    const int tk_begin = (static_cast<int>(blockIdx.y) * W + wave) * a.tw;
    int tk_end = tk_begin + a.tw;
    tk_end = tk_end < a.t_pad ? tk_end : a.t_pad;

    const bool is_x = cb < a.nbx;
    const int cc = is_x ? cb : cb - a.nbx;
    const int d = is_x ? a.d_in : a.d_out;
    const _Float16* src = is_x ? a.x : a.g;
    const float* small = is_x ? a.duT : a.tT;   // dt = beta du meets x, u = beta t meets g
    const int sstride = is_x ? a.du_stride : a.t_stride;

    const int rbe = a.rp >> 4;  // rank blocks per envelope
    float beta[RB];
    int row_of[RB];  // the lane's row in the small arrays: envelope * r + rank, clamped to a rank that exists (its values are then masked)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {   // block rb: envelope rb / (rp / 16), ranks 16 (rb % (rp / 16)) ..
        const int en = rb / rbe, rk = (rb - en * rbe) * 16 + li;
        row_of[rb] = en * a.r + (rk < a.r ? rk : a.r - 1);
        beta[rb] = rk < a.r ? static_cast<float>(a.s_rank[row_of[rb]]) : 0.f;
    }
    int col = cc * 128 + li * 8;
    col = col < d ? col : d - 8;  // past the end: a valid column group is re-read, its sums are never used

    f4 acc[RB][8];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[rb][e] = f4{0.f, 0.f, 0.f, 0.f};
    }
    // Power-of-two scaling per rank: 2^(140 - cur_e) brings an entry with biased exponent cur_e to [2^13, 2^14), so that
    // hi + lo (two fp16) keep 22 bits of it.  cur_e follows the largest entry of the rank seen so far, group by group; when
    // it grows, what has been accumulated is rescaled.  Entries far below the largest lose bits that do not matter to the sum.
    int cur_e[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) cur_e[rb] = 14;

    u4 xb[G][8];         // x (or g): step i of the group, 8 token rows x 8 columns per lane
    u4 sb[G][RB][2];     // du (or t): 8 tokens of the lane's rank per step, fp32
    u4 hl[G][RB][2];     // the same as fp16 hi and lo operands, scaled
    auto issue_x = [&](int i, int tk) {
        tk = tk < a.t_pad - 32 ? tk : a.t_pad - 32;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int row = tk + 8 * q + e;
            row = row < a.T ? row : a.T - 1;  // rows past T meet dt = u = 0
            xb[i][e] = load16_stream(src + static_cast<size_t>(row) * d + col);
        }
    };
    auto issue_small = [&](int tk0) {  // all G steps of the group that starts at token tk0
#pragma unroll
        for (int i = 0; i < G; ++i) {
            int tk = tk0 + 32 * i;
            tk = tk < a.t_pad - 32 ? tk : a.t_pad - 32;
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                // 32 bytes inside the row's t_pad entries; the array is defined for token < T only, the rest is masked
                const float* p = small + static_cast<size_t>(row_of[rb]) * sstride + tk + 8 * q;
                sb[i][rb][0] = load16(p);
                sb[i][rb][1] = load16(p + 4);
            }
        }
    };
    auto convert = [&](int tk0) {  // scale of the group, then its hi / lo operands
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            float v[G][8];
            float m = 0.f;
#pragma unroll
            for (int i = 0; i < G; ++i) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float raw = __uint_as_float(sb[i][rb][e >> 2][e & 3]);
                    // select, not multiply: the padding rows and the ranks past r hold undefined values
                    v[i][e] = (tk0 + 32 * i + 8 * q + e < a.T && beta[rb] != 0.f) ? raw * beta[rb] : 0.f;
                    m = fmaxf(m, fabsf(v[i][e]));
                }
            }
            m = fmaxf(m, __shfl_xor(m, 16, 64));
            m = fmaxf(m, __shfl_xor(m, 32, 64));
            int e_new = static_cast<int>((__float_as_uint(m) >> 23) & 0xffu);
            e_new = e_new > 254 ? 254 : e_new;
            if (__builtin_amdgcn_ballot_w64(e_new > cur_e[rb]) != 0ull) {   // scalar branch: rare after the first group
                const int sh = cur_e[rb] - e_new;                           // < 0 where this lane's rank grows
                const float f = sh >= 0 ? 1.f : (sh < -126 ? 0.f : __uint_as_float(static_cast<uint32_t>(127 + sh) << 23));
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[rb][e] *= f;
                cur_e[rb] = e_new > cur_e[rb] ? e_new : cur_e[rb];
            }
            const float mul = __uint_as_float(static_cast<uint32_t>(267 - cur_e[rb]) << 23);
#pragma unroll
            for (int i = 0; i < G; ++i) {
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const float v0 = v[i][2 * w] * mul, v1 = v[i][2 * w + 1] * mul;
                    h2 h, l;
                    h[0] = static_cast<_Float16>(v0);
                    h[1] = static_cast<_Float16>(v1);
                    l[0] = static_cast<_Float16>(v0 - static_cast<float>(h[0]));
                    l[1] = static_cast<_Float16>(v1 - static_cast<float>(h[1]));
                    hl[i][rb][0][w] = __builtin_bit_cast(uint32_t, h);
                    hl[i][rb][1][w] = __builtin_bit_cast(uint32_t, l);
                }
            }
        }
    };
    auto consume_x = [&](int i) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            // column e of the lane's 8 x 8 block: token pairs (0,1), (2,3), (4,5), (6,7)
            const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
            u4 col8;
#pragma unroll
            for (int pr = 0; pr < 4; ++pr)
                col8[pr] = __builtin_amdgcn_perm(xb[i][2 * pr + 1][e >> 1], xb[i][2 * pr][e >> 1], sel);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                acc[rb][e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(col8), as_h8(hl[i][rb][0]), acc[rb][e], 0, 0, 0);
                acc[rb][e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_h8(col8), as_h8(hl[i][rb][1]), acc[rb][e], 0, 0, 0);
            }
        }
    };
    // t_pad and tw are multiples of 32 G: a wave's range is a whole number of groups (possibly none).  The small loads of a
    // group are requested before the x loads that are issued while the previous group is consumed, so the conversion (a
    // dependent chain of vector-ALU work and two cross-lane exchanges) never waits for x.
    if (tk_begin < tk_end) {
        issue_small(tk_begin);
#pragma unroll
        for (int i = 0; i < G; ++i) issue_x(i, tk_begin + 32 * i);
        int tk = tk_begin;
        for (; tk + 32 * G < tk_end; tk += 32 * G) {
            convert(tk);
            issue_small(tk + 32 * G);
#pragma unroll
            for (int i = 0; i < G; ++i) {
                consume_x(i);
                issue_x(i, tk + 32 * (G + i));
            }
        }
        convert(tk);
#pragma unroll
        for (int i = 0; i < G; ++i) consume_x(i);
    }

    // Accumulator e, register i of lane (li, q): rank rb*16 + li, column 8 (4q + i) + e of the block.  Each wave brings its
    // tile back to true scale; the tiles are summed in wave order; with 4 waves wave w sums register i = w of all 8
    // accumulators and so ends up with 8 consecutive columns, with 8 waves it sums register i = w mod 4 of accumulators
    // 4 (w / 4) .. 4 (w / 4) + 3: 4 consecutive columns.
    float* out = a.part + static_cast<size_t>(blockIdx.y) * (RB * 16) * a.dcols + static_cast<size_t>(cb) * 128;
    constexpr int NE = W == 4 ? 8 : 4;
    const int ri = wave & 3, e0 = W == 4 ? 0 : 4 * (wave >> 2);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        if (rb > 0) __syncthreads();
        const float inv = __uint_as_float(static_cast<uint32_t>(cur_e[rb] - 13) << 23);
#pragma unroll
        for (int e = 0; e < 8; ++e) *reinterpret_cast<f4*>(&red[wave][e][lane][0]) = acc[rb][e] * inv;
        __syncthreads();
        float sum[NE];
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            float s = red[0][e0 + e][lane][ri];
#pragma unroll
            for (int w = 1; w < W; ++w) s += red[w][e0 + e][lane][ri];
            sum[e] = s;
        }
        float* dst = out + static_cast<size_t>(rb * 16 + li) * a.dcols + 8 * (4 * q + ri) + e0;
        *reinterpret_cast<f4*>(dst) = f4{sum[0], sum[1], sum[2], sum[3]};
        if constexpr (NE == 8) *reinterpret_cast<f4*>(dst + 4) = f4{sum[4], sum[5], sum[6], sum[7]};
    }
    if (cb != 0) return;
    // The workgroups of the first column block also take the share of d_beta_k = sum_t du[t,k] t[t,k] of their token rows
    // (a column of workgroups of its own would push the grid past one workgroup per compute unit, i.e. into a second
    // round): lane (li, q) takes rank li of each block and the tokens 8 q .. 8 q + 7 of every step; fixed order (lane, then
    // lane groups, then waves).
    __syncthreads();  // the sums below reuse the reduction area
    {
        float* sums = &red[0][0][0][0];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int en = rb / rbe, rk = (rb - en * rbe) * 16 + li;
            float s = 0.f;
            const int row = en * a.r + (rk < a.r ? rk : a.r - 1);  // a rank that exists; the result of a padded rank is dropped below
            const float* dup = a.duT + static_cast<size_t>(row) * a.du_stride + 8 * q;
            const float* tp = a.tT + static_cast<size_t>(row) * a.t_stride + 8 * q;
            for (int tk = tk_begin; tk < tk_end; tk += 32) {  // 32 bytes of each array per lane and step, inside t_pad entries
                const u4 d0 = load16(dup + tk), d1 = load16(dup + tk + 4), t0 = load16(tp + tk), t1 = load16(tp + tk + 4);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float dv = __uint_as_float(e < 4 ? d0[e & 3] : d1[e & 3]), tv = __uint_as_float(e < 4 ? t0[e & 3] : t1[e & 3]);
                    s += (tk + 8 * q + e < a.T) ? dv * tv : 0.f;   // select: entries past T are undefined
                }
            }
            if (rk >= a.r) s = 0.f;
            s += __shfl_xor(s, 16, 64);
            s += __shfl_xor(s, 32, 64);
            if (q == 0) sums[(rb * 16 + li) * W + wave] = s;
        }
        __syncthreads();
        if (tid < RB * 16) {
            float tot = 0.f;
#pragma unroll
            for (int w = 0; w < W; ++w) tot += sums[tid * W + w];
            a.dbeta_part[static_cast<size_t>(blockIdx.y) * (RB * 16) + tid] = tot;
        }
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
    __shared__ float sh[LORDBA_MAX_ENVELOPES][256];
    __shared__ float lat[32 * LORDBA_MAX_RANK];
    const int gx = a.d_in >> 5, gg = a.d_out >> 5;
    const int tid = threadIdx.x;
    const int r = a.r, ell = a.ell, rows = ell * a.rp;   // rows of one token range's plane of partial sums: all envelopes' rank blocks
    if (static_cast<int>(blockIdx.x) == gx + gg) {
        for (int o = tid; o < ell * r; o += 256) {  // d_beta of every envelope: the shares of the token ranges, in their order
            const int en = o / r, k = o - en * r;
            float tot = 0.f;
            for (int sp = 0; sp < a.splits; ++sp) tot += a.dbeta_part[static_cast<size_t>(sp) * rows + en * a.rp + k];
            a.d_s_rank[en * r + k] = tot;
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
    float scale[LORDBA_MAX_ENVELOPES], dscale[LORDBA_MAX_ENVELOPES];
#pragma unroll
    for (int en = 0; en < LORDBA_MAX_ENVELOPES; ++en) {
        const int ec = en < ell ? en : 0;
        scale[en] = static_cast<float>(is_x ? a.s_in[static_cast<size_t>(ec) * d + col] : a.s_out[static_cast<size_t>(ec) * d + col]);
        dscale[en] = 0.f;
    }
    if (!is_x && a.d_latB != nullptr) {  // latentB [d_out, r]: the group's 32 rows are 32 r contiguous floats; through LDS for coalesced accesses
        for (int e = tid; e < 32 * r; e += 256) lat[e] = a.latB[static_cast<size_t>(grp) * 32 * r + e];
        __syncthreads();
    }
    const bool with_lat = a.d_latA != nullptr;   // (null: the carriers are frozen, only the scale gradients are wanted)
    const bool lat_x = with_lat && is_x, add_x = lat_x && a.accumulate;
    for (int k = kq; k < r; k += 8) {
        // Everything this rank needs is requested before anything is used: the shares of the token ranges (eight at a
        // time, from a clamped index), the carrier word, the latent and, when accumulating, the gradient so far.  The
        // last two come from a harmless address when they are not wanted, so that no request hides behind a branch.
        const size_t n = static_cast<size_t>(k) * d + col;
        const uint32_t word = pk[k * (d >> 5) + grp];
        const float latent = *(lat_x ? a.latA + n : plane);
        const float so_far = *(add_x ? a.d_latA + n : plane);
        const uint32_t bit = (word >> c) & 1u;
        float weighted = 0.f;   // sum over the envelopes of scale_e * (Q_e or P_e)[k, col]: dL/dS[k, col]
#pragma unroll
        for (int en = 0; en < LORDBA_MAX_ENVELOPES; ++en) {
            if (en < ell) {
                float s = 0.f;
                for (int sp0 = 0; sp0 < a.splits; sp0 += 8) {
                    float v[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const int sp = sp0 + j < a.splits ? sp0 + j : a.splits - 1;
                        v[j] = plane[(static_cast<size_t>(sp) * rows + en * a.rp + k) * a.dcols];
                    }
#pragma unroll
                    for (int j = 0; j < 8; ++j) s += (sp0 + j < a.splits) ? v[j] : 0.f;
                }
                dscale[en] += flip(s, bit);
                weighted = ell == 1 ? scale[0] * s : fmaf(scale[en], s, weighted);
            }
        }
        if (lat_x) {
            const float val = weighted * smooth_sign_factor(latent, a.kappa);
            a.d_latA[n] = add_x ? so_far + val : val;
        } else if (with_lat) {
            lat[c * r + k] = weighted * smooth_sign_factor(lat[c * r + k], a.kappa);
        }
    }
#pragma unroll
    for (int en = 0; en < LORDBA_MAX_ENVELOPES; ++en) sh[en][tid] = dscale[en];
    __syncthreads();
    if (!is_x && a.d_latB != nullptr)
        for (int e = tid; e < 32 * r; e += 256) {
            float* dst = a.d_latB + static_cast<size_t>(grp) * 32 * r + e;
            *dst = a.accumulate ? *dst + lat[e] : lat[e];
        }
    if (kq < ell) {   // wave pair kq sums envelope kq's eight partial sums of every column
        float tot = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) tot += sh[kq][j * 32 + c];
        (is_x ? a.d_s_in : a.d_s_out)[static_cast<size_t>(kq) * d + col] = tot;
    }
}

// --------------------------------------------------------------------------------------- general kernel ----
// Q, P and everything that follows from them for any shape and alignment, on the vector ALU: one thread per column of x
// (Q[:, i], then d_s_in[i] and d_latentA[:, i]) or of g (P[:, j], d_s_out[j], d_latentB[j, :]) walks all token rows with
// its r sums in registers; r more threads take d_s_rank.  No partial sums, fixed order.  Slow (a column's T x r
// multiply-adds in one thread) but it is what a shape outside the matrix-core path gets, as in the forward pass.
template <int RP>
__global__ __launch_bounds__(256) void lordba_bwd_general_kernel(BwdArgs a) {
    __shared__ float beta_s[RP];
    const int r = a.r, tid = threadIdx.x;
    if (tid < RP) beta_s[tid] = tid < r ? static_cast<float>(a.s_rank[tid]) : 0.f;
    __syncthreads();
    const int64_t c = static_cast<int64_t>(blockIdx.x) * 256 + tid;
    const int64_t ncols = static_cast<int64_t>(a.d_in) + a.d_out;
    if (c >= ncols + r) return;
    if (c >= ncols) {  // d_beta_k = sum_t du[t, k] t[t, k]
        const int k = static_cast<int>(c - ncols);
        const float* dup = a.duT + static_cast<size_t>(k) * a.du_stride;
        const float* tp = a.tT + static_cast<size_t>(k) * a.t_stride;
        float s = 0.f;
        for (int t = 0; t < a.T; ++t) s = fmaf(dup[t], tp[t], s);
        a.d_s_rank[k] = s;
        return;
    }
    const bool is_x = c < a.d_in;
    const int col = static_cast<int>(is_x ? c : c - a.d_in);
    const int d = is_x ? a.d_in : a.d_out;
    const _Float16* src = (is_x ? a.x : a.g) + col;
    const float* small = is_x ? a.duT : a.tT;   // dt = beta du meets x, u = beta t meets g
    const int sstride = is_x ? a.du_stride : a.t_stride;
    float acc[RP];
#pragma unroll
    for (int k = 0; k < RP; ++k) acc[k] = 0.f;
    for (int t = 0; t < a.T; ++t) {
        const float v = static_cast<float>(src[static_cast<size_t>(t) * d]);
#pragma unroll
        for (int k = 0; k < RP; ++k)
            if (k < r) acc[k] = fmaf(small[static_cast<size_t>(k) * sstride + t] * beta_s[k], v, acc[k]);
    }
    const uint32_t* pk = is_x ? a.pA : a.pBt;   // both [r, d] bit streams
    const float scale = static_cast<float>(is_x ? a.s_in[col] : a.s_out[col]);
    const bool with_lat = a.d_latA != nullptr;
    float dscale = 0.f;
#pragma unroll
    for (int k = 0; k < RP; ++k) {
        if (k < r) {
            const int64_t n = static_cast<int64_t>(k) * d + col;
            dscale += flip(acc[k], (pk[n >> 5] >> (n & 31)) & 1u);
            if (with_lat) {
                const size_t at = is_x ? static_cast<size_t>(n) : static_cast<size_t>(col) * r + k;   // latentA [r, d_in], latentB [d_out, r]
                const float* lat = is_x ? a.latA : a.latB;
                float* out = is_x ? a.d_latA : a.d_latB;
                const float val = scale * acc[k] * smooth_sign_factor(lat[at], a.kappa);
                out[at] = a.accumulate ? out[at] + val : val;
            }
        }
    }
    (is_x ? a.d_s_in : a.d_s_out)[col] = dscale;
}

template <int RP>
lordba_status launch_general(const BwdArgs& a, hipStream_t st) {
    const int64_t n = static_cast<int64_t>(a.d_in) + a.d_out + a.r;
    hipLaunchKernelGGL((lordba_bwd_general_kernel<RP>), dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0, st, a);
    return hipGetLastError() == hipSuccess ? LORDBA_OK : LORDBA_ERR_LAUNCH;
}

// ------------------------------------------------------------------------------------------ host side ----
bool aligned_to(const void* p, size_t n) { return (reinterpret_cast<uintptr_t>(p) & (n - 1)) == 0; }

template <int RB>
lordba_status launch_all(const BwdArgs& a, hipStream_t st) {
    // (steps in flight and waves as make_plan laid the token ranges out)
    const dim3 grid(a.nbx + a.nbg, a.splits);
    if constexpr (RB <= 2) {
        if (a.waves == 2 * kWgradWaves)
            hipLaunchKernelGGL((lordba_bwd_wgrad_kernel<RB, kWgradGroup, 2 * kWgradWaves>), grid, dim3(2 * kWgradWaves * 64), 0, st, a);
        else
            hipLaunchKernelGGL((lordba_bwd_wgrad_kernel<RB, kWgradGroup, kWgradWaves>), grid, dim3(kWgradWaves * 64), 0, st, a);
    } else {
        hipLaunchKernelGGL((lordba_bwd_wgrad_kernel<RB, kWgradGroupWide, kWgradWaves>), grid, dim3(kWgradWaves * 64), 0, st, a);
    }
    if (hipGetLastError() != hipSuccess) return LORDBA_ERR_LAUNCH;
    hipLaunchKernelGGL(lordba_bwd_finish_kernel, dim3((a.d_in >> 5) + (a.d_out >> 5) + 1), dim3(256), 0, st, a);
    return hipGetLastError() == hipSuccess ? LORDBA_OK : LORDBA_ERR_LAUNCH;
}

bool supported(int64_t T, int64_t d_in, int64_t d_out, int64_t r) {
    return T >= 0 && d_in >= 1 && d_out >= 1 && r >= 1 && r <= LORDBA_MAX_RANK && T <= INT32_MAX - 128 && d_in <= (1 << 24) &&
           d_out <= (1 << 24);
}
// The matrix-core wgrad and the finish kernel read whole 128-column blocks and 32-column words.
bool fast_shape(int64_t d_in, int64_t d_out) { return d_in % 32 == 0 && d_out % 32 == 0; }

}  // namespace

extern "C" size_t lordba_backward_workspace_bytes(int64_t T, int64_t d_in, int64_t d_out, int64_t r) {
    if (!supported(T, d_in, d_out, r)) return 0;
    return make_plan(T, d_in, d_out, r).words * 4;
}

extern "C" size_t lordba_backward_multi_workspace_bytes(int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t ell) {
    if (!supported(T, d_in, d_out, r) || ell < 1 || ell > LORDBA_MAX_ENVELOPES) return 0;
    const bool one_pass = ell > 1 && fast_shape(d_in, d_out) && ell * ((r + 15) / 16) <= 4;
    return make_plan(T, d_in, d_out, r, one_pass ? ell : 1).words * 4;
}

namespace {

// Shared by the entry points.  ell envelopes: s_in, s_rank, s_out and their gradients have ell rows; everything is additive
// over the envelopes (DeltaW is their sum and g is fixed), so envelope e is one pass of the one-envelope machinery with its
// own scales: its own scale gradients, and latent gradients added to those of the envelopes before it.
lordba_status backward_impl(const void* x, const void* g,
                            const uint32_t* packedA, const uint32_t* packedAt, const uint32_t* packedBt,
                            const void* s_in, const void* s_rank, const void* s_out,
                            const float* latentA, const float* latentB, float kappa,
                            const float* t_saved, int64_t t_stride,
                            const void* dx_base, void* dx,
                            float* d_s_in, float* d_s_rank, float* d_s_out,
                            float* d_latentA, float* d_latentB,
                            void* workspace, size_t workspace_bytes,
                            int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t ell, void* stream) {
    if (!supported(T, d_in, d_out, r) || ell < 1 || ell > LORDBA_MAX_ENVELOPES) return LORDBA_ERR_DIM;
    if (!packedA || !packedAt || !packedBt || !s_in || !s_rank || !s_out || !d_s_in || !d_s_rank || !d_s_out || !workspace)
        return LORDBA_ERR_NULL;
    // frozen carriers (only the scales are trained): no latents, no latent gradients
    const bool with_latents = d_latentA != nullptr || d_latentB != nullptr;
    if (with_latents && (!latentA || !latentB || !d_latentA || !d_latentB)) return LORDBA_ERR_NULL;
    if (T > 0 && (!x || !g)) return LORDBA_ERR_NULL;
    if ((dx == nullptr) != (dx_base == nullptr)) return LORDBA_ERR_NULL;
    if (t_saved != nullptr && (t_stride < T || t_stride > INT32_MAX)) return LORDBA_ERR_DIM;
    // every pointer aligned to its element; the workspace to 16 bytes (its layout is this library's)
    if (!aligned_to(x, 2) || !aligned_to(g, 2) || !aligned_to(s_in, 2) || !aligned_to(s_out, 2) || !aligned_to(s_rank, 2) ||
        !aligned_to(packedA, 4) || !aligned_to(packedAt, 4) || !aligned_to(packedBt, 4) || !aligned_to(latentA, 4) ||
        !aligned_to(latentB, 4) || !aligned_to(d_s_in, 4) || !aligned_to(d_s_rank, 4) || !aligned_to(d_s_out, 4) ||
        !aligned_to(d_latentA, 4) || !aligned_to(d_latentB, 4) || !aligned_to(workspace, 16) || !aligned_to(t_saved, 4) ||
        !aligned_to(dx_base, 2) || !aligned_to(dx, 2))
        return LORDBA_ERR_ALIGN;
    // The matrix-core wgrad and the finish kernel need widths that are multiples of 32, 16-byte aligned activations and
    // carriers, and a kept t whose rows reach the padded token count (it is read in whole 32-row steps); anything else
    // takes the general kernel.
    const bool fast = fast_shape(d_in, d_out) && aligned_to(x, 16) && aligned_to(g, 16) && aligned_to(s_in, 16) && aligned_to(s_out, 16) &&
                      aligned_to(packedA, 16) && aligned_to(packedAt, 16) && aligned_to(dx_base, 16) && aligned_to(dx, 16) &&
                      (t_saved == nullptr || (aligned_to(t_saved, 16) && t_stride % 4 == 0 && t_stride >= (T + 127) / 128 * 128));
    // Several envelopes: with room for the partial sums of all of them (lordba_backward_multi_workspace_bytes) and at most
    // four rank blocks in all, one wgrad and one finish pass serve every envelope (x and g are read once); otherwise one
    // pass per envelope.
    const int64_t rbe = (r + 15) / 16;
    const bool fused = fast && ell > 1 && ell * rbe <= 4 && workspace_bytes >= make_plan(T, d_in, d_out, r, ell).words * 4;
    const BwdPlan p = make_plan(T, d_in, d_out, r, fused ? ell : 1);
    if (workspace_bytes < p.words * 4) return LORDBA_ERR_WORKSPACE;
    {
        // No output (and not the workspace) may overlap an input or another output; dx on top of dx_base is the one
        // exception and is checked by the forward call below.
        struct Span { const void* p; size_t n; };
        const size_t nx = static_cast<size_t>(T) * d_in * 2, ng = static_cast<size_t>(T) * d_out * 2;
        const size_t nA = static_cast<size_t>(r) * d_in, nB = static_cast<size_t>(d_out) * r;
        const size_t L = static_cast<size_t>(ell);
        const Span outs[] = {{d_s_in, L * d_in * 4}, {d_s_rank, L * r * 4},
                             {d_s_out, L * d_out * 4}, {d_latentA, nA * 4}, {d_latentB, nB * 4},
                             {workspace, p.words * 4}, {dx, dx ? nx : 0}};
        const Span ins[] = {{x, nx}, {g, ng}, {packedA, lordba_packed_words(r, d_in) * 4}, {packedAt, lordba_packed_words(d_in, r) * 4},
                            {packedBt, lordba_packed_words(r, d_out) * 4}, {s_in, L * d_in * 2},
                            {s_rank, L * r * 2}, {s_out, L * d_out * 2}, {latentA, nA * 4},
                            {latentB, nB * 4}, {t_saved, t_saved ? (static_cast<size_t>(ell * r - 1) * t_stride + T) * 4 : 0}};
        auto hit = [](const Span& a, const Span& b) {
            const uintptr_t pa = reinterpret_cast<uintptr_t>(a.p), pb = reinterpret_cast<uintptr_t>(b.p);
            return pa != 0 && pb != 0 && a.n != 0 && b.n != 0 && pa < pb + b.n && pb < pa + a.n;  // (optional arguments may be NULL)
        };
        constexpr int no = sizeof(outs) / sizeof(outs[0]), ni = sizeof(ins) / sizeof(ins[0]);
        for (int i = 0; i < no; ++i) {
            for (int j = 0; j < ni; ++j)
                if (hit(outs[i], ins[j])) return LORDBA_ERR_ALIAS;
            for (int j = i + 1; j < no; ++j)
                if (hit(outs[i], outs[j])) return LORDBA_ERR_ALIAS;
        }
    }
    hipStream_t st = static_cast<hipStream_t>(stream);

    if (T == 0) {  // no token rows: every parameter gradient is zero
        float* outs[5] = {d_s_in, d_s_rank, d_s_out, d_latentA, d_latentB};
        const int64_t ns[5] = {ell * d_in, ell * r, ell * d_out, r * d_in, d_out * r};
        for (int i = 0; i < (with_latents ? 5 : 3); ++i) {
            hipLaunchKernelGGL(bwd_zero_kernel, dim3(static_cast<unsigned>((ns[i] + 255) / 256)), dim3(256), 0, st, outs[i], ns[i]);
            if (hipGetLastError() != hipSuccess) return LORDBA_ERR_LAUNCH;
        }
        return LORDBA_OK;
    }

    float* ws = static_cast<float*>(workspace);
    float* duT = ws + p.off_du;
    float* t_own = ws + p.off_t;
    const _Float16* si = static_cast<const _Float16*>(s_in);
    const _Float16* sr = static_cast<const _Float16*>(s_rank);
    const _Float16* so = static_cast<const _Float16*>(s_out);
    lordba_status s;
    // du of every envelope, and dx = dx_base + g DeltaW^T if wanted (all envelopes at once, one rounding): the forward branch
    // of the transposed adapter (it validates its own arguments); du is that call's rank-r intermediate
    s = lordba_forward_multi_save_t(g, packedBt, packedAt, s_out, s_rank, s_in, dx_base, dx, duT, p.t_pad, T, d_out, d_in, r, ell, stream);
    if (s != LORDBA_OK) return s;
    if (t_saved == nullptr) {
        // t of every envelope: the forward branch of the adapter itself, stopped after its rank-r intermediate (its second
        // carrier is not read; packedAt stands in as a valid [d_in, r] carrier)
        s = lordba_forward_multi_save_t(x, packedA, packedAt, s_in, s_rank, s_in, nullptr, nullptr, t_own, p.t_pad, T, d_in, d_in, r, ell,
                                        stream);
        if (s != LORDBA_OK) return s;
    }
    for (int64_t e = 0; e < (fused ? 1 : ell); ++e) {
        const float* tT = t_saved ? t_saved + e * r * t_stride : t_own + e * r * p.t_pad;
        const int64_t tT_stride = t_saved ? t_stride : p.t_pad;

        BwdArgs a;
        a.x = static_cast<const _Float16*>(x);
        a.g = static_cast<const _Float16*>(g);
        a.pA = packedA;
        a.pBt = packedBt;
        a.s_in = si + e * d_in;
        a.s_rank = sr + e * r;
        a.s_out = so + e * d_out;
        a.latA = latentA;
        a.latB = latentB;
        a.kappa = kappa;
        a.d_s_in = d_s_in + e * d_in;
        a.d_s_rank = d_s_rank + e * r;
        a.d_s_out = d_s_out + e * d_out;
        a.d_latA = d_latentA;
        a.d_latB = d_latentB;
        a.tT = tT;
        a.duT = duT + e * r * p.t_pad;
        a.dbeta_part = ws + p.off_dbeta;
        a.part = ws + p.off_part;
        a.T = static_cast<int>(T);
        a.d_in = static_cast<int>(d_in);
        a.d_out = static_cast<int>(d_out);
        a.r = static_cast<int>(r);
        a.rp = p.rp;
        a.t_pad = p.t_pad;
        a.t_stride = static_cast<int>(tT_stride);
        a.du_stride = p.t_pad;
        a.nbx = p.nbx;
        a.nbg = p.nbg;
        a.dcols = p.dcols;
        a.tw = p.tw;
        a.splits = p.splits;
        a.waves = p.waves;
        a.accumulate = e > 0 ? 1 : 0;
        a.ell = fused ? static_cast<int>(ell) : 1;
        if (!fast) {
            s = r <= 8 ? launch_general<8>(a, st) : r <= 16 ? launch_general<16>(a, st) : r <= 32 ? launch_general<32>(a, st) : launch_general<64>(a, st);
        } else {
            switch (a.ell * (p.rp / 16)) {   // rank blocks held at once
                case 1: s = launch_all<1>(a, st); break;
                case 2: s = launch_all<2>(a, st); break;
                case 3: s = launch_all<3>(a, st); break;
                default: s = launch_all<4>(a, st); break;
            }
        }
        if (s != LORDBA_OK) return s;
    }
    return LORDBA_OK;
}

}  // namespace

extern "C" lordba_status lordba_backward(const void* x, const void* g,
                                         const uint32_t* packedA, const uint32_t* packedAt, const uint32_t* packedBt,
                                         const void* s_in, const void* s_rank, const void* s_out,
                                         const float* latentA, const float* latentB, float kappa,
                                         const float* t_saved, int64_t t_stride,
                                         const void* dx_base, void* dx,
                                         float* d_s_in, float* d_s_rank, float* d_s_out,
                                         float* d_latentA, float* d_latentB,
                                         void* workspace, size_t workspace_bytes,
                                         int64_t T, int64_t d_in, int64_t d_out, int64_t r, void* stream) {
    return backward_impl(x, g, packedA, packedAt, packedBt, s_in, s_rank, s_out, latentA, latentB, kappa, t_saved, t_stride, dx_base, dx,
                         d_s_in, d_s_rank, d_s_out, d_latentA, d_latentB, workspace, workspace_bytes, T, d_in, d_out, r, 1, stream);
}

extern "C" lordba_status lordba_backward_multi(const void* x, const void* g,
                                               const uint32_t* packedA, const uint32_t* packedAt, const uint32_t* packedBt,
                                               const void* s_in, const void* s_rank, const void* s_out,
                                               const float* latentA, const float* latentB, float kappa,
                                               const float* t_saved, int64_t t_stride,
                                               const void* dx_base, void* dx,
                                               float* d_s_in, float* d_s_rank, float* d_s_out,
                                               float* d_latentA, float* d_latentB,
                                               void* workspace, size_t workspace_bytes,
                                               int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t ell, void* stream) {
    return backward_impl(x, g, packedA, packedAt, packedBt, s_in, s_rank, s_out, latentA, latentB, kappa, t_saved, t_stride, dx_base, dx,
                         d_s_in, d_s_rank, d_s_out, d_latentA, d_latentB, workspace, workspace_bytes, T, d_in, d_out, r, ell, stream);
}

// ---------------------------------------------------------------------------- entry point that allocates nothing ----
// For callers that cannot allocate or pass a workspace: the scratch of the call (rank-r intermediates and partial sums, the
// layout of make_plan) lives in a device array of fixed size that belongs to the library.  Every GPU holds its own copy
// at its own address; in host code the array's name is only a handle, so the address is asked for once per device and
// that pointer is what the kernels get.
static __device__ __align__(256) unsigned char scratch[LORDBA_BACKWARD_NOALLOC_MAX_BYTES];

namespace {
lordba_status noalloc_scratch(void** out) {
    static std::mutex mu;
    static void* ptr[64] = {nullptr};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return LORDBA_ERR_NO_DEVICE; }
    if (dev < 0 || dev >= 64) return LORDBA_ERR_NO_DEVICE;
    std::lock_guard<std::mutex> g(mu);
    if (ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return LORDBA_ERR_NO_DEVICE;
        }
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return LORDBA_OK;
}
}  // namespace

extern "C" lordba_status lordba_backward_noalloc(const void* x, const void* g,
                                                 const uint32_t* packedA, const uint32_t* packedAt, const uint32_t* packedBt,
                                                 const void* s_in, const void* s_rank, const void* s_out,
                                                 const float* latentA, const float* latentB, float kappa,
                                                 const float* t_saved, int64_t t_stride,
                                                 const void* dx_base, void* dx,
                                                 float* d_s_in, float* d_s_rank, float* d_s_out,
                                                 float* d_latentA, float* d_latentB,
                                                 int64_t T, int64_t d_in, int64_t d_out, int64_t r, void* stream) {
    if (!supported(T, d_in, d_out, r)) return LORDBA_ERR_DIM;
    // the size check comes first: a shape beyond the array is refused whatever else is wrong with the call
    if (make_plan(T, d_in, d_out, r).words * 4 > static_cast<size_t>(LORDBA_BACKWARD_NOALLOC_MAX_BYTES)) return LORDBA_ERR_WORKSPACE;
    void* ws = nullptr;
    const lordba_status s = noalloc_scratch(&ws);
    if (s != LORDBA_OK) return s;
    // Nothing in the scratch has to start at zero: every word a kernel reads was written earlier in the same call.
    return backward_impl(x, g, packedA, packedAt, packedBt, s_in, s_rank, s_out, latentA, latentB, kappa, t_saved, t_stride, dx_base, dx,
                         d_s_in, d_s_rank, d_s_out, d_latentA, d_latentB, ws, LORDBA_BACKWARD_NOALLOC_MAX_BYTES, T, d_in, d_out, r, 1, stream);
}
