// PTQ-LoRDBA at envelope rank 1 on the device: the scaled consensus ADMM that fits diag(alpha) B1 diag(beta) B2 diag(gamma)
// to a low-rank update A* (B*)^T (appendix on post-training quantisation: Eq. (ptq-problem), the ordered updates
// Eq. (u-step-1), Eq. (u-step-2), Eq. (scales-step), Eq. (m-y-step), Alg. PTQ-LoRDBA; closed-form scale updates
// Eq. (alpha-update), Eq. (gamma-update), Eq. (beta-gram), Eq. (beta-pinv); warm start Eq. (svd-init)).
//
// The N x M target is never formed.  With the target kept as its factors, every quantity a sweep needs is a function of
// two small "Gram pairs", one per side of the adapter:
//     side 1 (rows i of U1, factor rows a*_i, scale alpha):  S1 = sum_i alpha_i^2 u_i u_i^T  [R, R],  K1 = sum_i alpha_i u_i a*_i^T  [R, r0]
//     side 2 (columns j of U2, factor rows b*_j, scale gamma): S2 = sum_j gamma_j^2 v_j v_j^T,        K2 = sum_j gamma_j v_j b*_j^T
// e.g. the Tikhonov step of row i of U1 is (alpha_i^2 (beta beta^T o S2) + rho_1 I) u = alpha_i beta o (K2 a*_i) + rho_1 (M1 - Y1)_i.
// The two sides are mirror images (the transposed target swaps them), so one kernel serves both.  U2 is held transposed,
// [M, R] row-major, which is also the layout of S_B.  All arithmetic is fp64; sums run in a fixed order (no atomics), so
// a call is reproducible bit for bit.
//
// Each row kernel works on blocks of 32 rows and ends by writing its block's share of its side's Gram pair; a small
// kernel adds the shares up (each workgroup of a row kernel doing so itself would pull every share through its own
// compute unit's 64 B/clk path to L2: measured 9 us per launch against 4.8 us for the extra launch).  A sweep is nine
// launches: two Tikhonov steps (each followed at once by the sign and dual update of its rows, which needs nothing
// else), alpha, gamma, each with its totals kernel, and beta with the penalty control.  A flag in device memory ends the
// loop: once the sign matrices repeat, the remaining launches return at once, so the host never waits on the device
// inside the loop (lordba_ptq_sweeps lets a caller that is willing to wait enqueue the run in pieces instead).
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <math.h>
#include <stdint.h>

#include <mutex>

#include "lordba.h"
#include "lordba_host_util.h"

namespace {

constexpr int kRows = 32;      // rows of one side per workgroup
constexpr int kThreads = 256;  // four waves: the warm-start and export kernels
constexpr int kRowThreads = 512;  // eight waves: the kernels of a sweep
static_assert(LORDBA_PTQ_MAX_RANK == 32, "the Tikhonov kernel is instantiated for ranks up to 16 and up to 32");
constexpr double kRankFloor = 1e-12;  // a singular value of the update below this fraction of the largest counts as zero
constexpr int kInfoHead = 8;   // info[0..7]: sweeps, frozen, rho, ||T||_F^2, degenerate, reserved; then one objective per sweep

enum Ctrl { kRho = 0, kYfac = 1, kDone = 2, kSweeps = 3, kNormT2 = 4, kFrozen = 5, kDegenerate = 6, kCtrlCount = 8 };

struct PtqArgs {
    const __half* F[2];  // A_star [N, r0], B_star [M, r0]
    int64_t n[2];        // N, M
    int R, r0;
    int nb[2];           // row blocks per side
    double* X[2];        // continuous iterates U1 [N, R], U2^T [M, R]
    double* Mm[2];       // their +-1 copies
    double* Y[2];        // scaled duals
    double* scale[2];    // alpha [N], gamma [M]
    double* beta;        // [R]
    double* part[2];     // per block shares of each side, [nb, pstride]: S (R*R), K (R*r0), then the block's squared
                         // consensus gap and its number of sign changes in the sweep (written by the Tikhonov kernel only)
    int pstride;
    double* tot[2];      // the shares of each side added up (same layout as one share), written by the totals kernel
    double* Z[2];        // warm start: [r0, R] maps from factor rows to singular-vector entries
    double* ctrl;        // [kCtrlCount]
    double* info;
    int K;
    double tau, mu;
};

__device__ inline void wave_sync() {
    // Lanes of one wave exchange data through LDS; the LDS serves a wave's requests in order, so only the compiler has to
    // be kept from moving accesses across this point.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// v rotated by N lanes within each row of 16 lanes (data-parallel primitive: no LDS traffic).
template <int N>
__device__ inline double row_rotate16(double v) {
    const int lo = __double2loint(v), hi = __double2hiint(v);
    constexpr int ctrl = 0x120 + N;   // row_ror:N
    return __hiloint2double(__builtin_amdgcn_update_dpp(0, hi, ctrl, 0xf, 0xf, false),
                            __builtin_amdgcn_update_dpp(0, lo, ctrl, 0xf, 0xf, false));
}

// Sum over each group of gs consecutive lanes (gs = 16, 32 or 64), returned in every lane of the group.  Within rows of 16
// lanes the partial sums travel by rotation, across rows by lane exchange.
__device__ inline double group_sum(double v, int gs) {
    for (int m = gs >> 1; m >= 16; m >>= 1) v += __shfl_xor(v, m, 64);
    v += row_rotate16<8>(v);
    v += row_rotate16<4>(v);
    v += row_rotate16<2>(v);
    v += row_rotate16<1>(v);
    return v;
}

__device__ inline int group_size_for(int R) { return R <= 16 ? 16 : (R <= 32 ? 32 : 64); }

// In-place Cholesky factor (lower triangle) of the n x n matrix H (leading dimension ld) by the lanes l = 0..gs-1 of one
// group; lane l owns column l.  Returns false (in every lane) if a pivot is not above `floor`.
__device__ inline bool group_cholesky(double* H, int ld, int n, int l, double floor = 0.0) {
    bool ok = true;
    for (int k = 0; k < n; ++k) {
        const double hkk = H[k * ld + k];
        ok = ok && (hkk > floor);
        const double d = sqrt(hkk);
        if (l > k && l < n) H[l * ld + k] = H[l * ld + k] / d;
        if (l == k) H[k * ld + k] = d;
        wave_sync();
        if (l > k && l < n) {
            const double ljk = H[l * ld + k];
            for (int i = l; i < n; ++i) H[i * ld + l] -= H[i * ld + k] * ljk;
        }
        wave_sync();
    }
    return ok;
}

// Solves L L^T x = b for the factor left by group_cholesky; lane l passes b_l and receives x_l.  `base` is the first
// lane of the group within the wave.
__device__ inline double group_solve(const double* H, int ld, int n, int l, int base, double b) {
    for (int k = 0; k < n; ++k) {
        const double yk = __shfl(b, base + k, 64) / H[k * ld + k];
        if (l == k) b = yk;
        if (l > k && l < n) b -= H[l * ld + k] * yk;
    }
    for (int k = n - 1; k >= 0; --k) {
        const double xk = __shfl(b, base + k, 64) / H[k * ld + k];
        if (l == k) b = xk;
        if (l < k) b -= H[k * ld + l] * xk;
    }
    return b;
}

// This block's share of a side's Gram pair from its rows in LDS: xs [kRows, R], cs [kRows] (0 past the end), fs [kRows, r0]
// with row stride fstride.  The rows are first scaled in place (xs <- cs o xs; the callers are done with xs), then every
// thread sums its output over the rows, eight rows' operands requested at a time.
__device__ inline void gram_share(double* xs, const double* cs, const double* fs, int fstride, int R, int r0, double* out) {
    for (int o = threadIdx.x; o < kRows * R; o += blockDim.x) xs[o] *= cs[o / R];
    __syncthreads();
    const int RR = R * R;
    for (int o = threadIdx.x; o < RR + R * r0; o += blockDim.x) {
        const bool gram = o < RR;
        const int k = gram ? o / R : (o - RR) / r0;
        const int j = gram ? o - k * R : (o - RR) - k * r0;
        const double* right = gram ? xs + j : fs + j;
        const int rstride = gram ? R : fstride;
        double acc = 0.0;
        for (int row0 = 0; row0 < kRows; row0 += 8) {
            double u[8], v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                u[e] = xs[(row0 + e) * R + k];
                v[e] = right[(row0 + e) * rstride];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) acc = fma(u[e], v[e], acc);
        }
        out[o] = acc;
    }
}

// Rows row0 .. row0 + kRows - 1 of a factor into LDS as doubles, row stride fstride (zeros past the end of the factor).
__device__ inline void load_factor_rows(const __half* F, int64_t n, int r0, int64_t row0, double* fs, int fstride) {
    for (int o = threadIdx.x; o < kRows * r0; o += blockDim.x) {
        const int row = o / r0, q = o - row * r0;
        fs[row * fstride + q] = row0 + row < n ? static_cast<double>(__half2float(F[row0 * r0 + o])) : 0.0;
    }
}

extern __shared__ double lds[];

// tot[side][o] = sum over the blocks of part[side][b][o], o < count: 64 outputs per workgroup of 256 threads.  Wave w adds
// up the shares b = w, w + 4, w + 8, ... (32 loads in flight per thread), and the four partial sums are added in the
// order of w: a fixed order, whatever the timing.
__global__ __launch_bounds__(256) void lordba_ptq_totals_kernel(PtqArgs a, int side, int count, int always) {
    if (!always && a.ctrl[kDone] != 0.0) return;
    __shared__ double partial[4][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int o = blockIdx.x * 64 + lane;
    const int oc = o < count ? o : count - 1;
    constexpr int kBatch = 32;
    const double* part = a.part[side] + oc;
    const int nb = a.nb[side];
    double acc = 0.0;
    for (int b0 = w; b0 < nb; b0 += 4 * kBatch) {
        double v[kBatch];
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const int b = b0 + 4 * j < nb ? b0 + 4 * j : nb - 1;
            v[j] = part[static_cast<int64_t>(b) * a.pstride];
        }
#pragma unroll
        for (int j = 0; j < kBatch; ++j) acc += (b0 + 4 * j < nb) ? v[j] : 0.0;
    }
    partial[w][lane] = acc;
    __syncthreads();
    if (w == 0 && o < count) a.tot[side][o] = (partial[0][lane] + partial[1][lane]) + (partial[2][lane] + partial[3][lane]);
}

// The totals of a side into LDS.
__device__ inline void load_totals(const double* tot, int count, double* dst) {
    for (int o = threadIdx.x; o < count; o += blockDim.x) dst[o] = tot[o];
}

// ---- warm start (Eq. (svd-init)) ----------------------------------------------------------------------------------

// Tall-skinny QR of the two factors: only the triangular factors are wanted (A* = Qa Ra, B* = Qb Rb with orthonormal Qa, Qb
// that are never formed).  One workgroup factors a panel of up to kQrRows rows by Householder reflections and writes the
// panel's r0 x r0 upper-triangular factor; the panels of level 0 are rows of the fp16 factor (taken at their exact
// values), those of a higher level the stacked factors of `group` panels of the level below, until one is left.  The
// triangular factor of a Householder QR is backward stable column by column, so the singular triplets of the update
// that the warm start takes from Ra Rb^T carry an error of eps sigma_1 / sigma_k, as a dense decomposition's would
// (through the Gram matrices A*^T A*, B*^T B* it would be the square of that ratio).
constexpr int kQrRows = 256;

struct QrLevel {
    const double* src[2];   // level >= 1: the factors of the level below, [count_in, r0, r0]
    double* dst[2];         // [count_out, r0, r0]
    int count_in[2];        // level 0: unused
    int count_out[2];       // 0: this side is finished (or has nothing at this level)
    int level, group;
};


__global__ __launch_bounds__(256) void lordba_ptq_qr_kernel(PtqArgs a, QrLevel lv) {
    const int side = static_cast<int>(blockIdx.x) < lv.count_out[0] ? 0 : 1;
    const int blk = side == 0 ? blockIdx.x : blockIdx.x - lv.count_out[0];
    const int n = a.r0, tid = threadIdx.x;
    const int m = lv.level == 0 ? kQrRows : lv.group * n;   // rows of the panel (zero rows where the input ends)
    double* P = lds;                    // [m, n] row-major
    double* partial = P + kQrRows * n;  // [slices, n]
    double* diag = partial + 256;       // [n]
    if (lv.level == 0) {
        const int64_t row0 = static_cast<int64_t>(blk) * kQrRows, rows = a.n[side];
        const __half* F = a.F[side];
        for (int o = tid; o < kQrRows * n; o += 256) {
            const int64_t row = row0 + o / n;
            P[o] = row < rows ? static_cast<double>(__half2float(F[row0 * n + o])) : 0.0;
        }
    } else {
        const int64_t first = static_cast<int64_t>(blk) * lv.group;
        const double* src = lv.src[side] + first * n * n;
        const int64_t have = (lv.count_in[side] - first < lv.group ? lv.count_in[side] - first : lv.group) * n;  // rows that exist
        for (int o = tid; o < m * n; o += 256) P[o] = o / n < have ? src[o] : 0.0;
    }
    // thread (j, s): column j, row slice s
    const int slices = 256 / n, rps = (m + slices - 1) / slices;
    const int j = tid % n, sl = tid / n;
    const bool active = sl < slices;
    const int i_lo = sl * rps, i_hi = (sl + 1) * rps < m ? (sl + 1) * rps : m;
    __syncthreads();
    for (int k = 0; k < n; ++k) {
        // the sums over the rows below the diagonal of (column k) x (column j), j >= k, slice by slice; row k's entries are
        // read here, before the barrier, because the update below rewrites them
        double alpha = 0.0, pkj = 0.0;
        if (active && j >= k) {
            alpha = P[k * n + k];
            pkj = P[k * n + j];
            double acc = 0.0;
            for (int i = (i_lo > k + 1 ? i_lo : k + 1); i < i_hi; ++i) acc = fma(P[i * n + k], P[i * n + j], acc);
            partial[sl * n + j] = acc;
        }
        __syncthreads();
        // Every thread forms the reflector's scalars itself (same values everywhere): x = column k from the diagonal down,
        // alpha its first entry; H = I - tau v v^T with v = (1, x_below / (alpha - beta)), beta = -sign(alpha) ||x||,
        // tau = (beta - alpha) / beta; H x = beta e_1.  A column that is zero below the diagonal is left as it is.
        if (active && j >= k) {
            double below2 = 0.0, dot = 0.0;
            for (int q = 0; q < slices; ++q) { below2 += partial[q * n + k]; dot += partial[q * n + j]; }
            if (below2 > 0.0) {
                const double beta = alpha < 0.0 ? sqrt(fma(alpha, alpha, below2)) : -sqrt(fma(alpha, alpha, below2));
                const double inv = 1.0 / (alpha - beta), tau = (beta - alpha) / beta;
                if (j == k) {
                    if (sl == 0) diag[k] = beta;
                } else {
                    const double w = fma(dot, inv, pkj);        // v^T (column j)
                    const double tw = tau * w, c = tw * inv;
                    for (int i = (i_lo > k + 1 ? i_lo : k + 1); i < i_hi; ++i) P[i * n + j] = fma(-c, P[i * n + k], P[i * n + j]);
                    if (sl == 0) P[k * n + j] = pkj - tw;
                }
            } else if (j == k && sl == 0) {
                diag[k] = alpha;
            }
        }
        __syncthreads();
    }
    double* dst = lv.dst[side] + static_cast<int64_t>(blk) * n * n;
    for (int o = tid; o < n * n; o += 256) {
        const int row = o / n, col = o - row * n;
        dst[o] = col > row ? P[o] : (col == row ? diag[row] : 0.0);
    }
}

// One-sided Jacobi iteration on the n x n matrix W (n <= 64) by one wave: plane rotations of column pairs, accumulated
// in V (which the caller sets to the identity), until all columns of W are orthogonal: W V_acc = (orthogonal columns).
// Round-robin order: the n / 2 column pairs of a round are disjoint, so groups of lanes rotate several pairs at once
// (lane i of a group owns row i of W and of V for the group's pair).
__device__ inline void jacobi_onesided(double* W, double* V, int n, int ld, int l) {
    const int gsz = n <= 16 ? 16 : (n <= 32 ? 32 : 64), ngroups = 64 / gsz;
    const int g = l / gsz, i = l - g * gsz;
    const int ne = n + (n & 1);  // an even number of players; with n odd, player n is a bye
    for (int sweep = 0; sweep < 60; ++sweep) {
        bool rotated = false;
        for (int round = 0; round + 1 < ne; ++round) {
            for (int m0 = 0; m0 < ne / 2; m0 += ngroups) {
                const int m = m0 + g;
                int p = 0, q = 0;
                bool valid = m < ne / 2;
                if (valid) {
                    const int lo = (round + m) % (ne - 1);
                    const int hi = m == 0 ? ne - 1 : (round + ne - 1 - m) % (ne - 1);
                    p = lo < hi ? lo : hi;
                    q = lo < hi ? hi : lo;
                    valid = q < n;
                }
                const bool mine = valid && i < n;
                const double wp = mine ? W[i * ld + p] : 0.0, wq = mine ? W[i * ld + q] : 0.0;
                const double app = group_sum(wp * wp, gsz), aqq = group_sum(wq * wq, gsz), apq = group_sum(wp * wq, gsz);
                const bool rot = valid && apq * apq > 1e-30 * (app * aqq);   // |apq| > 1e-15 sqrt(app aqq)
                if (rot && mine) {
                    // tangent of the rotation angle: with zeta = (aqq - app) / (2 apq), t = sign(zeta) / (|zeta| + sqrt(1 + zeta^2)),
                    // written with one square root and one division: t = sign(d) h / (|d| + sqrt(d^2 + h^2)), d = aqq - app, h = 2 apq
                    const double d = aqq - app, h = 2.0 * apq;
                    const double t = (signbit(d) ? -h : h) / (fabs(d) + sqrt(d * d + h * h));
                    const double cs = rsqrt(1.0 + t * t), sn = cs * t;
                    W[i * ld + p] = cs * wp - sn * wq;
                    W[i * ld + q] = sn * wp + cs * wq;
                    const double vp = V[i * ld + p], vq = V[i * ld + q];
                    V[i * ld + p] = cs * vp - sn * vq;
                    V[i * ld + q] = sn * vp + cs * vq;
                }
                rotated = rotated || (__builtin_amdgcn_ballot_w64(rot) != 0);
                wave_sync();
            }
        }
        if (!rotated) break;
    }
}

// norms[p] = the 2-norm of column p of the n x n matrix W (one wave; every lane returns after the values are in LDS).
__device__ inline void column_norms(const double* W, int n, int ld, int l, double* norms) {
    for (int p = 0; p < n; ++p) {
        const double wp = l < n ? W[l * ld + p] : 0.0;
        const double s2 = __shfl(group_sum(wp * wp, 64), 0, 64);
        if (l == 0) norms[p] = sqrt(s2);
    }
    wave_sync();
}

// One wave: the thin singular value decomposition of the target from the triangular factors of its two factors.
// With A* = Qa Ra and B* = Qb Rb (Qa, Qb with orthonormal columns, never formed) the target is Qa (Ra Rb^T) Qb^T, and a
// one-sided Jacobi iteration on the r0 x r0 core W = Ra Rb^T, W V = (orthogonal columns sigma_c u_c), gives the singular
// values of the target and its singular vectors Qb v_c, Qa u_c.  The warm start wants only their signs, and
//     (target) (Qb v_c) = A* (Rb^T v_c) = sigma_c (left vector c),     (target)^T (Qa u_c) = B* (Ra^T u_c) = sigma_c (right vector c),
// so the maps from factor rows to singular-vector entries are Z1 = Rb^T V and Z2 = Ra^T (rotated core), up to positive
// column factors that the signs do not see: no triangular system is solved, and factors without full column rank (a dead
// or repeated column, fewer rows than columns) need no other route.
__global__ __launch_bounds__(64) void lordba_ptq_svd_kernel(PtqArgs a, const double* RaG, const double* RbG) {
    const int r0 = a.r0, R = a.R, ld = r0 + 1, l = threadIdx.x;
    double* Ra = lds;
    double* Rb = Ra + r0 * ld;
    double* W = Rb + r0 * ld;
    double* V = W + r0 * ld;
    double* sig = V + r0 * ld;
    double* zs = sig + r0;   // [r0, R] one side's map before it goes to memory
    int* idx = reinterpret_cast<int*>(zs + r0 * R);
    for (int o = l; o < r0 * r0; o += 64) {
        Ra[(o / r0) * ld + o % r0] = RaG[o];
        Rb[(o / r0) * ld + o % r0] = RbG[o];
    }
    wave_sync();
    // core W = Ra Rb^T (both upper triangular), V = I; lane i owns row i of both from here on
    if (l < r0) {
        for (int j = 0; j < r0; ++j) {
            double acc = 0.0;
            for (int k = (l > j ? l : j); k < r0; ++k) acc = fma(Ra[l * ld + k], Rb[j * ld + k], acc);
            W[l * ld + j] = acc;
            V[l * ld + j] = (l == j) ? 1.0 : 0.0;
        }
    }
    wave_sync();
    jacobi_onesided(W, V, r0, ld, l);
    // singular values = column norms of the rotated core; order them (descending, ties by index)
    column_norms(W, r0, ld, l, sig);
    if (l < r0) idx[l] = l;   // (stays a valid index wherever non-finite values make the ranking below collide)
    wave_sync();
    if (l < r0) {   // position of column l in the descending order (ties by index)
        const double mine = sig[l];
        int before = 0;
        for (int q = 0; q < r0; ++q) {
            const double other = sig[q];
            before += (other > mine || (other == mine && q < l)) ? 1 : 0;
        }
        idx[before] = l;
    }
    wave_sync();
    if (l == 0) {
        double norm2 = 0.0;
        for (int p = 0; p < r0; ++p) norm2 += sig[idx[p]] * sig[idx[p]];
        // beyond the rank of the target the singular vectors are not defined: a singular value at the rounding level of the
        // largest one (a few eps sigma_1) is noise
        const bool good = norm2 > 0.0 && norm2 < INFINITY && sig[idx[R - 1]] > kRankFloor * sig[idx[0]];
        a.ctrl[kRho] = norm2 / (static_cast<double>(a.n[0]) * R + static_cast<double>(a.n[1]) * R);
        a.ctrl[kYfac] = 1.0;
        a.ctrl[kDone] = good ? 0.0 : 1.0;
        a.ctrl[kSweeps] = 0.0;
        a.ctrl[kNormT2] = norm2;
        a.ctrl[kFrozen] = 0.0;
        a.ctrl[kDegenerate] = good ? 0.0 : 1.0;
        a.ctrl[7] = 0.0;
    }
    wave_sync();
    if (l < R) a.beta[l] = sig[idx[l]];
    for (int side = 0; side < 2; ++side) {
        const double* Rt = side == 0 ? Rb : Ra;   // the OTHER factor's triangle, transposed: Z[i, l] = sum_{j <= i} Rt[j, i] src[j, c]
        const double* src = side == 0 ? V : W;
        if (l < R) {   // lane l: column l of the side's map, built in LDS (zs, [r0, R])
            const int c = idx[l];
            for (int i = 0; i < r0; ++i) {
                double acc = 0.0;
                for (int j = 0; j <= i; ++j) acc = fma(Rt[j * ld + i], src[j * ld + c], acc);
                zs[i * R + l] = acc;
            }
        }
        wave_sync();
        for (int o = l; o < r0 * R; o += 64) a.Z[side][o] = zs[o];
        wave_sync();
    }
}

// U = M = sign(factor row . Z), Y = 0, scale = 1, and the block's Gram share.
__global__ __launch_bounds__(kThreads) void lordba_ptq_init_rows_kernel(PtqArgs a) {
    const int side = static_cast<int>(blockIdx.x) < a.nb[0] ? 0 : 1;
    const int blk = side == 0 ? blockIdx.x : blockIdx.x - a.nb[0];
    const int R = a.R, r0 = a.r0;
    const int64_t n = a.n[side], row0 = static_cast<int64_t>(blk) * kRows;
    double* fs = lds;
    double* xs = fs + kRows * r0;
    double* cs = xs + kRows * R;
    double* zs = cs + kRows;
    load_factor_rows(a.F[side], n, r0, row0, fs, r0);
    for (int o = threadIdx.x; o < r0 * R; o += kThreads) zs[o] = a.Z[side][o];
    __syncthreads();
    for (int o = threadIdx.x; o < kRows * R; o += kThreads) {
        const int row = o / R, k = o - row * R;
        double acc = 0.0;
        for (int q = 0; q < r0; ++q) acc += fs[row * r0 + q] * zs[q * R + k];
        const double s = acc < 0.0 ? -1.0 : 1.0;
        const bool in = row0 + row < n;
        xs[o] = in ? s : 0.0;
        if (in) {
            const int64_t g = row0 * R + o;
            a.X[side][g] = s;
            a.Mm[side][g] = s;
            a.Y[side][g] = 0.0;
        }
    }
    for (int row = threadIdx.x; row < kRows; row += kThreads) {
        const bool in = row0 + row < n;
        cs[row] = in ? 1.0 : 0.0;
        if (in) a.scale[side][row0 + row] = 1.0;
    }
    __syncthreads();
    gram_share(xs, cs, fs, r0, R, r0, a.part[side] + static_cast<int64_t>(blk) * a.pstride);
}

// ---- one sweep ----------------------------------------------------------------------------------------------------

// LDS of the two row kernels: So [R*R], Ko [R*r0] (the other side's Gram pair), bs [R], fs [kRows, r0] with row stride
// r0 + 1, xs, cs, ys, kfs [kRows, R] (Ko f of every row), then the per-group areas of the Tikhonov step.
struct RowLds {
    double *So, *Ko, *bs, *fs, *xs, *cs, *ys, *kfs, *H;
    int fstride;
};
__device__ inline RowLds carve_rows(int R, int r0) {
    RowLds s;
    s.fstride = r0 + 1;
    s.So = lds;
    s.Ko = s.So + R * R;
    s.bs = s.Ko + R * r0;
    s.fs = s.bs + R;
    s.xs = s.fs + kRows * s.fstride;
    s.cs = s.xs + kRows * R;
    s.ys = s.cs + kRows;
    s.kfs = s.ys + kRows * R;
    s.H = s.kfs + kRows * R;
    return s;
}

// kfs[row][k] = Ko[k, :] . f_row for the block's rows (thread o: k = o / kRows, row = o % kRows, so that a wave reads one
// row of Ko and consecutive, padded rows of fs).  Call between two barriers.
__device__ inline void factor_products(const RowLds& s, int R, int r0) {
    for (int o = threadIdx.x; o < kRows * R; o += blockDim.x) {
        const int k = o / kRows, row = o - k * kRows;
        double acc = 0.0;
        for (int q = 0; q < r0; ++q) acc += s.Ko[k * r0 + q] * s.fs[row * s.fstride + q];
        s.kfs[row * R + k] = acc;
    }
}

// Solves H x = b for a symmetric positive definite RMAX x RMAX matrix by the RMAX lanes of one group (the wave's lanes
// base .. base + RMAX - 1; a smaller system is passed padded with an identity block, and R says how many pivots are its
// own).  Lane l passes column l of H in col[] (entries i >= l are used) and entry l of b, and receives entry l of x.
// Right-looking L D L^T factorisation with the columns in registers: a finished column is published once, unscaled, to
// Hs (LDS, RMAX x (RMAX + 1)), and the other lanes fold the scaling by its pivot into their rank-one updates.  The
// right-hand side rides along as one more row of the matrix (zrow, LDS, RMAX), which makes the forward substitution
// part of the factorisation; the backward substitution runs on lane shuffles with each lane's own column still in its
// registers.  Every loop has a fixed trip count and every LDS read is unconditional, so that the reads of a step are
// issued together.  No square root, one reciprocal per column (hardware estimate and two Newton steps).  Returns the
// smallest of the first R pivots in *min_pivot.
template <int RMAX>
__device__ inline double group_ldlt_solve(double (&col)[RMAX], double b, double* H, double* zrow, int R, int l, int base,
                                          double* min_pivot) {
    constexpr int ld = RMAX + 1;
    double minp = INFINITY, ipl = 0.0;
#pragma unroll
    for (int k = 0; k < RMAX; ++k) {
        if (l == k) {
#pragma unroll
            for (int i = k; i < RMAX; ++i) H[i * ld + k] = col[i];
            zrow[k] = b;
        }
        wave_sync();
        const double pk = H[k * ld + k], hl = H[l * ld + k], zk = zrow[k];
        double hk[RMAX];
#pragma unroll
        for (int i = k + 1; i < RMAX; ++i) hk[i] = H[i * ld + k];
        minp = fmin(minp, k < R ? pk : INFINITY);
        double ipk = __builtin_amdgcn_rcp(pk);
        ipk = fma(fma(-pk, ipk, 1.0), ipk, ipk);
        ipk = fma(fma(-pk, ipk, 1.0), ipk, ipk);
        ipl = (l == k) ? ipk : ipl;
        const double f = (l > k) ? hl * ipk : 0.0;   // L'[l][k] = H[l][k] / pivot_k for the lanes below the diagonal
#pragma unroll
        for (int i = k + 1; i < RMAX; ++i) col[i] = fma(-hk[i], f, col[i]);   // (entries i < l are updated too; they are never used)
        b = fma(-zk, f, b);                                                   // forward substitution: b as row RMAX of the matrix
    }
    // H = L' D L'^T with D the pivots and L' unit lower triangular; b now holds entry l of L'^{-1} b.
    b *= ipl;
#pragma unroll
    for (int k = RMAX - 1; k >= 1; --k) {
        const double xk = __shfl(b, base + k, 64);
        b = fma(-((l < k) ? col[k] * ipl : 0.0), xk, b);   // L'[k][l] = (lane l's own column, entry k) / pivot_l
    }
    *min_pivot = minp;
    return b;
}

// Eq. (u-step-1) / Eq. (u-step-2) for one side: per row, (c^2 (beta beta^T o So) + rho_k I) u = c beta o (Ko f) + rho_k (M - Y),
// then Eq. (m-y-step) for the same row: M = sign(u + Y), Y += u - M (a pending rescaling of Y after a penalty change is
// applied on the way).  A group of lanes solves one row: lane l keeps column l of the matrix in registers through a
// right-looking L D L^T factorisation; a finished column is published once, unscaled, to LDS together with the
// reciprocal of its pivot, and the other lanes fold the scaling into their updates (no square root, one reciprocal).
// `solve_waves` of the block's waves take part (as many as the LDS holds matrices for).
template <int RMAX>  // the carrier rank is at most RMAX (16 or 32): lanes per row and length of the register-resident column; the
                     // larger one runs with half the threads per block, so that a lane may hold twice the registers
__global__ __launch_bounds__(RMAX <= 16 ? kRowThreads : kRowThreads / 2) void lordba_ptq_ustep_kernel(PtqArgs a, int side, int solve_waves) {
    if (a.ctrl[kDone] != 0.0) return;
    const int R = a.R, r0 = a.r0, other = 1 - side, blk = blockIdx.x;
    const int64_t n = a.n[side], row0 = static_cast<int64_t>(blk) * kRows;
    const RowLds s = carve_rows(R, r0);
    const int count = R * R + R * r0;
    load_totals(a.tot[other], count, s.So);  // So and Ko are adjacent
    for (int k = threadIdx.x; k < R; k += blockDim.x) s.bs[k] = a.beta[k];
    load_factor_rows(a.F[side], n, r0, row0, s.fs, s.fstride);
    for (int row = threadIdx.x; row < kRows; row += blockDim.x) s.cs[row] = row0 + row < n ? a.scale[side][row0 + row] : 0.0;
    const double rho_k = a.ctrl[kRho] / (static_cast<double>(n) * R), yfac = a.ctrl[kYfac];
    for (int o = threadIdx.x; o < kRows * R; o += blockDim.x) {   // xs holds M until the row is solved, ys holds Y (its pending
        const bool in = row0 + o / R < n;                         // rescaling is applied where it is read, so that these loads
        s.xs[o] = in ? a.Mm[side][row0 * R + o] : 0.0;            // do not wait for the control words)
        s.ys[o] = in ? a.Y[side][row0 * R + o] : 0.0;
    }
    __syncthreads();
    factor_products(s, R, r0);
    __syncthreads();
    constexpr int gs = RMAX, groups = 64 / gs, ld = RMAX + 1;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int g = lane / gs, l = lane - g * gs, base = g * gs;
    double gap = 0.0, flips = 0.0;
    if (wave < solve_waves) {
        double* H = s.H + (wave * groups + g) * (RMAX * ld + RMAX);
        double* zrow = H + RMAX * ld;
        const int rows_per_pass = solve_waves * groups;
        const bool act = l < R;       // the other lanes of the group carry the identity block that pads the system
        const int lc = act ? l : 0;   // a valid column for their reads
        for (int pass = 0; pass < kRows / rows_per_pass; ++pass) {
            const int row = pass * rows_per_pass + wave * groups + g;
            const bool in = row0 + row < n;
            const double c = s.cs[row], c2 = c * c, bl = s.bs[lc];
            const double m_old = s.xs[row * R + lc], y_old = yfac * s.ys[row * R + lc];
            double b = act ? c * bl * s.kfs[row * R + lc] + rho_k * (m_old - y_old) : 0.0;
            double col[RMAX];
#pragma unroll
            for (int i = 0; i < RMAX; ++i) {
                const int ic = i < R ? i : 0;
                const double own = c2 * (s.bs[ic] * bl) * s.So[ic * R + lc] + (i == l ? rho_k : 0.0);
                col[i] = (act && i < R) ? own : (i == l ? 1.0 : 0.0);
            }
            double min_pivot;   // positive: the matrix is a Gram matrix plus rho_k I
            b = group_ldlt_solve<RMAX>(col, b, H, zrow, R, l, base, &min_pivot);
            if (act) {
                const double x = b;
                const double mn = (x + y_old) < 0.0 ? -1.0 : 1.0;
                s.xs[row * R + l] = in ? x : 0.0;
                if (in) {
                    const int64_t gi = (row0 + row) * R + l;
                    a.X[side][gi] = x;
                    a.Mm[side][gi] = mn;
                    a.Y[side][gi] = y_old + x - mn;
                    gap += (x - mn) * (x - mn);
                    flips += (mn != m_old) ? 1.0 : 0.0;
                }
            }
            wave_sync();
        }
    }
    gap = group_sum(gap, 64);
    flips = group_sum(flips, 64);
    double* red = s.ys;   // free once every row has taken its Y (the barrier below orders this after the last read)
    __syncthreads();
    if (lane == 0) { red[2 * wave] = gap; red[2 * wave + 1] = flips; }
    __syncthreads();
    double* share = a.part[side] + static_cast<int64_t>(blk) * a.pstride;
    gram_share(s.xs, s.cs, s.fs, s.fstride, R, r0, share);
    if (threadIdx.x == 0) {
        double gsum = 0.0, fsum = 0.0;
        for (int w = 0; w < static_cast<int>(blockDim.x >> 6); ++w) { gsum += red[2 * w]; fsum += red[2 * w + 1]; }
        share[count] = gsum;
        share[count + 1] = fsum;
    }
}

// Eq. (alpha-update) (side 0) / Eq. (gamma-update) (side 1): per row, with v = u o beta, <T_i, D_i> = v . (Ko f) and
// ||D_i||^2 = v^T So v; 0 where the denominator is 0.
__global__ __launch_bounds__(kRowThreads) void lordba_ptq_scale_kernel(PtqArgs a, int side) {
    if (a.ctrl[kDone] != 0.0) return;
    const int R = a.R, r0 = a.r0, other = 1 - side, blk = blockIdx.x;
    const int64_t n = a.n[side], row0 = static_cast<int64_t>(blk) * kRows;
    const RowLds s = carve_rows(R, r0);
    load_totals(a.tot[other], R * R + R * r0, s.So);
    for (int k = threadIdx.x; k < R; k += blockDim.x) s.bs[k] = a.beta[k];
    load_factor_rows(a.F[side], n, r0, row0, s.fs, s.fstride);
    for (int o = threadIdx.x; o < kRows * R; o += blockDim.x) s.xs[o] = row0 + o / R < n ? a.X[side][row0 * R + o] : 0.0;
    __syncthreads();
    factor_products(s, R, r0);
    __syncthreads();
    const int gs = group_size_for(R), groups = 64 / gs, waves = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int g = lane / gs, l = lane - g * gs;
    const int rows_per_pass = waves * groups;
    for (int pass = 0; pass < kRows / rows_per_pass; ++pass) {
        const int row = pass * rows_per_pass + wave * groups + g;
        double num = 0.0, den = 0.0;
        if (l < R) {
            const double v = s.xs[row * R + l] * s.bs[l];
            const double kf = s.kfs[row * R + l];
            double sv = 0.0;   // (So v)_l: So is symmetric, so lane l walks column l (consecutive lanes, consecutive words)
            for (int m0 = 0; m0 < R; m0 += 8) {
                double so[8], xv[8], bv[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int m = m0 + e < R ? m0 + e : R - 1;
                    so[e] = s.So[m * R + l];
                    xv[e] = s.xs[row * R + m];
                    bv[e] = s.bs[m];
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) sv += (m0 + e < R) ? so[e] * (xv[e] * bv[e]) : 0.0;
            }
            num = v * kf;
            den = v * sv;
        }
        num = group_sum(num, gs);
        den = group_sum(den, gs);
        const double c = den > 0.0 ? num / den : 0.0;
        const bool in = row0 + row < n;
        if (l == 0) {
            s.cs[row] = in ? c : 0.0;
            if (in) a.scale[side][row0 + row] = c;
        }
    }
    __syncthreads();
    gram_share(s.xs, s.cs, s.fs, s.fstride, R, r0, a.part[side] + static_cast<int64_t>(blk) * a.pstride);
}

// beta = pinv(G) h for a symmetric positive semidefinite R x R matrix G, by one wave (Eq. (beta-pinv)).  G [R, ld] and hv [R]
// are in LDS and are overwritten; N2 is an LDS area of max(R ld, 16 * 17 + 16) doubles; perm [R] must hold the identity.
// The result goes to bt [R].  A factorisation without pivoting is tried first (ranks up to 16: its columns stay in
// registers) and kept if every pivot clears the rank tolerance 64 eps max_k G_kk; otherwise a Cholesky factorisation with
// diagonal pivoting stops at the numerical rank: with G = L L^T, L of full column rank, pinv(G) = L (L^T L)^{-2} L^T (at
// full rank the ordinary solve).
__device__ inline void beta_pinv_solve(double* G, int ld, double* hv, double* N2, int* perm, double* bt, int R, int l) {
    double dmax = (l < R) ? G[l * ld + l] : 0.0;
    for (int m = 32; m >= 1; m >>= 1) dmax = fmax(dmax, __shfl_xor(dmax, m, 64));
    const double tol = 64.0 * 2.220446049250313e-16 * dmax;
    // Fast path: G is positive definite whenever both sides' iterates have full column rank, so try the factorisation
    // without pivoting first (columns in registers, N2 as its LDS area) and keep its result if every pivot clears the rank
    // tolerance; G itself is left untouched for the pivoted factorisation below.
    bool solved = false;
    double x = 0.0;
    if (R <= 16) {   // (a 32-entry column does not stay in registers beside the rest of this kernel: those ranks pivot at once)
        const int lg = l & 15;   // the wave's four groups of 16 lanes solve the same system; the first one's result is kept
        const int lc = lg < R ? lg : 0;
        double col[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int ic = i < R ? i : 0;
            const double own = G[ic * ld + lc];
            col[i] = (i < R && lg < R) ? own : (i == lg ? 1.0 : 0.0);
        }
        double min_pivot;
        const double xf = group_ldlt_solve<16>(col, lg < R ? hv[lc] : 0.0, N2, N2 + 16 * 17, R, lg, l & ~15, &min_pivot);
        wave_sync();
        if (min_pivot > tol) { solved = true; x = xf; }
    }
    int rank = 0;
    for (int k = 0; k < R && !solved; ++k) {
        // largest remaining diagonal entry, ties to the smallest index
        double best = (l >= k && l < R) ? G[l * ld + l] : -1.0;
        int arg = l;
        for (int m = 32; m >= 1; m >>= 1) {
            const double ob = __shfl_xor(best, m, 64);
            const int oa = __shfl_xor(arg, m, 64);
            if (ob > best || (ob == best && oa < arg)) { best = ob; arg = oa; }
        }
        best = __shfl(best, 0, 64);
        arg = __shfl(arg, 0, 64);
        if (!(best > tol)) break;
        if (arg != k) {
            if (l < R) { const double u = G[k * ld + l]; G[k * ld + l] = G[arg * ld + l]; G[arg * ld + l] = u; }
            wave_sync();
            if (l < R) { const double u = G[l * ld + k]; G[l * ld + k] = G[l * ld + arg]; G[l * ld + arg] = u; }
            if (l == 0) {
                const int pi = perm[k]; perm[k] = perm[arg]; perm[arg] = pi;
                const double u = hv[k]; hv[k] = hv[arg]; hv[arg] = u;
            }
            wave_sync();
        }
        const double d = sqrt(G[k * ld + k]);
        if (l > k && l < R) G[l * ld + k] = G[l * ld + k] / d;
        if (l == k) G[k * ld + k] = d;
        wave_sync();
        if (l > k && l < R) {
            const double ljk = G[l * ld + k];
            for (int i = k + 1; i < R; ++i) G[i * ld + l] -= G[i * ld + k] * ljk;  // both triangles are kept up to date
        }
        wave_sync();
        rank = k + 1;
    }
    if (solved) {
    } else if (rank == R) {
        x = group_solve(G, ld, R, l, 0, l < R ? hv[l] : 0.0);
    } else if (rank > 0) {
        double y = 0.0;
        if (l < rank) {
            for (int i = l; i < R; ++i) y += G[i * ld + l] * hv[i];
            for (int r = 0; r < rank; ++r) {
                double acc = 0.0;
                for (int i = (r > l ? r : l); i < R; ++i) acc += G[i * ld + r] * G[i * ld + l];
                N2[r * ld + l] = acc;
            }
        }
        wave_sync();
        group_cholesky(N2, ld, rank, l);
        const double z = group_solve(N2, ld, rank, l, 0, y);
        const double w = group_solve(N2, ld, rank, l, 0, z);
        for (int c = 0; c < rank; ++c) {
            const double wc = __shfl(w, c, 64);
            if (l < R && c <= l) x += G[l * ld + c] * wc;
        }
    }
    if (l < R) bt[perm[l]] = x;
    wave_sync();
}

// Eq. (beta-gram), Eq. (beta-Schur), Eq. (beta-pinv): G = S1 o S2, h_k = K1[k, :] . K2[k, :], beta = pinv(G) h by a
// Cholesky factorisation with diagonal pivoting that stops at the numerical rank (for a positive semidefinite G = L L^T
// with L of full column rank, pinv(G) = L (L^T L)^{-2} L^T; at full rank this is the ordinary solve, which is what runs
// then).  Also the objective of Eq. (admm-problem) at the continuous iterates, from the same Gram pairs:
// f = (||T||_F^2 - 2 beta.h + beta^T G beta) / 2.  Then the end of the sweep: residual balancing of the penalty (first
// half of the run) from the consensus gaps and sign changes the Tikhonov kernels left in their shares, and the end of
// the loop when no sign changed.
__global__ __launch_bounds__(kRowThreads) void lordba_ptq_beta_kernel(PtqArgs a, int t) {
    if (a.ctrl[kDone] != 0.0) return;
    const int R = a.R, r0 = a.r0, ld = R + 1, count = R * R + R * r0;
    double* P1 = lds;              // S1, K1, gap, sign changes of side 0
    double* P2 = P1 + count + 2;   // the same of side 1
    double* G = P2 + count + 2;    // [R, ld]
    double* N2 = G + R * ld;       // [R, ld]; the unpivoted attempt uses it as its 16 x 17 area plus the 16-entry extra row
    const int n2 = R * ld > 16 * 17 + 16 ? R * ld : 16 * 17 + 16;
    double* hv = N2 + n2;          // [R] permuted right-hand side
    double* h0 = hv + R;           // [R]
    double* bt = h0 + R;           // [R] result
    int* perm = reinterpret_cast<int*>(bt + R);
    load_totals(a.tot[0], count + 2, P1);
    load_totals(a.tot[1], count + 2, P2);
    __syncthreads();
    for (int o = threadIdx.x; o < R * R; o += blockDim.x) G[(o / R) * ld + o % R] = P1[o] * P2[o];
    for (int k = threadIdx.x; k < R; k += blockDim.x) {
        double acc = 0.0;
        for (int q = 0; q < r0; ++q) acc += P1[R * R + k * r0 + q] * P2[R * R + k * r0 + q];
        hv[k] = acc;
        h0[k] = acc;
        perm[k] = k;
    }
    __syncthreads();
    if (threadIdx.x >= 64) return;
    const int l = threadIdx.x;
    beta_pinv_solve(G, ld, hv, N2, perm, bt, R, l);
    double lin = 0.0, quad = 0.0;
    if (l < R) {
        const double bl = bt[l];
        a.beta[l] = bl;
        lin = bl * h0[l];
        for (int m = 0; m < R; ++m) quad += bl * bt[m] * (P1[l * R + m] * P2[l * R + m]);
    }
    lin = group_sum(lin, 64);
    quad = group_sum(quad, 64);
    if (l != 0) return;
    a.info[kInfoHead + t] = 0.5 * (a.ctrl[kNormT2] - 2.0 * lin + quad);
    const double gap = P1[count] + P2[count], f0 = P1[count + 1], f1 = P2[count + 1];
    double rho = a.ctrl[kRho], yfac = 1.0;
    if (2 * static_cast<int64_t>(t) < a.K) {
        const double rho0 = rho / (static_cast<double>(a.n[0]) * R), rho1 = rho / (static_cast<double>(a.n[1]) * R);
        const double r = sqrt(gap), sdual = sqrt(rho0 * rho0 * 4.0 * f0 + rho1 * rho1 * 4.0 * f1);
        if (r > a.mu * sdual) { rho *= a.tau; yfac = 1.0 / a.tau; }
        else if (sdual > a.mu * r) { rho /= a.tau; yfac = a.tau; }
    }
    a.ctrl[kRho] = rho;
    a.ctrl[kYfac] = yfac;
    a.ctrl[kSweeps] = t + 1;
    if (f0 + f1 == 0.0) { a.ctrl[kFrozen] = 1.0; a.ctrl[kDone] = 1.0; }
}

// The beta update on its own (lordba_ptq_beta_solve): G [R, R] row-major and h [R] from memory, beta [R] to memory.
__global__ __launch_bounds__(64) void lordba_ptq_beta_solve_kernel(const double* Gin, const double* hin, double* out, int R) {
    const int ld = R + 1, l = threadIdx.x;
    double* G = lds;
    const int n2 = R * ld > 16 * 17 + 16 ? R * ld : 16 * 17 + 16;
    double* N2 = G + R * ld;
    double* hv = N2 + n2;
    double* bt = hv + R;
    int* perm = reinterpret_cast<int*>(bt + R);
    for (int o = l; o < R * R; o += 64) G[(o / R) * ld + o % R] = Gin[o];
    if (l < R) { hv[l] = hin[l]; perm[l] = l; }
    wave_sync();
    beta_pinv_solve(G, ld, hv, N2, perm, bt, R, l);
    if (l < R) out[l] = bt[l];
}

// ---- export -------------------------------------------------------------------------------------------------------

struct ExportArgs {
    uint32_t* packedA;  // S_A = B1^T [R, N]
    uint32_t* packedB;  // S_B = B2^T [M, R]
    __half *s_in, *s_rank, *s_out;
    int64_t wordsA, wordsB;
};

// fp64 -> fp16, round to nearest even in one rounding: through an fp32 value rounded to odd (truncate, then set the last
// bit if anything was lost), which the final rounding to the 11-bit significand cannot tell from the exact value.
__device__ inline __half half_from_double(double x) {
    float f = static_cast<float>(x);
    if (static_cast<double>(f) != x && x == x && fabsf(f) < INFINITY) {
        uint32_t u = __float_as_uint(f);
        if (fabs(static_cast<double>(f)) > fabs(x)) u -= 1;  // step towards zero: the truncated value
        f = __uint_as_float(u | 1u);
    }
    return __float2half_rn(f);
}

__global__ __launch_bounds__(kThreads) void lordba_ptq_export_kernel(PtqArgs a, ExportArgs e) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    const int64_t N = a.n[0], M = a.n[1];
    const int R = a.R;
    // a word's 32 entries are requested together (from a clamped position), then tested
    if (i < e.wordsA) {
        double v[32];
#pragma unroll
        for (int bit = 0; bit < 32; ++bit) {
            const int nbit = static_cast<int>(i * 32 + bit < N * R ? i * 32 + bit : N * R - 1);   // (N R <= 2^27)
            const int k = nbit / static_cast<int>(N), row = nbit - k * static_cast<int>(N);
            v[bit] = a.Mm[0][row * R + k];
        }
        uint32_t w = 0;
#pragma unroll
        for (int bit = 0; bit < 32; ++bit)
            if (i * 32 + bit < N * R && v[bit] < 0.0) w |= 1u << bit;
        e.packedA[i] = w;
    }
    if (i < e.wordsB) {
        double v[32];
#pragma unroll
        for (int bit = 0; bit < 32; ++bit) v[bit] = a.Mm[1][i * 32 + bit < M * R ? i * 32 + bit : M * R - 1];
        uint32_t w = 0;
#pragma unroll
        for (int bit = 0; bit < 32; ++bit)
            if (i * 32 + bit < M * R && v[bit] < 0.0) w |= 1u << bit;
        e.packedB[i] = w;
    }
    if (e.s_in && i < N) e.s_in[i] = half_from_double(a.scale[0][i]);
    if (e.s_out && i < M) e.s_out[i] = half_from_double(a.scale[1][i]);
    if (e.s_rank && i < R) e.s_rank[i] = half_from_double(a.beta[i]);
    if (i < kCtrlCount) {
        const int map[kCtrlCount] = {kSweeps, kFrozen, kRho, kNormT2, kDegenerate, 7, 7, 7};
        a.info[i] = i < 5 ? a.ctrl[map[i]] : 0.0;
    }
}

__global__ __launch_bounds__(kThreads) void lordba_ptq_fill_kernel(double* p, int64_t n, double v) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (i < n) p[i] = v;
}

struct Layout {
    size_t x[2], m[2], y[2], part[2], tot[2], z[2], ctrl, total;
    int nb[2], pstride;
};

Layout make_layout(int64_t N, int64_t M, int64_t R, int64_t r0) {
    Layout L;
    const int64_t n[2] = {N, M};
    size_t off = 0;
    auto take = [&](size_t doubles) { const size_t at = off; off += (doubles + 31) / 32 * 32; return at; };
    for (int s = 0; s < 2; ++s) L.nb[s] = static_cast<int>((n[s] + kRows - 1) / kRows);
    const int64_t pair = R * R + R * r0 + 2, sq = r0 * r0;
    L.pstride = static_cast<int>(((pair > sq ? pair : sq) + 31) / 32 * 32);
    for (int s = 0; s < 2; ++s) L.x[s] = take(n[s] * R);   // the iterates come first: U1 [N, R], then U2^T [M, R]
    for (int s = 0; s < 2; ++s) L.m[s] = take(n[s] * R);
    for (int s = 0; s < 2; ++s) L.y[s] = take(n[s] * R);
    for (int s = 0; s < 2; ++s) L.part[s] = take(static_cast<size_t>(L.nb[s]) * L.pstride);
    for (int s = 0; s < 2; ++s) L.tot[s] = take(L.pstride);
    for (int s = 0; s < 2; ++s) L.z[s] = take(r0 * R);
    L.ctrl = take(kCtrlCount);
    L.total = off * sizeof(double);
    return L;
}

bool dims_ok(int64_t N, int64_t M, int64_t R, int64_t r0, int64_t K) {
    return N >= 1 && M >= 1 && N <= (1 << 22) && M <= (1 << 22) && R >= 1 && R <= LORDBA_PTQ_MAX_RANK && r0 >= R &&
           r0 <= LORDBA_PTQ_MAX_FACTOR_RANK && K >= 1 && K <= LORDBA_PTQ_MAX_SWEEPS;
}

}  // namespace

extern "C" size_t lordba_ptq_workspace_bytes(int64_t N, int64_t M, int64_t R, int64_t r0) {
    if (!dims_ok(N, M, R, r0, 1)) return 0;
    return make_layout(N, M, R, r0).total;
}

extern "C" lordba_status lordba_ptq_sweeps(const void* A_star, const void* B_star, uint32_t* packedA, uint32_t* packedB,
                                           double* alpha, double* beta, double* gamma, void* s_in, void* s_rank, void* s_out,
                                           double* info, void* workspace, size_t workspace_bytes, int64_t N, int64_t M, int64_t R,
                                           int64_t r0, int64_t K, int64_t t_begin, int64_t t_end, double tau, double mu,
                                           void* stream_) {
    if (!dims_ok(N, M, R, r0, K) || t_begin < 0 || t_end < t_begin || t_end > K) return LORDBA_ERR_DIM;
    if (!(tau > 1.0) || !(mu > 0.0) || !(tau < 1e6) || !(mu < 1e12)) return LORDBA_ERR_VALUE;
    if (!A_star || !B_star || !packedA || !packedB || !alpha || !beta || !gamma || !info || !workspace) return LORDBA_ERR_NULL;
    const uintptr_t p16 = reinterpret_cast<uintptr_t>(A_star) | reinterpret_cast<uintptr_t>(B_star) |
                          reinterpret_cast<uintptr_t>(s_in) | reinterpret_cast<uintptr_t>(s_rank) | reinterpret_cast<uintptr_t>(s_out);
    const uintptr_t p32 = reinterpret_cast<uintptr_t>(packedA) | reinterpret_cast<uintptr_t>(packedB);
    const uintptr_t p64 = reinterpret_cast<uintptr_t>(alpha) | reinterpret_cast<uintptr_t>(beta) | reinterpret_cast<uintptr_t>(gamma) |
                          reinterpret_cast<uintptr_t>(info) | reinterpret_cast<uintptr_t>(workspace);
    if ((p16 & 1) || (p32 & 3) || (p64 & 7)) return LORDBA_ERR_ALIGN;
    const Layout L = make_layout(N, M, R, r0);
    if (workspace_bytes < L.total) return LORDBA_ERR_WORKSPACE;
    const size_t wordsA = lordba_packed_words(R, N), wordsB = lordba_packed_words(M, R);
    {   // no output may overlap an input, another output or the workspace
        struct Span { uintptr_t p; size_t n; };
        const Span spans[] = {
            {reinterpret_cast<uintptr_t>(A_star), static_cast<size_t>(N * r0) * 2}, {reinterpret_cast<uintptr_t>(B_star), static_cast<size_t>(M * r0) * 2},
            {reinterpret_cast<uintptr_t>(packedA), wordsA * 4}, {reinterpret_cast<uintptr_t>(packedB), wordsB * 4},
            {reinterpret_cast<uintptr_t>(alpha), static_cast<size_t>(N) * 8}, {reinterpret_cast<uintptr_t>(beta), static_cast<size_t>(R) * 8},
            {reinterpret_cast<uintptr_t>(gamma), static_cast<size_t>(M) * 8}, {reinterpret_cast<uintptr_t>(s_in), static_cast<size_t>(N) * 2},
            {reinterpret_cast<uintptr_t>(s_rank), static_cast<size_t>(R) * 2}, {reinterpret_cast<uintptr_t>(s_out), static_cast<size_t>(M) * 2},
            {reinterpret_cast<uintptr_t>(info), static_cast<size_t>(kInfoHead + K) * 8}, {reinterpret_cast<uintptr_t>(workspace), L.total}};
        const int ns = static_cast<int>(sizeof(spans) / sizeof(spans[0]));
        for (int i = 2; i < ns; ++i)
            for (int j = 0; j < i; ++j)
                if (spans[i].p && spans[j].p && spans[i].p < spans[j].p + spans[j].n && spans[j].p < spans[i].p + spans[i].n)
                    return LORDBA_ERR_ALIAS;
    }
    {
        const lordba_status ds = check_device();   // the kernels are built for gfx950 only
        if (ds != LORDBA_OK) return ds;
    }
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return LORDBA_ERR_NO_DEVICE; }
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    double* ws = static_cast<double*>(workspace);
    PtqArgs a;
    a.F[0] = static_cast<const __half*>(A_star);
    a.F[1] = static_cast<const __half*>(B_star);
    a.n[0] = N;
    a.n[1] = M;
    a.R = static_cast<int>(R);
    a.r0 = static_cast<int>(r0);
    for (int s = 0; s < 2; ++s) {
        a.nb[s] = L.nb[s];
        a.X[s] = ws + L.x[s];
        a.Mm[s] = ws + L.m[s];
        a.Y[s] = ws + L.y[s];
        a.part[s] = ws + L.part[s];
        a.tot[s] = ws + L.tot[s];
        a.Z[s] = ws + L.z[s];
    }
    a.scale[0] = alpha;
    a.scale[1] = gamma;
    a.beta = beta;
    a.pstride = L.pstride;
    a.ctrl = ws + L.ctrl;
    a.info = info;
    a.K = static_cast<int>(K);
    a.tau = tau;
    a.mu = mu;

    const int iR = a.R, ir0 = a.r0, ld0 = ir0 + 1, ldR = iR + 1;
    const size_t lds_qr = sizeof(double) * (kQrRows * ir0 + 256 + ir0);
    const size_t lds_svd = sizeof(double) * (4 * ir0 * ld0 + ir0 + ir0 * iR) + sizeof(int) * ir0;
    const size_t lds_init = sizeof(double) * (kRows * ir0 + kRows * iR + kRows + ir0 * iR);
    const int gs = iR <= 16 ? 16 : 32;
    // the Tikhonov kernel: as many waves solve rows at once as the LDS has room for their matrices (8, 4, 2 or 1); the scale
    // kernel has the same layout without the matrices
    const size_t lds_fixed = sizeof(double) * (iR * iR + iR * ir0 + iR + kRows * (ir0 + 1) + 3 * kRows * iR + kRows);
    const size_t lds_wave = sizeof(double) * (64 / gs) * (gs * (gs + 1) + gs);   // (systems are padded to the group's 16 or 32 lanes)
    const int ustep_threads = iR <= 16 ? kRowThreads : kRowThreads / 2;
    int solve_waves = ustep_threads / 64;
    while (solve_waves > 1 && lds_fixed + solve_waves * lds_wave > 160 * 1024) solve_waves >>= 1;
    const size_t lds_rows = lds_fixed + solve_waves * lds_wave;
    const size_t lds_beta = sizeof(double) * (2 * (iR * iR + iR * ir0 + 2) + iR * ldR + (iR * ldR > 288 ? iR * ldR : 288) + 3 * iR) + sizeof(int) * iR;
    const int nb01 = a.nb[0] + a.nb[1];

    {   // More than 64 KiB of LDS per workgroup has to be asked for; the largest request so far is remembered per device and
        // kernel, so that a call whose shapes the process has already seen makes no runtime call besides its launches
        // (it can then be captured into a HIP graph).
        static std::mutex mu;
        static size_t granted[64][7];
        const struct { const void* fn; size_t bytes; int slot; } big[] = {
            {reinterpret_cast<const void*>(lordba_ptq_qr_kernel), lds_qr, 0}, {reinterpret_cast<const void*>(lordba_ptq_svd_kernel), lds_svd, 1},
            {reinterpret_cast<const void*>(lordba_ptq_init_rows_kernel), lds_init, 2},
            {reinterpret_cast<const void*>(iR <= 16 ? lordba_ptq_ustep_kernel<16> : lordba_ptq_ustep_kernel<32>), lds_rows, iR <= 16 ? 3 : 4},
            {reinterpret_cast<const void*>(lordba_ptq_scale_kernel), lds_fixed, 5}, {reinterpret_cast<const void*>(lordba_ptq_beta_kernel), lds_beta, 6}};
        std::lock_guard<std::mutex> guard(mu);
        for (const auto& b : big) {
            if (b.bytes > 160 * 1024) return LORDBA_ERR_DIM;
            size_t& have = granted[dev & 63][b.slot];
            if (b.bytes > 48 * 1024 && have < b.bytes) {
                if (hipFuncSetAttribute(b.fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(b.bytes)) != hipSuccess) {
                    (void)hipGetLastError();
                    return LORDBA_ERR_LAUNCH;
                }
                have = b.bytes;
            }
        }
    }
    // A launch the runtime refuses (say, an LDS request it does not grant) is reported at once, not only after the last one.
    bool launch_failed = false;
    auto launched = [&]() { if (hipGetLastError() != hipSuccess) launch_failed = true; };
    const int count = iR * iR + iR * ir0;
    auto totals = [&](int side, int n, int always) {
        hipLaunchKernelGGL(lordba_ptq_totals_kernel, dim3((n + 63) / 64), dim3(256), 0, stream, a, side, n, always);
    };
    if (t_begin == 0) {   // the warm start; a later call continues from the state the workspace holds
        hipLaunchKernelGGL(lordba_ptq_fill_kernel, dim3((kInfoHead + K + kThreads - 1) / kThreads), dim3(kThreads), 0, stream, info,
                           kInfoHead + K, 0.0);
        // The triangular factors of A* and B*: panels of kQrRows rows, then groups of panel factors, level by level until one
        // factor per side is left.  The factors of a level live in the area of the Gram shares (not in use yet): even
        // levels at its start, odd levels behind the level-0 factors.
        const double* Rfinal[2] = {nullptr, nullptr};
        {
            const int group = kQrRows / ir0;
            int count[2];
            const double* src[2] = {nullptr, nullptr};
            for (int s = 0; s < 2; ++s) count[s] = static_cast<int>((a.n[s] + kQrRows - 1) / kQrRows);
            const size_t c0[2] = {static_cast<size_t>(count[0]), static_cast<size_t>(count[1])};
            for (int level = 0; Rfinal[0] == nullptr || Rfinal[1] == nullptr; ++level) {
                QrLevel lv;
                lv.level = level;
                lv.group = group;
                for (int s = 0; s < 2; ++s) {
                    lv.src[s] = src[s];
                    lv.count_in[s] = count[s];
                    lv.count_out[s] = Rfinal[s] != nullptr ? 0 : (level == 0 ? count[s] : (count[s] + group - 1) / group);
                    lv.dst[s] = a.part[s] + ((level & 1) ? c0[s] * ir0 * ir0 : 0);
                }
                hipLaunchKernelGGL(lordba_ptq_qr_kernel, dim3(lv.count_out[0] + lv.count_out[1]), dim3(256), lds_qr, stream, a, lv);
                launched();
                for (int s = 0; s < 2; ++s) {
                    if (lv.count_out[s] == 0) continue;
                    src[s] = lv.dst[s];
                    count[s] = lv.count_out[s];
                    if (count[s] == 1) Rfinal[s] = lv.dst[s];
                }
            }
        }
        hipLaunchKernelGGL(lordba_ptq_svd_kernel, dim3(1), dim3(64), lds_svd, stream, a, Rfinal[0], Rfinal[1]);
        hipLaunchKernelGGL(lordba_ptq_init_rows_kernel, dim3(nb01), dim3(kThreads), lds_init, stream, a);
        launched();
        totals(1, count, 0);
        hipLaunchKernelGGL(lordba_ptq_scale_kernel, dim3(a.nb[0]), dim3(kRowThreads), lds_fixed, stream, a, 0);
        totals(0, count, 0);
        hipLaunchKernelGGL(lordba_ptq_scale_kernel, dim3(a.nb[1]), dim3(kRowThreads), lds_fixed, stream, a, 1);
        totals(1, count, 0);
        launched();
        if (launch_failed) return LORDBA_ERR_LAUNCH;
    }
    for (int t = static_cast<int>(t_begin); t < static_cast<int>(t_end); ++t) {
        for (int side = 0; side < 2; ++side) {
            if (iR <= 16)
                hipLaunchKernelGGL(lordba_ptq_ustep_kernel<16>, dim3(a.nb[side]), dim3(kRowThreads), lds_rows, stream, a, side, solve_waves);
            else
                hipLaunchKernelGGL(lordba_ptq_ustep_kernel<32>, dim3(a.nb[side]), dim3(ustep_threads), lds_rows, stream, a, side, solve_waves);
            totals(side, count + 2, 0);
        }
        hipLaunchKernelGGL(lordba_ptq_scale_kernel, dim3(a.nb[0]), dim3(kRowThreads), lds_fixed, stream, a, 0);
        totals(0, count, 0);
        hipLaunchKernelGGL(lordba_ptq_scale_kernel, dim3(a.nb[1]), dim3(kRowThreads), lds_fixed, stream, a, 1);
        totals(1, count, 0);
        hipLaunchKernelGGL(lordba_ptq_beta_kernel, dim3(1), dim3(kRowThreads), lds_beta, stream, a, t);
        launched();
        if (launch_failed) return LORDBA_ERR_LAUNCH;
    }
    ExportArgs e;
    e.packedA = packedA;
    e.packedB = packedB;
    e.s_in = static_cast<__half*>(s_in);
    e.s_rank = static_cast<__half*>(s_rank);
    e.s_out = static_cast<__half*>(s_out);
    e.wordsA = static_cast<int64_t>(wordsA);
    e.wordsB = static_cast<int64_t>(wordsB);
    int64_t most = static_cast<int64_t>(wordsA > wordsB ? wordsA : wordsB);
    if (N > most) most = N;
    if (M > most) most = M;
    if (most < kCtrlCount) most = kCtrlCount;
    hipLaunchKernelGGL(lordba_ptq_export_kernel, dim3(static_cast<unsigned>((most + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream, a, e);
    return hipGetLastError() == hipSuccess ? LORDBA_OK : LORDBA_ERR_LAUNCH;
}

extern "C" lordba_status lordba_ptq(const void* A_star, const void* B_star, uint32_t* packedA, uint32_t* packedB,
                                    double* alpha, double* beta, double* gamma, void* s_in, void* s_rank, void* s_out,
                                    double* info, void* workspace, size_t workspace_bytes, int64_t N, int64_t M, int64_t R,
                                    int64_t r0, int64_t K, double tau, double mu, void* stream) {
    return lordba_ptq_sweeps(A_star, B_star, packedA, packedB, alpha, beta, gamma, s_in, s_rank, s_out, info, workspace,
                             workspace_bytes, N, M, R, r0, K, 0, K, tau, mu, stream);
}

extern "C" lordba_status lordba_ptq_beta_solve(const double* G, const double* h, double* beta, int64_t R, void* stream) {
    if (R < 1 || R > LORDBA_PTQ_MAX_RANK) return LORDBA_ERR_DIM;
    if (!G || !h || !beta) return LORDBA_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(G) | reinterpret_cast<uintptr_t>(h) | reinterpret_cast<uintptr_t>(beta)) & 7) return LORDBA_ERR_ALIGN;
    const uintptr_t pb = reinterpret_cast<uintptr_t>(beta), pg = reinterpret_cast<uintptr_t>(G), ph = reinterpret_cast<uintptr_t>(h);
    const size_t nb = static_cast<size_t>(R) * 8, ng = static_cast<size_t>(R) * R * 8;
    if ((pb < pg + ng && pg < pb + nb) || (pb < ph + nb && ph < pb + nb)) return LORDBA_ERR_ALIAS;
    const lordba_status ds = check_device();
    if (ds != LORDBA_OK) return ds;
    const int iR = static_cast<int>(R), ld = iR + 1;
    const size_t lds_bytes = sizeof(double) * (iR * ld + (iR * ld > 288 ? iR * ld : 288) + 2 * iR) + sizeof(int) * iR;
    hipLaunchKernelGGL(lordba_ptq_beta_solve_kernel, dim3(1), dim3(64), lds_bytes, static_cast<hipStream_t>(stream), G, h, beta, iR);
    return hipGetLastError() == hipSuccess ? LORDBA_OK : LORDBA_ERR_LAUNCH;
}
