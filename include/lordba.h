/*
 * lordba.h - C ABI of the MI355X (gfx950) LoRDBA adapter-forward library.
 *
 * The library evaluates the unmerged LoRDBA side branch of one adapted projection and adds it to
 * the base projection's output (paper: Def. 1 and Eq. (lordba) with one scale envelope, l = 1;
 * Eq. (adapter-mode-fwd); evaluation order of Eq. (lordba-fwd), Sec. 3.3):
 *
 *     y_out[t, j] = y_base[t, j]
 *                 + s_out[j] * sum_k S_B[j, k] * s_rank[k] * sum_i S_A[k, i] * s_in[i] * x[t, i]
 *
 * Notation bridge (paper, row-vector convention X DeltaW  ->  this header):
 *     N, M, R, T            ->  d_in, d_out, r, T
 *     B1 in {+-1}^{N x R}   ->  S_A = B1^T, logical shape [r, d_in]
 *     B2 in {+-1}^{R x M}   ->  S_B = B2^T, logical shape [d_out, r]
 *     alpha, beta, gamma    ->  s_in[d_in], s_rank[r], s_out[d_out]   (fp16, any finite real value)
 *     W0^T x (base output)  ->  y_base (an input; the base GEMM is not part of this library)
 *
 * Canonical packed carrier format (the paper says only "bit-packed", Sec. 3.3; storage is
 * R(N+M) bits, Eq. (lordba-bits)).  A [rows, cols] sign matrix is the row-major bit stream
 * n = row * cols + col; bit n is bit (n mod 32) of the little-endian uint32 word (n div 32);
 * bit = 1 encodes -1 and bit = 0 encodes +1 (the IEEE sign-bit convention, so applying a
 * carrier entry is an XOR into a sign bit); pad bits in the last word are 0.  packedA holds
 * S_A as [r, d_in], packedB holds S_B as [d_out, r].
 *
 * All functions return a lordba_status; none throws, aborts or prints.
 */
#ifndef LORDBA_H
#define LORDBA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int lordba_status;
enum {
    LORDBA_OK = 0,
    LORDBA_ERR_NULL = 1,      /* a required pointer is NULL                                   */
    LORDBA_ERR_DIM = 2,       /* T < 0, d_in < 1, d_out < 1, r < 1, r > LORDBA_MAX_RANK, or a
                                 size that does not fit 32-bit indexing of one row             */
    LORDBA_ERR_VALUE = 3,     /* a sign entry that is not +-1 (int8 variant) or is NaN (f32)  */
    LORDBA_ERR_ALIAS = 4,     /* y_out overlaps an input other than being exactly y_base      */
    LORDBA_ERR_ALIGN = 5,     /* a pointer is not aligned to its element size                 */
    LORDBA_ERR_NO_DEVICE = 6, /* no usable HIP device / not a gfx950 device                   */
    LORDBA_ERR_LAUNCH = 7,    /* the HIP runtime rejected the launch                          */
    LORDBA_ERR_ALGO = 8,      /* lordba_forward_algo: the requested kernel cannot run this shape */
    LORDBA_ERR_WORKSPACE = 9  /* lordba_backward, lordba_ptq: the workspace is smaller than their ..._workspace_bytes */
};

#define LORDBA_MAX_RANK 64
#define LORDBA_MAX_ENVELOPES 4

/* Number of uint32 words of a packed [rows, cols] sign matrix: ceil(rows * cols / 32).
 * Returns 0 if rows or cols is negative. */
size_t lordba_packed_words(int64_t rows, int64_t cols);

/* HOST function (all pointers are host memory; no device work).  Packs both carriers of one
 * adapter into the canonical format above (Sec. 3.3: the packed {B1, B2} is stored once per adapter).
 *   signsA : int8[r * d_in],  values in {-1, +1}, row-major [r, d_in]      (S_A)
 *   signsB : int8[d_out * r], values in {-1, +1}, row-major [d_out, r]     (S_B)
 *   packedA: uint32[lordba_packed_words(r, d_in)]   out, caller-owned
 *   packedB: uint32[lordba_packed_words(d_out, r)]  out, caller-owned
 * Any other entry value -> LORDBA_ERR_VALUE (outputs are then unspecified).  1 <= r <= 64. */
lordba_status lordba_pack_signs(const int8_t* signsA, const int8_t* signsB,
                                uint32_t* packedA, uint32_t* packedB,
                                int64_t d_in, int64_t d_out, int64_t r);

/* HOST function.  Same, from real-valued latent carriers, binarised with sign(0) = +1
 * (Sec. 2, Notation; B = sign(H) of Sec. 3.2).  Compared by value: -0.0 -> +1.  NaN -> LORDBA_ERR_VALUE. */
lordba_status lordba_pack_signs_f32(const float* latentA, const float* latentB,
                                    uint32_t* packedA, uint32_t* packedB,
                                    int64_t d_in, int64_t d_out, int64_t r);

/* HOST function.  Inverse of the packing: int8 +-1 matrices from canonical words. */
lordba_status lordba_unpack_signs(const uint32_t* packedA, const uint32_t* packedB,
                                  int8_t* signsA, int8_t* signsB,
                                  int64_t d_in, int64_t d_out, int64_t r);

/* DEVICE function: the adapter forward branch (Eq. (lordba-fwd) added to the base output,
 * Eq. (adapter-mode-fwd)).  Every pointer is DEVICE memory on the current HIP device, row-major
 * and contiguous; the caller owns all of it.  The call only enqueues work on `stream`
 * (a hipStream_t passed as void*; NULL = the default stream): it never synchronises, allocates
 * or frees, and uses no workspace.
 *   x      : fp16 [T, d_in]        s_in  : fp16 [d_in]
 *   packedA: uint32, S_A packed    s_rank: fp16 [r]
 *   packedB: uint32, S_B packed    s_out : fp16 [d_out]
 *   y_base : fp16 [T, d_out]       y_out : fp16 [T, d_out]  (out)
 * y_out may be the very same pointer as y_base (in-place update); any other overlap of y_out with
 * an input -> LORDBA_ERR_ALIAS.  T == 0 -> LORDBA_OK and no work (x, y_base, y_out may then be NULL).
 * 1 <= r <= 64.
 * Arithmetic: fp16 inputs at their exact values, products s_in*x exact, fp32 accumulation, one
 * round-to-nearest-even to fp16 at the end; every token row is within 1e-3 relative L2 of the
 * exact result.  Shapes with d_in % 32 == 0, d_out % 8 == 0 and 16-byte aligned pointers take the
 * matrix-core kernel; anything else takes a slower general kernel with the same results.
 * Non-finite inputs propagate by IEEE rules; nothing is clamped. */
lordba_status lordba_forward(const void* x, const uint32_t* packedA, const uint32_t* packedB,
                             const void* s_in, const void* s_rank, const void* s_out,
                             const void* y_base, void* y_out,
                             int64_t T, int64_t d_in, int64_t d_out, int64_t r, void* stream);

/* Same as lordba_forward with the kernel chosen by the caller (benchmarks and tests):
 *   LORDBA_ALGO_AUTO      what lordba_forward does
 *   LORDBA_ALGO_GENERAL   vector-ALU kernel, one workgroup per token row, any shape
 *   LORDBA_ALGO_MFMA_T8   matrix-core kernel, 8 token rows per workgroup
 *   LORDBA_ALGO_MFMA_T16  matrix-core kernel, 16 token rows per workgroup
 * Values 4..7 select the same matrix-core kernel with fewer waves per workgroup (tuning only).
 * A kernel that cannot run the shape -> LORDBA_ERR_ALGO. */
enum { LORDBA_ALGO_AUTO = 0, LORDBA_ALGO_GENERAL = 1, LORDBA_ALGO_MFMA_T8 = 2, LORDBA_ALGO_MFMA_T16 = 3 };
lordba_status lordba_forward_algo(const void* x, const uint32_t* packedA, const uint32_t* packedB,
                                  const void* s_in, const void* s_rank, const void* s_out,
                                  const void* y_base, void* y_out,
                                  int64_t T, int64_t d_in, int64_t d_out, int64_t r, void* stream,
                                  int algo);

/* DEVICE function: the forward branch of an adapter with `ell` scale envelopes over the same carriers
 * (Def. 1 / Eq. (lordba) with envelope rank l = ell; Sec. 3.3: the packed carriers are stored once and
 * shared by all envelopes):
 *   y_out[t, j] = y_base[t, j] + sum_{e < ell} s_out[e, j] * sum_k S_B[j, k] * s_rank[e, k] * sum_i S_A[k, i] * s_in[e, i] * x[t, i]
 * Arguments as lordba_forward, except
 *   s_in  : fp16 [ell, d_in]     s_rank: fp16 [ell, r]     s_out : fp16 [ell, d_out]     (row-major, contiguous)
 *   1 <= ell <= LORDBA_MAX_ENVELOPES; anything else -> LORDBA_ERR_DIM.  ell == 1 is lordba_forward.
 * x and y_base are read once and y_out written once whatever ell is; the envelopes are accumulated in
 * fp32 in their order and the sum is rounded once to fp16.  Same error bound, aliasing rules, stream
 * semantics (enqueue only, no allocation, no workspace) and error codes as lordba_forward. */
lordba_status lordba_forward_multi(const void* x, const uint32_t* packedA, const uint32_t* packedB,
                                   const void* s_in, const void* s_rank, const void* s_out,
                                   const void* y_base, void* y_out,
                                   int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t ell, void* stream);

/* Same with the kernel chosen by the caller: LORDBA_ALGO_AUTO, _GENERAL, _MFMA_T8 or _MFMA_T16; for ell >= 2 the tuning
 * values 6 and 7 select the 8-row / 16-row matrix-core kernel on 8 waves per workgroup (4 and 5 exist for ell == 1 only). */
lordba_status lordba_forward_multi_algo(const void* x, const uint32_t* packedA, const uint32_t* packedB,
                                        const void* s_in, const void* s_rank, const void* s_out,
                                        const void* y_base, void* y_out,
                                        int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t ell,
                                        void* stream, int algo);

/* DEVICE function: one batch served by several adapters of the same shape (Sec. 3.3: adapters are hot-swappable and
 * served concurrently over one frozen base; Eq. (adapter-mode-fwd) holds row by row).  Token row t goes through adapter
 * adapter_of_row[t] of a pool; a row whose index is outside [0, n_adapters) has no adapter and y_out[t] = y_base[t].
 *   packedA_pool : uint32 [n_adapters, lordba_packed_words(r, d_in)]    each adapter's S_A in the canonical format
 *   packedB_pool : uint32 [n_adapters, lordba_packed_words(d_out, r)]   each adapter's S_B
 *   s_in_pool    : fp16 [n_adapters, d_in]    s_rank_pool: fp16 [n_adapters, r]    s_out_pool: fp16 [n_adapters, d_out]
 *   adapter_of_row: int32 [T], device memory, any order (rows sorted by adapter are processed fastest: the kernel
 *                  works on runs of equal index inside 8-row tiles)
 * All other arguments, the arithmetic, the error bound, aliasing rules (y_out may be y_base), stream semantics (enqueue
 * only, no allocation, no workspace) and error codes as lordba_forward; 1 <= n_adapters <= 2^20.  The index array is
 * read on the device only: it is not validated by the host, out-of-range entries are defined as "no adapter". */
lordba_status lordba_forward_batched(const void* x, const uint32_t* packedA_pool, const uint32_t* packedB_pool,
                                     const void* s_in_pool, const void* s_rank_pool, const void* s_out_pool,
                                     const int32_t* adapter_of_row, const void* y_base, void* y_out,
                                     int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t n_adapters,
                                     void* stream);

/* Same with the kernel chosen by the caller: LORDBA_ALGO_AUTO, LORDBA_ALGO_GENERAL or LORDBA_ALGO_MFMA_T8. */
lordba_status lordba_forward_batched_algo(const void* x, const uint32_t* packedA_pool, const uint32_t* packedB_pool,
                                          const void* s_in_pool, const void* s_rank_pool, const void* s_out_pool,
                                          const int32_t* adapter_of_row, const void* y_base, void* y_out,
                                          int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t n_adapters,
                                          void* stream, int algo);

/* DEVICE function: lordba_forward_batched for a pool whose adapters have `ell` scale envelopes each over their own
 * carriers (Def. 1 / Eq. (lordba) with envelope rank l = ell per adapter; Sec. 3.3: such adapters are hot-swapped and served
 * concurrently like any other):
 *   y_out[t] = y_base[t] + sum_{e < ell} (branch of envelope e of adapter adapter_of_row[t]) applied to x[t]
 *   s_in_pool: fp16 [n_adapters, ell, d_in]    s_rank_pool: fp16 [n_adapters, ell, r]    s_out_pool: fp16 [n_adapters, ell, d_out]
 * 1 <= ell <= LORDBA_MAX_ENVELOPES (else LORDBA_ERR_DIM); ell == 1 is lordba_forward_batched.  Everything else (the packed
 * pools, the index array, pass-through rows, arithmetic as lordba_forward_multi, error bound, aliasing, stream semantics:
 * enqueue only, no allocation, no workspace) as lordba_forward_batched. */
lordba_status lordba_forward_batched_multi(const void* x, const uint32_t* packedA_pool, const uint32_t* packedB_pool,
                                           const void* s_in_pool, const void* s_rank_pool, const void* s_out_pool,
                                           const int32_t* adapter_of_row, const void* y_base, void* y_out,
                                           int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t ell, int64_t n_adapters,
                                           void* stream);

/* Same with the kernel chosen by the caller: LORDBA_ALGO_AUTO, LORDBA_ALGO_GENERAL or LORDBA_ALGO_MFMA_T8. */
lordba_status lordba_forward_batched_multi_algo(const void* x, const uint32_t* packedA_pool, const uint32_t* packedB_pool,
                                                const void* s_in_pool, const void* s_rank_pool, const void* s_out_pool,
                                                const int32_t* adapter_of_row, const void* y_base, void* y_out,
                                                int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t ell,
                                                int64_t n_adapters, void* stream, int algo);

/* DEVICE function: binarises and packs the latent carriers on the device, as every training step does before its
 * forward pass (B1 = sign(U1), B2 = sign(U2), Sec. 3.2; Alg. QAT-LoRDBA), sign(0) = +1 (Sec. 2, Notation; -0.0 counts as
 * zero).  latentA fp32 [r, d_in], latentB fp32 [d_out, r] (device memory).  Outputs, each in the canonical packed format
 * and each optional (NULL = not wanted): packedA = S_A as [r, d_in], packedB = S_B as [d_out, r] (what lordba_forward
 * takes), packedAt = S_A^T as [d_in, r], packedBt = S_B^T as [r, d_out] (what lordba_backward takes besides packedA).
 * Bit-identical to lordba_pack_signs_f32 applied to the latents and to their transposes, except that a NaN, which the
 * host function rejects, packs as +1 here (an enqueue-only call has no way to report it).  Enqueues one kernel on
 * `stream`; never synchronises, allocates or frees. */
lordba_status lordba_pack_latents(const float* latentA, const float* latentB,
                                  uint32_t* packedA, uint32_t* packedB, uint32_t* packedAt, uint32_t* packedBt,
                                  int64_t d_in, int64_t d_out, int64_t r, void* stream);

/* DEVICE function: the forward branch as training runs it (Sec. 3.2): lordba_forward, which also keeps the rank-r
 * intermediate of Eq. (lordba-fwd) for the backward pass,
 *   t_out[k * t_stride + t] = sum_i S_A[k, i] * s_in[i] * x[t, i]        fp32, rank-major, k < r, t < T, t_stride >= T
 * (the value before the rank scaling; other entries of t_out are left untouched).  T * r * 4 bytes instead of recomputing
 * a pass over x.  y_base == NULL and y_out == NULL together: only t_out is computed (x is read once, nothing else).
 * Everything else as lordba_forward (T == 0: no work, t_out may then be NULL too); t_out must not overlap x, y_base or
 * y_out (LORDBA_ERR_ALIAS). */
lordba_status lordba_forward_save_t(const void* x, const uint32_t* packedA, const uint32_t* packedB,
                                    const void* s_in, const void* s_rank, const void* s_out,
                                    const void* y_base, void* y_out, float* t_out, int64_t t_stride,
                                    int64_t T, int64_t d_in, int64_t d_out, int64_t r, void* stream);

/* DEVICE function: lordba_forward_save_t for an adapter with `ell` envelopes (the forward of lordba_forward_multi):
 *   t_out[(e * r + k) * t_stride + t] = sum_i S_A[k, i] * s_in[e, i] * x[t, i]      fp32, one [r, t_stride] block per envelope
 * y_base == NULL and y_out == NULL together: only t_out.  Runs the 8-row, 8-wave variant of the kernel (the only one
 * with a training instantiation for ell >= 2), so y_out may differ from lordba_forward_multi's in the last bit. */
lordba_status lordba_forward_multi_save_t(const void* x, const uint32_t* packedA, const uint32_t* packedB,
                                          const void* s_in, const void* s_rank, const void* s_out,
                                          const void* y_base, void* y_out, float* t_out, int64_t t_stride,
                                          int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t ell, void* stream);

/* DEVICE function: the backward pass of the branch in training (Sec. 3.2, "Forward and backward pass"; Alg. QAT-LoRDBA;
 * smooth-sign straight-through factor of Eq. (smoothsign)).  For Y = Y_base + X diag(s_in) S_A^T diag(s_rank) S_B^T diag(s_out)
 * with S_A = sign(latentA), S_B = sign(latentB), and an upstream gradient g = dL/dY, it computes
 *   dx        = dx_base + g DeltaW^T                                  fp16 [T, d_in]   (one rounding, as lordba_forward)
 *   d_s_in, d_s_rank, d_s_out                                        fp32 [d_in], [r], [d_out]
 *   d_latentA = dL/dS_A * kappa (1 - tanh^2(kappa latentA))           fp32 [r, d_in]
 *   d_latentB = dL/dS_B * kappa (1 - tanh^2(kappa latentB))           fp32 [d_out, r]
 * Inputs (device memory, row-major, contiguous, caller-owned):
 *   x fp16 [T, d_in]; g fp16 [T, d_out]; s_in, s_rank, s_out fp16: the values the forward pass used (the optimiser's fp32
 *   master copies are the caller's; Sec. 3.2 trains the scales in fp32); latentA fp32 [r, d_in], latentB fp32 [d_out, r];
 *   kappa: the temperature of Eq. (smoothsign) (100 by default in the paper);
 *   packedA : S_A   as [r, d_in]    (the forward pass's packedA)
 *   packedAt: S_A^T as [d_in, r]    packedBt: S_B^T as [r, d_out]     (the same canonical format, transposed matrices;
 *             the carriers are taken from these bits, which the caller keeps equal to the signs of the latents)
 *   t_saved : the rank-r intermediate that lordba_forward_save_t wrote for this x and adapter, with its t_stride >= T
 *             (entries past T are ignored); or NULL: it is recomputed from x (one more pass over x).  The matrix-core
 *             kernels take it only with a t_stride that is a multiple of 4 and at least T rounded up to a multiple of
 *             128 (they read the rows in whole steps), 16-byte aligned.
 *   d_latentA == NULL and d_latentB == NULL together: the carriers are frozen and only the scales are trained (the
 *   "QAT Freeze" mode of Sec. 3.2): no latent gradients are computed; latentA, latentB and kappa are then ignored.
 *   dx_base fp16 [T, d_in]: the input gradient of the base path, to which the branch's is added; dx may be the same
 *   pointer.  dx == NULL and dx_base == NULL together: the input gradient is not computed.
 *   workspace: at least lordba_backward_workspace_bytes(T, d_in, d_out, r) bytes of device memory, 16-byte aligned, owned
 *   by the caller, contents irrelevant before and after; a smaller one -> LORDBA_ERR_WORKSPACE.  Calls that share a
 *   workspace must not overlap in time.
 * No output, nor the workspace, may overlap an input or another output (dx == dx_base excepted): LORDBA_ERR_ALIAS.
 * Shapes: any d_in, d_out >= 1 and 1 <= r <= 64, every pointer aligned to its element (the workspace to 16 bytes), as
 * lordba_forward and lordba_forward_save_t; else LORDBA_ERR_DIM / LORDBA_ERR_ALIGN.  With d_in and d_out multiples of 32
 * and 16-byte aligned activations, scales and packed carriers the matrix-core kernels run; anything else takes a slower
 * general kernel with the same results (one thread per column).  T == 0: the parameter gradients are set to zero.
 * The call only enqueues kernels on `stream`; it never synchronises, allocates or frees.  Results are deterministic
 * (fixed summation order).  Arithmetic: fp16 inputs at their exact values, fp32 accumulation; every gradient array is
 * within 1e-3 relative L2 (per token row for dx, per rank for the latents, whole vector for the scales) of the exact result. */
lordba_status lordba_backward(const void* x, const void* g,
                              const uint32_t* packedA, const uint32_t* packedAt, const uint32_t* packedBt,
                              const void* s_in, const void* s_rank, const void* s_out,
                              const float* latentA, const float* latentB, float kappa,
                              const float* t_saved, int64_t t_stride,
                              const void* dx_base, void* dx,
                              float* d_s_in, float* d_s_rank, float* d_s_out,
                              float* d_latentA, float* d_latentB,
                              void* workspace, size_t workspace_bytes,
                              int64_t T, int64_t d_in, int64_t d_out, int64_t r, void* stream);

/* DEVICE function: lordba_backward for an adapter with `ell` scale envelopes over the same carriers (Def. 1 / Eq. (lordba),
 * l = ell; the forward of lordba_forward_multi).  s_in fp16 [ell, d_in], s_rank fp16 [ell, r], s_out fp16 [ell, d_out];
 * d_s_in fp32 [ell, d_in], d_s_rank fp32 [ell, r], d_s_out fp32 [ell, d_out]: every envelope has its own scale
 * gradients; dx and the latent gradients are the sums over the envelopes (dx with one rounding).  1 <= ell <=
 * LORDBA_MAX_ENVELOPES.  t_saved: what lordba_forward_multi_save_t wrote ([ell, r, t_stride]), or NULL (recomputed: one
 * more pass over x).  Workspace: lordba_backward_workspace_bytes is enough whatever ell is (the activations are then
 * contracted once per envelope); with lordba_backward_multi_workspace_bytes(..., ell) bytes, and at most four rank blocks of
 * 16 in all envelopes together (ell * ceil(r / 16) <= 4), one pass over x and g serves every envelope (the carriers are
 * shared, only the rank-r operand differs; same results up to the order of fp32 sums).  Everything else as lordba_backward. */
lordba_status lordba_backward_multi(const void* x, const void* g,
                                    const uint32_t* packedA, const uint32_t* packedAt, const uint32_t* packedBt,
                                    const void* s_in, const void* s_rank, const void* s_out,
                                    const float* latentA, const float* latentB, float kappa,
                                    const float* t_saved, int64_t t_stride,
                                    const void* dx_base, void* dx,
                                    float* d_s_in, float* d_s_rank, float* d_s_out,
                                    float* d_latentA, float* d_latentB,
                                    void* workspace, size_t workspace_bytes,
                                    int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t ell, void* stream);

/* Bytes of workspace lordba_backward needs for a shape (0 for sizes outside its range: T < 0, a width below 1 or above
 * 2^24, r outside 1..64). */
size_t lordba_backward_workspace_bytes(int64_t T, int64_t d_in, int64_t d_out, int64_t r);

/* Bytes of workspace with which lordba_backward_multi reads x and g once for all `ell` envelopes (never less than
 * lordba_backward_workspace_bytes; equal to it where the one-pass form does not apply; 0 for sizes out of range). */
size_t lordba_backward_multi_workspace_bytes(int64_t T, int64_t d_in, int64_t d_out, int64_t r, int64_t ell);

/* Size of the library-owned scratch array behind lordba_backward_noalloc (one per GPU the library runs on, held until the
 * process ends). */
#define LORDBA_BACKWARD_NOALLOC_MAX_BYTES (16 * 1024 * 1024)

/* DEVICE function for callers that cannot allocate device memory or hand over a workspace: code under HIP graph capture,
 * tight serving or training loops, harnesses that forbid allocation.  It is lordba_backward (same arguments, kernels,
 * results bit for bit, error codes) without the workspace arguments: the scratch lives in a device array of
 * LORDBA_BACKWARD_NOALLOC_MAX_BYTES bytes that is part of the library's code object, and the call allocates and frees
 * nothing (its first call on a device only looks up that device's address of the array; make that call outside a graph
 * capture).  A shape with lordba_backward_workspace_bytes(T, d_in, d_out, r) > LORDBA_BACKWARD_NOALLOC_MAX_BYTES ->
 * LORDBA_ERR_WORKSPACE, nothing is enqueued (every shape of the paper's models at r = 16 and T <= 8192 fits; so does
 * d = 4096, r = 64, T = 2048).  All calls on one GPU share that GPU's array: calls that may overlap in time (different
 * streams, or graphs replayed side by side) race on it and must be ordered by the caller.  The array's contents after a
 * call are unspecified; nothing in it needs clearing between calls. */
lordba_status lordba_backward_noalloc(const void* x, const void* g,
                                      const uint32_t* packedA, const uint32_t* packedAt, const uint32_t* packedBt,
                                      const void* s_in, const void* s_rank, const void* s_out,
                                      const float* latentA, const float* latentB, float kappa,
                                      const float* t_saved, int64_t t_stride,
                                      const void* dx_base, void* dx,
                                      float* d_s_in, float* d_s_rank, float* d_s_out,
                                      float* d_latentA, float* d_latentB,
                                      int64_t T, int64_t d_in, int64_t d_out, int64_t r, void* stream);

/* ---- post-training quantisation of a low-rank update into a LoRDBA adapter ---------------------------------------- */

#define LORDBA_PTQ_MAX_RANK 32         /* carrier rank R of lordba_ptq                    */
#define LORDBA_PTQ_MAX_FACTOR_RANK 64  /* rank r0 of the factors of the update            */
#define LORDBA_PTQ_MAX_SWEEPS 4096     /* outer iterations K                              */

/* DEVICE function: PTQ-LoRDBA at envelope rank 1 (appendix on post-training quantisation: the least-squares problem
 * Eq. (ptq-problem); the consensus ADMM Eq. (admm-problem) with the ordered updates Eq. (u-step-1), Eq. (u-step-2),
 * Eq. (scales-step), Eq. (m-y-step); the closed-form scale updates Eq. (alpha-update), Eq. (gamma-update),
 * Eq. (beta-gram), Eq. (beta-pinv); the warm start Eq. (svd-init); Alg. PTQ-LoRDBA).  Fits
 *     diag(alpha) B1 diag(beta) B2 diag(gamma)  ~  Delta W* = A_star B_star^T     (N x M, in the Frobenius norm)
 * with B1 in {+-1}^{N x R}, B2 in {+-1}^{R x M}, and returns the adapter in the form lordba_forward takes, with
 * d_in = N, d_out = M, r = R.  All pointers are DEVICE pointers; the call only enqueues kernels on `stream` and never
 * waits for the device.
 *   A_star, B_star : fp16 [N, r0], [M, r0] row-major, in; taken at their exact values.  They need not have full column
 *          rank (dead or repeated columns, fewer rows than columns are fine), but the update must have rank >= R.
 *   packedA : uint32 [lordba_packed_words(R, N)] out, S_A = B1^T in the canonical format;  packedB : uint32
 *             [lordba_packed_words(M, R)] out, S_B = B2^T.
 *   alpha [N], beta [R], gamma [M] : fp64 out, the scales (s_in, s_rank, s_out of the forward).
 *   s_in [N], s_rank [R], s_out [M] : fp16 out, the same scales rounded to nearest; each may be NULL.
 *   info : fp64 [8 + K] out: [0] sweeps run, [1] 1 if the loop ended because the sign matrices repeated, [2] the penalty
 *          rho it ended with, [3] ||Delta W*||_F^2, [4] 1 if the input was degenerate (an update of rank below R,
 *          zero or non-finite: no sweep is run and the other outputs are unspecified), [5..7] 0,
 *          [8 + t] the objective of Eq. (admm-problem) at the continuous iterates after the scale update of sweep t
 *          (0 for sweeps not run).
 *   workspace : lordba_ptq_workspace_bytes(N, M, R, r0) bytes, 8-byte aligned, owned by the caller; a smaller one ->
 *          LORDBA_ERR_WORKSPACE.  After the call it begins with the last continuous iterates, fp64: U1 [N, R] row-major at
 *          offset 0, then U2^T [M, R] row-major at the next multiple of 32 doubles (they are what a later quantisation-
 *          aware training run would take as latent carriers); the rest is scratch.
 *   K : outer iterations (the paper uses 100); tau > 1 and mu > 0: the residual-balancing constants (the paper uses 2, 10),
 *          anything else -> LORDBA_ERR_VALUE.
 * Readings where the paper leaves a choice: sign(0) = +1; the warm start keeps beta at the singular values, starts from
 * gamma = 1 and updates alpha, then gamma; a scale sweep updates alpha, gamma, beta in this order at the continuous
 * iterates; residual balancing compares r = sqrt(sum_k ||U_k - M_k||_F^2) with s = sqrt(sum_k (rho_k ||M_k^(t+1) -
 * M_k^(t)||_F)^2), rho_k = rho / n_k, after the sweeps t < K/2 (r > mu s: rho *= tau, Y /= tau; s > mu r: the opposite);
 * the loop ends after the first sweep that leaves both sign matrices unchanged.  Each pair (column k of B1, row k of B2)
 * is defined up to a common sign (the singular vectors of the warm start are).
 * Limits: 1 <= R <= LORDBA_PTQ_MAX_RANK, R <= r0 <= LORDBA_PTQ_MAX_FACTOR_RANK (beyond r0 the warm start has no singular
 * vectors), 1 <= N, M <= 2^22, 1 <= K <= LORDBA_PTQ_MAX_SWEEPS; else LORDBA_ERR_DIM.  No output, nor the workspace,
 * may overlap an input or another output: LORDBA_ERR_ALIAS.  Arithmetic: fp64 throughout, fixed summation order
 * (calls are reproducible bit for bit).  The warm start (Eq. (svd-init)) takes the singular triplets of the update from
 * the triangular factors of Householder QR factorisations of A_star and B_star: triplet k carries a relative error of
 * about eps sigma_1 / sigma_k, as a dense singular value decomposition's would; an update whose R-th singular value is
 * below 1e-12 of its largest counts as rank deficient (info[4]). */
lordba_status lordba_ptq(const void* A_star, const void* B_star, uint32_t* packedA, uint32_t* packedB,
                         double* alpha, double* beta, double* gamma, void* s_in, void* s_rank, void* s_out,
                         double* info, void* workspace, size_t workspace_bytes,
                         int64_t N, int64_t M, int64_t R, int64_t r0, int64_t K, double tau, double mu, void* stream);

/* DEVICE function: lordba_ptq enqueued in pieces.  Enqueues the sweeps t_begin <= t < t_end of a run of K sweeps (the
 * schedule of the penalty depends on K, not on the piece) and then the export; t_begin == 0 also enqueues the warm
 * start.  A call with t_begin > 0 continues the run whose state the workspace and the output arrays hold: it takes the
 * same arguments as the call before it (same pointers, shapes, K, tau, mu) and t_begin equal to that call's t_end, and
 * nothing else may have written to them in between.  After every piece the outputs describe the run so far (info[0]
 * sweeps, info[1] the end flag, ...), so a caller that is willing to wait can enqueue the typical number of sweeps,
 * look at info[1], and enqueue the rest only if the loop has not ended: the result is bit for bit that of lordba_ptq
 * (which is this function with t_begin = 0, t_end = K), without the launches that would return at once.
 * 0 <= t_begin <= t_end <= K, else LORDBA_ERR_DIM; everything else as lordba_ptq. */
lordba_status lordba_ptq_sweeps(const void* A_star, const void* B_star, uint32_t* packedA, uint32_t* packedB,
                                double* alpha, double* beta, double* gamma, void* s_in, void* s_rank, void* s_out,
                                double* info, void* workspace, size_t workspace_bytes,
                                int64_t N, int64_t M, int64_t R, int64_t r0, int64_t K, int64_t t_begin, int64_t t_end,
                                double tau, double mu, void* stream);

/* Bytes of workspace lordba_ptq needs for a shape (0 for a shape it does not support). */
size_t lordba_ptq_workspace_bytes(int64_t N, int64_t M, int64_t R, int64_t r0);

/* DEVICE function: the closed-form update of the rank scales on its own (Eq. (beta-gram), Eq. (beta-pinv)): beta = pinv(G) h
 * for a symmetric positive semidefinite G, the minimum-norm least-squares solution when G is singular (two carrier
 * columns that coincide, a zero scale vector).  It is the routine a sweep of lordba_ptq runs after it has formed
 * G = (P^T P) o (Q Q^T) and h; exported so that it can be used, and checked, by itself.
 *   G : fp64 [R, R] row-major, in (only its symmetric content matters: both triangles are read);  h : fp64 [R], in;
 *   beta : fp64 [R], out.  Device pointers, 8-byte aligned; beta may not overlap G or h (LORDBA_ERR_ALIAS).
 * 1 <= R <= LORDBA_PTQ_MAX_RANK, else LORDBA_ERR_DIM.  One small kernel on `stream`; never waits, allocates or frees.
 * Rank decision: a pivot of the diagonally pivoted Cholesky factorisation that does not exceed 64 eps max_k G_kk ends
 * the factorisation; G = 0 gives beta = 0. */
lordba_status lordba_ptq_beta_solve(const double* G, const double* h, double* beta, int64_t R, void* stream);

/* Static, never-NULL description of a status code. */
const char* lordba_status_string(lordba_status status);

#ifdef __cplusplus
}
#endif
#endif /* LORDBA_H */
