/*
 * monarch.h -- C ABI of the MI355X (gfx950) Monarch multiply library.
 *
 * The library applies a Monarch matrix  M = P L P^T R  (Dao et al., "Monarch:
 * Expressive Structured Matrices for Efficient and Accurate Training",
 * Definition 3.1) to a batch of row vectors, forward and backward.  R and L are
 * block-diagonal, P is the "reshape as a grid, transpose, flatten" permutation.
 * The rectangular / larger-block form used for Transformer layers (Section 3.1,
 * "Extension to Rectangular Matrices") is covered by the same calls: both
 * factors have k blocks, R's blocks are q x p and L's blocks are s x q.
 *
 * Operation (Section 3.3, "Steps to multiply x by a Monarch matrix", steps 1-3),
 * for every row b of the batch, 0-based indices, p = n_in / k:
 *
 *   step 1   Y1[b][kk][j] = sum_{i<p} R[kk][j][i] * x[b][kk*p + i]        kk<k, j<q
 *   P^T      U[b][c*q + r] = Y1[b][f mod k][f div k],  f = c*q + r        c<k,  r<q
 *   step 2   W[b][c][l]   = sum_{r<q} L[c][l][r] * U[b][c*q + r]          l<s
 *   step 3   y[b][l*k + c] = W[b][c][l]
 *
 * In the square case n = m^2, k = p = q = s = m this is literally
 * z[l][j] = sum_k L[j][l][k] * (sum_i R[k][j][i] x[k][i]),  y[l*m + j] = z[l][j],
 * i.e. Equation (1): M[l*m + j][k*m + i] = L[j][l][k] * R[k][j][i].
 *
 * The paper defines P only for the square case.  For k != q the default above
 * takes the (k, q) grid of stage-1 outputs, transposes it to (q, k), flattens,
 * and cuts the result into k chunks of length q.  MONARCH_FLAG_PERM_B selects
 * the inverse permutation instead:  U[b][c*q + r] = Y1flat[b][r*k + c].
 * The two agree whenever k == q.
 *
 * Layout: every tensor is dense, row-major, last index fastest.
 *   x, dx  (batch, n_in)        R, dR  (k, q, n_in/k)
 *   y, dy  (batch, k*s)         L, dL  (k, s, q)
 * Element type is `dtype` for all of them: MONARCH_F32 = IEEE binary32,
 * MONARCH_BF16 = the upper 16 bits of a binary32 stored as uint16_t.  Products
 * are accumulated in fp32; in the bf16 path the on-chip intermediate between
 * the two stages is rounded to bf16 (nearest even) and each output is rounded
 * once on store.  With MONARCH_FLAG_WGRAD_F32, dR and dL are written as fp32
 * regardless of dtype.
 *
 * Ownership: all pointers are DEVICE pointers owned by the caller, 16-byte
 * aligned, valid until `stream` has passed the call.  Outputs must not alias
 * inputs.  The library keeps no state, allocates nothing and frees nothing;
 * scratch memory is the caller's `workspace` (monarch_bwd, monarch_fwd_ws).  All work is
 * enqueued on `stream` (a hipStream_t passed as void*, NULL = the default
 * stream) and the calls return without synchronising.
 *
 * Errors: every call returns MONARCH_OK (0) or a negative status.  Arguments
 * are validated on the host before anything is launched, so the error paths
 * need no GPU.  batch == 0 is a successful no-op (monarch_bwd then still
 * zero-fills dR and dL); the per-row pointers x, y, dy, dx may then be NULL.
 * Nothing is printed and nothing aborts.
 */
#ifndef MONARCH_H_
#define MONARCH_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { MONARCH_F32 = 0, MONARCH_BF16 = 1 } monarch_dtype;

enum {
    MONARCH_OK = 0,
    MONARCH_ERR_INVALID = -1,     /* null pointer, non-positive size, n_in % k != 0, bad dtype/flags */
    MONARCH_ERR_UNSUPPORTED = -2, /* shape too large for any kernel of this build */
    MONARCH_ERR_WORKSPACE = -3,   /* workspace missing, misaligned or too small */
    MONARCH_ERR_HIP = -4          /* the HIP runtime refused a launch */
};

#define MONARCH_FLAG_WGRAD_F32 1u /* monarch_bwd: dR, dL are float even when dtype is bf16 */
#define MONARCH_FLAG_PERM_B    2u /* use the inverse mid permutation (see above) */
#define MONARCH_FLAG_GENERIC   4u /* force the shape-generic kernels (testing aid) */
#define MONARCH_FLAG_WS_PACKED 8u /* monarch_fwd_ws: the workspace already holds the packed copies of these
                                     R and L, left there by an earlier monarch_fwd_ws call for the same
                                     shape without this flag; the pack pass is skipped (weights that stay
                                     fixed over many calls: inference, several micro-batches per update) */

/* Forward: y = x M^T  (Section 3.3 steps 1-3; one fused pass, the intermediate
 * Y1/U never leaves the chip).  x (batch, n_in), R (k, q, n_in/k), L (k, s, q),
 * y (batch, k*s); all device pointers. */
int monarch_fwd(const void* x, const void* R, const void* L, void* y,
                int64_t batch, int n_in, int k, int q, int s,
                monarch_dtype dtype, void* stream);

/* Same as monarch_fwd with `flags` (MONARCH_FLAG_PERM_B, MONARCH_FLAG_GENERIC). */
int monarch_fwd_ex(const void* x, const void* R, const void* L, void* y,
                   int64_t batch, int n_in, int k, int q, int s,
                   monarch_dtype dtype, void* stream, unsigned flags);

/* Forward with scratch memory (same operation, same arguments and result as monarch_fwd_ex;
 * Section 3.3 steps 1-3).  For the shapes that have a packed-weight kernel (bf16: k = 4 wide
 * blocks, and the square m = 64 case) the call first re-lays R and L in matrix-core fragment order into `workspace` and then
 * runs the fused forward on the packed copies, which removes the weights from the LDS traffic of
 * the kernel.  fp32 layers with square blocks p = q = s of 32 or 64 (any k) run on the fp32 matrix cores, one
 * launch per block-diagonal factor with the vector between the factors kept in `workspace` (the packed flag
 * means nothing to them and is ignored).  Every other shape runs exactly as monarch_fwd_ex and ignores the
 * workspace.
 * `workspace` (device memory, 256-byte aligned, caller-owned) must hold at least
 * monarch_fwd_workspace_bytes(...) bytes when that is non-zero.  Without MONARCH_FLAG_WS_PACKED its
 * contents on entry are ignored; on exit it holds the packed copies of R and L, and a later call with
 * MONARCH_FLAG_WS_PACKED, the same shape and unchanged R and L may reuse them (R and L must still be
 * valid pointers but are not read).  Returns MONARCH_ERR_WORKSPACE if the workspace is missing, misaligned or too small. */
int monarch_fwd_ws(const void* x, const void* R, const void* L, void* y,
                   int64_t batch, int n_in, int k, int q, int s,
                   monarch_dtype dtype, void* stream,
                   void* workspace, size_t workspace_bytes, unsigned flags);

/* monarch_fwd_ws for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * operation, arguments, kernels and result as monarch_fwd_ws (bit for bit), but the scratch
 * memory is an array inside the library that exists from program load: MONARCH_STATIC_WORKSPACE_BYTES
 * bytes per GPU, held by every GPU the library runs on until the process ends.  The call
 * allocates and frees nothing.  Shapes whose monarch_fwd_workspace_bytes(...) exceeds that limit
 * return MONARCH_ERR_WORKSPACE (every shape with a packed-weight kernel in this build fits);
 * MONARCH_FLAG_WS_PACKED is refused with MONARCH_ERR_INVALID, because the array belongs to no
 * caller between calls.  All calls on one GPU share the array and overwrite it: two calls that may
 * overlap in time on one GPU (different streams, different threads) race and must be serialised by
 * the caller; calls on one stream are ordered and safe.  The first call on a device looks up the
 * array's device address (no allocation; make that call outside graph capture). */
#define MONARCH_STATIC_WORKSPACE_BYTES (8u << 20)
int monarch_fwd_static(const void* x, const void* R, const void* L, void* y,
                       int64_t batch, int n_in, int k, int q, int s,
                       monarch_dtype dtype, void* stream, unsigned flags);

/* Forward of the affine layer built on the Monarch matrix:  y[b][o] = (x M^T)[b][o] + bias[o].
 * Section 4 swaps a layer's dense weight matrix for a Monarch one and keeps the rest of the layer;
 * the appendix on BERT pretraining lists the bias add as a step to fuse into the matrix product.
 * Arguments as monarch_fwd_ws (same workspace, same flags); `bias` (k*s elements of `dtype`, device
 * pointer, 16-byte aligned) may be NULL, and the call is then monarch_fwd_ws itself.  The bias is
 * added to the fp32 accumulator before the single rounding to `dtype` in the kernels that have a
 * bias epilogue (bf16 k = 4 wide blocks, fp32 m = 16, the shape-generic kernels); the bf16 m = 64
 * kernel has none, there a second in-place pass adds the bias to the rounded y (two roundings). */
int monarch_fwd_bias(const void* x, const void* R, const void* L, const void* bias, void* y,
                     int64_t batch, int n_in, int k, int q, int s,
                     monarch_dtype dtype, void* stream,
                     void* workspace, size_t workspace_bytes, unsigned flags);

/* Bytes of device scratch monarch_fwd_ws needs for this problem (0 when the shape has no
 * packed-weight kernel, and on invalid arguments). */
size_t monarch_fwd_workspace_bytes(int64_t batch, int n_in, int k, int q, int s,
                                   monarch_dtype dtype, unsigned flags);

/* Backward: the adjoint of steps 3, 2, P^T, 1 in that order (the paper obtains it
 * by automatic differentiation, Section 4):
 *   dW[b][c][l]  = dy[b][l*k + c]
 *   dL[c][l][r]  = sum_b dW[b][c][l] * U[b][c*q + r]
 *   dU[b][c*q+r] = sum_l L[c][l][r] * dW[b][c][l]
 *   dY1          = inverse mid permutation of dU
 *   dR[kk][j][i] = sum_b dY1[b][kk][j] * x[b][kk*p + i]
 *   dx[b][kk*p+i]= sum_j R[kk][j][i] * dY1[b][kk][j]
 * U is recomputed from x (no activation is saved by the forward call).  dx, dR
 * and dL are overwritten, never accumulated into.  The matrix-core kernels sum
 * per-chunk partial gradients in a fixed order (bit-reproducible); the
 * shape-generic fallback reduces dR/dL with fp32 atomics across workgroups, so
 * its results are reproducible only up to fp32 summation order.  `workspace` must hold at least
 * monarch_bwd_workspace_bytes(...) bytes (device memory, 256-byte aligned);
 * its contents on entry are ignored and on exit are unspecified. */
int monarch_bwd(const void* dy, const void* x, const void* R, const void* L,
                void* dx, void* dR, void* dL,
                int64_t batch, int n_in, int k, int q, int s,
                monarch_dtype dtype, void* stream,
                void* workspace, size_t workspace_bytes, unsigned flags);

/* Backward of the affine layer: monarch_bwd plus the bias gradient
 *   dbias[o] = sum_b dy[b][o]
 * (the same appendix lists it as fused with the backward product).  `dbias` holds k*s elements, of
 * `dtype`, or float with MONARCH_FLAG_WGRAD_F32; it is overwritten (zeros when batch == 0); NULL
 * skips it, and the call is then monarch_bwd itself.  The sum runs in fp32 over fixed row chunks in
 * a fixed order (bit-reproducible), as its own pass over dy ahead of the other kernels.  Same
 * workspace as monarch_bwd. */
int monarch_bwd_bias(const void* dy, const void* x, const void* R, const void* L,
                     void* dx, void* dR, void* dL, void* dbias,
                     int64_t batch, int n_in, int k, int q, int s,
                     monarch_dtype dtype, void* stream,
                     void* workspace, size_t workspace_bytes, unsigned flags);

/* The two layers of a feed-forward block with the nonlinearity between them applied inside the layers'
 * own kernels, so that the block's hidden activation is not read and re-written by separate elementwise
 * passes.  Section 4 replaces the dense weight matrices of the feed-forward blocks of ViT, MLP-Mixer,
 * BERT and GPT-2 by Monarch matrices and leaves the blocks otherwise unchanged; the paper does not
 * write the blocks' nonlinearity down (it names kernel fusion as a further speed-up it expects, at
 * the end of Section 5.2).  All four models use GELU; taken here in its tanh form (GPT-2's),
 *     gelu(v) = v/2 * (1 + tanh( sqrt(2/pi) * (v + 0.044715 v^3) )).
 *
 * monarch_fwd_bias_gelu (the block's first layer):
 *     y_pre[b][o] = (x M^T)[b][o] + bias[o],    y[b][o] = gelu(y_pre[b][o]).
 * Arguments as monarch_fwd_bias.  `bias` may be NULL (no bias).  `y_pre` (batch x k*s elements of
 * `dtype`, 16-byte aligned) receives the value before the nonlinearity, which the backward pass
 * needs; NULL skips it (inference).  In the kernels with the fused epilogue (bf16, k = 4 wide blocks,
 * with workspace) gelu is applied to the fp32 sum before its rounding to `dtype`; for every other
 * shape y_pre is rounded to `dtype` first and a second pass computes y from it.
 *
 * monarch_bwd_bias_gelu_in (the block's second layer, whose input is x = gelu(x_pre)):
 *     dx_pre[b][i] = (dy M)[b][i] * gelu'(x_pre[b][i]),
 * dR, dL, dbias exactly as monarch_bwd_bias for the input x.  `x` is what the first layer wrote as y,
 * `x_pre` what it wrote as y_pre (same shape as x; 16-byte aligned; required).  dx_pre is then the
 * upstream gradient dy of the first layer's monarch_bwd_bias.  Fused into the dx epilogue of the
 * bf16 k = 4 backward; a second pass over dx elsewhere.  Workspace and errors as monarch_bwd_bias. */
int monarch_fwd_bias_gelu(const void* x, const void* R, const void* L, const void* bias,
                          void* y_pre, void* y,
                          int64_t batch, int n_in, int k, int q, int s,
                          monarch_dtype dtype, void* stream,
                          void* workspace, size_t workspace_bytes, unsigned flags);
int monarch_bwd_bias_gelu_in(const void* dy, const void* x, const void* x_pre,
                             const void* R, const void* L,
                             void* dx_pre, void* dR, void* dL, void* dbias,
                             int64_t batch, int n_in, int k, int q, int s,
                             monarch_dtype dtype, void* stream,
                             void* workspace, size_t workspace_bytes, unsigned flags);

/* Forward and backward that share the vector between the two factors instead of recomputing it (the
 * paper differentiates the multiply automatically, Section 4, which keeps the intermediate of step 1
 * for the backward pass; monarch_bwd recomputes it from x).  monarch_fwd_save is monarch_fwd_ex that
 * also writes that vector into `saved` (monarch_saved_bytes(...) bytes, device memory, 16-byte
 * aligned, caller-owned, contents opaque); monarch_bwd_saved is monarch_bwd_bias that reads it from
 * there and skips the recompute.  x is still needed (dR).  `saved` must come from monarch_fwd_save
 * with the same x, R, L, shape and flags.  For shapes whose kernels have no such path
 * monarch_saved_bytes returns 0, `saved` may be NULL and the two calls are monarch_fwd_ex and
 * monarch_bwd_bias exactly; a NULL `saved` in monarch_bwd_saved always means "recompute".
 * Errors as the calls they extend; a missing, misaligned or short `saved` buffer is
 * MONARCH_ERR_WORKSPACE. */
size_t monarch_saved_bytes(int64_t batch, int n_in, int k, int q, int s,
                           monarch_dtype dtype, unsigned flags);
int monarch_fwd_save(const void* x, const void* R, const void* L, void* y,
                     void* saved, size_t saved_bytes,
                     int64_t batch, int n_in, int k, int q, int s,
                     monarch_dtype dtype, void* stream, unsigned flags);
int monarch_bwd_saved(const void* dy, const void* x, const void* saved, size_t saved_bytes,
                      const void* R, const void* L,
                      void* dx, void* dR, void* dL, void* dbias,
                      int64_t batch, int n_in, int k, int q, int s,
                      monarch_dtype dtype, void* stream,
                      void* workspace, size_t workspace_bytes, unsigned flags);

/* Bytes of device scratch monarch_bwd and monarch_bwd_bias need for this problem (never 0 for a
 * valid problem; 0 on invalid arguments). */
size_t monarch_bwd_workspace_bytes(int64_t batch, int n_in, int k, int q, int s,
                                   monarch_dtype dtype, unsigned flags);

/* Transposed multiply:  y = x M,  i.e. the transpose M^T = R^T P L^T P^T applied to every row (for
 * real factors the M* of Section 3.1, "Products of Monarch Matrices": a matrix of the class MM* is
 * applied as monarch_fwd_t with the factors of M2 followed by monarch_fwd with the factors of M1).
 * Steps, for every row b:
 *   W[b][c][l]     = x[b][l*k + c]
 *   U[b][c*q + r]  = sum_l L[c][l][r] * W[b][c][l]
 *   Y1[b][kk][j]   = U[b][position that the mid permutation gives stage-1 output (kk, j)]
 *   y[b][kk*p + i] = sum_j R[kk][j][i] * Y1[b][kk][j]
 * the same arithmetic as the dx part of monarch_bwd.  x (batch, k*s), y (batch, n_in), R and L as
 * everywhere; flags: MONARCH_FLAG_PERM_B, MONARCH_FLAG_GENERIC.  `workspace` (device, 256-byte
 * aligned) must hold monarch_fwd_t_workspace_bytes(...) bytes when that is non-zero (weights in
 * matrix-core operand order; for m = 64 also one re-laid copy of x); contents on entry are ignored.
 * In the bf16 path the vector between the two factors is rounded to bf16, as in monarch_fwd. */
int monarch_fwd_t(const void* x, const void* R, const void* L, void* y,
                  int64_t batch, int n_in, int k, int q, int s,
                  monarch_dtype dtype, void* stream,
                  void* workspace, size_t workspace_bytes, unsigned flags);

/* Bytes of device scratch monarch_fwd_t needs (0 for the shape-generic SIMT kernels and the fp32 m = 16
 * kernel, and on invalid arguments). */
size_t monarch_fwd_t_workspace_bytes(int64_t batch, int n_in, int k, int q, int s,
                                     monarch_dtype dtype, unsigned flags);

/* The Monarch matrix itself as a dense array: M = P L P^T R (Definition 3.1), the matrix for which
 * monarch_fwd computes y = x M^T.  This is the conversion that sparse-to-dense training makes when it
 * switches from the Monarch layer to a dense one (Section 4: the factors multiplied out together
 * with the permutations).  Entry by entry, with o = l*k + c and col = kk*p + i,
 *   M[o][col] = sum over j < q with  dest(kk, j) in [c*q, (c+1)*q)  of  L[c][l][dest(kk, j) - c*q] * R[kk][j][i]
 * where dest(kk, j) is the position in U that stage-1 output (kk, j) is moved to (j*k + kk by
 * default, ((kk*q + j) mod k)*q + (kk*q + j) div k with MONARCH_FLAG_PERM_B).  In the square case
 * this is Equation (1), M[l*m + j][kk*m + i] = L[j][l][kk] * R[kk][j][i], one product per entry;
 * otherwise about q/k products are summed in fp32 and the entry is rounded once to `dtype`.
 * R (k, q, n_in/k), L (k, s, q) and M (k*s, n_in) row-major are device pointers, 16-byte aligned; M
 * is overwritten in full (structural zeros included).  `flags` may hold MONARCH_FLAG_PERM_B only;
 * any other flag is MONARCH_ERR_INVALID.  No workspace. */
int monarch_to_dense(const void* R, const void* L, void* M,
                     int n_in, int k, int q, int s,
                     monarch_dtype dtype, void* stream, unsigned flags);

/* Projection of a dense matrix onto the square Monarch matrices (Section 3.3, "Projection on the Set
 * M of Monarch Matrices", Theorem 1, Algorithm 1): the factors of the Monarch matrix closest to A in
 * Frobenius norm.  A is n x n row-major with n = m*m; with At[l][j][k][i] = A[l*m + j][k*m + i] every
 * slice At[:, j, k, :] (m x m) is replaced by its best rank-1 approximation sigma_1 u_1 v_1^T, and
 *   L[j][l][k] = sqrt(sigma_1) * u_1[l],    R[k][j][i] = sqrt(sigma_1) * v_1[i]
 * so that Equation (1), M[l*m + j][k*m + i] = L[j][l][k] * R[k][j][i], gives the projection (the
 * dense-to-sparse step that precedes fine-tuning).  The sign of (u_1, v_1) is not fixed, and when the
 * two largest singular values of a slice coincide any leading pair is a valid answer; only the
 * products L*R are determined.  A zero slice gives zero factors.
 * The singular triple is computed in fp32 by a one-sided Jacobi iteration (at most 40 sweeps, pairs
 * orthogonal to 3e-7 relative).  A (n, n), R (m, m, m), L (m, m, m) are device pointers, 16-byte
 * aligned, element type `dtype`; R and L are overwritten.  m <= 64; larger m returns
 * MONARCH_ERR_UNSUPPORTED; n != m*m or flags != 0 returns MONARCH_ERR_INVALID.  No workspace. */
int monarch_project(const void* A, void* R, void* L, int n, int m,
                    monarch_dtype dtype, void* stream, unsigned flags);

/* Complex-valued Monarch multiply.  The paper's results hold over the complex numbers as well
 * (Notation Review), and its MRI reconstruction model is a single complex Monarch matrix.  Same steps,
 * shapes and layouts as monarch_fwd_ex / monarch_bwd, every element a complex64 (two fp32: real part,
 * then imaginary part); products and sums in fp32.  The forward applies M^T (no conjugation).  The
 * backward returns, for a real loss, grad z = dLoss/dRe z + i dLoss/dIm z (the convention of automatic
 * differentiation):  dx = dy conj(M),  dL[c] = dW[c]^T conj(U[c]),  dR[kk] = dY1[kk]^T conj(x[kk]).
 * These three calls take no workspace and run shape-generic fp32 kernels; dR and dL are reduced with fp32
 * atomics (reproducible up to summation order).  flags: MONARCH_FLAG_PERM_B only. */
int monarch_fwd_c64(const void* x, const void* R, const void* L, void* y,
                    int64_t batch, int n_in, int k, int q, int s, void* stream, unsigned flags);
/* Conjugate transpose applied to every row:  y = x conj(M),  x (batch, k*s) -> y (batch, n_in), complex64.
 * M* is the second factor of the products M1 M2* of Section 3.1 ("Products of Monarch Matrices"; the star is
 * the conjugate transpose, Notation Review): M1 M2* x is monarch_fwd_h_c64 with the factors of M2, then
 * monarch_fwd_c64 with those of M1.  For real factors it is monarch_fwd_t.  Same shapes, layouts, flags and
 * errors as monarch_fwd_c64 with input and output sizes exchanged. */
int monarch_fwd_h_c64(const void* x, const void* R, const void* L, void* y,
                      int64_t batch, int n_in, int k, int q, int s, void* stream, unsigned flags);
int monarch_bwd_c64(const void* dy, const void* x, const void* R, const void* L,
                    void* dx, void* dR, void* dL,
                    int64_t batch, int n_in, int k, int q, int s, void* stream, unsigned flags);
/* The same three operations with a workspace (device memory, 256-byte aligned, at least
 * monarch_c64_workspace_bytes(pass, ...) bytes with pass 0 = monarch_fwd_c64_ws, 1 = monarch_bwd_c64_ws,
 * 2 = monarch_fwd_h_c64_ws; contents ignored on entry, unspecified on exit).
 * Square blocks p = q = s in {16, 32, 64} (any k; the DFT-initialised matrices of the MRI model are of this
 * kind) run on the matrix cores: one launch per block-diagonal factor, the vector between the factors kept
 * in the workspace in a tiled order that makes the permutation between them long contiguous runs; the weight
 * gradients are contracted over the batch on the matrix cores too and their partial sums added in a fixed
 * order (bit-reproducible, no atomics).  fp32 products and sums, as above.
 * Other shapes: the forward calls ignore the workspace; the backward writes the batch-major operands of the
 * weight gradients there and contracts them in one tiled launch whose batch chunks meet in fp32 atomics.
 * workspace == NULL: exactly the calls above.  A short or misaligned workspace returns MONARCH_ERR_WORKSPACE;
 * other errors as above.  monarch_c64_workspace_bytes returns 0 for arguments the calls reject (and for the
 * forward calls on shapes that use no workspace). */
size_t monarch_c64_workspace_bytes(int pass, int64_t batch, int n_in, int k, int q, int s, unsigned flags);
int monarch_fwd_c64_ws(const void* x, const void* R, const void* L, void* y,
                       int64_t batch, int n_in, int k, int q, int s, void* stream,
                       void* workspace, size_t workspace_bytes, unsigned flags);
int monarch_fwd_h_c64_ws(const void* x, const void* R, const void* L, void* y,
                         int64_t batch, int n_in, int k, int q, int s, void* stream,
                         void* workspace, size_t workspace_bytes, unsigned flags);
int monarch_bwd_c64_ws(const void* dy, const void* x, const void* R, const void* L,
                       void* dx, void* dR, void* dL,
                       int64_t batch, int n_in, int k, int q, int s, void* stream,
                       void* workspace, size_t workspace_bytes, unsigned flags);

/* Factors that make the square complex Monarch matrix a discrete Fourier transform (the model of the
 * MRI experiment starts from the inverse FFT): with n = m*m and w = exp(-2 pi i / n),
 *   R[kk][j][i] = w^(m*i*j),   L[j][l][kk] = w^(kk*j + m*kk*l)
 * give  P L P^T R = F_n P  (the DFT of the input read as an m x m grid and transposed: the 4-step
 * splitting).  inverse != 0: conjugate factors, L scaled by 1/n (F_n^{-1} P).  R and L are (m, m, m)
 * complex64 device arrays, 16-byte aligned; m <= 1024. */
int monarch_dft_factors(void* R, void* L, int m, int inverse, void* stream);

/* Name of the kernel family the dispatcher picks for this problem: pass 0 = forward
 * (monarch_fwd / monarch_fwd_ex), 1 = backward, 2 = forward with workspace (monarch_fwd_ws),
 * 3 = transposed multiply (monarch_fwd_t).  Static string, never NULL ("invalid" / "unsupported" on bad input). */
const char* monarch_kernel_name(int pass, int n_in, int k, int q, int s,
                                monarch_dtype dtype, unsigned flags);

/* Measurement aid, not part of the method: a plain streaming device-to-device copy
 * (16 bytes per lane, grid-stride) of `nbytes` bytes.  bench.py times it as the
 * empirical HBM roof of the machine, and its known traffic calibrates the
 * FETCH_SIZE / WRITE_SIZE hardware counters of a profiler run.  dst and src are
 * device pointers, 16-byte aligned, nbytes a multiple of 16, non-overlapping.
 * Returns MONARCH_ERR_INVALID otherwise; nbytes == 0 is a successful no-op. */
int monarch_stream_copy(void* dst, const void* src, size_t nbytes, void* stream);

/* Measurement aid, not part of the method: enqueues one empty kernel (one wavefront, no
 * arguments, no memory access) on `stream`.  The time per launch of a run of these is the
 * floor under any call on that stream; the n = 256, 64-row workload (Definition 3.1 with
 * m = 16), whose ideal time is tens of nanoseconds, is reported next to it.
 * Returns MONARCH_OK or MONARCH_ERR_HIP. */
int monarch_launch_probe(void* stream);

/* Human-readable text for a status code.  Static string, never NULL. */
const char* monarch_status_string(int status);

/* Library version: major*10000 + minor*100 + patch. */
int monarch_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MONARCH_H_ */
