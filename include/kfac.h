/*
 * kfac.h -- C ABI of the MI355X (gfx950) K-FAC preconditioner library.
 *
 * The library computes, per layer, the steps of the K-FAC gradient
 * preconditioner of arXiv 2007.00784 ("Convolutional Neural Network Training
 * with Distributed K-FAC"):
 *   unfold conv inputs -> Kronecker factors A, G with running average ->
 *   symmetric eigendecomposition of each factor -> eigenbasis preconditioning.
 *
 * Conventions for every call
 *  - C linkage, plain structs, int status (0 = KFAC_OK, negative = error).
 *    No exception crosses the boundary.  kfac_strerror() names a status.
 *  - Every data pointer is a DEVICE pointer owned by the caller unless it is
 *    marked "host".  The library never allocates or frees user-visible memory
 *    and keeps no pointer after a call returns, except the workspace given to
 *    kfac_create(), which it uses as scratch until kfac_destroy().
 *  - Work is enqueued on the hipStream_t given to kfac_create().  All calls
 *    are asynchronous with respect to the host except kfac_eig(), which waits
 *    on the stream between sweeps to decide convergence and returns with its
 *    outputs complete.
 *  - Matrices are row-major, fp32 unless stated.  Outputs must not alias
 *    inputs except where a parameter is marked in/out.
 *  - A context is not thread-safe; use one context per stream.
 *  - Arguments are validated on the host before any kernel is launched; an
 *    invalid argument returns KFAC_EINVAL and launches nothing.
 */
#ifndef KFAC_H
#define KFAC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    KFAC_OK = 0,
    KFAC_EINVAL = -1,     /* NULL / out-of-range / unsupported argument            */
    KFAC_ENOCONV = -2,    /* eigensolver reached max_sweeps; outputs still written */
    KFAC_EHIP = -3,       /* a HIP runtime call failed                             */
    KFAC_EWORKSPACE = -4, /* the context's workspace is too small for this call    */
    KFAC_ESCRATCH = -5    /* the input needs more than the library's static scratch */
};

typedef enum { KFAC_F32 = 0, KFAC_BF16 = 1 } kfac_dtype;

/* Layout of a sample matrix X with R = N*T sample rows and d features.
 *   KFAC_LAYOUT_RD : [R][d], d contiguous (FC activations and gradients; T = 1 is typical)
 *   KFAC_LAYOUT_NDT: [N][d][T], T contiguous: per-example slabs.  This is the NCHW layout of
 *                    conv output gradients ([N][C_out][Ho*Wo]) and of the input of a 1x1
 *                    stride-1 unpadded conv, and it is what kfac_unfold() writes.          */
typedef enum { KFAC_LAYOUT_RD = 0, KFAC_LAYOUT_NDT = 1 } kfac_layout;

typedef struct {
    int N, C, H, W;          /* input tensor, NCHW                               */
    int kh, kw;              /* kernel                                           */
    int stride_h, stride_w;
    int pad_h, pad_w;        /* zero padding on each side                        */
    int dtype;               /* kfac_dtype of x and of the patches               */
} kfac_conv_desc;

typedef struct {
    int max_sweeps;          /* cap on Jacobi sweeps (<=0: 30)                    */
    float tol;               /* stop when off(F)_F <= tol * ||F||_F (<=0: 2e-6)   */
    int fp32_only;           /* 0 (default): for d >= 2048 the rank-256 update passes run as split-fp16
                                MFMA products (hi + lo halves, three products per fp32 product, fp32
                                accumulation): same tolerances met, errors bounded normwise (relative to
                                ||F||_F).  1: every product on the fp32 MFMA path: slower, keeps fp32's
                                elementwise accuracy on strongly graded spectra.                   */
    int warm_start;          /* 1: on entry every Q_i with d_i > 128 holds an orthonormal basis to start from
                                (typically the eigenvectors of the previous decomposition of a slowly moving
                                factor: the remark of Sec. V-C that the FIM becomes more stable as training progresses); the iteration then runs on Q_i^T F_i Q_i, which is close to
                                diagonal, and needs fewer sweeps.  Costs 4 d^3 flops per factor up front; a basis
                                that is not orthonormal to fp32 rounding gives wrong results.  0: start from I.   */
} kfac_eig_opts;

typedef struct {             /* host memory, filled when kfac_eig() returns       */
    int sweeps;              /* sweeps performed                                  */
    float off_norm_rel;      /* off(F)_F / ||F||_F of the rotated matrix at exit  */
    int converged;           /* 1 if the tolerance was met                        */
} kfac_eig_info;

typedef struct kfac_ctx kfac_ctx;

/* Create a context bound to HIP device `device` and stream `hip_stream` (a hipStream_t; NULL is
 * the default stream).  `workspace_dev` is caller-owned device scratch of `workspace_bytes` bytes,
 * 256-byte aligned, which must outlive the context; see kfac_workspace_bytes().  */
int kfac_create(kfac_ctx **ctx, int device, void *hip_stream, void *workspace_dev, size_t workspace_bytes);
int kfac_destroy(kfac_ctx *ctx);

/* Pure host functions: bytes of workspace that suffice for any call with factor dimension <= max_d,
 * at most max_batch_factors factors per kfac_eig() call and at most max_R sample rows; and the exact
 * requirement of one kfac_eig() call on the given host array of dimensions.  */
size_t kfac_workspace_bytes(int max_d, int max_batch_factors, int64_t max_R);
size_t kfac_eig_workspace_bytes(int batch, const int *d /* host */);

const char *kfac_strerror(int code);

/* Unfold of a conv input (the paper handles Conv2D layers, Sec. V, treating every output location
 * of every example as one sample): patches[n][(c*kh+ky)*kw+kx][ho*Wo+wo] = x[n][c][ho*sh-ph+ky][wo*sw-pw+kx],
 * zero outside the image; Ho = (H+2ph-kh)/sh+1, Wo likewise.
 *   x       : [N][C][H][W], dtype desc->dtype
 *   patches : [N][C*kh*kw][Ho*Wo] (KFAC_LAYOUT_NDT), same dtype, no bias row.
 * Size limit: kh padded input rows must fit the 16 KB staging tile, kh*(W+2pw) <= 4096 elements (fp32) or
 * 8192 (bf16); beyond that KFAC_EINVAL.  */
int kfac_unfold(kfac_ctx *ctx, const kfac_conv_desc *desc, const void *x, void *patches);

/* The same for n layers in one launch per element type (a network's late layers are a few microseconds of work
 * each, which separate launches cannot fill the machine with):
 *   descs   : HOST array of n descriptors
 *   x       : HOST array of n device pointers, x[i] as for kfac_unfold() with descs[i]
 *   patches : HOST array of n device pointers, distinct, patches[i] as for kfac_unfold()
 * Uses kfac_unfold_workspace_bytes(n) bytes at the start of the context's workspace (a table that the launch
 * reads; later calls on the same stream may overwrite it).  KFAC_EINVAL for any invalid layer: nothing is launched. */
int kfac_unfold_batched(kfac_ctx *ctx, int n, const kfac_conv_desc *descs /* host */, const void *const *x /* host */,
                        void *const *patches /* host */);
size_t kfac_unfold_workspace_bytes(int n);

/* Kronecker factor of a mini-batch folded into its running average (Sec. II-C: A = a a^T, G = g g^T
 * over the samples; Sec. IV-B: running average with parameter xi):
 *   F <- decay * F + (1 - decay) * scale * Xt^T Xt,   Xt = [X | 1] if append_ones else X
 *   X     : samples, dtype `dtype`, layout `layout`, N examples x T locations x d features
 *   F     : [D][D] fp32, D = d + append_ones, full symmetric storage, in/out
 *   decay : xi, weight of the history; decay = 0 overwrites F with the batch factor
 * The result is exactly symmetric.  Split-K partial sums are reduced in a fixed order, so the
 * result is bit-reproducible run to run.  */
int kfac_update_factors(kfac_ctx *ctx, const void *X, int dtype, int layout, int N, int d, int T,
                        int append_ones, float scale, float decay, float *F);

/* The same update for a batch of factors in as few launches as there are operand forms (layout x dtype):
 * every factor is cut into jobs of similar length that fill the machine together, so small layers cost
 * no launch of their own.  items: host array; fields as the arguments of kfac_update_factors.  The
 * factors of one call must be distinct.  Workspace: kfac_update_factors_workspace_bytes().  */
typedef struct {
    const void *X;
    int dtype, layout;
    int N, d, T;
    int append_ones;
    float scale, decay;
    float *F;
} kfac_factor_item;
int kfac_update_factors_batched(kfac_ctx *ctx, int n, const kfac_factor_item *items /* host */);
size_t kfac_update_factors_workspace_bytes(int n, const kfac_factor_item *items /* host; X, F not read */);

/* kfac_update_factors() for callers that cannot allocate device memory or provide a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Arguments, result and kernels are those
 * of kfac_update_factors() (bit-identical output); the job tables and split partials live in a static device
 * array of the library (kfac_static_scratch_bytes() = 48 MiB, held by every device the library runs on until the
 * process ends) instead of the context's workspace, and the call allocates nothing, on the device or in pinned
 * memory.  A factor whose split plan needs more than that returns KFAC_ESCRATCH and launches nothing (the plan
 * of a lone factor keeps at most 1536 partial tiles of 64.5 KB; 48 MiB hold 761 of them -- every plan that fills
 * the machine once).  All calls on a device share the array: two calls that overlap on one device (different
 * contexts or streams) race; calls on one stream are ordered and safe.  */
int kfac_update_factors_static(kfac_ctx *ctx, const void *X, int dtype, int layout, int N, int d, int T,
                               int append_ones, float scale, float decay, float *F);
size_t kfac_static_scratch_bytes(void);

/* Symmetric eigendecompositions F_i = Q_i diag(lam_i) Q_i^T (Sec. IV-A, Algorithm 1 step 2) of a
 * batch of factors by (block) Jacobi iteration; lam ascending, eigenvectors in the columns of Q.
 *   F, Q, lam : HOST arrays of `batch` device pointers; F_i is [d_i][d_i] (read only),
 *               Q_i [d_i][d_i], lam_i [d_i]
 *   d         : host array of dimensions, 1 <= d_i <= 8192
 *   opts      : host, may be NULL for defaults;  info: host array [batch], may be NULL
 * Returns KFAC_ENOCONV if any factor missed the tolerance within max_sweeps (all outputs are
 * still the current iterate).  Non-finite input gives non-finite output and KFAC_ENOCONV.  */
int kfac_eig(kfac_ctx *ctx, int batch, const float *const *F, const int *d, float *const *Q,
             float *const *lam, const kfac_eig_opts *opts, kfac_eig_info *info);

/* Eigenbasis preconditioning, Eqs. (v1), (v2), (kfac-eigen) of Sec. IV-A, in place:
 *   V1 = QG^T grad QA;  V2 = V1 / (max(lamG,0) max(lamA,0)^T + damping);  grad <- QG V2 QA^T
 *   QA [dA][dA], lamA [dA], QG [dG][dG], lamG [dG] : fp32
 *   grad : [dG][dA], dtype grad_dtype, in/out; its last column is the bias gradient when the
 *          A factor was built with append_ones.  damping > 0.  */
int kfac_precondition(kfac_ctx *ctx, const float *QA, const float *lamA, int dA, const float *QG,
                      const float *lamG, int dG, float damping, void *grad, int grad_dtype);

/* The same operation for a batch of layers in four launches (one per GEMM stage, covering the output
 * tiles of every layer): what a training step calls once per iteration (Algorithm 1, step 3).
 *   items : HOST array of n records; every pointer in a record is a device pointer with the meaning
 *           and shape of the kfac_precondition() argument of the same name.  Gradients must not alias
 *           one another.  kfac_precondition_workspace_bytes() gives the workspace the batch needs.  */
typedef struct {
    const float *QA, *lamA;
    int dA;
    const float *QG, *lamG;
    int dG;
    float damping;
    void *grad;
    int grad_dtype;
    int factored_damping;    /* 0: the step of Eqs. (v1), (v2), (kfac-eigen): divide by lamG lamA^T + damping (exact
                                Tikhonov damping of the Kronecker product).  1: the explicit-inverse method of
                                Sec. II-C, Eq. (kfac-damped): (G + damping I)^-1 grad (A + damping I)^-1, computed in
                                the eigenbasis as a division by (lamG + damping)(lamA + damping)^T              */
    int split_f16;           /* 0: the four GEMMs run on the fp32 matrix instructions.  1: every fp32 operand element
                                is split into two fp16 halves (22 significand bits) and a product is three fp16
                                matrix instructions with fp32 accumulation: about twice as fast, relative Frobenius
                                error of the result about 1e-6 instead of 1e-7 (entries more than 2^25 below the
                                largest of their matrix are not resolved).  Meant for bf16 gradients, whose own
                                rounding is 4e-3, and for callers who accept the normwise bound             */
} kfac_precond_item;
int kfac_precondition_batched(kfac_ctx *ctx, int n, const kfac_precond_item *items /* host */);
size_t kfac_precondition_workspace_bytes(int n, const kfac_precond_item *items /* host; only dA, dG are read */);

/* The explicit-inverse method (Sec. II-C, Eq. (kfac-damped); the method that Sec. IV-A and Table I set the
 * eigendecomposition against), as the paper describes it: the damped factors are inverted once,
 *     Finv[b] = (F[b] + damping I)^-1 ,
 * and a gradient is preconditioned by two plain products, grad <- Ginv grad Ainv.
 * kfac_invert_factors: blocked Cholesky factorisation, triangular inversion and L^-T L^-1, all in fp32; the factors
 * are taken one after another on the context's stream.
 *   F, d, Finv : HOST arrays of `batch` entries; F[b], Finv[b] device pointers to [d[b]][d[b]] fp32 matrices
 *                (F[b] symmetric positive semi-definite, read only; Finv[b] must not alias it), damping > 0.
 *   A factor that is not positive definite after damping (or not finite) gives a non-finite Finv; no error is
 *   reported for it.  Accuracy is that of an fp32 Cholesky inverse: relative error of the order of
 *   cond(F + damping I) * 6e-8.  Workspace: kfac_invert_workspace_bytes() (covered by kfac_workspace_bytes(max_d, ..)).
 *   Factors of equal size advance together, and with workspace to spare (four times the largest factor's need)
 *   groups run side by side on the context's internal streams; the caller's stream waits for all of them.
 * kfac_precondition_inverse[_batched]: grad [dG][dA] (fp32 or bf16, in/out) <- Ginv grad Ainv on the fp32 matrix
 *   instructions, two launches for the whole batch; items is a HOST array, every pointer in it a device pointer;
 *   gradients must not alias one another.  Workspace: kfac_precondition_inverse_workspace_bytes() (dG*dA floats per
 *   layer).  All calls are asynchronous with respect to the host.  */
int kfac_invert_factors(kfac_ctx *ctx, int batch, const float *const *F /* host array of device ptrs */,
                        const int *d /* host */, float damping, float *const *Finv /* host array of device ptrs */);
size_t kfac_invert_workspace_bytes(int batch, const int *d /* host */);
typedef struct {
    const float *Ainv;   /* [dA][dA] */
    int dA;
    const float *Ginv;   /* [dG][dG] */
    int dG;
    void *grad;          /* [dG][dA], in/out */
    int grad_dtype;
} kfac_precond_inv_item;
int kfac_precondition_inverse(kfac_ctx *ctx, const float *Ainv, int dA, const float *Ginv, int dG, void *grad,
                              int grad_dtype);
int kfac_precondition_inverse_batched(kfac_ctx *ctx, int n, const kfac_precond_inv_item *items /* host */);
size_t kfac_precondition_inverse_workspace_bytes(int n, const kfac_precond_inv_item *items /* host; only dA, dG are read */);

/* The same, followed by the gradient scaling of Sec. V-C ("K-FAC Hyper-Parameters"): every preconditioned
 * gradient P_l is multiplied by
 *     nu = min(1, sqrt(kappa / (lr^2 * sum_l |<P_l, grad_l>|)))
 * with grad_l the gradient as it was on entry and <.,.> the sum of elementwise products (for bf16 gradients
 * of the values as stored).  The inner products are taken in the last GEMM's epilogue (per-tile partial sums,
 * added in a fixed order: deterministic).  nu: DEVICE pointer to one float, written by the call (1 when the
 * sum is zero); kappa > 0, lr > 0.  Same workspace as kfac_precondition_batched.  */
int kfac_precondition_batched_scaled(kfac_ctx *ctx, int n, const kfac_precond_item *items /* host */, float kappa,
                                     float lr, float *nu /* device, out */);

/* Update-decoupled schedule (Sec. IV-C, Sec. V-C), host only: at iteration k refresh the factors
 * when k % f_fac == 0 and the eigendecompositions when k % f_eig == 0; precondition always.  */
int kfac_schedule_due(int64_t k, int f_fac, int f_eig, int *do_factors, int *do_eig);

/* Optional per-kernel timing, for benchmarks.  Between kfac_profile_begin() and kfac_profile_end()
 * every kernel launch of this context is bracketed by a pair of hipEvents on the context's stream.
 * kfac_profile_end() waits for the stream and fills up to `max` records (host memory), one per
 * kernel class that was launched, with the launch count, the summed duration and the summed
 * algorithmic work of those launches (flops for contractions and rotations, bytes for data
 * movement), and stores the number of records in *n.  */
typedef struct {
    char name[32];
    int launches;
    double ms;       /* total over the launches */
    double flops;    /* algorithmic floating-point operations, total */
    double bytes;    /* algorithmic HBM bytes, total */
} kfac_kernel_stat;
int kfac_profile_begin(kfac_ctx *ctx);
int kfac_profile_end(kfac_ctx *ctx, kfac_kernel_stat *out /* host */, int max, int *n /* host */);

#ifdef __cplusplus
}
#endif
#endif /* KFAC_H */
