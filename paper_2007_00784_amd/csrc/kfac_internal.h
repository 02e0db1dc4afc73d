// Internal declarations shared by the HIP translation units of libkfac_hip.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/kfac.h"

struct kfac_ctx {
    int device;
    hipStream_t stream;
    char *ws;            // caller-owned device workspace
    size_t ws_bytes;
    double *host_flags;  // pinned host scratch for the eigensolver's convergence read-back
    int max_lds;         // bytes of LDS one workgroup may use on this device
};

#define KFAC_HIP_CHECK(expr)                      \
    do {                                          \
        hipError_t _e = (expr);                   \
        if (_e != hipSuccess) return KFAC_EHIP;   \
    } while (0)

static inline size_t kfac_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Tiling constants shared between host-side sizing and kernels.
constexpr int KFAC_TILE = 128;       // GEMM / SYRK output tile edge
constexpr int KFAC_EIG_SMALL = 128;  // factors up to this size are solved inside one workgroup's LDS
constexpr int KFAC_EIG_B = 64;       // block size of the blocked Jacobi path (sub-problems are 2B x 2B)
constexpr int KFAC_MAX_D = 8192;

// ---- launchers implemented in the kernel files (all enqueue on ctx->stream) ----
int kfac_launch_unfold(kfac_ctx *ctx, const kfac_conv_desc *d, const void *x, void *patches);
size_t kfac_syrk_workspace_bytes(int D, int64_t R);
int kfac_launch_update_factors(kfac_ctx *ctx, const void *X, int dtype, int layout, int N, int d, int T,
                               int append_ones, float scale, float decay, float *F);
int kfac_launch_precondition(kfac_ctx *ctx, const float *QA, const float *lamA, int dA, const float *QG,
                             const float *lamG, int dG, float damping, void *grad, int grad_dtype);
size_t kfac_eig_ws_bytes_impl(int batch, const int *d);
int kfac_launch_eig(kfac_ctx *ctx, int batch, const float *const *F, const int *d, float *const *Q,
                    float *const *lam, const kfac_eig_opts *opts, kfac_eig_info *info);
