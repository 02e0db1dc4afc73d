// Internal declarations shared by the HIP translation units of libkfac_hip.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <vector>
#include "../../include/kfac.h"

// A pointer that the compiler cannot trace back to a kernel argument (one read from a descriptor table in memory)
// is generic to it, and a load through a generic pointer is a flat load: it counts on the vector-memory counter
// and on the LDS counter, so every wait for an LDS read also waits for all the loads from memory still in flight,
// which undoes a software pipeline that prefetches from memory while it multiplies out of LDS.  Every operand of
// this library lives in device global memory; as_global() says so at the point of access.
template <typename T> using global_ptr = T __attribute__((address_space(1))) *;
template <typename T> __device__ inline global_ptr<T> as_global(T *p) { return (global_ptr<T>)p; }

// Kernel classes for the optional per-kernel timing (kfac_profile_begin / kfac_profile_end).
enum KfacKernelClass {
    KC_UNFOLD = 0, KC_SYRK, KC_SYRK_REDUCE, KC_PRECOND_GEMM, KC_EIG_SMALL, KC_EIG_SOLVE, KC_EIG_APPLY,
    KC_EIG_MISC, KC_EIG_POST, KC_EIG_COPY, KC_EIG_OUTER, KC_PRECOND_SCALE, KC_SYRK_B16, KC_PRECOND_GEMM_X3, KC_EIG_OUTER_ROWS, KC_INVERSE, KC_COUNT
};
struct KfacProfRec { int cls; hipEvent_t t0, t1; double flops, bytes; };

constexpr int KFAC_NUM_AUX_STREAMS = 4;   // internal streams of the eigensolver (default priority)
constexpr int KFAC_MAX_GROUPS = 128;      // distinct block counts in one kfac_eig call (8192 / 64)
constexpr int KFAC_EIG_SLOTS = 3;         // convergence reports a group may have in flight (events, pinned norms)

struct kfac_ctx {
    int device;
    hipStream_t stream;
    hipStream_t aux[KFAC_NUM_AUX_STREAMS];
    hipEvent_t ev_fork, ev_join[KFAC_NUM_AUX_STREAMS], ev_group[KFAC_EIG_SLOTS * KFAC_MAX_GROUPS];
    double *pinned;      // pinned host scratch of the eigensolver: convergence read-back, then its tables and statistics
    size_t pinned_bytes;
    // pinned staging ring for the host tables that the batched calls upload on ctx->stream (two halves; a half is
    // reused only after the copies issued from it have completed)
    char *stage;
    size_t stage_bytes, stage_off;
    int stage_half;
    hipEvent_t stage_ev[2];
    bool stage_used[2];
    char *ws;            // caller-owned device workspace
    size_t ws_bytes;
    int max_lds;         // bytes of LDS one workgroup may use on this device
    bool prof_on;        // bracket every kernel launch with events
    std::vector<KfacProfRec> prof;
    std::vector<hipEvent_t> ev_pool;
};

// Brackets one kernel launch with a pair of events when profiling is on; `flops` and `bytes` are the
// algorithmic work of that launch.
struct KfacProfScope {
    kfac_ctx *c;
    KfacProfRec r;
    hipStream_t s;
    KfacProfScope(kfac_ctx *ctx, int cls, double flops, double bytes) : KfacProfScope(ctx, cls, flops, bytes, ctx->stream) {}
    KfacProfScope(kfac_ctx *ctx, int cls, double flops, double bytes, hipStream_t st) : c(ctx), s(st) {
        if (!c->prof_on) return;
        r.cls = cls; r.flops = flops; r.bytes = bytes;
        r.t0 = get(); r.t1 = get();
        (void)hipEventRecord(r.t0, s);
    }
    ~KfacProfScope() {
        if (!c->prof_on) return;
        (void)hipEventRecord(r.t1, s);
        c->prof.push_back(r);
    }
    hipEvent_t get() {
        if (!c->ev_pool.empty()) { hipEvent_t e = c->ev_pool.back(); c->ev_pool.pop_back(); return e; }
        hipEvent_t e; (void)hipEventCreate(&e); return e;
    }
};

#define KFAC_HIP_CHECK(expr)                      \
    do {                                          \
        hipError_t _e = (expr);                   \
        if (_e != hipSuccess) return KFAC_EHIP;   \
    } while (0)

#define KFAC_CHECK(expr)                          \
    do {                                          \
        const int _rc = (expr);                   \
        if (_rc != KFAC_OK) return _rc;           \
    } while (0)

static inline size_t kfac_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

constexpr size_t KFAC_PINNED_NORMS = (size_t)3 << 16;    // the eigensolver's norms: 2 doubles per factor and report slot, 4096 factors
constexpr size_t KFAC_PINNED_TABLES = (size_t)1 << 18;   // the eigensolver's item tables and small-factor statistics
constexpr size_t KFAC_STAGE_BYTES = (size_t)4 << 20;     // staging ring of the batched calls

// Copy a host table to device memory on ctx->stream through the pinned staging ring: the host buffer may be
// freed as soon as this returns, and the call does not wait for work already queued on the stream (a copy from
// pageable memory would).  Tables larger than half the ring go through the runtime's own staging instead.
int kfac_upload(kfac_ctx *ctx, void *dst_dev, const void *src_host, size_t bytes);

// Tiling constants shared between host-side sizing and kernels.
constexpr int KFAC_TILE = 128;       // GEMM / SYRK output tile edge
constexpr int KFAC_EIG_SMALL = 128;  // factors up to this size are solved inside one workgroup's LDS
constexpr int KFAC_EIG_B = 32;       // block size of the blocked Jacobi path (sub-problems are 2B x 2B)
constexpr int KFAC_MAX_D = 8192;
// A factor updated alone splits its contraction into at most this many partial tiles (or one per tile, if it has
// more tiles than that): what kfac_workspace_bytes() sizes the workspace of a single update for.
constexpr int KFAC_SYRK_MAX_SINGLE_PARTIALS = 1536;
constexpr size_t KFAC_STATIC_SCRATCH_BYTES = (size_t)48 << 20;   // the library's static device scratch (per device)

// ---- launchers implemented in the kernel files (all enqueue on ctx->stream) ----
int kfac_launch_unfold(kfac_ctx *ctx, const kfac_conv_desc *d, const void *x, void *patches);
int kfac_launch_unfold_batched(kfac_ctx *ctx, int n, const kfac_conv_desc *descs, const void *const *x, void *const *patches);
size_t kfac_unfold_ws_bytes_impl(int n);
size_t kfac_syrk_workspace_bytes(int D, int64_t R);
size_t kfac_syrk_ws_bytes_impl(int n, const kfac_factor_item *items);
int kfac_launch_update_factors_batched(kfac_ctx *ctx, int n, const kfac_factor_item *items);
// the same with the scratch (tables, split partials) in `ws` instead of the context's workspace
int kfac_launch_update_factors_ws(kfac_ctx *ctx, int n, const kfac_factor_item *items, char *ws, size_t ws_bytes);
bool kfac_valid_factor_item(const kfac_factor_item &it, bool pointers);
// Looks up, once per device and with that device current, the device address of the library's static scratch array.
int kfac_static_scratch_init(int device);
int kfac_launch_update_factors(kfac_ctx *ctx, const void *X, int dtype, int layout, int N, int d, int T,
                               int append_ones, float scale, float decay, float *F);
int kfac_launch_precondition(kfac_ctx *ctx, const float *QA, const float *lamA, int dA, const float *QG,
                             const float *lamG, int dG, float damping, void *grad, int grad_dtype);
int kfac_launch_precondition_batched(kfac_ctx *ctx, int n, const kfac_precond_item *items, bool scaled, float kappa, float lr,
                                     float *nu);
size_t kfac_precond_ws_bytes_impl(int n, const kfac_precond_item *items);
size_t kfac_eig_ws_bytes_impl(int batch, const int *d);
size_t kfac_invert_ws_bytes_impl(int batch, const int *d);
int kfac_launch_invert_factors(kfac_ctx *ctx, int batch, const float *const *F, const int *d, float damping, float *const *Finv);
size_t kfac_precondition_inverse_ws_bytes_impl(int n, const kfac_precond_inv_item *items);
int kfac_launch_precondition_inverse_batched(kfac_ctx *ctx, int n, const kfac_precond_inv_item *items);
int kfac_launch_eig(kfac_ctx *ctx, int batch, const float *const *F, const int *d, float *const *Q,
                    float *const *lam, const kfac_eig_opts *opts, kfac_eig_info *info);
