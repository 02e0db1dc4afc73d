// C-ABI entry points: argument validation, workspace accounting, dispatch to the kernel launchers.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string_view>
#include <vector>
#include "kfac_internal.h"

namespace {

bool valid_dtype(int t) { return t == KFAC_F32 || t == KFAC_BF16; }

// cheap sanity check that a pointer the caller calls "device" is usable from this device
bool is_device_ptr(const void *p) {
    if (!p) return false;
    hipPointerAttribute_t a;
    if (hipPointerGetAttributes(&a, p) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return a.type == hipMemoryTypeDevice;   // plain device memory only: no managed or host-mapped workspace
}

}  // namespace

int kfac_upload(kfac_ctx *c, void *dst_dev, const void *src_host, size_t bytes) {
    if (bytes == 0) return KFAC_OK;
    const size_t half = c->stage_bytes / 2, need = kfac_align_up(bytes, 64);
    if (need > half) {
        KFAC_HIP_CHECK(hipMemcpyAsync(dst_dev, src_host, bytes, hipMemcpyHostToDevice, c->stream));
        return KFAC_OK;
    }
    if (c->stage_off + need > half) {
        // this half is full: mark where its last copy sits in the stream, move to the other half and wait until
        // the copies issued from that one (a whole half ago) are through
        KFAC_HIP_CHECK(hipEventRecord(c->stage_ev[c->stage_half], c->stream));
        c->stage_used[c->stage_half] = true;
        c->stage_half ^= 1;
        c->stage_off = 0;
        if (c->stage_used[c->stage_half]) KFAC_HIP_CHECK(hipEventSynchronize(c->stage_ev[c->stage_half]));
    }
    char *slot = c->stage + (size_t)c->stage_half * half + c->stage_off;
    memcpy(slot, src_host, bytes);
    c->stage_off += need;
    KFAC_HIP_CHECK(hipMemcpyAsync(dst_dev, slot, bytes, hipMemcpyHostToDevice, c->stream));
    return KFAC_OK;
}

bool kfac_valid_factor_item(const kfac_factor_item &it, bool pointers) {
    if (pointers && (!it.X || !it.F || (const void *)it.F == it.X)) return false;
    if (!valid_dtype(it.dtype) || (it.layout != KFAC_LAYOUT_RD && it.layout != KFAC_LAYOUT_NDT)) return false;
    if (it.N < 1 || it.d < 1 || it.T < 1 || (it.append_ones != 0 && it.append_ones != 1)) return false;
    if (it.d + it.append_ones > KFAC_MAX_D) return false;
    if ((int64_t)it.N * it.T >= (int64_t)1 << 30) return false;
    if ((int64_t)it.d * it.T >= (int64_t)1 << 31) return false;   // 32-bit offsets inside one example's slab
    if (pointers && (!(it.decay >= 0.f && it.decay <= 1.f) || !std::isfinite(it.scale))) return false;
    return true;
}

extern "C" {

const char *kfac_strerror(int code) {
    switch (code) {
        case KFAC_OK: return "success";
        case KFAC_EINVAL: return "invalid or unsupported argument";
        case KFAC_ENOCONV: return "eigensolver did not reach the tolerance within max_sweeps";
        case KFAC_EHIP: return "HIP runtime failure";
        case KFAC_EWORKSPACE: return "workspace too small";
        case KFAC_ESCRATCH: return "input needs more scratch than the library's static device buffer holds";
        default: return "unknown status";
    }
}

int kfac_create(kfac_ctx **out, int device, void *hip_stream, void *workspace_dev, size_t workspace_bytes) {
    if (!out) return KFAC_EINVAL;
    *out = nullptr;
    int ndev = 0;
    KFAC_HIP_CHECK(hipGetDeviceCount(&ndev));
    if (device < 0 || device >= ndev) return KFAC_EINVAL;
    if (workspace_bytes > 0 && (!workspace_dev || ((uintptr_t)workspace_dev & 255))) return KFAC_EINVAL;
    KFAC_HIP_CHECK(hipSetDevice(device));
    KFAC_CHECK(kfac_static_scratch_init(device));   // device address of the library's static scratch on this device
    hipDeviceProp_t prop;
    KFAC_HIP_CHECK(hipGetDeviceProperties(&prop, device));
    if (std::string_view(prop.gcnArchName).substr(0, 6) != "gfx950") return KFAC_EINVAL;  // built for gfx950 only
    if (workspace_bytes > 0 && !is_device_ptr(workspace_dev)) return KFAC_EINVAL;
    kfac_ctx *c = new (std::nothrow) kfac_ctx();
    if (!c) return KFAC_EHIP;
    c->device = device;
    c->stream = (hipStream_t)hip_stream;
    c->ws = (char *)workspace_dev;
    c->ws_bytes = workspace_bytes;
    c->pinned = nullptr;
    c->pinned_bytes = KFAC_PINNED_NORMS + KFAC_PINNED_TABLES;
    c->stage = nullptr;
    c->stage_bytes = KFAC_STAGE_BYTES;
    c->stage_off = 0;
    c->stage_half = 0;
    c->stage_used[0] = c->stage_used[1] = false;
    bool ok = hipHostMalloc((void **)&c->pinned, c->pinned_bytes, hipHostMallocDefault) == hipSuccess;
    ok = ok && hipHostMalloc((void **)&c->stage, c->stage_bytes, hipHostMallocDefault) == hipSuccess;
    int made_streams = 0, made_events = 0;
    hipEvent_t *evs[4 + KFAC_NUM_AUX_STREAMS + KFAC_EIG_SLOTS * KFAC_MAX_GROUPS];
    int ne = 0;
    evs[ne++] = &c->ev_fork;
    evs[ne++] = &c->stage_ev[0];
    evs[ne++] = &c->stage_ev[1];
    for (int i = 0; i < KFAC_NUM_AUX_STREAMS; ++i) evs[ne++] = &c->ev_join[i];
    for (int i = 0; i < KFAC_EIG_SLOTS * KFAC_MAX_GROUPS; ++i) evs[ne++] = &c->ev_group[i];
    for (; ok && made_streams < KFAC_NUM_AUX_STREAMS; ++made_streams)
        ok = hipStreamCreateWithFlags(&c->aux[made_streams], hipStreamNonBlocking) == hipSuccess;
    for (; ok && made_events < ne; ++made_events)
        ok = hipEventCreateWithFlags(evs[made_events], hipEventDisableTiming) == hipSuccess;
    if (!ok) {
        for (int i = 0; i < made_events; ++i) (void)hipEventDestroy(*evs[i]);
        for (int i = 0; i < made_streams; ++i) (void)hipStreamDestroy(c->aux[i]);
        if (c->pinned) (void)hipHostFree(c->pinned);
        if (c->stage) (void)hipHostFree(c->stage);
        delete c;
        return KFAC_EHIP;
    }
    c->prof_on = false;
    int lds = 0;
    if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, device) != hipSuccess) lds = 65536;
    c->max_lds = lds;
    *out = c;
    return KFAC_OK;
}

int kfac_destroy(kfac_ctx *ctx) {
    if (!ctx) return KFAC_EINVAL;
    for (auto &r : ctx->prof) { (void)hipEventDestroy(r.t0); (void)hipEventDestroy(r.t1); }
    for (auto e : ctx->ev_pool) (void)hipEventDestroy(e);
    (void)hipEventDestroy(ctx->ev_fork);
    (void)hipEventDestroy(ctx->stage_ev[0]);
    (void)hipEventDestroy(ctx->stage_ev[1]);
    for (int i = 0; i < KFAC_NUM_AUX_STREAMS; ++i) (void)hipEventDestroy(ctx->ev_join[i]);
    for (int i = 0; i < KFAC_EIG_SLOTS * KFAC_MAX_GROUPS; ++i) (void)hipEventDestroy(ctx->ev_group[i]);
    for (int i = 0; i < KFAC_NUM_AUX_STREAMS; ++i) (void)hipStreamDestroy(ctx->aux[i]);
    (void)hipHostFree(ctx->pinned);
    (void)hipHostFree(ctx->stage);
    delete ctx;
    return KFAC_OK;
}

size_t kfac_eig_workspace_bytes(int batch, const int *d) {
    if (batch <= 0 || !d) return 0;
    for (int i = 0; i < batch; ++i)
        if (d[i] < 1 || d[i] > KFAC_MAX_D) return 0;
    return kfac_eig_ws_bytes_impl(batch, d);
}

size_t kfac_workspace_bytes(int max_d, int max_batch_factors, int64_t max_R) {
    if (max_d < 1 || max_d > KFAC_MAX_D || max_batch_factors < 1 || max_R < 1) return 0;
    // SYRK split partials of a factor updated alone, whatever its operand form: at most
    // max(KFAC_SYRK_MAX_SINGLE_PARTIALS, tiles) partial tiles of 128 x 128 + 128 floats, plus the job tables
    const size_t nt = (max_d + KFAC_TILE - 1) / KFAC_TILE, ntri = nt * (nt + 1) / 2;
    size_t need = std::max<size_t>(KFAC_SYRK_MAX_SINGLE_PARTIALS, ntri) * (size_t)(KFAC_TILE * KFAC_TILE + KFAC_TILE) * sizeof(float) +
                  (size_t)(1 << 20);
    (void)max_R;
    // precondition: two dG x dA temporaries
    need = std::max(need, 2 * kfac_align_up((size_t)max_d * max_d, 64) * sizeof(float) + (size_t)(1 << 20));
    // eig: every factor of the batch at the largest size, advanced together
    std::vector<int> d((size_t)max_batch_factors, max_d);
    need = std::max(need, kfac_eig_ws_bytes_impl(max_batch_factors, d.data()));
    // explicit inverses: one factor at a time
    need = std::max(need, kfac_invert_ws_bytes_impl(1, d.data()));
    return kfac_align_up(need, 256);
}

static bool valid_conv_desc(const kfac_conv_desc &d) {
    if (d.N < 1 || d.C < 1 || d.H < 1 || d.W < 1 || d.kh < 1 || d.kw < 1) return false;
    if (d.stride_h < 1 || d.stride_w < 1 || d.pad_h < 0 || d.pad_w < 0) return false;
    if (d.pad_h >= d.kh || d.pad_w >= d.kw) return false;  // every window must touch the image
    if (d.H + 2 * d.pad_h < d.kh || d.W + 2 * d.pad_w < d.kw) return false;
    if (!valid_dtype(d.dtype)) return false;
    return (int64_t)d.C * d.kh * d.kw <= KFAC_MAX_D;
}

int kfac_unfold(kfac_ctx *ctx, const kfac_conv_desc *desc, const void *x, void *patches) {
    if (!ctx || !desc || !x || !patches || x == patches) return KFAC_EINVAL;
    if (!valid_conv_desc(*desc)) return KFAC_EINVAL;
    return kfac_launch_unfold(ctx, desc, x, patches);
}

int kfac_unfold_batched(kfac_ctx *ctx, int n, const kfac_conv_desc *descs, const void *const *x, void *const *patches) {
    if (!ctx || n < 0 || (n > 0 && (!descs || !x || !patches))) return KFAC_EINVAL;
    for (int i = 0; i < n; ++i) {
        if (!x[i] || !patches[i] || x[i] == patches[i] || !valid_conv_desc(descs[i])) return KFAC_EINVAL;
        for (int j = 0; j < i; ++j)
            if (patches[j] == patches[i]) return KFAC_EINVAL;
    }
    if (n == 0) return KFAC_OK;
    return kfac_launch_unfold_batched(ctx, n, descs, x, patches);
}

size_t kfac_unfold_workspace_bytes(int n) { return n > 0 ? kfac_unfold_ws_bytes_impl(n) : 0; }

int kfac_update_factors(kfac_ctx *ctx, const void *X, int dtype, int layout, int N, int d, int T,
                        int append_ones, float scale, float decay, float *F) {
    if (!ctx) return KFAC_EINVAL;
    const kfac_factor_item it{X, dtype, layout, N, d, T, append_ones, scale, decay, F};
    if (!kfac_valid_factor_item(it, true)) return KFAC_EINVAL;
    return kfac_launch_update_factors_batched(ctx, 1, &it);
}

int kfac_update_factors_batched(kfac_ctx *ctx, int n, const kfac_factor_item *items) {
    if (!ctx || n < 0 || (n > 0 && !items)) return KFAC_EINVAL;
    for (int i = 0; i < n; ++i) {
        if (!kfac_valid_factor_item(items[i], true)) return KFAC_EINVAL;
        for (int j = 0; j < i; ++j)
            if (items[j].F == items[i].F) return KFAC_EINVAL;
    }
    if (n == 0) return KFAC_OK;
    return kfac_launch_update_factors_batched(ctx, n, items);
}

size_t kfac_update_factors_workspace_bytes(int n, const kfac_factor_item *items) {
    if (n <= 0 || !items) return 0;
    for (int i = 0; i < n; ++i)
        if (!kfac_valid_factor_item(items[i], false)) return 0;
    return kfac_syrk_ws_bytes_impl(n, items);
}

int kfac_eig(kfac_ctx *ctx, int batch, const float *const *F, const int *d, float *const *Q,
             float *const *lam, const kfac_eig_opts *opts, kfac_eig_info *info) {
    if (!ctx || batch < 0 || (batch > 0 && (!F || !d || !Q || !lam))) return KFAC_EINVAL;
    for (int i = 0; i < batch; ++i) {
        if (d[i] < 1 || d[i] > KFAC_MAX_D || !F[i] || !Q[i] || !lam[i] || (const float *)Q[i] == F[i]) return KFAC_EINVAL;
    }
    if (opts && (opts->max_sweeps > 1000 || !(opts->tol < 1.f))) return KFAC_EINVAL;
    if (batch == 0) return KFAC_OK;
    return kfac_launch_eig(ctx, batch, F, d, Q, lam, opts, info);
}

int kfac_precondition(kfac_ctx *ctx, const float *QA, const float *lamA, int dA, const float *QG,
                      const float *lamG, int dG, float damping, void *grad, int grad_dtype) {
    if (!ctx || !QA || !lamA || !QG || !lamG || !grad) return KFAC_EINVAL;
    if (dA < 1 || dG < 1 || dA > KFAC_MAX_D || dG > KFAC_MAX_D) return KFAC_EINVAL;
    if (!(damping > 0.f) || !std::isfinite(damping) || !valid_dtype(grad_dtype)) return KFAC_EINVAL;
    return kfac_launch_precondition(ctx, QA, lamA, dA, QG, lamG, dG, damping, grad, grad_dtype);
}

int kfac_invert_factors(kfac_ctx *ctx, int batch, const float *const *F, const int *d, float damping, float *const *Finv) {
    if (!ctx || batch < 0 || (batch > 0 && (!F || !d || !Finv))) return KFAC_EINVAL;
    if (!(damping > 0.f) || !std::isfinite(damping)) return KFAC_EINVAL;
    for (int i = 0; i < batch; ++i)
        if (d[i] < 1 || d[i] > KFAC_MAX_D || !F[i] || !Finv[i] || (const float *)Finv[i] == F[i]) return KFAC_EINVAL;
    if (batch == 0) return KFAC_OK;
    return kfac_launch_invert_factors(ctx, batch, F, d, damping, Finv);
}

size_t kfac_invert_workspace_bytes(int batch, const int *d) {
    if (batch < 0 || (batch > 0 && !d)) return 0;
    for (int i = 0; i < batch; ++i)
        if (d[i] < 1 || d[i] > KFAC_MAX_D) return 0;
    return kfac_invert_ws_bytes_impl(batch, d);
}

static bool valid_inv_item(const kfac_precond_inv_item &it, bool pointers) {
    if (pointers && (!it.Ainv || !it.Ginv || !it.grad)) return false;
    return it.dA >= 1 && it.dG >= 1 && it.dA <= KFAC_MAX_D && it.dG <= KFAC_MAX_D && valid_dtype(it.grad_dtype);
}

int kfac_precondition_inverse_batched(kfac_ctx *ctx, int n, const kfac_precond_inv_item *items) {
    if (!ctx || n < 0 || (n > 0 && !items)) return KFAC_EINVAL;
    for (int i = 0; i < n; ++i)
        if (!valid_inv_item(items[i], true)) return KFAC_EINVAL;
    if (n == 0) return KFAC_OK;
    return kfac_launch_precondition_inverse_batched(ctx, n, items);
}

size_t kfac_precondition_inverse_workspace_bytes(int n, const kfac_precond_inv_item *items) {
    if (n < 0 || (n > 0 && !items)) return 0;
    for (int i = 0; i < n; ++i)
        if (!valid_inv_item(items[i], false)) return 0;
    return kfac_precondition_inverse_ws_bytes_impl(n, items);
}

int kfac_precondition_inverse(kfac_ctx *ctx, const float *Ainv, int dA, const float *Ginv, int dG, void *grad, int grad_dtype) {
    const kfac_precond_inv_item it{Ainv, dA, Ginv, dG, grad, grad_dtype};
    return kfac_precondition_inverse_batched(ctx, 1, &it);
}

int kfac_profile_begin(kfac_ctx *ctx) {
    if (!ctx) return KFAC_EINVAL;
    for (auto &r : ctx->prof) { ctx->ev_pool.push_back(r.t0); ctx->ev_pool.push_back(r.t1); }
    ctx->prof.clear();
    ctx->prof_on = true;
    return KFAC_OK;
}

int kfac_profile_end(kfac_ctx *ctx, kfac_kernel_stat *out, int max, int *n) {
    if (!ctx || !out || !n || max < 0) return KFAC_EINVAL;
    static const char *names[KC_COUNT] = {"unfold", "syrk", "syrk_reduce", "precond_gemm", "eig_small",
                                          "eig_pivot_solve", "eig_apply", "eig_misc", "eig_post_gemm", "eig_copy", "eig_outer_cols",
                                          "precond_scale", "syrk_bf16", "precond_gemm_split", "eig_outer_rows", "factor_inverse"};
    ctx->prof_on = false;
    KFAC_HIP_CHECK(hipStreamSynchronize(ctx->stream));
    kfac_kernel_stat acc[KC_COUNT] = {};
    for (auto &r : ctx->prof) {
        float ms = 0.f;
        KFAC_HIP_CHECK(hipEventElapsedTime(&ms, r.t0, r.t1));
        acc[r.cls].launches += 1;
        acc[r.cls].ms += ms;
        acc[r.cls].flops += r.flops;
        acc[r.cls].bytes += r.bytes;
        ctx->ev_pool.push_back(r.t0);
        ctx->ev_pool.push_back(r.t1);
    }
    ctx->prof.clear();
    int k = 0;
    for (int c = 0; c < KC_COUNT && k < max; ++c) {
        if (!acc[c].launches) continue;
        out[k] = acc[c];
        snprintf(out[k].name, sizeof(out[k].name), "%s", names[c]);
        ++k;
    }
    *n = k;
    return KFAC_OK;
}

static bool valid_precond_item(const kfac_precond_item &p) {
    if (!p.QA || !p.lamA || !p.QG || !p.lamG || !p.grad) return false;
    if (p.dA < 1 || p.dG < 1 || p.dA > KFAC_MAX_D || p.dG > KFAC_MAX_D) return false;
    return p.damping > 0.f && std::isfinite(p.damping) && valid_dtype(p.grad_dtype) && (p.factored_damping == 0 || p.factored_damping == 1) &&
           (p.split_f16 == 0 || p.split_f16 == 1);
}

int kfac_precondition_batched(kfac_ctx *ctx, int n, const kfac_precond_item *items) {
    if (!ctx || n < 0 || (n > 0 && !items)) return KFAC_EINVAL;
    for (int i = 0; i < n; ++i)
        if (!valid_precond_item(items[i])) return KFAC_EINVAL;
    if (n == 0) return KFAC_OK;
    return kfac_launch_precondition_batched(ctx, n, items, false, 0.f, 0.f, nullptr);
}

int kfac_precondition_batched_scaled(kfac_ctx *ctx, int n, const kfac_precond_item *items, float kappa, float lr, float *nu) {
    if (!ctx || n < 1 || !items || !nu) return KFAC_EINVAL;
    if (!(kappa > 0.f) || !std::isfinite(kappa) || !(lr > 0.f) || !std::isfinite(lr)) return KFAC_EINVAL;
    for (int i = 0; i < n; ++i)
        if (!valid_precond_item(items[i])) return KFAC_EINVAL;
    return kfac_launch_precondition_batched(ctx, n, items, true, kappa, lr, nu);
}

size_t kfac_precondition_workspace_bytes(int n, const kfac_precond_item *items) {
    if (n <= 0 || !items) return 0;
    for (int i = 0; i < n; ++i)
        if (items[i].dA < 1 || items[i].dG < 1 || items[i].dA > KFAC_MAX_D || items[i].dG > KFAC_MAX_D) return 0;
    return kfac_precond_ws_bytes_impl(n, items);
}

int kfac_schedule_due(int64_t k, int f_fac, int f_eig, int *do_factors, int *do_eig) {
    if (k < 0 || f_fac < 1 || f_eig < 1 || !do_factors || !do_eig) return KFAC_EINVAL;
    *do_factors = (k % f_fac) == 0;
    *do_eig = (k % f_eig) == 0;
    return KFAC_OK;
}

}  // extern "C"
