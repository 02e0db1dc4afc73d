// Eigenbasis preconditioning, Eqs. (v1), (v2), (kfac-eigen) of Sec. IV-A, for one layer or a batch of
// layers:
//   T  = QG^T grad            (dG x dA, K = dG)
//   V2 = (T QA) / (lamG lamA^T + damping)     (K = dA, divide fused into the epilogue)
//   T  = QG V2                (K = dG)
//   grad = T QA^T             (K = dA)
// and optionally the gradient scaling of Sec. V-C on top: nu = min(1, sqrt(kappa / (lr^2 sum_l |<P_l, grad_l>|))),
// P_l the preconditioned and grad_l the original gradient of layer l, every P_l multiplied by nu.  The inner
// products cost no extra pass: the last stage overwrites grad element by element, so its epilogue reads the
// old value just before it stores the new one.
// Four dependent GEMM stages on the fp32 MFMA tile engine, or (per layer, on request) on the split-fp16 engine.  Each stage is ONE launch over the 128x128
// output tiles of every layer in the batch (a device table maps a workgroup to its layer and tile,
// longest contraction first), so small layers do not leave the machine idle and a 54-layer network
// costs four launches instead of 216.  T and V2 live in the context workspace.
#include <algorithm>
#include <vector>
#include "kfac_internal.h"
#include "mfma_gemm.h"
#include "mfma_gemm_x3.h"

using namespace kfac;

namespace {

struct LayerDev {
    const float *QA, *lamA, *QG, *lamG;
    void *grad;
    float *T, *V;
    int dA, dG;
    float damping;
    int grad_bf16;
    int tile_base;     // index of this layer's first tile in the per-tile inner-product array
    int factored;      // denominator (lamG + damping)(lamA + damping) instead of lamG lamA + damping
    int split;         // GEMM chain on the split-fp16 engine
    double *gnorm;     // split: NORM_PARTS partial sums of grad^2 (written by precond_norm_kernel)
    double *vnorm;     // split: per-tile partial sums of V2^2 (written by stage 1)
};
struct TileRef { int layer, tile; };   // tile = ti * tiles_n + tj

__device__ inline unsigned short f32_to_bf16_rne(float v) {
    unsigned u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

template <class OpA, class OpB, class Epi>
__device__ inline void run_tile(OpA a, OpB b, int i0, int j0, int K, int M, int N, TileSmem &sm, Epi epi) {
    gemm_tile_ragged(a, b, i0, j0, K, M, N, sm, epi);
}

template <int STAGE>
__global__ __launch_bounds__(NTHREADS) __attribute__((amdgpu_waves_per_eu(2))) void precond_stage_kernel(const LayerDev *layers, const TileRef *tiles,
                                                                                                       double *dots) {
    __shared__ TileSmem sm;
    const TileRef tr = tiles[blockIdx.x];
    const LayerDev L = layers[tr.layer];
    if (L.split) return;
    const int dA = L.dA, dG = L.dG;
    const int tn = (dA + BM - 1) / BM;
    const int i0 = (tr.tile / tn) * BM, j0 = (tr.tile % tn) * BM;
    if (STAGE == 0) {
        // T = QG^T grad : A(m,k) = QG[k][m] (m contiguous), B(k,n) = grad[k][n] (n contiguous)
        OpStrided<float, false> qgt{L.QG, 1, dG, dG, dG, -1};
        float *T = L.T;
        auto epi = [=](int r, int c, float v) { T[(int64_t)r * dA + c] = v; };
        if (L.grad_bf16) {
            OpStrided<unsigned short, false> g{(const unsigned short *)L.grad, 1, dA, dA, dG, -1};
            run_tile(qgt, g, i0, j0, dG, dG, dA, sm, epi);
        } else {
            OpStrided<float, false> g{(const float *)L.grad, 1, dA, dA, dG, -1};
            run_tile(qgt, g, i0, j0, dG, dG, dA, sm, epi);
        }
    } else if (STAGE == 1) {
        // V = (T QA) / (lamG lamA^T + damping) : A(m,k) = T[m][k] (k contiguous), B(k,n) = QA[k][n]
        OpStrided<float, true> t_mk{L.T, dA, 1, dG, dA, -1};
        OpStrided<float, false> qa_kn{L.QA, 1, dA, dA, dA, -1};
        float *V = L.V;
        const float *lamG = L.lamG, *lamA = L.lamA;
        const float damping = L.damping;
        const bool factored = L.factored != 0;
        run_tile(t_mk, qa_kn, i0, j0, dA, dG, dA, sm, [=](int r, int c, float v) {
            const float lg = fmaxf(lamG[r], 0.f), la = fmaxf(lamA[c], 0.f);
            V[(int64_t)r * dA + c] = v / (factored ? (lg + damping) * (la + damping) : lg * la + damping);
        });
    } else if (STAGE == 2) {
        // T = QG V : A(m,k) = QG[m][k] (k contiguous), B(k,n) = V[k][n]
        OpStrided<float, true> qg_mk{L.QG, dG, 1, dG, dG, -1};
        OpStrided<float, false> v_kn{L.V, 1, dA, dA, dG, -1};
        float *T = L.T;
        run_tile(qg_mk, v_kn, i0, j0, dG, dG, dA, sm, [=](int r, int c, float v) { T[(int64_t)r * dA + c] = v; });
    } else {
        // grad = T QA^T : A(m,k) = T[m][k], B(k,n) = QA[n][k] (k contiguous)
        OpStrided<float, true> t_mk{L.T, dA, 1, dG, dA, -1};
        OpStrided<float, true> qa_nk{L.QA, dA, 1, dA, dA, -1};
        // dot: this thread's share of <new grad, old grad> (the values as stored, i.e. after bf16 rounding)
        void *grad = L.grad;
        float dot = 0.f;
        if (L.grad_bf16)
            run_tile(t_mk, qa_nk, i0, j0, dA, dG, dA, sm, [&](int r, int c, float v) {
                unsigned short *p = (unsigned short *)grad + (int64_t)r * dA + c;
                const unsigned short nv = f32_to_bf16_rne(v);
                dot = fmaf(to_float(nv), to_float(*p), dot);
                *p = nv;
            });
        else
            run_tile(t_mk, qa_nk, i0, j0, dA, dG, dA, sm, [&](int r, int c, float v) {
                float *p = (float *)grad + (int64_t)r * dA + c;
                dot = fmaf(v, *p, dot);
                *p = v;
            });
        if (dots) {   // fixed-order sum over the workgroup, one double per tile
            __shared__ double red[NTHREADS];
            red[threadIdx.x] = (double)dot;
            __syncthreads();
            if (threadIdx.x == 0) {
                double t = 0.0;
                for (int i = 0; i < NTHREADS; ++i) t += red[i];
                dots[L.tile_base + tr.tile] = t;
            }
        }
    }
}

// ---- the same chain on the split-fp16 engine (three fp16 MFMA products per fp32 product, 22 significand bits) ----
// Operands are scaled by powers of two into fp16's range: eigenvector matrices (entries <= 1) by 2^14, the
// gradient-like operand of a stage by the power of two that puts its Frobenius norm (an upper bound of every
// entry) in [2^12, 2^13).  Multiplying by an orthogonal matrix keeps the Frobenius norm, so stages 0 and 1 share the
// scale of the incoming gradient and stages 2 and 3 that of V2, whose squares stage 1 sums in its epilogue.
constexpr int NORM_PARTS = 128;
constexpr float X3_QSCALE = 16384.f;

__global__ __launch_bounds__(256) void precond_norm_kernel(const LayerDev *layers) {
    const LayerDev L = layers[blockIdx.y];
    if (!L.split) return;
    const int64_t count = (int64_t)L.dG * L.dA;
    double acc = 0.0;
    for (int64_t e = blockIdx.x * 256 + threadIdx.x; e < count; e += (int64_t)NORM_PARTS * 256) {
        const float v = L.grad_bf16 ? to_float(((const unsigned short *)L.grad)[e]) : ((const float *)L.grad)[e];
        acc += (double)v * v;
    }
    __shared__ double red[256];
    red[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int i = 0; i < 256; ++i) t += red[i];
        L.gnorm[blockIdx.x] = t;
    }
}

// Power-of-two scale for an operand whose squared Frobenius norm is the sum of `parts` (every thread of the
// workgroup returns the same value).
__device__ inline float split_scale(const double *parts, int n) {
    __shared__ double red[NTHREADS];
    double t = 0.0;
    for (int i = threadIdx.x; i < n; i += NTHREADS) t += parts[i];
    red[threadIdx.x] = t;
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = 0.0;
        for (int i = 0; i < NTHREADS; ++i) s += red[i];
        red[0] = s;
    }
    __syncthreads();
    const double n2 = red[0];
    __syncthreads();
    if (!(n2 > 0.0) || !(n2 < 1e300)) return 1.f;
    const int e = ilogb(sqrt(n2));            // norm in [2^e, 2^(e+1))
    return ldexpf(1.f, min(max(12 - e, -100), 100));
}

template <class OpA, class OpB, class Epi>
__device__ inline void run_tile_x3(OpA a, OpB b, int i0, int j0, int K, int M, int N, float out_scale, X3Smem &sm, Epi epi) {
    floatx16 acc[2][2];
    a.start(threadIdx.x, i0);
    b.start(threadIdx.x, j0);
    gemm_tile_x3(a, b, K, sm, acc);
    for_each_acc(acc, [&](int r, int c, float v) {
        const int gr = i0 + r, gc = j0 + c;
        if (gr < M && gc < N) epi(gr, gc, v * out_scale);
    });
}

template <int STAGE>
__global__ __launch_bounds__(NTHREADS) __attribute__((amdgpu_waves_per_eu(2))) void precond_stage_x3_kernel(const LayerDev *layers, const TileRef *tiles,
                                                                                                          double *dots) {
    __shared__ X3Smem sm;
    const TileRef tr = tiles[blockIdx.x];
    const LayerDev L = layers[tr.layer];
    if (!L.split) return;
    const int dA = L.dA, dG = L.dG;
    const int tn = (dA + BM - 1) / BM;
    const int ntile = ((dG + BM - 1) / BM) * tn;
    const int i0 = (tr.tile / tn) * BM, j0 = (tr.tile % tn) * BM;
    const float s = STAGE < 2 ? split_scale(L.gnorm, NORM_PARTS) : split_scale(L.vnorm, ntile);
    const float out_scale = 1.f / (s * X3_QSCALE);
    if (STAGE == 0) {
        X3OpG<float, false> qgt{L.QG, dG, X3_QSCALE, dG, dG};                  // elem(m,k) = QG[k][m]
        float *T = L.T;
        auto epi = [=](int r, int c, float v) { T[(int64_t)r * dA + c] = v; };
        if (L.grad_bf16) {
            X3OpG<unsigned short, false> g{(const unsigned short *)L.grad, dA, s, dA, dG};   // elem(n,k) = grad[k][n]
            run_tile_x3(qgt, g, i0, j0, dG, dG, dA, out_scale, sm, epi);
        } else {
            X3OpG<float, false> g{(const float *)L.grad, dA, s, dA, dG};
            run_tile_x3(qgt, g, i0, j0, dG, dG, dA, out_scale, sm, epi);
        }
    } else if (STAGE == 1) {
        X3OpG<float, true> t_mk{L.T, dA, s, dG, dA};                           // elem(m,k) = T[m][k]
        X3OpG<float, false> qa_kn{L.QA, dA, X3_QSCALE, dA, dA};                // elem(n,k) = QA[k][n]
        float *V = L.V;
        const float *lamG = L.lamG, *lamA = L.lamA;
        const float damping = L.damping;
        const bool factored = L.factored != 0;
        float sq = 0.f;
        run_tile_x3(t_mk, qa_kn, i0, j0, dA, dG, dA, out_scale, sm, [&](int r, int c, float v) {
            const float lg = fmaxf(lamG[r], 0.f), la = fmaxf(lamA[c], 0.f);
            const float q = v / (factored ? (lg + damping) * (la + damping) : lg * la + damping);
            V[(int64_t)r * dA + c] = q;
            sq = fmaf(q, q, sq);
        });
        __shared__ double red[NTHREADS];
        red[threadIdx.x] = (double)sq;
        __syncthreads();
        if (threadIdx.x == 0) {
            double t = 0.0;
            for (int i = 0; i < NTHREADS; ++i) t += red[i];
            L.vnorm[tr.tile] = t;
        }
    } else if (STAGE == 2) {
        X3OpG<float, true> qg_mk{L.QG, dG, X3_QSCALE, dG, dG};                 // elem(m,k) = QG[m][k]
        X3OpG<float, false> v_kn{L.V, dA, s, dA, dG};                          // elem(n,k) = V[k][n]
        float *T = L.T;
        run_tile_x3(qg_mk, v_kn, i0, j0, dG, dG, dA, out_scale, sm, [=](int r, int c, float v) { T[(int64_t)r * dA + c] = v; });
    } else {
        X3OpG<float, true> t_mk{L.T, dA, s, dG, dA};                           // elem(m,k) = T[m][k]
        X3OpG<float, true> qa_nk{L.QA, dA, X3_QSCALE, dA, dA};                 // elem(n,k) = QA[n][k]
        void *grad = L.grad;
        float dot = 0.f;
        if (L.grad_bf16)
            run_tile_x3(t_mk, qa_nk, i0, j0, dA, dG, dA, out_scale, sm, [&](int r, int c, float v) {
                unsigned short *p = (unsigned short *)grad + (int64_t)r * dA + c;
                const unsigned short nv = f32_to_bf16_rne(v);
                dot = fmaf(to_float(nv), to_float(*p), dot);
                *p = nv;
            });
        else
            run_tile_x3(t_mk, qa_nk, i0, j0, dA, dG, dA, out_scale, sm, [&](int r, int c, float v) {
                float *p = (float *)grad + (int64_t)r * dA + c;
                dot = fmaf(v, *p, dot);
                *p = v;
            });
        if (dots) {
            __shared__ double red[NTHREADS];
            red[threadIdx.x] = (double)dot;
            __syncthreads();
            if (threadIdx.x == 0) {
                double t = 0.0;
                for (int i = 0; i < NTHREADS; ++i) t += red[i];
                dots[L.tile_base + tr.tile] = t;
            }
        }
    }
}

// nu from the per-tile inner products (layer sums and the sum over layers in fixed order), one thread.
__global__ void precond_nu_kernel(const LayerDev *layers, int n, const double *dots, float kappa, float lr, float *nu) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    double total = 0.0;
    for (int l = 0; l < n; ++l) {
        const int nt = ((layers[l].dG + BM - 1) / BM) * ((layers[l].dA + BM - 1) / BM);
        double d = 0.0;
        for (int t = 0; t < nt; ++t) d += dots[layers[l].tile_base + t];
        total += fabs(d);
    }
    double v = 1.0;
    if (total > 0.0) v = fmin(1.0, sqrt((double)kappa / ((double)lr * lr * total)));
    *nu = (float)v;
}

// grad_l <- nu grad_l for every layer (blockIdx.y); nothing to do when nu = 1.
__global__ __launch_bounds__(256) void precond_scale_kernel(const LayerDev *layers, const float *nu) {
    const float v = *nu;
    if (v == 1.f) return;
    const LayerDev L = layers[blockIdx.y];
    const int64_t count = (int64_t)L.dG * L.dA;
    for (int64_t e = blockIdx.x * 256 + threadIdx.x; e < count; e += (int64_t)gridDim.x * 256) {
        if (L.grad_bf16) {
            unsigned short *p = (unsigned short *)L.grad + e;
            *p = f32_to_bf16_rne(v * to_float(*p));
        } else {
            float *p = (float *)L.grad + e;
            *p = v * *p;
        }
    }
}

size_t layout(int n, const kfac_precond_item *it, size_t &off_tiles, size_t &off_tv, size_t &ntiles) {
    ntiles = 0;
    size_t tv = 0;
    for (int i = 0; i < n; ++i) {
        ntiles += (size_t)((it[i].dG + BM - 1) / BM) * ((it[i].dA + BM - 1) / BM);
        tv += 2 * kfac_align_up((size_t)it[i].dG * it[i].dA, 64);
    }
    off_tiles = kfac_align_up((size_t)n * sizeof(LayerDev), 256);
    // tile tables (two orders), per-tile inner products, per-tile V2 norms, per-layer gradient norm partials
    off_tv = off_tiles + kfac_align_up(2 * ntiles * sizeof(TileRef), 256) + 2 * kfac_align_up(ntiles * sizeof(double), 256) +
             kfac_align_up((size_t)n * NORM_PARTS * sizeof(double), 256);
    return off_tv + tv * sizeof(float);
}

}  // namespace

size_t kfac_precond_ws_bytes_impl(int n, const kfac_precond_item *items) {
    size_t a, b, c;
    return layout(n, items, a, b, c);
}

int kfac_launch_precondition_batched(kfac_ctx *ctx, int n, const kfac_precond_item *items, bool scaled, float kappa, float lr,
                                     float *nu) {
    size_t off_tiles, off_tv, ntiles;
    const size_t need = layout(n, items, off_tiles, off_tv, ntiles);
    if (need > ctx->ws_bytes) return KFAC_EWORKSPACE;
    std::vector<LayerDev> dev(n);
    float *tv = (float *)(ctx->ws + off_tv);
    const size_t off_dots = off_tiles + kfac_align_up(2 * ntiles * sizeof(TileRef), 256);
    double *d_vnorm = (double *)(ctx->ws + off_dots + kfac_align_up(ntiles * sizeof(double), 256));
    double *d_gnorm = (double *)(ctx->ws + off_dots + 2 * kfac_align_up(ntiles * sizeof(double), 256));
    bool any_split = false, any_plain = false;
    double flops = 0.0, bytes = 0.0;
    int tile_base = 0;
    for (int i = 0; i < n; ++i) {
        const kfac_precond_item &p = items[i];
        const size_t e = kfac_align_up((size_t)p.dG * p.dA, 64);
        dev[i] = LayerDev{p.QA, p.lamA, p.QG, p.lamG, p.grad, tv, tv + e, p.dA, p.dG, p.damping, p.grad_dtype == KFAC_BF16, tile_base, p.factored_damping,
                          p.split_f16, d_gnorm + (size_t)i * NORM_PARTS, d_vnorm + tile_base};
        (p.split_f16 ? any_split : any_plain) = true;
        tile_base += ((p.dG + BM - 1) / BM) * ((p.dA + BM - 1) / BM);
        tv += 2 * e;
        flops += 4.0 * p.dA * p.dG * ((double)p.dA + p.dG);
        bytes += 4.0 * ((double)p.dA * p.dA + (double)p.dG * p.dG) * 2 + 4.0 * 8 * p.dA * p.dG;
    }
    // tile lists, longest contraction first: stages 0 and 2 contract over dG, stages 1 and 3 over dA
    std::vector<TileRef> byG, byA;
    byG.reserve(ntiles);
    for (int i = 0; i < n; ++i) {
        const int nt = ((items[i].dG + BM - 1) / BM) * ((items[i].dA + BM - 1) / BM);
        for (int t = 0; t < nt; ++t) byG.push_back(TileRef{i, t});
    }
    byA = byG;
    std::stable_sort(byG.begin(), byG.end(), [&](const TileRef &a, const TileRef &b) { return items[a.layer].dG > items[b.layer].dG; });
    std::stable_sort(byA.begin(), byA.end(), [&](const TileRef &a, const TileRef &b) { return items[a.layer].dA > items[b.layer].dA; });
    LayerDev *d_layers = (LayerDev *)ctx->ws;
    TileRef *d_byG = (TileRef *)(ctx->ws + off_tiles), *d_byA = d_byG + ntiles;
    double *d_dots = scaled ? (double *)(ctx->ws + off_dots) : nullptr;
    KFAC_CHECK(kfac_upload(ctx, d_layers, dev.data(), n * sizeof(LayerDev)));
    KFAC_CHECK(kfac_upload(ctx, d_byG, byG.data(), ntiles * sizeof(TileRef)));
    KFAC_CHECK(kfac_upload(ctx, d_byA, byA.data(), ntiles * sizeof(TileRef)));
    const dim3 grid((unsigned)ntiles), block(NTHREADS);
    if (any_split) {
        KfacProfScope prof(ctx, KC_PRECOND_SCALE, 0.0, bytes / 16);   // one read of every gradient
        hipLaunchKernelGGL(precond_norm_kernel, dim3(NORM_PARTS, n), dim3(256), 0, ctx->stream, d_layers);
    }
    // every stage kernel runs over all tiles; a workgroup whose layer uses the other engine returns at once
    for (int stage = 0; stage < 4; ++stage) {
        const TileRef *order = (stage & 1) ? d_byA : d_byG;
        double *dots = stage == 3 ? d_dots : nullptr;
        if (any_plain) {
            KfacProfScope prof(ctx, KC_PRECOND_GEMM, any_split ? 0.0 : flops / 4, any_split ? 0.0 : bytes / 4);
            switch (stage) {
                case 0: hipLaunchKernelGGL(precond_stage_kernel<0>, grid, block, 0, ctx->stream, d_layers, order, dots); break;
                case 1: hipLaunchKernelGGL(precond_stage_kernel<1>, grid, block, 0, ctx->stream, d_layers, order, dots); break;
                case 2: hipLaunchKernelGGL(precond_stage_kernel<2>, grid, block, 0, ctx->stream, d_layers, order, dots); break;
                default: hipLaunchKernelGGL(precond_stage_kernel<3>, grid, block, 0, ctx->stream, d_layers, order, dots); break;
            }
        }
        if (any_split) {
            KfacProfScope prof(ctx, KC_PRECOND_GEMM_X3, flops / 4, bytes / 4);
            switch (stage) {
                case 0: hipLaunchKernelGGL(precond_stage_x3_kernel<0>, grid, block, 0, ctx->stream, d_layers, order, dots); break;
                case 1: hipLaunchKernelGGL(precond_stage_x3_kernel<1>, grid, block, 0, ctx->stream, d_layers, order, dots); break;
                case 2: hipLaunchKernelGGL(precond_stage_x3_kernel<2>, grid, block, 0, ctx->stream, d_layers, order, dots); break;
                default: hipLaunchKernelGGL(precond_stage_x3_kernel<3>, grid, block, 0, ctx->stream, d_layers, order, dots); break;
            }
        }
    }
    if (scaled) {
        double total = 0.0;
        for (int i = 0; i < n; ++i) total += (double)items[i].dG * items[i].dA;
        KfacProfScope prof(ctx, KC_PRECOND_SCALE, 0.0, 8.0 * total);   // read + write of every gradient (when nu < 1)
        hipLaunchKernelGGL(precond_nu_kernel, dim3(1), dim3(64), 0, ctx->stream, d_layers, n, d_dots, kappa, lr, nu);
        hipLaunchKernelGGL(precond_scale_kernel, dim3(64, n), dim3(256), 0, ctx->stream, d_layers, nu);
    }
    KFAC_HIP_CHECK(hipGetLastError());
    return KFAC_OK;
}

int kfac_launch_precondition(kfac_ctx *ctx, const float *QA, const float *lamA, int dA, const float *QG,
                             const float *lamG, int dG, float damping, void *grad, int grad_dtype) {
    kfac_precond_item it{QA, lamA, dA, QG, lamG, dG, damping, grad, grad_dtype, 0, 0};
    return kfac_launch_precondition_batched(ctx, 1, &it, false, 0.f, 0.f, nullptr);
}
