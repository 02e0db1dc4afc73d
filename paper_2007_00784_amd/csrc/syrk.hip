// Kronecker-factor update: F <- decay*F + (1-decay)*scale * Xt^T Xt  (Sec. II-C factors, Sec. IV-B
// running average).  The Gram matrix is a symmetric rank-R update on the fp32 MFMA engine: only the
// lower-triangular 128x128 tiles are computed and mirrored, the contraction over the sample rows is
// split across workgroups when there are few tiles, and the running average is applied where the
// final sum is formed (the SYRK epilogue, or the fixed-order split reducer).
#include "kfac_internal.h"
#include "mfma_gemm.h"

using namespace kfac;

namespace {

struct SyrkArgs {
    int D;            // factor dimension (d + append_ones)
    int ntile;        // tiles per edge
    int nsplit;       // workgroups along K per tile
    int kchunk;       // K rows per split (multiple of BK)
    int K;            // total sample rows
    float alpha;      // (1-decay)*scale
    float decay;
    float *F;
    float *partial;   // [nsplit][ntri][128][128] when nsplit > 1
};

__device__ inline void tri_decode(int idx, int &ti, int &tj) {
    // idx = ti*(ti+1)/2 + tj, tj <= ti
    int t = (int)((sqrtf(8.f * (float)idx + 1.f) - 1.f) * 0.5f);
    while ((t + 1) * (t + 2) / 2 <= idx) ++t;
    while (t * (t + 1) / 2 > idx) --t;
    ti = t;
    tj = idx - t * (t + 1) / 2;
}

__device__ inline void ema_store(float *F, int D, int r, int c, float v, float alpha, float decay, bool mirror) {
    const int64_t o = (int64_t)r * D + c;
    float out = alpha * v;
    if (decay != 0.f) out += decay * F[o];
    F[o] = out;
    if (mirror) F[(int64_t)c * D + r] = out;
}

template <class Op>
__global__ __launch_bounds__(NTHREADS) void syrk_kernel(Op opA, SyrkArgs g) {
    __shared__ TileSmem sm;
    int ti, tj;
    tri_decode(blockIdx.x, ti, tj);
    const int split = blockIdx.y;
    const int kbeg = split * g.kchunk;
    const int kend = min(g.K, kbeg + g.kchunk);
    Op a = opA, b = opA;
    a.K = kend;
    b.K = kend;
    floatx16 acc[2][2];
    gemm_tile(a, b, ti * BM, tj * BM, kbeg, kend, sm, acc);
    if (g.nsplit == 1) {
        const bool diag = ti == tj;
        for_each_acc(acc, [&](int r, int c, float v) {
            const int gr = ti * BM + r, gc = tj * BM + c;
            if (gr < g.D && gc < g.D && (!diag || gc <= gr))
                ema_store(g.F, g.D, gr, gc, v, g.alpha, g.decay, gr != gc);
        });
    } else {
        const int ntri = gridDim.x;
        float *dst = g.partial + ((int64_t)split * ntri + blockIdx.x) * (BM * BM);
        for_each_acc(acc, [&](int r, int c, float v) { dst[r * BM + c] = v; });
    }
}

// Sum the split partials of each tile in split order, then apply the running average and mirror.
// One thread per tile element (gridDim.y * 256 = 128 * 128); the loads of consecutive splits are
// independent, so they are issued eight at a time.
__global__ __launch_bounds__(256) void syrk_reduce_kernel(SyrkArgs g) {
    int ti, tj;
    tri_decode(blockIdx.x, ti, tj);
    const int ntri = gridDim.x;
    const bool diag = ti == tj;
    const int e = threadIdx.x + blockIdx.y * 256;
    const int r = e / BM, c = e % BM;
    const int gr = ti * BM + r, gc = tj * BM + c;
    if (gr >= g.D || gc >= g.D || (diag && gc > gr)) return;
    const float *src = g.partial + (int64_t)blockIdx.x * (BM * BM) + e;
    const int64_t stride = (int64_t)ntri * (BM * BM);
    float s = 0.f;
    int sp = 0;
    for (; sp + 8 <= g.nsplit; sp += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[(sp + u) * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; sp < g.nsplit; ++sp) s += src[sp * stride];
    ema_store(g.F, g.D, gr, gc, s, g.alpha, g.decay, gr != gc);
}

void plan(int D, int64_t R, int &ntile, int &ntri, int &nsplit, int &kchunk) {
    ntile = (D + BM - 1) / BM;
    ntri = ntile * (ntile + 1) / 2;
    int want = (256 + ntri - 1) / ntri;                 // aim at one workgroup per compute unit
    int64_t maxsplit = R / 256 > 0 ? R / 256 : 1;       // keep >= 256 rows per split
    nsplit = (int)(want < maxsplit ? want : maxsplit);
    if (nsplit < 1) nsplit = 1;
    int64_t chunk = (R + nsplit - 1) / nsplit;
    chunk = (chunk + BK - 1) / BK * BK;
    kchunk = (int)chunk;
    nsplit = (int)((R + chunk - 1) / chunk);
}

}  // namespace

size_t kfac_syrk_workspace_bytes(int D, int64_t R) {
    int ntile, ntri, nsplit, kchunk;
    plan(D, R, ntile, ntri, nsplit, kchunk);
    return nsplit > 1 ? (size_t)nsplit * ntri * BM * BM * sizeof(float) : 0;
}

int kfac_launch_update_factors(kfac_ctx *ctx, const void *X, int dtype, int layout, int N, int d, int T,
                               int append_ones, float scale, float decay, float *F) {
    const int64_t R = (int64_t)N * T;
    const int D = d + (append_ones ? 1 : 0);
    SyrkArgs g;
    int ntile, ntri;
    plan(D, R, ntile, ntri, g.nsplit, g.kchunk);
    g.ntile = ntile;
    g.D = D;
    g.K = (int)R;
    g.alpha = (1.f - decay) * scale;
    g.decay = decay;
    g.F = F;
    g.partial = (float *)ctx->ws;
    if (g.nsplit > 1 && (size_t)g.nsplit * ntri * BM * BM * sizeof(float) > ctx->ws_bytes) return KFAC_EWORKSPACE;
    const dim3 grid(ntri, g.nsplit), block(NTHREADS);
    const int ones_i = append_ones ? d : -1;
    const double esz = dtype == KFAC_F32 ? 4.0 : 2.0;
    {
    // useful flops of the symmetric update R*D*(D+1); bytes: the samples once, F read (if averaged) and written
    KfacProfScope prof(ctx, KC_SYRK, (double)R * D * (D + 1.0),
                       esz * (double)R * d + (g.nsplit == 1 ? (decay != 0.f ? 8.0 : 4.0) * D * D : 0.0));
    if (layout == KFAC_LAYOUT_NDT && T > 1) {
        if (dtype == KFAC_F32) {
            OpNDT<float> op{(const float *)X, d, T, 0, ones_i};
            hipLaunchKernelGGL(syrk_kernel<OpNDT<float>>, grid, block, 0, ctx->stream, op, g);
        } else {
            OpNDT<unsigned short> op{(const unsigned short *)X, d, T, 0, ones_i};
            hipLaunchKernelGGL(syrk_kernel<OpNDT<unsigned short>>, grid, block, 0, ctx->stream, op, g);
        }
    } else {
        // [R][d]: feature index contiguous, sample index strided by d
        if (dtype == KFAC_F32) {
            OpStrided<float, false> op{(const float *)X, 1, d, d, 0, ones_i};
            hipLaunchKernelGGL((syrk_kernel<OpStrided<float, false>>), grid, block, 0, ctx->stream, op, g);
        } else {
            OpStrided<unsigned short, false> op{(const unsigned short *)X, 1, d, d, 0, ones_i};
            hipLaunchKernelGGL((syrk_kernel<OpStrided<unsigned short, false>>), grid, block, 0, ctx->stream, op, g);
        }
    }
    }
    KFAC_HIP_CHECK(hipGetLastError());
    if (g.nsplit > 1) {
        KfacProfScope prof(ctx, KC_SYRK_REDUCE, 0.0, (decay != 0.f ? 8.0 : 4.0) * D * D);
        hipLaunchKernelGGL(syrk_reduce_kernel, dim3(ntri, BM * BM / 256), dim3(256), 0, ctx->stream, g);
        KFAC_HIP_CHECK(hipGetLastError());
    }
    return KFAC_OK;
}
