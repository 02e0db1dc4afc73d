// Kronecker-factor update: F <- decay*F + (1-decay)*scale * Xt^T Xt  (Sec. II-C factors, Sec. IV-B
// running average).  The Gram matrix is a symmetric rank-R update on the fp32 MFMA engine: only the
// lower-triangular 128x128 tiles of X^T X are computed and mirrored, the contraction over the sample
// rows is split across workgroups when there are few tiles, and the running average is applied where
// the final sum is formed (the SYRK epilogue, or the fixed-order split reducer).
//
// The appended ones column is not materialised and costs no MFMA tile: its row of the factor is the
// vector of column sums of X, which every diagonal tile accumulates for its own 128 columns from the
// operand elements it loads anyway; the corner entry is scale * R.
#include <cmath>
#include "kfac_internal.h"
#include "mfma_gemm.h"

using namespace kfac;

namespace {

constexpr int PART = BM * BM + BM;   // floats per split partial: the tile, then 128 column sums

struct SyrkArgs {
    int d;            // features (tile grid covers d x d)
    int D;            // factor dimension (d + append_ones), leading dimension of F
    int ones;         // 1: also produce the bias row/column
    int nsplit;       // workgroups along K per tile
    int kchunk;       // K rows per split (multiple of BK)
    int K;            // total sample rows
    float alpha;      // (1-decay)*scale
    float decay;
    float *F;
    float *partial;   // [nsplit][ntri][PART] when nsplit > 1
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

// Fixed-order reduction of the per-thread column sums of a diagonal tile into cs[0..127] (LDS).
template <bool KFAST>
__device__ inline void reduce_colsum(const float (&csum)[EPT], float *scratch /* >= 128*16 floats */, float *cs) {
    const int tid = threadIdx.x;
    __syncthreads();
    if (KFAST) {   // slot s holds column (tid>>4)+16s; the 16 threads tid&15 share it
#pragma unroll
        for (int s = 0; s < EPT; ++s) scratch[((tid >> 4) + 16 * s) * 16 + (tid & 15)] = csum[s];
    } else {       // every slot is column tid&127; two threads (tid>>7) share it
        float t = 0.f;
#pragma unroll
        for (int s = 0; s < EPT; ++s) t += csum[s];
        scratch[(tid & 127) * 16 + (tid >> 7)] = t;
    }
    __syncthreads();
    if (tid < BM) {
        float t = 0.f;
        const int n = KFAST ? 16 : 2;
        for (int u = 0; u < n; ++u) t += scratch[tid * 16 + u];
        cs[tid] = t;
    }
    __syncthreads();
}

template <class Op>
__global__ __launch_bounds__(NTHREADS) __attribute__((amdgpu_waves_per_eu(2))) void syrk_kernel(Op opA, SyrkArgs g) {
    __shared__ TileSmem sm;
    __shared__ float cs[BM];
    int ti, tj;
    tri_decode(blockIdx.x, ti, tj);
    const int split = blockIdx.y;
    const int kbeg = split * g.kchunk;
    const int kend = min(g.K, kbeg + g.kchunk);
    const bool diag = ti == tj;
    const bool want_cs = diag && g.ones;
    Op a = opA, b = opA;
    a.K = kend;
    b.K = kend;
    floatx16 acc[2][2];
    float csum[EPT];
#pragma unroll
    for (int s = 0; s < EPT; ++s) csum[s] = 0.f;
    if (want_cs) {
        gemm_tile<Op, Op, true>(a, b, ti * BM, tj * BM, kbeg, kend, sm, acc, csum);
        reduce_colsum<Op::KFAST>(csum, &sm.a[0][0][0], cs);
    } else {
        gemm_tile<Op, Op, false>(a, b, ti * BM, tj * BM, kbeg, kend, sm, acc);
    }
    if (g.nsplit == 1) {
        for_each_acc(acc, [&](int r, int c, float v) {
            const int gr = ti * BM + r, gc = tj * BM + c;
            if (gr < g.d && gc < g.d && (!diag || gc <= gr))
                ema_store(g.F, g.D, gr, gc, v, g.alpha, g.decay, gr != gc);
        });
        if (want_cs) {
            const int gc = ti * BM + threadIdx.x;
            if (threadIdx.x < BM && gc < g.d) ema_store(g.F, g.D, g.d, gc, cs[threadIdx.x], g.alpha, g.decay, true);
            if (blockIdx.x == 0 && threadIdx.x == 0) ema_store(g.F, g.D, g.d, g.d, (float)g.K, g.alpha, g.decay, false);
        }
    } else {
        const int ntri = gridDim.x;
        float *dst = g.partial + ((int64_t)split * ntri + blockIdx.x) * PART;
        for_each_acc(acc, [&](int r, int c, float v) { dst[r * BM + c] = v; });
        if (want_cs && threadIdx.x < BM) dst[BM * BM + threadIdx.x] = cs[threadIdx.x];
    }
}

// Sum the split partials of each tile in split order, then apply the running average and mirror.
// One thread per tile element (plus 128 for the column sums of diagonal tiles); the loads of
// consecutive splits are independent, so they are issued eight at a time.
__global__ __launch_bounds__(256) void syrk_reduce_kernel(SyrkArgs g) {
    int ti, tj;
    tri_decode(blockIdx.x, ti, tj);
    const int ntri = gridDim.x;
    const bool diag = ti == tj;
    const int e = threadIdx.x + blockIdx.y * 256;          // 0 .. PART-1 (grid covers PART rounded up)
    if (e >= PART) return;
    int gr, gc;
    bool mirror;
    if (e < BM * BM) {
        gr = ti * BM + e / BM;
        gc = tj * BM + e % BM;
        if (gr >= g.d || gc >= g.d || (diag && gc > gr)) return;
        mirror = gr != gc;
    } else {
        if (!diag || !g.ones) return;
        gr = g.d;
        gc = ti * BM + (e - BM * BM);
        if (gc >= g.d) return;
        mirror = true;
    }
    const float *src = g.partial + (int64_t)blockIdx.x * PART + e;
    const int64_t stride = (int64_t)ntri * PART;
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
    ema_store(g.F, g.D, gr, gc, s, g.alpha, g.decay, mirror);
    if (g.ones && blockIdx.x == 0 && e == 0) ema_store(g.F, g.D, g.d, g.d, (float)g.K, g.alpha, g.decay, false);
}

// Choose the number of K splits.  Two workgroups share a compute unit (register budget), so the
// machine has 512 slots; a launch takes ceil(workgroups / 512) rounds of (slabs per split + a fixed
// per-workgroup cost of about 12 slabs for prologue, epilogue and partial traffic).
void plan(int d, int64_t R, int &ntile, int &ntri, int &nsplit, int &kchunk) {
    ntile = (d + BM - 1) / BM;
    ntri = ntile * (ntile + 1) / 2;
    const int64_t slabs = (R + BK - 1) / BK;
    int best = 1;
    double best_cost = 1e300;
    for (int ns = 1; ns <= 512; ++ns) {
        if (ns > 1 && slabs / ns < 8) break;                 // keep >= 128 rows per split
        const double rounds = std::ceil((double)ntri * ns / 512.0);
        const double cost = rounds * ((double)((slabs + ns - 1) / ns) + 12.0);
        if (cost < best_cost * 0.999) { best_cost = cost; best = ns; }
    }
    nsplit = best;
    int64_t chunk = (R + nsplit - 1) / nsplit;
    chunk = (chunk + BK - 1) / BK * BK;
    kchunk = (int)chunk;
    nsplit = (int)((R + chunk - 1) / chunk);
}

}  // namespace

size_t kfac_syrk_workspace_bytes(int D, int64_t R) {
    int ntile, ntri, nsplit, kchunk;
    plan(D, R, ntile, ntri, nsplit, kchunk);
    return nsplit > 1 ? (size_t)nsplit * ntri * PART * sizeof(float) : 0;
}

int kfac_launch_update_factors(kfac_ctx *ctx, const void *X, int dtype, int layout, int N, int d, int T,
                               int append_ones, float scale, float decay, float *F) {
    const int64_t R = (int64_t)N * T;
    SyrkArgs g;
    int ntile, ntri;
    plan(d, R, ntile, ntri, g.nsplit, g.kchunk);
    g.d = d;
    g.D = d + (append_ones ? 1 : 0);
    g.ones = append_ones ? 1 : 0;
    g.K = (int)R;
    g.alpha = (1.f - decay) * scale;
    g.decay = decay;
    g.F = F;
    g.partial = (float *)ctx->ws;
    if (g.nsplit > 1 && (size_t)g.nsplit * ntri * PART * sizeof(float) > ctx->ws_bytes) return KFAC_EWORKSPACE;
    const dim3 grid(ntri, g.nsplit), block(NTHREADS);
    const double esz = dtype == KFAC_F32 ? 4.0 : 2.0;
    const double D = g.D;
    {
        // useful flops of the symmetric update R*D*(D+1); bytes: the samples once, F read (if averaged) and written
        KfacProfScope prof(ctx, KC_SYRK, (double)R * D * (D + 1.0),
                           esz * (double)R * d + (g.nsplit == 1 ? (decay != 0.f ? 8.0 : 4.0) * D * D : 0.0));
        if (layout == KFAC_LAYOUT_NDT && T > 1) {
            if (dtype == KFAC_F32) {
                OpNDT<float> op{(const float *)X, d, T, 0, -1};
                hipLaunchKernelGGL(syrk_kernel<OpNDT<float>>, grid, block, 0, ctx->stream, op, g);
            } else {
                OpNDT<unsigned short> op{(const unsigned short *)X, d, T, 0, -1};
                hipLaunchKernelGGL(syrk_kernel<OpNDT<unsigned short>>, grid, block, 0, ctx->stream, op, g);
            }
        } else {
            // [R][d]: feature index contiguous, sample index strided by d
            if (dtype == KFAC_F32) {
                OpStrided<float, false> op{(const float *)X, 1, d, d, 0, -1};
                hipLaunchKernelGGL((syrk_kernel<OpStrided<float, false>>), grid, block, 0, ctx->stream, op, g);
            } else {
                OpStrided<unsigned short, false> op{(const unsigned short *)X, 1, d, d, 0, -1};
                hipLaunchKernelGGL((syrk_kernel<OpStrided<unsigned short, false>>), grid, block, 0, ctx->stream, op, g);
            }
        }
    }
    KFAC_HIP_CHECK(hipGetLastError());
    if (g.nsplit > 1) {
        KfacProfScope prof(ctx, KC_SYRK_REDUCE, 0.0, (decay != 0.f ? 8.0 : 4.0) * D * D);
        hipLaunchKernelGGL(syrk_reduce_kernel, dim3(ntri, (PART + 255) / 256), dim3(256), 0, ctx->stream, g);
        KFAC_HIP_CHECK(hipGetLastError());
    }
    return KFAC_OK;
}
