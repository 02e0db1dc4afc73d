// The explicit-inverse method of Sec. II-C, Eq. (kfac-damped): Finv = (F + gamma I)^-1 for every Kronecker factor,
// then the preconditioned gradient as two plain products Ginv * grad * Ainv (the method Sec. IV-A and Table I
// compare the eigendecomposition with).  The inverse of a symmetric positive definite matrix is formed the
// classical way, in fp32: blocked Cholesky factorisation F + gamma I = L L^T (128-wide block columns: the diagonal
// block is factored, and inverted, by one workgroup in LDS; the panel below it is multiplied by that inverse and the
// trailing matrix gets its rank-128 update on the fp32 MFMA tile engine), then the triangular inverse L^-1 block
// row by block row, then L^-T L^-1 as one symmetric product.  n^3 flops in all, 5 n/128 + 1 launches per factor.
#include <algorithm>
#include <cmath>
#include "kfac_internal.h"
#include "mfma_gemm.h"

using namespace kfac;

namespace {

constexpr int NB = BM;            // block size of the factorisation = tile edge of the engine
constexpr int DLD = NB + 1;       // LDS pitch of a diagonal block

struct InvPtr { const float *F; float *out; };   // one factor: the caller's matrix and where its inverse goes

// One group of factors of the same size, advanced together (blockIdx.y: factor).  Per factor the workspace holds
//   L  [npad][npad]  F + gamma I on entry to the factorisation (both triangles), the Cholesky factor after
//   Li [npad][npad]  L^-1 (lower triangular)
//   D  [nt][NB][NB]  inverses of the diagonal blocks of L
//   R  [NB][npad]    one block row of L * Li during the triangular inversion
struct InvArgs {
    float *base;          // first factor's buffers; the next factor's are fstride floats further
    int64_t fstride;
    const InvPtr *tab;    // device table of the group's factors
    int64_t ld;           // npad
    int n, nt, k;         // k: block column (factorisation) or block row (triangular inversion) of this launch
    __device__ float *L(int f) const { return base + f * fstride; }
    __device__ float *Li(int f) const { return L(f) + ld * ld; }
    __device__ float *D(int f) const { return Li(f) + ld * ld; }
    __device__ float *R(int f) const { return D(f) + (int64_t)nt * NB * NB; }
};

// L = F + gamma I inside n x n, the identity on the padded part of the diagonal, zero elsewhere; Li = 0.
__global__ __launch_bounds__(256) void inv_init_kernel(float gamma, InvArgs a) {
    const int f = blockIdx.y, n = a.n;
    const float *F = a.tab[f].F;
    float *L = a.L(f), *Li = a.Li(f);
    const int64_t total = a.ld * a.ld;
    for (int64_t e = blockIdx.x * 256ll + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        const int r = (int)(e / a.ld), c = (int)(e - (int64_t)r * a.ld);
        float v = 0.f;
        if (r < n && c < n) v = F[(int64_t)r * n + c] + (r == c ? gamma : 0.f);
        else if (r == c) v = 1.f;
        L[e] = v;
        Li[e] = 0.f;
    }
}

// Diagonal block k: Cholesky factor in place (lower triangle; the upper is cleared) and its inverse, written to D[k]
// and to the diagonal block of Li.  One workgroup per factor; both matrices live in LDS.  A pivot that is not positive (the
// input was not positive definite, or not finite) yields NaNs from there on.
__global__ __launch_bounds__(256) void inv_diag_kernel(InvArgs a) {
    extern __shared__ float lds[];
    float *S = lds, *X = lds + NB * DLD;
    const int tid = threadIdx.x, f = blockIdx.x;
    float *blk = a.L(f) + ((int64_t)a.k * NB) * a.ld + (int64_t)a.k * NB;
    for (int e = tid; e < NB * NB; e += 256) {
        const int r = e / NB, c = e % NB;
        S[r * DLD + c] = r >= c ? blk[(int64_t)r * a.ld + c] : blk[(int64_t)c * a.ld + r];   // the lower triangle is the valid one
        X[r * DLD + c] = 0.f;
    }
    const int ty = tid >> 4, tx = tid & 15;
    for (int j = 0; j < NB; ++j) {
        __syncthreads();
        const float piv = S[j * DLD + j];
        const float sq = sqrtf(piv), rs = 1.f / sq;
        __syncthreads();
        if (tid < NB - 1 - j) S[(j + 1 + tid) * DLD + j] *= rs;
        if (tid == 255) S[j * DLD + j] = sq;
        __syncthreads();
        // trailing update of the lower triangle: S[i][c] -= S[i][j] S[c][j], j < c <= i
        for (int i = j + 1 + ty; i < NB; i += 16) {
            const float lij = S[i * DLD + j];
            for (int c = j + 1 + tx; c <= i; c += 16) S[i * DLD + c] -= lij * S[c * DLD + j];
        }
    }
    __syncthreads();
    // X = S^-1 by forward substitution, one column per thread; every thread walks the same (i, k) so the reads of S
    // are broadcasts (entries of X above the column's diagonal are zero and add nothing)
    if (tid < NB) {
        const int c = tid;
        for (int i = 0; i < NB; ++i) {
            float s = i == c ? 1.f : 0.f;
            for (int k = 0; k < i; ++k) s -= S[i * DLD + k] * X[k * DLD + c];
            if (i >= c) X[i * DLD + c] = s / S[i * DLD + i];
        }
    }
    __syncthreads();
    float *Dk = a.D(f) + (int64_t)a.k * NB * NB;
    float *Lik = a.Li(f) + ((int64_t)a.k * NB) * a.ld + (int64_t)a.k * NB;
    for (int e = tid; e < NB * NB; e += 256) {
        const int r = e / NB, c = e % NB;
        blk[(int64_t)r * a.ld + c] = r >= c ? S[r * DLD + c] : 0.f;
        const float x = r >= c ? X[r * DLD + c] : 0.f;
        Dk[e] = x;
        Lik[(int64_t)r * a.ld + c] = x;
    }
}

__device__ inline void inv_tri_decode(int idx, int &ti, int &tj) {   // idx = ti (ti + 1) / 2 + tj, tj <= ti
    int t = (int)((sqrtf(8.f * (float)idx + 1.f) - 1.f) * 0.5f);
    while ((t + 1) * (t + 2) / 2 <= idx) ++t;
    while (t * (t + 1) / 2 > idx) --t;
    ti = t;
    tj = idx - t * (t + 1) / 2;
}

// The five products, one 128 x 128 output tile per workgroup (all operands are padded to whole tiles):
//   PANEL   L[i,k] <- L[i,k] D_k^T                                      i > k              (grid: nt-k-1)
//   UPDATE  L[i,j] <- L[i,j] - L[i,k] L[j,k]^T                          i >= j > k         (grid: lower tiles)
//   ROW     R[:, j] <- sum_{c = j}^{i-1} L[i,c] Li[c,j]                 j < i = a.k        (grid: i)
//   SCALE   Li[i,j] <- -D_i R[:, j]                                     j < i = a.k        (grid: i)
//   GRAM    out[i,j] <- sum_{c >= i} Li[c,i]^T Li[c,j], and its mirror  i >= j             (grid: lower tiles)
enum { INV_PANEL = 0, INV_UPDATE, INV_ROW, INV_SCALE, INV_GRAM };
template <int MODE>
__global__ __launch_bounds__(NTHREADS) __attribute__((amdgpu_waves_per_eu(2))) void inv_gemm_kernel(InvArgs a) {
    __shared__ TileSmem sm;
    floatx16 acc[2][2];
    const int64_t ld = a.ld;
    const int npad = a.nt * NB, f = blockIdx.y;
    float *const L = a.L(f), *const Li = a.Li(f), *const D = a.D(f), *const R = a.R(f);
    if (MODE == INV_PANEL) {
        const int i = a.k + 1 + blockIdx.x;
        float *Lik = L + ((int64_t)i * NB) * ld + (int64_t)a.k * NB;
        OpStrided<float, true> A{Lik, ld, 1, NB, NB, -1};                                     // elem(m,c) = L[i,k][m][c]
        OpStrided<float, true> B{D + (int64_t)a.k * NB * NB, NB, 1, NB, NB, -1};              // elem(n,c) = D_k[n][c]
        gemm_tile(A, B, 0, 0, 0, NB, sm, acc);
        for_each_acc(acc, [&](int r, int c, float v) { Lik[(int64_t)r * ld + c] = v; });
    } else if (MODE == INV_UPDATE) {
        int ti, tj;
        inv_tri_decode(blockIdx.x, ti, tj);
        const int i = a.k + 1 + ti, j = a.k + 1 + tj;
        OpStrided<float, true> A{L + ((int64_t)i * NB) * ld + (int64_t)a.k * NB, ld, 1, NB, NB, -1};
        OpStrided<float, true> B{L + ((int64_t)j * NB) * ld + (int64_t)a.k * NB, ld, 1, NB, NB, -1};
        gemm_tile(A, B, 0, 0, 0, NB, sm, acc);
        float *Lij = L + ((int64_t)i * NB) * ld + (int64_t)j * NB;
        for_each_acc(acc, [&](int r, int c, float v) { Lij[(int64_t)r * ld + c] -= v; });
    } else if (MODE == INV_ROW) {
        const int i = a.k, j = blockIdx.x;
        OpStrided<float, true> A{L + ((int64_t)i * NB) * ld, ld, 1, NB, i * NB, -1};           // elem(m,c) = L[i*NB+m][c]
        OpStrided<float, false> B{Li + (int64_t)j * NB, 1, ld, NB, i * NB, -1};                // elem(n,c) = Li[c][j*NB+n]
        gemm_tile(A, B, 0, 0, j * NB, i * NB, sm, acc);
        float *Rj = R + (int64_t)j * NB;
        for_each_acc(acc, [&](int r, int c, float v) { Rj[(int64_t)r * ld + c] = v; });
    } else if (MODE == INV_SCALE) {
        const int i = a.k, j = blockIdx.x;
        OpStrided<float, true> A{D + (int64_t)i * NB * NB, NB, 1, NB, NB, -1};                 // elem(m,c) = D_i[m][c]
        OpStrided<float, false> B{R + (int64_t)j * NB, 1, ld, NB, NB, -1};                     // elem(n,c) = R[c][j*NB+n]
        gemm_tile(A, B, 0, 0, 0, NB, sm, acc);
        float *Lij = Li + ((int64_t)i * NB) * ld + (int64_t)j * NB;
        for_each_acc(acc, [&](int r, int c, float v) { Lij[(int64_t)r * ld + c] = -v; });
    } else {
        int i, j;
        inv_tri_decode(blockIdx.x, i, j);
        OpStrided<float, false> A{Li + (int64_t)i * NB, 1, ld, NB, npad, -1};                  // elem(m,c) = Li[c][i*NB+m]
        OpStrided<float, false> B{Li + (int64_t)j * NB, 1, ld, NB, npad, -1};                  // elem(n,c) = Li[c][j*NB+n]
        gemm_tile(A, B, 0, 0, i * NB, npad, sm, acc);                                          // Li[c, i] = 0 for c < i
        const int n = a.n;
        float *out = a.tab[f].out;
        for_each_acc(acc, [&](int r, int c, float v) {
            const int gr = i * NB + r, gc = j * NB + c;
            if (gr < n && gc < n) out[(int64_t)gr * n + gc] = v;
        });
        if (i != j)
            for_each_acc_transposed(acc, reinterpret_cast<float *>(&sm), [&](int r, int c, float v) {
                const int gr = j * NB + r, gc = i * NB + c;
                if (gr < n && gc < n) out[(int64_t)gr * n + gc] = v;
            });
    }
}

inline int inv_npad(int n) { return (n + NB - 1) / NB * NB; }
inline size_t inv_bytes_one(int n) {
    const size_t np = inv_npad(n), nt = np / NB;
    return kfac_align_up((2 * np * np + nt * NB * NB + (size_t)NB * np) * sizeof(float), 256);
}

// grad <- Ginv grad Ainv: T = grad Ainv into the workspace, then grad = Ginv T.
struct EpiStoreBf16 {
    unsigned short *C;
    int64_t ld;
    __device__ void operator()(int r, int c, float v) const {
        unsigned u = __float_as_uint(v);
        if ((u & 0x7fffffffu) > 0x7f800000u) { C[(int64_t)r * ld + c] = (unsigned short)((u >> 16) | 0x40u); return; }
        u += 0x7fffu + ((u >> 16) & 1u);    // round to nearest even
        C[(int64_t)r * ld + c] = (unsigned short)(u >> 16);
    }
};

}  // namespace

// Workspace: the table of pointers, then room for the largest group of equal-sized factors (a group too large for
// the workspace at hand is cut into several).  With room for more, up to four groups are in flight at once.
static size_t inv_table_bytes(int batch) { return kfac_align_up((size_t)batch * sizeof(InvPtr), 256); }
size_t kfac_invert_ws_bytes_impl(int batch, const int *d) {
    size_t m = 0;
    for (int b = 0; b < batch; ++b) m = std::max(m, inv_bytes_one(d[b]));
    return inv_table_bytes(batch) + m;
}

namespace {
struct InvGroup { int n, first, count; };   // `count` factors of size n, entries first.. of the sorted table

// The whole chain of one group on one stream.
int inv_enqueue_group(kfac_ctx *ctx, hipStream_t st, const InvGroup &g, const InvPtr *tab_dev, float *slot, float damping, size_t lds) {
    const int n = g.n, np = inv_npad(n), nt = np / NB, nm = g.count;
    InvArgs a;
    a.base = slot;
    a.fstride = (int64_t)(inv_bytes_one(n) / sizeof(float));
    a.tab = tab_dev + g.first;
    a.ld = np; a.n = n; a.nt = nt; a.k = 0;
    const double n3 = (double)nm * n * n * n;
    {
        KfacProfScope prof(ctx, KC_INVERSE, n3 / 3.0, 0.0, st);
        hipLaunchKernelGGL(inv_init_kernel, dim3((unsigned)std::min<int64_t>(((int64_t)np * np + 255) / 256, 2048), nm), dim3(256), 0, st,
                           damping, a);
        for (int k = 0; k < nt; ++k) {
            a.k = k;
            hipLaunchKernelGGL(inv_diag_kernel, dim3(nm), dim3(256), lds, st, a);
            const int rest = nt - k - 1;
            if (rest > 0) {
                hipLaunchKernelGGL(inv_gemm_kernel<INV_PANEL>, dim3(rest, nm), dim3(NTHREADS), 0, st, a);
                hipLaunchKernelGGL(inv_gemm_kernel<INV_UPDATE>, dim3(rest * (rest + 1) / 2, nm), dim3(NTHREADS), 0, st, a);
            }
        }
    }
    {
        KfacProfScope prof(ctx, KC_INVERSE, n3 / 3.0, 0.0, st);
        for (int i = 1; i < nt; ++i) {
            a.k = i;
            hipLaunchKernelGGL(inv_gemm_kernel<INV_ROW>, dim3(i, nm), dim3(NTHREADS), 0, st, a);
            hipLaunchKernelGGL(inv_gemm_kernel<INV_SCALE>, dim3(i, nm), dim3(NTHREADS), 0, st, a);
        }
    }
    KfacProfScope prof(ctx, KC_INVERSE, n3 / 3.0, 0.0, st);
    hipLaunchKernelGGL(inv_gemm_kernel<INV_GRAM>, dim3(nt * (nt + 1) / 2, nm), dim3(NTHREADS), 0, st, a);
    KFAC_HIP_CHECK(hipGetLastError());
    return KFAC_OK;
}
}  // namespace

int kfac_launch_invert_factors(kfac_ctx *ctx, int batch, const float *const *F, const int *d, float damping, float *const *Finv) {
    if (kfac_invert_ws_bytes_impl(batch, d) > ctx->ws_bytes) return KFAC_EWORKSPACE;
    const size_t lds = (size_t)2 * NB * DLD * sizeof(float);
    if ((int)lds > ctx->max_lds) return KFAC_EHIP;
    KFAC_HIP_CHECK(hipFuncSetAttribute((const void *)inv_diag_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    // factors sorted by size (largest first); equal sizes form groups
    std::vector<int> order(batch);
    for (int b = 0; b < batch; ++b) order[b] = b;
    std::stable_sort(order.begin(), order.end(), [&](int p, int q) { return d[p] > d[q]; });
    std::vector<InvPtr> tab(batch);
    for (int t = 0; t < batch; ++t) tab[t] = InvPtr{F[order[t]], Finv[order[t]]};
    InvPtr *tab_dev = (InvPtr *)ctx->ws;
    KFAC_CHECK(kfac_upload(ctx, tab_dev, tab.data(), (size_t)batch * sizeof(InvPtr)));
    char *pool = ctx->ws + inv_table_bytes(batch);
    const size_t pool_bytes = ctx->ws_bytes - inv_table_bytes(batch);
    // four equal regions, one per internal stream, if each then still holds the largest factor; else one region
    const size_t largest = inv_bytes_one(d[order[0]]);
    const int nstreams = pool_bytes / KFAC_NUM_AUX_STREAMS >= largest ? KFAC_NUM_AUX_STREAMS : 1;
    const size_t region = kfac_align_up(pool_bytes / nstreams - 255, 256) ;
    std::vector<InvGroup> groups;
    for (int t = 0; t < batch;) {
        int e = t;
        const size_t one = inv_bytes_one(d[order[t]]);
        const int cap = (int)std::max<size_t>(1, region / one);
        while (e < batch && d[order[e]] == d[order[t]] && e - t < cap) ++e;
        groups.push_back(InvGroup{d[order[t]], t, e - t});
        t = e;
    }
    // the internal streams start after everything already queued on the caller's stream (the table upload included) ...
    KFAC_HIP_CHECK(hipEventRecord(ctx->ev_fork, ctx->stream));
    for (int i = 0; i < nstreams; ++i) KFAC_HIP_CHECK(hipStreamWaitEvent(ctx->aux[i], ctx->ev_fork, 0));
    // groups dealt to the stream with the least work so far (largest first); a stream's groups use its region in turn
    double load[KFAC_NUM_AUX_STREAMS] = {0, 0, 0, 0};
    int rc = KFAC_OK;
    for (const InvGroup &g : groups) {
        int best = 0;
        for (int i = 1; i < nstreams; ++i) if (load[i] < load[best]) best = i;
        const double nt = inv_npad(g.n) / NB;
        load[best] += nt * 250e-6 + (double)g.count * g.n * (double)g.n * g.n / 60e12;   // launch-latency floor + products
        rc = inv_enqueue_group(ctx, ctx->aux[best], g, tab_dev, (float *)(pool + (size_t)best * region), damping, lds);
        if (rc != KFAC_OK) break;
    }
    // ... and the caller's stream continues after all of them
    for (int i = 0; i < nstreams; ++i) {
        if (hipEventRecord(ctx->ev_join[i], ctx->aux[i]) != hipSuccess) return KFAC_EHIP;
        if (hipStreamWaitEvent(ctx->stream, ctx->ev_join[i], 0) != hipSuccess) return KFAC_EHIP;
    }
    return rc;
}

// ---- grad <- Ginv grad Ainv for a batch of layers: two launches, each over the output tiles of every layer ----
namespace {
struct InvLayer {
    const float *Ainv, *Ginv;
    void *grad;
    float *T;          // [dG][dA] intermediate grad * Ainv
    int dA, dG, bf16;
    int tile0, tn;     // first tile of the layer in the launch, tiles per tile row
};

// STAGE 0: T = grad Ainv.  STAGE 1: grad = Ginv T.
template <int STAGE>
__global__ __launch_bounds__(NTHREADS) __attribute__((amdgpu_waves_per_eu(2))) void inv_precond_kernel(const InvLayer *layers, int nlayers) {
    __shared__ TileSmem sm;
    // the layer whose tile range holds this workgroup: the last one that starts at or before it
    int l = 0;
    for (int base = 0; base < nlayers; base += 64) {
        const int idx = base + (int)(threadIdx.x & 63);
        const bool le = idx < nlayers && layers[idx].tile0 <= (int)blockIdx.x;
        const unsigned long long m = __ballot(le);
        if (m == 0) break;
        l = base + 63 - __builtin_clzll(m);
    }
    l = __builtin_amdgcn_readfirstlane(l);
    const InvLayer L = layers[l];
    const int t = blockIdx.x - L.tile0;
    const int i0 = (t / L.tn) * BM, j0 = (t % L.tn) * BM;
    if (STAGE == 0) {
        OpStrided<float, false> b{L.Ainv, 1, L.dA, L.dA, L.dA, -1};            // elem(c,k) = Ainv[k][c]
        float *T = L.T;
        const int dA = L.dA;
        auto epi = [=](int r, int c, float v) { T[(int64_t)r * dA + c] = v; };
        if (L.bf16) {
            OpStrided<unsigned short, true> a{(const unsigned short *)L.grad, L.dA, 1, L.dG, L.dA, -1};
            gemm_tile_ragged(a, b, i0, j0, L.dA, L.dG, L.dA, sm, epi);
        } else {
            OpStrided<float, true> a{(const float *)L.grad, L.dA, 1, L.dG, L.dA, -1};
            gemm_tile_ragged(a, b, i0, j0, L.dA, L.dG, L.dA, sm, epi);
        }
    } else {
        OpStrided<float, true> a{L.Ginv, L.dG, 1, L.dG, L.dG, -1};
        OpStrided<float, false> b{L.T, 1, L.dA, L.dA, L.dG, -1};               // elem(c,k) = T[k][c]
        if (L.bf16) {
            const EpiStoreBf16 e{(unsigned short *)L.grad, L.dA};
            gemm_tile_ragged(a, b, i0, j0, L.dG, L.dG, L.dA, sm, [=](int r, int c, float v) { e(r, c, v); });
        } else {
            float *g = (float *)L.grad;
            const int dA = L.dA;
            gemm_tile_ragged(a, b, i0, j0, L.dG, L.dG, L.dA, sm, [=](int r, int c, float v) { g[(int64_t)r * dA + c] = v; });
        }
    }
}
}  // namespace

size_t kfac_precondition_inverse_ws_bytes_impl(int n, const kfac_precond_inv_item *items) {
    size_t b = kfac_align_up((size_t)n * sizeof(InvLayer), 256);
    for (int i = 0; i < n; ++i) b += kfac_align_up((size_t)items[i].dA * items[i].dG * sizeof(float), 256);
    return b;
}

int kfac_launch_precondition_inverse_batched(kfac_ctx *ctx, int n, const kfac_precond_inv_item *items) {
    if (kfac_precondition_inverse_ws_bytes_impl(n, items) > ctx->ws_bytes) return KFAC_EWORKSPACE;
    std::vector<InvLayer> layers(n);
    char *p = ctx->ws + kfac_align_up((size_t)n * sizeof(InvLayer), 256);
    int tiles = 0;
    double fl0 = 0.0, fl1 = 0.0;
    for (int i = 0; i < n; ++i) {
        const kfac_precond_inv_item &it = items[i];
        const int tm = (it.dG + BM - 1) / BM, tn = (it.dA + BM - 1) / BM;
        layers[i] = InvLayer{it.Ainv, it.Ginv, it.grad, (float *)p, it.dA, it.dG, it.grad_dtype == KFAC_BF16 ? 1 : 0, tiles, tn};
        p += kfac_align_up((size_t)it.dA * it.dG * sizeof(float), 256);
        tiles += tm * tn;
        fl0 += 2.0 * it.dG * (double)it.dA * it.dA;
        fl1 += 2.0 * it.dG * (double)it.dG * it.dA;
    }
    InvLayer *d_layers = (InvLayer *)ctx->ws;
    KFAC_CHECK(kfac_upload(ctx, d_layers, layers.data(), (size_t)n * sizeof(InvLayer)));
    {
        KfacProfScope prof(ctx, KC_PRECOND_GEMM, fl0, 0.0);
        hipLaunchKernelGGL(inv_precond_kernel<0>, dim3(tiles), dim3(NTHREADS), 0, ctx->stream, (const InvLayer *)d_layers, n);
    }
    KfacProfScope prof(ctx, KC_PRECOND_GEMM, fl1, 0.0);
    hipLaunchKernelGGL(inv_precond_kernel<1>, dim3(tiles), dim3(NTHREADS), 0, ctx->stream, (const InvLayer *)d_layers, n);
    KFAC_HIP_CHECK(hipGetLastError());
    return KFAC_OK;
}
