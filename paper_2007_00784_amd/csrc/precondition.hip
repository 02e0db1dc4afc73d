// Eigenbasis preconditioning of one layer's gradient, Eqs. (v1), (v2), (kfac-eigen) of Sec. IV-A:
//   T  = QG^T grad            (dG x dA, K = dG)
//   V2 = (T QA) / (lamG lamA^T + damping)     (K = dA, divide fused into the epilogue)
//   T  = QG V2                (K = dG)
//   grad = T QA^T             (K = dA)
// Four dependent GEMMs on the fp32 MFMA tile engine; T and V2 live in the context workspace.
#include "kfac_internal.h"
#include "mfma_gemm.h"

using namespace kfac;

namespace {

enum { EPI_STORE = 0, EPI_DIVIDE = 1, EPI_STORE_BF16 = 2 };

struct GemmOut {
    float *C;
    unsigned short *Cb;
    int M, N;
    int64_t ldc;
    const float *lamG, *lamA;
    float damping;
};

__device__ inline unsigned short f32_to_bf16_rne(float v) {
    unsigned u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

template <class OpA, class OpB, int EPI>
__global__ __launch_bounds__(NTHREADS) void gemm_kernel(OpA a, OpB b, GemmOut o, int K) {
    __shared__ TileSmem sm;
    const int i0 = blockIdx.y * BM, j0 = blockIdx.x * BM;
    floatx16 acc[2][2];
    gemm_tile(a, b, i0, j0, 0, K, sm, acc);
    for_each_acc(acc, [&](int r, int c, float v) {
        const int gr = i0 + r, gc = j0 + c;
        if (gr < o.M && gc < o.N) {
            if (EPI == EPI_DIVIDE) {
                const float lg = fmaxf(o.lamG[gr], 0.f), la = fmaxf(o.lamA[gc], 0.f);
                v = v / (lg * la + o.damping);
            }
            if (EPI == EPI_STORE_BF16) o.Cb[(int64_t)gr * o.ldc + gc] = f32_to_bf16_rne(v);
            else o.C[(int64_t)gr * o.ldc + gc] = v;
        }
    });
}

template <class OpA, class OpB, int EPI>
int launch(kfac_ctx *ctx, OpA a, OpB b, GemmOut o, int K) {
    const dim3 grid((o.N + BM - 1) / BM, (o.M + BM - 1) / BM);
    KfacProfScope prof(ctx, KC_PRECOND_GEMM, 2.0 * o.M * o.N * K, 4.0 * ((double)o.M * K + (double)K * o.N + (double)o.M * o.N));
    hipLaunchKernelGGL((gemm_kernel<OpA, OpB, EPI>), grid, dim3(NTHREADS), 0, ctx->stream, a, b, o, K);
    KFAC_HIP_CHECK(hipGetLastError());
    return KFAC_OK;
}

}  // namespace

int kfac_launch_precondition(kfac_ctx *ctx, const float *QA, const float *lamA, int dA, const float *QG,
                             const float *lamG, int dG, float damping, void *grad, int grad_dtype) {
    const size_t elems = (size_t)dG * dA;
    if (2 * elems * sizeof(float) > ctx->ws_bytes) return KFAC_EWORKSPACE;
    float *T = (float *)ctx->ws;
    float *V = T + kfac_align_up(elems, 64);
    if (2 * kfac_align_up(elems, 64) * sizeof(float) > ctx->ws_bytes) return KFAC_EWORKSPACE;
    GemmOut o{nullptr, nullptr, dG, dA, dA, lamG, lamA, damping};
    int rc;
    // T = QG^T grad : A(m,k) = QG[k][m] (m contiguous), B(k,n) = grad[k][n] (n contiguous)
    o.C = T;
    OpStrided<float, false> qgt{QG, 1, dG, dG, dG, -1};
    if (grad_dtype == KFAC_F32) {
        OpStrided<float, false> g{(const float *)grad, 1, dA, dA, dG, -1};
        rc = launch<decltype(qgt), decltype(g), EPI_STORE>(ctx, qgt, g, o, dG);
    } else {
        OpStrided<unsigned short, false> g{(const unsigned short *)grad, 1, dA, dA, dG, -1};
        rc = launch<decltype(qgt), decltype(g), EPI_STORE>(ctx, qgt, g, o, dG);
    }
    if (rc) return rc;
    // V = (T QA) / (lamG lamA^T + damping) : A(m,k) = T[m][k] (k contiguous), B(k,n) = QA[k][n]
    o.C = V;
    OpStrided<float, true> t_mk{T, dA, 1, dG, dA, -1};
    OpStrided<float, false> qa_kn{QA, 1, dA, dA, dA, -1};
    rc = launch<decltype(t_mk), decltype(qa_kn), EPI_DIVIDE>(ctx, t_mk, qa_kn, o, dA);
    if (rc) return rc;
    // T = QG V : A(m,k) = QG[m][k] (k contiguous), B(k,n) = V[k][n]
    o.C = T;
    OpStrided<float, true> qg_mk{QG, dG, 1, dG, dG, -1};
    OpStrided<float, false> v_kn{V, 1, dA, dA, dG, -1};
    rc = launch<decltype(qg_mk), decltype(v_kn), EPI_STORE>(ctx, qg_mk, v_kn, o, dG);
    if (rc) return rc;
    // grad = T QA^T : A(m,k) = T[m][k], B(k,n) = QA[n][k] (k contiguous)
    OpStrided<float, true> qa_nk{QA, dA, 1, dA, dA, -1};
    if (grad_dtype == KFAC_F32) {
        o.C = (float *)grad;
        rc = launch<decltype(t_mk), decltype(qa_nk), EPI_STORE>(ctx, t_mk, qa_nk, o, dA);
    } else {
        o.Cb = (unsigned short *)grad;
        rc = launch<decltype(t_mk), decltype(qa_nk), EPI_STORE_BF16>(ctx, t_mk, qa_nk, o, dA);
    }
    return rc;
}
