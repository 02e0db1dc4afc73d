// fp32 MFMA tile engine for gfx950: one 256-thread workgroup (4 wave64s, 2x2) computes a
// 128x128 block of C = A * B, streaming K in slabs of 16 through double-buffered LDS.
// Each wave owns a 64x64 quadrant as 2x2 v_mfma_f32_32x32x2f32 accumulators (64 AccVGPRs).
//
// Operands are described by small loader objects, so the same engine serves the factor SYRK
// (sample matrices in [R][d] or [N][d][T] layout, fp32 or bf16, optional ones column), the
// preconditioner GEMM chain (transposed and plain eigenvector matrices) and the eigensolver's
// post-processing.  A loader presents the operand as elem(i, k), i = output row (A) or output
// column (B), k = contraction index, and returns zero outside the operand's extent, so ragged
// edges need no special handling anywhere else.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef float floatx16 __attribute__((ext_vector_type(16)));

namespace kfac {

constexpr int BM = 128;       // tile edge (both M and N)
constexpr int BK = 16;        // K slab
constexpr int LDT = BM + 4;   // LDS row pitch in floats
constexpr int NTHREADS = 256;
constexpr int EPT = BM * BK / NTHREADS;  // elements per thread per operand per slab = 8

__device__ inline float to_float(float v) { return v; }
__device__ inline float to_float(unsigned short v) { return __uint_as_float(((unsigned)v) << 16); }  // bf16 bits

// ---- operand loaders ------------------------------------------------------------------------
// Every loader defines:  KFAST  (thread mapping: consecutive threads walk k, else walk i)
//                        start(tid, i0, k0), fetch(float r[EPT]), next()
// Thread mapping, KFAST : kk = tid & 15,  ii = (tid >> 4) + 16*s
//                 IFAST : ii = tid & 127, kk = (tid >> 7) + 2*s          (s = 0..7)

// elem(i,k) = p[i*si + k*sk] for i < I, k < K; 1.0 on row ones_i (if >= 0); else 0.
template <typename E, bool KFAST_>
struct OpStrided {
    static constexpr bool KFAST = KFAST_;
    const E *p;
    int64_t si, sk;
    int I, K, ones_i;
    int i_t, k_t;  // thread state: first element's (i, k)
    __device__ void start(int tid, int i0, int k0) {
        if (KFAST) { i_t = i0 + (tid >> 4); k_t = k0 + (tid & 15); }
        else       { i_t = i0 + (tid & 127); k_t = k0 + (tid >> 7); }
    }
    __device__ void fetch(float (&r)[EPT]) const {
#pragma unroll
        for (int s = 0; s < EPT; ++s) {
            const int i = KFAST ? i_t + 16 * s : i_t;
            const int k = KFAST ? k_t : k_t + 2 * s;
            float v = 0.f;
            if (k < K) {
                if (i < I) v = to_float(p[(int64_t)i * si + (int64_t)k * sk]);
                else if (i == ones_i) v = 1.f;
            }
            r[s] = v;
        }
    }
    __device__ void next() { k_t += BK; }
};

// Samples in [N][d][T] layout with the contraction index k = n*T + t running over all sample rows:
// elem(i,k) = p[n*d*T + i*T + t], i < d; 1.0 on row ones_i; zero for k >= K (= end of this split).
template <typename E>
struct OpNDT {
    static constexpr bool KFAST = true;
    const E *p;
    int d, T, K, ones_i;
    int i_t, k_t, n_t, t_t;
    __device__ void start(int tid, int i0, int k0) {
        i_t = i0 + (tid >> 4);
        k_t = k0 + (tid & 15);
        n_t = k_t / T;
        t_t = k_t - n_t * T;
    }
    __device__ void fetch(float (&r)[EPT]) const {
        const E *base = p + ((int64_t)n_t * d) * T + t_t;
#pragma unroll
        for (int s = 0; s < EPT; ++s) {
            const int i = i_t + 16 * s;
            float v = 0.f;
            if (k_t < K) {
                if (i < d) v = to_float(base[(int64_t)i * T]);
                else if (i == ones_i) v = 1.f;
            }
            r[s] = v;
        }
    }
    __device__ void next() {
        k_t += BK;
        t_t += BK;
        while (t_t >= T) { t_t -= T; ++n_t; }
    }
};

template <bool KFAST>
__device__ inline void store_slab(float (*dst)[LDT], const float (&r)[EPT], int tid) {
#pragma unroll
    for (int s = 0; s < EPT; ++s) {
        if (KFAST) dst[tid & 15][(tid >> 4) + 16 * s] = r[s];
        else       dst[(tid >> 7) + 2 * s][tid & 127] = r[s];
    }
}

struct TileSmem {
    float a[2][BK][LDT];
    float b[2][BK][LDT];
};

// acc[i][j] accumulates rows wm+32i.., cols wn+32j.. of the tile; element r of a 32x32 accumulator
// sits at row 8*(r/4) + 4*(lane/32) + r%4, column lane%32.
template <class OpA, class OpB>
__device__ inline void gemm_tile(OpA &A, OpB &B, int i0, int j0, int kbeg, int kend, TileSmem &sm,
                                 floatx16 (&acc)[2][2]) {
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int lk = lane >> 5, lc = lane & 31;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    const int nslab = (kend - kbeg + BK - 1) / BK;
    if (nslab <= 0) return;
    float ra[EPT], rb[EPT];
    A.start(tid, i0, kbeg);
    B.start(tid, j0, kbeg);
    A.fetch(ra);
    B.fetch(rb);
    store_slab<OpA::KFAST>(sm.a[0], ra, tid);
    store_slab<OpB::KFAST>(sm.b[0], rb, tid);
    __syncthreads();
    for (int s = 0; s < nslab; ++s) {
        const int cur = s & 1;
        const bool more = s + 1 < nslab;
        if (more) {
            A.next();
            B.next();
            A.fetch(ra);
            B.fetch(rb);
        }
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            float a0 = sm.a[cur][kk + lk][wm + lc];
            float a1 = sm.a[cur][kk + lk][wm + 32 + lc];
            float b0 = sm.b[cur][kk + lk][wn + lc];
            float b1 = sm.b[cur][kk + lk][wn + 32 + lc];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
        }
        if (more) {
            store_slab<OpA::KFAST>(sm.a[cur ^ 1], ra, tid);
            store_slab<OpB::KFAST>(sm.b[cur ^ 1], rb, tid);
        }
        __syncthreads();
    }
}

// Visit every accumulator element of this thread: f(row_in_tile, col_in_tile, value).
template <class F>
__device__ inline void for_each_acc(const floatx16 (&acc)[2][2], F f) {
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int lk = lane >> 5, lc = lane & 31;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                f(wm + 32 * i + 8 * (r >> 2) + 4 * lk + (r & 3), wn + 32 * j + lc, acc[i][j][r]);
}

// C = A * B over a rectangular grid of tiles (blockIdx.y: row tile, blockIdx.x: column tile); the
// epilogue object is called as epi(row, col, value) for every in-range element.
template <class OpA, class OpB, class Epi>
__global__ __launch_bounds__(NTHREADS) void gemm_generic_kernel(OpA a, OpB b, Epi epi, int M, int N, int K) {
    __shared__ TileSmem sm;
    const int i0 = blockIdx.y * BM, j0 = blockIdx.x * BM;
    floatx16 acc[2][2];
    gemm_tile(a, b, i0, j0, 0, K, sm, acc);
    for_each_acc(acc, [&](int r, int c, float v) {
        const int gr = i0 + r, gc = j0 + c;
        if (gr < M && gc < N) epi(gr, gc, v);
    });
}

struct EpiStore {
    float *C;
    int64_t ld;
    __device__ void operator()(int r, int c, float v) const { C[(int64_t)r * ld + c] = v; }
};

}  // namespace kfac
