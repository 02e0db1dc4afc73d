// Batched symmetric eigensolver F = Q diag(lam) Q^T (Sec. IV-A; Algorithm 1, step 2) by two-sided
// Jacobi iteration in fp32.
//
//  * d <= 128: one workgroup per factor.  The rotated matrix and the accumulated eigenvectors both
//    stay in LDS for the whole solve; every round applies d/2 disjoint plane rotations (round-robin
//    tournament ordering), each computed by one lane and applied by the whole workgroup.
//  * d  > 128: blocked Jacobi.  The matrix is cut into EB-wide blocks; a round pairs the blocks by
//    the same tournament, gives each 2EB x 2EB pivot sub-problem ONE sweep of the LDS solver above
//    (one workgroup per pair; only the pairs between the two blocks after a block's first visit of the
//    sweep), and applies the resulting orthogonal transforms to the whole matrix and to the eigenvector
//    accumulator as fp32 MFMA products, one workgroup per 2EB x 2EB block.  Only the lower
//    block-triangle is computed; the mirror image is written from LDS, so the working matrix stays
//    exactly symmetric.
//  * d >= 2048: two-level.  128-wide super-blocks are paired by an outer tournament; each 256 x 256
//    super-pair runs the rounds above on a compact copy that stays in L2 and accumulates its transform,
//    which is then applied to the whole matrix and accumulator by two passes of 128 x 128 x 256 GEMM
//    tiles on split-fp16 MFMAs (or fp32 MFMAs on request).
//  * Factors of similar size are padded into common groups that advance together; all groups are in
//    flight at once on the context's internal streams.
//  * When a factor has converged, one Newton-Schulz step re-orthogonalises the accumulated
//    eigenvectors, Rayleigh quotients against the caller's matrix give the eigenvalues, and the
//    columns are sorted.
//
// Convergence is decided on the host once per sweep from off(F)_F / ||F||_F.
#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstdio>
#include <cmath>
#include <deque>
#include <thread>
#include <cstdlib>
#include <type_traits>
#include <vector>
#include "kfac_internal.h"
#include "mfma_gemm.h"
#include "mfma_gemm_x3.h"

namespace {

constexpr int EB = KFAC_EIG_B;       // block width of the blocked path
constexpr int KP = 2 * EB;           // pivot sub-problem size
constexpr int PLD = KP + 1;          // LDS pitch of a pivot (odd: column walks are conflict free)
constexpr int SMALL_MAX = KFAC_EIG_SMALL;
constexpr int NT = 256;
static_assert(NT == 256 && (KP == 64 || KP == 128) && SMALL_MAX == 128, "thread mappings below assume these sizes");

struct SmallItem { const float *F; float *Q; float *lam; int n; int pad_; };
struct EigStat { float sweeps, off_rel, converged, rotations; };

// Tournament schedule on `players` (even) players: round r in [0, players-1), pair j in [0, players/2).
__host__ __device__ inline void rr_pair(int players, int r, int j, int &p, int &q) {
    int a, b;
    const int m1 = players - 1;
    if (j == 0) { a = m1; b = r; }
    else { a = (r + j) % m1; b = (r - j + m1) % m1; }
    p = a < b ? a : b;
    q = a < b ? b : a;
}

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;
}

// Sum over the workgroup; result valid in all threads.  red: one float of LDS per wave.
__device__ inline float block_sum(float v, float *red) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float s = 0.f;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) s += red[w];
    return s;
}

struct JacobiResult { int sweeps; float off2, nrm2; int rotations; };
struct RotEntry { int p, q; float c, s; };

// Two-sided Jacobi on the k x k symmetric matrix S (k even), accumulating V <- V J, both in LDS with
// pitch ld.  Stops when off(S)^2 <= tol^2 * ||S||^2 or after max_sweeps.  Rotations use the smaller
// angle, so the accumulated transform stays close to the identity ordering.  Entries whose magnitude
// is below skip_rel * ||S||_F / k are left alone (and exact zeros always are, which keeps zero-padded
// rows and columns decoupled).  KC > 0 fixes k at compile time (index arithmetic becomes shifts and
// each thread's column pair is loop invariant); KC == 0 takes k at run time.
// CROSS: a sweep visits only the pairs (i, k/2 + j) between the two halves, in k/2 rounds (the pairs inside
// each half are left to the caller's schedule).
// LAST_NORMS = false: the caller has no use for the norms after the last sweep (off2 and nrm2 are those before it).
template <int KC, bool CROSS = false, int NTH = NT, bool LAST_NORMS = true>
__device__ JacobiResult jacobi_lds(float *S, float *V, int k_rt, int ld, int max_sweeps, float tol, float skip_rel,
                                   float *red, RotEntry *rot, int *rotflag) {
    const int tid = threadIdx.x;
    const int k = KC > 0 ? KC : k_rt;
    const int half = k >> 1;
    JacobiResult res{0, 0.f, 0.f, 0};
    if (tid == 0) *rotflag = 0;
    for (int sweep = 0;; ++sweep) {
        if (!LAST_NORMS && sweep > 0 && sweep >= max_sweeps) {
            res.sweeps = sweep;
            break;
        }
        float o2 = 0.f, d2 = 0.f;
        for (int e = tid; e < k * k; e += NTH) {
            const int i = e / k, j = e - i * k;
            const float v = S[i * ld + j];
            if (i == j) d2 += v * v; else o2 += v * v;
        }
        o2 = block_sum(o2, red);
        d2 = block_sum(d2, red);
        res.off2 = o2;
        res.nrm2 = o2 + d2;
        res.sweeps = sweep;
        if (!(o2 > tol * tol * res.nrm2) || sweep >= max_sweeps) break;
        const float thr = skip_rel * sqrtf(res.nrm2) / (float)k;
        const int nrounds = CROSS ? half : k - 1;
        for (int r = 0; r < nrounds; ++r) {
            if (tid < half) {
                int p, q;
                if (CROSS) { p = tid; q = half + (tid + r) % half; }
                else rr_pair(k, r, tid, p, q);
                const float app = S[p * ld + p], aqq = S[q * ld + q], apq = S[p * ld + q];
                float c = 1.f, s = 0.f;
                if (fabsf(apq) > thr) {
                    // smaller rotation angle: with dd = aqq - app, b = 2 apq,
                    //   tan = sign(dd b) |b| / (|dd| + sqrt(dd^2 + b^2)),  c = 1/sqrt(1 + tan^2),  s = tan c
                    // on operands scaled by max(|dd|, |b|), with the hardware reciprocal, square root and
                    // reciprocal square root; one Newton step on c removes the bias of the 1 ulp reciprocal
                    // square root, which would otherwise scale S and V a little at every rotation
                    const float dd = aqq - app, b = 2.f * apq;
                    const float rm = __builtin_amdgcn_rcpf(fmaxf(fabsf(dd), fabsf(b)));
                    const float dn = fabsf(dd) * rm, bn = fabsf(b) * rm;
                    const float h = __builtin_amdgcn_sqrtf(fmaf(dn, dn, bn * bn));
                    const float ta = bn * __builtin_amdgcn_rcpf(dn + h);
                    const float t = copysignf(ta, __uint_as_float(__float_as_uint(dd) ^ (__float_as_uint(b) & 0x80000000u)));
                    const float w = fmaf(t, t, 1.f);
                    c = __builtin_amdgcn_rsqf(w);
                    c = c * fmaf(-0.5f * w, c * c, 1.5f);
                    s = t * c;
                    *rotflag = 1;
                }
                rot[tid] = RotEntry{p, q, c, s};
            }
            __syncthreads();
            if constexpr (KC > 0) {
                // S <- J^T S J on 2x2 blocks (a thread's column pair is fixed, its row pairs vary) and V <- V J
                // (a thread's row is fixed, the column pairs vary).  Loads of a batch are issued together before
                // any store, so they overlap.  With NTH = NT every thread does its share of both; with more
                // threads the lower half of the workgroup takes S and the upper half V, which run side by side
                // (the rounds are bound by LDS latency, not by its throughput).
                constexpr int HALF = KC / 2;
                constexpr bool SPLIT = NTH > NT;
                constexpr int NS = SPLIT ? NTH / 2 : NTH;               // threads on S, threads on V
                constexpr int NSB = HALF * HALF / NS;                   // blocks per thread
                constexpr int SB = NSB < 4 ? NSB : 4;                   // blocks per batch
                constexpr int JSTEP = NS / HALF;
                constexpr int NVB = KC * HALF / NS;                     // items per thread
                constexpr int VB = NVB < 8 ? NVB : 8;
                constexpr int VSTEP = NS / KC;
                static_assert(NSB >= 1 && NVB >= 1 && NS % HALF == 0 && NS % KC == 0, "thread counts");
                if (!SPLIT || tid < NS) {
                    const RotEntry r2 = rot[tid & (HALF - 1)];
                    const float *c0 = S + r2.p, *c1p = S + r2.q;
                    for (int t0 = 0; t0 < NSB; t0 += SB) {
                        RotEntry r1[SB];
                        float a[SB], b[SB], c_[SB], d[SB];
#pragma unroll
                        for (int u = 0; u < SB; ++u) {
                            r1[u] = rot[tid / HALF + JSTEP * (t0 + u)];
                            a[u] = c0[r1[u].p * ld]; b[u] = c1p[r1[u].p * ld];
                            c_[u] = c0[r1[u].q * ld]; d[u] = c1p[r1[u].q * ld];
                        }
#pragma unroll
                        for (int u = 0; u < SB; ++u) {
                            // columns: [a b; c d] * [[c2, s2], [-s2, c2]], then rows: [[c1, -s1], [s1, c1]] * [...]
                            const float a1 = r2.c * a[u] - r2.s * b[u], b1 = r2.s * a[u] + r2.c * b[u];
                            const float cc1 = r2.c * c_[u] - r2.s * d[u], d1 = r2.s * c_[u] + r2.c * d[u];
                            S[r1[u].p * ld + r2.p] = r1[u].c * a1 - r1[u].s * cc1;
                            S[r1[u].p * ld + r2.q] = r1[u].c * b1 - r1[u].s * d1;
                            S[r1[u].q * ld + r2.p] = r1[u].s * a1 + r1[u].c * cc1;
                            S[r1[u].q * ld + r2.q] = r1[u].s * b1 + r1[u].c * d1;
                        }
                    }
                }
                if (!SPLIT || tid >= NS) {
                    const int vt = SPLIT ? tid - NS : tid;
                    float *vrow = V + (vt & (KC - 1)) * ld;
                    for (int t0 = 0; t0 < NVB; t0 += VB) {
                        RotEntry rc[VB];
                        float vp[VB], vq[VB];
#pragma unroll
                        for (int u = 0; u < VB; ++u) {
                            rc[u] = rot[vt / KC + VSTEP * (t0 + u)];
                            vp[u] = vrow[rc[u].p]; vq[u] = vrow[rc[u].q];
                        }
#pragma unroll
                        for (int u = 0; u < VB; ++u) {
                            vrow[rc[u].p] = rc[u].c * vp[u] - rc[u].s * vq[u];
                            vrow[rc[u].q] = rc[u].s * vp[u] + rc[u].c * vq[u];
                        }
                    }
                }
            } else {
                for (int e = tid; e < half * half; e += NT) {
                    const int j1 = e / half, j2 = e - j1 * half;
                    const RotEntry r1 = rot[j1], r2 = rot[j2];
                    float a = S[r1.p * ld + r2.p], b = S[r1.p * ld + r2.q], c_ = S[r1.q * ld + r2.p], d = S[r1.q * ld + r2.q];
                    const float a1 = r2.c * a - r2.s * b, b1 = r2.s * a + r2.c * b;
                    const float cc1 = r2.c * c_ - r2.s * d, d1 = r2.s * c_ + r2.c * d;
                    S[r1.p * ld + r2.p] = r1.c * a1 - r1.s * cc1;
                    S[r1.p * ld + r2.q] = r1.c * b1 - r1.s * d1;
                    S[r1.q * ld + r2.p] = r1.s * a1 + r1.c * cc1;
                    S[r1.q * ld + r2.q] = r1.s * b1 + r1.c * d1;
                }
                for (int e = tid; e < k * half; e += NT) {
                    const int j = e / k, i = e - j * k;
                    const RotEntry rc = rot[j];
                    const float vp = V[i * ld + rc.p], vq = V[i * ld + rc.q];
                    V[i * ld + rc.p] = rc.c * vp - rc.s * vq;
                    V[i * ld + rc.q] = rc.s * vp + rc.c * vq;
                }
            }
            __syncthreads();
        }
    }
    res.rotations = *rotflag;
    return res;
}

// Dynamic LDS layout shared by the small solver and the pivot solver (auxiliary arrays sized for 128).
struct JacobiSmem {
    float *S, *V, *red;
    RotEntry *rot;
    int *rotflag, *rank;
    float *diag;
    __device__ JacobiSmem(char *base, int k, int ld) {
        S = (float *)base;
        V = S + k * ld;
        red = V + k * ld;
        rot = (RotEntry *)(red + 16);
        rotflag = (int *)(rot + SMALL_MAX / 2);
        rank = rotflag + 4;
        diag = (float *)(rank + SMALL_MAX);
    }
    static size_t bytes(int k, int ld) {
        return ((size_t)2 * k * ld + 16 + 4 * (SMALL_MAX / 2) + 4 + 2 * SMALL_MAX) * sizeof(float);
    }
};

// ---- Newton-Schulz step V <- V (3I - V^T V)/2 in LDS ------------------------------------------------
// Hundreds of fp32 rotations leave V orthogonal only to ~1e-6; one step restores ~1e-7.

// KP x KP x KP product on LDS operands for the pivot size: acc = A * B, A(m,k) = Am[m*am + k*ak],
// B(k,n) = Bm[k*PLD + n].  KP = 128: 2x2 accumulators per wave; KP = 64: one (acc[0][0]).
__device__ inline void lds_gemm_pivot(const float *Am, int am, int ak, const float *Bm, floatx16 (&acc)[2][2]) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int Q = KP / 2;   // quadrant edge per wave
    const int wm = (wave >> 1) * Q, wn = (wave & 1) * Q;
    const int lk = lane >> 5, lc = lane & 31;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
#pragma unroll 4
    for (int kk = 0; kk < KP; kk += 2) {
        const float a0 = Am[(wm + lc) * am + (kk + lk) * ak];
        const float b0 = Bm[(kk + lk) * PLD + wn + lc];
        acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
        if (KP == 128) {
            const float a1 = Am[(wm + 32 + lc) * am + (kk + lk) * ak];
            const float b1 = Bm[(kk + lk) * PLD + wn + 32 + lc];
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
        }
    }
}

// f(row, col, value) over this thread's elements of the pivot-sized accumulators.
template <class F>
__device__ inline void for_each_pivot_acc(const floatx16 (&acc)[2][2], F f) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int Q = KP / 2, NI = KP / 64;
    const int wm = (wave >> 1) * Q, wn = (wave & 1) * Q;
    const int lk = lane >> 5, lc = lane & 31;
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                f(wm + 32 * i + 8 * (r >> 2) + 4 * lk + (r & 3), wn + 32 * j + lc, acc[i][j][r]);
}

// Called by the whole workgroup; the first four waves do the products.
__device__ void polish_pivot_mfma(float *V, float *Y) {
    const bool act = threadIdx.x < NT;
    floatx16 acc[2][2];
    if (act) {
        lds_gemm_pivot(V, 1, PLD, V, acc);  // V^T V
        for_each_pivot_acc(acc, [&](int r, int c, float v) { Y[r * PLD + c] = (r == c ? 1.5f : 0.f) - 0.5f * v; });
    }
    __syncthreads();
    if (act) lds_gemm_pivot(V, PLD, 1, Y, acc);  // V Y
    __syncthreads();
    if (act) for_each_pivot_acc(acc, [&](int r, int c, float v) { V[r * PLD + c] = v; });
    __syncthreads();
}

// The same step with plain FMAs for a run-time size k <= 128 (Y is k x k scratch, same pitch).
__device__ void polish_lds_valu(float *V, float *Y, int k, int ld) {
    const int tid = threadIdx.x;
    for (int e = tid; e < k * k; e += NT) {
        const int i = e / k, j = e - i * k;
        float s = 0.f;
        for (int r = 0; r < k; ++r) s = fmaf(V[r * ld + i], V[r * ld + j], s);
        Y[i * ld + j] = (i == j ? 1.5f : 0.f) - 0.5f * s;
    }
    __syncthreads();
    float out[SMALL_MAX * SMALL_MAX / NT];
#pragma unroll
    for (int t = 0; t < SMALL_MAX * SMALL_MAX / NT; ++t) {
        const int e = tid + t * NT;
        float s = 0.f;
        if (e < k * k) {
            const int i = e / k, j = e - i * k;
            for (int r = 0; r < k; ++r) s = fmaf(V[i * ld + r], Y[r * ld + j], s);
        }
        out[t] = s;
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < SMALL_MAX * SMALL_MAX / NT; ++t) {
        const int e = tid + t * NT;
        if (e < k * k) V[(e / k) * ld + (e % k)] = out[t];
    }
    __syncthreads();
}

// ------------------------------------------------------------------------------------------------
// d <= 128: whole factor in LDS
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(NT) void eig_small_kernel(const SmallItem *items, EigStat *stats, int max_sweeps,
                                                       float tol) {
    extern __shared__ __align__(16) char smem[];
    const SmallItem it = items[blockIdx.x];
    const int n = it.n;
    const int k = (n + 1) & ~1;
    const int ld = k + 1;
    JacobiSmem sm(smem, k, ld);
    const int tid = threadIdx.x;
    for (int e = tid; e < k * k; e += NT) {
        const int i = e / k, j = e - i * k;
        sm.S[i * ld + j] = (i < n && j < n) ? it.F[(int64_t)i * n + j] : 0.f;
        sm.V[i * ld + j] = (i == j) ? 1.f : 0.f;
    }
    __syncthreads();
    const JacobiResult res = jacobi_lds<0>(sm.S, sm.V, k, ld, max_sweeps, tol, 1e-9f, sm.red, sm.rot, sm.rotflag);
    if (!(res.nrm2 < INFINITY)) {
        // non-finite input: nothing was rotated (every comparison with a NaN fails); say so in every output element
        const float nan = __uint_as_float(0x7fc00000u);
        for (int i = tid; i < n; i += NT) it.lam[i] = nan;
        for (int e = tid; e < n * n; e += NT) it.Q[e] = nan;
        if (tid == 0) stats[blockIdx.x] = EigStat{(float)res.sweeps, nan, 0.f, 0.f};
        return;
    }
    for (int i = tid; i < k; i += NT) sm.diag[i] = sm.S[i * ld + i];
    __syncthreads();
    if (res.rotations > 0) polish_lds_valu(sm.V, sm.S, k, ld);
    // rank of every eigenvalue (ascending, ties by index)
    for (int i = tid; i < n; i += NT) {
        const float li = sm.diag[i];
        int rank = 0;
        for (int j = 0; j < n; ++j) {
            const float lj = sm.diag[j];
            rank += (lj < li) || (lj == li && j < i);
        }
        sm.rank[i] = rank;
        it.lam[rank] = li;
    }
    __syncthreads();
    for (int e = tid; e < n * n; e += NT) {
        const int i = e / n, j = e - i * n;
        it.Q[(int64_t)i * n + sm.rank[j]] = sm.V[i * ld + j];
    }
    if (tid == 0) {
        EigStat st;
        st.sweeps = (float)res.sweeps;
        st.off_rel = res.nrm2 > 0.f ? sqrtf(res.off2 / res.nrm2) : 0.f;
        st.converged = (res.off2 <= tol * tol * res.nrm2) ? 1.f : 0.f;
        st.rotations = (float)res.rotations;
        stats[blockIdx.x] = st;
    }
}

// ------------------------------------------------------------------------------------------------
// d > 128: blocked path.  Per group of `nmat` factors with `nblk` EB-wide blocks (npad = EB*nblk):
//   W  [nmat][npad][npad]   rotated matrix         Qw [nmat][npad][npad]  accumulated eigenvectors
//   J  [nmat][npairs][KP][KP] pivot transforms     idt[nmat][npairs]      1 = transform is identity
// ------------------------------------------------------------------------------------------------
struct BlkGroup {
    float *W, *Qw, *J;
    int *idt;
    double *norms;   // [nmat][2] = off^2, diag^2
    int nmat, nblk, npad, players, npairs;
    int bipartite;   // 0: tournament over all blocks; 1: block j of the first half with a block of the second
    const int *done; // [factors]: 1 once a factor has met the tolerance; its workgroups return at once
    int per_factor;  // matrices of this group per factor (units of a two-level group; 1 otherwise)
    // Unit mode (the inner rounds of a two-level group): matrix m is unit m % per_factor of factor m / per_factor, W points
    // to the factors' full matrices [factors][ldw][ldw] and the unit's small blocks are rotated in place there (block b
    // of the unit is quarter b % 4 of super-block b0 (b < 4) or b1 of the outer round's pair), while Qw is the unit's own
    // compact accumulator [nmat][npad][npad].
    int unit_mode, ldw, outer_round, sp_players, sp_nsuper;
    int qw_identity;        // the accumulator is taken to be the identity instead of being read (first inner round)
    int qw_minus_identity;  // the identity is subtracted from the accumulator as it is written (last inner round)
};
__device__ inline bool blk_done(const BlkGroup &g, int m) { return g.done[m / g.per_factor] != 0; }

// Where matrix m of a group lives: base pointer and leading dimension of the matrix its blocks are part of, and
// (unit mode) the two super-blocks of the unit, -1 for an absent one.
struct BlkWhere { float *W; int64_t ld; int b0, b1; };
__device__ inline BlkWhere blk_where(const BlkGroup &g, int m) {
    BlkWhere w;
    if (!g.unit_mode) {
        w.W = g.W + (int64_t)m * g.npad * g.npad;
        w.ld = g.npad;
        w.b0 = w.b1 = 0;
        return w;
    }
    const int f = m / g.per_factor, u = m - f * g.per_factor;
    w.W = g.W + (int64_t)f * g.ldw * g.ldw;
    w.ld = g.ldw;
    if (g.outer_round < 0) { w.b0 = u; w.b1 = -1; }      // diagonal phase: super-block u alone
    else {
        int p, q;
        rr_pair(g.sp_players, g.outer_round, u, p, q);
        w.b0 = p;
        w.b1 = q < g.sp_nsuper ? q : -1;
    }
    return w;
}

// Pair j of round `round`: tournament over `players` blocks, or (bipartite) block j with block
// half + (j + round) % half, which meets every cross pair of the two halves in `half` rounds.
__device__ inline void sched_pair(const BlkGroup &g, int round, int j, int &p, int &q) {
    if (g.bipartite) {
        const int half = g.players >> 1;
        p = j;
        q = half + (j + round) % half;
    } else {
        rr_pair(g.players, round, j, p, q);
    }
}
struct BlkItem { const float *F; float *Q; float *lam; int n; int pad_; };

// W <- F (zero padded), accumulator <- I, or with `warm` <- the basis the caller left in Q (identity on the padding).
__global__ void blk_init_kernel(BlkGroup g, const BlkItem *items, int warm) {
    const int m = blockIdx.y;
    const BlkItem it = items[m];
    const int64_t np2 = (int64_t)g.npad * g.npad;
    float *W = g.W + m * np2, *Qw = g.Qw + m * np2;
    for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < np2; e += (int64_t)gridDim.x * blockDim.x) {
        const int i = (int)(e / g.npad), j = (int)(e - (int64_t)i * g.npad);
        const bool in = i < it.n && j < it.n;
        W[e] = in ? it.F[(int64_t)i * it.n + j] : 0.f;
        Qw[e] = (warm && in) ? it.Q[(int64_t)i * it.n + j] : ((i == j) ? 1.f : 0.f);
    }
}

// W <- (W + W^T) / 2 inside the 128 x 128 tiles on the diagonal, for every factor of a group (blockIdx.y).  It follows
// a symmetric product (gemm_batched_kernel with SYM), whose tiles below the diagonal and their mirror images agree
// to the last bit already; only a diagonal tile computes both of its halves, each with its own rounding.
__global__ __launch_bounds__(NT) void blk_symmetrise_tiles_kernel(float *W, int64_t stride, int64_t ld, const BlkItem *items) {
    const int n = items[blockIdx.y].n;
    float *Wm = W + blockIdx.y * stride;
    const int64_t count = (int64_t)n * kfac::BM;
    for (int64_t e = blockIdx.x * (int64_t)NT + threadIdx.x; e < count; e += (int64_t)gridDim.x * NT) {
        const int i = (int)(e / kfac::BM), j = (i / kfac::BM) * kfac::BM + (int)(e % kfac::BM);
        if (j >= i) continue;
        const float v = 0.5f * (Wm[(int64_t)i * ld + j] + Wm[(int64_t)j * ld + i]);
        Wm[(int64_t)i * ld + j] = v;
        Wm[(int64_t)j * ld + i] = v;
    }
}

// Squared Frobenius norms of the off-diagonal and of the diagonal part of every matrix of a group, in two
// steps whose summation order is fixed (the eigenvalues' stopping decision is then the same run to run):
// workgroup (b, m) leaves its share in part[m][b][2], one workgroup per matrix adds the shares in order.
constexpr int NORM_PARTS_MAX = 512;

__global__ __launch_bounds__(NT) void blk_offnorm_kernel(BlkGroup g, double *part) {
    __shared__ float red[8];
    const int m = blockIdx.y;
    const int64_t np2 = (int64_t)g.npad * g.npad;
    const float *W = g.W + m * np2;
    float o2 = 0.f, d2 = 0.f;
    for (int64_t e = blockIdx.x * (int64_t)NT + threadIdx.x; e < np2; e += (int64_t)gridDim.x * NT) {
        const int i = (int)(e / g.npad), j = (int)(e - (int64_t)i * g.npad);
        const float v = W[e];
        if (i == j) d2 += v * v; else o2 += v * v;
    }
    o2 = block_sum(o2, red);
    d2 = block_sum(d2, red);
    if (threadIdx.x == 0) {
        double *dst = part + ((int64_t)m * gridDim.x + blockIdx.x) * 2;
        dst[0] = (double)o2;
        dst[1] = (double)d2;
    }
}

// norms[m] = (off^2, diag^2) from the nparts shares of matrix m; done[m] = 1 when the factor has met the
// tolerance (the host applies the same test to the same sums) or its norms are not finite (nothing more
// can be done for it: its workgroups return at once from then on).
__global__ __launch_bounds__(NT) void blk_norm_reduce_kernel(const double *part, int nparts, double *norms, int *done, double tol2) {
    __shared__ double so[NT], sd[NT];
    const int m = blockIdx.x, t = threadIdx.x;
    const double *src = part + (int64_t)m * nparts * 2;
    double o = 0.0, d = 0.0;
    for (int i = t; i < nparts; i += NT) { o += src[2 * i]; d += src[2 * i + 1]; }
    so[t] = o;
    sd[t] = d;
    __syncthreads();
    for (int w = NT / 2; w > 0; w >>= 1) {
        if (t < w) { so[t] += so[t + w]; sd[t] += sd[t + w]; }
        __syncthreads();
    }
    if (t == 0) {
        const double o2 = so[0], n2 = so[0] + sd[0];
        norms[2 * m] = o2;
        norms[2 * m + 1] = sd[0];
        done[m] = !(o2 > tol2 * n2) ? 1 : 0;
    }
}

// Row/column index in the padded matrix of element a (0..KP-1) of the pair (p, q); -1 if the block is
// the phantom one that completes an odd block count.
__device__ inline int pair_index(int a, int p, int q, int nblk) {
    const int blk = a < EB ? p : q;
    return blk < nblk ? blk * EB + (a & (EB - 1)) : -1;
}
// The same inside the matrix the group's W points to: in unit mode small block b of the unit is quarter b % 4 of
// super-block b0 (b < 4) or b1 (128-wide super-blocks of four small blocks).
__device__ inline int blk_index(const BlkGroup &g, const BlkWhere &w, int a, int p, int q) {
    if (!g.unit_mode) return pair_index(a, p, q, g.nblk);
    const int blk = a < EB ? p : q;
    if (blk >= g.nblk) return -1;
    const int sb = blk < 4 ? w.b0 : w.b1;
    return sb < 0 ? -1 : sb * (4 * EB) + (blk & 3) * EB + (a & (EB - 1));
}

// One sweep of the LDS Jacobi solver over the pivot sub-problem of every pair of this round; writes
// the accumulated (and re-orthogonalised) transform J and whether it is the identity.
constexpr int SOLVE_NT = 512;    // threads of a pivot solve: half of them rotate S, the other half V (more threads
                                 // are no faster, and a smaller workgroup leaves room for other groups' kernels)

__global__ __launch_bounds__(SOLVE_NT) void blk_solve_kernel(BlkGroup g, int round, int inner_sweeps, float inner_tol) {
    extern __shared__ __align__(16) char smem[];
    JacobiSmem sm(smem, KP, PLD);
    const int m = blockIdx.y, pj = blockIdx.x, tid = threadIdx.x;
    if (blk_done(g, m)) return;
    const BlkWhere wh = blk_where(g, m);
    const float *W = wh.W;
    int p, q;
    sched_pair(g, round, pj, p, q);
    constexpr int PER = KP * KP / SOLVE_NT;
    float v[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int e = tid + SOLVE_NT * u;
        const int a = e / KP, b = e % KP;
        const int gi = blk_index(g, wh, a, p, q), gj = blk_index(g, wh, b, p, q);
        // read the lower triangle only, so the sub-problem is exactly symmetric
        v[u] = 0.f;
        if (gi >= 0 && gj >= 0) v[u] = (gi >= gj) ? W[(int64_t)gi * wh.ld + gj] : W[(int64_t)gj * wh.ld + gi];
    }
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int e = tid + SOLVE_NT * u;
        const int a = e / KP, b = e % KP;
        sm.S[a * PLD + b] = v[u];
        sm.V[a * PLD + b] = (a == b) ? 1.f : 0.f;
    }
    __syncthreads();
    // The pairs inside a block need one visit per sweep: a tournament gives it in its round 0 (where every
    // block plays, possibly against the phantom), a bipartite schedule leaves it to its caller.  Every
    // other visit rotates only the pairs between the two blocks.
    const JacobiResult res =
        (g.bipartite || round > 0) ? jacobi_lds<KP, true, SOLVE_NT, false>(sm.S, sm.V, KP, PLD, inner_sweeps, inner_tol, 1e-9f, sm.red, sm.rot, sm.rotflag)
                                   : jacobi_lds<KP, false, SOLVE_NT, false>(sm.S, sm.V, KP, PLD, inner_sweeps, inner_tol, 1e-9f, sm.red, sm.rot, sm.rotflag);
    if (res.rotations > 0) polish_pivot_mfma(sm.V, sm.S);
    float *J = g.J + ((int64_t)m * g.npairs + pj) * (KP * KP);
    for (int e = tid; e < KP * KP; e += SOLVE_NT) J[e] = sm.V[(e / KP) * PLD + (e % KP)];
    if (tid == 0) g.idt[m * g.npairs + pj] = res.rotations == 0;
}

__device__ inline void tri_decode(int idx, int &ti, int &tj) {
    int t = (int)((sqrtf(8.f * (float)idx + 1.f) - 1.f) * 0.5f);
    while ((t + 1) * (t + 2) / 2 <= idx) ++t;
    while (t * (t + 1) / 2 > idx) --t;
    ti = t;
    tj = idx - t * (t + 1) / 2;
}

// ---- round application ---------------------------------------------------------------------------
// One workgroup per KP x KP block of pivot pairs: block (I, J) of W becomes J_I^T W_IJ J_J (pairs I >= J;
// the mirror image is written from LDS, so W stays exactly symmetric), and every KP-row slab of the
// accumulator is multiplied by the transform of its column pair.  The work of a round is bound by latency,
// not by arithmetic, so the blocks are small and many share a compute unit (17 KB of LDS, one 32 x 32
// accumulator per wave): the transforms are read from global memory (L2) straight into MFMA operand
// registers while the block itself is on its way into LDS.
constexpr int BLD = KP + 1;          // LDS pitch of a block
static_assert(KP == 64, "the block application assumes 64 x 64 pivots (four 32 x 32 wave quadrants)");

// acc = A * B over KP: A(m,k) from LDS (Xs[m][k]) and B(k,n) in registers (bj[j] = B[2j + lk][n]), or
// A(m,k) in registers (aj[j] = A[m][2j + lk]) and B(k,n) from LDS (Xs[k][n]).
template <bool A_IN_LDS>
__device__ inline floatx16 block_gemm(const float *Xs, const float (&reg)[KP / 2], int wm, int wn, int lk, int lc) {
    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
    for (int j = 0; j < KP / 2; ++j) {
        const int k = 2 * j + lk;
        if (A_IN_LDS) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(Xs[(wm + lc) * BLD + k], reg[j], acc, 0, 0, 0);
        else acc = __builtin_amdgcn_mfma_f32_32x32x2f32(reg[j], Xs[k * BLD + wn + lc], acc, 0, 0, 0);
    }
    return acc;
}

// Block <-> global memory, four consecutive columns per access.  rowf(a) / colf(b) give the global row and
// column of block row a / block column b (b a multiple of 4; the four columns are contiguous), or -1.
// G is uniform over the workgroup (buffer accesses: a block row or column outside the matrix is given an offset the
// range check rejects, which reads zeros and drops the store -- no branch around any access).
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
template <class RowF, class ColF>
__device__ inline void block_load(float *Xs, const float *G, int64_t ld, RowF rowf, ColF colf) {
    const __amdgpu_buffer_rsrc_t rs = kfac::buffer_at(G);
    uintx4 v[KP * KP / 4 / NT];
#pragma unroll
    for (int u = 0; u < KP * KP / 4 / NT; ++u) {
        const int e4 = threadIdx.x + NT * u;
        const int a = e4 >> 4, b = (e4 & 15) * 4;
        const int gi = rowf(a), gj = colf(b);
        const unsigned off = (gi >= 0 && gj >= 0) ? (unsigned)(((int64_t)gi * ld + gj) * 4) : kfac::BUF_OUTSIDE;
        v[u] = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < KP * KP / 4 / NT; ++u) {
        const int e4 = threadIdx.x + NT * u;
        float *dst = Xs + (e4 >> 4) * BLD + (e4 & 15) * 4;
        dst[0] = __uint_as_float(v[u].x); dst[1] = __uint_as_float(v[u].y); dst[2] = __uint_as_float(v[u].z); dst[3] = __uint_as_float(v[u].w);
    }
}

// TRANSPOSED: write Xs^T, i.e. global (colf(b), rowf(a..a+3)) <- Xs[a..a+3][b].
template <bool TRANSPOSED, class RowF, class ColF>
__device__ inline void block_store(const float *Xs, float *G, int64_t ld, RowF rowf, ColF colf) {
    const __amdgpu_buffer_rsrc_t rs = kfac::buffer_at(G);
#pragma unroll
    for (int u = 0; u < KP * KP / 4 / NT; ++u) {
        const int e4 = threadIdx.x + NT * u;
        if (!TRANSPOSED) {
            const int a = e4 >> 4, b = (e4 & 15) * 4;
            const int gi = rowf(a), gj = colf(b);
            const float *src = Xs + a * BLD + b;
            const unsigned off = (gi >= 0 && gj >= 0) ? (unsigned)(((int64_t)gi * ld + gj) * 4) : kfac::BUF_OUTSIDE;
            const uintx4 q = {__float_as_uint(src[0]), __float_as_uint(src[1]), __float_as_uint(src[2]), __float_as_uint(src[3])};
            __builtin_amdgcn_raw_buffer_store_b128(q, rs, off, 0, 0);
        } else {
            const int b = e4 >> 4, a = (e4 & 15) * 4;
            const int gi = rowf(a), gj = colf(b);
            const float *src = Xs + a * BLD + b;
            const unsigned off = (gi >= 0 && gj >= 0) ? (unsigned)(((int64_t)gj * ld + gi) * 4) : kfac::BUF_OUTSIDE;
            const uintx4 q = {__float_as_uint(src[0]), __float_as_uint(src[BLD]), __float_as_uint(src[2 * BLD]), __float_as_uint(src[3 * BLD])};
            __builtin_amdgcn_raw_buffer_store_b128(q, rs, off, 0, 0);
        }
    }
}

__device__ inline void acc_to_block(const floatx16 &acc, float *Xs, int wm, int wn, int lk, int lc) {
#pragma unroll
    for (int r = 0; r < 16; ++r) Xs[(wm + 8 * (r >> 2) + 4 * lk + (r & 3)) * BLD + wn + lc] = acc[r];
}

// grid.x: nblocks_w lower-triangular blocks of W, then ceil(nrb / 2) pairs of row slabs x npairs column pairs of the
// accumulator.  A workgroup of the accumulator part takes TWO 64-row slabs of one column pair: the transform is read
// once for both, both blocks travel to LDS together, and the barriers of the three phases are shared -- the launch of
// a unit-mode round (54 units x 18 instead of 26 workgroups) then fits the machine in one go.
// (waves_per_eu(4): with the register budget of four waves per SIMD the compiler keeps both transforms and the
// staged block in flight; left to itself it aims at six, and the flat groups' rounds take 8 % longer)
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(4))) void blk_apply_kernel(BlkGroup g, int round, int nblocks_w, int nrb) {
    __shared__ float Xs2[2][KP * BLD];
    float *const Xs = Xs2[0];
    const int m = blockIdx.y;
    if (blk_done(g, m)) return;
    const int64_t np2 = (int64_t)g.npad * g.npad;
    const int *idt = g.idt + m * g.npairs;
    const float *Jall = g.J + (int64_t)m * g.npairs * (KP * KP);
    const int nblk = g.nblk;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave >> 1) * 32, wn = (wave & 1) * 32, lk = lane >> 5, lc = lane & 31;
    if ((int)blockIdx.x < nblocks_w) {
        const BlkWhere wh = blk_where(g, m);
        float *W = wh.W;
        int I, Jp;
        tri_decode(blockIdx.x, I, Jp);
        const bool idI = idt[I] != 0, idJ = idt[Jp] != 0;
        if (idI && idJ) return;
        int pI, qI, pJ, qJ;
        sched_pair(g, round, I, pI, qI);
        sched_pair(g, round, Jp, pJ, qJ);
        auto rowf = [&](int a) { return blk_index(g, wh, a, pI, qI); };
        auto colf = [&](int b) { return blk_index(g, wh, b, pJ, qJ); };
        // operands of both products in registers: bj[j] = J_J[2j + lk][wn + lc], aj[j] = J_I[2j + lk][wm + lc]
        float bj[KP / 2], aj[KP / 2];
        const float *Jc = Jall + (int64_t)Jp * (KP * KP) + wn + lc, *Jr = Jall + (int64_t)I * (KP * KP) + wm + lc;
#pragma unroll
        for (int j = 0; j < KP / 2; ++j) bj[j] = Jc[(2 * j + lk) * KP];
        block_load(Xs, W, wh.ld, rowf, colf);
#pragma unroll
        for (int j = 0; j < KP / 2; ++j) aj[j] = Jr[(2 * j + lk) * KP];
        __syncthreads();
        if (!idJ) {
            const floatx16 t = block_gemm<true>(Xs, bj, wm, wn, lk, lc);    // T = X J_J
            __syncthreads();
            acc_to_block(t, Xs, wm, wn, lk, lc);
            __syncthreads();
        }
        if (!idI) {
            const floatx16 w = block_gemm<false>(Xs, aj, wm, wn, lk, lc);   // W' = J_I^T T
            __syncthreads();
            acc_to_block(w, Xs, wm, wn, lk, lc);
            __syncthreads();
        }
        if (I == Jp) {
            // a diagonal block holds both halves of itself: keep the lower one
            for (int e = threadIdx.x; e < KP * KP; e += NT) {
                const int a = e >> 6, b = e & 63;
                if (b > a) Xs[a * BLD + b] = Xs[b * BLD + a];
            }
            __syncthreads();
        }
        block_store<false>(Xs, W, wh.ld, rowf, colf);
        if (I != Jp) block_store<true>(Xs, W, wh.ld, rowf, colf);
    } else {
        float *Qw = g.Qw + m * np2;
        const int t = blockIdx.x - nblocks_w;
        const int nrb2 = (nrb + 1) >> 1;
        const int rb2 = t % nrb2, Jp = t / nrb2;
        // an identity transform leaves the accumulator as it is -- unless this launch also starts it or takes the
        // identity off it, which every block has to see
        if (idt[Jp] && !g.qw_identity && !g.qw_minus_identity) return;
        int pJ, qJ;
        sched_pair(g, round, Jp, pJ, qJ);
        const int npad = g.npad;
        const int nslab = 2 * rb2 + 1 < nrb ? 2 : 1;   // uniform over the workgroup
        auto colf = [&](int b) { return pair_index(b, pJ, qJ, nblk); };
        float bj[KP / 2];
        const float *Jc = Jall + (int64_t)Jp * (KP * KP) + wn + lc;
#pragma unroll
        for (int j = 0; j < KP / 2; ++j) bj[j] = Jc[(2 * j + lk) * KP];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            if (h >= nslab) break;
            const int row0 = (2 * rb2 + h) * KP;
            auto rowf = [&](int a) { return row0 + a < npad ? row0 + a : -1; };
            if (g.qw_identity) {
                for (int e = threadIdx.x; e < KP * KP; e += NT) {
                    const int a = e >> 6, b = e & 63;
                    Xs2[h][a * BLD + b] = (row0 + a == colf(b)) ? 1.f : 0.f;
                }
            } else {
                block_load(Xs2[h], Qw, g.npad, rowf, colf);
            }
        }
        __syncthreads();
        floatx16 t2[2];
#pragma unroll
        for (int h = 0; h < 2; ++h)
            if (h < nslab) t2[h] = block_gemm<true>(Xs2[h], bj, wm, wn, lk, lc);
        __syncthreads();
#pragma unroll
        for (int h = 0; h < 2; ++h)
            if (h < nslab) acc_to_block(t2[h], Xs2[h], wm, wn, lk, lc);
        __syncthreads();
        if (g.qw_minus_identity) {
            for (int h = 0; h < nslab; ++h) {
                const int row0 = (2 * rb2 + h) * KP;
                for (int e = threadIdx.x; e < KP * KP; e += NT) {
                    const int a = e >> 6, b = e & 63;
                    if (row0 + a == colf(b)) Xs2[h][a * BLD + b] -= 1.f;
                }
            }
            __syncthreads();
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            if (h >= nslab) break;
            const int row0 = (2 * rb2 + h) * KP;
            auto rowf = [&](int a) { return row0 + a < npad ? row0 + a : -1; };
            block_store<false>(Xs2[h], Qw, g.npad, rowf, colf);
        }
    }
}

// ---- post-processing of a converged factor -------------------------------------------------------
// Y = (3I - Q^T Q)/2 : epilogue of the Newton-Schulz orthogonalisation step Q <- Q Y.
struct EpiNewtonSchulz {
    float *Y;
    int64_t ld;
    __device__ void operator()(int r, int c, float v) const { Y[(int64_t)r * ld + c] = (r == c ? 1.5f : 0.f) - 0.5f * v; }
};

// The same step on the split-fp16 engine, in delta form: D = (I - Q^T Q)/2 (entries of the size of the accumulated
// rounding, 1e-6), then Q + Q D with the first term added in fp32 -- the split engine's 2^-22 then applies to a
// correction that is itself 1e-6 of Q.  Operands are scaled by 2^14 (entries of Q and D are below 1).
struct EpiNewtonSchulzDelta {
    float *D;
    int64_t ld;
    __device__ void operator()(int r, int c, float v) const { D[(int64_t)r * ld + c] = (r == c ? 0.5f : 0.f) - 0.5f * v; }
};
struct EpiAddStore {
    const float *X;
    int64_t ldx;
    float *C;
    int64_t ldc;
    __device__ void operator()(int r, int c, float v) const { C[(int64_t)r * ldc + c] = X[(int64_t)r * ldx + c] + v; }
};
// ---- n x n products for every factor of a group in one launch (blockIdx.z: factor; y, x: row and column tile) ----
// The post-processing and refresh products of the mid-size factors are a few hundred tiles each, half a machine at
// best; launched one factor after another they left it half empty (and the flat groups' 25-tile products nearly
// idle).  An operand is one of the group's buffers (factor z at base + z * stride, the group's pitch) or one of the
// caller's arrays of that factor (F or Q, pitch n), looked up in the group's item table.
struct BatchOperand {
    const float *base;
    int64_t stride;
    int kind;   // 0: group buffer, 1: the caller's F, 2: the caller's Q
};
__device__ inline float *batch_ptr(const BatchOperand &o, const BlkItem &it, int z, int64_t ldg, int64_t &ld) {
    if (o.kind == 0) {
        ld = ldg;
        return const_cast<float *>(o.base) + z * o.stride;
    }
    ld = it.n;
    return o.kind == 1 ? const_cast<float *>(it.F) : it.Q;
}
enum { EPI_STORE, EPI_NS, EPI_NS_DELTA, EPI_ADD_STORE };
template <int EPI> struct EpiOf;
template <> struct EpiOf<EPI_STORE> { using type = kfac::EpiStore; };
template <> struct EpiOf<EPI_NS> { using type = EpiNewtonSchulz; };
template <> struct EpiOf<EPI_NS_DELTA> { using type = EpiNewtonSchulzDelta; };
template <> struct EpiOf<EPI_ADD_STORE> { using type = EpiAddStore; };
template <int EPI>
__device__ inline typename EpiOf<EPI>::type make_epi(float *c, int64_t ldc, const float *x, int64_t ldx) {
    if constexpr (EPI == EPI_ADD_STORE) return EpiAddStore{x, ldx, c, ldc};
    else return typename EpiOf<EPI>::type{c, ldc};
}
// C = A B (elem(i,k) operands; AK / BK: the contraction index is the fast one in memory) on the fp32 engine, or with X3
// on the split-fp16 engine (operands scaled by sc, result by out_scale).  SYM: the product is known to be symmetric;
// tiles above the diagonal return at once and every tile below it also delivers its mirror image, epi(col, row,
// value) -- half the matrix-core work, and the two halves agree to the last bit.
template <bool AK, bool BK, int EPI, bool SYM, bool X3>
__global__ __launch_bounds__(kfac::NTHREADS) __attribute__((amdgpu_waves_per_eu(2))) void gemm_batched_kernel(BatchOperand A, BatchOperand B, BatchOperand C,
                                                                                                            BatchOperand X, const BlkItem *items,
                                                                                                            int64_t ldg, float sc, float out_scale) {
    using namespace kfac;
    __shared__ typename std::conditional<X3, X3Smem, TileSmem>::type sm;
    const int z = blockIdx.z;
    const BlkItem it = items[z];
    const int n = it.n;
    const int i0 = blockIdx.y * BM, j0 = blockIdx.x * BM;
    if (i0 >= n || j0 >= n || (SYM && j0 > i0)) return;
    int64_t lda, ldb, ldc, ldx = 0;
    const float *pa = batch_ptr(A, it, z, ldg, lda), *pb = batch_ptr(B, it, z, ldg, ldb);
    float *pc = batch_ptr(C, it, z, ldg, ldc);
    const float *px = EPI == EPI_ADD_STORE ? batch_ptr(X, it, z, ldg, ldx) : nullptr;
    const auto epi = make_epi<EPI>(pc, ldc, px, ldx);
    floatx16 acc[2][2];
    if constexpr (X3) {
        X3OpG<float, AK> a{pa, lda, sc, n, n};
        X3OpG<float, BK> b{pb, ldb, sc, n, n};
        a.start(threadIdx.x, i0);
        b.start(threadIdx.x, j0);
        gemm_tile_x3(a, b, n, sm, acc);
    } else {
        OpStrided<float, AK> a{pa, AK ? lda : 1, AK ? 1 : lda, n, n, -1};
        OpStrided<float, BK> b{pb, BK ? ldb : 1, BK ? 1 : ldb, n, n, -1};
        if (!SYM) {
            gemm_tile_ragged(a, b, i0, j0, n, n, n, sm, epi);
            return;
        }
        gemm_tile(a, b, i0, j0, 0, n, sm, acc);
    }
    const float os = X3 ? out_scale : 1.f;
    for_each_acc(acc, [&](int r, int c, float v) {
        const int gr = i0 + r, gc = j0 + c;
        if (gr < n && gc < n) epi(gr, gc, v * os);
    });
    if (SYM && j0 < i0)
        for_each_acc_transposed(acc, reinterpret_cast<float *>(&sm), [&](int r, int c, float v) {
            const int gr = j0 + r, gc = i0 + c;
            if (gr < n && gc < n) epi(gr, gc, v * os);
        });
}

// Rayleigh quotients lam[i] = q_i^T (F q_i) from Q [n][ldq] and Z = F Q [n][ldz]: the rows are split over
// blockIdx.y, whose shares land in part[y][i] and are added in order by the kernel below.
constexpr int RAY_PARTS = 32;
__global__ __launch_bounds__(NT) void blk_rayleigh_kernel(const float *Q, int64_t ldq, const float *Z, int64_t ldz,
                                                          int n, double *part) {
    const int i = blockIdx.x * NT + threadIdx.x;
    if (i >= n) return;
    const int rows_per = (n + gridDim.y - 1) / gridDim.y;
    const int r0 = blockIdx.y * rows_per, r1 = min(n, r0 + rows_per);
    double s = 0.0;
    for (int r = r0; r < r1; ++r) s += (double)Q[(int64_t)r * ldq + i] * (double)Z[(int64_t)r * ldz + i];
    part[(int64_t)blockIdx.y * n + i] = s;
}
__global__ __launch_bounds__(NT) void blk_rayleigh_sum_kernel(const double *part, int n, double *lam64) {
    const int i = blockIdx.x * NT + threadIdx.x;
    if (i >= n) return;
    double s = 0.0;
    for (int y = 0; y < RAY_PARTS; ++y) s += part[(int64_t)y * n + i];
    lam64[i] = s;
}

// perm[rank] = index of the rank-th smallest eigenvalue (ties by index); lam[rank] = that eigenvalue (if asked for).
// n^2 comparisons: a workgroup ranks RANK_IPB values, sixteen threads sharing the comparisons of each (the values
// they compare against pass through LDS a workgroup-load at a time), so a 4609-wide spectrum is 289 workgroups.
constexpr int RANK_IPB = 16;
__device__ inline void rank_block(const double *lam64, int n, int *perm, float *lam_out) {
    __shared__ float chunk[NT];
    __shared__ int part[NT];
    const int ii = threadIdx.x & (RANK_IPB - 1), js = threadIdx.x / RANK_IPB;
    const int i = blockIdx.x * RANK_IPB + ii;
    const float li = i < n ? (float)lam64[i] : 0.f;
    const bool nan_i = li != li;
    int rank = 0;
    for (int j0 = 0; j0 < n; j0 += NT) {
        __syncthreads();
        chunk[threadIdx.x] = j0 + (int)threadIdx.x < n ? (float)lam64[j0 + threadIdx.x] : 0.f;
        __syncthreads();
        const int cnt = min(NT, n - j0);
        for (int k = js; k < cnt; k += NT / RANK_IPB) {   // NaNs order after every number, among themselves by index: always a permutation
            const float lj = chunk[k];
            const int j = j0 + k;
            const bool nan_j = lj != lj;
            rank += nan_i ? (!nan_j || j < i) : (!nan_j && ((lj < li) || (lj == li && j < i)));
        }
    }
    part[threadIdx.x] = rank;
    __syncthreads();
    if (js == 0 && i < n) {
        int total = 0;
        for (int t = 0; t < NT / RANK_IPB; ++t) total += part[t * RANK_IPB + ii];
        perm[total] = i;
        if (lam_out) lam_out[total] = li;
    }
}
__global__ __launch_bounds__(NT) void blk_rank_kernel(const double *lam64, int n, int *perm, float *lam_out) {
    rank_block(lam64, n, perm, lam_out);
}

__global__ __launch_bounds__(NT) void blk_fill_kernel(float *dst, int64_t count, float v) {
    for (int64_t e = blockIdx.x * (int64_t)NT + threadIdx.x; e < count; e += (int64_t)gridDim.x * NT) dst[e] = v;
}

__global__ __launch_bounds__(NT) void blk_copy_kernel(const float *src, float *dst, int64_t count) {
    for (int64_t e = blockIdx.x * (int64_t)NT + threadIdx.x; e < count; e += (int64_t)gridDim.x * NT) dst[e] = src[e];
}

// Qout[i][j] = Qin[i][perm[j]]
__global__ __launch_bounds__(NT) void blk_gather_kernel(const float *Qin, int64_t ldin, float *Qout, int64_t ldout, int n, const int *perm) {
    const int64_t n2 = (int64_t)n * n;
    for (int64_t e = blockIdx.x * (int64_t)NT + threadIdx.x; e < n2; e += (int64_t)gridDim.x * NT) {
        const int i = (int)(e / n), j = (int)(e - (int64_t)i * n);
        int c = perm[j];
        c = c < 0 ? 0 : (c >= n ? n - 1 : c);  // ranks collide only when the input holds NaNs
        Qout[(int64_t)i * ldout + j] = Qin[(int64_t)i * ldin + c];
    }
}

// out[i] = W[i][i]
__global__ __launch_bounds__(NT) void blk_diag_kernel(const float *W, int64_t ld, int n, double *out) {
    const int i = blockIdx.x * NT + threadIdx.x;
    if (i < n) out[i] = (double)W[(int64_t)i * ld + i];
}

// ------------------------------------------------------------------------------------------------
// d >= 2048: two-level blocked Jacobi.  At these sizes the round application above is bound by HBM
// traffic (a 64-wide contraction per pass over the matrix), so rounds are grouped: 128-wide
// super-blocks are paired by an outer tournament; each 256 x 256 super-pair is gathered into a compact
// buffer that stays in L2, where the block rounds above run on it alone (4 bipartite rounds meet every
// cross pair of its 4 + 4 small blocks) and accumulate its 256 x 256 orthogonal transform; that
// transform is then applied to the whole matrix and to the eigenvector accumulator in two passes of
// ordinary 128 x 128 x 256 GEMM tiles (columns, then rows), which are MFMA bound.  Pairs of small
// blocks inside one super-block are met in a "diagonal" phase once per sweep, so every pair of small
// blocks is still visited exactly once per sweep.
// ------------------------------------------------------------------------------------------------
constexpr int SB = 128;                 // super-block width
constexpr int LDI = 2 * SB;             // edge of a super-pair (unit)
static_assert(SB == 4 * EB, "a super-block is four small blocks (blk_index)");
constexpr int TWO_LEVEL_MIN = 2048;     // factors at least this large take the two-level path

struct SpGroup {
    float *W, *T;          // [nmat][npad][npad]: rotated matrix, column-pass result
    float *Vi;             // accumulated transforms of the units: [nmat*U][s][s]
    float *scale;          // [nmat][2]: power of two that brings ||W||_F into [2^12, 2^13), and its inverse
    const int *done;       // [nmat]: as in BlkGroup
    int nmat, npad, nsuper, players;
};

// The passes below run on the split-fp16 engine (template argument X3; the fp32 engine otherwise).  Its
// operands are scaled into fp16's range: W and T by the factor's own power of two (no entry of an
// orthogonally rotated matrix exceeds its Frobenius norm, which the rotations preserve), the transforms
// and the eigenvector accumulator, whose entries are at most 1, by 2^14.
constexpr float X3_UNIT = 16384.f;

__global__ void sp_scale_kernel(SpGroup g, const double *norms) {
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    if (m >= g.nmat) return;
    const double n2 = norms[2 * m] + norms[2 * m + 1];
    float sc = 1.f, inv = 1.f;
    if (n2 > 0.0 && n2 < 1e300) {
        const int e = ilogb(sqrt(n2));          // ||W||_F in [2^e, 2^(e+1))
        const int k = min(max(12 - e, -100), 100);
        sc = ldexpf(1.f, k);
        inv = ldexpf(1.f, -k);
    }
    g.scale[2 * m] = sc;
    g.scale[2 * m + 1] = inv;
}

// Super-blocks of unit u: outer tournament pair of round `round`, or super-block u alone in the
// diagonal phase (round < 0).  b1 = -1 when the unit has a single super-block.
__device__ inline void unit_blocks(const SpGroup &g, int round, int u, int &b0, int &b1) {
    if (round < 0) { b0 = u; b1 = -1; return; }
    int p, q;
    rr_pair(g.players, round, u, p, q);
    b0 = p;
    b1 = q < g.nsuper ? q : -1;
}

// Column pass.  W part: T[blk(I,a), blk(J,b)] = sum_c W[blk(I,a), blk(J,c)] V_J[c, b] for unit pairs I > J;
// accumulator part: Qout[rb, blk(J,b)] = sum_c Qin[rb, blk(J,c)] V_J[c, b] for every 128-row slab rb.
template <bool X3>
__global__ __launch_bounds__(kfac::NTHREADS) __attribute__((amdgpu_waves_per_eu(3))) void sp_pass_cols_kernel(SpGroup g, int round, int U, int s, int nW, int nrb,
                                                                      const float *Qin, float *Qout, int bx0) {
    using namespace kfac;
    __shared__ typename std::conditional<X3, X3Smem, TileSmem>::type sm;
    const int m = blockIdx.y;
    if (g.done[m]) return;
    const int64_t np2 = (int64_t)g.npad * g.npad;
    const int ld = g.npad;
    int J, b, rowblk;          // unit and column part; global row super-block of the output tile
    const float *src;          // matrix whose rows [rowblk] are multiplied
    float *dst;
    // The fp16 MFMA's fp32 accumulation truncates toward minus infinity: a bias of about 2^-25 of every
    // result, always downwards.  Summed down a column of the accumulator, against the all-positive leading
    // eigenvector of a factor, such a bias adds up coherently over the rounds.  Feeding the negated operand in
    // every other round (and negating the result) turns it upwards there, so it cancels over two rounds.
    const float sgn = (round & 1) ? -1.f : 1.f;
    float in_scale = X3_UNIT, out_scale = 1.f / (X3_UNIT * X3_UNIT);   // split engine: accumulator part
    // Workgroup order: the two tiles that share an A operand (column halves b = 0, 1 of one unit) are 8 apart in
    // the launch, i.e. they run at the same time on the same XCD (workgroups go round the 8 XCDs), so the second
    // read of the operand is an L2 hit instead of a second trip to memory.  c counts the (operand, unit) pairs.
    const int bx = blockIdx.x + bx0;
    if (bx < nW) {
        if (X3) { in_scale = g.scale[2 * m]; out_scale = g.scale[2 * m + 1] * (1.f / X3_UNIT); }
        const int c = (bx >> 4) * 8 + (bx & 7);
        if (c >= (U * (U - 1) / 2) * 2) return;
        const int a = c & 1;
        b = (bx >> 3) & 1;
        int i1;
        tri_decode(c >> 1, i1, J);
        int I0, I1;
        unit_blocks(g, round, i1 + 1, I0, I1);
        rowblk = a ? I1 : I0;
        if (rowblk < 0) return;
        src = g.W + m * np2;
        dst = g.T + m * np2;
    } else {
        const int idx = bx - nW;
        const int c = (idx >> 4) * 8 + (idx & 7);
        if (c >= nrb * U) return;
        rowblk = c % nrb;
        J = c / nrb;
        b = (idx >> 3) & 1;
        src = Qin + m * np2;
        dst = Qout + m * np2;
    }
    int J0, J1;
    unit_blocks(g, round, J, J0, J1);
    const int cb = b ? J1 : J0;
    if (cb < 0) return;
    const float *V = g.Vi + ((int64_t)m * U + J) * s * s;
    // one contraction over both column blocks of the unit: the A operand jumps from block J0 to block J1
    // half way, the rows of V are contiguous
    floatx16 acc[2][2];
    const int K = J1 >= 0 ? 2 * SB : SB;
    float *out = dst + (int64_t)rowblk * SB * ld + cb * SB;
    if constexpr (X3) {
        X3Op<true> A{src + (int64_t)rowblk * SB * ld + J0 * SB, ld, sgn * in_scale, 0, 0};
        out_scale *= sgn;
        if (J1 >= 0) A.set_segment(SB, (int64_t)(J1 - J0 - 1) * SB);
        X3Op<false> B{V + b * SB, s, X3_UNIT, 0, 0};      // V holds V - I here: X V = X + X (V - I)
        A.start(threadIdx.x);
        B.start(threadIdx.x);
        gemm_tile_x3(A, B, K, sm, acc);
        // all loads of the input tile are issued before the first store (the two may alias for the compiler)
        const float *in = src + (int64_t)rowblk * SB * ld + cb * SB;
        floatx16 xin[2][2];
        fill_acc(xin, [&](int r, int c) { return in[(int64_t)r * ld + c]; });
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = acc[i][j] * out_scale + xin[i][j];
        for_each_acc(acc, [&](int r, int c, float v) { out[(int64_t)r * ld + c] = v; });
    } else {
        OpStrided<float, true> A{src + (int64_t)rowblk * SB * ld + J0 * SB, ld, 1, SB, K, -1};
        if (J1 >= 0) A.set_segment(SB, (int64_t)(J1 - J0 - 1) * SB);
        OpStrided<float, false> B{V + b * SB, 1, s, SB, K, -1};
        gemm_tile(A, B, 0, 0, 0, K, sm, acc);
        for_each_acc(acc, [&](int r, int c, float v) { out[(int64_t)r * ld + c] = v; });
    }
}

// Row pass: W[blk(I,a), blk(J,b)] = sum_c V_I[c, a]^T T[blk(I,c), blk(J,b)] for unit pairs I > J, mirrored.
template <bool X3>
__global__ __launch_bounds__(kfac::NTHREADS) __attribute__((amdgpu_waves_per_eu(3))) void sp_pass_rows_kernel(SpGroup g, int round, int U, int s) {
    using namespace kfac;
    __shared__ typename std::conditional<X3, X3Smem, TileSmem>::type sm;
    const int m = blockIdx.y;
    if (g.done[m]) return;
    const int64_t np2 = (int64_t)g.npad * g.npad;
    const int ld = g.npad;
    // the two tiles that share the B operand (row halves a = 0, 1 of one unit) are 8 apart: see the column pass
    const int idx = blockIdx.x;
    const int c = (idx >> 4) * 8 + (idx & 7);
    if (c >= (U * (U - 1) / 2) * 2) return;
    const int a = (idx >> 3) & 1, b = c & 1;
    int i1, J;
    tri_decode(c >> 1, i1, J);
    const int I = i1 + 1;
    int I0, I1, J0, J1;
    unit_blocks(g, round, I, I0, I1);
    unit_blocks(g, round, J, J0, J1);
    const int rb = a ? I1 : I0, cb = b ? J1 : J0;
    if (rb < 0 || cb < 0) return;
    const float *V = g.Vi + ((int64_t)m * U + I) * s * s;
    const float *T = g.T + m * np2;
    float *W = g.W + m * np2;
    floatx16 acc[2][2];
    const int K = I1 >= 0 ? 2 * SB : SB;
    float out_scale = 1.f;
    if constexpr (X3) {
        const float sgn = (round & 1) ? -1.f : 1.f;   // alternating sign: see the column pass
        X3Op<false> A{V + a * SB, s, sgn * X3_UNIT, 0, 0};                              // elem(m,k) = (V - I)[k][m]
        X3Op<false> B{T + (int64_t)I0 * SB * ld + cb * SB, ld, g.scale[2 * m], 0, 0};   // elem(n,k) = T[k][n]
        if (I1 >= 0) B.set_segment(SB, (int64_t)(I1 - I0 - 1) * SB * ld);
        A.start(threadIdx.x);
        B.start(threadIdx.x);
        gemm_tile_x3(A, B, K, sm, acc);
        out_scale = sgn * g.scale[2 * m + 1] * (1.f / X3_UNIT);
    } else {
        OpStrided<float, false> A{V + a * SB, 1, s, SB, K, -1};                                    // elem(m,k) = V[k][m]
        OpStrided<float, false> B{T + (int64_t)I0 * SB * ld + cb * SB, 1, ld, SB, K, -1};         // elem(n,k) = T[k][n]
        if (I1 >= 0) B.set_segment(SB, (int64_t)(I1 - I0 - 1) * SB * ld);
        gemm_tile(A, B, 0, 0, 0, K, sm, acc);
    }
    float *out = W + (int64_t)rb * SB * ld + cb * SB;
    float *mir = W + (int64_t)cb * SB * ld + rb * SB;
    if constexpr (X3) {
        const float *tin = T + (int64_t)rb * SB * ld + cb * SB;   // V^T T = T + (V - I)^T T
        floatx16 xin[2][2];
        fill_acc(xin, [&](int r, int c) { return tin[(int64_t)r * ld + c]; });
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = acc[i][j] * out_scale + xin[i][j];
    }
    for_each_acc(acc, [&](int r, int c, float v) { out[(int64_t)r * ld + c] = v; });
    store_acc_transposed(acc, reinterpret_cast<float *>(&sm), mir, ld);
}

// ---- ordering of the diagonal ------------------------------------------------------------------------
// A symmetric permutation that puts the diagonal of W (the eigenvalue estimates) in ascending order, applied to W
// and to the columns of the accumulator; all factors of a group in one launch each (blockIdx.y: factor).  A factor
// that has met the tolerance is left alone.  `T` is n x n scratch per factor: the group's own (pitch npad) or, for
// groups that have none, the caller's eigenvector buffer (pitch n), which nothing else uses before the very end.
struct SortArgs {
    float *W, *Qw, *T;
    int64_t np2;
    int npad;
    const BlkItem *items;
    const int *done;
    double *lam64;        // [factor][lam_stride]
    int64_t lam_stride;
    int *perm;            // [factor][npad]
};
__device__ inline float *sort_scratch(const SortArgs &a, int m, int64_t &ld) {
    if (a.T) { ld = a.npad; return a.T + m * a.np2; }
    ld = a.items[m].n;
    return a.items[m].Q;
}
__global__ __launch_bounds__(NT) void sort_diag_kernel(SortArgs a) {
    const int m = blockIdx.y, i = blockIdx.x * NT + threadIdx.x;
    if (a.done[m] || i >= a.items[m].n) return;
    a.lam64[m * a.lam_stride + i] = (double)a.W[m * a.np2 + (int64_t)i * a.npad + i];
}
__global__ __launch_bounds__(NT) void sort_rank_kernel(SortArgs a) {
    const int m = blockIdx.y;
    if (a.done[m]) return;
    const int n = a.items[m].n;
    if ((int)(blockIdx.x * RANK_IPB) >= n) return;
    rank_block(a.lam64 + m * a.lam_stride, n, a.perm + (int64_t)m * a.npad, nullptr);
}
// which = 0: scratch = P W P^T; which = 1: scratch[:, j] = Q[:, perm[j]]
__global__ __launch_bounds__(NT) void sort_permute_kernel(SortArgs a, int which) {
    const int m = blockIdx.y;
    if (a.done[m]) return;
    const int n = a.items[m].n;
    const int *perm = a.perm + (int64_t)m * a.npad;
    int64_t lds;
    float *S = sort_scratch(a, m, lds);
    const float *src = (which == 0 ? a.W : a.Qw) + m * a.np2;
    const int64_t n2 = (int64_t)n * n;
    for (int64_t e = blockIdx.x * (int64_t)NT + threadIdx.x; e < n2; e += (int64_t)gridDim.x * NT) {
        const int i = (int)(e / n), j = (int)(e - (int64_t)i * n);
        int c = perm[j];
        c = c < 0 ? 0 : (c >= n ? n - 1 : c);
        int r = i;
        if (which == 0) {
            r = perm[i];
            r = r < 0 ? 0 : (r >= n ? n - 1 : r);
        }
        S[(int64_t)i * lds + j] = src[(int64_t)r * a.npad + c];
    }
}
__global__ __launch_bounds__(NT) void sort_copyback_kernel(SortArgs a, int which) {
    const int m = blockIdx.y;
    if (a.done[m]) return;
    const int n = a.items[m].n;
    int64_t lds;
    const float *S = sort_scratch(a, m, lds);
    float *dst = (which == 0 ? a.W : a.Qw) + m * a.np2;
    const int64_t n2 = (int64_t)n * n;
    for (int64_t e = blockIdx.x * (int64_t)NT + threadIdx.x; e < n2; e += (int64_t)gridDim.x * NT) {
        const int i = (int)(e / n), j = (int)(e - (int64_t)i * n);
        dst[(int64_t)i * a.npad + j] = S[(int64_t)i * lds + j];
    }
}

// ---- host side ---------------------------------------------------------------------------------
struct GroupPlan {
    int nblk, npad, players, npairs;
    bool two_level;
    int nsuper, splayers, U;      // two-level: super-blocks, outer players (even), units per outer round
    std::vector<int> members;
    size_t inner_mats() const { return members.size() * (size_t)std::max(U, nsuper); }
    size_t bytes() const {
        const size_t nm = members.size();
        size_t b = 0;
        b += kfac_align_up(nm * (two_level ? 4 : 2) * (size_t)npad * npad * sizeof(float), 256);   // W, Qw (+ T, Qw')
        if (two_level) {
            b += kfac_align_up(nm * (size_t)U * LDI * LDI * sizeof(float), 256);                  // Vi
            b += kfac_align_up(inner_mats() * 4 * KP * KP * sizeof(float), 256);                   // inner J
            b += kfac_align_up(inner_mats() * 4 * sizeof(int), 256);                               // inner idt
            b += kfac_align_up(nm * 2 * sizeof(float), 256);                                       // scale
        } else {
            b += kfac_align_up(nm * (size_t)npairs * KP * KP * sizeof(float), 256);                // J
            b += kfac_align_up(nm * (size_t)npairs * sizeof(int), 256);                            // idt
        }
        b += kfac_align_up(nm * 2 * sizeof(double), 256);                            // norms
        b += kfac_align_up(nm * 2 * NORM_PARTS_MAX * sizeof(double), 256);           // their per-workgroup shares
        b += kfac_align_up(nm * sizeof(int), 256);                                   // done flags
        b += kfac_align_up(nm * (size_t)npad * sizeof(int), 256);                    // perm
        b += kfac_align_up(nm * (size_t)npad * (RAY_PARTS + 1) * sizeof(double), 256);   // Rayleigh quotients and their shares
        b += kfac_align_up(nm * sizeof(BlkItem), 256);                               // items
        return b;
    }
};

// Factors of similar size advance together as one group, each padded with zero blocks (which no rotation
// ever touches) to the group's block count: one chain of launches serves them all, and a round's launches
// are large enough to fill the machine.  Block counts are rounded up along a ladder of odd numbers about
// 15 % apart (odd: the tournament then needs no phantom block).
int bucket(int n) {
    static const int ladder[] = {3, 5, 7, 9, 11, 13, 15, 19, 23, 27, 33, 37, 45, 53, 65, 75, 87, 101, 117, 135, 155, 179, 205, 235, 257};
    for (int b : ladder) if (b >= n) return b;
    return n | 1;
}

void make_plan(int batch, const int *d, std::vector<int> &small, std::vector<GroupPlan> &groups) {
    for (int i = 0; i < batch; ++i) {
        if (d[i] <= SMALL_MAX) { small.push_back(i); continue; }
        const bool two = d[i] >= TWO_LEVEL_MIN;
        const int unit = two ? SB : EB;
        // small blocks along the ladder; super-blocks only up to the next odd count (padding a large factor
        // by 15 % would cost more than a chain of its own)
        const int nunit = (d[i] + unit - 1) / unit;
        const int npad = (two ? (nunit | 1) : bucket(nunit)) * unit;
        const int nblk = npad / EB;
        GroupPlan *gp = nullptr;
        for (auto &g : groups) if (g.nblk == nblk && g.two_level == two) gp = &g;
        if (!gp) {
            GroupPlan g;
            g.two_level = two;
            g.nblk = nblk;
            g.npad = npad;
            g.players = (nblk + 1) & ~1;
            g.npairs = g.players / 2;
            g.nsuper = npad / SB;
            g.splayers = (g.nsuper + 1) & ~1;
            g.U = g.splayers / 2;
            groups.push_back(g);
            gp = &groups.back();
        }
        gp->members.push_back(i);
    }
    std::sort(groups.begin(), groups.end(), [](const GroupPlan &a, const GroupPlan &b) { return a.nblk > b.nblk; });
}

size_t small_bytes(size_t nsmall) {
    return kfac_align_up(nsmall * sizeof(SmallItem), 256) + kfac_align_up(nsmall * sizeof(EigStat), 256);
}

// Everything one group of equally sized factors needs while it is in flight on its stream.
struct GroupRun {
    GroupPlan *plan;
    BlkGroup g;           // flat view: W, Qw (current accumulator), J, idt, norms
    SpGroup sp;           // two-level view
    BlkGroup gi, gd;      // two-level: inner groups of the regular rounds and of the diagonal phase
    float *Qalt;          // two-level: the other accumulator buffer
    hipStream_t st;
    hipEvent_t ev[KFAC_EIG_SLOTS];   // one per report slot; slot 0 also marks the end of the post-processing
    struct Report { int slot, sweeps; bool final_ok; };   // norms after `sweeps` sweeps; final_ok: taken after the refresh
    std::deque<Report> reports;      // enqueued, not yet read by the host (oldest first)
    int next_slot;
    std::vector<BlkItem> items;
    BlkItem *d_items;
    int *perm;
    double *lam64;
    double *normpart;     // [nm][norm_blocks][2]
    int norm_blocks;
    double *h_norms;      // pinned, KFAC_EIG_SLOTS x 2 per factor
    int nm, ntiles_w, nrb, ntiles, nmax, fill_blocks;
    double apply_flops, solve_flops;
    int sweep;
    bool done;
    bool x3;              // two-level: outer passes on the split-fp16 engine
    bool refreshed;       // x3: W has been recomputed as Q^T F Q in fp32 (or never left fp32)
    int *d_done;          // device flags, one per factor
    double tol2;
    std::vector<char> conv;
    std::vector<char> bad;        // norms not finite: the factor is given up (outputs filled with NaN)
    std::vector<int> sweeps_done;
    std::vector<float> offrel;
};

int enqueue_offnorm(kfac_ctx *ctx, GroupRun &r) {
    {
        KfacProfScope prof(ctx, KC_EIG_MISC, 0.0, 0.0, r.st);
        hipLaunchKernelGGL(blk_offnorm_kernel, dim3(r.norm_blocks, r.nm), dim3(NT), 0, r.st, r.g, r.normpart);
        hipLaunchKernelGGL(blk_norm_reduce_kernel, dim3(r.nm), dim3(NT), 0, r.st, (const double *)r.normpart, r.norm_blocks, r.g.norms,
                           r.d_done, r.tol2);
    }
    KFAC_HIP_CHECK(hipGetLastError());
    const int slot = r.next_slot;
    r.next_slot = (slot + 1) % KFAC_EIG_SLOTS;
    KFAC_HIP_CHECK(hipMemcpyAsync(r.h_norms + (size_t)slot * 2 * r.nm, r.g.norms, 2 * r.nm * sizeof(double), hipMemcpyDeviceToHost, r.st));
    KFAC_HIP_CHECK(hipEventRecord(r.ev[slot], r.st));
    r.reports.push_back(GroupRun::Report{slot, r.sweep, r.refreshed || r.sweep == 0});
    return KFAC_OK;
}

// One round of (pivot solves, application) on a block group.
void enqueue_round(kfac_ctx *ctx, hipStream_t st, const BlkGroup &g, int rd, int ntiles, int ntiles_w, int nrb,
                   size_t lds_solve, int inner_cap, float inner_tol, double solve_flops, double apply_flops, double apply_bytes) {
    {
        KfacProfScope prof(ctx, KC_EIG_SOLVE, solve_flops, 0.0, st);
        hipLaunchKernelGGL(blk_solve_kernel, dim3(g.npairs, g.nmat), dim3(SOLVE_NT), lds_solve, st, g, rd, inner_cap, inner_tol);
    }
    {
        KfacProfScope prof(ctx, KC_EIG_APPLY, apply_flops, apply_bytes, st);
        hipLaunchKernelGGL(blk_apply_kernel, dim3(ntiles, g.nmat), dim3(NT), 0, st, g, rd, ntiles_w, nrb);
    }
}

// Ascending order of the eigenvalue estimates along the diagonal (see SortArgs): six launches for the whole group.
int enqueue_sort(kfac_ctx *ctx, GroupRun &r) {
    const GroupPlan &gp = *r.plan;
    SortArgs a{r.g.W, r.g.Qw, gp.two_level ? r.sp.T : nullptr, (int64_t)gp.npad * gp.npad, gp.npad, r.d_items, r.d_done,
               r.lam64, (int64_t)gp.npad * (RAY_PARTS + 1), r.perm};
    const dim3 gv((r.nmax + NT - 1) / NT, r.nm), gm(std::min(r.fill_blocks, 1024), r.nm);
    KfacProfScope prof(ctx, KC_EIG_MISC, 0.0, 0.0, r.st);
    hipLaunchKernelGGL(sort_diag_kernel, gv, dim3(NT), 0, r.st, a);
    hipLaunchKernelGGL(sort_rank_kernel, dim3((r.nmax + RANK_IPB - 1) / RANK_IPB, r.nm), dim3(NT), 0, r.st, a);
    for (int which = 0; which < 2; ++which) {
        hipLaunchKernelGGL(sort_permute_kernel, gm, dim3(NT), 0, r.st, a, which);
        hipLaunchKernelGGL(sort_copyback_kernel, gm, dim3(NT), 0, r.st, a, which);
    }
    KFAC_HIP_CHECK(hipGetLastError());
    return KFAC_OK;
}

int enqueue_sweep_flat(kfac_ctx *ctx, GroupRun &r, size_t lds_solve, int inner_cap, float inner_tol) {
    for (int rd = 0; rd < r.plan->players - 1; ++rd)
        enqueue_round(ctx, r.st, r.g, rd, r.ntiles, r.ntiles_w, r.nrb, lds_solve, inner_cap, inner_tol, r.solve_flops, r.apply_flops,
                      2.0 * r.apply_flops / EB);   // W and the accumulator read and written once: 16 n^2 bytes per factor
    KFAC_HIP_CHECK(hipGetLastError());
    return KFAC_OK;
}

// One phase of the two-level sweep: the inner rounds of every unit, then the passes that apply the units' transforms.
void enqueue_phase(kfac_ctx *ctx, GroupRun &r, int round, size_t lds_solve, int inner_cap, float inner_tol) {
    const GroupPlan &gp = *r.plan;
    hipStream_t st = r.st;
    const bool diag = round < 0;
    const int U = diag ? gp.nsuper : gp.U;
    const int s = diag ? SB : LDI;
    const BlkGroup &gin = diag ? r.gd : r.gi;
    const int inner_rounds = diag ? gin.players - 1 : gin.players / 2;
    // The unit's own blocks of W are rotated in place by the inner rounds (the passes below touch only blocks between
    // different units); its transform is accumulated in the compact Vi, started from the identity by the first round
    // and, for the split engine, left as V - I by the last.
    const int in_tw = gin.npairs * (gin.npairs + 1) / 2, in_nrb = s / KP, in_tiles = in_tw + ((in_nrb + 1) / 2) * gin.npairs;
    const double in_solve = (double)gin.nmat * gin.npairs * 9.0 * KP * KP * (KP / 2);
    const double in_apply = (double)gin.nmat * 8.0 * s * s * EB;
    for (int ri = 0; ri < inner_rounds; ++ri) {
        BlkGroup gr = gin;
        gr.outer_round = round;
        gr.qw_identity = ri == 0;
        gr.qw_minus_identity = r.x3 && ri == inner_rounds - 1;
        enqueue_round(ctx, st, gr, ri, in_tiles, in_tw, in_nrb, lds_solve, inner_cap, inner_tol, in_solve, in_apply, 2.0 * in_apply / EB);
    }
    const int nW = ((2 * (U * (U - 1) / 2) + 7) / 8) * 16;      // padded to whole groups of 8 pairs x 2 halves
    const int nrb = gp.npad / SB;
    const int nQ = ((nrb * U + 7) / 8) * 16;
    // algorithmic work of the two passes: every element of half the symmetric matrix and of the
    // accumulator gets two (one) dot products of the unit edge s
    // algorithmic bytes: the column pass reads Q and the lower half of W and writes as much (12 n^2 bytes), the
    // row pass reads the half-size T and writes W with its mirror image (6 n^2)
    double fl = 0.0, n2 = 0.0;
    for (int i = 0; i < r.nm; ++i) {
        fl += 4.0 * (double)r.items[i].n * r.items[i].n * s;
        n2 += (double)r.items[i].n * r.items[i].n;
    }
    {
        KfacProfScope prof(ctx, KC_EIG_OUTER, 0.75 * fl, 12.0 * n2, st);
        if (r.x3)
            hipLaunchKernelGGL(sp_pass_cols_kernel<true>, dim3(nW + nQ, r.nm), dim3(kfac::NTHREADS), 0, st, r.sp, round, U, s,
                               nW, nrb, (const float *)r.g.Qw, r.Qalt, 0);
        else
            hipLaunchKernelGGL(sp_pass_cols_kernel<false>, dim3(nW + nQ, r.nm), dim3(kfac::NTHREADS), 0, st, r.sp, round, U, s,
                               nW, nrb, (const float *)r.g.Qw, r.Qalt, 0);
    }
    if (nW > 0) {
        KfacProfScope prof(ctx, KC_EIG_OUTER_ROWS, 0.25 * fl, 6.0 * n2, st);
        if (r.x3) hipLaunchKernelGGL(sp_pass_rows_kernel<true>, dim3(nW, r.nm), dim3(kfac::NTHREADS), 0, st, r.sp, round, U, s);
        else hipLaunchKernelGGL(sp_pass_rows_kernel<false>, dim3(nW, r.nm), dim3(kfac::NTHREADS), 0, st, r.sp, round, U, s);
    }
    std::swap(r.g.Qw, r.Qalt);
}

int enqueue_sweep_two_level(kfac_ctx *ctx, GroupRun &r, size_t lds_solve, int inner_cap, float inner_tol) {
    enqueue_phase(ctx, r, -1, lds_solve, inner_cap, inner_tol);
    for (int rd = 0; rd < r.plan->splayers - 1; ++rd) enqueue_phase(ctx, r, rd, lds_solve, inner_cap, inner_tol);
    KFAC_HIP_CHECK(hipGetLastError());
    return KFAC_OK;
}

// Flops a symmetric n x n product over a contraction of n is credited with when only the tiles on and below the
// diagonal are computed.
inline double sym_product_flops(int n) {
    const double nt = (n + kfac::BM - 1) / kfac::BM;
    return 2.0 * n * n * n * (nt + 1.0) / (2.0 * nt);
}

// One Newton-Schulz step out = Q (3I - Q^T Q)/2 on the leading n x n part of Q (pitch ld); `scratch` (same pitch) is
// overwritten.  On the fp32 engine, or (split: groups whose passes run there anyway) on the split-fp16 engine in delta form.
void enqueue_newton_schulz(kfac_ctx *ctx, GroupRun &r, BatchOperand Qm, BatchOperand scratch, BatchOperand out, bool split) {
    using namespace kfac;
    const int64_t ld = r.plan->npad;
    const int tiles = (r.nmax + BM - 1) / BM;
    const dim3 grid(tiles, tiles, r.nm), block(NTHREADS);
    double f_sym = 0.0, f_full = 0.0;
    for (int i = 0; i < r.nm; ++i) {
        const double n = r.items[i].n;
        f_sym += sym_product_flops(r.items[i].n);
        f_full += 2.0 * n * n * n;
    }
    const BatchOperand none{nullptr, 0, 0};
    hipStream_t st = r.st;
    if (split) {
        constexpr float SC = 16384.f, OUT = 1.f / (SC * SC);
        {   // D = (I - Q^T Q) / 2
            KfacProfScope prof(ctx, KC_EIG_POST, f_sym, 0.0, st);
            hipLaunchKernelGGL((gemm_batched_kernel<false, false, EPI_NS_DELTA, true, true>), grid, block, 0, st, Qm, Qm, scratch, none,
                               (const BlkItem *)r.d_items, ld, SC, OUT);
        }
        KfacProfScope prof(ctx, KC_EIG_POST, f_full, 0.0, st);   // Q + Q D
        hipLaunchKernelGGL((gemm_batched_kernel<true, false, EPI_ADD_STORE, false, true>), grid, block, 0, st, Qm, scratch, out, Qm,
                           (const BlkItem *)r.d_items, ld, SC, OUT);
        return;
    }
    {   // Y = (3I - Q^T Q) / 2
        KfacProfScope prof(ctx, KC_EIG_POST, f_sym, 0.0, st);
        hipLaunchKernelGGL((gemm_batched_kernel<false, false, EPI_NS, true, false>), grid, block, 0, st, Qm, Qm, scratch, none,
                           (const BlkItem *)r.d_items, ld, 1.f, 1.f);
    }
    KfacProfScope prof(ctx, KC_EIG_POST, f_full, 0.0, st);       // Q Y
    hipLaunchKernelGGL((gemm_batched_kernel<true, false, EPI_STORE, false, false>), grid, block, 0, st, Qm, scratch, out, none,
                       (const BlkItem *)r.d_items, ld, 1.f, 1.f);
}

// C = A B (A with the contraction index fast, e.g. the caller's F; B with it slow) and C = A^T B made of lower tiles
// and their mirror images, for every factor of the group, on the fp32 engine.
void enqueue_product(kfac_ctx *ctx, GroupRun &r, BatchOperand A, BatchOperand B, BatchOperand C, bool sym) {
    using namespace kfac;
    const int64_t ld = r.plan->npad;
    const int tiles = (r.nmax + BM - 1) / BM;
    const dim3 grid(tiles, tiles, r.nm), block(NTHREADS);
    double flops = 0.0;
    for (int i = 0; i < r.nm; ++i) {
        const double n = r.items[i].n;
        flops += sym ? sym_product_flops(r.items[i].n) : 2.0 * n * n * n;
    }
    const BatchOperand none{nullptr, 0, 0};
    KfacProfScope prof(ctx, KC_EIG_POST, flops, 0.0, r.st);
    if (sym)
        hipLaunchKernelGGL((gemm_batched_kernel<false, false, EPI_STORE, true, false>), grid, block, 0, r.st, A, B, C, none,
                           (const BlkItem *)r.d_items, ld, 1.f, 1.f);
    else
        hipLaunchKernelGGL((gemm_batched_kernel<true, false, EPI_STORE, false, false>), grid, block, 0, r.st, A, B, C, none,
                           (const BlkItem *)r.d_items, ld, 1.f, 1.f);
}

// Refresh of a group whose passes run on the split engine.  Those passes carry 22 significand bits and an error
// bounded relative to ||F||, so after several sweeps the working matrix W has drifted a little from Q^T F Q for
// the accumulator Q that goes with it.  Once the off-norm is small the drift is removed: Q is re-orthogonalised
// (one Newton-Schulz step) and W is recomputed from the caller's F as Q^T F Q, both on the fp32 engine.  From
// then on the iteration is a Jacobi iteration started from a good basis -- what came before only chose that
// basis -- and its remaining rounds are small corrections, which the split passes add to fp32 operands
// (X + X (V - I)) with an error far below fp32 rounding.  Every factor of the group takes part, converged or not.
// The refresh also puts the columns in ascending order of their eigenvalue estimates (it costs one more pass over Q).
// Cyclic Jacobi keeps its quadratic end phase in the presence of a multiple eigenvalue only if the diagonal entries
// that converge to it are neighbours; the null space of a rank-deficient factor (1500 to 3000 wide for the largest
// K-FAC factors of a small batch) is scattered over the diagonal otherwise, and the end phase was linear (off-norm
// x 0.3 per sweep at d = 4609, two to three sweeps more than a full-rank factor of that size needs).
int enqueue_refresh(kfac_ctx *ctx, GroupRun &r) {
    using namespace kfac;
    const GroupPlan &gp = *r.plan;
    const size_t np2 = (size_t)gp.npad * gp.npad;
    hipStream_t st = r.st;
    const int64_t ld = gp.npad;
    const BatchOperand bW{r.g.W, (int64_t)np2, 0}, bQ{r.g.Qw, (int64_t)np2, 0}, bQo{r.Qalt, (int64_t)np2, 0}, bT{r.sp.T, (int64_t)np2, 0};
    const BatchOperand bF{nullptr, 0, 1};
    // Every product below is one launch for the whole group (a factor with non-finite input rides along: its
    // matrices are its own).
    for (int i = 0; i < r.nm; ++i) {
        if (r.bad[i]) continue;
        const int n = r.items[i].n;
        const float *Wm = r.g.W + i * np2;
        // The diagonal of W, i.e. the eigenvalue estimates, before W becomes scratch: their ascending order is the order the
        // columns take below.
        double *l64 = r.lam64 + (size_t)i * gp.npad * (RAY_PARTS + 1);
        int *pm = r.perm + (size_t)i * gp.npad;
        KfacProfScope prof(ctx, KC_EIG_MISC, 0.0, 0.0, st);
        hipLaunchKernelGGL(blk_diag_kernel, dim3((n + NT - 1) / NT), dim3(NT), 0, st, Wm, ld, n, l64);
        hipLaunchKernelGGL(blk_rank_kernel, dim3((n + RANK_IPB - 1) / RANK_IPB), dim3(NT), 0, st, (const double *)l64, n, pm, r.items[i].lam);
    }
    // Q (3I - Q^T Q)/2 into the other accumulator buffer; W, free from here on, is the scratch
    enqueue_newton_schulz(ctx, r, bQ, bW, bQo, true);
    for (int i = 0; i < r.nm; ++i) {   // ... and back with the columns in ascending order of their eigenvalue estimates (the padding keeps its identity)
        if (r.bad[i]) continue;
        KfacProfScope prof(ctx, KC_EIG_MISC, 0.0, 0.0, st);
        hipLaunchKernelGGL(blk_gather_kernel, dim3(std::min(r.fill_blocks, 2048)), dim3(NT), 0, st, (const float *)(r.Qalt + i * np2), ld,
                           r.g.Qw + i * np2, ld, r.items[i].n, r.perm + (size_t)i * gp.npad);
    }
    enqueue_product(ctx, r, bF, bQ, bT, false);   // T = F Q1
    enqueue_product(ctx, r, bQ, bT, bW, true);    // W = Q1^T T, made exactly symmetric
    {
        KfacProfScope prof(ctx, KC_EIG_MISC, 0.0, 0.0, st);
        hipLaunchKernelGGL(blk_symmetrise_tiles_kernel, dim3((r.nmax * BM + NT - 1) / NT, r.nm), dim3(NT), 0, st, r.g.W, (int64_t)np2, ld,
                           (const BlkItem *)r.d_items);
    }
    r.refreshed = true;
    KFAC_HIP_CHECK(hipGetLastError());
    return KFAC_OK;
}

// Post-processing per factor: one Newton-Schulz step restores the orthogonality that thousands of fp32
// transforms have eroded, Rayleigh quotients against the caller's F give the eigenvalues, and the
// columns are put in ascending order.  W is dead by now and serves as scratch.
int enqueue_post(kfac_ctx *ctx, GroupRun &r) {
    using namespace kfac;
    const GroupPlan &gp = *r.plan;
    const size_t np2 = (size_t)gp.npad * gp.npad;
    hipStream_t st = r.st;
    const int64_t ld = gp.npad;
    const BatchOperand bW{r.g.W, (int64_t)np2, 0}, bQ{r.g.Qw, (int64_t)np2, 0}, bF{nullptr, 0, 1}, bOut{nullptr, 0, 2};
    // one launch per product for the whole group: the orthogonalised accumulator goes to the caller's Q, F Q into the
    // accumulator's place
    enqueue_newton_schulz(ctx, r, bQ, bW, bOut, r.x3);
    enqueue_product(ctx, r, bF, bOut, bQ, false);
    for (int i = 0; i < r.nm; ++i) {
        const int n = r.items[i].n;
        if (r.bad[i]) {   // non-finite input: non-finite output
            const float nan = std::nanf("");
            hipLaunchKernelGGL(blk_fill_kernel, dim3(std::min(r.fill_blocks, 2048)), dim3(NT), 0, st, r.items[i].Q, (int64_t)n * n, nan);
            hipLaunchKernelGGL(blk_fill_kernel, dim3(1), dim3(NT), 0, st, r.items[i].lam, (int64_t)n, nan);
            continue;
        }
        float *Wm = r.g.W + i * np2, *Qm = r.g.Qw + i * np2;
        double *l64 = r.lam64 + (size_t)i * gp.npad * (RAY_PARTS + 1), *lpart = l64 + gp.npad;
        int *pm = r.perm + (size_t)i * gp.npad;
        {
            KfacProfScope prof(ctx, KC_EIG_MISC, 0.0, 0.0, st);
            hipLaunchKernelGGL(blk_rayleigh_kernel, dim3((n + NT - 1) / NT, RAY_PARTS), dim3(NT), 0, st, r.items[i].Q, (int64_t)n, Qm, ld, n, lpart);
            hipLaunchKernelGGL(blk_rayleigh_sum_kernel, dim3((n + NT - 1) / NT), dim3(NT), 0, st, (const double *)lpart, n, l64);
            hipLaunchKernelGGL(blk_rank_kernel, dim3((n + RANK_IPB - 1) / RANK_IPB), dim3(NT), 0, st, l64, n, pm, r.items[i].lam);
        }
        {
            // plain copy of n*n floats (read + write): also the reference point for HBM traffic counters
            KfacProfScope prof(ctx, KC_EIG_COPY, 0.0, 8.0 * n * n, st);
            hipLaunchKernelGGL(blk_copy_kernel, dim3(std::min(r.fill_blocks, 2048)), dim3(NT), 0, st, r.items[i].Q, Wm, (int64_t)n * n);
        }
        KfacProfScope prof(ctx, KC_EIG_MISC, 0.0, 0.0, st);
        hipLaunchKernelGGL(blk_gather_kernel, dim3(std::min(r.fill_blocks, 2048)), dim3(NT), 0, st, Wm, (int64_t)n, r.items[i].Q, (int64_t)n, n, pm);
    }
    KFAC_HIP_CHECK(hipGetLastError());
    KFAC_HIP_CHECK(hipEventRecord(r.ev[0], st));
    return KFAC_OK;
}

}  // namespace

// All groups are in flight at once, each on one of the context's internal streams, so the workspace
// holds every group's buffers side by side.
size_t kfac_eig_ws_bytes_impl(int batch, const int *d) {
    std::vector<int> small;
    std::vector<GroupPlan> groups;
    make_plan(batch, d, small, groups);
    size_t need = small_bytes(small.size());
    for (auto &g : groups) need += g.bytes();
    return need;
}

// Everything between the fork onto the internal streams and the join back: may return early with an error, the
// caller joins in every case.
static int eig_run(kfac_ctx *ctx, int batch, const float *const *F, const int *d, float *const *Q, float *const *lam,
                   const kfac_eig_opts *opts, kfac_eig_info *info, std::vector<int> &small, std::vector<GroupPlan> &groups) {
    const int max_sweeps = (opts && opts->max_sweeps > 0) ? opts->max_sweeps : 30;
    const float tol = (opts && opts->tol > 0.f) ? opts->tol : 2e-6f;
    const bool fp32_outer = opts && opts->fp32_only != 0;
    const bool warm = opts && opts->warm_start != 0;
    const float refresh_at = 3e-4f;   // off(W)/||W|| at which a split-engine group recomputes W = Q^T F Q in fp32
    const int inner_cap = 1;       // one Jacobi sweep over a pivot per visit: fewest total rotations
    const float inner_tol = 1e-7f;
    const size_t lds_solve = JacobiSmem::bytes(KP, PLD);
    if (!groups.empty()) {
        if ((int)lds_solve > ctx->max_lds) return KFAC_EHIP;
        KFAC_HIP_CHECK(hipFuncSetAttribute((const void *)blk_solve_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_solve));
    }
    bool all_conv = true;

    char *wsp = ctx->ws;
    // host tables and the statistics that come back live in the context's pinned memory (after the norms), so
    // that no copy waits for the stream it is queued on
    char *ptab = (char *)ctx->pinned + KFAC_PINNED_NORMS;
    // ---- small factors: one launch, on the last internal stream ----
    SmallItem *sitems = nullptr;
    EigStat *sstats = nullptr;
    hipStream_t st_small = ctx->aux[(ctx->prof_on || getenv("KFAC_EIG_SERIAL")) ? 0 : KFAC_NUM_AUX_STREAMS - 1];
    if (!small.empty()) {
        const size_t ns = small.size();
        sitems = (SmallItem *)ptab; ptab += kfac_align_up(ns * sizeof(SmallItem), 64);
        sstats = (EigStat *)ptab; ptab += kfac_align_up(ns * sizeof(EigStat), 64);
        int kmax = 2;
        for (size_t i = 0; i < ns; ++i) {
            sitems[i] = SmallItem{F[small[i]], Q[small[i]], lam[small[i]], d[small[i]], 0};
            kmax = std::max(kmax, (d[small[i]] + 1) & ~1);
        }
        SmallItem *d_items = (SmallItem *)wsp;
        EigStat *d_stats = (EigStat *)(wsp + kfac_align_up(ns * sizeof(SmallItem), 256));
        wsp += small_bytes(ns);
        KFAC_HIP_CHECK(hipMemcpyAsync(d_items, sitems, ns * sizeof(SmallItem), hipMemcpyHostToDevice, st_small));
        const size_t lds = JacobiSmem::bytes(kmax, kmax + 1);
        if ((int)lds > ctx->max_lds) return KFAC_EHIP;
        KFAC_HIP_CHECK(hipFuncSetAttribute((const void *)eig_small_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        {
            KfacProfScope prof(ctx, KC_EIG_SMALL, 0.0, 0.0, st_small);
            hipLaunchKernelGGL(eig_small_kernel, dim3((unsigned)ns), dim3(NT), lds, st_small, d_items, d_stats, max_sweeps, tol);
        }
        KFAC_HIP_CHECK(hipGetLastError());
        KFAC_HIP_CHECK(hipMemcpyAsync(sstats, d_stats, ns * sizeof(EigStat), hipMemcpyDeviceToHost, st_small));
    }

    // ---- blocked groups: set up, then drive them sweep by sweep as their norms arrive ----
    std::vector<GroupRun> runs(groups.size());
    // A group's sweeps are one dependent chain of launches on one stream.  Groups are dealt to the internal
    // streams longest chain first, each to the stream with the least work so far; the estimate per round is
    // a launch-latency floor plus the round's products at the rate those kernels reach.
    std::vector<int> stream_of(groups.size(), 0);
    // Measurement aid: while per-kernel timing is on (kfac_profile_begin) or KFAC_EIG_SERIAL is set, all groups share
    // one stream, so an event bracket (or a profiler's kernel duration) is the kernel's own time and not also its
    // wait behind the other groups' kernels.
    const bool serial = ctx->prof_on || getenv("KFAC_EIG_SERIAL") != nullptr;
    {
        std::vector<std::pair<double, size_t>> cost(groups.size());
        for (size_t gi = 0; gi < groups.size(); ++gi) {
            const GroupPlan &gp = groups[gi];
            double n2 = 0.0;
            for (int b : gp.members) n2 += (double)d[b] * d[b];
            double t;
            if (gp.two_level) t = gp.splayers * (350e-6 + 4.0 * n2 * LDI / 130e12);
            else t = (gp.players - 1) * std::max(90e-6, 8.0 * n2 * EB / 20e12);
            cost[gi] = {t, gi};
        }
        std::sort(cost.begin(), cost.end(), [](const std::pair<double, size_t> &a, const std::pair<double, size_t> &b) { return a.first > b.first; });
        double load[KFAC_NUM_AUX_STREAMS] = {0};
        if (!small.empty()) load[KFAC_NUM_AUX_STREAMS - 1] += 0.5e-3;   // the small factors' one launch
        for (auto &c : cost) {
            int best = 0;
            for (int i = 1; i < KFAC_NUM_AUX_STREAMS && !serial; ++i) if (load[i] < load[best]) best = i;
            stream_of[c.second] = best;
            load[best] += c.first;
        }
    }
    double *pinned = ctx->pinned;
    for (size_t gi = 0; gi < groups.size(); ++gi) {
        GroupPlan &gp = groups[gi];
        GroupRun &r = runs[gi];
        r.plan = &gp;
        r.nm = (int)gp.members.size();
        r.tol2 = (double)tol * tol;
        r.st = ctx->aux[stream_of[gi]];
        for (int k = 0; k < KFAC_EIG_SLOTS; ++k) r.ev[k] = ctx->ev_group[KFAC_EIG_SLOTS * gi + k];
        r.next_slot = 0;
        const size_t np2 = (size_t)gp.npad * gp.npad;
        const int nm = r.nm;
        char *p = wsp;
        BlkGroup &g = r.g;
        g.nmat = nm; g.nblk = gp.nblk; g.npad = gp.npad; g.players = gp.players; g.npairs = gp.npairs;
        g.bipartite = 0;
        g.W = (float *)p;
        g.Qw = g.W + nm * np2;
        r.Qalt = nullptr;
        if (gp.two_level) {
            SpGroup &sp = r.sp;
            sp.W = g.W;
            sp.T = g.W + 2 * nm * np2;
            r.Qalt = g.W + 3 * nm * np2;
            sp.nmat = nm; sp.npad = gp.npad; sp.nsuper = gp.nsuper; sp.players = gp.splayers;
            p += kfac_align_up(nm * 4 * np2 * sizeof(float), 256);
            sp.Vi = (float *)p;
            p += kfac_align_up((size_t)nm * gp.U * LDI * LDI * sizeof(float), 256);
            float *Jin = (float *)p; p += kfac_align_up(gp.inner_mats() * 4 * KP * KP * sizeof(float), 256);
            int *idtin = (int *)p; p += kfac_align_up(gp.inner_mats() * 4 * sizeof(int), 256);
            sp.scale = (float *)p; p += kfac_align_up((size_t)nm * 2 * sizeof(float), 256);
            g.J = Jin; g.idt = idtin;   // unused by the flat kernels for this group
            // inner group of a regular outer round: units of 4 + 4 small blocks, bipartite pairing
            r.gi = BlkGroup{sp.W, sp.Vi, Jin, idtin, nullptr, nm * gp.U, 2 * SB / EB, LDI, 2 * SB / EB, SB / EB, 1, nullptr, 1,
                            1, gp.npad, 0, gp.splayers, gp.nsuper, 0, 0};
            // inner group of the diagonal phase: one super-block of 4 small blocks each, tournament pairing
            r.gd = BlkGroup{sp.W, sp.Vi, Jin, idtin, nullptr, nm * gp.nsuper, SB / EB, SB, SB / EB, SB / EB / 2, 0, nullptr, 1,
                            1, gp.npad, -1, gp.splayers, gp.nsuper, 0, 0};
        } else {
            p += kfac_align_up(nm * 2 * np2 * sizeof(float), 256);
            g.J = (float *)p; p += kfac_align_up((size_t)nm * gp.npairs * KP * KP * sizeof(float), 256);
            g.idt = (int *)p; p += kfac_align_up((size_t)nm * gp.npairs * sizeof(int), 256);
        }
        g.norms = (double *)p; p += kfac_align_up((size_t)nm * 2 * sizeof(double), 256);
        r.normpart = (double *)p; p += kfac_align_up((size_t)nm * 2 * NORM_PARTS_MAX * sizeof(double), 256);
        int *done = (int *)p; p += kfac_align_up((size_t)nm * sizeof(int), 256);
        g.done = done;
        g.per_factor = 1;
        r.d_done = done;
        if (gp.two_level) {
            r.sp.done = done;
            r.gi.done = done; r.gi.per_factor = gp.U;
            r.gd.done = done; r.gd.per_factor = gp.nsuper;
        }
        KFAC_HIP_CHECK(hipMemsetAsync(done, 0, (size_t)nm * sizeof(int), r.st));
        r.perm = (int *)p; p += kfac_align_up((size_t)nm * gp.npad * sizeof(int), 256);
        r.lam64 = (double *)p; p += kfac_align_up((size_t)nm * gp.npad * (RAY_PARTS + 1) * sizeof(double), 256);
        r.d_items = (BlkItem *)p;
        wsp += gp.bytes();
        r.h_norms = pinned;
        pinned += (size_t)KFAC_EIG_SLOTS * 2 * nm;
        r.items.resize(nm);
        r.nmax = 0;
        r.apply_flops = 0.0;
        for (int i = 0; i < nm; ++i) {
            const int b = gp.members[i];
            r.items[i] = BlkItem{F[b], Q[b], lam[b], d[b], 0};
            r.nmax = std::max(r.nmax, d[b]);
            // algorithmic work of one round: W <- J^T W J on half the (symmetric) matrix and Q <- Q J,
            // each element a length-2*EB dot product: 8 n^2 EB flops per factor
            r.apply_flops += 8.0 * (double)d[b] * d[b] * EB;
        }
        // one visit of a pivot: KP/2 rounds over the cross pairs (the first round of a sweep also does the
        // pairs inside the blocks; not counted), 9 flops per element per round (S rotated twice, V once)
        r.solve_flops = (double)nm * gp.npairs * 9.0 * KP * KP * (KP / 2);
        r.ntiles_w = gp.npairs * (gp.npairs + 1) / 2;
        r.nrb = (r.nmax + KP - 1) / KP;
        r.ntiles = r.ntiles_w + ((r.nrb + 1) / 2) * gp.npairs;   // the accumulator part: two row slabs per workgroup
        r.fill_blocks = (int)std::min<size_t>((np2 + NT - 1) / NT, 4096);
        r.norm_blocks = std::min(r.fill_blocks, NORM_PARTS_MAX);
        r.sweep = 0;
        r.done = false;
        r.conv.assign(nm, 0);
        r.bad.assign(nm, 0);
        r.sweeps_done.assign(nm, 0);
        r.offrel.assign(nm, 0.f);
        BlkItem *h_items = (BlkItem *)ptab; ptab += kfac_align_up(nm * sizeof(BlkItem), 64);
        std::copy(r.items.begin(), r.items.end(), h_items);
        KFAC_HIP_CHECK(hipMemcpyAsync(r.d_items, h_items, nm * sizeof(BlkItem), hipMemcpyHostToDevice, r.st));
        {
            KfacProfScope prof(ctx, KC_EIG_MISC, 0.0, 0.0, r.st);
            hipLaunchKernelGGL(blk_init_kernel, dim3(r.fill_blocks, nm), dim3(NT), 0, r.st, g, r.d_items, warm ? 1 : 0);
        }
        KFAC_HIP_CHECK(hipGetLastError());
        if (warm) {
            // W <- Q0^T F Q0 for the start basis Q0 now in the accumulator; the caller's Q buffer (to be overwritten
            // anyway) holds the intermediate F Q0
            const BatchOperand bW{g.W, (int64_t)np2, 0}, bQ{g.Qw, (int64_t)np2, 0}, bF{nullptr, 0, 1}, bOut{nullptr, 0, 2};
            enqueue_product(ctx, r, bF, bQ, bOut, false);   // F Q0
            enqueue_product(ctx, r, bQ, bOut, bW, true);    // Q0^T (F Q0)
            KfacProfScope prof(ctx, KC_EIG_MISC, 0.0, 0.0, r.st);
            hipLaunchKernelGGL(blk_symmetrise_tiles_kernel, dim3((r.nmax * kfac::BM + NT - 1) / NT, nm), dim3(NT), 0, r.st, g.W, (int64_t)np2,
                               (int64_t)gp.npad, (const BlkItem *)r.d_items);
            KFAC_HIP_CHECK(hipGetLastError());
        }
        int rc = enqueue_offnorm(ctx, r);
        if (rc) return rc;
        r.x3 = gp.two_level && !fp32_outer;
        r.refreshed = !r.x3 || warm;   // a warm start begins from W = Q0^T F Q0 formed in fp32
        if (r.x3) {
            hipLaunchKernelGGL(sp_scale_kernel, dim3((nm + 63) / 64), dim3(64), 0, r.st, r.sp, (const double *)g.norms);
            KFAC_HIP_CHECK(hipGetLastError());
        }
    }
    // One sweep of a group = one chain of launches followed by a report (norms -> pinned memory, event).  The host
    // keeps one sweep queued behind the one whose report it is waiting for, so a stream never idles while the host
    // reads norms or enqueues another group's launches; the device-side flags make the workgroups of a factor
    // that converged meanwhile return at once, so a sweep queued in vain costs only its empty launches.
    // state per group: waiting for reports (post == 0) or for its post-processing (post == 1)
    const auto t_start = std::chrono::steady_clock::now();
    const bool trace = getenv("KFAC_EIG_TRACE") != nullptr;
    double host_enqueue_ms = 0.0;
    auto now_ms = [&]() { return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t_start).count(); };
    auto enqueue_sweep = [&](GroupRun &r) -> int {
        // The diagonal is put in order once the estimates are good enough to tell the clusters apart (after four sweeps:
        // off-norm below 1e-2), and once more near the end -- for split-engine groups that is part of the refresh.  A
        // sweep right after a reordering gains a little less than it would have, so more often does not pay (every
        // sweep: two sweeps more; after two sweeps already: one more).
        int rc = KFAC_OK;
        if (r.sweep == 4 || (r.sweep == 7 && !r.x3)) rc = enqueue_sort(ctx, r);
        if (rc != KFAC_OK) return rc;
        rc = r.plan->two_level ? enqueue_sweep_two_level(ctx, r, lds_solve, inner_cap, inner_tol)
                               : enqueue_sweep_flat(ctx, r, lds_solve, inner_cap, inner_tol);
        ++r.sweep;
        if (rc == KFAC_OK) rc = enqueue_offnorm(ctx, r);
        // measurement mode: all groups share one stream; keep its queue short (one group's sweep at a time), a
        // profiler that wraps every dispatch in packets of its own has little room behind thousands of launches
        if (rc == KFAC_OK && serial && hipStreamSynchronize(r.st) != hipSuccess) rc = KFAC_EHIP;
        return rc;
    };
    for (auto &r : runs)   // the first sweep goes out before its norms are known
        if (r.sweep < max_sweeps) KFAC_CHECK(enqueue_sweep(r));
    std::vector<char> post(runs.size(), 0);
    size_t remaining = runs.size();
    while (remaining > 0) {
        bool progressed = false;
        for (size_t gi = 0; gi < runs.size(); ++gi) {
            GroupRun &r = runs[gi];
            if (r.done) continue;
            if (post[gi]) {
                const hipError_t q = hipEventQuery(r.ev[0]);
                if (q == hipErrorNotReady) continue;
                if (q != hipSuccess) return KFAC_EHIP;
                progressed = true;
                r.done = true;
                --remaining;
                if (trace)
                    fprintf(stderr, "[kfac_eig] group nblk=%d (%d factors, stream %d) finished at %.1f ms\n", r.plan->nblk, r.nm,
                            (int)stream_of[gi], now_ms());
                continue;
            }
            if (r.reports.empty()) return KFAC_EHIP;   // cannot happen: a group that is not finishing has a report queued
            const GroupRun::Report R = r.reports.front();
            const hipError_t q = hipEventQuery(r.ev[R.slot]);
            if (q == hipErrorNotReady) continue;
            if (q != hipSuccess) return KFAC_EHIP;
            progressed = true;
            r.reports.pop_front();
            const double *hn = r.h_norms + (size_t)R.slot * 2 * r.nm;
            bool all = true;
            float worst = 0.f;
            for (int i = 0; i < r.nm; ++i) {
                const double o2 = hn[2 * i], n2 = o2 + hn[2 * i + 1];
                r.offrel[i] = n2 > 0 ? (float)std::sqrt(o2 / n2) : 0.f;
                const bool c = o2 <= (double)tol * tol * n2;   // false for NaN
                r.bad[i] = !std::isfinite(n2);
                all &= c || r.bad[i];
                if (!r.bad[i]) worst = std::max(worst, r.offrel[i]);
                if (R.final_ok) {   // no factor of a split-engine group counts as converged before the refresh
                    if (c && !r.conv[i]) r.sweeps_done[i] = R.sweeps;
                    r.conv[i] = c;
                }
            }
            if (trace) {   // debugging aid: the convergence history on stderr
                fprintf(stderr, "[kfac_eig] %.1f ms group nblk=%d sweep %d%s off/norm:", now_ms(), r.plan->nblk, R.sweeps, R.final_ok ? "" : " (before refresh)");
                for (int i = 0; i < r.nm; ++i) fprintf(stderr, " %.2e", r.offrel[i]);
                fprintf(stderr, "\n");
            }
            const double t_enq = now_ms();
            int rc = KFAC_OK;
            if (R.final_ok && (all || R.sweeps >= max_sweeps)) {
                rc = enqueue_post(ctx, r);     // after whatever is still queued, which no longer changes anything
                post[gi] = 1;
                r.reports.clear();
            } else {
                if (!r.refreshed && R.sweeps > 0 && (all || worst <= refresh_at || R.sweeps >= max_sweeps)) {
                    rc = enqueue_refresh(ctx, r);
                    if (rc == KFAC_OK) rc = enqueue_offnorm(ctx, r);
                }
                while (rc == KFAC_OK && r.reports.size() < 2 && r.sweep < max_sweeps) rc = enqueue_sweep(r);
            }
            host_enqueue_ms += now_ms() - t_enq;
            if (rc) return rc;
        }
        // nothing ready: poll again shortly.  (Blocking on one group's event would leave every other group
        // that finishes its sweep earlier waiting for the host.)
        if (!progressed) std::this_thread::sleep_for(std::chrono::microseconds(20));
    }
    if (trace) fprintf(stderr, "[kfac_eig] all groups done at %.1f ms; host time spent enqueueing %.1f ms\n", now_ms(), host_enqueue_ms);
    // the statistics of the small factors are read below
    KFAC_HIP_CHECK(hipStreamSynchronize(st_small));

    for (size_t i = 0; i < small.size(); ++i) {
        const bool conv = sstats[i].converged > 0.5f;
        all_conv &= conv;
        const double k = (d[small[i]] + 1) & ~1;   // 9 flops per element per round: S twice, V once
        if (ctx->prof_on)
            for (auto it = ctx->prof.rbegin(); it != ctx->prof.rend(); ++it)
                if (it->cls == KC_EIG_SMALL) { it->flops += sstats[i].sweeps * 9.0 * k * k * (k - 1); break; }
        if (info) info[small[i]] = kfac_eig_info{(int)sstats[i].sweeps, sstats[i].off_rel, conv ? 1 : 0};
    }
    for (auto &r : runs) {
        for (int i = 0; i < r.nm; ++i) {
            all_conv &= (bool)r.conv[i];
            if (info) info[r.plan->members[i]] = kfac_eig_info{r.conv[i] ? r.sweeps_done[i] : r.sweep, r.offrel[i], r.conv[i] ? 1 : 0};
        }
    }
    return all_conv ? KFAC_OK : KFAC_ENOCONV;
}

int kfac_launch_eig(kfac_ctx *ctx, int batch, const float *const *F, const int *d, float *const *Q,
                    float *const *lam, const kfac_eig_opts *opts, kfac_eig_info *info) {
    std::vector<int> small;
    std::vector<GroupPlan> groups;
    make_plan(batch, d, small, groups);
    if (kfac_eig_ws_bytes_impl(batch, d) > ctx->ws_bytes) return KFAC_EWORKSPACE;
    if (groups.size() > (size_t)KFAC_MAX_GROUPS) return KFAC_EINVAL;
    size_t norms_need = 0, tables_need = kfac_align_up(small.size() * sizeof(SmallItem), 64) + kfac_align_up(small.size() * sizeof(EigStat), 64);
    for (auto &gp : groups) {
        norms_need += (size_t)KFAC_EIG_SLOTS * 2 * gp.members.size() * sizeof(double);
        tables_need += kfac_align_up(gp.members.size() * sizeof(BlkItem), 64);
    }
    if (norms_need > KFAC_PINNED_NORMS || tables_need > KFAC_PINNED_TABLES) return KFAC_EINVAL;   // more than 4096 factors
    // the internal streams start after everything already queued on the caller's stream ...
    KFAC_HIP_CHECK(hipEventRecord(ctx->ev_fork, ctx->stream));
    for (int i = 0; i < KFAC_NUM_AUX_STREAMS; ++i) KFAC_HIP_CHECK(hipStreamWaitEvent(ctx->aux[i], ctx->ev_fork, 0));
    const int rc = eig_run(ctx, batch, F, d, Q, lam, opts, info, small, groups);
    // ... and the caller's stream continues after all of them.  On an error, too: whatever was queued before it is
    // waited for here, so no kernel of this call is in flight, and no pointer of the caller in use, after the return.
    int jrc = KFAC_OK;
    for (int i = 0; i < KFAC_NUM_AUX_STREAMS; ++i) {
        if (hipEventRecord(ctx->ev_join[i], ctx->aux[i]) != hipSuccess) jrc = KFAC_EHIP;
        else if (hipStreamWaitEvent(ctx->stream, ctx->ev_join[i], 0) != hipSuccess) jrc = KFAC_EHIP;
    }
    for (int i = 0; i < KFAC_NUM_AUX_STREAMS; ++i)
        if (hipStreamSynchronize(ctx->aux[i]) != hipSuccess) jrc = KFAC_EHIP;
    return (rc != KFAC_OK && rc != KFAC_ENOCONV) ? rc : (jrc != KFAC_OK ? jrc : rc);
}
