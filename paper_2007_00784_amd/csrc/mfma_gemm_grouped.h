// Grouped-load MFMA tile engine for gfx950, for the Gram matrices of samples in [N][d][T] layout (row i of
// example n holds T consecutive positions), fp32 or bf16: the same 128x128 workgroup tile and accumulator layout
// as the generic fp32 engine, but every operand access is 16 bytes wide from HBM to the matrix core.
//
// The contraction runs over "groups" of EPG = 16 / sizeof(E) consecutive positions of one example (4 fp32, 8 bf16),
// q = n * gpe + gi with gpe = ceil(T / EPG); group gi covers positions EPG gi .. EPG gi + EPG - 1.  A group travels
// from global memory straight into LDS (one 16-byte direct load per lane) and a lane's MFMA operands of a group
// are one 16-byte LDS read: no staging registers, no LDS store instructions and a quarter (fp32) or an eighth
// (bf16) of the LDS reads of the element-wise engine.
// Rows are not 16-byte aligned when T is odd, so the loads are unaligned ones (global memory allows that).  The
// last group of an example, when T is not a multiple of EPG, is loaded from position T - EPG instead and the
// positions that the previous group already covered are cleared in LDS once the load has landed: no load ever
// leaves its row, and since both operands of a product use the same grouping the sum over positions is
// unchanged.  Requires T >= EPG.
//
// bf16 operands stay bf16 all the way (v_mfma_f32_32x32x16_bf16: exact products, fp32 accumulation, 16 times the
// fp32 MFMA rate); at that rate the tile is bound by operand delivery through LDS, not by the matrix core.
// A K slab is 8 groups (128 bytes per operand row: whole cache lines), and a diagonal tile of a symmetric product
// loads its operand once.
#pragma once
#include "mfma_gemm.h"

namespace kfac {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int GRP_GROUPS = 8;                  // groups per K slab
constexpr int GRP_ROWB = 16 * GRP_GROUPS;      // LDS bytes per operand row: 128 B, no padding; the group slots of a
                                               // row are permuted instead (physical slot = group ^ ((row >> 1) & 7)),
                                               // which keeps both the 16-byte fragment reads and the landing
                                               // loads free of bank conflicts
constexpr int GRP_RPT = BM * GRP_GROUPS / NTHREADS;   // (row, group) pairs per thread per slab = 4

struct GrpSmem {
    __attribute__((aligned(16))) char a[2][BM * GRP_ROWB];
    __attribute__((aligned(16))) char b[2][BM * GRP_ROWB];
};

// Source of the groups that lie outside an operand (rows >= d, groups past the end of the contraction).
static __device__ __attribute__((aligned(16))) unsigned grp_zero16[4];

// s_waitcnt vmcnt(0) with the other counters unconstrained (gfx9 encoding: vmcnt in bits 3:0 and 15:14,
// expcnt 6:4, lgkmcnt 11:8): all of this wave's loads, including those that land in LDS, have completed.
__device__ inline void grp_wait_loads() { __builtin_amdgcn_s_waitcnt((0x7 << 4) | (0xF << 8)); }

template <typename E> struct GrpTraits;
template <> struct GrpTraits<float> {
    static constexpr int EPG = 4;
    // keep elements sh.. of a group: one mask per dword
    __device__ static void masks(int sh, unsigned (&m)[4]) {
#pragma unroll
        for (int w = 0; w < 4; ++w) m[w] = w >= sh ? 0xffffffffu : 0u;
    }
    __device__ static float sum(const uint4 &x) {
        return (__uint_as_float(x.x) + __uint_as_float(x.y)) + (__uint_as_float(x.z) + __uint_as_float(x.w));
    }
};
template <> struct GrpTraits<unsigned short> {   // bf16 bits
    static constexpr int EPG = 8;
    __device__ static void masks(int sh, unsigned (&m)[4]) {
#pragma unroll
        for (int w = 0; w < 4; ++w) m[w] = (2 * w >= sh ? 0x0000ffffu : 0u) | (2 * w + 1 >= sh ? 0xffff0000u : 0u);
    }
    __device__ static float sum(const uint4 &x) {
        const unsigned w[4] = {x.x, x.y, x.z, x.w};
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) s += __uint_as_float(w[i] << 16) + __uint_as_float(w[i] & 0xffff0000u);
        return s;
    }
};

// Thread mapping: physical slot tid & 7 of rows (tid >> 3) + 32 u, u = 0..3, i.e. group (tid & 7) ^ ((tid >> 4) & 7)
// (the permutation term is the same for the four rows).  A slab is moved by global_load_lds_dwordx4: every lane
// names its own 16 bytes of global memory and the wave's 64 groups land in 1 KB of consecutive LDS (lane l at
// 16 l, i.e. eight whole rows), with no trip through registers and no LDS store instructions -- staging through
// registers was what bound this engine (a probe of the bf16 loop: 450 TFLOP/s with register staging even without
// any global loads, 700 with direct loads).
template <typename E>
struct GrpOpNDT {
    static constexpr int EPG = GrpTraits<E>::EPG;
    const E *p;
    int d, T, gpe;
    int q_end;            // groups q >= q_end read as zero
    // thread state
    int rowoff[GRP_RPT];  // row * T (row clamped into the operand; d * T < 2^31 is checked on the host)
    unsigned rowmask;     // per u: row inside the operand
    int q, n, gi;
    __device__ void start(int tid, int i0, int q0) {
        q = q0 + ((tid & 7) ^ ((tid >> 4) & 7));
        n = q / gpe;
        gi = q - n * gpe;
        rowmask = 0;
#pragma unroll
        for (int u = 0; u < GRP_RPT; ++u) {
            const int row = i0 + (tid >> 3) + 32 * u;
            rowmask |= (row < d ? 1u : 0u) << u;
            rowoff[u] = min(row, d - 1) * T;
        }
    }
    // Start the loads of this thread's groups of the current slab into `slab` (this operand's 16 KB buffer).
    // Returns how many leading positions of the landed groups belong to the previous group of the example
    // (the last, overlapping group when T is not a multiple of EPG) and must be cleared by patch().
    __device__ int issue(char *slab, int tid) const {
        const bool valid = q < q_end;
        const int t0 = min(EPG * gi, T - EPG);
        const E *base = p + (valid ? (int64_t)n * d * T + t0 : (int64_t)0);
        const int wave = tid >> 6;
#pragma unroll
        for (int u = 0; u < GRP_RPT; ++u) {
            const bool ok = valid && ((rowmask >> u) & 1u);
            const void *src = ok ? (const void *)(base + rowoff[u]) : (const void *)grp_zero16;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                             (__attribute__((address_space(3))) void *)(slab + (8 * wave + 32 * u) * GRP_ROWB), 16, 0, 0);
        }
        return valid ? EPG * gi - t0 : 0;
    }
    // After the loads have landed: clear the first `sh` positions of this thread's groups.
    __device__ void patch(char *slab, int tid, int sh) const {
        if (sh == 0) return;
        unsigned m[4];
        GrpTraits<E>::masks(sh, m);
#pragma unroll
        for (int u = 0; u < GRP_RPT; ++u) {
            uint4 *x = reinterpret_cast<uint4 *>(slab + ((tid >> 3) + 32 * u) * GRP_ROWB + (tid & 7) * 16);
            uint4 v = *x;
            v.x &= m[0]; v.y &= m[1]; v.z &= m[2]; v.w &= m[3];
            *x = v;
        }
    }
    // Sum of the elements of this thread's landed (and patched) group of row u.
    __device__ static float landed_sum(const char *slab, int tid, int u) {
        return GrpTraits<E>::sum(*reinterpret_cast<const uint4 *>(slab + ((tid >> 3) + 32 * u) * GRP_ROWB + (tid & 7) * 16));
    }
    __device__ void next() {
        q += GRP_GROUPS;
        gi += GRP_GROUPS;
        while (gi >= gpe) { gi -= gpe; ++n; }
    }
};

// One slab of MFMAs from fragments: lane (c, g) holds group 2 ks + g of row (column) c in k-step ks.  Any
// assignment of contraction indices to MFMA k-lanes works as long as both operands share it.  `blocks` (uniform
// over the wave) has bit 2 i + j set for the 32 x 32 accumulator blocks that anybody will read: blocks past the
// edge of the operand and, in a diagonal tile, blocks strictly above the diagonal are left at zero and cost
// no matrix-core time (a seventh of a ResNet-50 factor update's MFMAs otherwise).  `ksteps` has bit ks set for the
// k-steps of the slab this wave multiplies (all four, except where two waves share a quadrant).
template <int KS0, int KS1>
__device__ inline void grp_mfma(const uint4 (&fa)[4][2], const uint4 (&fb)[4][2], floatx16 (&acc)[2][2], unsigned blocks, unsigned ksteps, float) {
#pragma unroll
    for (int ks = KS0; ks < KS1; ++ks) {
        if (!((ksteps >> ks) & 1u)) continue;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                if (!((blocks >> (2 * i + j)) & 1u)) continue;
                const unsigned a[4] = {fa[ks][i].x, fa[ks][i].y, fa[ks][i].z, fa[ks][i].w};
                const unsigned b[4] = {fb[ks][j].x, fb[ks][j].y, fb[ks][j].z, fb[ks][j].w};
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[e]), __uint_as_float(b[e]), acc[i][j], 0, 0, 0);
            }
    }
}
template <int KS0, int KS1>
__device__ inline void grp_mfma(const uint4 (&fa)[4][2], const uint4 (&fb)[4][2], floatx16 (&acc)[2][2], unsigned blocks, unsigned ksteps, unsigned short) {
#pragma unroll
    for (int ks = KS0; ks < KS1; ++ks) {
        if (!((ksteps >> ks) & 1u)) continue;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                if (!((blocks >> (2 * i + j)) & 1u)) continue;
                bf16x8 x, y;
                __builtin_memcpy(&x, &fa[ks][i], 16);
                __builtin_memcpy(&y, &fb[ks][j], 16);
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, acc[i][j], 0, 0, 0);
            }
    }
}

// acc = A B^T over groups [q0, q_end) (both operands as elem(row, position)); DIAG: B is the same row block
// as A and is neither loaded nor staged.  With COLSUM every thread also accumulates, per u, the sum of the
// A-operand elements it fetches (csum[u]); summed over the eight threads that share a row this is the row's
// sum over all positions.
template <typename E, bool DIAG, bool COLSUM>
__device__ inline void gemm_tile_grouped(GrpOpNDT<E> &A, GrpOpNDT<E> &B, int i0, int j0, int q0, int q_end, GrpSmem &sm,
                                         floatx16 (&acc)[2][2], float *csum) {
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    // In a diagonal tile the quadrant above the diagonal (wave 1's) is never read, while the one below it is the
    // only quadrant with four blocks to compute (the two on the diagonal have three).  Wave 1 therefore takes half
    // of wave 2's work: both multiply the lower-left quadrant, each over two of a slab's four k-steps, and the two
    // sums are added through LDS at the end.  No wave then has more than 12 of a slab's block-steps instead of 16.
    const bool helper = DIAG && wave == 1;
    const int wm = helper ? 64 : (wave >> 1) * 64, wn = helper ? 0 : (wave & 1) * 64;
    const unsigned ksteps = __builtin_amdgcn_readfirstlane(!DIAG ? 0xFu : wave == 1 ? 0xCu : wave == 2 ? 0x3u : 0xFu);
    const int lk = lane >> 5, lc = lane & 31;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    const int nslab = (q_end - q0 + GRP_GROUPS - 1) / GRP_GROUPS;
    if (nslab <= 0) return;
    // Two LDS buffers.  Step s: wait for this wave's loads of slab s, clear overlapping positions, barrier (slab s is
    // complete and nobody reads slab s-1 any more), start the loads of slab s+1 into the buffer slab s-1 used, then
    // multiply slab s.  The loads fly during the MFMAs of the slab before; the second workgroup on the compute unit
    // covers what is left of their latency.
    A.q_end = q_end;
    B.q_end = q_end;
    A.start(tid, i0, q0);
    if (!DIAG) B.start(tid, j0, q0);
    int sha = A.issue(sm.a[0], tid), shb = 0;
    if (!DIAG) shb = B.issue(sm.b[0], tid);
    const int swz = (lc >> 1) & 7;   // (row >> 1) & 7 of this lane's fragment rows (they differ by multiples of 32)
    unsigned blocks = 0;             // this wave's accumulator blocks that hold entries of the factor's lower triangle
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
            if (i0 + wm + 32 * i < A.d && j0 + wn + 32 * j < A.d && (!DIAG || wn + 32 * j <= wm + 32 * i)) blocks |= 1u << (2 * i + j);
    blocks = __builtin_amdgcn_readfirstlane(blocks);
    for (int s = 0; s < nslab; ++s) {
        const int cur = s & 1;
        grp_wait_loads();
        A.patch(sm.a[cur], tid, sha);
        if (!DIAG) B.patch(sm.b[cur], tid, shb);
        if (COLSUM) {
#pragma unroll
            for (int u = 0; u < GRP_RPT; ++u) csum[u] += GrpOpNDT<E>::landed_sum(sm.a[cur], tid, u);
        }
        __syncthreads();
        const char *pa = sm.a[cur];
        const char *pb = DIAG ? sm.a[cur] : sm.b[cur];
        uint4 fa[4][2], fb[4][2];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                fa[ks][i] = *reinterpret_cast<const uint4 *>(pa + (wm + 32 * i + lc) * GRP_ROWB + (((2 * ks + lk) ^ swz) * 16));
                fb[ks][i] = *reinterpret_cast<const uint4 *>(pb + (wn + 32 * i + lc) * GRP_ROWB + (((2 * ks + lk) ^ swz) * 16));
            }
        __builtin_amdgcn_sched_barrier(0);
        grp_mfma<0, 1>(fa, fb, acc, blocks, ksteps, E());
        __builtin_amdgcn_sched_barrier(0);
        if (s + 1 < nslab) {   // address arithmetic and load issue in the shadow of the MFMAs just queued
            A.next();
            sha = A.issue(sm.a[cur ^ 1], tid);
            if (!DIAG) {
                B.next();
                shb = B.issue(sm.b[cur ^ 1], tid);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        grp_mfma<1, 4>(fa, fb, acc, blocks, ksteps, E());
    }
    __syncthreads();   // callers reuse the slab buffers
    if (DIAG) {        // wave 2 += wave 1 (16 KB through LDS); wave 1 ends with the zeros of the quadrant it stands for
        float *x = reinterpret_cast<float *>(&sm);
        if (wave == 1) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        x[((i * 2 + j) * 16 + r) * 64 + lane] = acc[i][j][r];
                        acc[i][j][r] = 0.f;
                    }
        }
        __syncthreads();
        if (wave == 2) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] += x[((i * 2 + j) * 16 + r) * 64 + lane];
        }
        __syncthreads();
    }
}

// The single (diagonal) tile of a factor with at most 64 rows.  A 128 x 128 tile would spend three quarters of its
// MFMAs on rows and columns that do not exist; here all four waves compute the same 64 x 64 block, each over a
// quarter of every slab (k-step `wave`), and the four partial sums are added through LDS at the end.  On return
// wave 0 holds the block in the usual accumulator layout and the other waves hold zeros.
template <typename E, bool COLSUM>
__device__ inline void gemm_tile_grouped_small(GrpOpNDT<E> &A, int q0, int q_end, GrpSmem &sm, floatx16 (&acc)[2][2], float *csum) {
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lk = lane >> 5, lc = lane & 31;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    const int nslab = (q_end - q0 + GRP_GROUPS - 1) / GRP_GROUPS;
    if (nslab <= 0) return;
    A.q_end = q_end;
    A.start(tid, 0, q0);
    int sha = A.issue(sm.a[0], tid);
    const int swz = (lc >> 1) & 7;
    for (int s = 0; s < nslab; ++s) {
        const int cur = s & 1;
        grp_wait_loads();
        A.patch(sm.a[cur], tid, sha);
        if (COLSUM) {
#pragma unroll
            for (int u = 0; u < GRP_RPT; ++u) csum[u] += GrpOpNDT<E>::landed_sum(sm.a[cur], tid, u);
        }
        __syncthreads();
        uint4 f[2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
            f[i] = *reinterpret_cast<const uint4 *>(sm.a[cur] + (32 * i + lc) * GRP_ROWB + (((2 * wave + lk) ^ swz) * 16));
        __builtin_amdgcn_sched_barrier(0);
        if (s + 1 < nslab) {
            A.next();
            sha = A.issue(sm.a[cur ^ 1], tid);
        }
        if (sizeof(E) == 4) {
            const unsigned a[2][4] = {{f[0].x, f[0].y, f[0].z, f[0].w}, {f[1].x, f[1].y, f[1].z, f[1].w}};
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[i][e]), __uint_as_float(a[j][e]), acc[i][j], 0, 0, 0);
        } else {
            bf16x8 x[2];
            __builtin_memcpy(&x[0], &f[0], 16);
            __builtin_memcpy(&x[1], &f[1], 16);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x[i], x[j], acc[i][j], 0, 0, 0);
        }
    }
    __syncthreads();
    float *scratch = reinterpret_cast<float *>(&sm);   // 3 waves x 64 values x 64 lanes = 48 KB of the 64 KB
    if (wave > 0) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    scratch[(((wave - 1) * 64) + (i * 2 + j) * 16 + r) * 64 + lane] = acc[i][j][r];
                    acc[i][j][r] = 0.f;
                }
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int w = 0; w < 3; ++w)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] += scratch[((w * 64) + (i * 2 + j) * 16 + r) * 64 + lane];
    }
    __syncthreads();   // callers reuse the slab buffers
}

}  // namespace kfac
