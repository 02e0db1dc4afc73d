// Grouped-load MFMA tile engine for gfx950, for the Gram matrices of samples in [N][d][T] layout (row i of
// example n holds T consecutive positions), fp32 or bf16: the same 128x128 workgroup tile and accumulator layout
// as the generic fp32 engine, but every operand access is 16 bytes wide from HBM to the matrix core.
//
// The contraction runs over "groups" of EPG = 16 / sizeof(E) consecutive positions of one example (4 fp32, 8 bf16),
// q = n * gpe + gi with gpe = ceil(T / EPG); group gi covers positions EPG gi .. EPG gi + EPG - 1.  A thread moves a
// group with one 16-byte load and one 16-byte LDS store, and a lane's MFMA operands of a group are one 16-byte LDS
// read: a quarter (fp32) or an eighth (bf16) of the memory instructions of the element-wise engine, which is what
// separated that engine (102-117 TFLOP/s fp32 on a probe) from what its LDS reads and MFMAs alone sustain (142).
// Rows are not 16-byte aligned when T is odd, so the loads are unaligned ones (global memory allows that).  The
// last group of an example, when T is not a multiple of EPG, is loaded from position T - EPG instead and the
// positions that the previous group already covered are masked to zero: no load ever leaves its row, and since
// both operands of a product use the same grouping the sum over positions is unchanged.  Requires T >= EPG.
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
constexpr int GRP_ROWB = 16 * GRP_GROUPS + 16; // LDS bytes per operand row: 128 B of data, 16 B pad
                                               // (144 B = 36 banks: sixteen 16-byte accesses at this pitch
                                               // hit distinct banks)
constexpr int GRP_RPT = BM * GRP_GROUPS / NTHREADS;   // (row, group) pairs per thread per slab = 4

struct GrpSmem {
    __attribute__((aligned(16))) char a[2][BM * GRP_ROWB];
    __attribute__((aligned(16))) char b[2][BM * GRP_ROWB];
};

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

// Thread mapping: group slot gs = tid & 7, rows (tid >> 3) + 32 u, u = 0..3.
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
        q = q0 + (tid & 7);
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
    // Issue the loads of this thread's groups; `m` receives the element masks that apply() puts on them.  Kept
    // apart so that nothing touches the loaded registers until the slab is moved to LDS, one or two steps later.
    __device__ void fetch(uint4 (&v)[GRP_RPT], unsigned (&m)[4]) const {
        const bool valid = q < q_end;
        const int t0 = min(EPG * gi, T - EPG);
        const int sh = valid ? EPG * gi - t0 : EPG;   // positions below sh belong to the previous group (or nothing is valid)
        const E *base = p + (valid ? (int64_t)n * d * T + t0 : (int64_t)0);
        GrpTraits<E>::masks(sh, m);
#pragma unroll
        for (int u = 0; u < GRP_RPT; ++u) __builtin_memcpy(&v[u], base + rowoff[u], 16);
    }
    __device__ void apply(uint4 (&v)[GRP_RPT], const unsigned (&m)[4]) const {
#pragma unroll
        for (int u = 0; u < GRP_RPT; ++u) {
            const unsigned keep = ((rowmask >> u) & 1u) ? 0xffffffffu : 0u;
            v[u].x &= m[0] & keep;
            v[u].y &= m[1] & keep;
            v[u].z &= m[2] & keep;
            v[u].w &= m[3] & keep;
        }
    }
    __device__ void next() {
        q += GRP_GROUPS;
        gi += GRP_GROUPS;
        while (gi >= gpe) { gi -= gpe; ++n; }
    }
    __device__ static void store(char *slab, const uint4 (&v)[GRP_RPT], int tid) {
#pragma unroll
        for (int u = 0; u < GRP_RPT; ++u)
            *reinterpret_cast<uint4 *>(slab + ((tid >> 3) + 32 * u) * GRP_ROWB + (tid & 7) * 16) = v[u];
    }
};

// One slab of MFMAs from fragments: lane (c, g) holds group 2 ks + g of row (column) c in k-step ks.  Any
// assignment of contraction indices to MFMA k-lanes works as long as both operands share it.
__device__ inline void grp_mfma(const uint4 (&fa)[4][2], const uint4 (&fb)[4][2], floatx16 (&acc)[2][2], float) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const unsigned a[2][4] = {{fa[ks][0].x, fa[ks][0].y, fa[ks][0].z, fa[ks][0].w}, {fa[ks][1].x, fa[ks][1].y, fa[ks][1].z, fa[ks][1].w}};
        const unsigned b[2][4] = {{fb[ks][0].x, fb[ks][0].y, fb[ks][0].z, fb[ks][0].w}, {fb[ks][1].x, fb[ks][1].y, fb[ks][1].z, fb[ks][1].w}};
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[i][e]), __uint_as_float(b[j][e]), acc[i][j], 0, 0, 0);
    }
}
__device__ inline void grp_mfma(const uint4 (&fa)[4][2], const uint4 (&fb)[4][2], floatx16 (&acc)[2][2], unsigned short) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                bf16x8 x, y;
                __builtin_memcpy(&x, &fa[ks][i], 16);
                __builtin_memcpy(&y, &fb[ks][j], 16);
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, acc[i][j], 0, 0, 0);
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
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int lk = lane >> 5, lc = lane & 31;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    const int nslab = (q_end - q0 + GRP_GROUPS - 1) / GRP_GROUPS;
    if (nslab <= 0) return;
    // Pipeline: slab s is multiplied out of LDS while slab s+1 waits in registers for its LDS buffer and the
    // loads of slab s+2 are in flight: at the bf16 MFMA rate one slab of arithmetic is much shorter than a trip
    // to L2, so a single slab of look-ahead leaves the matrix core idle most of the time.  Slabs past the end read
    // as zero (q >= q_end), so the look-ahead needs no special case.
    uint4 ra[2][GRP_RPT], rb[2][GRP_RPT];
    unsigned ma[2][4], mb[2][4];
    A.q_end = q_end;
    B.q_end = q_end;
    A.start(tid, i0, q0);
    A.fetch(ra[0], ma[0]);
    if (!DIAG) {
        B.start(tid, j0, q0);
        B.fetch(rb[0], mb[0]);
    }
    A.next();
    A.fetch(ra[1], ma[1]);   // slab 1
    if (!DIAG) {
        B.next();
        B.fetch(rb[1], mb[1]);
    }
    A.apply(ra[0], ma[0]);
    if (!DIAG) B.apply(rb[0], mb[0]);
    if (COLSUM) {
#pragma unroll
        for (int u = 0; u < GRP_RPT; ++u) csum[u] += GrpTraits<E>::sum(ra[0][u]);
    }
    GrpOpNDT<E>::store(sm.a[0], ra[0], tid);
    if (!DIAG) GrpOpNDT<E>::store(sm.b[0], rb[0], tid);
    __syncthreads();
    // one step: start the loads of slab s+2 into set f (free since slab s went to LDS), multiply slab s out of
    // LDS buffer s & 1, then move slab s+1, whose loads have had two steps to land, from set o to the other buffer
    auto step = [&](int s, int f, int o) {
        const int cur = s & 1;
        if (s + 2 < nslab) {
            A.next();
            A.fetch(ra[f], ma[f]);
            if (!DIAG) {
                B.next();
                B.fetch(rb[f], mb[f]);
            }
        }
        const char *pa = sm.a[cur];
        const char *pb = DIAG ? sm.a[cur] : sm.b[cur];
        uint4 fa[4][2], fb[4][2];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                fa[ks][i] = *reinterpret_cast<const uint4 *>(pa + (wm + 32 * i + lc) * GRP_ROWB + (2 * ks + lk) * 16);
                fb[ks][i] = *reinterpret_cast<const uint4 *>(pb + (wn + 32 * i + lc) * GRP_ROWB + (2 * ks + lk) * 16);
            }
        __builtin_amdgcn_sched_barrier(0);
        grp_mfma(fa, fb, acc, E());
        if (s + 1 < nslab) {
            A.apply(ra[o], ma[o]);
            if (!DIAG) B.apply(rb[o], mb[o]);
            if (COLSUM) {
#pragma unroll
                for (int u = 0; u < GRP_RPT; ++u) csum[u] += GrpTraits<E>::sum(ra[o][u]);
            }
            GrpOpNDT<E>::store(sm.a[cur ^ 1], ra[o], tid);
            if (!DIAG) GrpOpNDT<E>::store(sm.b[cur ^ 1], rb[o], tid);
        }
        __syncthreads();
    };
    for (int s = 0; s < nslab; s += 2) {
        step(s, 0, 1);           // slab s+1 sits in set 1; slab s+2 is fetched into set 0
        if (s + 1 < nslab) step(s + 1, 1, 0);
    }
}

}  // namespace kfac
