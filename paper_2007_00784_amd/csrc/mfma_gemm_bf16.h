// bf16 MFMA tile engine for gfx950, for the Gram matrices of bf16 samples: the same 128x128 workgroup tile
// and accumulator layout as the fp32 engine, but the operands stay bf16 from HBM to the matrix core
// (v_mfma_f32_32x32x16_bf16: exact products, fp32 accumulation), which runs at 16 times the fp32 MFMA rate.
// At that rate the tile is bound by operand delivery (L2 -> LDS -> registers), not by the matrix core, so the
// K slab is deep (64 sample rows: whole 128-byte lines per operand row) and a diagonal tile of a symmetric
// product loads its operand once.
//
// Samples are in [N][d][T] layout: row i of example n holds T consecutive positions.  The contraction runs
// over "groups" of eight positions of one example, q = n * gpe + gi with gpe = ceil(T / 8); group gi covers
// positions 8 gi .. 8 gi + 7.  Rows are not 16-byte aligned when T is odd, so the 16-byte loads are
// unaligned ones (global memory allows that).  The last group of an example, when T is not a multiple of
// eight, is loaded from position T - 8 instead and the positions that the previous group already covered are
// masked to zero: no load ever leaves its row, and since both operands of a product use the same grouping
// the sum over positions is unchanged.  Requires T >= 8.
#pragma once
#include "mfma_gemm.h"

namespace kfac {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int B16_GROUPS = 8;                  // groups per K slab
constexpr int B16_ROWB = 16 * B16_GROUPS + 16; // LDS bytes per operand row: 128 B of data, 16 B pad
                                               // (144 B = 36 banks: sixteen 16-byte accesses at this pitch
                                               // hit distinct banks)
constexpr int B16_RPT = BM * B16_GROUPS / NTHREADS;   // (row, group) pairs per thread per slab = 4

struct B16Smem {
    __attribute__((aligned(16))) char a[2][BM * B16_ROWB];
    __attribute__((aligned(16))) char b[2][BM * B16_ROWB];
};

// Thread mapping: group slot gs = tid & 7, rows (tid >> 3) + 32 u, u = 0..3.
struct B16OpNDT {
    const unsigned short *p;
    int d, T, gpe;
    int q_end;            // groups q >= q_end read as zero
    // thread state
    int rowoff[B16_RPT];  // row * T (row clamped into the operand; d * T < 2^31 is checked on the host)
    unsigned rowmask;     // per u: row inside the operand
    int q, n, gi;
    __device__ void start(int tid, int i0, int q0) {
        q = q0 + (tid & 7);
        n = q / gpe;
        gi = q - n * gpe;
        rowmask = 0;
#pragma unroll
        for (int u = 0; u < B16_RPT; ++u) {
            const int row = i0 + (tid >> 3) + 32 * u;
            rowmask |= (row < d ? 1u : 0u) << u;
            rowoff[u] = min(row, d - 1) * T;
        }
    }
    // Issue the loads of this thread's groups; `m` receives the element masks that apply() puts on them.  Kept
    // apart so that nothing touches the loaded registers until the slab is moved to LDS, one step later.
    __device__ void fetch(uint4 (&v)[B16_RPT], unsigned (&m)[4]) const {
        const bool valid = q < q_end;
        const int t0 = min(8 * gi, T - 8);
        const int sh = valid ? 8 * gi - t0 : 8;   // positions below sh belong to the previous group (or nothing is valid)
        const unsigned short *base = p + (valid ? (int64_t)n * d * T + t0 : (int64_t)0);
#pragma unroll
        for (int w = 0; w < 4; ++w) m[w] = (2 * w >= sh ? 0x0000ffffu : 0u) | (2 * w + 1 >= sh ? 0xffff0000u : 0u);
#pragma unroll
        for (int u = 0; u < B16_RPT; ++u) __builtin_memcpy(&v[u], base + rowoff[u], 16);
    }
    __device__ void apply(uint4 (&v)[B16_RPT], const unsigned (&m)[4]) const {
#pragma unroll
        for (int u = 0; u < B16_RPT; ++u) {
            const unsigned keep = ((rowmask >> u) & 1u) ? 0xffffffffu : 0u;
            v[u].x &= m[0] & keep;
            v[u].y &= m[1] & keep;
            v[u].z &= m[2] & keep;
            v[u].w &= m[3] & keep;
        }
    }
    __device__ void next() {
        q += B16_GROUPS;
        gi += B16_GROUPS;
        while (gi >= gpe) { gi -= gpe; ++n; }
    }
    __device__ static void store(char *slab, const uint4 (&v)[B16_RPT], int tid) {
#pragma unroll
        for (int u = 0; u < B16_RPT; ++u)
            *reinterpret_cast<uint4 *>(slab + ((tid >> 3) + 32 * u) * B16_ROWB + (tid & 7) * 16) = v[u];
    }
};

__device__ inline float b16_sum8(const uint4 &x) {
    const unsigned w[4] = {x.x, x.y, x.z, x.w};
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) s += __uint_as_float(w[i] << 16) + __uint_as_float(w[i] & 0xffff0000u);
    return s;
}

// acc = A B^T over groups [q0, q_end) (both operands as elem(row, position)); DIAG: B is the same row block
// as A and is neither loaded nor staged.  With COLSUM every thread also accumulates, per u, the sum of the
// A-operand elements it fetches (csum[u]); summed over the eight threads that share a row this is the row's
// sum over all positions.
template <bool DIAG, bool COLSUM>
__device__ inline void gemm_tile_b16(B16OpNDT &A, B16OpNDT &B, int i0, int j0, int q0, int q_end, B16Smem &sm,
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
    const int nslab = (q_end - q0 + B16_GROUPS - 1) / B16_GROUPS;
    if (nslab <= 0) return;
    // Pipeline: slab s is multiplied out of LDS while slab s+1 waits in registers for its LDS buffer and the
    // loads of slab s+2 are in flight: at the bf16 MFMA rate one slab of arithmetic is much shorter than a trip
    // to L2, so a single slab of look-ahead leaves the matrix core idle most of the time.  Slabs past the end read
    // as zero (q >= q_end), so the look-ahead needs no special case.
    uint4 ra[2][B16_RPT], rb[2][B16_RPT];
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
        for (int u = 0; u < B16_RPT; ++u) csum[u] += b16_sum8(ra[0][u]);
    }
    B16OpNDT::store(sm.a[0], ra[0], tid);
    if (!DIAG) B16OpNDT::store(sm.b[0], rb[0], tid);
    __syncthreads();
    // one step: start the loads of slab s+2 into `f*` (free since slab s went to LDS), multiply slab s out of
    // LDS buffer s & 1, then move slab s+1, whose loads have had two steps to land, from `s*` to the other buffer
    auto step = [&](int s, int f, int o) {   // f = s & 1: register set to fetch into, o = 1 - f: set to move to LDS
        const int cur = s & 1;
        uint4 (&fa_)[B16_RPT] = ra[f], (&fb_)[B16_RPT] = rb[f], (&sa_)[B16_RPT] = ra[o], (&sb_)[B16_RPT] = rb[o];
        if (s + 2 < nslab) {
            A.next();
            A.fetch(fa_, ma[f]);
            if (!DIAG) {
                B.next();
                B.fetch(fb_, mb[f]);
            }
        }
        const char *pa = sm.a[cur];
        const char *pb = DIAG ? sm.a[cur] : sm.b[cur];
        // lane (c, g) of a 32x32x16 MFMA operand holds eight consecutive contraction indices of row (column) c:
        // group 2 ks + g of the slab in k-step ks (any assignment works as long as both operands share it)
        bf16x8 fa[4][2], fb[4][2];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                fa[ks][i] = *reinterpret_cast<const bf16x8 *>(pa + (wm + 32 * i + lc) * B16_ROWB + (2 * ks + lk) * 16);
                fb[ks][i] = *reinterpret_cast<const bf16x8 *>(pb + (wn + 32 * i + lc) * B16_ROWB + (2 * ks + lk) * 16);
            }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks][i], fb[ks][j], acc[i][j], 0, 0, 0);
        if (s + 1 < nslab) {
            A.apply(sa_, ma[o]);
            if (!DIAG) B.apply(sb_, mb[o]);
            if (COLSUM) {
#pragma unroll
                for (int u = 0; u < B16_RPT; ++u) csum[u] += b16_sum8(sa_[u]);
            }
            B16OpNDT::store(sm.a[cur ^ 1], sa_, tid);
            if (!DIAG) B16OpNDT::store(sm.b[cur ^ 1], sb_, tid);
        }
        __syncthreads();
    };
    for (int s = 0; s < nslab; s += 2) {
        step(s, 0, 1);           // slab s+1 sits in set 1; slab s+2 is fetched into set 0
        if (s + 1 < nslab) step(s + 1, 1, 0);
    }
}

}  // namespace kfac
