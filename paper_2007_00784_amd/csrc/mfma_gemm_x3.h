// Split-fp16 MFMA tile engine for gfx950: the same 128x128 workgroup tile as the fp32 engine, but every
// fp32 operand element x is written to LDS as two halves, hi = fp16(x) and lo = fp16(x - hi), and the
// product is accumulated in fp32 as  lo*hi + hi*lo + hi*hi  with v_mfma_f32_32x32x16_f16 (three MFMAs that
// each run at 16 times the fp32 MFMA rate).  hi + lo carries 22 significand bits, so a product is good to
// about 2^-21 relative as long as hi stays in fp16's normal range; callers therefore scale their operands
// by powers of two (exact) so that magnitudes that matter sit well inside [2^-14, 2^15], and undo the
// scaling on the accumulator.  What falls below the normal range is kept to an absolute 2^-25 of the
// scaled unit, i.e. the engine is accurate normwise, not elementwise.
//
// For a near-identity transform V a caller does best to compute X (V - I) here and to add X itself in
// fp32: the split engine's error then scales with |V - I|.
//
// Two loaders: X3Op for whole, aligned tiles (the eigensolver's outer passes meet its restrictions by
// construction: full 128-row operand tiles, K a multiple of 16, 16-byte aligned k-contiguous operands) and
// X3OpG for operands of any extent and alignment (the preconditioner's GEMM chain).
#pragma once
#include "mfma_gemm.h"

namespace kfac {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

constexpr int X3_ROWB = 80;   // LDS bytes per operand row and slab: hi[16], lo[16] halves, 16 B pad
                              // (80 B = 20 banks: sixteen 16-byte accesses at this pitch hit distinct banks)

struct X3Smem {
    __attribute__((aligned(16))) char a[2][BM * X3_ROWB];
    __attribute__((aligned(16))) char b[2][BM * X3_ROWB];
};

// elem(i,k) = p[i*ld + k] (KFAST) or p[k*ld + i]; i in [0,128), k in [0,K).  Each thread owns one row i and
// eight consecutive k of every slab.  set_segment(k, delta): as for the fp32 loaders.
template <bool KFAST_>
struct X3Op {
    static constexpr bool KFAST = KFAST_;
    static constexpr bool HAS_BULK = false;   // its one fetch is already free of checks
    __device__ void fetch_bulk(float (&r)[8]) const { fetch(r); }
    const float *p;
    int64_t ld;
    float scale;          // power of two applied before the split
    int seg_k;
    int64_t seg_delta;
    // thread state
    const float *pb;      // uniform over the workgroup: the loads are buffer loads (scalar base, fixed offset per lane)
    unsigned off;         // byte offset of this thread's first element of a slab
    int k_slab, row, kg;
    __device__ void set_segment(int k, int64_t delta) { seg_k = k; seg_delta = delta; }
    __device__ void start(int tid) {
        row = KFAST ? tid >> 1 : tid & 127;
        kg = KFAST ? tid & 1 : tid >> 7;
        pb = p;
        k_slab = 0;
        off = 4u * (KFAST ? (unsigned)(row * ld + 8 * kg) : (unsigned)(8 * kg * ld + row));
    }
    __device__ void fetch(float (&r)[8]) const {
        const __amdgpu_buffer_rsrc_t rs = buffer_at(pb);
        if (KFAST) {
            typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
            const uintx4 x = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0);
            const uintx4 y = __builtin_amdgcn_raw_buffer_load_b128(rs, off + 16, 0, 0);
            r[0] = __uint_as_float(x.x); r[1] = __uint_as_float(x.y); r[2] = __uint_as_float(x.z); r[3] = __uint_as_float(x.w);
            r[4] = __uint_as_float(y.x); r[5] = __uint_as_float(y.y); r[6] = __uint_as_float(y.z); r[7] = __uint_as_float(y.w);
        } else {
#pragma unroll
            for (int s = 0; s < 8; ++s) buffer_load(rs, off + 4u * (unsigned)(s * ld), r[s]);
        }
    }
    __device__ void next() {
        k_slab += BK;
        pb += KFAST ? (int64_t)BK : (int64_t)BK * ld;
        if (seg_k != 0 && k_slab == seg_k) pb += seg_delta;
    }
    // split the eight fetched values and write them to this thread's place in an LDS slab
    __device__ void store(char *slab, const float (&r)[8]) const {
        half8 hi, lo;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            // two mixed-precision FMAs per element: hi = rne(r * scale), lo = rne(r * scale - hi).  The scaling by a
            // power of two and the difference are exact, so these are the values of the plain expressions.
            const _Float16 h = (_Float16)__builtin_fmaf(r[s], scale, 0.f);
            hi[s] = h;
            lo[s] = (_Float16)__builtin_fmaf(r[s], scale, -(float)h);
        }
        *reinterpret_cast<half8 *>(slab + row * X3_ROWB + kg * 16) = hi;
        *reinterpret_cast<half8 *>(slab + row * X3_ROWB + 32 + kg * 16) = lo;
    }
};

// General operand for the same engine: any extent and alignment, fp32 or bf16 elements.  elem(i,k) = p[i*ld + k]
// (KFAST) or p[k*ld + i], zero for i >= I or k >= K (i counted from the operand's first row; the tile's first row
// i0 is given to start()).  Two ways to fetch a slab.  fetch_bulk(), for slabs that lie wholly below K: buffer loads
// from a base in scalar registers that moves with the slab, at a byte offset per thread that never changes (a row
// outside the operand has an offset the range check rejects, and reads zeros) -- no comparison, no select and no
// address arithmetic in vector registers, which is what bound the products of this engine before (some 230 vector
// instructions a slab beside its 12 MFMAs).  fetch(), for the ragged last slab: element by element, every index
// checked.
template <typename E, bool KFAST_>
struct X3OpG {
    static constexpr bool KFAST = KFAST_;
    static constexpr bool HAS_BULK = true;
    const E *p;
    int64_t ld;
    float scale;
    int I, K;
    // thread state
    global_ptr<const E> pb;   // KFAST: first element of this thread's row; else p + this thread's i
    const E *ub;              // bulk: element (i0, first k of the current slab), uniform over the workgroup
    unsigned boff;            // bulk: byte offset of this thread's first element from ub
    int row, kg, k;    // k: first of this thread's eight contraction indices in the current slab
    bool row_ok;
    __device__ void start(int tid, int i0) {
        row = KFAST ? tid >> 1 : tid & 127;
        kg = KFAST ? tid & 1 : tid >> 7;
        k = 8 * kg;
        row_ok = i0 + row < I;
        const int i = row_ok ? i0 + row : 0;
        pb = KFAST ? as_global(p) + (int64_t)i * ld : as_global(p) + i;
        ub = KFAST ? p + (int64_t)i0 * ld : p + i0;
        const int64_t e = KFAST ? (int64_t)row * ld + 8 * kg : (int64_t)8 * kg * ld + row;
        boff = row_ok ? (unsigned)(e * (int64_t)sizeof(E)) : BUF_OUTSIDE;
    }
    __device__ void fetch_bulk(float (&r)[8]) const {
        typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
        const __amdgpu_buffer_rsrc_t rs = buffer_at(ub);
        if (KFAST) {
            if (sizeof(E) == 4) {
                const uintx4 x = __builtin_amdgcn_raw_buffer_load_b128(rs, boff, 0, 0);
                const uintx4 y = __builtin_amdgcn_raw_buffer_load_b128(rs, boff + 16, 0, 0);
                r[0] = __uint_as_float(x.x); r[1] = __uint_as_float(x.y); r[2] = __uint_as_float(x.z); r[3] = __uint_as_float(x.w);
                r[4] = __uint_as_float(y.x); r[5] = __uint_as_float(y.y); r[6] = __uint_as_float(y.z); r[7] = __uint_as_float(y.w);
            } else {
                const uintx4 x = __builtin_amdgcn_raw_buffer_load_b128(rs, boff, 0, 0);
                const unsigned w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
                for (int t = 0; t < 4; ++t) { r[2 * t] = __uint_as_float(w[t] << 16); r[2 * t + 1] = __uint_as_float(w[t] & 0xffff0000u); }
            }
        } else {
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                E v;
                buffer_load(rs, boff + (unsigned)(s * ld) * (unsigned)sizeof(E), v);
                r[s] = to_float(v);
            }
        }
    }
    __device__ void fetch(float (&r)[8]) const {
        if (KFAST) {
            if (row_ok && k + 8 <= K) {
                if (sizeof(E) == 4) {
                    uint4 x, y;
                    __builtin_memcpy(&x, pb + k, 16);
                    __builtin_memcpy(&y, pb + k + 4, 16);
                    r[0] = __uint_as_float(x.x); r[1] = __uint_as_float(x.y); r[2] = __uint_as_float(x.z); r[3] = __uint_as_float(x.w);
                    r[4] = __uint_as_float(y.x); r[5] = __uint_as_float(y.y); r[6] = __uint_as_float(y.z); r[7] = __uint_as_float(y.w);
                } else {
                    uint4 x;
                    __builtin_memcpy(&x, pb + k, 16);
                    const unsigned w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
                    for (int t = 0; t < 4; ++t) { r[2 * t] = __uint_as_float(w[t] << 16); r[2 * t + 1] = __uint_as_float(w[t] & 0xffff0000u); }
                }
            } else {
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    const bool ok = row_ok && k + s < K;
                    const float v = to_float(pb[ok ? k + s : 0]);
                    r[s] = ok ? v : 0.f;
                }
            }
        } else {
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const bool ok = row_ok && k + s < K;
                const float v = to_float(pb[ok ? (int64_t)(k + s) * ld : (int64_t)0]);
                r[s] = ok ? v : 0.f;
            }
        }
    }
    __device__ void next() {
        k += BK;
        ub += KFAST ? (int64_t)BK : (int64_t)BK * ld;
    }
    __device__ void store(char *slab, const float (&r)[8]) const {
        half8 hi, lo;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const _Float16 h = (_Float16)__builtin_fmaf(r[s], scale, 0.f);   // as in X3Op::store
            hi[s] = h;
            lo[s] = (_Float16)__builtin_fmaf(r[s], scale, -(float)h);
        }
        *reinterpret_cast<half8 *>(slab + row * X3_ROWB + kg * 16) = hi;
        *reinterpret_cast<half8 *>(slab + row * X3_ROWB + 32 + kg * 16) = lo;
    }
};

// `nslab` slabs of the product, from the loaders' current position (with ADVANCE they first move on one slab);
// BULK: the slabs lie wholly inside the contraction and are fetched with fetch_bulk().  Ends with a barrier, so
// the slab buffers are free again.
template <bool BULK, class OpA, class OpB>
__device__ inline void x3_slabs(OpA &A, OpB &B, int nslab, bool advance, X3Smem &sm, floatx16 (&acc)[2][2]) {
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int lk = lane >> 5, lc = lane & 31;
    float ra[8], rb[8];
    if (advance) {
        A.next();
        B.next();
    }
    if (BULK) { A.fetch_bulk(ra); B.fetch_bulk(rb); } else { A.fetch(ra); B.fetch(rb); }
    A.store(sm.a[0], ra);
    B.store(sm.b[0], rb);
    __syncthreads();
    for (int s = 0; s < nslab; ++s) {
        const int cur = s & 1;
        const bool more = s + 1 < nslab;
        if (more) {
            A.next();
            B.next();
            if (BULK) { A.fetch_bulk(ra); B.fetch_bulk(rb); } else { A.fetch(ra); B.fetch(rb); }
        }
        // lane (c, g) of a 32x32x16 MFMA operand holds k = 8g .. 8g+7 of row (column) c
        half8 ah[2], al[2], bh[2], bl[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            ah[i] = *reinterpret_cast<const half8 *>(sm.a[cur] + (wm + 32 * i + lc) * X3_ROWB + lk * 16);
            al[i] = *reinterpret_cast<const half8 *>(sm.a[cur] + (wm + 32 * i + lc) * X3_ROWB + 32 + lk * 16);
            bh[i] = *reinterpret_cast<const half8 *>(sm.b[cur] + (wn + 32 * i + lc) * X3_ROWB + lk * 16);
            bl[i] = *reinterpret_cast<const half8 *>(sm.b[cur] + (wn + 32 * i + lc) * X3_ROWB + 32 + lk * 16);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al[i], bh[j], acc[i][j], 0, 0, 0);
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah[i], bl[j], acc[i][j], 0, 0, 0);
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah[i], bh[j], acc[i][j], 0, 0, 0);
            }
        __builtin_amdgcn_sched_barrier(0);
        if (more) {
            A.store(sm.a[cur ^ 1], ra);
            B.store(sm.b[cur ^ 1], rb);
        }
        __syncthreads();
    }
}

// acc = (scaleA A) (scaleB B)^T-style product over K (operands as elem(i,k)); same accumulator layout as
// gemm_tile, so for_each_acc applies.  Loaders that have a bulk fetch run the whole slabs of the contraction on it
// and the ragged last slab, if there is one, on the checked fetch, as a second short pipeline.
// The caller has already called start() on both loaders.
template <class OpA, class OpB>
__device__ inline void gemm_tile_x3(OpA &A, OpB &B, int K, X3Smem &sm, floatx16 (&acc)[2][2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    const int nslab = (K + BK - 1) / BK;   // loaders without an extent of their own are given whole slabs
    if (nslab <= 0) return;
    constexpr bool TWO = OpA::HAS_BULK && OpB::HAS_BULK;
    const int nbulk = TWO ? K / BK : 0;
    if (TWO && nbulk > 0) x3_slabs<true>(A, B, nbulk, false, sm, acc);
    if (nslab > nbulk) x3_slabs<false>(A, B, nslab - nbulk, nbulk > 0, sm, acc);
}

}  // namespace kfac
