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
#include "kfac_internal.h"

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
//                        Raw    (the element type as it sits in memory)
//                        start(tid, i0, k0), fetch(Raw r[EPT]), value(r, s), next()
// fetch() only issues the loads of a slab (from a clamped address where the element is outside the operand) and notes
// which slots are inside; value() turns slot s of what was fetched into the operand element (zero outside, converted
// to fp32).  Nothing may touch the loaded registers between the two: the engine calls value() after the MFMAs of the
// slab before, so the loads stay in flight behind them.
// Thread mapping, KFAST : kk = tid & 15,  ii = (tid >> 4) + 16*s
//                 IFAST : ii = tid & 127, kk = (tid >> 7) + 2*s          (s = 0..7)

// Buffer loads: the address is a descriptor in scalar registers (base, extent) plus a 32-bit byte offset per lane, and
// the hardware returns zero for an offset outside the extent.  A load slot that is outside its operand is given
// such an offset, so a slab's loads need no address arithmetic, no comparison and no select in vector registers
// (in a probe of this engine's loop the vector instructions around the loads, not the loads, cost a fifth of the
// MFMA rate).
constexpr unsigned BUF_EXTENT = 0x7ffffff0u;   // bytes a descriptor covers from its base (offsets of real elements are far below)
constexpr unsigned BUF_OUTSIDE = 0x7ffffff8u;  // an offset the range check rejects: the load returns zero
__device__ inline __amdgpu_buffer_rsrc_t buffer_at(const void *base, unsigned extent = BUF_EXTENT) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, extent, 0x00020000);
}
__device__ inline void buffer_load(__amdgpu_buffer_rsrc_t rs, unsigned off, float &v) {
    v = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, off, 0, 0));
}
__device__ inline void buffer_load(__amdgpu_buffer_rsrc_t rs, unsigned off, unsigned short &v) {
    v = __builtin_amdgcn_raw_buffer_load_b16(rs, off, 0, 0);
}

// elem(i,k) = p[i*si + k*sk] for i < I, k < K, else 0  (ones_i is unused and kept at -1).
// Addressing: a base pointer that is uniform over the workgroup (it advances by a whole slab, so it lives in
// scalar registers) plus an unsigned 32-bit byte offset per load slot that never changes; the offset of a slot
// whose row is outside the operand is BUF_OUTSIDE.  The end of the contraction, k >= K: where k is the slow index
// in memory (IFAST; (i0 + i) si < sk is assumed, a row of the tile lies inside one leading dimension) the
// descriptor's extent ends with row K - 1, where k is the fast one the thread's one k per slab is compared with K.
// (127 si + 15 sk) * sizeof(E) must stay below 2^31: leading dimensions here are at most a few thousand.
// A contraction index may run over two separate memory ranges: set_segment(k, delta) moves the base by
// `delta` more elements when the slab starting at contraction index k is entered (k a multiple of BK).
template <typename E, bool KFAST_>
struct OpStrided {
    static constexpr bool KFAST = KFAST_;
    using Raw = E;
    const E *p;
    int64_t si, sk;
    int I, K, ones_i;
    int seg_k;
    int64_t seg_delta;
    // thread state
    const E *pb;          // tile base for the current slab (uniform)
    unsigned off[EPT];    // byte offsets of the slots relative to pb
    int k_t, k_slab;      // k of slot 0; first k of the current slab
    int64_t row0;         // i0 * si
    __device__ void set_segment(int k, int64_t delta) { seg_k = k; seg_delta = delta; }
    __device__ void start(int tid, int i0, int k0) {
        const int di = KFAST ? (tid >> 4) : (tid & 127);
        const int dk = KFAST ? (tid & 15) : (tid >> 7);
        row0 = (int64_t)i0 * si;
        pb = p + row0 + (int64_t)k0 * sk;
        k_t = k0 + dk;
        k_slab = k0;
#pragma unroll
        for (int s = 0; s < EPT; ++s) {
            const int i = KFAST ? di + 16 * s : di;
            const int k = KFAST ? dk : dk + 2 * s;
            off[s] = i0 + i < I ? (unsigned)(((int64_t)i * si + (int64_t)k * sk) * (int64_t)sizeof(E)) : BUF_OUTSIDE;
        }
    }
    __device__ void fetch(E (&r)[EPT]) const {
        if (KFAST) {
            const __amdgpu_buffer_rsrc_t rs = buffer_at(pb);
            const bool in = k_t < K;
#pragma unroll
            for (int s = 0; s < EPT; ++s) buffer_load(rs, in ? off[s] : BUF_OUTSIDE, r[s]);
        } else {
            const int64_t left = ((int64_t)(K - k_slab) * sk - row0) * (int64_t)sizeof(E);   // bytes from pb to the end of row K - 1
            const __amdgpu_buffer_rsrc_t rs = buffer_at(pb, (unsigned)min(max(left, (int64_t)0), (int64_t)BUF_EXTENT));
#pragma unroll
            for (int s = 0; s < EPT; ++s) buffer_load(rs, off[s], r[s]);
        }
    }
    __device__ float value(const E (&r)[EPT], int s) const { return to_float(r[s]); }
    __device__ void next() {
        k_t += BK;
        k_slab += BK;
        pb += (int64_t)BK * sk;
        if (seg_k != 0 && k_slab == seg_k) pb += seg_delta;
    }
};

// Samples in [N][d][T] layout with the contraction index k = n*T + t running over all sample rows:
// elem(i,k) = p[n*d*T + i*T + t], i < d; 1.0 on row ones_i; zero for k >= K (= end of this split).
template <typename E>
struct OpNDT {
    static constexpr bool KFAST = true;
    const E *p;
    int d, T, K, ones_i;
    // thread state
    int64_t base;       // n*d*T + t of this thread's k
    int ioff[EPT];      // i*T per slot (d*T < 2^31 is checked on the host)
    int k_t, t_t;
    unsigned in_mask, ones_mask;
    unsigned ok, one;   // per slot, for what was fetched last: inside the operand; on the ones row
    using Raw = E;
    __device__ void start(int tid, int i0, int k0) {
        const int i_t = i0 + (tid >> 4);
        k_t = k0 + (tid & 15);
        const int n_t = k_t / T;
        t_t = k_t - n_t * T;
        base = (int64_t)n_t * d * T + t_t;
        in_mask = ones_mask = 0;
#pragma unroll
        for (int s = 0; s < EPT; ++s) {
            const int i = i_t + 16 * s;
            ioff[s] = i * T;
            in_mask |= (i < d ? 1u : 0u) << s;
            ones_mask |= (i == ones_i ? 1u : 0u) << s;
        }
    }
    __device__ void fetch(E (&r)[EPT]) {
        const bool kv = k_t < K;
        ok = kv ? in_mask : 0u;
        one = kv ? ones_mask : 0u;
#pragma unroll
        for (int s = 0; s < EPT; ++s) r[s] = as_global(p)[((ok >> s) & 1u) ? base + ioff[s] : 0];
    }
    __device__ float value(const E (&r)[EPT], int s) const {
        return ((ok >> s) & 1u) ? to_float(r[s]) : (((one >> s) & 1u) ? 1.f : 0.f);
    }
    __device__ void next() {
        k_t += BK;
        t_t += BK;
        base += BK;
        while (t_t >= T) { t_t -= T; base += (int64_t)(d - 1) * T; }
    }
};

// The slab fetched last through `op`, as operand elements, into its place in LDS; with COLSUM, csum[s] += element s.
template <bool COLSUM, class Op>
__device__ inline void store_slab(float (*dst)[LDT], const Op &op, const typename Op::Raw (&r)[EPT], int tid, float *csum) {
#pragma unroll
    for (int s = 0; s < EPT; ++s) {
        const float v = op.value(r, s);
        if (COLSUM) csum[s] += v;
        if (Op::KFAST) dst[tid & 15][(tid >> 4) + 16 * s] = v;
        else           dst[(tid >> 7) + 2 * s][tid & 127] = v;
    }
}

struct TileSmem {
    float a[2][BK][LDT];
    float b[2][BK][LDT];
};

// How the four waves share a tile.  A wave's accumulator acc[i][j] covers rows wm+32i.., columns wn+32j.. of the
// tile and is computed only if bit 2i+j of `blocks` is set (the value is uniform over the wave).
struct WaveMap {
    int wm, wn;
    unsigned blocks;
};
// Every wave a 64x64 quadrant, all four accumulators: the whole 128x128 tile.
__device__ inline WaveMap wave_map_full() {
    const int wave = threadIdx.x >> 6;
    return WaveMap{(wave >> 1) * 64, (wave & 1) * 64, 0xFu};
}
// For a tile of which only the first mext rows and next columns are wanted (an edge tile of a ragged matrix):
// 32x32 accumulator blocks wholly outside are not computed, and a tile that is at most 64 wide (tall) is cut into
// four slices along the other side, so that all four waves - one per SIMD - share what is left.  An operand
// dimension of 128 m + 1 (a factor with its bias column) costs a quarter of a tile's time for the last column
// instead of a whole one.
__device__ inline WaveMap wave_map_edge(int mext, int next) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    WaveMap m;
    unsigned rows, cols;   // bit i: accumulator row block i wanted; bit j: column block j
    if (next <= 64 || mext <= 64) {
        const bool tall = next <= 64;                 // slices of 32 rows (tall) or of 32 columns
        m.wm = tall ? 32 * wave : 0;
        m.wn = tall ? 0 : 32 * wave;
        const int se = tall ? mext : next, oe = tall ? next : mext;   // extent along / across the slices
        const unsigned mine = 32 * wave < se ? 1u : 0u;
        const unsigned other = oe > 32 ? 3u : 1u;
        rows = tall ? mine : other;
        cols = tall ? other : mine;
    } else {
        m.wm = (wave >> 1) * 64;
        m.wn = (wave & 1) * 64;
        rows = (m.wm < mext ? 1u : 0u) | (m.wm + 32 < mext ? 2u : 0u);
        cols = (m.wn < next ? 1u : 0u) | (m.wn + 32 < next ? 2u : 0u);
    }
    m.blocks = 0;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
            if (((rows >> i) & 1u) && ((cols >> j) & 1u)) m.blocks |= 1u << (2 * i + j);
    return m;
}

// acc[i][j] accumulates rows wm+32i.., cols wn+32j.. of the tile; element r of a 32x32 accumulator
// sits at row 8*(r/4) + 4*(lane/32) + r%4, column lane%32.
// With COLSUM the thread also accumulates, per load slot, the sum over k of the A-operand elements it
// fetches (csum[s]); summed over the threads that share a row index this is sum_k elem_A(i, k).
template <class OpA, class OpB, bool COLSUM = false, bool EDGE = false>
__device__ inline void gemm_tile(OpA &A, OpB &B, int i0, int j0, int kbeg, int kend, TileSmem &sm,
                                 floatx16 (&acc)[2][2], float *csum = nullptr, bool zero_acc = true,
                                 const WaveMap map = wave_map_full()) {
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wm = map.wm, wn = map.wn;
    const unsigned blocks = map.blocks;   // EDGE: the accumulators to compute; else all four
    const int lk = lane >> 5, lc = lane & 31;
    if (zero_acc) {   // false: keep accumulating into acc (a contraction given in several segments)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    }
    const int nslab = (kend - kbeg + BK - 1) / BK;
    if (nslab <= 0) return;
    typename OpA::Raw ra[EPT];
    typename OpB::Raw rb[EPT];
    A.start(tid, i0, kbeg);
    B.start(tid, j0, kbeg);
    A.fetch(ra);
    B.fetch(rb);
    store_slab<COLSUM>(sm.a[0], A, ra, tid, csum);
    store_slab<false>(sm.b[0], B, rb, tid, nullptr);
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
        // all MFMA operands of the slab are read from LDS up front (32 registers), so the LDS latency is
        // paid once per slab instead of once per k-step and the 32 MFMAs issue back to back
        float a0[BK / 2], a1[BK / 2], b0[BK / 2], b1[BK / 2];
        if (!EDGE) {
#pragma unroll
            for (int j = 0; j < BK / 2; ++j) {
                a0[j] = sm.a[cur][2 * j + lk][wm + lc];
                a1[j] = sm.a[cur][2 * j + lk][wm + 32 + lc];
                b0[j] = sm.b[cur][2 * j + lk][wn + lc];
                b1[j] = sm.b[cur][2 * j + lk][wn + 32 + lc];
            }
            __builtin_amdgcn_sched_barrier(0);   // keep the reads above ahead of the MFMAs below
#pragma unroll
            for (int j = 0; j < BK / 2; ++j) {
                acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[j], b0[j], acc[0][0], 0, 0, 0);
                acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[j], b1[j], acc[0][1], 0, 0, 0);
                acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[j], b0[j], acc[1][0], 0, 0, 0);
                acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[j], b1[j], acc[1][1], 0, 0, 0);
            }
        } else if (blocks != 0u) {   // only the wanted blocks (the operands of a second block may lie outside the slab)
#pragma unroll
            for (int j = 0; j < BK / 2; ++j) {
                a0[j] = sm.a[cur][2 * j + lk][wm + lc];
                b0[j] = sm.b[cur][2 * j + lk][wn + lc];
            }
            if (blocks & 0xCu) {
#pragma unroll
                for (int j = 0; j < BK / 2; ++j) a1[j] = sm.a[cur][2 * j + lk][wm + 32 + lc];
            }
            if (blocks & 0xAu) {
#pragma unroll
                for (int j = 0; j < BK / 2; ++j) b1[j] = sm.b[cur][2 * j + lk][wn + 32 + lc];
            }
            __builtin_amdgcn_sched_barrier(0);
            if (blocks & 1u) {
#pragma unroll
                for (int j = 0; j < BK / 2; ++j) acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[j], b0[j], acc[0][0], 0, 0, 0);
            }
            if (blocks & 2u) {
#pragma unroll
                for (int j = 0; j < BK / 2; ++j) acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[j], b1[j], acc[0][1], 0, 0, 0);
            }
            if (blocks & 4u) {
#pragma unroll
                for (int j = 0; j < BK / 2; ++j) acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[j], b0[j], acc[1][0], 0, 0, 0);
            }
            if (blocks & 8u) {
#pragma unroll
                for (int j = 0; j < BK / 2; ++j) acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[j], b1[j], acc[1][1], 0, 0, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);   // nothing that reads the fetched registers moves up in front of the MFMAs
        if (more) {
            store_slab<COLSUM>(sm.a[cur ^ 1], A, ra, tid, csum);
            store_slab<false>(sm.b[cur ^ 1], B, rb, tid, nullptr);
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

// The same for a tile computed under `map`: only the accumulators that were computed are visited.
template <class F>
__device__ inline void for_each_acc(const floatx16 (&acc)[2][2], const WaveMap map, F f) {
    const int lane = threadIdx.x & 63;
    const int lk = lane >> 5, lc = lane & 31;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            if (!((map.blocks >> (2 * i + j)) & 1u)) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                f(map.wm + 32 * i + 8 * (r >> 2) + 4 * lk + (r & 3), map.wn + 32 * j + lc, acc[i][j][r]);
        }
}

// Fill every accumulator element of this thread: acc(row, col) = f(row_in_tile, col_in_tile).
template <class F>
__device__ inline void fill_acc(floatx16 (&acc)[2][2], F f) {
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
                acc[i][j][r] = f(wm + 32 * i + 8 * (r >> 2) + 4 * lk + (r & 3), wn + 32 * j + lc);
}

// dst[c * ld + r] = acc(r, c) for the whole tile: the transposed tile, written with coalesced rows.  Every
// wave turns its 32x32 accumulator blocks round in a private 32 x 33 patch of LDS (scratch: 4 * 32 * 33
// floats, free once the K loop is over).  All threads of the workgroup must call it.
__device__ inline void store_acc_transposed(const floatx16 (&acc)[2][2], float *scratch, float *dst, int64_t ld) {
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int lk = lane >> 5, lc = lane & 31;
    float *patch = scratch + wave * (32 * 33);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            __syncthreads();
#pragma unroll
            for (int r = 0; r < 16; ++r) patch[lc * 33 + 8 * (r >> 2) + 4 * lk + (r & 3)] = acc[i][j][r];   // patch[col][row]
            __syncthreads();
            float *d = dst + (int64_t)(wn + 32 * j) * ld + wm + 32 * i;
#pragma unroll
            for (int t = 0; t < 16; ++t) {
                const int c = lk + 2 * t;
                d[(int64_t)c * ld + lc] = patch[c * 33 + lc];
            }
        }
}

// f(c, r, acc(r, c)) for the whole tile, i.e. the transposed tile, visited so that a wave's lanes run along its rows
// (coalesced if f stores).  Same LDS patches as store_acc_transposed; all threads of the workgroup must call it.
template <class F>
__device__ inline void for_each_acc_transposed(const floatx16 (&acc)[2][2], float *scratch, F f) {
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int lk = lane >> 5, lc = lane & 31;
    float *patch = scratch + wave * (32 * 33);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            __syncthreads();
#pragma unroll
            for (int r = 0; r < 16; ++r) patch[lc * 33 + 8 * (r >> 2) + 4 * lk + (r & 3)] = acc[i][j][r];   // patch[col][row]
            __syncthreads();
#pragma unroll
            for (int t = 0; t < 16; ++t) {
                const int c = lk + 2 * t;
                f(wn + 32 * j + c, wm + 32 * i + lc, patch[c * 33 + lc]);
            }
        }
}

// One tile of an M x N product with ragged edges: epi(row, col, value) for every element of the tile inside the
// matrix.  A full tile runs under the full map; at an edge the waves share the blocks that hold something.
template <class OpA, class OpB, class Epi>
__device__ inline void gemm_tile_ragged(OpA &a, OpB &b, int i0, int j0, int K, int M, int N, TileSmem &sm, Epi epi) {
    floatx16 acc[2][2];
    const int mext = min(BM, M - i0), next = min(BM, N - j0);
    if (mext == BM && next == BM) {
        gemm_tile(a, b, i0, j0, 0, K, sm, acc);
        for_each_acc(acc, [&](int r, int c, float v) { epi(i0 + r, j0 + c, v); });
    } else {
        const WaveMap map = wave_map_edge(mext, next);
        gemm_tile<OpA, OpB, false, true>(a, b, i0, j0, 0, K, sm, acc, nullptr, true, map);
        for_each_acc(acc, map, [&](int r, int c, float v) {
            const int gr = i0 + r, gc = j0 + c;
            if (gr < M && gc < N) epi(gr, gc, v);
        });
    }
}

// Epilogue objects are called as epi(row, col, value) for every in-range element of a tile.
struct EpiStore {
    float *C;
    int64_t ld;
    __device__ void operator()(int r, int c, float v) const { C[(int64_t)r * ld + c] = v; }
};

}  // namespace kfac
