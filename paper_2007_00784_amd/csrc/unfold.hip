// Unfold (im2col) of a conv input into per-example patch slabs [N][C*kh*kw][Ho*Wo].
// Pure data movement, HBM-bound: each workgroup stages the input rows of a group of channels it
// needs once in LDS (zero padding materialised there), then writes the kh*kw shifted copies.  For a
// fixed example and channel the kh*kw patch rows are adjacent in the output, so a workgroup's
// output is one contiguous run (full-height chunks) or kh*kw runs of whole output rows, and both
// the global reads (along W) and the global writes (along Ho*Wo) are coalesced.
#include <algorithm>
#include <vector>
#include "kfac_internal.h"

namespace {

constexpr int UNFOLD_LDS_BYTES = 16384; // staged input per workgroup.  With the offset table that is 20 KB of LDS: seven
                                        // workgroups per compute unit.  The phases of a workgroup (load, barrier, write) do not
                                        // overlap, so occupancy is what hides them: 32 KB tiles (three workgroups per compute
                                        // unit) measured 0.50 ms for the ResNet-50 set, these 0.47 ms
constexpr int UNFOLD_TILE_SLACK = 8;    // elements past the tile that a 16-byte read at its very end may touch
constexpr int UNFOLD_MAX_PROWS = 2048;  // patch rows (channels of the workgroup x kh x kw) whose LDS offsets are tabulated

struct UnfoldArgs {
    int N, C, H, W, kh, kw, sh, sw, ph, pw, Ho, Wo;
    int cpb;       // channels per workgroup
    int rows_out;  // output rows per workgroup
    int rows_in;   // staged input rows = (rows_out-1)*sh + kh
    int Wp;        // staged row width = W + 2*pw
    int deint;     // 1 (column stride 2): even and odd staged columns are kept in separate half planes, so that the
                   // columns one patch row needs (2*wo + kx: one parity) are contiguous in LDS
    int Wq;        // LDS row pitch: Wp, or ceil(Wp / 2) when deinterleaved
    int plane;     // LDS elements per staged channel: rows_in * Wp, or 2 * rows_in * Wq
    int compact;   // 1 (1 x 1 kernel): only the pixels the windows touch are staged, as [rows_out][Wo] per channel, so the
                   // output slab of a channel is one contiguous copy of its staged plane (Wq = Wo, plane = rows_out * Wo)
    float inv_Wp, inv_rows_in, inv_Tc, inv_Wo, inv_kw, inv_kh;
};

// q = e / d, r = e % d for 0 <= e < 2^24 using a float reciprocal and one correction step each way.
__device__ inline void fdivmod(int e, int d, float inv_d, int &q, int &r) {
    q = (int)((float)e * inv_d);
    r = e - q * d;
    if (r < 0) { --q; r += d; }
    if (r >= d) { ++q; r -= d; }
}

template <typename E>
__device__ inline void unfold_block(const E *__restrict__ x_, E *__restrict__ out_, const UnfoldArgs &a, int bx, int by, int bz, E *tile,
                                    unsigned short *rowoff) {
    // global loads and stores, not flat ones (the batched kernel reads its pointers from a table): a flat access
    // counts on the LDS counter too, and every wait for an LDS read of the write phase would wait for the stores
    typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
    const global_ptr<const E> x = as_global(x_);
    const global_ptr<E> out = as_global(out_);
    const int n = bz;
    const int c0 = by * a.cpb;
    const int ho0 = bx * a.rows_out;
    const int nch = min(a.cpb, a.C - c0);
    const int rows_out = min(a.rows_out, a.Ho - ho0);
    const int rows_in = (rows_out - 1) * a.sh + a.kh;
    const int h_first = ho0 * a.sh - a.ph;
    const int plane = a.plane;             // LDS pitch per channel
    const int hplane = a.rows_in * a.Wq;   // deinterleaved: pitch between the even and the odd half plane
    // ---- stage: tile[cc][hr][wc] = x[n][c0+cc][h_first+hr][wc-pw] or 0 ----
    // Eight elements per thread at a time: all eight addresses first, then the eight loads back to back, then the LDS
    // stores -- so a thread waits for memory once per batch, not once per element.  (1 x 1 kernels: tile[cc][hoo][wo] =
    // x[n][c0+cc][(ho0+hoo)*sh-ph][wo*sw-pw], only the pixels a window touches.)
    const int srows = a.compact ? rows_out : rows_in, scols = a.compact ? a.Wo : a.Wp;   // staged rows and columns per channel
    const int stage_n = nch * srows * scols;
    const float inv_rows = 1.0f / (float)srows, inv_cols = a.compact ? a.inv_Wo : a.inv_Wp;
    constexpr int SBATCH = 8;
    for (int base = threadIdx.x; base < stage_n; base += 256 * SBATCH) {
        E v[SBATCH];
        int dst[SBATCH];
        global_ptr<const E> src[SBATCH];
#pragma unroll
        for (int u = 0; u < SBATCH; ++u) {
            const int e = min(base + 256 * u, stage_n - 1);
            int row, wc, cc, hr;
            fdivmod(e, scols, inv_cols, row, wc);
            fdivmod(row, srows, inv_rows, cc, hr);
            const int h = a.compact ? (ho0 + hr) * a.sh - a.ph : h_first + hr, w = a.compact ? wc * a.sw - a.pw : wc - a.pw;
            const bool in = h >= 0 && h < a.H && w >= 0 && w < a.W;
            src[u] = in ? x + ((((int64_t)n * a.C + c0 + cc) * a.H + h) * a.W + w) : nullptr;
            dst[u] = a.deint ? cc * plane + (wc & 1) * hplane + hr * a.Wq + (wc >> 1) : cc * plane + hr * a.Wq + wc;
            if (base + 256 * u >= stage_n) dst[u] = -1;
        }
#pragma unroll
        for (int u = 0; u < SBATCH; ++u) v[u] = src[u] ? *src[u] : (E)0;
#pragma unroll
        for (int u = 0; u < SBATCH; ++u)
            if (dst[u] >= 0) tile[dst[u]] = v[u];
    }
    // ---- write ----
    // For (cc, ky, kx) the outputs of this workgroup are the run of Tc = rows_out*Wo positions starting at
    // (ho0, 0).  With full-height chunks (Tc == T) the runs of consecutive patch rows are adjacent, so the whole
    // workgroup writes ONE contiguous run; otherwise one run per patch row.  A run is cut into 16-byte vectors
    // aligned in global memory (the first and last may be partial and are stored element by element).
    // The kernel is bound by its index arithmetic, not by memory, so a vector costs two divisions (position in the
    // run -> patch row and output position -> output row and column) and one look-up of the patch row's LDS offset
    // (tabulated once per workgroup).  Where consecutive output columns are consecutive in LDS (column stride 1, or 2
    // with the parity-split staging) a vector inside one output row is one 16-byte LDS read, and one that runs over
    // the end of a row into the next is two such reads merged; anything else goes element by element with carries.
    constexpr int VEC = 16 / (int)sizeof(E);
    const int Tc = rows_out * a.Wo;
    const int T = a.Ho * a.Wo;
    const int khw = a.kh * a.kw;
    const bool one_run = Tc == T;
    const int nrun = one_run ? 1 : nch * khw;
    const int L = one_run ? nch * khw * T : Tc;
    const float inv_Tc = 1.0f / (float)Tc;
    const float inv_khw = 1.0f / (float)khw;
    for (int pr = threadIdx.x; pr <= nch * khw; pr += 256) {      // one entry past the end: read, never used
        int cc, kk, ky, kx;
        fdivmod(pr, khw, inv_khw, cc, kk);
        fdivmod(kk, a.kw, a.inv_kw, ky, kx);
        const int o = a.deint ? cc * plane + (kx & 1) * hplane + ky * a.Wq + (kx >> 1) : cc * plane + ky * a.Wq + kx;
        rowoff[pr] = (unsigned short)(pr < nch * khw ? o : 0);
    }
    __syncthreads();
    const int es = (a.deint || a.compact) ? 1 : a.sw;  // LDS step between consecutive output columns
    const int rp = a.compact ? a.Wq : a.sh * a.Wq;     // ... and between consecutive output rows
    const int row_step = rp - a.Wo * es;               // from the end of an output row to the start of the next
    const global_ptr<E> out0 = out + ((int64_t)n * a.C + c0) * khw * T + (int64_t)ho0 * a.Wo;   // run 0, element 0
    for (int run = 0; run < nrun; ++run) {
        const global_ptr<E> dst = out0 + (int64_t)run * T;
        const int g0 = (int)(((uintptr_t)dst / sizeof(E)) % VEC);   // elements past a 16-byte boundary
        const int nvec = (L + g0 + VEC - 1) / VEC;
        for (int v = threadIdx.x; v < nvec; v += 256) {
            const int j0 = v * VEC - g0;             // first element of the vector inside the run (may be < 0)
            const int jb = max(j0, 0), je = min(j0 + VEC, L);
            int prow, t, hoo, wo;
            if (one_run) fdivmod(jb, Tc, inv_Tc, prow, t);
            else { prow = run; t = jb; }
            fdivmod(t, a.Wo, a.inv_Wo, hoo, wo);
            int off = rowoff[prow] + hoo * rp + wo * es;     // LDS index of the vector's first element
            const bool whole = jb == j0 && je == j0 + VEC;
            if (whole && es == 1) {
                const int c1 = a.Wo - wo;                     // elements left in this output row
                if (c1 >= VEC) {
                    uintx4 q;
                    __builtin_memcpy(&q, tile + off, 16);     // element aligned only: an unaligned LDS read
                    *(global_ptr<uintx4>)(dst + j0) = q;
                    continue;
                }
                // the rest of the vector comes from the start of the next output row (or of the next patch row)
                const int off2 = (hoo + 1 == rows_out) ? rowoff[prow + 1] : off - wo + rp;
                if (c1 + a.Wo >= VEC && off2 >= c1) {
                    E va[VEC], vb[VEC];
                    __builtin_memcpy(va, tile + off, 16);
                    __builtin_memcpy(vb, tile + (off2 - c1), 16);
#pragma unroll
                    for (int i = 0; i < VEC; ++i) va[i] = i < c1 ? va[i] : vb[i];
                    uintx4 q;
                    __builtin_memcpy(&q, va, 16);
                    *(global_ptr<uintx4>)(dst + j0) = q;
                    continue;
                }
            }
            E vals[VEC];
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                const int j = j0 + i;
                E xv = 0;
                if (j >= jb && j < je) {
                    xv = tile[off];
                    off += es;
                    if (++wo == a.Wo) {
                        wo = 0;
                        off += row_step;
                        if (++hoo == rows_out) {     // only reached inside the single run: next patch row
                            hoo = 0;
                            off = rowoff[++prow];
                        }
                    }
                }
                vals[i] = xv;
            }
            if (whole) {
                uintx4 q;
                __builtin_memcpy(&q, vals, 16);
                *(global_ptr<uintx4>)(dst + j0) = q;
            } else {
#pragma unroll
                for (int i = 0; i < VEC; ++i)
                    if (j0 + i >= jb && j0 + i < je) dst[j0 + i] = vals[i];
            }
        }
    }
}

template <typename E>
__global__ __launch_bounds__(256) void unfold_kernel(const E *__restrict__ x, E *__restrict__ out, UnfoldArgs a) {
    __shared__ __align__(16) E tile[UNFOLD_LDS_BYTES / sizeof(E) + UNFOLD_TILE_SLACK];
    __shared__ unsigned short rowoff[UNFOLD_MAX_PROWS + 2];
    unfold_block<E>(x, out, a, blockIdx.x, blockIdx.y, blockIdx.z, tile, rowoff);
}

// Several layers in one launch: workgroup b belongs to the layer l with first[l] <= b < first[l+1] and is
// workgroup (bx, by, bz) of that layer's own grid (gx, gy, gz), bx fastest.
struct UnfoldItem {
    const void *x;
    void *out;
    UnfoldArgs a;
    int gx, gy;
    int first;     // index of the layer's first workgroup in the launch
};
template <typename E>
__global__ __launch_bounds__(256) void unfold_batched_kernel(const UnfoldItem *items, int n) {
    __shared__ __align__(16) E tile[UNFOLD_LDS_BYTES / sizeof(E) + UNFOLD_TILE_SLACK];
    __shared__ unsigned short rowoff[UNFOLD_MAX_PROWS + 2];
    const int b = blockIdx.x;
    // last layer whose first workgroup is <= b: the first wave counts, 64 layers per step with one load each, the
    // layers that start at or before b (their firsts ascend)
    __shared__ int layer_of;
    if (threadIdx.x < 64) {
        int cnt = 0;
        for (int base = 0; base < n; base += 64) {
            const int l = base + (int)threadIdx.x;
            const bool le = l < n && items[l].first <= b;
            cnt += __popcll(__ballot(le));
        }
        if (threadIdx.x == 0) layer_of = cnt - 1;
    }
    __syncthreads();
    const int lo = layer_of;
    const UnfoldItem &it = items[lo];
    const int r = b - it.first;
    const int bx = r % it.gx, t = r / it.gx;
    unfold_block<E>((const E *)it.x, (E *)it.out, it.a, bx, t % it.gy, t / it.gy, tile, rowoff);
}

}  // namespace

namespace {
// Tiling of one layer: fills `a` and the grid; false when the shape does not fit the kernel's limits.
bool plan_unfold(const kfac_conv_desc *d, UnfoldArgs &a, dim3 &grid, bool batched = false) {
    a.N = d->N; a.C = d->C; a.H = d->H; a.W = d->W; a.kh = d->kh; a.kw = d->kw;
    a.sh = d->stride_h; a.sw = d->stride_w; a.ph = d->pad_h; a.pw = d->pad_w;
    a.Ho = (d->H + 2 * d->pad_h - d->kh) / d->stride_h + 1;
    a.Wo = (d->W + 2 * d->pad_w - d->kw) / d->stride_w + 1;
    a.Wp = d->W + 2 * d->pad_w;
    a.compact = (a.kh == 1 && a.kw == 1) ? 1 : 0;
    a.deint = (!a.compact && a.sw == 2) ? 1 : 0;
    a.Wq = a.compact ? a.Wo : (a.deint ? (a.Wp + 1) / 2 : a.Wp);
    const int row_elems = a.deint ? 2 * a.Wq : a.Wq;             // LDS elements per staged row
    const int UNFOLD_LDS_ELEMS = UNFOLD_LDS_BYTES / (d->dtype == KFAC_F32 ? 4 : 2);
    const int rows_in_full = a.compact ? a.Ho : (a.Ho - 1) * a.sh + a.kh;   // staged rows of a full-height chunk
    if ((int64_t)d->kh * row_elems > UNFOLD_LDS_ELEMS) return false;  // one output row must fit
    if ((int64_t)rows_in_full * row_elems <= UNFOLD_LDS_ELEMS) {
        a.rows_out = a.Ho;
        int cpb = UNFOLD_LDS_ELEMS / (rows_in_full * row_elems);
        // a layer launched alone keeps its grid large enough to fill 256 CUs several times over; in a batch the other
        // layers fill the machine and fatter workgroups amortise their fixed costs
        int64_t want_blocks = batched ? 32 : 2048;
        int64_t cap = ((int64_t)d->N * d->C + want_blocks - 1) / want_blocks;
        if (cap < 1) cap = 1;
        if (cpb > cap) cpb = (int)cap;
        if (cpb > d->C) cpb = d->C;
        if (cpb > UNFOLD_MAX_PROWS / (d->kh * d->kw)) cpb = UNFOLD_MAX_PROWS / (d->kh * d->kw);   // the offset table holds them
        a.cpb = cpb < 1 ? 1 : cpb;
    } else {
        a.cpb = 1;
        a.rows_out = a.compact ? UNFOLD_LDS_ELEMS / row_elems : (UNFOLD_LDS_ELEMS / row_elems - a.kh) / a.sh + 1;
        if (a.rows_out < 1) a.rows_out = 1;
    }
    a.rows_in = (a.rows_out - 1) * a.sh + a.kh;
    a.plane = (a.compact ? a.rows_out : a.rows_in) * row_elems;
    // the flattened per-workgroup counters must stay exactly representable in fp32
    if ((int64_t)a.cpb * a.kh * a.kw * a.rows_out * a.Wo >= (1 << 24)) return false;
    a.inv_Wp = 1.0f / (float)a.Wp;
    a.inv_Wo = 1.0f / (float)a.Wo;
    a.inv_kw = 1.0f / (float)a.kw;
    a.inv_kh = 1.0f / (float)a.kh;
    a.inv_rows_in = 0.f;
    a.inv_Tc = 0.f;
    grid = dim3((a.Ho + a.rows_out - 1) / a.rows_out, (d->C + a.cpb - 1) / a.cpb, d->N);
    return grid.y <= 65535 && grid.z <= 65535;
}
double unfold_bytes(const kfac_conv_desc *d, const UnfoldArgs &a) {
    const double esz = d->dtype == KFAC_F32 ? 4.0 : 2.0;
    return esz * ((double)d->N * d->C * d->H * d->W + (double)d->N * d->C * d->kh * d->kw * a.Ho * a.Wo);
}
}  // namespace

int kfac_launch_unfold(kfac_ctx *ctx, const kfac_conv_desc *d, const void *x, void *patches) {
    UnfoldArgs a;
    dim3 grid;
    if (!plan_unfold(d, a, grid)) return KFAC_EINVAL;
    KfacProfScope prof(ctx, KC_UNFOLD, 0.0, unfold_bytes(d, a));
    if (d->dtype == KFAC_F32)
        hipLaunchKernelGGL(unfold_kernel<float>, grid, dim3(256), 0, ctx->stream, (const float *)x, (float *)patches, a);
    else
        hipLaunchKernelGGL(unfold_kernel<unsigned short>, grid, dim3(256), 0, ctx->stream,
                           (const unsigned short *)x, (unsigned short *)patches, a);
    KFAC_HIP_CHECK(hipGetLastError());
    return KFAC_OK;
}

size_t kfac_unfold_ws_bytes_impl(int n) { return kfac_align_up((size_t)n * sizeof(UnfoldItem), 256); }

// All layers of one element type in one launch (two launches for a mixed batch), largest layers first.
int kfac_launch_unfold_batched(kfac_ctx *ctx, int n, const kfac_conv_desc *descs, const void *const *x, void *const *patches) {
    if (kfac_unfold_ws_bytes_impl(n) > ctx->ws_bytes) return KFAC_EWORKSPACE;
    std::vector<UnfoldItem> items[2];
    double bytes[2] = {0.0, 0.0};
    std::vector<int> order(n);
    std::vector<int64_t> work(n);
    for (int i = 0; i < n; ++i) {
        order[i] = i;
        work[i] = (int64_t)descs[i].N * descs[i].C * descs[i].kh * descs[i].kw * descs[i].H * descs[i].W;
    }
    std::stable_sort(order.begin(), order.end(), [&](int p, int q) { return work[p] > work[q]; });
    int64_t total[2] = {0, 0};
    for (int i : order) {
        UnfoldItem it;
        dim3 grid;
        if (!plan_unfold(&descs[i], it.a, grid, true)) return KFAC_EINVAL;
        const int f = descs[i].dtype == KFAC_F32 ? 0 : 1;
        it.x = x[i];
        it.out = patches[i];
        it.gx = (int)grid.x;
        it.gy = (int)grid.y;
        if (total[f] + (int64_t)grid.x * grid.y * grid.z >= ((int64_t)1 << 31)) return KFAC_EINVAL;
        it.first = (int)total[f];
        total[f] += (int64_t)grid.x * grid.y * grid.z;
        bytes[f] += unfold_bytes(&descs[i], it.a);
        items[f].push_back(it);
    }
    UnfoldItem *d_items = (UnfoldItem *)ctx->ws;
    size_t at = 0;
    for (int f = 0; f < 2; ++f) {
        if (items[f].empty()) continue;
        KFAC_CHECK(kfac_upload(ctx, d_items + at, items[f].data(), items[f].size() * sizeof(UnfoldItem)));
        KfacProfScope prof(ctx, KC_UNFOLD, 0.0, bytes[f]);
        if (f == 0)
            hipLaunchKernelGGL(unfold_batched_kernel<float>, dim3((unsigned)total[f]), dim3(256), 0, ctx->stream, d_items + at, (int)items[f].size());
        else
            hipLaunchKernelGGL(unfold_batched_kernel<unsigned short>, dim3((unsigned)total[f]), dim3(256), 0, ctx->stream, d_items + at, (int)items[f].size());
        at += items[f].size();
    }
    KFAC_HIP_CHECK(hipGetLastError());
    return KFAC_OK;
}
