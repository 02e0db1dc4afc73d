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

constexpr int UNFOLD_LDS_ELEMS = 8192;  // staged input elements per workgroup (32 KB as fp32)

struct UnfoldArgs {
    int N, C, H, W, kh, kw, sh, sw, ph, pw, Ho, Wo;
    int cpb;       // channels per workgroup
    int rows_out;  // output rows per workgroup
    int rows_in;   // staged input rows = (rows_out-1)*sh + kh
    int Wp;        // staged row width = W + 2*pw
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
__device__ inline void unfold_block(const E *__restrict__ x, E *__restrict__ out, const UnfoldArgs &a, int bx, int by, int bz, E *tile) {
    const int n = bz;
    const int c0 = by * a.cpb;
    const int ho0 = bx * a.rows_out;
    const int nch = min(a.cpb, a.C - c0);
    const int rows_out = min(a.rows_out, a.Ho - ho0);
    const int rows_in = (rows_out - 1) * a.sh + a.kh;
    const int h_first = ho0 * a.sh - a.ph;
    const int plane = a.rows_in * a.Wp;  // LDS pitch per channel
    // ---- stage: tile[cc][hr][wc] = x[n][c0+cc][h_first+hr][wc-pw] or 0 ----
    const int stage_n = nch * rows_in * a.Wp;
    for (int e = threadIdx.x; e < stage_n; e += 256) {
        int row, wc, cc, hr;
        fdivmod(e, a.Wp, a.inv_Wp, row, wc);
        fdivmod(row, rows_in, 1.0f / (float)rows_in, cc, hr);
        const int h = h_first + hr, w = wc - a.pw;
        E v = 0;
        if (h >= 0 && h < a.H && w >= 0 && w < a.W) v = x[(((int64_t)n * a.C + c0 + cc) * a.H + h) * a.W + w];
        tile[cc * plane + hr * a.Wp + wc] = v;
    }
    __syncthreads();
    // ---- write ----
    // For (cc, ky, kx) the outputs of this workgroup are the run of Tc = rows_out*Wo positions starting at
    // (ho0, 0).  With full-height chunks (Tc == T) the runs of consecutive patch rows are adjacent, so the whole
    // workgroup writes ONE contiguous run; otherwise one run per patch row.  A run is cut into 16-byte vectors
    // aligned in global memory (the first and last may be partial and are stored element by element); the
    // decode of a vector's first element costs a few divisions, the rest of the vector is reached by carries.
    constexpr int VEC = 16 / (int)sizeof(E);
    const int Tc = rows_out * a.Wo;
    const int T = a.Ho * a.Wo;
    const int khw = a.kh * a.kw;
    const bool one_run = Tc == T;
    const int nrun = one_run ? 1 : nch * khw;
    const int L = one_run ? nch * khw * T : Tc;
    const float inv_Tc = 1.0f / (float)Tc;
    const float inv_khw = 1.0f / (float)khw;
    E *const out0 = out + ((int64_t)n * a.C + c0) * khw * T + (int64_t)ho0 * a.Wo;   // run 0, element 0
    for (int run = 0; run < nrun; ++run) {
        E *const dst = out0 + (int64_t)run * T;
        const int g0 = (int)((reinterpret_cast<uintptr_t>(dst) / sizeof(E)) % VEC);   // elements past a 16-byte boundary
        const int nvec = (L + g0 + VEC - 1) / VEC;
        for (int v = threadIdx.x; v < nvec; v += 256) {
            const int j0 = v * VEC - g0;             // first element of the vector inside the run (may be < 0)
            const int jb = max(j0, 0), je = min(j0 + VEC, L);
            int prow, t, cc, kk, ky, kx, hoo, wo;
            if (one_run) fdivmod(jb, Tc, inv_Tc, prow, t);
            else { prow = run; t = jb; }
            fdivmod(prow, khw, inv_khw, cc, kk);
            fdivmod(kk, a.kw, a.inv_kw, ky, kx);
            fdivmod(t, a.Wo, a.inv_Wo, hoo, wo);
            E vals[VEC];
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                const int j = j0 + i;
                E x = 0;
                if (j >= jb && j < je) {
                    x = tile[cc * plane + (hoo * a.sh + ky) * a.Wp + wo * a.sw + kx];
                    if (++wo == a.Wo) {
                        wo = 0;
                        if (++hoo == rows_out) {     // only reached inside the single run: next patch row
                            hoo = 0;
                            if (++kx == a.kw) {
                                kx = 0;
                                if (++ky == a.kh) { ky = 0; ++cc; }
                            }
                        }
                    }
                }
                vals[i] = x;
            }
            if (jb == j0 && je == j0 + VEC) {
                uint4 q;
                __builtin_memcpy(&q, vals, 16);
                *reinterpret_cast<uint4 *>(dst + j0) = q;
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
    __shared__ E tile[UNFOLD_LDS_ELEMS];
    unfold_block<E>(x, out, a, blockIdx.x, blockIdx.y, blockIdx.z, tile);
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
    __shared__ E tile[UNFOLD_LDS_ELEMS];
    const int b = blockIdx.x;
    int lo = 0, hi = n - 1;                 // last layer whose first workgroup is <= b
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (items[mid].first <= b) lo = mid; else hi = mid - 1;
    }
    const UnfoldItem &it = items[lo];
    const int r = b - it.first;
    const int bx = r % it.gx, t = r / it.gx;
    unfold_block<E>((const E *)it.x, (E *)it.out, it.a, bx, t % it.gy, t / it.gy, tile);
}

}  // namespace

namespace {
// Tiling of one layer: fills `a` and the grid; false when the shape does not fit the kernel's limits.
bool plan_unfold(const kfac_conv_desc *d, UnfoldArgs &a, dim3 &grid) {
    a.N = d->N; a.C = d->C; a.H = d->H; a.W = d->W; a.kh = d->kh; a.kw = d->kw;
    a.sh = d->stride_h; a.sw = d->stride_w; a.ph = d->pad_h; a.pw = d->pad_w;
    a.Ho = (d->H + 2 * d->pad_h - d->kh) / d->stride_h + 1;
    a.Wo = (d->W + 2 * d->pad_w - d->kw) / d->stride_w + 1;
    a.Wp = d->W + 2 * d->pad_w;
    const int rows_in_full = (a.Ho - 1) * a.sh + a.kh;
    if ((int64_t)d->kh * a.Wp > UNFOLD_LDS_ELEMS) return false;  // one output row must fit
    if ((int64_t)rows_in_full * a.Wp <= UNFOLD_LDS_ELEMS) {
        a.rows_out = a.Ho;
        int cpb = UNFOLD_LDS_ELEMS / (rows_in_full * a.Wp);
        int64_t want_blocks = 2048;  // keep the grid large enough to fill 256 CUs several times over
        int64_t cap = ((int64_t)d->N * d->C + want_blocks - 1) / want_blocks;
        if (cap < 1) cap = 1;
        if (cpb > cap) cpb = (int)cap;
        if (cpb > d->C) cpb = d->C;
        a.cpb = cpb < 1 ? 1 : cpb;
    } else {
        a.cpb = 1;
        a.rows_out = (UNFOLD_LDS_ELEMS / a.Wp - a.kh) / a.sh + 1;
        if (a.rows_out < 1) a.rows_out = 1;
    }
    a.rows_in = (a.rows_out - 1) * a.sh + a.kh;
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
        if (!plan_unfold(&descs[i], it.a, grid)) return KFAC_EINVAL;
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
