// Kronecker-factor update: F <- decay*F + (1-decay)*scale * Xt^T Xt  (Sec. II-C factors, Sec. IV-B
// running average).  The Gram matrix is a symmetric rank-R update on the matrix cores: only the
// lower-triangular 128x128 tiles of X^T X are computed and mirrored, the contraction over the sample
// rows is split across workgroups when there are few tiles, and the running average is applied where
// the final sum is formed (the SYRK epilogue, or the fixed-order split reducer).  Samples in [N][d][T]
// layout (every conv factor) run on the grouped-load engine -- fp32 MFMAs for fp32 samples, bf16 MFMAs
// for bf16 ones -- the rest ([R][d] layout, T below one 16-byte group) on the element-wise fp32 engine.
//
// The appended ones column is not materialised and costs no MFMA tile: its row of the factor is the
// vector of column sums of X, which every diagonal tile accumulates for its own 128 columns from the
// operand elements it loads anyway; the corner entry is scale * R.
#include <algorithm>
#include <cmath>
#include <vector>
#include "kfac_internal.h"
#include "mfma_gemm.h"
#include "mfma_gemm_grouped.h"

using namespace kfac;

namespace {

constexpr int PART = BM * BM + BM;   // floats per split partial: the tile, then 128 column sums

struct SyrkArgs {     // one factor update of a batch
    const void *X;
    int d;            // features (tile grid covers d x d)
    int D;            // factor dimension (d + append_ones), leading dimension of F
    int ones;         // 1: also produce the bias row/column
    int nsplit;       // workgroups along K per tile
    int kchunk;       // K rows per split (multiple of BK)
    int K;            // total sample rows
    int T;            // [N][d][T] layout: positions per example
    int gpe;          // grouped engine: groups of 16 bytes of positions per example, ceil(T / EPG); kchunk counts groups
    int Q;            // grouped engine: groups in all, N * gpe
    int ntri;         // lower-triangular tiles
    float alpha;      // (1-decay)*scale
    float decay;
    float *F;
    float *partial;   // [nsplit][ntri][PART] when nsplit > 1
};
struct SyrkJob { int item, tri, split; };   // one workgroup's share: tile `tri` of factor `item`, K split `split`

__device__ inline void tri_decode(int idx, int &ti, int &tj) {
    // idx = ti*(ti+1)/2 + tj, tj <= ti
    int t = (int)((sqrtf(8.f * (float)idx + 1.f) - 1.f) * 0.5f);
    while ((t + 1) * (t + 2) / 2 <= idx) ++t;
    while (t * (t + 1) / 2 > idx) --t;
    ti = t;
    tj = idx - t * (t + 1) / 2;
}

__device__ inline void ema_store(float *F, int D, int r, int c, float v, float alpha, float decay, bool mirror) {
    const int64_t o = (int64_t)r * D + c;
    float out = alpha * v;
    if (decay != 0.f) out += decay * F[o];
    F[o] = out;
    if (mirror) F[(int64_t)c * D + r] = out;
}

// Fixed-order reduction of the per-thread column sums of a diagonal tile into cs[0..127] (LDS).
template <bool KFAST>
__device__ inline void reduce_colsum(const float (&csum)[EPT], float *scratch /* >= 128*16 floats */, float *cs) {
    const int tid = threadIdx.x;
    __syncthreads();
    if (KFAST) {   // slot s holds column (tid>>4)+16s; the 16 threads tid&15 share it
#pragma unroll
        for (int s = 0; s < EPT; ++s) scratch[((tid >> 4) + 16 * s) * 16 + (tid & 15)] = csum[s];
    } else {       // every slot is column tid&127; two threads (tid>>7) share it
        float t = 0.f;
#pragma unroll
        for (int s = 0; s < EPT; ++s) t += csum[s];
        scratch[(tid & 127) * 16 + (tid >> 7)] = t;
    }
    __syncthreads();
    if (tid < BM) {
        float t = 0.f;
        const int n = KFAST ? 16 : 2;
        for (int u = 0; u < n; ++u) t += scratch[tid * 16 + u];
        cs[tid] = t;
    }
    __syncthreads();
}

template <class Op> __device__ inline Op make_op(const SyrkArgs &g);
template <> __device__ inline OpNDT<float> make_op(const SyrkArgs &g) { return OpNDT<float>{(const float *)g.X, g.d, g.T, 0, -1}; }
template <> __device__ inline OpNDT<unsigned short> make_op(const SyrkArgs &g) {
    return OpNDT<unsigned short>{(const unsigned short *)g.X, g.d, g.T, 0, -1};
}
// [R][d]: feature index contiguous, sample index strided by d
template <> __device__ inline OpStrided<float, false> make_op(const SyrkArgs &g) {
    return OpStrided<float, false>{(const float *)g.X, 1, g.d, g.d, 0, -1};
}
template <> __device__ inline OpStrided<unsigned short, false> make_op(const SyrkArgs &g) {
    return OpStrided<unsigned short, false>{(const unsigned short *)g.X, 1, g.d, g.d, 0, -1};
}

// Final sum of a tile (running average applied, mirrored) or this split's partial.
__device__ inline void syrk_epilogue(const SyrkArgs &g, const SyrkJob &job, int ti, int tj, bool want_cs,
                                     const floatx16 (&acc)[2][2], const float *cs) {
    const bool diag = ti == tj;
    if (g.nsplit == 1) {
        for_each_acc(acc, [&](int r, int c, float v) {
            const int gr = ti * BM + r, gc = tj * BM + c;
            if (gr < g.d && gc < g.d && (!diag || gc <= gr))
                ema_store(g.F, g.D, gr, gc, v, g.alpha, g.decay, gr != gc);
        });
        if (want_cs) {
            const int gc = ti * BM + threadIdx.x;
            if (threadIdx.x < BM && gc < g.d) ema_store(g.F, g.D, g.d, gc, cs[threadIdx.x], g.alpha, g.decay, true);
            if (job.tri == 0 && threadIdx.x == 0) ema_store(g.F, g.D, g.d, g.d, (float)g.K, g.alpha, g.decay, false);
        }
    } else {
        float *dst = g.partial + ((int64_t)job.split * g.ntri + job.tri) * PART;
        for_each_acc(acc, [&](int r, int c, float v) { dst[r * BM + c] = v; });
        if (want_cs && threadIdx.x < BM) dst[BM * BM + threadIdx.x] = cs[threadIdx.x];
    }
}

// One launch serves every factor of a batch that shares an operand form: workgroup b takes jobs[b].
template <class Op>
__global__ __launch_bounds__(NTHREADS) __attribute__((amdgpu_waves_per_eu(2))) void syrk_kernel(const SyrkArgs *items, const SyrkJob *jobs) {
    __shared__ TileSmem sm;
    __shared__ float cs[BM];
    const SyrkJob job = jobs[blockIdx.x];
    if (job.item < 0) return;   // padding of the launch order
    const SyrkArgs g = items[job.item];
    int ti, tj;
    tri_decode(job.tri, ti, tj);
    const int split = job.split;
    const int kbeg = split * g.kchunk;
    const int kend = min(g.K, kbeg + g.kchunk);
    const bool diag = ti == tj;
    const bool want_cs = diag && g.ones;
    Op a = make_op<Op>(g), b = a;
    a.K = kend;
    b.K = kend;
    floatx16 acc[2][2];
    float csum[EPT];
#pragma unroll
    for (int s = 0; s < EPT; ++s) csum[s] = 0.f;
    if (want_cs) {
        gemm_tile<Op, Op, true>(a, b, ti * BM, tj * BM, kbeg, kend, sm, acc, csum);
        reduce_colsum<Op::KFAST>(csum, &sm.a[0][0][0], cs);
    } else {
        gemm_tile<Op, Op, false>(a, b, ti * BM, tj * BM, kbeg, kend, sm, acc);
    }
    syrk_epilogue(g, job, ti, tj, want_cs, acc, cs);
}

// The same for samples in [N][d][T] layout with T >= EPG (4 fp32, 8 bf16), on the grouped-load engine.  kchunk
// and Q count groups of EPG positions.  Dynamic LDS: GrpSmem, then 128 floats of column sums.
template <typename E>
__global__ __launch_bounds__(NTHREADS) __attribute__((amdgpu_waves_per_eu(2))) void syrk_grouped_kernel(const SyrkArgs *items, const SyrkJob *jobs) {
    extern __shared__ __align__(16) char smem[];
    GrpSmem &sm = *reinterpret_cast<GrpSmem *>(smem);
    float *cs = reinterpret_cast<float *>(smem + sizeof(GrpSmem));
    const SyrkJob job = jobs[blockIdx.x];
    if (job.item < 0) return;   // padding of the launch order
    const SyrkArgs g = items[job.item];
    int ti, tj;
    tri_decode(job.tri, ti, tj);
    const int q0 = job.split * g.kchunk;
    const int q_end = min(g.Q, q0 + g.kchunk);
    const bool diag = ti == tj;
    const bool want_cs = diag && g.ones;
    GrpOpNDT<E> a{(const E *)g.X, g.d, g.T, g.gpe, 0}, b = a;
    floatx16 acc[2][2];
    float csum[GRP_RPT];
#pragma unroll
    for (int u = 0; u < GRP_RPT; ++u) csum[u] = 0.f;
    if (g.d <= 64) {   // one tile, a quarter of it in use: contraction split over the waves instead
        if (want_cs) gemm_tile_grouped_small<E, true>(a, q0, q_end, sm, acc, csum);
        else gemm_tile_grouped_small<E, false>(a, q0, q_end, sm, acc, csum);
    } else if (want_cs) gemm_tile_grouped<E, true, true>(a, b, ti * BM, tj * BM, q0, q_end, sm, acc, csum);
    else if (diag) gemm_tile_grouped<E, true, false>(a, b, ti * BM, tj * BM, q0, q_end, sm, acc, csum);
    else gemm_tile_grouped<E, false, false>(a, b, ti * BM, tj * BM, q0, q_end, sm, acc, csum);
    if (want_cs) {   // the K loop ended on a barrier, so the slab buffers are free: sum the eight threads of a row in order
        const int tid = threadIdx.x;
        float *scratch = reinterpret_cast<float *>(sm.a[0]);
#pragma unroll
        for (int u = 0; u < GRP_RPT; ++u) scratch[((tid >> 3) + 32 * u) * 8 + (tid & 7)] = csum[u];
        __syncthreads();
        if (tid < BM) {
            float t = 0.f;
            for (int k = 0; k < 8; ++k) t += scratch[tid * 8 + k];
            cs[tid] = t;
        }
        __syncthreads();
    }
    syrk_epilogue(g, job, ti, tj, want_cs, acc, cs);
}

// Sum the split partials of each tile in split order, then apply the running average and mirror.
// One thread per tile element (plus 128 for the column sums of diagonal tiles); the loads of
// consecutive splits are independent, so they are issued eight at a time.  jobs: (item, tile) pairs.
__global__ __launch_bounds__(256) void syrk_reduce_kernel(const SyrkArgs *items, const SyrkJob *jobs) {
    const SyrkJob job = jobs[blockIdx.x];
    const SyrkArgs g = items[job.item];
    int ti, tj;
    tri_decode(job.tri, ti, tj);
    const bool diag = ti == tj;
    const int e = threadIdx.x + blockIdx.y * 256;          // 0 .. PART-1 (grid covers PART rounded up)
    if (e >= PART) return;
    int gr, gc;
    bool mirror;
    if (e < BM * BM) {
        gr = ti * BM + e / BM;
        gc = tj * BM + e % BM;
        if (gr >= g.d || gc >= g.d || (diag && gc > gr)) return;
        mirror = gr != gc;
    } else {
        if (!diag || !g.ones) return;
        gr = g.d;
        gc = ti * BM + (e - BM * BM);
        if (gc >= g.d) return;
        mirror = true;
    }
    const float *src = g.partial + (int64_t)job.tri * PART + e;
    const int64_t stride = (int64_t)g.ntri * PART;
    float s = 0.f;
    int sp = 0;
    for (; sp + 8 <= g.nsplit; sp += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[(sp + u) * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; sp < g.nsplit; ++sp) s += src[sp * stride];
    ema_store(g.F, g.D, gr, gc, s, g.alpha, g.decay, mirror);
    if (g.ones && job.tri == 0 && e == 0) ema_store(g.F, g.D, g.d, g.d, (float)g.K, g.alpha, g.decay, false);
}

// Choose the number of K splits of one factor launched alone.  Two workgroups share a compute unit
// (register budget), so the machine has 512 slots; a launch takes ceil(workgroups / 512) rounds of (slabs
// per split + a fixed per-workgroup cost, in slabs, for prologue, epilogue and partial traffic: about 12
// slabs of the fp32 engine).  R counts contraction units (sample rows; groups on the bf16 engine) and `slab`
// is the engine's slab in those units.
void plan_single(int d, int64_t R, int slab, double fixed, int &ntri, int &nsplit, int &kchunk) {
    const int ntile = (d + BM - 1) / BM;
    ntri = ntile * (ntile + 1) / 2;
    const int64_t slabs = (R + slab - 1) / slab;
    int best = 1;
    double best_cost = 1e300;
    for (int ns = 1; ns <= 512; ++ns) {
        if (ns > 1 && slabs / ns < 8) break;                 // keep >= 8 slabs per split
        if (ns > 1 && (int64_t)ntri * ns > KFAC_SYRK_MAX_SINGLE_PARTIALS) break;   // bounds the workspace of a lone factor
        const double rounds = std::ceil((double)ntri * ns / 512.0);
        const double cost = rounds * ((double)((slabs + ns - 1) / ns) + fixed);
        if (cost < best_cost * 0.999) { best_cost = cost; best = ns; }
    }
    nsplit = best;
    int64_t chunk = (R + nsplit - 1) / nsplit;
    chunk = (chunk + slab - 1) / slab * slab;
    kchunk = (int)chunk;
    nsplit = (int)((R + chunk - 1) / chunk);
}

// In a batch the other factors fill the machine, so a factor is cut into jobs of about JOB_SLABS slabs
// each: long enough to amortise a job's fixed cost and its 64 KB partial, short enough that the longest
// job is a small part of the launch.
constexpr int XCD_PAD = 8 * 16;   // no-op jobs that the XCD-aware launch order may add to one operand form
constexpr int JOB_SLABS = 512;
constexpr int JOB_SLABS_GRP_F32 = 256;   // grouped engine, fp32: slabs of 32 sample rows
constexpr int JOB_SLABS_GRP_B16 = 256;   // grouped engine, bf16: slabs of 64 sample rows
void plan_batched(int d, int64_t R, int slab, int job_slabs, int &ntri, int &nsplit, int &kchunk) {
    const int ntile = (d + BM - 1) / BM;
    ntri = ntile * (ntile + 1) / 2;
    const int64_t slabs = (R + slab - 1) / slab;
    nsplit = (int)std::max<int64_t>(1, (slabs + job_slabs / 2) / job_slabs);
    int64_t chunk = (R + nsplit - 1) / nsplit;
    chunk = (chunk + slab - 1) / slab * slab;
    kchunk = (int)chunk;
    nsplit = (int)((R + chunk - 1) / chunk);
}

// Operand forms, one launch each.  0: [N][d][T] fp32 with T < 4, 1: [N][d][T] bf16 with T < 8, 2: [R][d] fp32,
// 3: [R][d] bf16 (all on the element-wise fp32 engine); 4: [N][d][T] bf16, 5: [N][d][T] fp32 on the grouped engine.
constexpr int NFORM = 6;
int form_of(const kfac_factor_item &it) {
    const bool ndt = it.layout == KFAC_LAYOUT_NDT && it.T > 1;
    if (it.dtype == KFAC_F32) return !ndt ? 2 : (it.T >= 4 ? 5 : 0);
    return !ndt ? 3 : (it.T >= 8 ? 4 : 1);
}

void plan_item(int n, const kfac_factor_item &it, int &ntri, int &nsplit, int &kchunk) {
    const int form = form_of(it);
    if (form >= 4) {   // contraction units are groups of 16 bytes
        const int epg = form == 4 ? 8 : 4;
        const int64_t Q = (int64_t)it.N * ((it.T + epg - 1) / epg);
        if (n == 1) plan_single(it.d, Q, GRP_GROUPS, form == 4 ? 30.0 : 6.0, ntri, nsplit, kchunk);
        else plan_batched(it.d, Q, GRP_GROUPS, form == 4 ? JOB_SLABS_GRP_B16 : JOB_SLABS_GRP_F32, ntri, nsplit, kchunk);
        return;
    }
    const int64_t R = (int64_t)it.N * it.T;
    if (n == 1) plan_single(it.d, R, BK, 12.0, ntri, nsplit, kchunk);
    else plan_batched(it.d, R, BK, JOB_SLABS, ntri, nsplit, kchunk);
}

// Workspace layout: SyrkArgs[n], the job table, the reducer's job table, then every factor's partials.
size_t layout(int n, const kfac_factor_item *items, size_t &off_jobs, size_t &off_rjobs, size_t &off_part, size_t &njobs, size_t &nrjobs) {
    njobs = nrjobs = 0;
    size_t part = 0;
    for (int i = 0; i < n; ++i) {
        int ntri, nsplit, kchunk;
        plan_item(n, items[i], ntri, nsplit, kchunk);
        njobs += (size_t)ntri * nsplit;
        if (nsplit > 1) {
            nrjobs += ntri;
            part += (size_t)nsplit * ntri * PART;
        }
    }
    off_jobs = kfac_align_up((size_t)n * sizeof(SyrkArgs), 256);
    off_rjobs = off_jobs + kfac_align_up((njobs + NFORM * XCD_PAD) * sizeof(SyrkJob), 256);   // + padding of the XCD order
    off_part = off_rjobs + kfac_align_up(nrjobs * sizeof(SyrkJob), 256);
    return off_part + part * sizeof(float);
}

// Launch order of one operand form.  Workgroups go round the 8 XCDs (workgroup b runs on XCD b % 8), each with its
// own L2.  Tiles that share operand panels -- the tiles of one 4 x 4 block of tiles of one K range of one factor:
// 16 tiles, 8 panels -- are therefore placed 8 apart, one after the other on the same XCD, where they run at the
// same time and fetch each panel from memory once instead of once per tile.  Blocks are dealt to the XCD whose list
// is shortest; lists are padded to equal length with no-op jobs (item -1) so that the positions stay aligned.
constexpr int XCDS = 8, SUPER = 4;
void xcd_order(std::vector<SyrkJob> &jobs) {
    if (jobs.size() < 2 * XCDS) return;
    std::vector<SyrkJob> lists[XCDS];
    auto tile_of = [](int tri, int &ti, int &tj) {
        int t = (int)((std::sqrt(8.0 * tri + 1.0) - 1.0) * 0.5);
        while ((t + 1) * (t + 2) / 2 <= tri) ++t;
        while (t * (t + 1) / 2 > tri) --t;
        ti = t;
        tj = tri - t * (t + 1) / 2;
    };
    size_t i = 0;
    while (i < jobs.size()) {
        // the jobs of one (factor, K range) are contiguous; cut them into blocks of SUPER x SUPER tiles
        size_t e = i;
        while (e < jobs.size() && jobs[e].item == jobs[i].item && jobs[e].split == jobs[i].split) ++e;
        std::vector<std::pair<int, SyrkJob>> keyed;
        keyed.reserve(e - i);
        for (size_t k = i; k < e; ++k) {
            int ti, tj;
            tile_of(jobs[k].tri, ti, tj);
            keyed.push_back({(ti / SUPER) * 4096 + tj / SUPER, jobs[k]});
        }
        std::stable_sort(keyed.begin(), keyed.end(), [](const std::pair<int, SyrkJob> &a, const std::pair<int, SyrkJob> &b) { return a.first < b.first; });
        size_t k = 0;
        while (k < keyed.size()) {
            size_t ke = k;
            while (ke < keyed.size() && keyed[ke].first == keyed[k].first) ++ke;
            int best = 0;
            for (int x = 1; x < XCDS; ++x) if (lists[x].size() < lists[best].size()) best = x;
            for (; k < ke; ++k) lists[best].push_back(keyed[k].second);
        }
        i = e;
    }
    size_t len = 0;
    for (auto &l : lists) len = std::max(len, l.size());
    jobs.assign(len * XCDS, SyrkJob{-1, 0, 0});
    for (int x = 0; x < XCDS; ++x)
        for (size_t k = 0; k < lists[x].size(); ++k) jobs[k * XCDS + x] = lists[x][k];
}

template <class Op>
void launch_class(kfac_ctx *ctx, const SyrkArgs *d_items, const SyrkJob *d_jobs, size_t count, double flops, double bytes) {
    if (count == 0) return;
    KfacProfScope prof(ctx, KC_SYRK, flops, bytes);
    hipLaunchKernelGGL((syrk_kernel<Op>), dim3((unsigned)count), dim3(NTHREADS), 0, ctx->stream, d_items, d_jobs);
}

}  // namespace

size_t kfac_syrk_ws_bytes_impl(int n, const kfac_factor_item *items) {
    size_t a, b, c, d, e;
    return layout(n, items, a, b, c, d, e);
}

size_t kfac_syrk_workspace_bytes(int D, int64_t R) {
    kfac_factor_item it{};
    it.N = 1;
    it.T = (int)std::min<int64_t>(R, (int64_t)1 << 30);
    it.d = D;
    return kfac_syrk_ws_bytes_impl(1, &it);
}

int kfac_launch_update_factors_batched(kfac_ctx *ctx, int n, const kfac_factor_item *items) {
    return kfac_launch_update_factors_ws(ctx, n, items, ctx->ws, ctx->ws_bytes);
}

int kfac_launch_update_factors_ws(kfac_ctx *ctx, int n, const kfac_factor_item *items, char *ws, size_t ws_bytes) {
    size_t off_jobs, off_rjobs, off_part, njobs, nrjobs;
    const size_t need = layout(n, items, off_jobs, off_rjobs, off_part, njobs, nrjobs);
    if (need > ws_bytes) return KFAC_EWORKSPACE;
    std::vector<SyrkArgs> args(n);
    // jobs grouped by operand form, inside a form the longest contraction first
    std::vector<SyrkJob> jobs[NFORM], rjobs;
    double flops[NFORM] = {}, bytes[NFORM] = {}, rbytes = 0.0;
    float *part = (float *)(ws + off_part);
    for (int i = 0; i < n; ++i) {
        const kfac_factor_item &it = items[i];
        SyrkArgs &g = args[i];
        const int64_t R = (int64_t)it.N * it.T;
        plan_item(n, it, g.ntri, g.nsplit, g.kchunk);
        g.X = it.X;
        g.d = it.d;
        g.D = it.d + (it.append_ones ? 1 : 0);
        g.ones = it.append_ones ? 1 : 0;
        g.K = (int)R;
        g.T = it.T;
        const int epg = it.dtype == KFAC_F32 ? 4 : 8;
        g.gpe = (it.T + epg - 1) / epg;
        g.Q = it.N * g.gpe;
        g.alpha = (1.f - it.decay) * it.scale;
        g.decay = it.decay;
        g.F = it.F;
        g.partial = part;
        if (g.nsplit > 1) part += (size_t)g.nsplit * g.ntri * PART;
        const int form = form_of(it);
        // all tiles of one K range next to one another: they run at the same time and share their operand panels
        // in L2 and the Infinity Cache instead of each fetching them from memory
        for (int sp = 0; sp < g.nsplit; ++sp)
            for (int t = 0; t < g.ntri; ++t) jobs[form].push_back(SyrkJob{i, t, sp});
        if (g.nsplit > 1)
            for (int t = 0; t < g.ntri; ++t) rjobs.push_back(SyrkJob{i, t, 0});
        // useful flops of the symmetric update R*D*(D+1); bytes: the samples once, F read (if averaged) and written
        const double esz = it.dtype == KFAC_F32 ? 4.0 : 2.0, D = g.D;
        const double fbytes = (it.decay != 0.f ? 8.0 : 4.0) * D * D;
        flops[form] += (double)R * D * (D + 1.0);
        bytes[form] += esz * (double)R * it.d + (g.nsplit == 1 ? fbytes : 0.0);
        if (g.nsplit > 1) rbytes += fbytes;
    }
    SyrkArgs *d_items = (SyrkArgs *)ws;
    SyrkJob *d_jobs = (SyrkJob *)(ws + off_jobs), *d_rjobs = (SyrkJob *)(ws + off_rjobs);
    KFAC_CHECK(kfac_upload(ctx, d_items, args.data(), n * sizeof(SyrkArgs)));
    size_t at[NFORM], pos = 0;
    for (int f = 0; f < NFORM; ++f) {
        std::stable_sort(jobs[f].begin(), jobs[f].end(), [&](const SyrkJob &a, const SyrkJob &b) { return args[a.item].kchunk > args[b.item].kchunk; });
        xcd_order(jobs[f]);
        at[f] = pos;
        if (!jobs[f].empty())
            KFAC_CHECK(kfac_upload(ctx, d_jobs + pos, jobs[f].data(), jobs[f].size() * sizeof(SyrkJob)));
        pos += jobs[f].size();
    }
    if (!rjobs.empty())
        KFAC_CHECK(kfac_upload(ctx, d_rjobs, rjobs.data(), rjobs.size() * sizeof(SyrkJob)));
    launch_class<OpNDT<float>>(ctx, d_items, d_jobs + at[0], jobs[0].size(), flops[0], bytes[0]);
    launch_class<OpNDT<unsigned short>>(ctx, d_items, d_jobs + at[1], jobs[1].size(), flops[1], bytes[1]);
    launch_class<OpStrided<float, false>>(ctx, d_items, d_jobs + at[2], jobs[2].size(), flops[2], bytes[2]);
    launch_class<OpStrided<unsigned short, false>>(ctx, d_items, d_jobs + at[3], jobs[3].size(), flops[3], bytes[3]);
    const int lds = (int)(sizeof(GrpSmem) + BM * sizeof(float));
    if ((!jobs[4].empty() || !jobs[5].empty()) && lds > ctx->max_lds) return KFAC_EHIP;
    if (!jobs[5].empty()) {
        KFAC_HIP_CHECK(hipFuncSetAttribute((const void *)syrk_grouped_kernel<float>, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        KfacProfScope prof(ctx, KC_SYRK, flops[5], bytes[5]);
        hipLaunchKernelGGL(syrk_grouped_kernel<float>, dim3((unsigned)jobs[5].size()), dim3(NTHREADS), lds, ctx->stream, d_items, d_jobs + at[5]);
    }
    if (!jobs[4].empty()) {
        KFAC_HIP_CHECK(hipFuncSetAttribute((const void *)syrk_grouped_kernel<unsigned short>, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        KfacProfScope prof(ctx, KC_SYRK_B16, flops[4], bytes[4]);
        hipLaunchKernelGGL(syrk_grouped_kernel<unsigned short>, dim3((unsigned)jobs[4].size()), dim3(NTHREADS), lds, ctx->stream, d_items, d_jobs + at[4]);
    }
    KFAC_HIP_CHECK(hipGetLastError());
    if (!rjobs.empty()) {
        KfacProfScope prof(ctx, KC_SYRK_REDUCE, 0.0, rbytes);
        hipLaunchKernelGGL(syrk_reduce_kernel, dim3((unsigned)rjobs.size(), (PART + 255) / 256), dim3(256), 0, ctx->stream, d_items, d_rjobs);
        KFAC_HIP_CHECK(hipGetLastError());
    }
    return KFAC_OK;
}

int kfac_launch_update_factors(kfac_ctx *ctx, const void *X, int dtype, int layout, int N, int d, int T,
                               int append_ones, float scale, float decay, float *F) {
    kfac_factor_item it{X, dtype, layout, N, d, T, append_ones, scale, decay, F};
    return kfac_launch_update_factors_batched(ctx, 1, &it);
}
