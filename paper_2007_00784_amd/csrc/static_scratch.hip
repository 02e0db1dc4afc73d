// kfac_update_factors_static: the factor update for callers that cannot allocate device memory or hand over
// a workspace (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same
// kernels and split plan as kfac_update_factors(); the job tables and split partials live in a file-scope
// device array of this library instead of the context's workspace.
//
// Every device the library runs on holds its own copy of the array, at its own address, until the process ends.
// The array's name is a host-side stand-in and never a kernel argument: its device address is looked up once per
// device (from kfac_create(), with that device current) and that pointer is what the kernels and copies get.
// All calls on one device share the array: calls that overlap on one device race.  Nothing in it has to start
// at zero: the tables are uploaded whole and every partial tile that the reducer reads was written by a SYRK
// workgroup of the same call.
#include <mutex>
#include "kfac_internal.h"

namespace {

constexpr size_t SCRATCH_BYTES = KFAC_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
void *scratch_ptr[MAX_DEVICES];   // device address of `scratch` per device; nullptr until looked up
std::mutex scratch_mutex;

}  // namespace

int kfac_static_scratch_init(int device) {
    if (device < 0 || device >= MAX_DEVICES) return KFAC_EINVAL;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (scratch_ptr[device]) return KFAC_OK;
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
        (void)hipGetLastError();
        return KFAC_EHIP;
    }
    scratch_ptr[device] = p;
    return KFAC_OK;
}

extern "C" {

size_t kfac_static_scratch_bytes(void) { return SCRATCH_BYTES; }

int kfac_update_factors_static(kfac_ctx *ctx, const void *X, int dtype, int layout, int N, int d, int T,
                               int append_ones, float scale, float decay, float *F) {
    if (!ctx) return KFAC_EINVAL;
    const kfac_factor_item it{X, dtype, layout, N, d, T, append_ones, scale, decay, F};
    if (!kfac_valid_factor_item(it, true)) return KFAC_EINVAL;
    void *ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(scratch_mutex);
        ptr = scratch_ptr[ctx->device];
    }
    if (!ptr) return KFAC_EHIP;   // kfac_create() looks the address up; a context cannot exist without it
    if (kfac_syrk_ws_bytes_impl(1, &it) > SCRATCH_BYTES) return KFAC_ESCRATCH;
    return kfac_launch_update_factors_ws(ctx, 1, &it, (char *)ptr, SCRATCH_BYTES);
}

}  // extern "C"
