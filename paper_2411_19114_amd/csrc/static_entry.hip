// prep_resize_normalize_static: resize + centre crop + normalize for callers that cannot
// allocate (code under HIP graph capture, tight serving loops, harnesses that forbid
// hipMalloc).  The same kernels as prep_resize_normalize; what that entry point keeps in
// buffers of a handle, the per-image mapping records that the kernels read from device
// memory, lives here in a file-scope device array that every GPU holds until the process
// ends.  The call allocates nothing: no handle, no hipMalloc / hipFree, no copy through a
// staging buffer (the records travel as kernel arguments).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "../../include/prep.h"
#include "kernels.h"
#include "prep_internal.h"

namespace prep {

namespace {

constexpr int kMaxDevices = 64;
constexpr int kPack = 32;  // records per fill launch (1792 bytes of kernel arguments)

// The scratch buffer: the mapping records of one call, PREP_STATIC_MAX_IMAGES of them (56 KiB).
// In host code this name is only a handle for hipGetSymbolAddress; kernels and copies get the
// device address that call returns, one per device.
static __device__ __align__(256) ResizeRec scratch[PREP_STATIC_MAX_IMAGES];

std::mutex g_lock;
ResizeRec *g_scratch_of[kMaxDevices];  // device address of `scratch` on each device, once known

struct RecPack {
    ResizeRec r[kPack];
};

__global__ void store_resize_recs(RecPack pack, ResizeRec *__restrict__ dst, int count)
{
    const int i = (int)threadIdx.x;
    if (i < count) dst[i] = pack.r[i];
}

// Device address of the scratch array on `device`, which must be the current device.
int scratch_on(int device, ResizeRec **out)
{
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_scratch_of[device]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return PREP_E_HIP;
        }
        g_scratch_of[device] = static_cast<ResizeRec *>(p);
    }
    *out = g_scratch_of[device];
    return PREP_OK;
}

}  // namespace

}  // namespace prep

using namespace prep;

extern "C" int prep_resize_normalize_static(int32_t device, const uint8_t *rgb, const uint64_t *rgb_offsets,
                                            const int32_t *widths, const int32_t *heights,
                                            const int32_t *pitches, int32_t n, const prep_params *params,
                                            void *out, void *stream)
{
    if (device < 0 || device >= kMaxDevices || !rgb || !rgb_offsets || !widths || !heights || !pitches ||
        !out || n < 0 || !params_ok(params))
        return PREP_E_INVALID_ARG;
    if (n > PREP_STATIC_MAX_IMAGES) return PREP_E_TOO_LARGE;
    if (n == 0) return PREP_OK;
    // the host's copy of the records, on the stack (the antialiased filter deals the images
    // to its two launches by their scales)
    ResizeRec host_rr[PREP_STATIC_MAX_IMAGES];
    for (int32_t i = 0; i < n; i++) {
        if (widths[i] < 1 || heights[i] < 1 || widths[i] > 65535 || heights[i] > 65535 ||
            pitches[i] < widths[i] * 3)
            return PREP_E_INVALID_ARG;
        if (!make_resize_rec(widths[i], heights[i], params, rgb_offsets[i], (uint32_t)pitches[i], &host_rr[i]))
            return PREP_E_INVALID_ARG;
    }
    if (hipSetDevice(device) != hipSuccess) {
        (void)hipGetLastError();
        return PREP_E_HIP;
    }
    ResizeRec *d_rr = nullptr;
    const int rc = scratch_on(device, &d_rr);
    if (rc != PREP_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    for (int32_t at = 0; at < n; at += kPack) {
        RecPack pack;
        const int count = n - at < kPack ? n - at : kPack;
        for (int k = 0; k < count; k++) pack.r[k] = host_rr[at + k];
        for (int k = count; k < kPack; k++) pack.r[k] = host_rr[at];
        hipLaunchKernelGGL(store_resize_recs, dim3(1), dim3(64), 0, st, pack, d_rr + at, count);
    }
    launch_resize_normalize(rgb, d_rr, nullptr, n, params->crop_h, params->crop_w, params->out_dtype,
                            params->filter, host_rr, params->mean, params->std, out, false, st);
    if (hipGetLastError() != hipSuccess) return PREP_E_HIP;
    return PREP_OK;
}
