// Bilinear resize + centre crop + mean/std normalize -> planar NCHW, fused (gfx950).
//
// The Resize, Crop and Normalize functional units of the image CU (PREBA
// section 4.2, Table 1), streamed through one kernel as the paper streams them
// through FIFOs: no resized image is ever materialised.  Pixel centres sit at
// half-integers, the two scales are in/out per axis, taps are clamped at the
// border, nothing is rounded before the final cast.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/prep.h"
#include "kernels.h"
#include "prep_internal.h"

namespace prep {

namespace {

constexpr int kResizeThreads = 256;

struct NormConst {
    float scale[3];  // 1 / (255 std)
    float bias[3];   // -mean / std
};

__device__ inline void store4(float *p, const float v[4])
{
    *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
__device__ inline void store4(__half *p, const float v[4])
{
    __half2 a = __floats2half2_rn(v[0], v[1]);
    __half2 b = __floats2half2_rn(v[2], v[3]);
    uint2 u;
    u.x = *reinterpret_cast<uint32_t *>(&a);
    u.y = *reinterpret_cast<uint32_t *>(&b);
    *reinterpret_cast<uint2 *>(p) = u;
}
__device__ inline void store1(float *p, float v) { *p = v; }
__device__ inline void store1(__half *p, float v) { *p = __float2half_rn(v); }

}  // namespace

// One thread produces 4 horizontally adjacent output pixels of all 3 planes.
template <typename OutT>
__global__ __launch_bounds__(kResizeThreads) void resize_crop_normalize(
    const uint8_t *__restrict__ rgb, const ResizeRec *__restrict__ rr,
    const int32_t *__restrict__ status, int crop_h, int crop_w, NormConst nc,
    OutT *__restrict__ out)
{
    const int img = blockIdx.y;
    const int quads = (crop_w + 3) >> 2;
    const int item = blockIdx.x * kResizeThreads + threadIdx.x;
    if (item >= quads * crop_h) return;
    const int y = item / quads, x0 = (item - y * quads) * 4;
    const int nx = min(4, crop_w - x0);
    const size_t plane = (size_t)crop_h * crop_w;
    OutT *o = out + (size_t)img * 3 * plane + (size_t)y * crop_w + x0;
    // 4-wide stores need the plane row start to keep their alignment
    const bool vec = nx == 4 && (crop_w & 3) == 0;
    float res[3][4];
    const bool ok = status == nullptr || status[img] == PREP_OK;
    if (!ok) {
#pragma unroll
        for (int c = 0; c < 3; c++)
#pragma unroll
            for (int j = 0; j < 4; j++) res[c][j] = 0.0f;
    } else {
        const ResizeRec R = rr[img];
        const uint8_t *src = rgb + R.src_off;
        // source coordinates in double: a float has too few bits left at x ~ 2000
        const double sy = fma((double)y, R.scale_y, R.off_y);
        const double fy0 = floor(sy);
        const float fy = (float)(sy - fy0);
        const int ya = min(max((int)fy0, 0), R.src_h - 1), yb = min(max((int)fy0 + 1, 0), R.src_h - 1);
        const uint8_t *ra = src + (size_t)ya * R.src_pitch, *rb = src + (size_t)yb * R.src_pitch;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const double sx = fma((double)(x0 + j), R.scale_x, R.off_x);
            const double fx0 = floor(sx);
            const float fx = (float)(sx - fx0);
            const int xa = min(max((int)fx0, 0), R.src_w - 1) * 3;
            const int xb = min(max((int)fx0 + 1, 0), R.src_w - 1) * 3;
#pragma unroll
            for (int c = 0; c < 3; c++) {
                const float p00 = ra[xa + c], p01 = ra[xb + c], p10 = rb[xa + c], p11 = rb[xb + c];
                const float top = fmaf(fx, p01 - p00, p00), bot = fmaf(fx, p11 - p10, p10);
                const float v = fmaf(fy, bot - top, top);
                res[c][j] = fmaf(v, nc.scale[c], nc.bias[c]);
            }
        }
    }
#pragma unroll
    for (int c = 0; c < 3; c++) {
        if (vec) {
            store4(o + c * plane, res[c]);
        } else {
            for (int j = 0; j < nx; j++) store1(o + c * plane + j, res[c][j]);
        }
    }
}

void launch_resize_normalize(const uint8_t *rgb, const ResizeRec *rr, const int32_t *status,
                             int n_images, int crop_h, int crop_w, int out_dtype,
                             const float mean[3], const float std[3], void *out,
                             hipStream_t stream)
{
    if (n_images <= 0) return;
    NormConst nc;
    for (int c = 0; c < 3; c++) {
        nc.scale[c] = (float)(1.0 / (255.0 * (double)std[c]));
        nc.bias[c] = (float)(-(double)mean[c] / (double)std[c]);
    }
    const int quads = (crop_w + 3) >> 2;
    const int items = quads * crop_h;
    dim3 grid((items + kResizeThreads - 1) / kResizeThreads, n_images);
    if (out_dtype == PREP_F16)
        hipLaunchKernelGGL(resize_crop_normalize<__half>, grid, dim3(kResizeThreads), 0, stream, rgb,
                           rr, status, crop_h, crop_w, nc, (__half *)out);
    else
        hipLaunchKernelGGL(resize_crop_normalize<float>, grid, dim3(kResizeThreads), 0, stream, rgb,
                           rr, status, crop_h, crop_w, nc, (float *)out);
}

}  // namespace prep
