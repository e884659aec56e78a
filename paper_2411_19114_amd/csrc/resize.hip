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

constexpr int kPx = 4;  // horizontally adjacent outputs per thread

// kPx adjacent outputs of one plane row as one vector store (p is 16-byte aligned for
// float, 8-byte aligned for half)
__device__ inline void store_row(float *p, const float v[kPx])
{
    *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
__device__ inline void store_row(__half *p, const float v[kPx])
{
    __half2 a = __floats2half2_rn(v[0], v[1]);
    __half2 b = __floats2half2_rn(v[2], v[3]);
    uint2 u;
    u.x = *reinterpret_cast<uint32_t *>(&a);
    u.y = *reinterpret_cast<uint32_t *>(&b);
    *reinterpret_cast<uint2 *>(p) = u;
}
static_assert(kPx == 4, "store_row writes four values");
__device__ inline void store1(float *p, float v) { *p = v; }
__device__ inline void store1(__half *p, float v) { *p = __float2half_rn(v); }

}  // namespace

// Source coordinate of output index i: integer part (may be -1 at the border) and fraction.
__device__ __forceinline__ void map_coord(uint64_t off, uint64_t scale, int i, int *whole, float *frac)
{
    const uint64_t t = off + (uint64_t)(uint32_t)i * scale;
    *whole = (int)(t >> kCoordFrac) - kCoordBias;
    *frac = (float)(uint32_t)(t & ((1ull << kCoordFrac) - 1)) * (1.0f / (float)(1u << kCoordFrac));
}

// Two horizontally adjacent RGB pixels (6 bytes) starting at p, as one 8-byte load.  The
// address has no alignment; the two bytes past the pixels must be readable.
__device__ __forceinline__ uint2 load_pixel_pair(const uint8_t *p)
{
    uint2 v;
    __builtin_memcpy(&v, p, 8);
    return v;
}

// channel c of the left (i = 0) or right (i = 1) pixel of a pair
__device__ __forceinline__ float pair_channel(const uint2 v, int i, int c)
{
    const int b = 3 * i + c;  // byte index 0..5
    const uint32_t w = b < 4 ? v.x : v.y;
    return (float)((w >> (8 * (b & 3))) & 255u);
}

// One thread produces kPx horizontally adjacent output pixels of all 3 planes.
// kWide: the source rows may be read two bytes past a pixel pair (true for the library's
// own RGB workspace, which keeps slack after every image); otherwise bytes are loaded singly.
template <typename OutT, bool kWide>
__global__ __launch_bounds__(kResizeThreads) void resize_crop_normalize(
    const uint8_t *__restrict__ rgb, const ResizeRec *__restrict__ rr,
    const int32_t *__restrict__ status, int crop_h, int crop_w, int vec_ok, NormConst nc,
    OutT *__restrict__ out)
{
    const int img = blockIdx.y;
    const int groups = (crop_w + kPx - 1) / kPx;
    const int item = blockIdx.x * kResizeThreads + threadIdx.x;
    if (item >= groups * crop_h) return;
    const int y = item / groups, x0 = (item - y * groups) * kPx;
    const int nx = min(kPx, crop_w - x0);
    const size_t plane = (size_t)crop_h * crop_w;
    OutT *o = out + (size_t)img * 3 * plane + (size_t)y * crop_w + x0;
    const bool vec = nx == kPx && vec_ok;
    float res[3][kPx];
    const bool ok = status == nullptr || status[img] == PREP_OK;
    if (!ok) {
#pragma unroll
        for (int c = 0; c < 3; c++)
#pragma unroll
            for (int j = 0; j < kPx; j++) res[c][j] = 0.0f;
    } else {
        const ResizeRec R = rr[img];
        const uint8_t *src = rgb + R.src_off;
        // source coordinates in 64-bit fixed point: a float has too few bits left at x ~ 2000
        int iy;
        float fy;
        map_coord(R.off_y, R.scale_y, y, &iy, &fy);
        const int ya = min(max(iy, 0), R.src_h - 1), yb = min(max(iy + 1, 0), R.src_h - 1);
        const uint8_t *ra = src + (size_t)ya * R.src_pitch, *rb = src + (size_t)yb * R.src_pitch;
#pragma unroll
        for (int j = 0; j < kPx; j++) {
            int ix;
            float fx;
            map_coord(R.off_x, R.scale_x, x0 + j, &ix, &fx);
            const int xa = min(max(ix, 0), R.src_w - 1);
            const int xb = min(max(ix + 1, 0), R.src_w - 1);
            if (kWide) {
                // the right tap is the next pixel except where clamping makes both taps one pixel
                const int right = xb != xa;
                const uint2 a = load_pixel_pair(ra + xa * 3), b = load_pixel_pair(rb + xa * 3);
#pragma unroll
                for (int c = 0; c < 3; c++) {
                    const float p00 = pair_channel(a, 0, c), p01 = right ? pair_channel(a, 1, c) : p00;
                    const float p10 = pair_channel(b, 0, c), p11 = right ? pair_channel(b, 1, c) : p10;
                    const float top = fmaf(fx, p01 - p00, p00), bot = fmaf(fx, p11 - p10, p10);
                    res[c][j] = fmaf(fmaf(fy, bot - top, top), nc.scale[c], nc.bias[c]);
                }
            } else {
#pragma unroll
                for (int c = 0; c < 3; c++) {
                    const float p00 = ra[xa * 3 + c], p01 = ra[xb * 3 + c];
                    const float p10 = rb[xa * 3 + c], p11 = rb[xb * 3 + c];
                    const float top = fmaf(fx, p01 - p00, p00), bot = fmaf(fx, p11 - p10, p10);
                    res[c][j] = fmaf(fmaf(fy, bot - top, top), nc.scale[c], nc.bias[c]);
                }
            }
        }
    }
#pragma unroll
    for (int c = 0; c < 3; c++) {
        if (vec) {
            store_row(o + c * plane, res[c]);
        } else {
            for (int j = 0; j < nx; j++) store1(o + c * plane + j, res[c][j]);
        }
    }
}

void launch_resize_normalize(const uint8_t *rgb, const ResizeRec *rr, const int32_t *status,
                             int n_images, int crop_h, int crop_w, int out_dtype,
                             const float mean[3], const float std[3], void *out, bool wide_reads,
                             hipStream_t stream)
{
    if (n_images <= 0) return;
    NormConst nc;
    for (int c = 0; c < 3; c++) {
        nc.scale[c] = (float)(1.0 / (255.0 * (double)std[c]));
        nc.bias[c] = (float)(-(double)mean[c] / (double)std[c]);
    }
    const int groups = (crop_w + kPx - 1) / kPx;
    const int items = groups * crop_h;
    // vector stores need every group of kPx outputs to start 16-byte aligned
    const int vec_ok = crop_w % kPx == 0 && ((uintptr_t)out & 15u) == 0;
    dim3 grid((items + kResizeThreads - 1) / kResizeThreads, n_images);
    dim3 block(kResizeThreads);
    if (out_dtype == PREP_F16) {
        if (wide_reads)
            hipLaunchKernelGGL((resize_crop_normalize<__half, true>), grid, block, 0, stream, rgb, rr,
                               status, crop_h, crop_w, vec_ok, nc, (__half *)out);
        else
            hipLaunchKernelGGL((resize_crop_normalize<__half, false>), grid, block, 0, stream, rgb, rr,
                               status, crop_h, crop_w, vec_ok, nc, (__half *)out);
    } else {
        if (wide_reads)
            hipLaunchKernelGGL((resize_crop_normalize<float, true>), grid, block, 0, stream, rgb, rr,
                               status, crop_h, crop_w, vec_ok, nc, (float *)out);
        else
            hipLaunchKernelGGL((resize_crop_normalize<float, false>), grid, block, 0, stream, rgb, rr,
                               status, crop_h, crop_w, vec_ok, nc, (float *)out);
    }
}

}  // namespace prep
