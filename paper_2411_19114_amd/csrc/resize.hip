// Resize (two-tap bilinear or antialiased) + centre crop + mean/std normalize -> planar NCHW,
// or without normalize -> 8-bit NHWC, fused (gfx950).
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
// 8-bit output: a resized sample (0 .. 255, no Normalize) to the nearest integer, halves
// upwards.  Exact halves are common (rational scales) and fp32 interpolation lands up to a few
// 1e-5 to either side of them, so a sample within 2^-12 below a half is taken for the half.
__device__ inline uint32_t to_byte(float v) { return min((uint32_t)(v + (0.5f + 1.0f / 4096.0f)), 255u); }

__device__ inline void store1(float *p, float v) { *p = v; }
__device__ inline void store1(__half *p, float v) { *p = __float2half_rn(v); }
__device__ inline void store1(uint8_t *p, float v) { *p = (uint8_t)to_byte(v); }

// Where channel 0 of output (img, y, x) goes and how far apart its channels are (*plane):
// planar [n][3][h][w], or interleaved [n][h][w][3] for the 8-bit output.
template <typename OutT>
__device__ inline OutT *output_at(OutT *out, int img, int y, int x, int crop_h, int crop_w, size_t *plane)
{
    const size_t in_image = (size_t)y * crop_w + x, image = (size_t)crop_h * crop_w;
    if (sizeof(OutT) == 1) {
        *plane = 1;
        return out + ((size_t)img * image + in_image) * 3;
    }
    *plane = image;
    return out + (size_t)img * 3 * image + in_image;
}

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
    size_t plane;
    OutT *o = output_at(out, img, y, x0, crop_h, crop_w, &plane);
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
    if constexpr (sizeof(OutT) == 1) {
        // kPx pixels = 12 adjacent bytes
        uint32_t b[3 * kPx];
#pragma unroll
        for (int j = 0; j < kPx; j++)
#pragma unroll
            for (int c = 0; c < 3; c++) b[3 * j + c] = to_byte(res[c][j]);
        if (vec) {
            uint32_t *w = reinterpret_cast<uint32_t *>(o);
#pragma unroll
            for (int k = 0; k < 3; k++)
                w[k] = b[4 * k] | (b[4 * k + 1] << 8) | (b[4 * k + 2] << 16) | (b[4 * k + 3] << 24);
        } else {
            for (int j = 0; j < 3 * nx; j++) o[j] = (uint8_t)b[j];
        }
    } else {
#pragma unroll
        for (int c = 0; c < 3; c++) {
            if (vec) {
                store_row(o + c * plane, res[c]);
            } else {
                for (int j = 0; j < nx; j++) store1(o + c * plane + j, res[c][j]);
            }
        }
    }
}

// ---- antialiased variant -------------------------------------------------------
//
// Where an axis shrinks, an output sample is the mean of the source samples under a triangle
// centred on it and as wide as an output sample (support = in / out source samples each way),
// the window cut at the image's edge and the weights scaled to sum 1: the resize of image
// libraries when they reduce.  Where an axis grows the support is one sample and this is the
// two-tap interpolation above.  (PREBA section 4.2 names the Resize unit and no filter.)

// The window of one output index along one axis and what its weights need.
struct Window {
    int first, end;  // source samples first .. end-1, inside the image
    int whole;       // floor of the output sample's source coordinate (centre - 1/2)
    float frac;      // and its fraction
    float inv;       // 1 / support
    __device__ __forceinline__ float weight(int j) const
    {
        return fmaxf(0.0f, fmaf(-fabsf((float)(j - whole) - frac), inv, 1.0f));
    }
};

__device__ __forceinline__ Window make_window(uint64_t off, uint64_t scale, int i, int size)
{
    const uint64_t one = 1ull << kCoordFrac;
    const uint64_t t = off + (uint64_t)(uint32_t)i * scale;
    const uint64_t support = scale > one ? scale : one;
    Window w;
    // floor(centre - support + 1/2) and floor(centre + support + 1/2) with centre - 1/2 = t
    w.first = max((int)((int64_t)(t + one - support) >> kCoordFrac) - kCoordBias, 0);
    w.end = min((int)((t + one + support) >> kCoordFrac) - kCoordBias, size);
    w.whole = (int)(t >> kCoordFrac) - kCoordBias;
    w.frac = (float)(uint32_t)(t & (one - 1)) * (1.0f / (float)(1u << kCoordFrac));
    w.inv = 1.0f / fmaxf(1.0f, (float)scale * (1.0f / (float)(1u << kCoordFrac)));
    return w;
}

// A pixel's three bytes as floats.  kWide: read as four bytes (the byte past the pixel is
// readable); otherwise the bytes are loaded singly.
template <bool kWide>
__device__ __forceinline__ void load_pixel(const uint8_t *p, float v[3])
{
    if (kWide) {
        uint32_t u;
        __builtin_memcpy(&u, p, 4);
        v[0] = (float)(u & 255u);
        v[1] = (float)((u >> 8) & 255u);
        v[2] = (float)((u >> 16) & 255u);
    } else {
#pragma unroll
        for (int c = 0; c < 3; c++) v[c] = (float)p[c];
    }
}

// One thread produces one output pixel of all 3 planes, a workgroup a tile of 64 x 4 outputs,
// a wave the 64 outputs of one row.  The outputs of a wave share their row window and their
// column windows overlap, so the wave first sums every source column under its triangles
// over the rows (weights from LDS, the columns dealt to the lanes: coalesced loads), then
// every lane sums its own columns from LDS: (64 s + 2 s) n + 64 n taps instead of 64 n^2 for
// n taps per axis.  That pays from reductions of about 2.5 times on (measured: full-HD frames
// to 384 rows 220 -> 181 us, photos reduced 1.2 to 2.5 times 125 -> 142 us: the set-up and the
// two barriers outweigh the fewer taps there), so smaller reductions, and tiles whose columns
// or rows do not fit the LDS arrays (reductions beyond about 7.5 times), take the direct
// double sum.
constexpr int kTileW = 64, kTileH = kResizeThreads / kTileW;
constexpr int kMaxCols = 512, kMaxRows = 64;
constexpr int kTwoPassRows = 7;  // row windows at least this tall: support of 2.5 samples or more

// Which of the two ways an image's tiles (the 64 x 4 outputs of a workgroup) are summed: columns
// first through LDS when its row windows are tall enough for that to pay and the rows and the
// columns of a tile fit the LDS arrays.  A property of the image's scales alone, so that the
// host knows which launches a batch needs.
__host__ __device__ inline bool sums_columns_first(const ResizeRec &R)
{
    const uint64_t one = 1ull << kCoordFrac;
    const uint64_t sup_x = R.scale_x > one ? R.scale_x : one, sup_y = R.scale_y > one ? R.scale_y : one;
    // the tallest row window (a window holds at most 2 support + 1 samples) and the most columns
    // under the triangles of 64 adjacent outputs
    const uint64_t ny_max = ((2 * sup_y) >> kCoordFrac) + 2;
    const uint64_t cols_max = (((kTileW - 1) * R.scale_x + 2 * sup_x) >> kCoordFrac) + 2;
    return ny_max >= (uint64_t)kTwoPassRows && ny_max <= (uint64_t)kMaxRows && cols_max <= (uint64_t)kMaxCols;
}

// kColumnsFirst: this launch does the images that sum their columns first and leaves the
// others to the launch with kColumnsFirst = false (which holds no LDS and so keeps more
// waves on a compute unit), and the other way round.
template <typename OutT, bool kWide, bool kColumnsFirst>
__global__ __launch_bounds__(kResizeThreads) void resize_antialias_crop_normalize(
    const uint8_t *__restrict__ rgb, const ResizeRec *__restrict__ rr,
    const int32_t *__restrict__ status, int crop_h, int crop_w, NormConst nc, OutT *__restrict__ out)
{
    const int img = blockIdx.z;
    const int lane = threadIdx.x % kTileW, wave = threadIdx.x / kTileW;
    const int x_first = blockIdx.x * kTileW;
    const int x = x_first + lane, y = blockIdx.y * kTileH + wave;
    const bool inside = x < crop_w && y < crop_h;
    float res[3] = {0.0f, 0.0f, 0.0f};
    // everything up to the stores is the same for all threads of the workgroup or of a wave
    // except what `inside` guards, so the barriers are reached by all or by none
    const ResizeRec R = rr[img];
    if (sums_columns_first(R) != kColumnsFirst) return;  // the other launch's image
    if (status == nullptr || status[img] == PREP_OK) {
        const uint8_t *src = rgb + R.src_off;
        const Window wx = make_window(R.off_x, R.scale_x, min(x, crop_w - 1), R.src_w);
        const Window wy = make_window(R.off_y, R.scale_y, min(y, crop_h - 1), R.src_h);
        const int nx = wx.end - wx.first, ny = wy.end - wy.first;
        const float dx0 = (float)(wx.first - wx.whole) - wx.frac;  // then one more per tap
        // the columns under the triangles of this tile's outputs (windows move right with x)
        const int c_lo = make_window(R.off_x, R.scale_x, x_first, R.src_w).first;
        const int c_hi = make_window(R.off_x, R.scale_x, min(x_first + kTileW, crop_w) - 1, R.src_w).end;
        if constexpr (kColumnsFirst) {
            __shared__ float column_sum[kTileH][3][kMaxCols];
            __shared__ float row_weight[kTileH][kMaxRows];
            // row weights, scaled to sum 1
            float sum_y = 0.0f;
            for (int j = wy.first; j < wy.end; j++) sum_y += wy.weight(j);
            for (int j = lane; j < ny; j += kTileW) row_weight[wave][j] = wy.weight(wy.first + j) / sum_y;
            __syncthreads();
            if (y < crop_h) {
                for (int c = c_lo + lane; c < c_hi; c += kTileW) {
                    const uint8_t *p = src + (size_t)wy.first * R.src_pitch + (size_t)c * 3;
                    float a[3] = {0.0f, 0.0f, 0.0f};
                    // two rows at a time, so that their loads are in flight together
                    for (int j = 0; j < ny; j += 2, p += 2 * (size_t)R.src_pitch) {
                        const bool two = j + 1 < ny;
                        float u[3], v[3];
                        load_pixel<kWide>(p, u);
                        load_pixel<kWide>(two ? p + R.src_pitch : p, v);  // a row of the window either way
                        const float w0 = row_weight[wave][j], w1 = two ? row_weight[wave][j + 1] : 0.0f;
#pragma unroll
                        for (int ch = 0; ch < 3; ch++) a[ch] = fmaf(w0, u[ch], fmaf(w1, v[ch], a[ch]));
                    }
#pragma unroll
                    for (int ch = 0; ch < 3; ch++) column_sum[wave][ch][c - c_lo] = a[ch];
                }
            }
            __syncthreads();
            if (inside) {
                float sum_x = 0.0f, acc[3] = {0.0f, 0.0f, 0.0f};
                const float *v = &column_sum[wave][0][wx.first - c_lo];
                float d = dx0;
                for (int k = 0; k < nx; k++, d += 1.0f) {
                    const float w = fmaxf(0.0f, fmaf(-fabsf(d), wx.inv, 1.0f));
                    sum_x += w;
#pragma unroll
                    for (int ch = 0; ch < 3; ch++) acc[ch] = fmaf(w, v[ch * kMaxCols + k], acc[ch]);
                }
                // a window holds at least the sample nearest to the centre, so the sum is positive
                const float norm = 1.0f / sum_x;
#pragma unroll
                for (int ch = 0; ch < 3; ch++) res[ch] = fmaf(acc[ch] * norm, nc.scale[ch], nc.bias[ch]);
            }
        } else if (inside) {
            float sum_x = 0.0f, sum_y = 0.0f;
            for (int j = wx.first; j < wx.end; j++) sum_x += wx.weight(j);
            for (int j = wy.first; j < wy.end; j++) sum_y += wy.weight(j);
            float acc[3] = {0.0f, 0.0f, 0.0f};
            // two rows at a time: one column weight serves both, and their loads are in
            // flight together
            for (int r = wy.first; r < wy.end; r += 2) {
                const bool two = r + 1 < wy.end;
                const uint8_t *p0 = src + (size_t)r * R.src_pitch + (size_t)wx.first * 3;
                const uint8_t *p1 = two ? p0 + R.src_pitch : p0;  // a row of the window either way
                float a[3] = {0.0f, 0.0f, 0.0f}, b[3] = {0.0f, 0.0f, 0.0f};
                float d = dx0;
                for (int k = 0; k < nx; k++, p0 += 3, p1 += 3, d += 1.0f) {
                    const float w = fmaxf(0.0f, fmaf(-fabsf(d), wx.inv, 1.0f));
                    float u[3], v[3];
                    load_pixel<kWide>(p0, u);
                    load_pixel<kWide>(p1, v);
#pragma unroll
                    for (int ch = 0; ch < 3; ch++) {
                        a[ch] = fmaf(w, u[ch], a[ch]);
                        b[ch] = fmaf(w, v[ch], b[ch]);
                    }
                }
                const float w0 = wy.weight(r), w1 = two ? wy.weight(r + 1) : 0.0f;
#pragma unroll
                for (int ch = 0; ch < 3; ch++) acc[ch] = fmaf(w0, a[ch], fmaf(w1, b[ch], acc[ch]));
            }
            const float norm = 1.0f / (sum_x * sum_y);
#pragma unroll
            for (int ch = 0; ch < 3; ch++) res[ch] = fmaf(acc[ch] * norm, nc.scale[ch], nc.bias[ch]);
        }
    }
    if (inside) {
        size_t plane;
        OutT *o = output_at(out, img, y, x, crop_h, crop_w, &plane);
#pragma unroll
        for (int ch = 0; ch < 3; ch++) store1(o + ch * plane, res[ch]);
    }
}

void resize_antialias_classes(const ResizeRec *rr, int n, bool *any_direct, bool *any_columns_first)
{
    *any_direct = *any_columns_first = false;
    for (int i = 0; i < n; i++) *(sums_columns_first(rr[i]) ? any_columns_first : any_direct) = true;
}

namespace {

// The launches of one output type.
template <typename OutT>
void launch_for(const uint8_t *rgb, const ResizeRec *rr, const int32_t *status, int n_images, int crop_h,
                int crop_w, int filter, const ResizeRec *host_rr, const NormConst &nc, OutT *out,
                bool wide_reads, hipStream_t stream)
{
    dim3 block(kResizeThreads);
    if (filter == PREP_FILTER_ANTIALIAS) {
        dim3 grid((crop_w + kTileW - 1) / kTileW, (crop_h + kTileH - 1) / kTileH, n_images);
        auto launch = [&](auto kernel) {
            hipLaunchKernelGGL(kernel, grid, block, 0, stream, rgb, rr, status, crop_h, crop_w, nc, out);
        };
        // every image is done by exactly one of the two launches
        bool direct, columns;
        resize_antialias_classes(host_rr, n_images, &direct, &columns);
        if (wide_reads) {
            if (direct) launch(resize_antialias_crop_normalize<OutT, true, false>);
            if (columns) launch(resize_antialias_crop_normalize<OutT, true, true>);
        } else {
            if (direct) launch(resize_antialias_crop_normalize<OutT, false, false>);
            if (columns) launch(resize_antialias_crop_normalize<OutT, false, true>);
        }
        return;
    }
    const int groups = (crop_w + kPx - 1) / kPx;
    const int items = groups * crop_h;
    // vector stores need every group of kPx outputs to start 16-byte aligned (4-byte aligned
    // for the 8-bit output, which the same test covers)
    const int vec_ok = crop_w % kPx == 0 && ((uintptr_t)out & 15u) == 0;
    dim3 grid((items + kResizeThreads - 1) / kResizeThreads, n_images);
    if (wide_reads)
        hipLaunchKernelGGL((resize_crop_normalize<OutT, true>), grid, block, 0, stream, rgb, rr, status,
                           crop_h, crop_w, vec_ok, nc, out);
    else
        hipLaunchKernelGGL((resize_crop_normalize<OutT, false>), grid, block, 0, stream, rgb, rr, status,
                           crop_h, crop_w, vec_ok, nc, out);
}

}  // namespace

void launch_resize_normalize(const uint8_t *rgb, const ResizeRec *rr, const int32_t *status,
                             int n_images, int crop_h, int crop_w, int out_dtype, int filter,
                             const ResizeRec *host_rr, const float mean[3], const float std[3], void *out,
                             bool wide_reads, hipStream_t stream)
{
    if (n_images <= 0) return;
    NormConst nc;
    for (int c = 0; c < 3; c++) {
        // the 8-bit output is the resized sample itself
        nc.scale[c] = out_dtype == PREP_U8_NHWC ? 1.0f : (float)(1.0 / (255.0 * (double)std[c]));
        nc.bias[c] = out_dtype == PREP_U8_NHWC ? 0.0f : (float)(-(double)mean[c] / (double)std[c]);
    }
    if (out_dtype == PREP_F16)
        launch_for(rgb, rr, status, n_images, crop_h, crop_w, filter, host_rr, nc, (__half *)out, wide_reads, stream);
    else if (out_dtype == PREP_U8_NHWC)
        launch_for(rgb, rr, status, n_images, crop_h, crop_w, filter, host_rr, nc, (uint8_t *)out, wide_reads, stream);
    else
        launch_for(rgb, rr, status, n_images, crop_h, crop_w, filter, host_rr, nc, (float *)out, wide_reads, stream);
}

}  // namespace prep
