// Dequantise + 8x8 inverse DCT + chroma upsampling + YCbCr->RGB, fused (gfx950).
//
// The second half of the "Decode" functional unit (PREBA section 4.2, Table 1):
// T.81 A.3.4 (dequantisation, zig-zag), A.3.3 (IDCT), A.3.1 (level shift),
// sample replication for subsampled chroma (or, as a variant, interpolation under a centred
// triangle by a second kernel), JFIF colour transform.  One
// workgroup handles a run of MCUs of one MCU row: coefficients are read once
// (128 B per block), everything else lives in LDS, and RGB leaves as aligned
// 32-bit stores covering the whole MCU grid (the row pitch includes padding).
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/prep.h"
#include "kernels.h"
#include "prep_internal.h"

namespace prep {

namespace {

constexpr int kTileStride = 9;               // doubles per tile row: spreads rows over LDS banks
constexpr int kTileSize = 8 * kTileStride;   // one 8x8 block
constexpr int kLumaPitch = 256;              // bytes per row of the luma sample plane
constexpr int kChromaPitch = 96;

// zig-zag position k -> natural index v*8+u (T.81 Figure A.6), found by walking
// the anti-diagonals alternately down-left and up-right
struct ZigZag {
    uint8_t nat[64];
    constexpr ZigZag() : nat()
    {
        int v = 0, u = 0;
        for (int k = 0; k < 64; k++) {
            nat[k] = (uint8_t)(v * 8 + u);
            if (((v + u) & 1) == 0) {          // moving up-right
                if (u == 7) v++;
                else if (v == 0) u++;
                else { v--; u++; }
            } else {                           // moving down-left
                if (v == 7) u++;
                else if (u == 0) v++;
                else { v++; u--; }
            }
        }
    }
};

// for column u, the zig-zag positions of its eight coefficients F(v, u), v = 0..7, packed a
// byte each: lane u of a block fetches them in one 8-byte load
struct ZigZagColumns {
    unsigned long long pos[8];
    constexpr ZigZagColumns() : pos()
    {
        ZigZag z;
        for (int k = 0; k < 64; k++) {
            const int v = z.nat[k] >> 3, u = z.nat[k] & 7;
            pos[u] |= (unsigned long long)k << (8 * v);
        }
    }
};
__device__ const ZigZagColumns kZigZagColumns{};

// 8-point inverse DCT with basis m(x,0) = 1, m(x,u) = sqrt(2) cos((2x+1) u pi/16):
// the 2-D result still needs a factor 1/8.  Even and odd frequencies are summed
// separately because the odd basis is antisymmetric about the centre.
//
// Double precision on purpose: a decoded sample is rounded to 8 bits and a chroma
// sample that rounds the other way moves blue by two levels after colour
// conversion.  With ~1e-13 of evaluation noise only samples that the definition
// puts exactly half way can flip, and those are settled by kTieEps below.  With
// this basis m(x,4) = +-1 exactly, so DC-only and DC+F(.,4) blocks are exact.
__device__ inline void idct8(const double F[8], double out[8])
{
    constexpr double c1 = 1.3870398453221475, c2 = 1.3065629648763766, c3 = 1.1758756024193588,
                     c5 = 0.7856949583871022, c6 = 0.5411961001461970, c7 = 0.2758993792829431;
    const double a = F[0] + F[4], b = F[0] - F[4];
    const double e0 = a + (c2 * F[2] + c6 * F[6]);
    const double e3 = a - (c2 * F[2] + c6 * F[6]);
    const double e1 = b + (c6 * F[2] - c2 * F[6]);
    const double e2 = b - (c6 * F[2] - c2 * F[6]);
    const double o0 = c1 * F[1] + c3 * F[3] + c5 * F[5] + c7 * F[7];
    const double o1 = c3 * F[1] - c7 * F[3] - c1 * F[5] - c5 * F[7];
    const double o2 = c5 * F[1] - c1 * F[3] + c7 * F[5] + c3 * F[7];
    const double o3 = c7 * F[1] - c5 * F[3] + c3 * F[5] - c1 * F[7];
    out[0] = e0 + o0; out[7] = e0 - o0;
    out[1] = e1 + o1; out[6] = e1 - o1;
    out[2] = e2 + o2; out[5] = e2 - o2;
    out[3] = e3 + o3; out[4] = e3 - o3;
}

// Samples closer than this below a half-way point count as half way and round up:
// rational results of the IDCT definition carry ~1e-13 of evaluation noise.
constexpr double kTieEps = 1.0 / 1048576.0;

// One colour value -> byte `lane` of `word`: round to nearest, clamp to 0..255, in one
// conversion instruction.  It rounds exact half-way values to even, where the rounding of
// T.81 A.3.1 (used for the colour conversion too) goes up; see chroma_terms.
__device__ inline uint32_t put_u8(float v, uint32_t lane, uint32_t word)
{
    return __builtin_amdgcn_cvt_pk_u8_f32(v, lane, word);
}

// JFIF colour values are sums of an integer and one or two products of small integers with
// three- or six-decimal constants, so single precision decides the rounding wherever a value
// is not within ~1e-5 of a half-way point.  Exactly half way lie: red never (1.402 Cr has no
// fraction .5 for |Cr| <= 128); blue for Cb = +-125 only (1.772 * 125 = 221.5), and its
// fractions are multiples of .004, so adding .001 to the blue term turns round-to-nearest
// into round-half-up without moving any other value across a half-way point; green for
// (Cb, Cr) = (+-50, -+50), with fractions too fine for such a shift, so green is rounded as
// floor(value + 1/2) before the conversion, which then only clamps and packs.
struct ChromaTerms {
    float r, g, b;  // 1.402 Cr, -0.344136 Cb - 0.714136 Cr + .5, 1.772 Cb + .001 (Cb, Cr less 128)
};
__device__ inline ChromaTerms chroma_terms(uint32_t cb_byte, uint32_t cr_byte)
{
    const float cb = (float)((int)cb_byte - 128), cr = (float)((int)cr_byte - 128);
    ChromaTerms t;
    t.r = 1.402f * cr;
    t.g = fmaf(-0.714136f, cr, fmaf(-0.344136f, cb, 0.5f));
    t.b = fmaf(1.772f, cb, 0.001f);
    return t;
}
// Four pixels of one row -> twelve bytes R G B R G B ... as three words; pixel j has luma byte
// j of y4 and the chroma terms t[j].  Every value is converted straight into its byte.
__device__ inline void store_rgb4(uint8_t *dst, uint32_t y4, const ChromaTerms &t0, const ChromaTerms &t1,
                                  const ChromaTerms &t2, const ChromaTerms &t3)
{
    const float y0 = (float)(y4 & 255u), y1 = (float)((y4 >> 8) & 255u);
    const float y2 = (float)((y4 >> 16) & 255u), y3 = (float)(y4 >> 24);
    uint32_t d0 = 0, d1 = 0, d2 = 0;
    d0 = put_u8(y0 + t0.r, 0, d0); d0 = put_u8(floorf(y0 + t0.g), 1, d0); d0 = put_u8(y0 + t0.b, 2, d0);
    d0 = put_u8(y1 + t1.r, 3, d0); d1 = put_u8(floorf(y1 + t1.g), 0, d1); d1 = put_u8(y1 + t1.b, 1, d1);
    d1 = put_u8(y2 + t2.r, 2, d1); d1 = put_u8(floorf(y2 + t2.g), 3, d1); d2 = put_u8(y2 + t2.b, 0, d2);
    d2 = put_u8(y3 + t3.r, 1, d2); d2 = put_u8(floorf(y3 + t3.g), 2, d2); d2 = put_u8(y3 + t3.b, 3, d2);
    uint32_t *d = reinterpret_cast<uint32_t *>(dst);
    d[0] = d0;
    d[1] = d1;
    d[2] = d2;
}
// four gray pixels: every byte of y4 three times
__device__ inline void store_gray4(uint8_t *dst, uint32_t y4)
{
    const uint32_t a = y4 & 255u, b = (y4 >> 8) & 255u, c = (y4 >> 16) & 255u, e = y4 >> 24;
    uint32_t *d = reinterpret_cast<uint32_t *>(dst);
    d[0] = a * 0x010101u | (b << 24);
    d[1] = b * 0x0101u | (c * 0x0101u << 16);
    d[2] = c | (e * 0x010101u << 8);
}

}  // namespace

// A group's raw coefficients land in LDS block by block, 64 in zig-zag order, kRawPitch
// int16 apart: 72 = 36 words keeps the 16-byte stores aligned and puts the blocks of a wave
// four banks apart, so that lanes of different blocks reading the same zig-zag position do
// not meet in one bank.
constexpr int kRawPitch = 72;

struct ReconShared {
    double tile[kReconBlocks * kTileSize];
    int32_t qi[3][64];
    // the sample planes, luma first; free between a group's colour conversion and the next
    // group's row pass, which is when the raw coefficients use the same bytes
    uint32_t luma[16 * kLumaPitch / 4];
    uint32_t chroma[2][8 * kChromaPitch / 4];
};
static_assert(offsetof(ReconShared, chroma) == offsetof(ReconShared, luma) + sizeof(uint32_t) * 16 * kLumaPitch / 4,
              "the chroma planes follow the luma plane");
static_assert(kReconBlocks * kRawPitch * sizeof(int16_t) <=
                  sizeof(uint32_t) * (16 * kLumaPitch / 4 + 2 * 8 * kChromaPitch / 4),
              "the raw coefficients fit in the sample planes");

// Where the interpolating variant keeps an image's chroma samples between its two kernels:
// two planes of (8 mcu_cols) x (8 mcu_rows) bytes, Cb then Cr, in a workspace that mirrors the
// RGB workspace at a third of its offsets (a subsampled image has at most half as many chroma
// samples as pixels, and its RGB rows take three bytes per pixel).
struct ChromaPlanes {
    size_t off, plane;
    uint32_t pitch;
};
__device__ inline ChromaPlanes chroma_planes_of(const ImageRec &R)
{
    ChromaPlanes c;
    c.off = (size_t)(R.rgb_off / 12u) * 4u;
    c.pitch = (uint32_t)R.mcu_cols * 8u;
    c.plane = (size_t)c.pitch * R.mcu_rows * 8u;
    return c;
}

// The work of one workgroup: groups gi0 .. gi0 + n_groups - 1 of one image (a group is a run
// of MCUs of one MCU row, numbered row by row), one after the other.  The sampling mode is
// a compile-time constant so that every block / pixel index is divided by constants.
//
// A group's time is mostly the latency of its coefficient loads, and LDS limits a compute
// unit to six workgroups, so the coefficients of the next group are fetched into registers
// while the current one is transformed and converted.
//
// kPlanes (the interpolating variant, subsampled images only): the colour step is left to
// interpolate_chroma_rgb.  The group writes its luma as gray pixels and its chroma samples
// into the image's two chroma planes in chroma_all.
template <int sampling, bool kPlanes>
__device__ __forceinline__ void reconstruct_groups(ReconShared &S, const uint8_t *__restrict__ bits,
                                                   const ImageRec &R, uint32_t gi0, uint32_t n_groups,
                                                   const int16_t *__restrict__ coef_all,
                                                   uint8_t *__restrict__ rgb_all,
                                                   uint8_t *__restrict__ chroma_all)
{
    double *tile = S.tile;
    int32_t (*qi)[64] = S.qi;
    uint32_t *luma = S.luma;
    uint32_t (*chroma)[8 * kChromaPitch / 4] = S.chroma;
    const int tid = threadIdx.x;
    constexpr int bpm = blocks_per_mcu_of(sampling);
    constexpr int hs = luma_h(sampling), vs = luma_v(sampling);  // luma blocks per MCU along x, y
    constexpr int n_luma = hs * vs;
    constexpr int per_group = recon_mcus_per_group(sampling);
    static_assert(per_group * 8 * hs <= kLumaPitch && 8 * vs <= 16, "a group's luma fits its plane");
    static_assert(bpm == 1 || per_group * 8 <= kChromaPitch, "a group's chroma fits its plane");

    const uint8_t *file = bits + R.file_off;
    if (tid < 192) qi[tid >> 6][tid & 63] = (int32_t)file[R.dqt_off[tid >> 6] + (tid & 63)];

    const int b = tid >> 3, l = tid & 7;
    const int mcu = b / bpm, blk = b % bpm;  // of the lane's block, if the group has that many
    const int comp = blk < n_luma ? 0 : blk - n_luma + 1;
    double *T = tile + b * kTileSize;
    // the sample planes double as the landing place of a group's raw coefficients: they are
    // free until the row pass
    int16_t *zz16 = reinterpret_cast<int16_t *>(luma);
    const unsigned long long pos = kZigZagColumns.pos[l];
    // the lane's column of its component's quantisation table, kept for all groups
    __syncthreads();
    int32_t qcol[8];
#pragma unroll
    for (int v = 0; v < 8; v++) qcol[v] = qi[comp][(int)((pos >> (8 * v)) & 63u)];

    // groups are numbered row by row inside the image's region of interest
    const uint32_t gcol_end = (uint32_t)R.roi_gcol0 + R.roi_gcols;
    uint32_t mrow = gi0 / R.roi_gcols, gcol = gi0 - mrow * R.roi_gcols;
    mrow += R.roi_row0;
    gcol += R.roi_gcol0;
    // the lane's eight coefficients of group (mrow, gcol), or zeros past the group's blocks
    auto fetch = [&](uint32_t row, uint32_t col) {
        const uint32_t x0 = col * per_group;
        const int count = min(per_group, (int)R.mcu_cols - (int)x0);
        if (b >= count * bpm) return make_uint4(0, 0, 0, 0);
        const size_t gb = (size_t)R.coef_block0 + ((size_t)row * R.mcu_cols + x0 + mcu) * bpm + blk;
        return *reinterpret_cast<const uint4 *>(coef_all + gb * 64 + l * 8);
    };
    uint4 raw = fetch(mrow, gcol);
    for (uint32_t g = 0; g < n_groups; g++) {
        const uint32_t mcu_x0 = gcol * per_group;
        const int gcount = min(per_group, (int)R.mcu_cols - (int)mcu_x0);
        const bool have = b < gcount * bpm;  // <= kReconBlocks blocks
        if (have) *reinterpret_cast<uint4 *>(zz16 + b * kRawPitch + l * 8) = raw;
        __syncthreads();
        // next group of this workgroup, row by row
        uint32_t next_row = mrow, next_col = gcol + 1;
        if (next_col == gcol_end) { next_col = R.roi_gcol0; next_row++; }
        // ---- columns: lane l gathers column u = l through the zig-zag (A.3.4), dequantises
        // and transforms it ----------------------------------------------------------------
        if (have) {
            double F[8], o[8];
#pragma unroll
            for (int v = 0; v < 8; v++) {
                const int k = (int)((pos >> (8 * v)) & 63u);
                F[v] = (double)__mul24((int)zz16[b * kRawPitch + k], qcol[v]);  // 16 x 8 bits: exact
            }
            idct8(F, o);
#pragma unroll
            for (int y = 0; y < 8; y++) T[y * kTileStride + l] = o[y];
        }
        if (g + 1 < n_groups) raw = fetch(next_row, next_col);
        __syncthreads();
        // ---- rows: lane l transforms row y = l, level shift, round, clamp (A.3.1) ---------
        if (have) {
            double F[8], o[8];
#pragma unroll
            for (int u = 0; u < 8; u++) F[u] = T[l * kTileStride + u];
            idct8(F, o);
            uint32_t pk[2] = {0, 0};
#pragma unroll
            for (int x = 0; x < 8; x++) {
                // level shift and round half up; truncation instead of floor differs only below
                // zero, where both clamp to 0
                const int sample = (int)fma(o[x], 0.125, 128.5 + kTieEps);
                pk[x >> 2] |= (uint32_t)min(max(sample, 0), 255) << (8 * (x & 3));
            }
            if (comp == 0) {
                const int bx = blk % hs, by = blk / hs;  // luma blocks of an MCU run row by row (A.2.3)
                const int row = by * 8 + l, col = (mcu * hs + bx) * 8;
                luma[(row * kLumaPitch + col) / 4] = pk[0];
                luma[(row * kLumaPitch + col) / 4 + 1] = pk[1];
            } else {
                chroma[comp - 1][(l * kChromaPitch + mcu * 8) / 4] = pk[0];
                chroma[comp - 1][(l * kChromaPitch + mcu * 8) / 4 + 1] = pk[1];
            }
        }
        __syncthreads();
        // ---- colour ---------------------------------------------------------------------------
        const int rows = 8 * vs, width = gcount * 8 * hs, quads = width >> 2;
        uint8_t *dst0 = rgb_all + R.rgb_off + (size_t)mrow * rows * R.rgb_pitch +
                        (size_t)mcu_x0 * 8 * hs * 3;
        if (sampling == PREP_SAMPLING_GRAY || kPlanes) {
            // an item is 4 pixels of one row
            const int items = rows * quads;
            for (int it = tid; it < items; it += kReconThreads) {
                const int row = it / quads, q = it - row * quads;
                store_gray4(dst0 + (size_t)row * R.rgb_pitch + q * 12, luma[(row * kLumaPitch) / 4 + q]);
            }
            if (kPlanes) {
                // the group's 8 rows of gcount * 8 samples of each chroma plane, a word per item
                const ChromaPlanes cp = chroma_planes_of(R);
                const int words = gcount * 2;
                for (int it = tid; it < 2 * 8 * words; it += kReconThreads) {
                    const int c = it / (8 * words), r = (it / words) & 7, wd = it % words;
                    uint8_t *dst = chroma_all + cp.off + (size_t)c * cp.plane +
                                   (size_t)(mrow * 8u + (uint32_t)r) * cp.pitch + mcu_x0 * 8u + (uint32_t)wd * 4u;
                    *reinterpret_cast<uint32_t *>(dst) = chroma[c][(r * kChromaPitch) / 4 + wd];
                }
            }
        } else {
            // an item is 4 pixels of vs rows: the pixels that 4 / hs chroma samples of one chroma
            // row serve, so the terms of a chroma sample are formed once for all of them
            const int items = (rows / vs) * quads;
            for (int it = tid; it < items; it += kReconThreads) {
                const int rp = it / quads, q = it - rp * quads;
                ChromaTerms t[4];
                if (hs == 2) {
                    const uint16_t *cb16 = reinterpret_cast<const uint16_t *>(chroma[0]);
                    const uint16_t *cr16 = reinterpret_cast<const uint16_t *>(chroma[1]);
                    const uint32_t cbp = cb16[(rp * kChromaPitch) / 2 + q], crp = cr16[(rp * kChromaPitch) / 2 + q];
                    t[0] = t[1] = chroma_terms(cbp & 255u, crp & 255u);
                    t[2] = t[3] = chroma_terms(cbp >> 8, crp >> 8);
                } else {
                    const uint32_t cb4 = chroma[0][(rp * kChromaPitch) / 4 + q];
                    const uint32_t cr4 = chroma[1][(rp * kChromaPitch) / 4 + q];
#pragma unroll
                    for (int j = 0; j < 4; j++) t[j] = chroma_terms((cb4 >> (8 * j)) & 255u, (cr4 >> (8 * j)) & 255u);
                }
#pragma unroll
                for (int r = 0; r < vs; r++) {
                    const int row = vs * rp + r;
                    store_rgb4(dst0 + (size_t)row * R.rgb_pitch + q * 12, luma[(row * kLumaPitch) / 4 + q],
                               t[0], t[1], t[2], t[3]);
                }
            }
        }
        mrow = next_row;
        gcol = next_col;
        __syncthreads();  // the sample planes are free again
    }
}

// group0[i] = first workgroup of image i (ascending); a workgroup takes groups_per_wg
// consecutive groups of its image.  The image of workgroup wg is the last one whose entry
// does not exceed wg: every lane tests one entry and the hits are counted.
template <bool kPlanes>
__global__ __launch_bounds__(kReconThreads) void reconstruct_rgb(
    const uint8_t *__restrict__ bits, const ImageRec *__restrict__ recs,
    const uint32_t *__restrict__ group0, int n_images, uint32_t groups_per_wg,
    const int16_t *__restrict__ coef_all, uint8_t *__restrict__ rgb_all, uint8_t *__restrict__ chroma_all)
{
    __shared__ ReconShared S;
    __shared__ uint32_t s_hits[kReconThreads / 64];
    const uint32_t wg = blockIdx.x;
    uint32_t hits = 0;
    for (int base = 0; base < n_images; base += kReconThreads) {
        const int i = base + (int)threadIdx.x;
        hits += (uint32_t)__popcll(__ballot(i < n_images && group0[i] <= wg));
    }
    if ((threadIdx.x & 63) == 0) s_hits[threadIdx.x >> 6] = hits;
    __syncthreads();
    hits = 0;
    for (int w = 0; w < kReconThreads / 64; w++) hits += s_hits[w];
    if (hits == 0) return;
    const ImageRec &R = recs[hits - 1];
    if (R.status != PREP_OK) return;
    const uint32_t total = (uint32_t)R.roi_gcols * (uint32_t)R.roi_rows;
    const uint32_t gi0 = (wg - R.group0) * groups_per_wg;
    if (gi0 >= total) return;
    const uint32_t n = min(groups_per_wg, total - gi0);
    if (R.sampling == PREP_SAMPLING_420)
        reconstruct_groups<PREP_SAMPLING_420, kPlanes>(S, bits, R, gi0, n, coef_all, rgb_all, chroma_all);
    else if (R.sampling == PREP_SAMPLING_444)
        reconstruct_groups<PREP_SAMPLING_444, false>(S, bits, R, gi0, n, coef_all, rgb_all, chroma_all);
    else if (R.sampling == PREP_SAMPLING_422)
        reconstruct_groups<PREP_SAMPLING_422, kPlanes>(S, bits, R, gi0, n, coef_all, rgb_all, chroma_all);
    else if (R.sampling == PREP_SAMPLING_440)
        reconstruct_groups<PREP_SAMPLING_440, kPlanes>(S, bits, R, gi0, n, coef_all, rgb_all, chroma_all);
    else
        reconstruct_groups<PREP_SAMPLING_GRAY, false>(S, bits, R, gi0, n, coef_all, rgb_all, chroma_all);
}

// The second kernel of the interpolating variant (a decode variant under the flexibility
// objective of PREBA section 4.2): subsampled chroma brought to full resolution under a centred
// triangle, then the colour transform.  A chroma sample of a 2:1 axis lies midway between two
// pixels; a pixel takes 3/4 of the sample it belongs to and 1/4 of the next one on its side
// (9, 3, 3, 1 sixteenths over two axes), rounded to the nearest integer with halves upwards,
// and a neighbour outside the image's samples is the sample at the edge.  Reads the gray
// pixels and the chroma planes that reconstruct_rgb<true> left, and writes the pixels in
// place.  A thread takes four adjacent pixels of one row of the image's reconstructed region;
// neighbours outside that region are clamped to it, so its outermost pixels are exact only
// where the region ends with the image.
__global__ __launch_bounds__(kReconThreads) void interpolate_chroma_rgb(
    const ImageRec *__restrict__ recs, const uint8_t *__restrict__ chroma_all, uint8_t *__restrict__ rgb_all)
{
    const ImageRec &R = recs[blockIdx.y];
    if (R.status != PREP_OK) return;
    const int fx = luma_h(R.sampling), fy = luma_v(R.sampling);
    if (R.sampling == PREP_SAMPLING_GRAY || fx * fy == 1) return;
    const int per_group = recon_mcus_per_group(R.sampling);
    // the region in pixels and in chroma samples
    const int x_lo = R.roi_gcol0 * per_group * 8 * fx;
    const int x_hi = min((R.roi_gcol0 + R.roi_gcols) * per_group, (int)R.mcu_cols) * 8 * fx;
    const int y_lo = R.roi_row0 * 8 * fy, y_hi = (R.roi_row0 + R.roi_rows) * 8 * fy;
    const int quads = (x_hi - x_lo) >> 2;
    const int item = blockIdx.x * kReconThreads + threadIdx.x;
    if (item >= quads * (y_hi - y_lo)) return;
    const int y = y_lo + item / quads, x0 = x_lo + (item % quads) * 4;
    const int cx_lo = x_lo / fx, cx_hi = min(x_hi / fx, ((int)R.width + fx - 1) / fx) - 1;
    const int cy_lo = y_lo / fy, cy_hi = min(y_hi / fy, ((int)R.height + fy - 1) / fy) - 1;
    const ChromaPlanes cp = chroma_planes_of(R);
    // rows: the sample row the pixel belongs to, the next one on its side, and the nearer row's
    // weight in quarters
    const int y_near = min(y / fy, cy_hi);
    int y_far = y_near, wy = 4;
    if (fy == 2) { y_far = min(max((y & 1) ? y / 2 + 1 : y / 2 - 1, cy_lo), cy_hi); wy = 3; }
    uint32_t up[2][4];  // the four pixels' chroma, Cb and Cr
#pragma unroll
    for (int c = 0; c < 2; c++) {
        const uint8_t *near = chroma_all + cp.off + (size_t)c * cp.plane + (size_t)y_near * cp.pitch;
        const uint8_t *far = chroma_all + cp.off + (size_t)c * cp.plane + (size_t)y_far * cp.pitch;
        // quarters along the row, of the nearer and of the farther sample row
        int hn[4], hf[4];
        if (fx == 2) {
            const int c0 = x0 / 2;
            int sn[4], sf[4];  // samples c0 - 1 .. c0 + 2
#pragma unroll
            for (int k = 0; k < 4; k++) {
                const int cx = min(max(c0 - 1 + k, cx_lo), cx_hi);
                sn[k] = near[cx];
                sf[k] = far[cx];
            }
            hn[0] = 3 * sn[1] + sn[0]; hn[1] = 3 * sn[1] + sn[2]; hn[2] = 3 * sn[2] + sn[1]; hn[3] = 3 * sn[2] + sn[3];
            hf[0] = 3 * sf[1] + sf[0]; hf[1] = 3 * sf[1] + sf[2]; hf[2] = 3 * sf[2] + sf[1]; hf[3] = 3 * sf[2] + sf[3];
        } else {
#pragma unroll
            for (int k = 0; k < 4; k++) {
                const int cx = min(x0 + k, cx_hi);
                hn[k] = 4 * near[cx];
                hf[k] = 4 * far[cx];
            }
        }
#pragma unroll
        for (int k = 0; k < 4; k++) up[c][k] = (uint32_t)(wy * hn[k] + (4 - wy) * hf[k] + 8) >> 4;
    }
    uint8_t *px = rgb_all + R.rgb_off + (size_t)y * R.rgb_pitch + (size_t)x0 * 3;
    const uint32_t *g = reinterpret_cast<const uint32_t *>(px);  // gray pixels: Y Y Y Y Y Y ...
    const uint32_t g0 = g[0], g1 = g[1], g2 = g[2];
    const uint32_t y4 = (g0 & 255u) | ((g0 >> 24) << 8) | (((g1 >> 16) & 255u) << 16) | (((g2 >> 8) & 255u) << 24);
    store_rgb4(px, y4, chroma_terms(up[0][0], up[1][0]), chroma_terms(up[0][1], up[1][1]),
               chroma_terms(up[0][2], up[1][2]), chroma_terms(up[0][3], up[1][3]));
}

void launch_reconstruct(const uint8_t *bits, const ImageRec *recs, const uint32_t *group0, int n_images,
                        uint32_t n_workgroups, uint32_t groups_per_wg, const int16_t *coef, uint8_t *rgb,
                        uint8_t *chroma, uint32_t max_region_pixels, hipStream_t stream)
{
    if (n_workgroups == 0) return;
    if (!chroma) {
        hipLaunchKernelGGL(reconstruct_rgb<false>, dim3(n_workgroups), dim3(kReconThreads), 0, stream, bits,
                           recs, group0, n_images, groups_per_wg, coef, rgb, chroma);
        return;
    }
    hipLaunchKernelGGL(reconstruct_rgb<true>, dim3(n_workgroups), dim3(kReconThreads), 0, stream, bits, recs,
                       group0, n_images, groups_per_wg, coef, rgb, chroma);
    const uint32_t items = max_region_pixels / 4;  // four pixels per thread
    if (items)
        hipLaunchKernelGGL(interpolate_chroma_rgb, dim3((items + kReconThreads - 1) / kReconThreads, n_images),
                           dim3(kReconThreads), 0, stream, recs, chroma, rgb);
}

}  // namespace prep
