/*
 * CPU oracle (test infrastructure): the arithmetic definitions.
 * Zig-zag order, 8x8 DCT pair, JFIF colour transforms, quality-scaled
 * quantisation tables, and resize + centre crop + normalize.
 * Everything is the textbook definition evaluated in double precision.
 */
#include "oracle.h"
#include <math.h>
#include <stdlib.h>

/* T.81 Figure A.6.  Diagonal d = v+u runs 0..14; odd diagonals are walked
 * with v increasing (towards the lower left), even ones with v decreasing. */
void oracle_zigzag_pos(int k, int *v, int *u)
{
    int n = 0;
    for (int d = 0; d <= 14; d++) {
        int vlo = d > 7 ? d - 7 : 0;
        int vhi = d < 7 ? d : 7;
        int len = vhi - vlo + 1;
        if (k < n + len) {
            int i = k - n;
            int vv = (d & 1) ? vlo + i : vhi - i;
            *v = vv;
            *u = d - vv;
            return;
        }
        n += len;
    }
    *v = *u = -1;
}

/* C(u) C(v) of A.3.3 with C(0) = 1/sqrt(2), C(k>0) = 1.  The product is formed
 * exactly (C(0)^2 = 1/2) so that a block holding only a DC term reconstructs to
 * exactly DC/8 and the half-way cases of the final rounding fall where the
 * definition puts them.                                                     */
static double dct_scale2(int u, int v)
{
    if (u == 0 && v == 0) return 0.5;
    if (u == 0 || v == 0) return sqrt(0.5);
    return 1.0;
}

/* cos((2i+1) k pi/16) for i,k = 0..7: the 64 distinct cosine factors of A.3.3 */
static void cosine_factors(double ct[8][8])
{
    const double pi = acos(-1.0);
    for (int i = 0; i < 8; i++)
        for (int k = 0; k < 8; k++) ct[i][k] = cos((2 * i + 1) * k * pi / 16.0);
}

/* T.81 A.3.3:  s(y,x) = 1/4 sum_u sum_v C(u) C(v) S(v,u)
 *                         cos((2x+1) u pi/16) cos((2y+1) v pi/16)          */
void oracle_idct8x8(const double F[64], double f[64])
{
    double ct[8][8];
    cosine_factors(ct);
    for (int y = 0; y < 8; y++)
        for (int x = 0; x < 8; x++) {
            double s = 0.0;
            for (int v = 0; v < 8; v++)
                for (int u = 0; u < 8; u++)
                    s += dct_scale2(u, v) * F[v * 8 + u] * ct[x][u] * ct[y][v];
            f[y * 8 + x] = 0.25 * s;
        }
}

/* T.81 A.3.3:  S(v,u) = 1/4 C(u) C(v) sum_x sum_y s(y,x) cos(..) cos(..)   */
void oracle_fdct8x8(const double f[64], double F[64])
{
    double ct[8][8];
    cosine_factors(ct);
    for (int v = 0; v < 8; v++)
        for (int u = 0; u < 8; u++) {
            double s = 0.0;
            for (int y = 0; y < 8; y++)
                for (int x = 0; x < 8; x++) s += f[y * 8 + x] * ct[x][u] * ct[y][v];
            F[v * 8 + u] = 0.25 * dct_scale2(u, v) * s;
        }
}

static uint8_t round_clamp_u8(double v)
{
    double r = floor(v + 0.5);
    if (r < 0.0) r = 0.0;
    if (r > 255.0) r = 255.0;
    return (uint8_t)r;
}

/* JFIF (ITU-R BT.601 full range) inverse transform.                        */
void oracle_ycc_to_rgb(int y, int cb, int cr, uint8_t rgb[3])
{
    double Y = y, Cb = cb - 128.0, Cr = cr - 128.0;
    rgb[0] = round_clamp_u8(Y + 1.402 * Cr);
    rgb[1] = round_clamp_u8(Y - 0.344136 * Cb - 0.714136 * Cr);
    rgb[2] = round_clamp_u8(Y + 1.772 * Cb);
}

/* JFIF forward transform.                                                  */
void oracle_rgb_to_ycc(int r, int g, int b, uint8_t ycc[3])
{
    double R = r, G = g, B = b;
    ycc[0] = round_clamp_u8(0.299 * R + 0.587 * G + 0.114 * B);
    ycc[1] = round_clamp_u8(-0.168736 * R - 0.331264 * G + 0.5 * B + 128.0);
    ycc[2] = round_clamp_u8(0.5 * R - 0.418688 * G - 0.081312 * B + 128.0);
}

/* T.81 Annex K, Tables K.1 (luminance) and K.2 (chrominance), row-major.   */
static const uint8_t k1_luma[64] = {
    16, 11, 10, 16, 24,  40,  51,  61,
    12, 12, 14, 19, 26,  58,  60,  55,
    14, 13, 16, 24, 40,  57,  69,  56,
    14, 17, 22, 29, 51,  87,  80,  62,
    18, 22, 37, 56, 68,  109, 103, 77,
    24, 35, 55, 64, 81,  104, 113, 92,
    49, 64, 78, 87, 103, 121, 120, 101,
    72, 92, 95, 98, 112, 100, 103, 99};
static const uint8_t k2_chroma[64] = {
    17, 18, 24, 47, 99, 99, 99, 99,
    18, 21, 26, 66, 99, 99, 99, 99,
    24, 26, 56, 99, 99, 99, 99, 99,
    47, 66, 99, 99, 99, 99, 99, 99,
    99, 99, 99, 99, 99, 99, 99, 99,
    99, 99, 99, 99, 99, 99, 99, 99,
    99, 99, 99, 99, 99, 99, 99, 99,
    99, 99, 99, 99, 99, 99, 99, 99};

void oracle_quant_table(int quality, int chroma, uint16_t q[64])
{
    if (quality < 1) quality = 1;
    if (quality > 100) quality = 100;
    int s = quality < 50 ? 5000 / quality : 200 - 2 * quality;
    const uint8_t *base = chroma ? k2_chroma : k1_luma;
    for (int i = 0; i < 64; i++) {
        int v = (base[i] * s + 50) / 100;
        if (v < 1) v = 1;
        if (v > 255) v = 255;
        q[i] = (uint16_t)v;
    }
}

void oracle_resized_size(int w, int h, int s, int *ow, int *oh)
{
    if (s <= 0) { *ow = w; *oh = h; return; }
    if (w <= h) {
        *ow = s;
        *oh = (int)(((int64_t)s * h) / w);
    } else {
        *oh = s;
        *ow = (int)(((int64_t)s * w) / h);
    }
}

static int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

/* The resized and cropped samples on the 0..255 scale, planar out[c][y][x], not yet normalized. */
static int resample_plain(const uint8_t *rgb, int w, int h, int resize_short, int crop_h, int crop_w,
                          double *out)
{
    if (!rgb || !out || w < 1 || h < 1 || crop_h < 1 || crop_w < 1) return ORACLE_E_ARG;
    int ow, oh;
    oracle_resized_size(w, h, resize_short, &ow, &oh);
    if (crop_w > ow || crop_h > oh) return ORACLE_E_ARG;
    int top = (oh - crop_h) / 2, left = (ow - crop_w) / 2;
    double scale_x = (double)w / (double)ow, scale_y = (double)h / (double)oh;
    for (int c = 0; c < 3; c++)
        for (int y = 0; y < crop_h; y++)
            for (int x = 0; x < crop_w; x++) {
                /* centre of output pixel mapped into source pixel units */
                double sx = (x + left + 0.5) * scale_x - 0.5;
                double sy = (y + top + 0.5) * scale_y - 0.5;
                int x0 = (int)floor(sx), y0 = (int)floor(sy);
                double fx = sx - x0, fy = sy - y0;
                int xa = clampi(x0, 0, w - 1), xb = clampi(x0 + 1, 0, w - 1);
                int ya = clampi(y0, 0, h - 1), yb = clampi(y0 + 1, 0, h - 1);
                double p00 = rgb[((size_t)ya * w + xa) * 3 + c];
                double p01 = rgb[((size_t)ya * w + xb) * 3 + c];
                double p10 = rgb[((size_t)yb * w + xa) * 3 + c];
                double p11 = rgb[((size_t)yb * w + xb) * 3 + c];
                out[((size_t)c * crop_h + y) * crop_w + x] =
                    (1.0 - fy) * ((1.0 - fx) * p00 + fx * p01) + fy * ((1.0 - fx) * p10 + fx * p11);
            }
    return ORACLE_OK;
}

/* Normalize (PREBA Table 1) in place: (v / 255 - mean[c]) / std[c]. */
static int normalize_planes(double *v, int crop_h, int crop_w, const double mean[3], const double std[3])
{
    for (int c = 0; c < 3; c++)
        if (!(std[c] > 0.0)) return ORACLE_E_ARG;
    for (int c = 0; c < 3; c++)
        for (size_t i = 0; i < (size_t)crop_h * crop_w; i++) {
            double *p = &v[(size_t)c * crop_h * crop_w + i];
            *p = (*p / 255.0 - mean[c]) / std[c];
        }
    return ORACLE_OK;
}

int oracle_preprocess(const uint8_t *rgb, int w, int h, int resize_short,
                      int crop_h, int crop_w, const double mean[3], const double std[3],
                      double *out)
{
    for (int c = 0; c < 3; c++)
        if (!(std[c] > 0.0)) return ORACLE_E_ARG;
    int rc = resample_plain(rgb, w, h, resize_short, crop_h, crop_w, out);
    return rc ? rc : normalize_planes(out, crop_h, crop_w, mean, std);
}

/* Weights of the source samples that one output sample of the antialiased resize reads along
 * one axis: a triangle centred on the output sample's centre (in source units), as wide as
 * the larger of one source sample and one output sample, cut at the image's edge and scaled
 * to sum 1.  Returns the first source index; *count = number of weights written to wt.     */
static int triangle_window(int out_index, double scale, int in_size, double *wt, int *count)
{
    double support = scale > 1.0 ? scale : 1.0;
    double centre = (out_index + 0.5) * scale;
    int first = (int)floor(centre - support + 0.5);
    int end = (int)floor(centre + support + 0.5);
    if (first < 0) first = 0;
    if (end > in_size) end = in_size;
    double total = 0.0;
    for (int j = first; j < end; j++) {
        double d = fabs(j + 0.5 - centre) / support;
        wt[j - first] = d < 1.0 ? 1.0 - d : 0.0;
        total += wt[j - first];
    }
    for (int j = first; j < end; j++) wt[j - first] /= total;
    *count = end - first;
    return first;
}

static int resample_antialias(const uint8_t *rgb, int w, int h, int resize_short, int crop_h, int crop_w,
                              double *out)
{
    if (!rgb || !out || w < 1 || h < 1 || crop_h < 1 || crop_w < 1) return ORACLE_E_ARG;
    int ow, oh;
    oracle_resized_size(w, h, resize_short, &ow, &oh);
    if (crop_w > ow || crop_h > oh) return ORACLE_E_ARG;
    int top = (oh - crop_h) / 2, left = (ow - crop_w) / 2;
    double scale_x = (double)w / (double)ow, scale_y = (double)h / (double)oh;
    /* at most 2 * support + 2 samples fall under a triangle */
    size_t cap_x = (size_t)(2.0 * (scale_x > 1.0 ? scale_x : 1.0)) + 3;
    size_t cap_y = (size_t)(2.0 * (scale_y > 1.0 ? scale_y : 1.0)) + 3;
    double *wx = malloc(cap_x * sizeof *wx), *wy = malloc(cap_y * sizeof *wy);
    if (!wx || !wy) { free(wx); free(wy); return ORACLE_E_ARG; }
    for (int y = 0; y < crop_h; y++) {
        int ny, y0 = triangle_window(y + top, scale_y, h, wy, &ny);
        for (int x = 0; x < crop_w; x++) {
            int nx, x0 = triangle_window(x + left, scale_x, w, wx, &nx);
            for (int c = 0; c < 3; c++) {
                double v = 0.0;
                for (int r = 0; r < ny; r++) {
                    double row = 0.0;
                    for (int k = 0; k < nx; k++)
                        row += wx[k] * rgb[((size_t)(y0 + r) * w + (x0 + k)) * 3 + c];
                    v += wy[r] * row;
                }
                out[((size_t)c * crop_h + y) * crop_w + x] = v;
            }
        }
    }
    free(wx);
    free(wy);
    return ORACLE_OK;
}

int oracle_preprocess_antialias(const uint8_t *rgb, int w, int h, int resize_short,
                                int crop_h, int crop_w, const double mean[3], const double std[3],
                                double *out)
{
    for (int c = 0; c < 3; c++)
        if (!(std[c] > 0.0)) return ORACLE_E_ARG;
    int rc = resample_antialias(rgb, w, h, resize_short, crop_h, crop_w, out);
    return rc ? rc : normalize_planes(out, crop_h, crop_w, mean, std);
}

/* ---- 8-bit output: the resized sample rounded to the nearest integer, halves upwards ------
 * Computed in exact integers, not from the double-precision planes above: the weights of both
 * filters are rationals with small denominators (2 * out size for the two-tap filter, the
 * window's weight sum for the antialiased one), rational scales put samples exactly half way
 * between two integers all the time, and floor(v + 1/2) must not depend on which side of such
 * a point a floating-point evaluation happens to land.                                      */

typedef __int128 wide_t;

static int64_t floor_div(int64_t a, int64_t b) /* b > 0 */
{
    int64_t q = a / b;
    return (a % b != 0 && a < 0) ? q - 1 : q;
}

/* Two-tap weights along one axis for output index i (crop offset included): source
 * coordinate (2 i + 1) in / (2 out) - 1/2 = n / d with d = 2 out; taps floor and floor + 1,
 * clamped, with weights (d - a) / d and a / d.                                             */
static void two_taps(int i, int in_size, int out_size, int *t0, int *t1, int64_t *a, int64_t *d)
{
    int64_t n = (int64_t)(2 * (int64_t)i + 1) * in_size - out_size;
    *d = 2 * (int64_t)out_size;
    int64_t f = floor_div(n, *d);
    *a = n - f * *d;
    *t0 = clampi((int)f, 0, in_size - 1);
    *t1 = clampi((int)f + 1, 0, in_size - 1);
}

/* Triangle weights along one axis for output index i, as integers u[j - first] >= 0 whose sum
 * is the normalising denominator.  With scale = in / out and support = max(scale, 1) = s / out,
 * s = max(in, out): the centre is (2 i + 1) in / (2 out), the window is
 * [floor(centre - support + 1/2), floor(centre + support + 1/2)) cut to the image, and
 * 1 - |j + 1/2 - centre| / support = (2 s - |(2 j + 1) out - (2 i + 1) in|) / (2 s).          */
static int triangle_units(int i, int in_size, int out_size, int64_t *u, int *count)
{
    int64_t s = in_size > out_size ? in_size : out_size;
    int64_t c2 = (int64_t)(2 * (int64_t)i + 1) * in_size;            /* centre * 2 out */
    int64_t first = floor_div(c2 - 2 * s + out_size, 2 * (int64_t)out_size);
    int64_t end = floor_div(c2 + 2 * s + out_size, 2 * (int64_t)out_size);
    if (first < 0) first = 0;
    if (end > in_size) end = in_size;
    for (int64_t j = first; j < end; j++) {
        int64_t dist = (2 * j + 1) * out_size - c2;
        if (dist < 0) dist = -dist;
        u[j - first] = 2 * s > dist ? 2 * s - dist : 0;
    }
    *count = (int)(end - first);
    return (int)first;
}

int oracle_resize_crop_u8(const uint8_t *rgb, int w, int h, int resize_short, int crop_h, int crop_w,
                          int antialias, uint8_t *out)
{
    if (!rgb || !out || w < 1 || h < 1 || crop_h < 1 || crop_w < 1) return ORACLE_E_ARG;
    int ow, oh;
    oracle_resized_size(w, h, resize_short, &ow, &oh);
    if (crop_w > ow || crop_h > oh) return ORACLE_E_ARG;
    int top = (oh - crop_h) / 2, left = (ow - crop_w) / 2;
    if (!antialias) {
        for (int y = 0; y < crop_h; y++) {
            int ya, yb;
            int64_t b, e;
            two_taps(y + top, h, oh, &ya, &yb, &b, &e);
            for (int x = 0; x < crop_w; x++) {
                int xa, xb;
                int64_t a, d;
                two_taps(x + left, w, ow, &xa, &xb, &a, &d);
                for (int c = 0; c < 3; c++) {
                    int64_t p00 = rgb[((size_t)ya * w + xa) * 3 + c], p01 = rgb[((size_t)ya * w + xb) * 3 + c];
                    int64_t p10 = rgb[((size_t)yb * w + xa) * 3 + c], p11 = rgb[((size_t)yb * w + xb) * 3 + c];
                    /* v = num / (d e); floor(v + 1/2) = floor((2 num + d e) / (2 d e)) */
                    int64_t num = (e - b) * ((d - a) * p00 + a * p01) + b * ((d - a) * p10 + a * p11);
                    out[((size_t)y * crop_w + x) * 3 + c] = (uint8_t)((2 * num + d * e) / (2 * d * e));
                }
            }
        }
        return ORACLE_OK;
    }
    size_t cap_x = 2 * (size_t)(w > ow ? w / ow + 1 : 1) + 4, cap_y = 2 * (size_t)(h > oh ? h / oh + 1 : 1) + 4;
    int64_t *ux = malloc(cap_x * sizeof *ux), *uy = malloc(cap_y * sizeof *uy);
    if (!ux || !uy) { free(ux); free(uy); return ORACLE_E_ARG; }
    for (int y = 0; y < crop_h; y++) {
        int ny, y0 = triangle_units(y + top, h, oh, uy, &ny);
        wide_t sum_y = 0;
        for (int r = 0; r < ny; r++) sum_y += uy[r];
        for (int x = 0; x < crop_w; x++) {
            int nx, x0 = triangle_units(x + left, w, ow, ux, &nx);
            wide_t sum_x = 0;
            for (int k = 0; k < nx; k++) sum_x += ux[k];
            for (int c = 0; c < 3; c++) {
                wide_t num = 0;
                for (int r = 0; r < ny; r++) {
                    wide_t row = 0;
                    for (int k = 0; k < nx; k++) row += (wide_t)ux[k] * rgb[((size_t)(y0 + r) * w + (x0 + k)) * 3 + c];
                    num += (wide_t)uy[r] * row;
                }
                wide_t den = sum_x * sum_y;
                out[((size_t)y * crop_w + x) * 3 + c] = (uint8_t)((2 * num + den) / (2 * den));
            }
        }
    }
    free(ux);
    free(uy);
    return ORACLE_OK;
}
