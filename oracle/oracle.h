/*
 * CPU oracle for batched JPEG -> model-input-tensor preprocessing.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the plain, slow, single-threaded
 * definition of what the GPU library computes (PREBA, section 2.3 "Data
 * preprocessing": decode JPEG->RGB, resize, crop; Table 1 "Normalize" unit).
 * The paper names the operations and nothing else, so the decoder follows
 * ITU-T T.81 (baseline sequential DCT, Huffman) and the JFIF colour
 * convention, and the resize follows the half-pixel bilinear convention.
 * Nothing in the GPU library includes, links or calls this code, and this
 * code shares no source, table or helper with it.
 *
 * Parity status of each function is stated beside it ("pinned by").
 */
#ifndef ORACLE_H
#define ORACLE_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    ORACLE_OK = 0,
    ORACLE_E_ARG = -1,      /* bad argument / buffer too small            */
    ORACLE_E_CORRUPT = -2,  /* stream violates T.81 syntax                */
    ORACLE_E_UNSUPPORTED = -3 /* valid JPEG outside the baseline subset   */
};

enum { ORACLE_444 = 0, ORACLE_420 = 1, ORACLE_GRAY = 2, ORACLE_422 = 3, ORACLE_440 = 4 };

typedef struct {
    int32_t width, height;        /* SOF0 X, Y                             */
    int32_t ncomp;                /* 1 or 3                                */
    int32_t hs[3], vs[3];         /* sampling factors per component        */
    int32_t hmax, vmax;
    int32_t mcu_cols, mcu_rows;   /* ceil(X/(8 hmax)), ceil(Y/(8 vmax))    */
    int32_t blocks_per_mcu;
    int32_t restart_interval;     /* DRI value, 0 = none                   */
    int64_t nblocks;              /* mcu_cols*mcu_rows*blocks_per_mcu      */
    /* statistics filled by oracle_jpeg_decode (0 after oracle_jpeg_info) */
    int64_t entropy_bytes;        /* bytes from end of SOS header to EOI   */
    int64_t symbols;              /* Huffman symbols decoded               */
    int64_t coded_bits;           /* code bits + appended magnitude bits   */
} oracle_info;

/* ---- building blocks, exported so tests can pin each one ------------- */

/* T.81 Figure A.6: position k of the zig-zag sequence -> (row v, column u).
 * Computed by walking the anti-diagonals, not from a stored table.
 * pinned by: permutation property, first/last entries, diagonal order.   */
void oracle_zigzag_pos(int k, int *v, int *u);

/* T.81 A.3.3 inverse DCT, direct four-fold sum in double.
 * F and f are 8x8 row-major: F[v*8+u], f[y*8+x]. No level shift, no rounding.
 * pinned by: scipy.fft.idctn(norm='ortho'), DC-only closed form, Parseval. */
void oracle_idct8x8(const double F[64], double f[64]);

/* T.81 A.3.3 forward DCT, direct definition (encoder side only).          */
void oracle_fdct8x8(const double f[64], double F[64]);

/* JFIF inverse colour transform on 8-bit samples, result rounded half-up
 * and clamped to 0..255.
 * pinned by: Cb=Cr=128 -> R=G=B=Y, forward/inverse within 1 LSB.          */
void oracle_ycc_to_rgb(int y, int cb, int cr, uint8_t rgb[3]);
/* JFIF forward colour transform (encoder side only).                      */
void oracle_rgb_to_ycc(int r, int g, int b, uint8_t ycc[3]);

/* T.81 Annex C: canonical code assignment from BITS[1..16] / HUFFVAL.
 * bits[0] is unused, bits[l] = number of codes of length l.
 * Writes code[i], size[i] for the i-th HUFFVAL entry; returns the number of
 * codes or a negative error when the lengths over-subscribe the code space.
 * pinned by: Kraft sum, prefix-freeness brute force.                      */
int oracle_huff_codes(const uint8_t bits[17], uint16_t code[256], uint8_t size[256]);

/* T.81 K.2: length-limited (16) Huffman code lengths from symbol counts,
 * with one code point reserved so that no code is all ones.
 * freq[256]; outputs bits[17] and huffval[] (returns number of symbols).   */
int oracle_huff_from_freq(const int64_t freq[256], uint8_t bits[17], uint8_t huffval[256]);

/* Quantisation table (natural order q[v*8+u]) for a "quality" 1..100:
 * T.81 Table K.1 (chroma=0) or K.2 (chroma=1) scaled by the usual
 * 5000/q | 200-2q rule.  Encoder side only (decoders read DQT).            */
void oracle_quant_table(int quality, int chroma, uint16_t q[64]);

/* ---- encoder (produces test inputs and the round-trip pin) ------------ */

/* RGB8 HWC -> quantised coefficients in scan order (MCU by MCU; inside an
 * MCU the components in order, each V_i rows x H_i columns of blocks), 64
 * int16 per block in zig-zag order, DC stored as the absolute value.
 * mode: ORACLE_444 / ORACLE_420 / ORACLE_GRAY (gray = luma of the RGB) / ORACLE_422 (luma
 * 2 x 1: chroma halved horizontally) / ORACLE_440 (luma 1 x 2: chroma halved vertically).
 * qluma/qchroma natural order.  coef must hold info->nblocks*64 entries.   */
int oracle_forward_blocks(const uint8_t *rgb, int w, int h, int mode,
                          const uint16_t qluma[64], const uint16_t qchroma[64],
                          int16_t *coef, size_t coef_cap, oracle_info *info);

/* Quantised coefficients (layout above) -> complete JFIF-less baseline file
 * (SOI DQT SOF0 DHT [DRI] SOS data EOI).
 * table_mode 0: Huffman tables built (K.2 procedure) from this image's own
 * symbol counts; 1: built from a fixed smooth count model that gives every
 * baseline symbol a code; 2: as 1 for DC, and for AC a fixed valid prefix code
 * whose codes are sixteen bits long for all but fourteen rare symbols (decoders
 * with short lookup tables meet their long-code path on every block).
 * dri = restart interval in MCUs (0 = none).
 * Returns bytes written or a negative error.                              */
int64_t oracle_write_jpeg(const int16_t *coef, int w, int h, int mode,
                          const uint16_t qluma[64], const uint16_t qchroma[64],
                          int dri, int table_mode, uint8_t *out, size_t cap);

/* ---- decoder ---------------------------------------------------------- */

/* Marker walk only (T.81 Annex B): geometry of the first frame/scan.      */
int oracle_jpeg_info(const uint8_t *data, size_t len, oracle_info *info);

/* Full decode.  Any output pointer may be NULL.
 * coef : nblocks*64 int16, scan order x zig-zag index, absolute DC
 *        (checkpoint A, the entropy decoder's result);
 * rgb  : height*width*3 bytes, interleaved, padding discarded
 *        (checkpoint B).
 * pinned by: write->decode round trip equals the encoder's coefficients for
 * every mode x DRI x odd size; PIL decodes the same files to within a few
 * LSB; DC-only blocks give constant blocks.                               */
int oracle_jpeg_decode(const uint8_t *data, size_t len, int16_t *coef, size_t coef_cap,
                       uint8_t *rgb, size_t rgb_cap, oracle_info *info);

/* Centred-triangle upsampling of one subsampled plane (a decode variant in the sense of the
 * flexibility objective of PREBA section 4.2): the cw x ch samples of `plane` (rows `pitch`
 * apart), subsampled fx : 1 across and fy : 1 down (each 1 or 2), to w x h samples in `out`.
 * A sample of a 2 : 1 axis lies midway between two output samples, and an output sample is
 * the linear interpolation between the two input samples nearest to it (weights 3/4, 1/4;
 * 9, 3, 3, 1 sixteenths for 2 x 2), the edge sample standing in for a neighbour outside,
 * rounded to the nearest integer with halves upwards.
 * pinned by: an impulse (90, 30, 30, 10 of 160 and where they land), a ramp reproduced at the
 * quarter positions, the edge columns, the rounding of sums of 8 and 7 sixteenths, and the
 * decoder of an image library on smooth chroma.                                          */
int oracle_upsample_triangle(const uint8_t *plane, int pitch, int cw, int ch, int fx, int fy,
                             int w, int h, uint8_t *out);

/* oracle_jpeg_decode with the chroma planes of a subsampled image brought to full
 * resolution by oracle_upsample_triangle instead of sample replication.                 */
int oracle_jpeg_decode_smooth(const uint8_t *data, size_t len, int16_t *coef, size_t coef_cap,
                              uint8_t *rgb, size_t rgb_cap, oracle_info *info);

/* ---- resize + centre crop + normalize ---------------------------------- */

/* Resized size for "short side -> s" (s = 0 keeps the size): the short side
 * becomes s, the long side floor(s*long/short).                            */
void oracle_resized_size(int w, int h, int s, int *ow, int *oh);

/* Bilinear (half-pixel centres, edge clamp, no prefilter) resize of the RGB8
 * HWC image to the size above, centre crop crop_h x crop_w (origin
 * floor(margin/2)), then (v/255 - mean[c]) / std[c]; planar output
 * out[c][y][x] in double (checkpoint C).
 * pinned by: constant image, linear ramp, identity scale, closed-form
 * normalize.                                                              */
int oracle_preprocess(const uint8_t *rgb, int w, int h, int resize_short,
                      int crop_h, int crop_w, const double mean[3], const double std[3],
                      double *out);

/* The same with the antialiased bilinear resize that image libraries apply when they
 * shrink (Pillow's BILINEAR resize, torch's interpolate(mode="bilinear", antialias=True)):
 * along each axis an output sample is the triangle-weighted mean of the source samples
 * within max(scale, 1) source samples of its centre (scale = in / out), the window cut at
 * the image's edge and the weights scaled to sum 1; where the image grows this is the plain
 * bilinear resize above.  PREBA names a Resize unit (section 4.2, Table 1) and no filter.
 * pinned by: torch's CPU interpolate, Pillow's resize within its 8-bit rounding, the
 * 1/8 3/8 3/8 1/8 weights of an exact 2:1 reduction, equality with oracle_preprocess
 * when enlarging, constant images.                                                     */
int oracle_preprocess_antialias(const uint8_t *rgb, int w, int h, int resize_short,
                                int crop_h, int crop_w, const double mean[3], const double std[3],
                                double *out);

/* Resize (either filter) and centre crop without Normalize: the resized samples rounded to
 * the nearest integer, halves upwards, floor(v + 1/2), evaluated in exact integer arithmetic
 * (both filters' weights are rationals), as interleaved RGB8 out[y][x][c].
 * pinned by: the source pixels themselves at scale 1, integer means of 2:1 and 8:1 reductions
 * with their halves, both filters at scales with weights in sixths and fifteenths against the
 * definition in exact fractions (images built so that many samples lie exactly half way),
 * Pillow's 8-bit resize within one level.                                                 */
int oracle_resize_crop_u8(const uint8_t *rgb, int w, int h, int resize_short, int crop_h, int crop_w,
                          int antialias, uint8_t *out);

#ifdef __cplusplus
}
#endif
#endif
