/*
 * CPU oracle (test infrastructure): baseline JPEG decoder.
 * One image at a time, one bit at a time.  T.81 Annex B (marker syntax),
 * C and F.2.2.3 (Huffman decode by MINCODE/MAXCODE/VALPTR), F.2.2.1/2 (DC
 * differences, AC run/size), F.1.2.3 (byte stuffing), E.2.4 (restart
 * intervals), A.3.4 + A.3.3 (dequantise, IDCT), level shift and clamp;
 * chroma upsampling by sample replication, or by the centred triangle
 * (oracle_upsample_triangle); JFIF colour transform.
 */
#include "oracle.h"
#include <math.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int defined;
    uint8_t huffval[256];
    int32_t mincode[17], maxcode[17], valptr[17]; /* per code length 1..16 */
} dectable;

typedef struct {
    oracle_info g;
    uint16_t q[4][64]; /* zig-zag order, as transmitted */
    int qdefined[4];
    dectable dc[4], ac[4];
    int comp_id[3], comp_tq[3], comp_td[3], comp_ta[3];
    size_t scan_start; /* first entropy-coded byte */
    int have_frame, have_scan;
} header;

static int be16(const uint8_t *p) { return (p[0] << 8) | p[1]; }

static int build_dectable(dectable *t, const uint8_t *bits16, const uint8_t *vals, int nvals)
{
    uint8_t bits[17];
    bits[0] = 0;
    int total = 0;
    for (int l = 1; l <= 16; l++) { bits[l] = bits16[l - 1]; total += bits[l]; }
    if (total != nvals || total > 256) return ORACLE_E_CORRUPT;
    uint16_t code[256];
    uint8_t size[256];
    int n = oracle_huff_codes(bits, code, size);
    if (n != total) return ORACLE_E_CORRUPT;
    memcpy(t->huffval, vals, (size_t)nvals);
    int p = 0;
    for (int l = 1; l <= 16; l++) {
        if (bits[l] == 0) {
            t->maxcode[l] = -1;
            t->mincode[l] = 0;
            t->valptr[l] = 0;
        } else {
            t->valptr[l] = p;
            t->mincode[l] = code[p];
            p += bits[l];
            t->maxcode[l] = code[p - 1];
        }
    }
    t->defined = 1;
    return ORACLE_OK;
}

/* Annex B marker walk up to and including the first SOS header.            */
static int parse_headers(const uint8_t *d, size_t len, header *H)
{
    memset(H, 0, sizeof *H);
    if (len < 4 || d[0] != 0xFF || d[1] != 0xD8) return ORACLE_E_CORRUPT;
    size_t i = 2;
    while (1) {
        if (i + 4 > len) return ORACLE_E_CORRUPT;
        if (d[i] != 0xFF) return ORACLE_E_CORRUPT;
        while (i < len && d[i] == 0xFF) i++; /* fill bytes */
        if (i >= len) return ORACLE_E_CORRUPT;
        int m = d[i++];
        if (m == 0xD8 || m == 0x01 || (m >= 0xD0 && m <= 0xD7)) continue; /* no payload */
        if (m == 0xD9) return ORACLE_E_CORRUPT; /* EOI before any scan */
        if (i + 2 > len) return ORACLE_E_CORRUPT;
        int L = be16(d + i);
        if (L < 2 || i + (size_t)L > len) return ORACLE_E_CORRUPT;
        const uint8_t *p = d + i + 2;
        int n = L - 2;
        if (m == 0xDB) { /* DQT */
            while (n > 0) {
                int pq = p[0] >> 4, tq = p[0] & 15;
                if (tq > 3) return ORACLE_E_CORRUPT;
                if (pq != 0) return ORACLE_E_UNSUPPORTED; /* 16-bit tables: not baseline */
                if (n < 65) return ORACLE_E_CORRUPT;
                for (int k = 0; k < 64; k++) H->q[tq][k] = p[1 + k];
                H->qdefined[tq] = 1;
                p += 65;
                n -= 65;
            }
        } else if (m == 0xC4) { /* DHT */
            while (n > 0) {
                if (n < 17) return ORACLE_E_CORRUPT;
                int tc = p[0] >> 4, th = p[0] & 15;
                if (tc > 1 || th > 3) return ORACLE_E_CORRUPT;
                int total = 0;
                for (int l = 0; l < 16; l++) total += p[1 + l];
                if (n < 17 + total) return ORACLE_E_CORRUPT;
                int rc = build_dectable(tc ? &H->ac[th] : &H->dc[th], p + 1, p + 17, total);
                if (rc) return rc;
                p += 17 + total;
                n -= 17 + total;
            }
        } else if (m == 0xC0) { /* SOF0 */
            if (H->have_frame) return ORACLE_E_CORRUPT;
            if (n < 6) return ORACLE_E_CORRUPT;
            if (p[0] != 8) return ORACLE_E_UNSUPPORTED;
            oracle_info *g = &H->g;
            g->height = be16(p + 1);
            g->width = be16(p + 3);
            g->ncomp = p[5];
            if (g->ncomp != 1 && g->ncomp != 3) return ORACLE_E_UNSUPPORTED;
            if (n != 6 + 3 * g->ncomp) return ORACLE_E_CORRUPT;
            if (g->width < 1 || g->height < 1) return ORACLE_E_UNSUPPORTED;
            g->hmax = g->vmax = 1;
            for (int c = 0; c < g->ncomp; c++) {
                H->comp_id[c] = p[6 + 3 * c];
                g->hs[c] = p[7 + 3 * c] >> 4;
                g->vs[c] = p[7 + 3 * c] & 15;
                H->comp_tq[c] = p[8 + 3 * c];
                if (g->hs[c] < 1 || g->hs[c] > 2 || g->vs[c] < 1 || g->vs[c] > 2)
                    return ORACLE_E_UNSUPPORTED;
                if (H->comp_tq[c] > 3) return ORACLE_E_CORRUPT;
                if (g->hs[c] > g->hmax) g->hmax = g->hs[c];
                if (g->vs[c] > g->vmax) g->vmax = g->vs[c];
            }
            if (g->ncomp == 1) g->hs[0] = g->vs[0] = g->hmax = g->vmax = 1; /* A.2.2 */
            g->mcu_cols = (g->width + 8 * g->hmax - 1) / (8 * g->hmax);
            g->mcu_rows = (g->height + 8 * g->vmax - 1) / (8 * g->vmax);
            g->blocks_per_mcu = 0;
            for (int c = 0; c < g->ncomp; c++) g->blocks_per_mcu += g->hs[c] * g->vs[c];
            g->nblocks = (int64_t)g->mcu_cols * g->mcu_rows * g->blocks_per_mcu;
            H->have_frame = 1;
        } else if (m >= 0xC1 && m <= 0xCF && m != 0xC8) {
            return ORACLE_E_UNSUPPORTED; /* other frame types, arithmetic coding */
        } else if (m == 0xDD) { /* DRI */
            if (n != 2) return ORACLE_E_CORRUPT;
            H->g.restart_interval = be16(p);
        } else if (m == 0xDA) { /* SOS */
            if (!H->have_frame) return ORACLE_E_CORRUPT;
            if (n < 1) return ORACLE_E_CORRUPT;
            int ns = p[0];
            if (ns != H->g.ncomp) return ORACLE_E_UNSUPPORTED; /* one interleaved scan only */
            if (n != 4 + 2 * ns) return ORACLE_E_CORRUPT;
            for (int c = 0; c < ns; c++) {
                if (p[1 + 2 * c] != H->comp_id[c]) return ORACLE_E_UNSUPPORTED;
                H->comp_td[c] = p[2 + 2 * c] >> 4;
                H->comp_ta[c] = p[2 + 2 * c] & 15;
                if (H->comp_td[c] > 3 || H->comp_ta[c] > 3) return ORACLE_E_CORRUPT;
                if (!H->dc[H->comp_td[c]].defined || !H->ac[H->comp_ta[c]].defined)
                    return ORACLE_E_CORRUPT;
                if (!H->qdefined[H->comp_tq[c]]) return ORACLE_E_CORRUPT;
            }
            if (p[1 + 2 * ns] != 0 || p[2 + 2 * ns] != 63 || p[3 + 2 * ns] != 0)
                return ORACLE_E_UNSUPPORTED;
            H->scan_start = i + (size_t)L;
            H->have_scan = 1;
            return ORACLE_OK;
        }
        /* APPn, COM and anything else with a length: skipped */
        i += (size_t)L;
    }
}

int oracle_jpeg_info(const uint8_t *data, size_t len, oracle_info *info)
{
    if (!data || !info) return ORACLE_E_ARG;
    header H;
    int rc = parse_headers(data, len, &H);
    if (rc) return rc;
    *info = H.g;
    return ORACLE_OK;
}

/* ---- bit-serial entropy decoding --------------------------------------- */

typedef struct {
    const uint8_t *d;
    size_t len, pos;
    int cur, nleft; /* current byte and bits left in it */
    int marker;     /* marker met while fetching (0 = none) */
    int64_t bits_read;
} bitreader;

/* F.2.2.5 NEXTBIT: most significant bit first; FF 00 is a data byte FF; any
 * other FF xx is a marker, after which the reader supplies zero bits.      */
static int next_bit(bitreader *br)
{
    if (br->nleft == 0) {
        if (br->marker || br->pos >= br->len) {
            br->marker = br->marker ? br->marker : 0xD9;
            br->cur = 0;
        } else {
            br->cur = br->d[br->pos++];
            if (br->cur == 0xFF) {
                int b2 = br->pos < br->len ? br->d[br->pos] : 0xD9;
                if (b2 == 0) br->pos++;
                else { br->marker = b2; br->pos--; br->cur = 0; }
            }
        }
        br->nleft = 8;
    }
    br->nleft--;
    br->bits_read++;
    return (br->cur >> br->nleft) & 1;
}

/* F.2.2.3 DECODE */
static int decode_symbol(bitreader *br, const dectable *t)
{
    int32_t code = 0;
    for (int l = 1; l <= 16; l++) {
        code = (code << 1) | next_bit(br);
        if (t->maxcode[l] >= 0 && code <= t->maxcode[l] && code >= t->mincode[l])
            return t->huffval[t->valptr[l] + code - t->mincode[l]];
    }
    return -1;
}
/* F.2.2.4 RECEIVE + F.2.2.1 EXTEND */
static int receive_extend(bitreader *br, int t)
{
    if (t == 0) return 0;
    int v = 0;
    for (int i = 0; i < t; i++) v = (v << 1) | next_bit(br);
    return v < (1 << (t - 1)) ? v - (1 << t) + 1 : v;
}

/* A.3.3 + level shift (A.3.1): nearest integer, half-way cases up, clamped to 8 bits.
 * Cosine products that are rational in exact arithmetic (C(0)^2 = 1/2,
 * C(0) cos(pi/4) = 1/2, ...) can put a sample exactly half way; evaluated in
 * double they land within ~1e-12 of it, on either side.  Values closer than
 * ORACLE_TIE_EPS below a half-way point are therefore taken to be half way.    */
#define ORACLE_TIE_EPS (1.0 / 1048576.0)
static uint8_t clamp_sample(double v)
{
    double r = floor(v + 0.5 + ORACLE_TIE_EPS) + 128.0;
    if (r < 0.0) r = 0.0;
    if (r > 255.0) r = 255.0;
    return (uint8_t)r;
}

/* A subsampled plane brought to full resolution by linear interpolation between sample
 * centres.  With fx = 2 a sample sits between output columns 2i and 2i + 1, so column 2i
 * is a quarter of a sample spacing left of sample i and three quarters right of sample
 * i - 1: weights 3/4 and 1/4; column 2i + 1 takes 3/4 of sample i and 1/4 of sample
 * i + 1.  Rows likewise with fy = 2, the two axes multiplied (9, 3, 3, 1 sixteenths).  A
 * neighbour outside the cw x ch samples that the image owns is the sample at the edge.
 * The result is rounded to the nearest integer, halves upwards.  fx = 1 or fy = 1 leaves
 * that axis as it is.                                                                   */
int oracle_upsample_triangle(const uint8_t *plane, int pitch, int cw, int ch, int fx, int fy,
                             int w, int h, uint8_t *out)
{
    if (!plane || !out || cw < 1 || ch < 1 || w < 1 || h < 1) return ORACLE_E_ARG;
    if ((fx != 1 && fx != 2) || (fy != 1 && fy != 2)) return ORACLE_E_ARG;
    if ((w + fx - 1) / fx > cw || (h + fy - 1) / fy > ch) return ORACLE_E_ARG;
    for (int y = 0; y < h; y++)
        for (int x = 0; x < w; x++) {
            /* nearer sample, the farther one, and the nearer one's weight in quarters */
            int x_near = x / fx, x_far = x_near, wx = 4;
            if (fx == 2) { x_far = (x & 1) ? x_near + 1 : x_near - 1; wx = 3; }
            int y_near = y / fy, y_far = y_near, wy = 4;
            if (fy == 2) { y_far = (y & 1) ? y_near + 1 : y_near - 1; wy = 3; }
            if (x_far < 0) x_far = 0;
            if (x_far > cw - 1) x_far = cw - 1;
            if (y_far < 0) y_far = 0;
            if (y_far > ch - 1) y_far = ch - 1;
            int nn = plane[(size_t)y_near * pitch + x_near], nf = plane[(size_t)y_near * pitch + x_far];
            int fn = plane[(size_t)y_far * pitch + x_near], ff = plane[(size_t)y_far * pitch + x_far];
            int sum = wy * (wx * nn + (4 - wx) * nf) + (4 - wy) * (wx * fn + (4 - wx) * ff); /* sixteenths */
            out[(size_t)y * w + x] = (uint8_t)((sum + 8) >> 4);
        }
    return ORACLE_OK;
}

static int decode_with(const uint8_t *data, size_t len, int16_t *coef, size_t coef_cap,
                       uint8_t *rgb, size_t rgb_cap, oracle_info *info, int triangle)
{
    if (!data) return ORACLE_E_ARG;
    header H;
    int rc = parse_headers(data, len, &H);
    if (rc) return rc;
    oracle_info *g = &H.g;
    if (coef && coef_cap < (size_t)g->nblocks * 64) return ORACLE_E_ARG;
    if (rgb && rgb_cap < (size_t)g->width * g->height * 3) return ORACLE_E_ARG;

    int16_t *zz = (int16_t *)calloc((size_t)g->nblocks * 64, sizeof(int16_t));
    if (!zz) return ORACLE_E_ARG;
    bitreader br = {data, len, H.scan_start, 0, 0, 0, 0};
    int pred[3] = {0, 0, 0};
    int64_t nmcu = (int64_t)g->mcu_cols * g->mcu_rows;
    int ri = g->restart_interval;
    int16_t *blk = zz;
    int64_t symbols = 0;
    rc = ORACLE_OK;
    for (int64_t m = 0; m < nmcu && rc == ORACLE_OK; m++) {
        if (ri > 0 && m > 0 && m % ri == 0) {
            /* E.2.4: drop the padding bits, expect RSTn with n counting modulo 8 */
            br.nleft = 0;
            if (!br.marker) { /* marker not met yet: it must be next */
                if (br.pos + 1 < br.len && br.d[br.pos] == 0xFF) br.marker = br.d[br.pos + 1];
                else { rc = ORACLE_E_CORRUPT; break; }
            }
            int expect = 0xD0 + (int)((m / ri - 1) & 7);
            if (br.marker != expect) { rc = ORACLE_E_CORRUPT; break; }
            br.pos += 2;
            br.marker = 0;
            pred[0] = pred[1] = pred[2] = 0;
        }
        for (int c = 0; c < g->ncomp && rc == ORACLE_OK; c++) {
            const dectable *tdc = &H.dc[H.comp_td[c]], *tac = &H.ac[H.comp_ta[c]];
            for (int b = 0; b < g->hs[c] * g->vs[c]; b++, blk += 64) {
                int t = decode_symbol(&br, tdc);
                symbols++;
                if (t < 0 || t > 11) { rc = ORACLE_E_CORRUPT; break; }
                pred[c] += receive_extend(&br, t);
                blk[0] = (int16_t)pred[c];
                int k = 1;
                while (k <= 63) {
                    int rs = decode_symbol(&br, tac);
                    symbols++;
                    if (rs < 0) { rc = ORACLE_E_CORRUPT; break; }
                    int r = rs >> 4, s = rs & 15;
                    if (s == 0) {
                        if (r == 15) { k += 16; continue; }
                        break; /* EOB (runs 1..14 with size 0 are not baseline codes) */
                    }
                    k += r;
                    if (k > 63) { rc = ORACLE_E_CORRUPT; break; }
                    blk[k] = (int16_t)receive_extend(&br, s);
                    k++;
                }
                if (rc) break;
                if (br.marker) { rc = ORACLE_E_CORRUPT; break; } /* data ran into a marker */
            }
        }
    }
    g->entropy_bytes = (int64_t)(br.pos - H.scan_start);
    g->symbols = symbols;
    g->coded_bits = br.bits_read;
    if (rc) { free(zz); return rc; }
    if (coef) memcpy(coef, zz, (size_t)g->nblocks * 64 * sizeof(int16_t));

    if (rgb) {
        int zv[64], zu[64];
        for (int k = 0; k < 64; k++) oracle_zigzag_pos(k, &zv[k], &zu[k]);
        /* component planes covering the whole MCU grid */
        uint8_t *plane[3] = {0, 0, 0};
        int cw[3], ch[3];
        for (int c = 0; c < g->ncomp; c++) {
            cw[c] = g->mcu_cols * g->hs[c] * 8;
            ch[c] = g->mcu_rows * g->vs[c] * 8;
            plane[c] = (uint8_t *)malloc((size_t)cw[c] * ch[c]);
        }
        blk = zz;
        for (int my = 0; my < g->mcu_rows; my++)
            for (int mx = 0; mx < g->mcu_cols; mx++)
                for (int c = 0; c < g->ncomp; c++) {
                    const uint16_t *q = H.q[H.comp_tq[c]];
                    for (int by = 0; by < g->vs[c]; by++)
                        for (int bx = 0; bx < g->hs[c]; bx++, blk += 64) {
                            double F[64], f[64];
                            for (int k = 0; k < 64; k++) /* A.3.4 dequantise, undo zig-zag */
                                F[zv[k] * 8 + zu[k]] = (double)blk[k] * (double)q[k];
                            oracle_idct8x8(F, f);
                            int x0 = (mx * g->hs[c] + bx) * 8, y0 = (my * g->vs[c] + by) * 8;
                            for (int y = 0; y < 8; y++)
                                for (int x = 0; x < 8; x++)
                                    plane[c][(size_t)(y0 + y) * cw[c] + x0 + x] =
                                        clamp_sample(f[y * 8 + x]);
                        }
                }
        uint8_t *full[3] = {0, 0, 0};
        if (triangle && g->ncomp == 3) {
            /* chroma at full resolution first; the image owns ceil(size * factor share) samples */
            for (int c = 1; c < 3; c++) {
                int fx = g->hmax / g->hs[c], fy = g->vmax / g->vs[c];
                full[c] = (uint8_t *)malloc((size_t)g->width * g->height);
                rc = oracle_upsample_triangle(plane[c], cw[c], (g->width + fx - 1) / fx,
                                              (g->height + fy - 1) / fy, fx, fy, g->width, g->height, full[c]);
                if (rc) break;
            }
        }
        for (int y = 0; y < g->height && !rc; y++)
            for (int x = 0; x < g->width; x++) {
                uint8_t *o = rgb + ((size_t)y * g->width + x) * 3;
                int Y = plane[0][(size_t)y * cw[0] + x];
                if (g->ncomp == 1) {
                    o[0] = o[1] = o[2] = (uint8_t)Y;
                } else if (full[1]) {
                    oracle_ycc_to_rgb(Y, full[1][(size_t)y * g->width + x], full[2][(size_t)y * g->width + x], o);
                } else {
                    /* replicate each chroma sample over the pixels it covers */
                    int cx1 = x * g->hs[1] / g->hmax, cy1 = y * g->vs[1] / g->vmax;
                    int cx2 = x * g->hs[2] / g->hmax, cy2 = y * g->vs[2] / g->vmax;
                    int Cb = plane[1][(size_t)cy1 * cw[1] + cx1];
                    int Cr = plane[2][(size_t)cy2 * cw[2] + cx2];
                    oracle_ycc_to_rgb(Y, Cb, Cr, o);
                }
            }
        for (int c = 0; c < 3; c++) { free(plane[c]); free(full[c]); }
        if (rc) { free(zz); return rc; }
    }
    free(zz);
    if (info) *info = *g;
    return ORACLE_OK;
}

int oracle_jpeg_decode(const uint8_t *data, size_t len, int16_t *coef, size_t coef_cap,
                       uint8_t *rgb, size_t rgb_cap, oracle_info *info)
{
    return decode_with(data, len, coef, coef_cap, rgb, rgb_cap, info, 0);
}

int oracle_jpeg_decode_smooth(const uint8_t *data, size_t len, int16_t *coef, size_t coef_cap,
                              uint8_t *rgb, size_t rgb_cap, oracle_info *info)
{
    return decode_with(data, len, coef, coef_cap, rgb, rgb_cap, info, 1);
}
