/*
 * CPU oracle (test infrastructure): baseline JPEG encoder.
 * Produces test inputs and the encode -> decode round-trip pin.  T.81 Annex A
 * (FDCT, quantisation, zig-zag), F.1 (Huffman coding of DC differences and AC
 * run/size pairs, byte stuffing, restart intervals), Annex B (file syntax).
 */
#include "oracle.h"
#include <math.h>
#include <stdlib.h>
#include <string.h>

static void geometry(int w, int h, int mode, oracle_info *g)
{
    memset(g, 0, sizeof *g);
    g->width = w;
    g->height = h;
    g->ncomp = mode == ORACLE_GRAY ? 1 : 3;
    for (int c = 0; c < 3; c++) g->hs[c] = g->vs[c] = 1;
    /* luma sampling factors (T.81 A.1.1); the chroma components are 1 x 1 */
    if (mode == ORACLE_420) g->hs[0] = g->vs[0] = 2;
    if (mode == ORACLE_422) g->hs[0] = 2;
    if (mode == ORACLE_440) g->vs[0] = 2;
    g->hmax = g->hs[0];
    g->vmax = g->vs[0];
    g->mcu_cols = (w + 8 * g->hmax - 1) / (8 * g->hmax);
    g->mcu_rows = (h + 8 * g->vmax - 1) / (8 * g->vmax);
    g->blocks_per_mcu = 0;
    for (int c = 0; c < g->ncomp; c++) g->blocks_per_mcu += g->hs[c] * g->vs[c];
    g->nblocks = (int64_t)g->mcu_cols * g->mcu_rows * g->blocks_per_mcu;
}

/* quantise: nearest integer, halves away from zero */
static int quantise(double F, int q)
{
    double r = F / q;
    return (int)(r < 0 ? -floor(-r + 0.5) : floor(r + 0.5));
}

int oracle_forward_blocks(const uint8_t *rgb, int w, int h, int mode,
                          const uint16_t qluma[64], const uint16_t qchroma[64],
                          int16_t *coef, size_t coef_cap, oracle_info *info)
{
    if (!rgb || !coef || w < 1 || h < 1 || mode < 0 || mode > ORACLE_440) return ORACLE_E_ARG;
    oracle_info g;
    geometry(w, h, mode, &g);
    if (coef_cap < (size_t)g.nblocks * 64) return ORACLE_E_ARG;
    int pw = g.mcu_cols * 8 * g.hmax, ph = g.mcu_rows * 8 * g.vmax; /* padded luma size */
    /* full-resolution Y, Cb, Cr planes, padded by repeating the last row/column */
    uint8_t *plane[3];
    for (int c = 0; c < 3; c++) plane[c] = (uint8_t *)malloc((size_t)pw * ph);
    for (int y = 0; y < ph; y++)
        for (int x = 0; x < pw; x++) {
            int sy = y < h ? y : h - 1, sx = x < w ? x : w - 1;
            const uint8_t *p = rgb + ((size_t)sy * w + sx) * 3;
            uint8_t ycc[3];
            oracle_rgb_to_ycc(p[0], p[1], p[2], ycc);
            for (int c = 0; c < 3; c++) plane[c][(size_t)y * pw + x] = ycc[c];
        }
    /* component planes at their own resolution */
    uint8_t *comp[3] = {0, 0, 0};
    int cw[3], ch[3];
    for (int c = 0; c < g.ncomp; c++) {
        cw[c] = pw * g.hs[c] / g.hmax;
        ch[c] = ph * g.vs[c] / g.vmax;
        comp[c] = (uint8_t *)malloc((size_t)cw[c] * ch[c]);
        int fx = g.hmax / g.hs[c], fy = g.vmax / g.vs[c];
        for (int y = 0; y < ch[c]; y++)
            for (int x = 0; x < cw[c]; x++) {
                int sum = 0;
                for (int dy = 0; dy < fy; dy++)
                    for (int dx = 0; dx < fx; dx++)
                        sum += plane[c][(size_t)(y * fy + dy) * pw + (x * fx + dx)];
                int n = fx * fy;
                comp[c][(size_t)y * cw[c] + x] = (uint8_t)((sum + n / 2) / n);
            }
    }
    int zv[64], zu[64];
    for (int k = 0; k < 64; k++) oracle_zigzag_pos(k, &zv[k], &zu[k]);
    int16_t *dst = coef;
    for (int my = 0; my < g.mcu_rows; my++)
        for (int mx = 0; mx < g.mcu_cols; mx++)
            for (int c = 0; c < g.ncomp; c++) {
                const uint16_t *q = c == 0 ? qluma : qchroma;
                for (int by = 0; by < g.vs[c]; by++)
                    for (int bx = 0; bx < g.hs[c]; bx++) {
                        int x0 = (mx * g.hs[c] + bx) * 8, y0 = (my * g.vs[c] + by) * 8;
                        double f[64], F[64];
                        for (int y = 0; y < 8; y++)
                            for (int x = 0; x < 8; x++)
                                f[y * 8 + x] = comp[c][(size_t)(y0 + y) * cw[c] + x0 + x] - 128.0;
                        oracle_fdct8x8(f, F);
                        for (int k = 0; k < 64; k++) {
                            int n = zv[k] * 8 + zu[k];
                            dst[k] = (int16_t)quantise(F[n], q[n]);
                        }
                        dst += 64;
                    }
            }
    for (int c = 0; c < 3; c++) { free(plane[c]); free(comp[c]); }
    if (info) *info = g;
    return ORACLE_OK;
}

/* ---- entropy coding --------------------------------------------------- */

typedef struct {
    uint8_t *out;
    size_t cap, len;
    uint32_t acc;  /* pending bits, right aligned */
    int nacc;
    int overflow;
} bitwriter;

static void put_byte_raw(bitwriter *bw, int b)
{
    if (bw->len < bw->cap) bw->out[bw->len] = (uint8_t)b; else bw->overflow = 1;
    bw->len++;
}
static void put_bits(bitwriter *bw, uint32_t v, int n)
{
    for (int i = n - 1; i >= 0; i--) {
        bw->acc = (bw->acc << 1) | ((v >> i) & 1u);
        if (++bw->nacc == 8) {
            put_byte_raw(bw, bw->acc & 0xFF);
            if ((bw->acc & 0xFF) == 0xFF) put_byte_raw(bw, 0x00); /* F.1.2.3 stuffing */
            bw->acc = 0;
            bw->nacc = 0;
        }
    }
}
static void pad_ones(bitwriter *bw)
{
    while (bw->nacc != 0) put_bits(bw, 1, 1);
}
static void put_u16(bitwriter *bw, int v)
{
    put_byte_raw(bw, (v >> 8) & 0xFF);
    put_byte_raw(bw, v & 0xFF);
}

static int magnitude_category(int v)
{
    int a = v < 0 ? -v : v, n = 0;
    while (a) { n++; a >>= 1; }
    return n;
}
/* F.1.2.1.1: the appended bits are v for v >= 0, v-1 (low n bits) otherwise */
static uint32_t magnitude_bits(int v, int n)
{
    return (uint32_t)(v >= 0 ? v : v + (1 << n) - 1) & ((1u << n) - 1u);
}

typedef struct {
    uint8_t bits[17], huffval[256];
    int nval;
    uint16_t code_of[256];
    uint8_t size_of[256];
} enctable;

static int finish_table(enctable *t)
{
    uint16_t code[256];
    uint8_t size[256];
    int n = oracle_huff_codes(t->bits, code, size);
    if (n != t->nval) return ORACLE_E_ARG;
    memset(t->size_of, 0, sizeof t->size_of);
    for (int i = 0; i < n; i++) {
        t->code_of[t->huffval[i]] = code[i];
        t->size_of[t->huffval[i]] = size[i];
    }
    return ORACLE_OK;
}

/* Walk the blocks in scan order and either count symbols (bw == NULL) or
 * emit them.  table index: 0 DC luma, 1 AC luma, 2 DC chroma, 3 AC chroma. */
static int code_scan(const int16_t *coef, const oracle_info *g, int dri,
                     int64_t freq[4][256], const enctable *tab, bitwriter *bw)
{
    int pred[3] = {0, 0, 0};
    int64_t nmcu = (int64_t)g->mcu_cols * g->mcu_rows;
    const int16_t *blk = coef;
    for (int64_t m = 0; m < nmcu; m++) {
        if (dri > 0 && m > 0 && m % dri == 0) {
            if (bw) {
                pad_ones(bw);
                put_byte_raw(bw, 0xFF);
                put_byte_raw(bw, 0xD0 + (int)((m / dri - 1) & 7));
            }
            pred[0] = pred[1] = pred[2] = 0;
        }
        for (int c = 0; c < g->ncomp; c++) {
            int tdc = c == 0 ? 0 : 2, tac = tdc + 1;
            for (int b = 0; b < g->hs[c] * g->vs[c]; b++, blk += 64) {
                int diff = blk[0] - pred[c];
                pred[c] = blk[0];
                int t = magnitude_category(diff);
                if (t > 11) return ORACLE_E_ARG;
                if (bw) {
                    if (!tab[tdc].size_of[t]) return ORACLE_E_ARG;
                    put_bits(bw, tab[tdc].code_of[t], tab[tdc].size_of[t]);
                    put_bits(bw, magnitude_bits(diff, t), t);
                } else
                    freq[tdc][t]++;
                int run = 0;
                for (int k = 1; k < 64; k++) {
                    int v = blk[k];
                    if (v == 0) { run++; continue; }
                    while (run > 15) {
                        if (bw) {
                            if (!tab[tac].size_of[0xF0]) return ORACLE_E_ARG;
                            put_bits(bw, tab[tac].code_of[0xF0], tab[tac].size_of[0xF0]);
                        } else
                            freq[tac][0xF0]++;
                        run -= 16;
                    }
                    int s = magnitude_category(v);
                    if (s > 10) return ORACLE_E_ARG;
                    int rs = (run << 4) | s;
                    if (bw) {
                        if (!tab[tac].size_of[rs]) return ORACLE_E_ARG;
                        put_bits(bw, tab[tac].code_of[rs], tab[tac].size_of[rs]);
                        put_bits(bw, magnitude_bits(v, s), s);
                    } else
                        freq[tac][rs]++;
                    run = 0;
                }
                if (run > 0) { /* trailing zeros: end of block */
                    if (bw) {
                        if (!tab[tac].size_of[0]) return ORACLE_E_ARG;
                        put_bits(bw, tab[tac].code_of[0], tab[tac].size_of[0]);
                    } else
                        freq[tac][0]++;
                }
            }
        }
    }
    if (bw) pad_ones(bw);
    return ORACLE_OK;
}

/* A smooth count model that gives every baseline symbol a code: DC
 * categories 0..11, AC run 0..15 x size 1..10, EOB and ZRL.               */
static void model_counts(int64_t freq[4][256])
{
    memset(freq, 0, sizeof(int64_t) * 4 * 256);
    for (int t = 0; t <= 11; t++) {
        int d = t > 4 ? t - 4 : 4 - t;
        freq[0][t] = freq[2][t] = 1 + (1 << 20 >> (2 * d));
    }
    for (int ti = 1; ti < 4; ti += 2) {
        for (int r = 0; r < 16; r++)
            for (int s = 1; s <= 10; s++)
                freq[ti][(r << 4) | s] = 1 + ((int64_t)1 << 24 >> (r + 2 * s)) / (r + 1);
        freq[ti][0x00] = 1 << 22;
        freq[ti][0xF0] = 1 << 8;
    }
}

/* An AC table that is a valid prefix code (Annex C) and a poor one on purpose: one
 * code of each length 2..15 for the symbols that occur least (long runs of large
 * values), sixteen-bit codes for all the others, EOB and the short runs of small
 * values last.  The Kraft sum is just above one half, so no code is all ones.       */
static void lopsided_ac_table(enctable *t)
{
    int n = 0;
    for (int r = 15; r >= 0; r--)
        for (int s = 10; s >= 1; s--) t->huffval[n++] = (uint8_t)((r << 4) | s);
    t->huffval[n++] = 0xF0;
    t->huffval[n++] = 0x00;
    t->nval = n;
    memset(t->bits, 0, sizeof t->bits);
    for (int l = 2; l <= 15; l++) t->bits[l] = 1;
    t->bits[16] = (uint8_t)(n - 14);
}

int64_t oracle_write_jpeg(const int16_t *coef, int w, int h, int mode,
                          const uint16_t qluma[64], const uint16_t qchroma[64],
                          int dri, int table_mode, uint8_t *out, size_t cap)
{
    if (!coef || !out || w < 1 || h < 1 || w > 65535 || h > 65535 || mode < 0 || mode > ORACLE_440 ||
        dri < 0 || dri > 65535)
        return ORACLE_E_ARG;
    oracle_info g;
    geometry(w, h, mode, &g);
    int ntab = g.ncomp == 1 ? 2 : 4;
    int64_t freq[4][256];
    if (table_mode == 0) {
        memset(freq, 0, sizeof freq);
        int rc = code_scan(coef, &g, dri, freq, NULL, NULL);
        if (rc) return rc;
    } else
        model_counts(freq);
    enctable tab[4];
    for (int t = 0; t < ntab; t++) {
        int64_t any = 0;
        for (int i = 0; i < 256; i++) any += freq[t][i];
        if (!any) freq[t][0] = 1; /* a table must hold at least one code */
        if (table_mode == 2 && (t & 1)) {
            lopsided_ac_table(&tab[t]);
        } else {
            tab[t].nval = oracle_huff_from_freq(freq[t], tab[t].bits, tab[t].huffval);
            if (tab[t].nval < 0) return tab[t].nval;
        }
        int rc = finish_table(&tab[t]);
        if (rc) return rc;
    }
    int zv[64], zu[64];
    for (int k = 0; k < 64; k++) oracle_zigzag_pos(k, &zv[k], &zu[k]);
    bitwriter bw = {out, cap, 0, 0, 0, 0};
    put_u16(&bw, 0xFFD8); /* SOI */
    for (int t = 0; t < (g.ncomp == 1 ? 1 : 2); t++) { /* DQT, B.2.4.1 */
        const uint16_t *q = t == 0 ? qluma : qchroma;
        put_u16(&bw, 0xFFDB);
        put_u16(&bw, 2 + 1 + 64);
        put_byte_raw(&bw, t); /* Pq = 0 (8 bit), Tq = t */
        for (int k = 0; k < 64; k++) {
            int v = q[zv[k] * 8 + zu[k]];
            if (v < 1 || v > 255) return ORACLE_E_ARG;
            put_byte_raw(&bw, v);
        }
    }
    put_u16(&bw, 0xFFC0); /* SOF0, B.2.2 */
    put_u16(&bw, 8 + 3 * g.ncomp);
    put_byte_raw(&bw, 8);
    put_u16(&bw, h);
    put_u16(&bw, w);
    put_byte_raw(&bw, g.ncomp);
    for (int c = 0; c < g.ncomp; c++) {
        put_byte_raw(&bw, c + 1);
        put_byte_raw(&bw, (g.hs[c] << 4) | g.vs[c]);
        put_byte_raw(&bw, c == 0 ? 0 : 1);
    }
    for (int t = 0; t < ntab; t++) { /* DHT, B.2.4.2 */
        put_u16(&bw, 0xFFC4);
        put_u16(&bw, 2 + 1 + 16 + tab[t].nval);
        put_byte_raw(&bw, ((t & 1) << 4) | (t >> 1)); /* Tc = AC?, Th = luma/chroma */
        for (int l = 1; l <= 16; l++) put_byte_raw(&bw, tab[t].bits[l]);
        for (int i = 0; i < tab[t].nval; i++) put_byte_raw(&bw, tab[t].huffval[i]);
    }
    if (dri > 0) { /* DRI, B.2.4.4 */
        put_u16(&bw, 0xFFDD);
        put_u16(&bw, 4);
        put_u16(&bw, dri);
    }
    put_u16(&bw, 0xFFDA); /* SOS, B.2.3 */
    put_u16(&bw, 6 + 2 * g.ncomp);
    put_byte_raw(&bw, g.ncomp);
    for (int c = 0; c < g.ncomp; c++) {
        put_byte_raw(&bw, c + 1);
        put_byte_raw(&bw, c == 0 ? 0x00 : 0x11);
    }
    put_byte_raw(&bw, 0);
    put_byte_raw(&bw, 63);
    put_byte_raw(&bw, 0);
    int rc = code_scan(coef, &g, dri, NULL, tab, &bw);
    if (rc) return rc;
    put_u16(&bw, 0xFFD9); /* EOI */
    if (bw.overflow) return ORACLE_E_ARG;
    return (int64_t)bw.len;
}
