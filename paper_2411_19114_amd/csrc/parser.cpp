// Host-side marker/table parser (T.81 Annex B).  Reads each file up to the end
// of its start-of-scan header, validates the supported subset and records where
// the tables and the entropy-coded segment lie.  It never touches the
// entropy-coded bytes themselves except to find the EOI marker from the back.
#include "parser.h"

#include <string.h>

#include "prep_internal.h"

namespace prep {

namespace {

inline uint32_t be16(const uint8_t *p) { return (uint32_t(p[0]) << 8) | p[1]; }

// T.81 Annex C: BITS must describe a prefix code that fits the code space and
// leaves the all-ones code word of the longest length unused.
bool huffman_spec_ok(const uint8_t *bits16, uint32_t nval)
{
    uint32_t total = 0;
    uint64_t kraft = 0;  // sum of 2^(16-len) over all code words
    for (int len = 1; len <= 16; len++) {
        total += bits16[len - 1];
        kraft += uint64_t(bits16[len - 1]) << (16 - len);
    }
    if (total != nval || total == 0 || total > 256) return false;
    return kraft < (1ull << 16);
}

}  // namespace

int parse_image(const uint8_t *d, uint64_t len, ParsedImage *out)
{
    memset(out, 0, sizeof *out);
    prep_image_info &I = out->info;
    I.status = PREP_E_CORRUPT;
    if (len >= 0xFFFFFFF0ull) { I.status = PREP_E_UNSUPPORTED; return I.status; }
    if (len < 4 || d[0] != 0xFF || d[1] != 0xD8) return I.status;

    bool have_frame = false;
    bool qdef[4] = {false, false, false, false};
    uint32_t qoff[4] = {0, 0, 0, 0};
    bool hdef[2][4] = {{false}};
    uint32_t hoff[2][4] = {{0}}, hnval[2][4] = {{0}};
    int comp_id[3] = {0, 0, 0}, comp_tq[3] = {0, 0, 0}, comp_h[3] = {1, 1, 1}, comp_v[3] = {1, 1, 1};
    int ncomp = 0;
    uint64_t i = 2;
    for (;;) {
        if (i + 4 > len || d[i] != 0xFF) return I.status;
        while (i < len && d[i] == 0xFF) i++;  // fill bytes before a marker code
        if (i >= len) return I.status;
        const int m = d[i++];
        if (m == 0x01 || (m >= 0xD0 && m <= 0xD8)) continue;  // stand-alone markers
        if (m == 0xD9 || m == 0x00) return I.status;          // EOI before a scan / not a marker
        if (i + 2 > len) return I.status;
        const uint32_t L = be16(d + i);
        if (L < 2 || i + L > len) return I.status;
        const uint8_t *p = d + i + 2;
        int n = int(L) - 2;
        if (m == 0xDB) {  // DQT, B.2.4.1
            while (n > 0) {
                const int pq = p[0] >> 4, tq = p[0] & 15;
                if (tq > 3) return I.status;
                if (pq != 0) { I.status = PREP_E_UNSUPPORTED; return I.status; }
                if (n < 65) return I.status;
                for (int k = 0; k < 64; k++)
                    if (p[1 + k] == 0) return I.status;  // a zero quantiser is not allowed
                qdef[tq] = true;
                qoff[tq] = uint32_t(p + 1 - d);
                p += 65;
                n -= 65;
            }
        } else if (m == 0xC4) {  // DHT, B.2.4.2
            while (n > 0) {
                if (n < 17) return I.status;
                const int tc = p[0] >> 4, th = p[0] & 15;
                if (tc > 1 || th > 3) return I.status;
                uint32_t total = 0;
                for (int l = 0; l < 16; l++) total += p[1 + l];
                if (uint32_t(n) < 17 + total) return I.status;
                if (!huffman_spec_ok(p + 1, total)) return I.status;
                hdef[tc][th] = true;
                hoff[tc][th] = uint32_t(p + 1 - d);
                hnval[tc][th] = total;
                p += 17 + total;
                n -= int(17 + total);
            }
        } else if (m == 0xC0) {  // SOF0, B.2.2
            if (have_frame || n < 6) return I.status;
            if (p[0] != 8) { I.status = PREP_E_UNSUPPORTED; return I.status; }
            I.height = int32_t(be16(p + 1));
            I.width = int32_t(be16(p + 3));
            ncomp = p[5];
            if (ncomp != 1 && ncomp != 3) { I.status = PREP_E_UNSUPPORTED; return I.status; }
            if (n != 6 + 3 * ncomp) return I.status;
            if (I.width < 1 || I.height < 1) { I.status = PREP_E_UNSUPPORTED; return I.status; }
            for (int c = 0; c < ncomp; c++) {
                comp_id[c] = p[6 + 3 * c];
                comp_h[c] = p[7 + 3 * c] >> 4;
                comp_v[c] = p[7 + 3 * c] & 15;
                comp_tq[c] = p[8 + 3 * c];
                if (comp_h[c] < 1 || comp_h[c] > 4 || comp_v[c] < 1 || comp_v[c] > 4 ||
                    comp_tq[c] > 3)
                    return I.status;
            }
            if (ncomp == 1) {
                I.sampling = PREP_SAMPLING_GRAY;  // A.2.2: one component is never interleaved
            } else if (comp_h[1] == 1 && comp_v[1] == 1 && comp_h[2] == 1 && comp_v[2] == 1 &&
                       comp_h[0] <= 2 && comp_v[0] <= 2) {
                I.sampling = comp_h[0] == 1 ? (comp_v[0] == 1 ? PREP_SAMPLING_444 : PREP_SAMPLING_440)
                                            : (comp_v[0] == 1 ? PREP_SAMPLING_422 : PREP_SAMPLING_420);
            } else {
                I.status = PREP_E_UNSUPPORTED;
                return I.status;
            }
            const int mcu_w = 8 * luma_h(I.sampling), mcu_h = 8 * luma_v(I.sampling);
            I.mcu_cols = (I.width + mcu_w - 1) / mcu_w;
            I.mcu_rows = (I.height + mcu_h - 1) / mcu_h;
            I.blocks_per_mcu = blocks_per_mcu_of(I.sampling);
            have_frame = true;
        } else if (m >= 0xC1 && m <= 0xCF && m != 0xC8) {
            I.status = PREP_E_UNSUPPORTED;  // extended, progressive, lossless, arithmetic
            return I.status;
        } else if (m == 0xDD) {  // DRI, B.2.4.4
            if (n != 2) return I.status;
            I.restart_interval = int32_t(be16(p));
        } else if (m == 0xDA) {  // SOS, B.2.3
            if (!have_frame || n < 1) return I.status;
            const int ns = p[0];
            if (n != 4 + 2 * ns) return I.status;
            if (ns != ncomp) { I.status = PREP_E_UNSUPPORTED; return I.status; }
            for (int c = 0; c < ns; c++) {
                if (p[1 + 2 * c] != comp_id[c]) { I.status = PREP_E_UNSUPPORTED; return I.status; }
                const int td = p[2 + 2 * c] >> 4, ta = p[2 + 2 * c] & 15;
                if (td > 3 || ta > 3) return I.status;
                if (!hdef[0][td] || !hdef[1][ta] || !qdef[comp_tq[c]]) return I.status;
                // table slots: 0/1 = DC/AC of component 0, 2/3 = DC/AC of the chroma pair
                if (c == 0) {
                    out->dht_off[0] = hoff[0][td]; out->dht_nval[0] = hnval[0][td];
                    out->dht_off[1] = hoff[1][ta]; out->dht_nval[1] = hnval[1][ta];
                } else if (c == 1) {
                    out->dht_off[2] = hoff[0][td]; out->dht_nval[2] = hnval[0][td];
                    out->dht_off[3] = hoff[1][ta]; out->dht_nval[3] = hnval[1][ta];
                } else if (hoff[0][td] != out->dht_off[2] || hoff[1][ta] != out->dht_off[3]) {
                    I.status = PREP_E_UNSUPPORTED;  // Cb and Cr must share their tables
                    return I.status;
                }
                out->dqt_off[c] = qoff[comp_tq[c]];
            }
            if (ns == 1) {
                out->dht_off[2] = out->dht_off[0]; out->dht_nval[2] = out->dht_nval[0];
                out->dht_off[3] = out->dht_off[1]; out->dht_nval[3] = out->dht_nval[1];
                out->dqt_off[1] = out->dqt_off[2] = out->dqt_off[0];
            }
            if (p[1 + 2 * ns] != 0 || p[2 + 2 * ns] != 63 || p[3 + 2 * ns] != 0) {
                I.status = PREP_E_UNSUPPORTED;
                return I.status;
            }
            const uint64_t start = i + L;
            // The entropy-coded segment is taken up to the last EOI marker of the file, found from
            // the back without reading the data; if the file goes on after its image, the scan
            // kernel finds the first EOI marker inside and the decoder stops there.
            uint64_t e = len;
            while (e >= start + 2 && !(d[e - 2] == 0xFF && d[e - 1] == 0xD9)) e--;
            if (e < start + 2) return I.status;  // truncated: no EOI
            I.entropy_offset = start;
            I.entropy_bytes = e - 2 - start;
            const int64_t nmcu = int64_t(I.mcu_cols) * I.mcu_rows;
            I.n_intervals = I.restart_interval > 0
                                ? int32_t((nmcu + I.restart_interval - 1) / I.restart_interval)
                                : 1;
            I.status = PREP_OK;
            return I.status;
        }
        // APPn, COM and every other segment with a length is skipped
        i += L;
    }
}

}  // namespace prep
