// Driver of the CPU build of libprep (test infrastructure): reads a batch file,
// runs the C ABI end to end on host threads and dumps every checkpoint.
//   in : int32 n, resize_short, crop_h, crop_w, out_dtype; float mean[3], std[3];
//        uint64 offsets[n+1]; bytes
//   out: per image int32 status, int64 n_coef, int16 coef[], int64 n_rgb, uint8 rgb[];
//        then the output tensor
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/prep.h"

static void die(const char *what, int rc)
{
    fprintf(stderr, "prep_emul: %s failed: %d (%s)\n", what, rc, prep_strerror(rc));
    exit(2);
}

int main(int argc, char **argv)
{
    if (argc < 3) { fprintf(stderr, "usage: prep_emul in.bin out.bin\n"); return 1; }
    FILE *f = fopen(argv[1], "rb");
    if (!f) return 1;
    int32_t hdr[5];
    prep_params P;
    if (fread(hdr, 4, 5, f) != 5) return 1;
    const int32_t n = hdr[0];
    P.resize_short = hdr[1]; P.crop_h = hdr[2]; P.crop_w = hdr[3]; P.out_dtype = hdr[4];
    if (fread(P.mean, 4, 3, f) != 3 || fread(P.std, 4, 3, f) != 3) return 1;
    P.filter = PREP_FILTER_BILINEAR;
    if (const char *v = getenv("PREP_EMUL_FILTER")) P.filter = atoi(v);
    std::vector<uint64_t> off((size_t)n + 1);
    if (fread(off.data(), 8, off.size(), f) != off.size()) return 1;
    std::vector<uint8_t> bits(off[n] ? off[n] : 1);
    if (off[n] && fread(bits.data(), 1, off[n], f) != off[n]) return 1;
    fclose(f);

    std::vector<prep_image_info> info((size_t)n);
    int rc = prep_parse_headers(bits.data(), off.data(), n, info.data());
    if (rc) die("prep_parse_headers", rc);
    prep_config cfg = {};
    cfg.device = 0;
    cfg.max_batch = n > 0 ? n : 1;
    cfg.max_width = cfg.max_height = 1;
    uint64_t px = 0;
    for (auto &i : info)
        if (i.status == PREP_OK) {
            if (i.width > cfg.max_width) cfg.max_width = i.width;
            if (i.height > cfg.max_height) cfg.max_height = i.height;
            px += (uint64_t)i.width * i.height;
        }
    cfg.max_total_pixels = px ? px : 1;
    cfg.max_bitstream_bytes = off[n] ? off[n] : 1;
    if (const char *f = getenv("PREP_EMUL_FLAGS")) cfg.flags = (uint32_t)atoi(f);
    prep_handle *h = nullptr;
    rc = prep_create(&h, &cfg);
    if (rc) die("prep_create", rc);
    const size_t esz = P.out_dtype == PREP_F32 ? 4 : P.out_dtype == PREP_F16 ? 2 : 1;
    std::vector<uint8_t> out((size_t)n * 3 * P.crop_h * P.crop_w * esz + 16, 0xAB);
    rc = prep_decode_resize_batch(h, bits.data(), off.data(), n, &P, out.data(), nullptr);
    if (rc) die("prep_decode_resize_batch", rc);
    std::vector<int32_t> status((size_t)n);
    rc = prep_get_status(h, status.data(), n);
    if (rc) die("prep_get_status", rc);

    FILE *o = fopen(argv[2], "wb");
    if (!o) return 1;
    for (int32_t i = 0; i < n; i++) {
        fwrite(&status[i], 4, 1, o);
        int64_t nc = 0, nr = 0;
        int32_t rect[4] = {0, 0, 0, 0};
        std::vector<int16_t> coef;
        std::vector<uint8_t> rgb;
        if (status[i] == PREP_OK || status[i] == PREP_E_CORRUPT) {
            if (info[i].status == PREP_OK) {
                coef.resize((size_t)info[i].mcu_cols * info[i].mcu_rows * info[i].blocks_per_mcu * 64);
                nc = prep_debug_last_coefficients(h, i, coef.data(), coef.size());
                rgb.resize((size_t)info[i].width * info[i].height * 3);
                nr = prep_debug_last_rgb(h, i, rgb.data(), rgb.size());
                if (nc < 0) nc = 0;
                if (nr < 0) nr = 0;
                if (nr && prep_debug_last_region(h, i, rect) != PREP_OK) nr = 0;
            }
        }
        fwrite(&nc, 8, 1, o);
        if (nc) fwrite(coef.data(), 2, (size_t)nc, o);
        fwrite(rect, 4, 4, o);
        fwrite(&nr, 8, 1, o);
        if (nr) fwrite(rgb.data(), 1, (size_t)nr, o);
    }
    fwrite(out.data(), 1, out.size() - 16, o);
    fclose(o);
    for (size_t k = out.size() - 16; k < out.size(); k++)
        if (out[k] != 0xAB) { fprintf(stderr, "prep_emul: wrote past the output tensor\n"); return 3; }
    prep_destroy(h);
    return 0;
}
