// Launchers of libprep's HIP kernels (one translation unit per stage).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/prep.h"
#include "prep_internal.h"

namespace prep {

// entropy.hip
// bytes of one slot of expanded Huffman tables
size_t huff_tables_bytes();
// table_rep[s] = an image whose tables go into slot s of `tables` (n_tables slots);
// window_bytes = raw bytes between workgroup starts (the ImageRecs' n_windows count such windows);
// data_end[i] = length of image i's entropy-coded segment as the host found it, lowered by the
// kernel to the offset of the first EOI marker inside it
void launch_scan_restart_markers(const uint8_t *bits, const ImageRec *recs, int n_images,
                                 uint32_t n_windows, uint32_t window_bytes, uint32_t *win_count, uint32_t *win_first,
                                 uint32_t *data_end,
                                 int32_t *status, const uint32_t *table_rep, uint32_t n_tables,
                                 uint8_t *tables, hipStream_t stream);
// coef + side_off: one int16 per block of the coefficient workspace, in the same allocation
// behind the coefficients (the DC differences, which the decoder turns into values in a second
// step of the same launch); side_off plus the number of blocks must stay below 2^32;
// small_windows: the windows are small (the decoder variant for small calls), and
// hyp_span_bits = what a lane of its hypothesis passes takes, 512 or 256 bits
void launch_decode_entropy(const uint8_t *bits, const ImageRec *recs, int n_images,
                           uint32_t n_windows, const uint32_t *win_count, const uint32_t *win_first,
                           const uint32_t *data_end, int16_t *coef, uint32_t side_off, int32_t *status,
                           const uint8_t *tables, bool small_windows, uint32_t hyp_span_bits, hipStream_t stream);

// reconstruct.hip
// chroma: nullptr = subsampled chroma is replicated; else the workspace of the interpolating
// variant (a third of the RGB workspace's size), and max_region_pixels = the most pixels that
// the reconstructed region of one image holds (a multiple of four).
void launch_reconstruct(const uint8_t *bits, const ImageRec *recs, const uint32_t *group0, int n_images,
                        uint32_t n_workgroups, uint32_t groups_per_wg, const int16_t *coef, uint8_t *rgb,
                        uint8_t *chroma, uint32_t max_region_pixels, hipStream_t stream);

// resize.hip
// host_rr: the host's copy of rr (the records of all n_images must be initialised); read for
// PREP_FILTER_ANTIALIAS only, where the images are dealt to two launches by their scales.
void launch_resize_normalize(const uint8_t *rgb, const ResizeRec *rr, const int32_t *status,
                             int n_images, int crop_h, int crop_w, int out_dtype, int filter,
                             const ResizeRec *host_rr, const float mean[3], const float std[3], void *out,
                             bool wide_reads, hipStream_t stream);

// api.cpp: host-side checks and geometry shared by the entry points
bool params_ok(const prep_params *p);
// Mapping constants of one image (source offset and row pitch in bytes); false when the crop
// does not fit the resized image.
bool make_resize_rec(int w, int h, const prep_params *p, uint64_t src_off, uint32_t pitch, ResizeRec *r);

}  // namespace prep
