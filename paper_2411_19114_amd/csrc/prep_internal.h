// Shared between the host code and the HIP kernels of libprep: plain-old-data
// records that travel to the GPU and the launch geometry constants.
#pragma once
#include <stdint.h>

namespace prep {

// ---- entropy decoder geometry -------------------------------------------
// One workgroup owns a contiguous run of restart intervals of one image and
// decodes it chunk by chunk.  A chunk is kChunkRaw raw bytes staged into LDS
// with stuffing and markers removed; in the speculative regime each lane owns
// one subsequence of kSubseqBytes clean bytes.
constexpr int kDecodeThreads = 256;
constexpr int kSubseqBytes = 64;                            // clean bytes per lane
constexpr int kChunkRaw = kDecodeThreads * kSubseqBytes;    // raw bytes staged per chunk
constexpr int kChunkTail = 16;                              // bytes a non-final chunk keeps back
constexpr int kWindowBytes = 12288;                         // raw bytes between workgroup starts
// A call with little entropy-coded data would leave most of the chip idle behind a few lanes
// that walk whole restart intervals one symbol after the other.  Such a call is cut into
// smaller windows (more workgroups, a few restart intervals each) and its workgroups find the
// decoder states inside an interval by phase hypotheses instead (see decode_entropy).
constexpr int kSmallWindowBytes = 2048;
constexpr uint64_t kSmallCallBytes = 1536 << 10;            // entropy-coded bytes of a call up to which it is cut small
// The smallest calls (a single image, a batch of a few dozen small ones) still leave most
// compute units idle with 2 KiB windows: they are cut into windows of about one restart
// interval of a small image, and a lane of the hypothesis passes takes half a subsequence
// (measured on batches of 256 x 256 images: 86 against 142 us up to 16 images, 96 against 140
// at 32 = 375 KB, even at 48 = 562 KB, worse from there on).
constexpr int kTinyWindowBytes = 512;
constexpr uint64_t kTinyCallBytes = 448 << 10;
constexpr int kLutBits = 10;                                // first-level Huffman lookup width
// Images of a batch mostly share their Huffman tables (encoders write the tables of T.81
// Annex K unless asked to optimise): each distinct set of four tables is expanded once per
// batch into a slot of device memory and copied into LDS by the workgroups that need it.
constexpr uint32_t kMaxTableSlots = 1024;
constexpr uint32_t kNoTableSlot = 0xFFFFFFFFu;             // expand the tables in the workgroup

// ---- reconstruction geometry ----------------------------------------------
// Sampling modes (the PREP_SAMPLING_* values): luma blocks per MCU along x and y (T.81
// A.1.1, chroma is 1 x 1) and blocks per MCU (A.2.3).
inline constexpr int luma_h(int sampling) { return sampling == 1 || sampling == 3 ? 2 : 1; }
inline constexpr int luma_v(int sampling) { return sampling == 1 || sampling == 4 ? 2 : 1; }
inline constexpr int blocks_per_mcu_of(int sampling)
{
    return sampling == 2 ? 1 : luma_h(sampling) * luma_v(sampling) + 2;
}
// One workgroup turns kReconBlocks 8x8 blocks (a run of MCUs of one MCU row)
// into RGB pixels: 5 MCUs of 4:2:0, 10 of 4:4:4, 8 of 4:2:2 or 4:4:0, 32 of grayscale.
constexpr int kReconThreads = 256;
constexpr int kReconBlocks = 32;
inline constexpr int recon_mcus_per_group(int sampling) { return kReconBlocks / blocks_per_mcu_of(sampling); }
// A workgroup takes up to kReconMaxGroupsPerWg consecutive groups of one image: as many as
// leave about kReconGroupsPerWgDivisor workgroups in the launch (two rounds of a full chip).
constexpr uint32_t kReconMaxGroupsPerWg = 8;
constexpr uint32_t kReconGroupsPerWgDivisor = 3072;

// Per-image record, written by the host parser (T.81 Annex B) and read by
// every kernel.  file_off is the byte offset of the file in the device copy of
// the batch's bitstreams; entropy_rel, dht_off and dqt_off count from there.
struct ImageRec {
    uint64_t file_off;      // first byte (SOI) of this file
    uint64_t rgb_off;       // this image's RGB plane in the workspace (bytes)
    uint32_t entropy_rel;   // first entropy-coded byte
    uint32_t entropy_len;   // bytes up to the EOI marker
    uint32_t coef_block0;   // first block of this image in the coefficient workspace
    uint32_t n_blocks;      // mcu_cols * mcu_rows * blocks_per_mcu
    uint32_t window0;       // first decode window (= workgroup) of this image
    uint32_t n_windows;
    uint32_t rgb_pitch;     // bytes between RGB rows (covers the whole MCU grid)
    uint32_t group0;        // first reconstruction workgroup of this image
    // The groups (runs of MCUs of one MCU row) that reconstruction produces: MCU rows
    // roi_row0 .. + roi_rows - 1, groups roi_gcol0 .. + roi_gcols - 1 of each.  It is what the
    // bilinear taps of the crop window touch, or the whole MCU grid.
    uint16_t roi_row0, roi_rows;
    uint16_t roi_gcol0, roi_gcols;
    uint32_t dht_off[4];    // offset of BITS[16] of: DC luma, AC luma, DC chroma, AC chroma
    uint32_t dht_nval[4];   // number of HUFFVAL bytes that follow the 16 BITS bytes
    uint32_t dqt_off[3];    // offset of the 64 zig-zag ordered table bytes per component
    uint16_t width, height;
    uint16_t mcu_cols, mcu_rows;
    uint16_t restart_interval;  // MCUs, 0 = none
    uint8_t sampling;           // PREP_SAMPLING_*
    uint8_t blocks_per_mcu;
    int32_t status;             // host verdict; kernels skip images that are not PREP_OK
    uint32_t table_slot;        // expanded Huffman tables of this image, or kNoTableSlot
};
static_assert(sizeof(ImageRec) % 8 == 0, "ImageRec must keep 8-byte alignment in arrays");

// Resize/crop/normalize geometry of one image, computed on the host in double precision
// and handed over in fixed point so that every lane maps coordinates with integer
// arithmetic: source coordinate of output pixel i = (off + i * scale) / 2^kCoordFrac - kCoordBias.
constexpr int kCoordFrac = 30;   // fraction bits (scale < 2^17 and i < 2^16 keep the product in 64 bits)
constexpr int kCoordBias = 16;   // added so that the slightly negative coordinates at the border stay positive
struct ResizeRec {
    uint64_t scale_x, scale_y;  // source pixels per output pixel
    uint64_t off_x, off_y;      // source coordinate of output pixel (0,0), biased
    int32_t src_w, src_h;
    uint32_t src_pitch;
    uint32_t pad_;
    uint64_t src_off;           // byte offset of the source image
};

}  // namespace prep
