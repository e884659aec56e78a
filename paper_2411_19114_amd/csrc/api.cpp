// C ABI of libprep: handle, workspace, host-side batch planning and the launch
// sequence  parse -> (copy) -> restart-marker scan -> entropy decode ->
// reconstruct RGB -> resize/crop/normalize  (PREBA section 2.3 item 1, 4.2).
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <condition_variable>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "../../include/prep.h"
#include "kernels.h"
#include "parser.h"
#include "prep_internal.h"

using namespace prep;

namespace prep {

bool params_ok(const prep_params *p)
{
    if (!p) return false;
    if (p->resize_short < 0 || p->resize_short > 65535) return false;
    if (p->crop_h < 1 || p->crop_w < 1 || p->crop_h > 65535 || p->crop_w > 65535) return false;
    if (p->out_dtype != PREP_F32 && p->out_dtype != PREP_F16 && p->out_dtype != PREP_U8_NHWC) return false;
    if (p->filter != PREP_FILTER_BILINEAR && p->filter != PREP_FILTER_ANTIALIAS) return false;
    if (p->out_dtype == PREP_U8_NHWC) return true;  // no Normalize: mean and std are not looked at
    for (int c = 0; c < 3; c++)
        if (!(p->std[c] > 0.0f) || !isfinite(p->std[c]) || !isfinite(p->mean[c])) return false;
    return true;
}

// Resized size: the short side becomes s, the long side floor(s * long / short).
static void resized_size(int w, int h, int s, int *ow, int *oh)
{
    if (s <= 0) { *ow = w; *oh = h; return; }
    if (w <= h) { *ow = s; *oh = (int)(((int64_t)s * h) / w); }
    else { *oh = s; *ow = (int)(((int64_t)s * w) / h); }
}

// Mapping constants of one image; false when the crop does not fit.
bool make_resize_rec(int w, int h, const prep_params *p, uint64_t src_off, uint32_t pitch,
                     ResizeRec *r)
{
    int ow, oh;
    resized_size(w, h, p->resize_short, &ow, &oh);
    if (p->crop_w > ow || p->crop_h > oh) return false;
    const int top = (oh - p->crop_h) / 2, left = (ow - p->crop_w) / 2;
    const double sx = (double)w / (double)ow, sy = (double)h / (double)oh;
    const double one = (double)(1ull << kCoordFrac);
    r->scale_x = (uint64_t)llround(sx * one);
    r->scale_y = (uint64_t)llround(sy * one);
    r->off_x = (uint64_t)llround(((left + 0.5) * sx - 0.5 + kCoordBias) * one);
    r->off_y = (uint64_t)llround(((top + 0.5) * sy - 0.5 + kCoordBias) * one);
    r->src_w = w;
    r->src_h = h;
    r->src_pitch = pitch;
    r->pad_ = 0;
    r->src_off = src_off;
    return true;
}

}  // namespace prep

namespace {

// The host's copy of a large batch into pinned memory is as long as the GPU's work on the
// batch (tens of GB/s on one thread against a 38 MB batch of full-HD frames in 2 ms), so it
// is dealt to a few helper threads and runs while the calling thread parses the headers.
// One pool per process, started at the first large copy and never torn down (its threads
// sleep on a condition variable); a second caller that finds it busy copies by itself.
constexpr size_t kPooledCopyBytes = 1 << 20;  // copies from this size on go to the pool
class CopyPool {
public:
    static CopyPool *get()
    {
        static CopyPool *pool = new (std::nothrow) CopyPool;  // (never deleted: its threads never end)
        return pool;
    }
    // Starts copying n bytes; false if the pool is in use or has no threads (nothing started).
    bool start(uint8_t *dst, const uint8_t *src, size_t n)
    {
        std::unique_lock<std::mutex> lock(m_);
        if (busy_) return false;
        if (!started_) {
            started_ = true;
            for (int i = 0; i < kWorkers; i++) {
                try {
                    std::thread(&CopyPool::work, this, i).detach();
                    alive_++;
                } catch (...) {
                    break;
                }
            }
        }
        if (alive_ == 0) return false;
        busy_ = true;
        const size_t per = ((n + (size_t)alive_ - 1) / (size_t)alive_ + 63) & ~(size_t)63;
        for (int i = 0; i < alive_; i++) {
            const size_t lo = std::min(n, per * (size_t)i), hi = std::min(n, lo + per);
            job_[i] = {dst + lo, src + lo, hi - lo};
        }
        pending_ = alive_;
        generation_++;
        lock.unlock();
        cv_work_.notify_all();
        return true;
    }
    // Blocks until the copy that start() began is done.
    void wait()
    {
        std::unique_lock<std::mutex> lock(m_);
        cv_done_.wait(lock, [&] { return pending_ == 0; });
        busy_ = false;
    }

private:
    static constexpr int kWorkers = 3;
    struct Job {
        uint8_t *dst;
        const uint8_t *src;
        size_t n;
    };
    void work(int i)
    {
        uint64_t seen = 0;
        for (;;) {
            Job j;
            {
                std::unique_lock<std::mutex> lock(m_);
                cv_work_.wait(lock, [&] { return generation_ != seen; });
                seen = generation_;
                j = job_[i];
            }
            if (j.n) memcpy(j.dst, j.src, j.n);
            {
                std::lock_guard<std::mutex> lock(m_);
                pending_--;
            }
            cv_done_.notify_all();
        }
    }
    std::mutex m_;
    std::condition_variable cv_work_, cv_done_;
    Job job_[kWorkers] = {};
    int alive_ = 0, pending_ = 0;
    uint64_t generation_ = 0;
    bool busy_ = false, started_ = false;
};

constexpr int kSlots = 2;            // pinned staging is double buffered
constexpr size_t kBitsPad = 256;     // readable slack after the last file
constexpr size_t kRgbAlign = 256;
constexpr size_t kRgbSlack = 16;     // readable bytes kept after every image's RGB rows
constexpr int kTimedCalls = 256;     // calls whose stage events are kept
constexpr uint64_t kCopyStreamMinBytes = 64 << 10;  // bitstream uploads from this size on use the copy stream
constexpr int32_t kCopyStreamMinImages = 128;       // and so do the records of batches from this size on

// What one call uploads lives in one of kSlots sets of buffers, pinned host side and device
// side, so that the upload of a call (on the handle's copy stream) overlaps the kernels of the
// call before it (on the caller's stream).
struct Slot {
    uint8_t *h_bits = nullptr;
    // One block, host side and device side, holds what a call uploads besides the bitstreams,
    // so that it goes up in one copy: n ResizeRecs, then n ImageRecs, then n first-workgroup
    // indices, then <= n table owners, then n lengths of the entropy-coded data (which the scan
    // kernel lowers to the first EOI marker).  The pointers below are set per call.
    uint8_t *h_block = nullptr, *d_block = nullptr;
    ImageRec *h_recs = nullptr;
    ResizeRec *h_rr = nullptr;
    int32_t *h_status = nullptr;
    uint8_t *d_bits = nullptr;
    ImageRec *d_recs = nullptr;
    ResizeRec *d_rr = nullptr;
    uint32_t *h_data_end = nullptr, *d_data_end = nullptr;
    hipEvent_t copied = nullptr;  // uploads of the slot's call are done
    hipEvent_t done = nullptr;    // kernels of the slot's call are done
    bool pending = false;
};

// bytes of a slot's block for n images, and the pointers into it
inline size_t block_bytes(size_t n) { return (sizeof(ResizeRec) + sizeof(ImageRec) + 3 * sizeof(uint32_t)) * n; }
inline void place_block(Slot *s, size_t n)
{
    static_assert(sizeof(ResizeRec) % 8 == 0, "the ImageRecs behind the ResizeRecs stay 8-byte aligned");
    s->h_rr = reinterpret_cast<ResizeRec *>(s->h_block);
    s->d_rr = reinterpret_cast<ResizeRec *>(s->d_block);
    s->h_recs = reinterpret_cast<ImageRec *>(s->h_block + sizeof(ResizeRec) * n);
    s->d_recs = reinterpret_cast<ImageRec *>(s->d_block + sizeof(ResizeRec) * n);
    const size_t before = (sizeof(ResizeRec) + sizeof(ImageRec) + 2 * sizeof(uint32_t)) * n;
    s->h_data_end = reinterpret_cast<uint32_t *>(s->h_block + before);
    s->d_data_end = reinterpret_cast<uint32_t *>(s->d_block + before);
}

struct Plan {                         // what one call will run
    uint32_t n_windows = 0;
    uint32_t n_groups = 0;      // reconstruction groups of all images
    uint32_t recon_wgs = 0;     // reconstruction workgroups
    uint32_t groups_per_wg = 1; // consecutive groups of one image that a workgroup takes
    uint32_t n_tables = 0;     // distinct sets of Huffman tables (<= the handle's table slots)
    uint64_t n_blocks = 0;
    uint64_t rgb_bytes = 0;
    uint32_t max_region_pixels = 0;  // most pixels in the reconstructed region of one image
    uint32_t window_bytes = kWindowBytes;  // raw bytes between the decoder's workgroup starts
};

}  // namespace

struct prep_handle {
    prep_config cfg{};
    uint64_t cap_blocks = 0, cap_rgb = 0, cap_windows = 0, cap_bits = 0;
    hipStream_t copy_stream = nullptr;
    int16_t *d_coef = nullptr;
    uint8_t *d_rgb = nullptr;
    uint8_t *d_chroma = nullptr;  // PREP_FLAG_SMOOTH_CHROMA: chroma planes between the two reconstruction kernels
    uint8_t *d_tables = nullptr;  // table_slots expanded Huffman table sets
    uint32_t table_slots = 0;
    std::vector<uint32_t> table_rep;   // image that owns each slot of this call
    std::vector<uint32_t> table_hash;  // open-addressed: slot + 1 of a table set by the hash of its DHT bytes, 0 = free
    int32_t *d_status = nullptr;
    uint32_t *d_win_count = nullptr, *d_win_first = nullptr;
    Slot slot[kSlots];
    int next_slot = 0;
    // stage timing: one set of 5 events per call, kept for the last kTimedCalls calls
    std::vector<hipEvent_t> ev;
    bool timing = false;
    uint64_t timed_calls = 0;
    // last call
    int32_t last_n = 0;
    hipStream_t last_stream = nullptr;
    std::vector<ParsedImage> parsed;
    std::vector<ImageRec> recs;
    std::vector<ResizeRec> rr;
    std::vector<uint64_t> rel;         // file offsets relative to the batch's first byte
};

namespace {

#define HIP_TRY(expr)                       \
    do {                                    \
        if ((expr) != hipSuccess) {         \
            (void)hipGetLastError();        \
            return PREP_E_HIP;              \
        }                                   \
    } while (0)

// First and last source row (or column) whose pixels count in n_out outputs: the same
// fixed-point mapping as the resize kernel's, taps i and i + 1 clamped to the image; the
// second tap of the last output does not count where its weight is exactly zero.
void tap_span(uint64_t off, uint64_t scale, int n_out, int size, int *lo, int *hi)
{
    const uint64_t t_last = off + (uint64_t)(n_out - 1) * scale;
    const bool weighted = (t_last & ((1ull << kCoordFrac) - 1)) != 0;
    const int64_t first = (int64_t)(off >> kCoordFrac) - kCoordBias;
    const int64_t last = (int64_t)(t_last >> kCoordFrac) - kCoordBias + (weighted ? 1 : 0);
    *lo = (int)std::min<int64_t>(std::max<int64_t>(first, 0), size - 1);
    *hi = (int)std::min<int64_t>(std::max<int64_t>(last, 0), size - 1);
}

// The same for the antialiased filter: the first sample under the first output's triangle and
// the last under the last output's, by the kernel's own window arithmetic (a sample at the very
// edge of a triangle, weight zero, may be counted).
void window_span(uint64_t off, uint64_t scale, int n_out, int size, int *lo, int *hi)
{
    const uint64_t one = 1ull << kCoordFrac;
    const uint64_t support = std::max(scale, one);
    const uint64_t t_last = off + (uint64_t)(n_out - 1) * scale;
    const int64_t first = ((int64_t)(off + one - support) >> kCoordFrac) - kCoordBias;
    const int64_t last = (int64_t)((t_last + one + support) >> kCoordFrac) - kCoordBias - 1;
    *lo = (int)std::min<int64_t>(std::max<int64_t>(first, 0), size - 1);
    *hi = (int)std::min<int64_t>(std::max<int64_t>(last, 0), size - 1);
}

// Images with the same four Huffman tables share one expanded copy: the slot of image i's
// tables, found by the bytes of its DHT segments (BITS and HUFFVAL of the four tables), or
// kNoTableSlot when the handle's slots are used up.  h->parsed[i] must be filled.
uint32_t table_slot_of(prep_handle *h, const uint8_t *bits, const uint64_t *offsets, int32_t i)
{
    const ParsedImage &pi = h->parsed[(size_t)i];
    const uint8_t *file = bits + offsets[i];
    auto len_of = [](const ParsedImage &p, int t) { return 16u + std::min<uint32_t>(p.dht_nval[t], 256u); };
    uint64_t hash = 1469598103934665603ull;  // FNV-1a
    for (int t = 0; t < 4; t++)
        for (uint32_t k = 0; k < len_of(pi, t); k++) hash = (hash ^ file[pi.dht_off[t] + k]) * 1099511628211ull;
    const size_t mask = h->table_hash.size() - 1;  // a power of two, twice the slots
    for (size_t at = (size_t)hash & mask;; at = (at + 1) & mask) {
        const uint32_t entry = h->table_hash[at];
        if (entry == 0) {
            if (h->table_rep.size() >= h->table_slots) return kNoTableSlot;
            h->table_rep.push_back((uint32_t)i);
            h->table_hash[at] = (uint32_t)h->table_rep.size();
            return (uint32_t)h->table_rep.size() - 1;
        }
        const uint32_t j = h->table_rep[entry - 1];
        const ParsedImage &pj = h->parsed[j];
        const uint8_t *other = bits + offsets[j];
        bool same = true;
        for (int t = 0; t < 4 && same; t++)
            same = len_of(pi, t) == len_of(pj, t) &&
                   memcmp(file + pi.dht_off[t], other + pj.dht_off[t], len_of(pi, t)) == 0;
        if (same) return entry - 1;
    }
}

// Parse every file and lay the batch out in the workspace.
int plan_batch(prep_handle *h, const uint8_t *bits, const uint64_t *offsets, int32_t n,
               const prep_params *params, Plan *plan)
{
    h->parsed.resize((size_t)n);
    h->recs.resize((size_t)n);
    h->rr.resize((size_t)n);
    h->table_rep.clear();
    std::fill(h->table_hash.begin(), h->table_hash.end(), 0u);
    Plan P;
    uint64_t entropy_total = 0;
    for (int32_t i = 0; i < n; i++) {
        if (offsets[i + 1] < offsets[i]) return PREP_E_INVALID_ARG;
        ParsedImage &pi = h->parsed[(size_t)i];
        parse_image(bits + offsets[i], offsets[i + 1] - offsets[i], &pi);
        if (pi.info.status == PREP_OK) entropy_total += pi.info.entropy_bytes;
    }
    // a call with little data is cut into small windows, for the decoder variant that fills
    // the chip with hypotheses instead of walking whole restart intervals lane by lane
    if (entropy_total <= kSmallCallBytes && !(h->cfg.flags & PREP_FLAG_LARGE_WINDOWS))
        P.window_bytes = entropy_total <= kTinyCallBytes ? kTinyWindowBytes : kSmallWindowBytes;
    for (int32_t i = 0; i < n; i++) {
        ParsedImage &pi = h->parsed[(size_t)i];
        prep_image_info &I = pi.info;
        ImageRec &R = h->recs[(size_t)i];
        memset(&R, 0, sizeof R);
        ResizeRec &Z = h->rr[(size_t)i];
        memset(&Z, 0, sizeof Z);
        if (I.status == PREP_OK && (I.width > h->cfg.max_width || I.height > h->cfg.max_height))
            return PREP_E_TOO_LARGE;
        R.file_off = offsets[i];
        R.window0 = P.n_windows;
        R.group0 = P.n_groups;
        R.coef_block0 = (uint32_t)P.n_blocks;
        R.rgb_off = P.rgb_bytes;
        R.status = I.status;
        R.n_windows = 1;
        if (I.status == PREP_OK) {
            const int hs = luma_h(I.sampling);
            R.entropy_rel = (uint32_t)I.entropy_offset;
            R.entropy_len = (uint32_t)I.entropy_bytes;
            R.n_blocks = (uint32_t)((uint64_t)I.mcu_cols * I.mcu_rows * I.blocks_per_mcu);
            R.n_windows = (uint32_t)((I.entropy_bytes + P.window_bytes - 1) / P.window_bytes);
            if (R.n_windows == 0) R.n_windows = 1;
            R.rgb_pitch = (uint32_t)I.mcu_cols * 8u * hs * 3u;
            for (int t = 0; t < 4; t++) { R.dht_off[t] = pi.dht_off[t]; R.dht_nval[t] = pi.dht_nval[t]; }
            R.table_slot = table_slot_of(h, bits, offsets, i);
            for (int c = 0; c < 3; c++) R.dqt_off[c] = pi.dqt_off[c];
            R.width = (uint16_t)I.width;
            R.height = (uint16_t)I.height;
            R.mcu_cols = (uint16_t)I.mcu_cols;
            R.mcu_rows = (uint16_t)I.mcu_rows;
            R.restart_interval = (uint16_t)I.restart_interval;
            R.sampling = (uint8_t)I.sampling;
            R.blocks_per_mcu = (uint8_t)I.blocks_per_mcu;
            if (!make_resize_rec(I.width, I.height, params, R.rgb_off, R.rgb_pitch, &Z)) {
                // the crop window does not fit this image after resizing
                I.status = R.status = PREP_E_UNSUPPORTED;
            }
        }
        if (R.status == PREP_OK) {
            // Region of interest of the reconstruction, in groups of MCUs: the whole MCU grid,
            // or the MCUs whose pixels the crop window's bilinear taps read.
            const int per = recon_mcus_per_group(I.sampling);
            const int mcu_w = 8 * luma_h(I.sampling), mcu_h = 8 * luma_v(I.sampling);
            int x_lo = 0, x_hi = I.width - 1, y_lo = 0, y_hi = I.height - 1;
            if (!(h->cfg.flags & PREP_FLAG_FULL_RGB)) {
                const auto span = params->filter == PREP_FILTER_ANTIALIAS ? window_span : tap_span;
                span(Z.off_x, Z.scale_x, params->crop_w, I.width, &x_lo, &x_hi);
                span(Z.off_y, Z.scale_y, params->crop_h, I.height, &y_lo, &y_hi);
                if (h->cfg.flags & PREP_FLAG_SMOOTH_CHROMA) {
                    // an interpolated pixel also reads the chroma sample next to its own
                    x_lo = std::max(x_lo - luma_h(I.sampling), 0);
                    x_hi = std::min(x_hi + luma_h(I.sampling), (int)I.width - 1);
                    y_lo = std::max(y_lo - luma_v(I.sampling), 0);
                    y_hi = std::min(y_hi + luma_v(I.sampling), (int)I.height - 1);
                }
            }
            R.roi_row0 = (uint16_t)(y_lo / mcu_h);
            R.roi_rows = (uint16_t)(y_hi / mcu_h - y_lo / mcu_h + 1);
            R.roi_gcol0 = (uint16_t)(x_lo / mcu_w / per);
            R.roi_gcols = (uint16_t)(x_hi / mcu_w / per - x_lo / mcu_w / per + 1);
        }
        if (R.status == PREP_OK) {
            const uint64_t rows = (uint64_t)R.mcu_rows * 8u * (uint32_t)luma_v(R.sampling);
            P.n_blocks += R.n_blocks;
            P.rgb_bytes += ((uint64_t)R.rgb_pitch * rows + kRgbSlack + kRgbAlign - 1) / kRgbAlign * kRgbAlign;
            P.n_groups += (uint32_t)R.roi_gcols * R.roi_rows;
            const uint32_t region_cols = std::min<uint32_t>((uint32_t)(R.roi_gcol0 + R.roi_gcols) * (uint32_t)recon_mcus_per_group(R.sampling), R.mcu_cols) -
                                         (uint32_t)R.roi_gcol0 * (uint32_t)recon_mcus_per_group(R.sampling);
            P.max_region_pixels = std::max<uint32_t>(P.max_region_pixels,
                                                     region_cols * 8u * (uint32_t)luma_h(R.sampling) * (uint32_t)R.roi_rows * 8u * (uint32_t)luma_v(R.sampling));
        }
        P.n_windows += R.n_windows;
    }
    P.n_tables = (uint32_t)h->table_rep.size();
    // A reconstruction workgroup takes several groups of its image when there are plenty, so
    // that it can fetch one while it works on another; group0 counts workgroups.
    P.groups_per_wg = std::min<uint32_t>(std::max<uint32_t>(P.n_groups / kReconGroupsPerWgDivisor, 1u), kReconMaxGroupsPerWg);
    for (int32_t i = 0; i < n; i++) {
        ImageRec &R = h->recs[(size_t)i];
        R.group0 = P.recon_wgs;
        if (R.status == PREP_OK)
            P.recon_wgs += ((uint32_t)R.roi_gcols * R.roi_rows + P.groups_per_wg - 1) / P.groups_per_wg;
    }
    if (P.n_blocks > h->cap_blocks || P.rgb_bytes > h->cap_rgb || P.n_windows > h->cap_windows)
        return PREP_E_TOO_LARGE;
    *plan = P;
    return PREP_OK;
}

int take_slot(prep_handle *h, Slot **out)
{
    Slot &s = h->slot[h->next_slot];
    h->next_slot = (h->next_slot + 1) % kSlots;
    if (s.pending) {
        HIP_TRY(hipEventSynchronize(s.done));
        s.pending = false;
    }
    *out = &s;
    return PREP_OK;
}

int run_batch(prep_handle *h, const uint8_t *bits_host, const uint8_t *bits_dev,
              const uint64_t *offsets, int32_t n, const prep_params *params, void *out,
              hipStream_t stream, const int16_t *coef_host, uint64_t n_coef)
{
    if (!h || !bits_host || !offsets || !out || n < 0 || !params_ok(params)) return PREP_E_INVALID_ARG;
    if (n > h->cfg.max_batch) return PREP_E_TOO_LARGE;
    h->last_n = 0;
    if (n == 0) return PREP_OK;
    const uint64_t total = offsets[n] - offsets[0];
    if (offsets[n] < offsets[0] || total > h->cfg.max_bitstream_bytes) return PREP_E_TOO_LARGE;
    HIP_TRY(hipSetDevice(h->cfg.device));
    Plan P;
    // offsets are taken relative to the first file so that a batch may start anywhere
    const uint8_t *base_host = bits_host + offsets[0];
    std::vector<uint64_t> &rel = h->rel;
    rel.resize((size_t)n + 1);
    for (int32_t i = 0; i <= n; i++) {
        if (offsets[i] < offsets[0]) return PREP_E_INVALID_ARG;
        rel[(size_t)i] = offsets[i] - offsets[0];
    }
    // the slot first: its pinned buffer takes the bitstreams while the headers are parsed
    Slot *s;
    int rc = take_slot(h, &s);
    if (rc != PREP_OK) return rc;
    CopyPool *pool = !bits_dev && total >= kPooledCopyBytes && total <= h->cap_bits ? CopyPool::get() : nullptr;
    const bool pooled = pool && pool->start(s->h_bits, base_host, total);
    rc = plan_batch(h, base_host, rel.data(), n, params, &P);
    if (rc == PREP_OK && coef_host && n_coef != P.n_blocks * 64) rc = PREP_E_INVALID_ARG;
    if (pooled) pool->wait();
    if (rc != PREP_OK) return rc;
    place_block(s, (size_t)n);
    memcpy(s->h_recs, h->recs.data(), sizeof(ImageRec) * (size_t)n);
    // the first reconstruction workgroup of every image, packed behind the records: the
    // kernel finds its image by counting the entries that do not exceed its index
    uint32_t *h_group0 = reinterpret_cast<uint32_t *>(s->h_recs + n);
    for (int32_t i = 0; i < n; i++) h_group0[i] = h->recs[(size_t)i].group0;
    for (uint32_t t = 0; t < P.n_tables; t++) h_group0[n + (int32_t)t] = h->table_rep[t];
    for (int32_t i = 0; i < n; i++) s->h_data_end[i] = h->recs[(size_t)i].entropy_len;
    memcpy(s->h_rr, h->rr.data(), sizeof(ResizeRec) * (size_t)n);
    // Large uploads go on the handle's copy stream and the caller's stream waits for them, so
    // that they overlap the kernels of the call before.  Small ones stay on the caller's
    // stream: there the hop between streams costs more than it hides (with several handles
    // at work it also couples their streams through the few hardware queues).
    const bool aside = (!bits_dev && total >= kCopyStreamMinBytes) || n >= kCopyStreamMinImages;
    hipStream_t up = aside ? h->copy_stream : stream;
    const uint8_t *d_bits = bits_dev ? bits_dev + offsets[0] : s->d_bits;
    if (!bits_dev) {
        if (!pooled) memcpy(s->h_bits, base_host, total);
        HIP_TRY(hipMemcpyAsync(s->d_bits, s->h_bits, total, hipMemcpyHostToDevice, up));
    }
    HIP_TRY(hipMemcpyAsync(s->d_block, s->h_block, block_bytes((size_t)n), hipMemcpyHostToDevice, up));
    if (aside) {
        HIP_TRY(hipEventRecord(s->copied, h->copy_stream));
        HIP_TRY(hipStreamWaitEvent(stream, s->copied, 0));
    }
    const bool timing = h->timing;
    hipEvent_t *ev = timing ? &h->ev[(size_t)(h->timed_calls % kTimedCalls) * 5] : nullptr;
    if (timing) HIP_TRY(hipEventRecord(ev[0], stream));
    if (coef_host) {
        for (int32_t i = 0; i < n; i++) s->h_status[i] = h->recs[(size_t)i].status;
        HIP_TRY(hipMemcpyAsync(h->d_status, s->h_status, sizeof(int32_t) * (size_t)n, hipMemcpyHostToDevice, stream));
        if (P.n_blocks)
            HIP_TRY(hipMemcpyAsync(h->d_coef, coef_host, P.n_blocks * 128, hipMemcpyHostToDevice, stream));
        if (timing) { HIP_TRY(hipEventRecord(ev[1], stream)); HIP_TRY(hipEventRecord(ev[2], stream)); }
    } else {
        // (P.n_windows >= n > 0: the scan also sets every image's status)
        launch_scan_restart_markers(d_bits, s->d_recs, n, P.n_windows, P.window_bytes, h->d_win_count, h->d_win_first,
                                    s->d_data_end,
                                    h->d_status, reinterpret_cast<const uint32_t *>(s->d_recs + n) + n,
                                    P.n_tables, h->d_tables, stream);
        if (timing) HIP_TRY(hipEventRecord(ev[1], stream));
        launch_decode_entropy(d_bits, s->d_recs, n, P.n_windows, h->d_win_count, h->d_win_first, s->d_data_end,
                              h->d_coef, (uint32_t)(h->cap_blocks * 64), h->d_status, h->d_tables,
                              P.window_bytes != (uint32_t)kWindowBytes,
                              P.window_bytes == (uint32_t)kTinyWindowBytes ? 256u : 512u, stream);
        if (timing) HIP_TRY(hipEventRecord(ev[2], stream));
    }
    launch_reconstruct(d_bits, s->d_recs, reinterpret_cast<const uint32_t *>(s->d_recs + n), n, P.recon_wgs,
                       P.groups_per_wg, h->d_coef, h->d_rgb, h->d_chroma, P.max_region_pixels, stream);
    if (timing) HIP_TRY(hipEventRecord(ev[3], stream));
    launch_resize_normalize(h->d_rgb, s->d_rr, h->d_status, n, params->crop_h, params->crop_w,
                            params->out_dtype, params->filter, s->h_rr, params->mean,
                            params->std, out, true, stream);
    if (timing) HIP_TRY(hipEventRecord(ev[4], stream));
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipEventRecord(s->done, stream));
    s->pending = true;
    if (timing) h->timed_calls++;
    h->last_n = n;
    h->last_stream = stream;
    return PREP_OK;
}

}  // namespace

extern "C" {

int prep_create(prep_handle **out, const prep_config *cfg)
{
    if (!out) return PREP_E_INVALID_ARG;
    *out = nullptr;
    if (!cfg || cfg->max_batch < 1 || cfg->max_batch > 65535 || cfg->max_width < 1 ||
        cfg->max_height < 1 || cfg->max_width > 65535 || cfg->max_height > 65535 ||
        cfg->max_bitstream_bytes < 1 || cfg->max_bitstream_bytes > 0x7FFF0000ull ||
        (cfg->flags & ~(uint32_t)(PREP_FLAG_TABLES_PER_WORKGROUP | PREP_FLAG_FULL_RGB | PREP_FLAG_SMOOTH_CHROMA | PREP_FLAG_LARGE_WINDOWS)) != 0)
        return PREP_E_INVALID_ARG;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || cfg->device < 0 || cfg->device >= ndev) {
        (void)hipGetLastError();
        return PREP_E_HIP;
    }
    prep_handle *h = new (std::nothrow) prep_handle;
    if (!h) return PREP_E_NOMEM;
    h->cfg = *cfg;
    const uint64_t n = (uint64_t)cfg->max_batch;
    const uint64_t wh = (uint64_t)cfg->max_width * cfg->max_height;
    uint64_t px = cfg->max_total_pixels ? cfg->max_total_pixels : n * wh;
    if (px > n * wh) px = n * wh;
    // padded to whole 16x16 MCUs an image of w x h has at most (w+15)(h+15) pixels
    const uint64_t padded = px + 15ull * n * ((uint64_t)cfg->max_width + cfg->max_height) + 225ull * n;
    h->cap_blocks = padded * 3 / 64 + 6 * n;       // 4:4:4 worst case: 3 blocks per 64 pixels
    h->cap_rgb = padded * 3 + (kRgbAlign + kRgbSlack) * n;
    // (windows of either size: a call cut into small ones holds at most kSmallCallBytes)
    h->cap_windows = std::max<uint64_t>(cfg->max_bitstream_bytes / kWindowBytes,
                                        std::max<uint64_t>(std::min<uint64_t>(cfg->max_bitstream_bytes, kSmallCallBytes) / kSmallWindowBytes,
                                                           std::min<uint64_t>(cfg->max_bitstream_bytes, kTinyCallBytes) / kTinyWindowBytes)) + n + 1;
    h->cap_bits = cfg->max_bitstream_bytes + kBitsPad;
    // (the kernels index the workspace and its side array with 32-bit element offsets)
    if (h->cap_blocks * 65 > 0xFFFFFFFFull) { delete h; return PREP_E_TOO_LARGE; }

    bool ok = hipSetDevice(cfg->device) == hipSuccess;
    ok = ok && hipStreamCreateWithFlags(&h->copy_stream, hipStreamNonBlocking) == hipSuccess;
    // 64 coefficients per block, and behind them one more int16 per block: the DC differences
    // between the decoder's two steps
    ok = ok && hipMalloc((void **)&h->d_coef, h->cap_blocks * 130 + 16) == hipSuccess;
    ok = ok && hipMalloc((void **)&h->d_rgb, h->cap_rgb) == hipSuccess;
    if (cfg->flags & PREP_FLAG_SMOOTH_CHROMA)
        ok = ok && hipMalloc((void **)&h->d_chroma, h->cap_rgb / 3 + 16) == hipSuccess;
    h->table_slots = (cfg->flags & PREP_FLAG_TABLES_PER_WORKGROUP) ? 0u : std::min<uint32_t>((uint32_t)n, kMaxTableSlots);
    h->table_rep.reserve(h->table_slots);
    h->table_hash.assign(2 * (size_t)kMaxTableSlots, 0u);
    ok = ok && hipMalloc((void **)&h->d_tables, (size_t)std::max<uint32_t>(h->table_slots, 1u) * huff_tables_bytes()) == hipSuccess;
    ok = ok && hipMalloc((void **)&h->d_status, sizeof(int32_t) * n) == hipSuccess;
    ok = ok && hipMalloc((void **)&h->d_win_count, sizeof(uint32_t) * h->cap_windows) == hipSuccess;
    ok = ok && hipMalloc((void **)&h->d_win_first, sizeof(uint32_t) * h->cap_windows) == hipSuccess;
    for (int i = 0; ok && i < kSlots; i++) {
        Slot &s = h->slot[i];
        ok = ok && hipHostMalloc((void **)&s.h_bits, h->cap_bits, hipHostMallocDefault) == hipSuccess;
        ok = ok && hipHostMalloc((void **)&s.h_block, block_bytes(n), hipHostMallocDefault) == hipSuccess;
        ok = ok && hipHostMalloc((void **)&s.h_status, sizeof(int32_t) * n, hipHostMallocDefault) == hipSuccess;
        ok = ok && hipMalloc((void **)&s.d_bits, h->cap_bits) == hipSuccess;
        ok = ok && hipMalloc((void **)&s.d_block, block_bytes(n)) == hipSuccess;
        ok = ok && hipEventCreateWithFlags(&s.copied, hipEventDisableTiming) == hipSuccess;
        ok = ok && hipEventCreateWithFlags(&s.done, hipEventDisableTiming) == hipSuccess;
    }
    h->ev.assign((size_t)kTimedCalls * 5, nullptr);
    for (size_t i = 0; ok && i < h->ev.size(); i++) ok = hipEventCreate(&h->ev[i]) == hipSuccess;
    if (ok) ok = hipMemset(h->d_status, 0, sizeof(int32_t) * n) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        prep_destroy(h);
        return PREP_E_NOMEM;
    }
    *out = h;
    return PREP_OK;
}

int prep_destroy(prep_handle *h)
{
    if (!h) return PREP_E_INVALID_ARG;
    (void)hipSetDevice(h->cfg.device);
    (void)hipDeviceSynchronize();
    (void)hipFree(h->d_coef);
    (void)hipFree(h->d_rgb);
    (void)hipFree(h->d_chroma);
    (void)hipFree(h->d_tables);
    (void)hipFree(h->d_status);
    (void)hipFree(h->d_win_count);
    (void)hipFree(h->d_win_first);
    for (int i = 0; i < kSlots; i++) {
        Slot &s = h->slot[i];
        if (s.h_bits) (void)hipHostFree(s.h_bits);
        if (s.h_block) (void)hipHostFree(s.h_block);
        if (s.h_status) (void)hipHostFree(s.h_status);
        (void)hipFree(s.d_bits);
        (void)hipFree(s.d_block);
        if (s.copied) (void)hipEventDestroy(s.copied);
        if (s.done) (void)hipEventDestroy(s.done);
    }
    for (hipEvent_t e : h->ev)
        if (e) (void)hipEventDestroy(e);
    if (h->copy_stream) (void)hipStreamDestroy(h->copy_stream);
    (void)hipGetLastError();
    delete h;
    return PREP_OK;
}

int prep_decode_resize_batch(prep_handle *h, const uint8_t *bitstreams, const uint64_t *offsets,
                             int32_t n, const prep_params *params, void *out, void *stream)
{
    return run_batch(h, bitstreams, nullptr, offsets, n, params, out, (hipStream_t)stream, nullptr, 0);
}

int prep_decode_resize_batch_resident(prep_handle *h, const uint8_t *bitstreams,
                                      const uint8_t *bitstreams_device, const uint64_t *offsets,
                                      int32_t n, const prep_params *params, void *out, void *stream)
{
    if (!bitstreams_device) return PREP_E_INVALID_ARG;
    return run_batch(h, bitstreams, bitstreams_device, offsets, n, params, out, (hipStream_t)stream,
                     nullptr, 0);
}

int prep_reconstruct_from_coefficients(prep_handle *h, const uint8_t *bitstreams,
                                       const uint64_t *offsets, int32_t n,
                                       const int16_t *coefficients, uint64_t n_coefficients,
                                       const prep_params *params, void *out, void *stream)
{
    if (!coefficients) return PREP_E_INVALID_ARG;
    int rc = run_batch(h, bitstreams, nullptr, offsets, n, params, out, (hipStream_t)stream,
                       coefficients, n_coefficients);
    // the coefficients were copied from pageable memory: make sure the copy is over
    if (rc == PREP_OK && hipStreamSynchronize((hipStream_t)stream) != hipSuccess) rc = PREP_E_HIP;
    return rc;
}

int prep_get_status(prep_handle *h, int32_t *per_image_status, int32_t n)
{
    if (!h || !per_image_status || n < 0 || n > h->last_n) return PREP_E_INVALID_ARG;
    if (n == 0) return PREP_OK;
    HIP_TRY(hipSetDevice(h->cfg.device));
    HIP_TRY(hipStreamSynchronize(h->last_stream));
    HIP_TRY(hipMemcpy(per_image_status, h->d_status, sizeof(int32_t) * (size_t)n, hipMemcpyDeviceToHost));
    for (int32_t i = 0; i < n; i++)
        if (h->recs[(size_t)i].status != PREP_OK) per_image_status[i] = h->recs[(size_t)i].status;
    return PREP_OK;
}

const char *prep_strerror(int code)
{
    switch (code) {
    case PREP_OK: return "ok";
    case PREP_E_INVALID_ARG: return "invalid argument";
    case PREP_E_TOO_LARGE: return "batch exceeds the capacity the handle was created with";
    case PREP_E_HIP: return "HIP runtime call failed";
    case PREP_E_UNSUPPORTED: return "JPEG outside the supported baseline subset";
    case PREP_E_CORRUPT: return "corrupt JPEG stream";
    case PREP_E_NOMEM: return "out of memory";
    default: return "unknown error code";
    }
}

int prep_parse_headers(const uint8_t *bitstreams, const uint64_t *offsets, int32_t n,
                       prep_image_info *info)
{
    if (!bitstreams || !offsets || !info || n < 0) return PREP_E_INVALID_ARG;
    for (int32_t i = 0; i < n; i++) {
        if (offsets[i + 1] < offsets[i]) return PREP_E_INVALID_ARG;
        ParsedImage p;
        parse_image(bitstreams + offsets[i], offsets[i + 1] - offsets[i], &p);
        info[i] = p.info;
    }
    return PREP_OK;
}

int64_t prep_interval_descriptors(const prep_image_info *info, int32_t n, prep_interval_desc *desc,
                                  int64_t cap)
{
    if (!info || n < 0 || cap < 0 || (cap > 0 && !desc)) return PREP_E_INVALID_ARG;
    int64_t k = 0;
    for (int32_t i = 0; i < n; i++) {
        if (info[i].status != PREP_OK) continue;
        const int64_t nmcu = (int64_t)info[i].mcu_cols * info[i].mcu_rows;
        const int64_t ri = info[i].restart_interval > 0 ? info[i].restart_interval : nmcu;
        for (int64_t m = 0, j = 0; m < nmcu; m += ri, j++, k++) {
            if (k < cap) {
                desc[k].image = i;
                desc[k].first_mcu = (int32_t)m;
                desc[k].n_mcu = (int32_t)(nmcu - m < ri ? nmcu - m : ri);
                desc[k].rst_index = j == 0 ? -1 : (int32_t)((j - 1) & 7);
            }
        }
    }
    return k;
}

int prep_resize_normalize(prep_handle *h, const uint8_t *rgb, const uint64_t *rgb_offsets,
                          const int32_t *widths, const int32_t *heights, const int32_t *pitches,
                          int32_t n, const prep_params *params, void *out, void *stream)
{
    if (!h || !rgb || !rgb_offsets || !widths || !heights || !pitches || !out || n < 0 ||
        !params_ok(params))
        return PREP_E_INVALID_ARG;
    if (n > h->cfg.max_batch) return PREP_E_TOO_LARGE;
    if (n == 0) return PREP_OK;
    HIP_TRY(hipSetDevice(h->cfg.device));
    Slot *s;
    int rc = take_slot(h, &s);
    if (rc != PREP_OK) return rc;
    place_block(s, (size_t)n);
    for (int32_t i = 0; i < n; i++) {
        if (widths[i] < 1 || heights[i] < 1 || pitches[i] < widths[i] * 3) return PREP_E_INVALID_ARG;
        if (!make_resize_rec(widths[i], heights[i], params, rgb_offsets[i], (uint32_t)pitches[i], &s->h_rr[i]))
            return PREP_E_INVALID_ARG;
    }
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(hipMemcpyAsync(s->d_rr, s->h_rr, sizeof(ResizeRec) * (size_t)n, hipMemcpyHostToDevice, st));
    launch_resize_normalize(rgb, s->d_rr, nullptr, n, params->crop_h, params->crop_w,
                            params->out_dtype, params->filter, s->h_rr, params->mean,
                            params->std, out, false, st);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipEventRecord(s->done, st));
    s->pending = true;
    return PREP_OK;
}

int64_t prep_debug_last_coefficients(prep_handle *h, int32_t image, int16_t *host_out, uint64_t cap)
{
    if (!h || !host_out || image < 0 || image >= h->last_n) return PREP_E_INVALID_ARG;
    const ImageRec &R = h->recs[(size_t)image];
    if (R.status != PREP_OK) return R.status;
    const uint64_t count = (uint64_t)R.n_blocks * 64;
    if (cap < count) return PREP_E_INVALID_ARG;
    HIP_TRY(hipSetDevice(h->cfg.device));
    HIP_TRY(hipStreamSynchronize(h->last_stream));
    HIP_TRY(hipMemcpy(host_out, h->d_coef + (size_t)R.coef_block0 * 64, count * 2, hipMemcpyDeviceToHost));
    return (int64_t)count;
}

int64_t prep_debug_last_rgb(prep_handle *h, int32_t image, uint8_t *host_out_hwc, uint64_t cap)
{
    if (!h || !host_out_hwc || image < 0 || image >= h->last_n) return PREP_E_INVALID_ARG;
    const ImageRec &R = h->recs[(size_t)image];
    if (R.status != PREP_OK) return R.status;
    const uint64_t row = (uint64_t)R.width * 3, count = row * R.height;
    if (cap < count) return PREP_E_INVALID_ARG;
    HIP_TRY(hipSetDevice(h->cfg.device));
    HIP_TRY(hipStreamSynchronize(h->last_stream));
    HIP_TRY(hipMemcpy2D(host_out_hwc, row, h->d_rgb + R.rgb_off, R.rgb_pitch, row, R.height,
                        hipMemcpyDeviceToHost));
    return (int64_t)count;
}

int prep_debug_last_region(prep_handle *h, int32_t image, int32_t rect[4])
{
    if (!h || !rect || image < 0 || image >= h->last_n) return PREP_E_INVALID_ARG;
    const ImageRec &R = h->recs[(size_t)image];
    if (R.status != PREP_OK) return R.status;
    const int mcu_h = 8 * luma_v(R.sampling);
    const int group_px = 8 * luma_h(R.sampling) * recon_mcus_per_group(R.sampling);
    rect[0] = std::min<int>(R.roi_gcol0 * group_px, R.width);
    rect[1] = std::min<int>(R.roi_row0 * mcu_h, R.height);
    rect[2] = std::min<int>((R.roi_gcol0 + R.roi_gcols) * group_px, R.width);
    rect[3] = std::min<int>((R.roi_row0 + R.roi_rows) * mcu_h, R.height);
    if ((h->cfg.flags & PREP_FLAG_SMOOTH_CHROMA) && R.sampling != PREP_SAMPLING_GRAY) {
        // interpolated chroma is exact up to the last chroma sample but one of the region,
        // except where the region ends with the image
        const int fx = luma_h(R.sampling) > 1 ? luma_h(R.sampling) : 0, fy = luma_v(R.sampling) > 1 ? luma_v(R.sampling) : 0;
        if (rect[0] > 0) rect[0] += fx;
        if (rect[1] > 0) rect[1] += fy;
        if ((R.roi_gcol0 + R.roi_gcols) * recon_mcus_per_group(R.sampling) < R.mcu_cols) rect[2] -= fx;
        if (R.roi_row0 + R.roi_rows < R.mcu_rows) rect[3] -= fy;
    }
    return PREP_OK;
}

int prep_set_timing(prep_handle *h, int32_t enabled)
{
    if (!h) return PREP_E_INVALID_ARG;
    h->timing = enabled != 0;
    h->timed_calls = 0;
    return PREP_OK;
}

int prep_stage_ms(prep_handle *h, int32_t calls_back, float ms[4])
{
    if (!h || !ms || calls_back < 0 || calls_back >= kTimedCalls ||
        (uint64_t)calls_back >= h->timed_calls)
        return PREP_E_INVALID_ARG;
    const hipEvent_t *ev = &h->ev[(size_t)((h->timed_calls - 1 - (uint64_t)calls_back) % kTimedCalls) * 5];
    HIP_TRY(hipSetDevice(h->cfg.device));
    HIP_TRY(hipEventSynchronize(ev[4]));
    for (int i = 0; i < 4; i++) HIP_TRY(hipEventElapsedTime(&ms[i], ev[i], ev[i + 1]));
    return PREP_OK;
}

}  // extern "C"
