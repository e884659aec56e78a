// GPU Huffman entropy decoder for baseline JPEG (T.81 F.2.2), gfx950.
//
// The first half of the "Decode" functional unit (PREBA section 4.2, Table 1).
// The FPGA decodes one stream serially per compute unit; here one workgroup owns
// a run of whole restart intervals (T.81 E.2.4) of one image and decodes it with
// all of its lanes by self-synchronisation:
//
//   1. scan_restart_markers counts the RSTn markers in fixed windows of every
//      image's entropy-coded segment, so that a workgroup starting at the first
//      marker of its window knows which restart interval (hence which MCU) it
//      starts at, without any serial pass over the stream.
//   2. decode_entropy stages a chunk of the stream in LDS with byte stuffing
//      (FF 00) and markers removed, gives every lane one fixed-size subsequence,
//      and lets each lane decode from a guessed state (code-word boundary, block
//      0 of an MCU, DC coefficient).  Lane j then re-decodes from the end state
//      lane j-1 reached, until no end state changes.  Lane 0 starts from a known
//      state, so the fixed point is the sequential decode, exactly.  Restart
//      boundaries inside the chunk are hard synchronisation points.
//   3. A prefix sum of the blocks each lane completed gives every lane its
//      absolute block index; a last pass decodes once more from the now-true
//      start states and writes the coefficients; DC differences are turned into
//      absolute values with a segmented scan over the lanes.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/prep.h"
#include "kernels.h"
#include "prep_internal.h"

namespace prep {

namespace {

constexpr int kT = kDecodeThreads;
constexpr int kCleanWords = kChunkRaw / 4 + 8;      // destuffed stream + zero tail
constexpr int kMaskWords = kChunkRaw / 32 + 2;      // one bit per clean byte
constexpr uint32_t kNoMarker = 0xFFFFFFFFu;
constexpr uint32_t kSubBits = kSubseqBytes * 8;
static_assert(kSubseqBytes == 64, "one 64-bit keep mask per lane");

struct HuffTable {
    uint16_t lut[1 << kLutBits];   // (length << 8) | symbol for codes up to kLutBits bits, else 0
    int32_t first[17];             // first code of each length
    int32_t count[17];             // BITS
    int32_t valptr[17];            // index of the first symbol of each length
    uint8_t huffval[256];
};

struct DecodeShared {
    uint32_t clean[kCleanWords];   // big-endian packed: bit 31 of a word is the earliest bit
    uint32_t bmask[kMaskWords];    // bit q set: a restart interval begins at clean byte q
    uint32_t next_boundary[kT + 1];  // first interval start at or after the lane's subsequence
    HuffTable tab[4];              // DC luma, AC luma, DC chroma, AC chroma
    unsigned long long keep[kT];   // which of the lane's 64 raw bytes survived destuffing
    uint32_t keep_off[kT + 1];     // clean offset of the lane's first surviving byte
    uint32_t state[kT];            // end state of every subsequence
    uint32_t scan_a[kT / 64 + 1];  // per-wave totals for workgroup scans
    int32_t dc_val[3][kT / 64 + 1];
    int32_t dc_flag[3][kT / 64 + 1];
    uint32_t bcast[8];
};

__device__ inline uint32_t pack_state(uint32_t p, uint32_t blk, uint32_t zz)
{
    return (p << 9) | (blk << 6) | zz;
}

// ---- workgroup-wide helpers (kT threads, wave64) ---------------------------

__device__ inline uint32_t wave_incl_scan(uint32_t v)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t o = __shfl_up(v, d, 64);
        if (lane >= d) v += o;
    }
    return v;
}

// exclusive prefix sum over the workgroup; *total receives the sum
__device__ inline uint32_t block_excl_scan(uint32_t v, uint32_t *wave_tot, uint32_t *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = wave_incl_scan(v);
    __syncthreads();
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kT / 64; w++) {
        uint32_t t = wave_tot[w];
        if (w < wave) base += t;
        tot += t;
    }
    *total = tot;
    return base + inc - v;
}

// Segmented running sum (value, reset flag): a reset discards what came before.
// Returns the value carried INTO this lane (exclusive); carry_in seeds lane 0.
__device__ inline int32_t block_seg_excl_scan(int32_t v, int32_t f, int32_t carry_in,
                                              int32_t *wave_val, int32_t *wave_flag,
                                              int32_t *carry_out)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int32_t iv = v, ifl = f;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int32_t ov = __shfl_up(iv, d, 64);
        int32_t of = __shfl_up(ifl, d, 64);
        if (lane >= d) {
            if (!ifl) iv += ov;
            ifl |= of;
        }
    }
    __syncthreads();
    if (lane == 63) { wave_val[wave] = iv; wave_flag[wave] = ifl; }
    __syncthreads();
    // carry into this wave
    int32_t cv = carry_in, all_v = carry_in;
#pragma unroll
    for (int w = 0; w < kT / 64; w++) {
        int32_t wv = wave_val[w], wf = wave_flag[w];
        int32_t nv = wf ? wv : all_v + wv;
        if (w < wave) cv = nv;
        all_v = nv;
    }
    *carry_out = all_v;
    // exclusive value for this lane: inclusive of the previous lane
    int32_t pv = __shfl_up(iv, 1, 64);
    int32_t pf = __shfl_up(ifl, 1, 64);
    if (lane == 0) return cv;
    return pf ? pv : cv + pv;
}

// ---- bit-level decoding ------------------------------------------------------

struct Geometry {
    uint32_t bpm;        // blocks per MCU
    uint32_t n_luma;     // luma blocks per MCU (blocks >= n_luma use the chroma tables)
    uint32_t ri_blocks;  // blocks per restart interval, 0 = none
    uint32_t n_blocks;   // blocks in the image
};

__device__ inline uint32_t comp_of_block(const Geometry &g, uint32_t blk_in_mcu)
{
    return blk_in_mcu < g.n_luma ? 0u : blk_in_mcu - g.n_luma + 1u;
}

// first interval start at or after clean byte q (in bits), limit if none
__device__ inline uint32_t boundary_from(const DecodeShared &S, uint32_t q, uint32_t limit_bits)
{
    uint32_t j = q >> 6;
    if (j >= (uint32_t)kT) return limit_bits;
    unsigned long long m = ((unsigned long long)S.bmask[2 * j + 1] << 32) | S.bmask[2 * j];
    m >>= (q & 63);
    uint32_t r = m ? q + (uint32_t)__builtin_ctzll(m) : S.next_boundary[j + 1];
    r = r > 0x0FFFFFFFu ? limit_bits : r * 8u;
    return r < limit_bits ? r : limit_bits;
}

struct WriteCtx {
    int16_t *coef;       // this image's first block
    uint32_t block;      // absolute index of the block being decoded
    int32_t dcsum[3];    // running DC per component since the lane began or the last reset
    int32_t dcreset[3];
    uint32_t dc_first;   // first block whose DC this lane decoded
    uint32_t dc_count;
    int32_t need_restart;  // the next thing in the stream must be a restart boundary
    int32_t bad;
};

__device__ inline bool first_of_interval(const Geometry &g, uint32_t block)
{
    // the first block of each component in the first MCU of an interval restarts DC prediction
    uint32_t r = g.ri_blocks ? block % g.ri_blocks : block;
    return r == 0 || (r >= g.n_luma && r < g.bpm);
}

// Decode from packed state `st` until the bit position reaches end_bit.
// limit_bits = end of the staged data.  Returns the end state; *nblk = blocks completed.
template <bool kWrite>
__device__ inline uint32_t decode_span(const DecodeShared &S, const Geometry &g, uint32_t st,
                                       uint32_t end_bit, uint32_t limit_bits, uint32_t *nblk,
                                       WriteCtx *wc)
{
    uint32_t p = st >> 9, blk = (st >> 6) & 7u, zz = st & 63u;
    uint32_t done = 0;
    uint32_t widx = p >> 5;
    uint64_t acc;
    int cnt;
    auto reload = [&]() {
        widx = p >> 5;
        uint32_t w0 = S.clean[min(widx, (uint32_t)kCleanWords - 1)];
        uint32_t w1 = S.clean[min(widx + 1, (uint32_t)kCleanWords - 1)];
        acc = (((uint64_t)w0 << 32) | w1) << (p & 31);
        cnt = 64 - (int)(p & 31);
        widx += 2;
    };
    reload();
    uint32_t nb = boundary_from(S, (p + 7) >> 3, limit_bits);
    while (p < end_bit) {
        const bool dc = zz == 0;
        const HuffTable &T = S.tab[(blk >= g.n_luma ? 2u : 0u) + (dc ? 0u : 1u)];
        uint32_t e = T.lut[(uint32_t)(acc >> (64 - kLutBits))];
        uint32_t len = e >> 8, sym = e & 255u;
        bool found = true;
        if (len == 0) {  // code longer than the first-level table, or no code at all
            const uint32_t peek = (uint32_t)(acc >> 48);
            len = 16;
            sym = 0;
            found = false;
            for (int l = kLutBits + 1; l <= 16; l++) {
                int32_t c = (int32_t)(peek >> (16 - l)) - T.first[l];
                if (c >= 0 && c < T.count[l]) {
                    len = l;
                    sym = T.huffval[(T.valptr[l] + c) & 255];
                    found = true;
                    break;
                }
            }
        }
        const uint32_t s = sym & 15u;
        const uint32_t adv = len + s;
        if (kWrite && wc->need_restart && p + adv <= nb) wc->bad = 1;  // a restart marker is missing
        if (p + adv > nb) {
            // the symbol does not fit before the next restart boundary / end of data
            if (nb >= limit_bits) {
                if (kWrite && (blk != 0 || zz != 0 || limit_bits - p >= 8)) wc->bad = 1;
                p = limit_bits;
                break;
            }
            if (kWrite) {
                if (blk != 0 || zz != 0 || nb - p >= 8) wc->bad = 1;
                if (g.ri_blocks == 0 || wc->block % g.ri_blocks != 0) wc->bad = 1;
                wc->need_restart = 0;
            }
            p = nb;
            blk = 0;
            zz = 0;
            reload();
            nb = boundary_from(S, (p >> 3) + 1, limit_bits);
            continue;
        }
        if (kWrite && !found) wc->bad = 1;  // bits that are no code word (padding is met above)
        // appended bits (T.81 F.2.2.4 RECEIVE) and sign extension (F.2.2.1 EXTEND)
        const uint32_t after = (uint32_t)((acc << len) >> 32);
        const uint32_t extra = s ? after >> (32 - s) : 0u;
        const int32_t val = s ? ((extra >> (s - 1)) ? (int32_t)extra
                                                    : (int32_t)extra - (int32_t)((1u << s) - 1u))
                              : 0;
        acc <<= adv;
        cnt -= (int)adv;
        p += adv;
        if (cnt < 32) {
            uint32_t w = S.clean[min(widx, (uint32_t)kCleanWords - 1)];
            widx++;
            acc |= (uint64_t)w << (32 - cnt);
            cnt += 32;
        }
        if (dc) {
            if (kWrite) {
                if (sym > 11) wc->bad = 1;
                if (wc->block < g.n_blocks) {
                    const uint32_t c = comp_of_block(g, blk);
                    if (first_of_interval(g, wc->block)) {
                        wc->dcsum[c] = val;
                        wc->dcreset[c] = 1;
                    } else {
                        wc->dcsum[c] += val;
                    }
                    wc->coef[(size_t)wc->block * 64] = (int16_t)wc->dcsum[c];
                    if (wc->dc_count == 0) wc->dc_first = wc->block;
                    wc->dc_count++;
                } else {
                    wc->bad = 1;
                }
            }
            zz = 1;
        } else {
            const uint32_t r = sym >> 4;
            if (s == 0) {
                zz = (r == 15) ? zz + 16 : 64;  // ZRL or end of block
            } else {
                zz += r;
                if (zz < 64) {
                    if (kWrite && wc->block < g.n_blocks)
                        wc->coef[(size_t)wc->block * 64 + zz] = (int16_t)val;
                } else if (kWrite) {
                    wc->bad = 1;
                }
                zz++;
            }
        }
        if (zz >= 64) {
            zz = 0;
            blk = blk + 1 == g.bpm ? 0 : blk + 1;
            done++;
            if (kWrite) {
                wc->block++;
                if (g.ri_blocks && wc->block % g.ri_blocks == 0 && wc->block < g.n_blocks)
                    wc->need_restart = 1;
            }
        }
    }
    *nblk = done;
    return pack_state(p, blk, zz);
}

__device__ inline uint32_t load_byte(const uint8_t *p) { return *p; }

// binary search: largest i with key(i) <= x over records sorted by a uint32 field
template <typename F>
__device__ inline int find_image(int n, uint32_t x, F key)
{
    int lo = 0, hi = n - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (key(mid) <= x) lo = mid; else hi = mid - 1;
    }
    return lo;
}

}  // namespace

// ---- kernel 1: restart markers per window -----------------------------------
// window w of an image = raw bytes [w*kWindowBytes, (w+1)*kWindowBytes) of its
// entropy-coded segment.  cnt = RSTn markers whose FF byte lies in the window,
// first = offset (from the segment start) of the first such FF byte.
__global__ __launch_bounds__(kDecodeThreads) void scan_restart_markers(
    const uint8_t *__restrict__ bits, const ImageRec *__restrict__ recs, int n_images,
    uint32_t *__restrict__ win_count, uint32_t *__restrict__ win_first,
    int32_t *__restrict__ status)
{
    __shared__ uint32_t s_cnt[kT / 64], s_first[kT / 64];
    const uint32_t wg = blockIdx.x;
    const int img = find_image(n_images, wg, [&](int i) { return recs[i].window0; });
    const ImageRec &R = recs[img];
    const uint32_t w = wg - R.window0;
    // the per-image verdict starts as the host parser's; the decoder may lower it
    if (w == 0 && threadIdx.x == 0) status[img] = R.status;
    uint32_t cnt = 0, first = kNoMarker;
    if (R.status == PREP_OK && R.restart_interval != 0 && w < R.n_windows) {
        const uint8_t *seg = bits + R.file_off + R.entropy_rel;
        const uint32_t lo = w * (uint32_t)kWindowBytes;
        const uint32_t hi = min(lo + (uint32_t)kWindowBytes, R.entropy_len);
        constexpr uint32_t per = kWindowBytes / kT;
        uint32_t a = lo + threadIdx.x * per;
        uint32_t b = min(a + per, hi);
        if (a < b) {
            uint32_t prev = load_byte(seg + a);
            for (uint32_t i = a; i < b; i++) {
                // the byte after the last one of the segment is the EOI marker's FF
                uint32_t next = i + 1 < R.entropy_len ? load_byte(seg + i + 1) : 0xFFu;
                if (prev == 0xFFu && next >= 0xD0u && next <= 0xD7u) {
                    cnt++;
                    if (first == kNoMarker) first = i;
                }
                prev = next;
            }
        }
    }
    // workgroup reduction
    for (int d = 32; d >= 1; d >>= 1) {
        cnt += __shfl_xor(cnt, d, 64);
        first = min(first, (uint32_t)__shfl_xor(first, d, 64));
    }
    if ((threadIdx.x & 63) == 0) { s_cnt[threadIdx.x >> 6] = cnt; s_first[threadIdx.x >> 6] = first; }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t c = 0, f = kNoMarker;
        for (int i = 0; i < kT / 64; i++) { c += s_cnt[i]; f = min(f, s_first[i]); }
        win_count[wg] = c;
        win_first[wg] = f;
    }
}

// ---- kernel 2: the decoder -----------------------------------------------------
__global__ __launch_bounds__(kDecodeThreads) void decode_entropy(
    const uint8_t *__restrict__ bits, const ImageRec *__restrict__ recs, int n_images,
    const uint32_t *__restrict__ win_count, const uint32_t *__restrict__ win_first,
    int16_t *__restrict__ coef_all, int32_t *__restrict__ status)
{
    __shared__ DecodeShared S;
    const int tid = threadIdx.x;
    const uint32_t wg = blockIdx.x;
    const int img = find_image(n_images, wg, [&](int i) { return recs[i].window0; });
    const ImageRec &R = recs[img];
    const uint32_t w = wg - R.window0;
    if (R.status != PREP_OK || w >= R.n_windows) return;

    Geometry g;
    g.bpm = R.blocks_per_mcu;
    g.n_luma = R.sampling == PREP_SAMPLING_420 ? 4u : 1u;
    g.ri_blocks = (uint32_t)R.restart_interval * g.bpm;
    g.n_blocks = R.n_blocks;

    // ---- which part of the stream is ours -------------------------------------
    // window 0 starts at the segment start; window w > 0 starts after the first
    // marker of its window, if it has one, and runs to the first marker of the
    // next window that has one.
    uint32_t range_lo = 0, range_hi = R.entropy_len, block0 = 0, block_end = R.n_blocks;
    {
        const uint32_t *wc = win_count + R.window0, *wf = win_first + R.window0;
        uint32_t my_first = w == 0 ? 0u : wf[w];
        if (w != 0 && my_first == kNoMarker) return;  // uniform over the workgroup
        uint32_t before = 0, next_first = kNoMarker, next_w = kNoMarker;
        for (uint32_t i = tid; i < w; i += kT) before += wc[i];
        for (uint32_t i = w + 1 + tid; i < R.n_windows; i += kT)
            if (wf[i] != kNoMarker) { next_w = i; next_first = wf[i]; break; }
        for (int d = 32; d >= 1; d >>= 1) {
            before += __shfl_xor(before, d, 64);
            uint32_t ow = __shfl_xor(next_w, d, 64), of = __shfl_xor(next_first, d, 64);
            if (ow < next_w) { next_w = ow; next_first = of; }
        }
        if ((tid & 63) == 0) {
            S.scan_a[tid >> 6] = before;
            S.dc_val[0][tid >> 6] = (int32_t)next_w;
            S.dc_val[1][tid >> 6] = (int32_t)next_first;
        }
        __syncthreads();
        before = 0;
        next_w = kNoMarker;
        for (int i = 0; i < kT / 64; i++) {
            before += S.scan_a[i];
            if ((uint32_t)S.dc_val[0][i] < next_w) {
                next_w = (uint32_t)S.dc_val[0][i];
                next_first = (uint32_t)S.dc_val[1][i];
            }
        }
        __syncthreads();
        if (w != 0) {
            range_lo = my_first + 2;
            block0 = (before + 1) * g.ri_blocks;  // markers before ours + ours = intervals done
        }
        if (next_w != kNoMarker) {
            range_hi = next_first;
            // markers up to and including the first one of window next_w
            uint32_t upto = 0;
            for (uint32_t i = tid; i < next_w; i += kT) upto += wc[i];
            for (int d = 32; d >= 1; d >>= 1) upto += __shfl_xor(upto, d, 64);
            if ((tid & 63) == 0) S.scan_a[tid >> 6] = upto;
            __syncthreads();
            upto = 0;
            for (int i = 0; i < kT / 64; i++) upto += S.scan_a[i];
            __syncthreads();
            block_end = (upto + 1) * g.ri_blocks;
        }
    }
    if (block0 >= R.n_blocks || block_end > R.n_blocks || range_lo > range_hi) {
        if (tid == 0) atomicMin(&status[img], (int32_t)PREP_E_CORRUPT);
        return;
    }

    // ---- Huffman tables into LDS (T.81 Annex C) ---------------------------------
    const uint8_t *file = bits + R.file_off;
    if (tid < 4) {
        const uint8_t *b = file + R.dht_off[tid];
        HuffTable &T = S.tab[tid];
        int32_t code = 0, k = 0;
        T.first[0] = T.count[0] = T.valptr[0] = 0;
        for (int l = 1; l <= 16; l++) {
            int32_t c = b[l - 1];
            T.first[l] = code;
            T.count[l] = c;
            T.valptr[l] = k;
            code = (code + c) << 1;
            k += c;
        }
    }
    for (int t = 0; t < 4; t++) {
        const uint32_t nval = min(R.dht_nval[t], 256u);
        S.tab[t].huffval[tid] = (uint32_t)tid < nval ? file[R.dht_off[t] + 16 + tid] : 0;
    }
    __syncthreads();
    for (int t = 0; t < 4; t++) {
        HuffTable &T = S.tab[t];
        for (int x = tid; x < (1 << kLutBits); x += kT) {
            uint32_t e = 0;
            for (int l = 1; l <= kLutBits; l++) {
                int32_t c = (x >> (kLutBits - l)) - T.first[l];
                if (c >= 0 && c < T.count[l]) {
                    e = ((uint32_t)l << 8) | T.huffval[(T.valptr[l] + c) & 255];
                    break;
                }
            }
            T.lut[x] = (uint16_t)e;
        }
    }

    const uint8_t *seg = file + R.entropy_rel;
    int16_t *coef = coef_all + (size_t)R.coef_block0 * 64;
    // raw offsets are signed: the aligned span of the first chunk may begin a few bytes
    // before the segment (inside the file's headers)
    const int32_t seg_len = (int32_t)R.entropy_len;
    const int32_t rhi = (int32_t)range_hi;
    int32_t cs = (int32_t)range_lo;      // raw offset where the next chunk starts
    uint32_t st0 = pack_state(0, 0, 0);  // true state at the start of the chunk
    uint32_t block_base = block0;
    int32_t dc_carry[3] = {0, 0, 0};
    int32_t bad = 0;

    const uint32_t max_chunks = (range_hi - range_lo) / (kChunkRaw / 4) + 2;
    for (uint32_t iter = 0; iter < max_chunks && cs < rhi; iter++) {
        // ---- stage: destuff raw bytes [cs, ce) into S.clean --------------------------
        // lanes own 64-byte pieces of the 16-byte aligned span that contains cs
        const int32_t mis = (int32_t)((uintptr_t)(seg + cs) & 15u);
        const int32_t a0 = cs - mis;
        const int32_t ce = min(a0 + (int32_t)kChunkRaw, rhi);
        const bool last = ce == rhi;
        __syncthreads();
        for (int i = tid; i < kCleanWords; i += kT) S.clean[i] = 0;
        for (int i = tid; i < kMaskWords; i += kT) S.bmask[i] = 0;
        const int32_t my_lo = a0 + tid * 64;  // raw offset of my first byte
        unsigned long long keep = 0, bound = 0;
        uint32_t raw[16];
        {
            const uint4 *src = reinterpret_cast<const uint4 *>(seg + my_lo);
#pragma unroll
            for (int k = 0; k < 4; k++) {
                uint4 v = make_uint4(0, 0, 0, 0);
                // load a 16-byte piece only if it overlaps [cs, ce]: the byte at ce (the FF
                // of the marker that ends the run) is looked at, not consumed
                const int32_t plo = my_lo + 16 * k;
                if (plo + 16 > cs && plo <= ce) v = src[k];
                raw[4 * k + 0] = v.x; raw[4 * k + 1] = v.y; raw[4 * k + 2] = v.z; raw[4 * k + 3] = v.w;
            }
        }
        {
            // byte before my piece and byte after it, for the FF xx pairs that straddle;
            // past the segment comes the FF of the EOI marker
            uint32_t prev = 0, nextb = 0xFFu;
            if (my_lo > cs && my_lo <= ce) prev = load_byte(seg + my_lo - 1);
            if (my_lo + 64 < seg_len && my_lo + 64 > cs && my_lo + 64 <= ce) nextb = load_byte(seg + my_lo + 64);
#pragma unroll
            for (int i = 0; i < 64; i++) {
                const uint32_t cur = (raw[i >> 2] >> (8 * (i & 3))) & 255u;
                const uint32_t nxt = i < 63 ? (raw[(i + 1) >> 2] >> (8 * ((i + 1) & 3))) & 255u : nextb;
                const int32_t pos = my_lo + i;
                const bool inside = pos >= cs && pos < ce;
                // a byte after FF is stuffing or a marker code; FF itself is data only before 00
                const bool k = cur == 0xFFu ? nxt == 0u : prev != 0xFFu;
                if (inside && k) keep |= 1ull << i;
                if (inside && prev == 0xFFu && cur != 0u) {
                    if (cur >= 0xD0u && cur <= 0xD7u) bound |= 1ull << i;
                    else if (cur != 0xFFu) bad = 1;  // a marker that may not occur inside a scan
                }
                prev = cur;
            }
        }
        uint32_t clean_len;
        const uint32_t my_off = block_excl_scan((uint32_t)__popcll(keep), S.scan_a, &clean_len);
        S.keep[tid] = keep;
        S.keep_off[tid] = my_off;
        if (tid == 0) S.keep_off[kT] = clean_len;
        __syncthreads();  // zero fill done before bytes are written
        {
            uint8_t *cb = reinterpret_cast<uint8_t *>(S.clean);
            uint32_t o = my_off;
#pragma unroll
            for (int i = 0; i < 64; i++) {
                if ((bound >> i) & 1ull) atomicOr(&S.bmask[o >> 5], 1u << (o & 31));
                if ((keep >> i) & 1ull) {
                    cb[o ^ 3u] = (uint8_t)((raw[i >> 2] >> (8 * (i & 3))) & 255u);
                    o++;
                }
            }
        }
        __syncthreads();
        {
            // first interval start at or after each lane's subsequence: suffix minimum
            unsigned long long m = ((unsigned long long)S.bmask[2 * tid + 1] << 32) | S.bmask[2 * tid];
            uint32_t mine = m ? (uint32_t)tid * 64u + (uint32_t)__builtin_ctzll(m) : kNoMarker;
            // suffix min inside the wave, then across waves
            const int lane = tid & 63, wave = tid >> 6;
            for (int d = 1; d < 64; d <<= 1) {
                uint32_t o = __shfl_down(mine, d, 64);
                if (lane + d < 64) mine = min(mine, o);
            }
            if (lane == 0) S.scan_a[wave] = mine;
            __syncthreads();
            uint32_t later = kNoMarker;
            for (int ww = wave + 1; ww < kT / 64; ww++) later = min(later, S.scan_a[ww]);
            S.next_boundary[tid] = min(mine, later);
            if (tid == 0) S.next_boundary[kT] = kNoMarker;
        }
        __syncthreads();

        const uint32_t limit_bits = clean_len * 8u;
        // a chunk that is not the last keeps a tail back so that no symbol straddles its end
        const uint32_t own_bits = last ? limit_bits
                                       : (clean_len > (uint32_t)kChunkTail ? (clean_len - kChunkTail) * 8u : 0u);
        const uint32_t nsub = (own_bits + kSubBits - 1) / kSubBits;  // <= kT
        const bool active = (uint32_t)tid < nsub;
        const uint32_t end_bit = min(((uint32_t)tid + 1u) * kSubBits, own_bits);

        // ---- synchronise: iterate end states to their fixed point ---------------------
        uint32_t in_state = tid == 0 ? st0 : pack_state((uint32_t)tid * kSubBits, 0, 0);
        uint32_t out_state = in_state, nblk = 0;
        if (active) out_state = decode_span<false>(S, g, in_state, end_bit, limit_bits, &nblk, nullptr);
        S.state[tid] = out_state;
        for (uint32_t round = 0; round <= nsub; round++) {
            __syncthreads();
            int changed = 0;
            uint32_t prev_state = tid > 0 ? S.state[tid - 1] : st0;
            __syncthreads();
            if (active && tid > 0 && prev_state != in_state) {
                in_state = prev_state;
                uint32_t o = in_state;
                // a predecessor that already ran past my subsequence leaves me nothing to decode
                if ((in_state >> 9) < end_bit) o = decode_span<false>(S, g, in_state, end_bit, limit_bits, &nblk, nullptr);
                else nblk = 0;
                if (o != out_state) { out_state = o; changed = 1; }
                S.state[tid] = out_state;
            }
            if (!__syncthreads_or(changed)) break;
        }

        // ---- write: decode once more from the true states -----------------------------
        uint32_t total_blocks;
        const uint32_t my_block = block_base + block_excl_scan(active ? nblk : 0u, S.scan_a, &total_blocks);
        WriteCtx wc;
        wc.coef = coef;
        wc.block = my_block;
        wc.dcsum[0] = wc.dcsum[1] = wc.dcsum[2] = 0;
        wc.dcreset[0] = wc.dcreset[1] = wc.dcreset[2] = 0;
        wc.dc_first = 0;
        wc.dc_count = 0;
        wc.bad = 0;
        // a lane that begins on an MCU boundary where an interval ends must meet the boundary
        // first; lane 0 of a chunk may begin just after one (start of the run, or a boundary
        // consumed at the very end of the previous chunk)
        wc.need_restart = (in_state & 511u) == 0 && g.ri_blocks != 0 && my_block % g.ri_blocks == 0 &&
                          my_block < g.n_blocks && tid != 0;
        uint32_t final_state = out_state;
        if (active && (in_state >> 9) < end_bit) {
            uint32_t nb2;
            final_state = decode_span<true>(S, g, in_state, end_bit, limit_bits, &nb2, &wc);
            if (final_state != out_state || nb2 != nblk) wc.bad = 1;
        }
        bad |= wc.bad;
        // DC differences -> absolute values (T.81 F.2.2.1): carry each component's
        // running value across lanes, restarting where an interval begins
        int32_t carry[3];
#pragma unroll
        for (int c = 0; c < 3; c++) {
            int32_t out_c;
            carry[c] = block_seg_excl_scan(wc.dcsum[c], wc.dcreset[c], dc_carry[c], S.dc_val[c],
                                           S.dc_flag[c], &out_c);
            dc_carry[c] = out_c;
        }
        for (uint32_t i = 0; i < wc.dc_count; i++) {
            const uint32_t b = wc.dc_first + i;
            if (b >= g.n_blocks) break;
            const uint32_t c = comp_of_block(g, b % g.bpm);
            if (first_of_interval(g, b)) carry[c] = 0;
            if (carry[c] == 0 && carry[0] == 0 && carry[1] == 0 && carry[2] == 0) break;
            if (carry[c] != 0) coef[(size_t)b * 64] = (int16_t)(coef[(size_t)b * 64] + carry[c]);
        }

        // ---- carry the true end state into the next chunk -----------------------------
        __syncthreads();
        if (tid == 0) {
            const uint32_t fs = nsub ? S.state[nsub - 1] : st0;
            S.bcast[0] = fs;
        }
        __syncthreads();
        const uint32_t fs = S.bcast[0];
        block_base += total_blocks;
        if (last) { cs = rhi; st0 = fs; break; }
        // raw position of the clean byte the end state points into
        const uint32_t pbit = fs >> 9;
        const uint32_t qc = pbit >> 3;
        if (qc >= clean_len || nsub == 0) {
            // cannot happen for a chunk that is not the last; stop rather than loop
            bad = 1;
            cs = rhi;
            break;
        }
        if (S.keep_off[tid] <= qc && qc < S.keep_off[tid] + (uint32_t)__popcll(S.keep[tid])) {
            unsigned long long m = S.keep[tid];
            uint32_t skip = qc - S.keep_off[tid];
            for (uint32_t i = 0; i < skip; i++) m &= m - 1;  // drop the lowest set bits
            S.bcast[1] = (uint32_t)(a0 + tid * 64 + (int32_t)__builtin_ctzll(m));
        }
        __syncthreads();
        const int32_t next_cs = (int32_t)S.bcast[1];
        if (next_cs <= cs || next_cs >= rhi) { bad = 1; cs = rhi; break; }  // no progress: refuse to spin
        cs = next_cs;
        st0 = pack_state(pbit & 7u, (fs >> 6) & 7u, fs & 63u);
    }

    // the run must end on an MCU boundary with exactly the blocks it should hold
    if (tid == 0 && (block_base != block_end || (st0 & 511u) != 0)) bad = 1;
    if (__syncthreads_or(bad)) {
        if (tid == 0) atomicMin(&status[img], (int32_t)PREP_E_CORRUPT);
    }
}

void launch_scan_restart_markers(const uint8_t *bits, const ImageRec *recs, int n_images,
                                 uint32_t n_windows, uint32_t *win_count, uint32_t *win_first,
                                 int32_t *status, hipStream_t stream)
{
    if (n_windows == 0) return;
    hipLaunchKernelGGL(scan_restart_markers, dim3(n_windows), dim3(kDecodeThreads), 0, stream, bits,
                       recs, n_images, win_count, win_first, status);
}

void launch_decode_entropy(const uint8_t *bits, const ImageRec *recs, int n_images,
                           uint32_t n_windows, const uint32_t *win_count, const uint32_t *win_first,
                           int16_t *coef, int32_t *status, hipStream_t stream)
{
    if (n_windows == 0) return;
    hipLaunchKernelGGL(decode_entropy, dim3(n_windows), dim3(kDecodeThreads), 0, stream, bits, recs,
                       n_images, win_count, win_first, coef, status);
}

}  // namespace prep
