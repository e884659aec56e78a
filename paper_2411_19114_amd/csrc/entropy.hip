// GPU Huffman entropy decoder for baseline JPEG (T.81 F.2.2), gfx950.
//
// The first half of the "Decode" functional unit (PREBA section 4.2, Table 1).
// The FPGA decodes one stream serially per compute unit; here one workgroup owns
// a run of whole restart intervals (T.81 E.2.4) of one image:
//
//   1. scan_restart_markers counts the RSTn markers in fixed windows of every
//      image's entropy-coded segment, so that a workgroup starting at the first
//      marker of its window knows which restart interval (hence which MCU) it
//      starts at, without any serial pass over the stream.
//   2. decode_entropy stages a chunk of the stream in LDS with byte stuffing
//      (FF 00) and markers removed and the interval starts marked, then decodes
//      it in one of two ways:
//      - short intervals: one lane per restart interval, a single sequential pass
//        that writes coefficients directly (start state and MCU index are known);
//      - long intervals or none: every lane takes a fixed-size subsequence and
//        decodes from a guessed state (code-word boundary, block 0 of an MCU, DC
//        coefficient); lane j then re-decodes from the end state lane j-1 reached
//        until no end state changes.  Lane 0 starts from a known state, so the
//        fixed point is the sequential decode, exactly.  A prefix sum of completed
//        blocks gives every lane its block index, a last pass writes coefficients,
//        and a segmented scan turns DC differences into absolute values.
//      - calls with little data (small windows, kHyp): the states at the subsequence
//        borders inside restart intervals are found by phase hypotheses in two passes
//        (resolve_by_hypotheses) instead of by iteration, then written as above.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/prep.h"
#include "kernels.h"
#include "prep_internal.h"

namespace prep {

namespace {

constexpr int kT = kDecodeThreads;
constexpr int kPadShift = 4;                        // rows of 16 words (= one subsequence) + 1 (copy of the next)
constexpr int kCleanWords = kChunkRaw / 4 + kT + 16;  // destuffed stream, the rows' last words, zero tail
constexpr int kMaskWords = kChunkRaw / 32 + 2;      // one bit per clean byte
constexpr int kSubEntries = 256;                    // second-level lookup entries per table
constexpr int kMaxBoundaries = 1024;                // listed interval starts per chunk
constexpr uint32_t kShortInterval = 1024;           // mean clean bytes up to which a lane takes a whole interval
constexpr uint32_t kNoMarker = 0xFFFFFFFFu;
constexpr uint32_t kSubBits = kSubseqBytes * 8;
static_assert(kSubseqBytes == 64 && (kSubseqBytes / 4) == (1 << kPadShift), "one 64-bit keep mask per lane");

// Lookup entry of a Huffman code (16 bits):
//   bits 15..11 code length + number of appended bits (1..31); 0 = not a code entry
//   bits 10..4  zig-zag advance - 1 (DC 1, AC run+1, ZRL 16, EOB 128).  Added to the zig-zag
//               index it gives the index k of the symbol's coefficient, which must not exceed
//               63 except for EOB, whose coefficient is the block's last: k <= 63 is in order,
//               64 <= k < 128 is a run past the block's end, k >= 128 is EOB (bit 6 of k tells)
//   bits 3..0   number of appended bits
// A first-level entry that is not a code entry refers to the table's second-level pool:
// bits 10..8 = extra index bits (0..6), bits 7..0 = offset of its block.  Two pool entries are
// set aside so that every first-level miss is resolved by the same read: entry 0 holds 0 (no
// such code; the first-level entry is 0 too), entry 1 holds kUseLoop (the table's blocks did
// not fit the pool: search the canonical code lists instead).
constexpr uint32_t kUseLoop = 0x07FFu;
constexpr uint32_t kPoolReserved = 2, kPoolSearchRef = 1;
constexpr uint32_t kInvalidEntry = (16u << 11) | (127u << 4);  // 16 bits, ends the block

struct alignas(16) HuffTables {
    // first level: entry (prefix << 2) | table for the next kLutBits bits, the four tables
    // (DC luma, AC luma, DC chroma, AC chroma) interleaved, so that a decoder forms an entry's
    // address from the bits and its table number with one AND-OR
    alignas(8) uint16_t lut[4 << kLutBits];
    uint16_t sub[4 * kSubEntries];   // second level
    int32_t first[4][17];            // first code of each length
    int32_t count[4][17];            // BITS
    int32_t valptr[4][17];           // index of the first symbol of each length
    uint8_t huffval[4][256];
    uint32_t sub_used[4];
};

struct DecodeShared {
    // The destuffed stream, big-endian packed (bit 31 of a word is the earliest bit).  In the
    // subsequence passes every 16 words (a subsequence) are followed by a copy of the next
    // word: rows of 17, so that lanes that read at similar offsets of their subsequences hit
    // different LDS banks, and a lane's reads stay in its row (see clean_row_of_bit).
    uint32_t clean[kCleanWords];
    uint32_t bmask[kMaskWords];      // bit q set: a restart interval begins at clean byte q
    uint32_t next_boundary[kT + 1];  // first interval start at or after the lane's subsequence
    uint16_t bpos[kMaxBoundaries];   // interval starts of the chunk in order (clean byte offsets)
    HuffTables tab;                  // DC luma, AC luma, DC chroma, AC chroma
    unsigned long long keep[kT];     // which of the lane's 64 raw bytes survived destuffing
    uint32_t keep_off[kT + 1];       // clean offset of the lane's first surviving byte
    uint32_t state[kT];              // end state of every subsequence
    uint32_t scan_a[kT / 64 + 1];    // per-wave totals for workgroup scans
    int32_t dc_val[kT / 64 + 1];
    int32_t dc_flag[kT / 64 + 1];
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

// sum over the workgroup
__device__ inline uint32_t block_sum(uint32_t v, uint32_t *wave_tot)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) wave_tot[threadIdx.x >> 6] = v;
    __syncthreads();
    uint32_t tot = 0;
#pragma unroll
    for (int w = 0; w < kT / 64; w++) tot += wave_tot[w];
    return tot;
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
    int32_t cv = carry_in, all_v = carry_in;
#pragma unroll
    for (int w = 0; w < kT / 64; w++) {
        int32_t wv = wave_val[w], wf = wave_flag[w];
        int32_t nv = wf ? wv : all_v + wv;
        if (w < wave) cv = nv;
        all_v = nv;
    }
    *carry_out = all_v;
    int32_t pv = __shfl_up(iv, 1, 64);
    int32_t pf = __shfl_up(ifl, 1, 64);
    if (lane == 0) return cv;
    return pf ? pv : cv + pv;
}

// ---- Huffman tables (T.81 Annex C) --------------------------------------------

// canonical search among the code lengths lo..hi for the code that starts `peek16`
__device__ inline bool canonical_lookup(const HuffTables &T, int t, uint32_t peek16, int lo, int hi,
                                        uint32_t *len, uint32_t *sym)
{
    for (int l = lo; l <= hi; l++) {
        const int32_t c = (int32_t)(peek16 >> (16 - l)) - T.first[t][l];
        if (c >= 0 && c < T.count[t][l]) {
            *len = (uint32_t)l;
            *sym = T.huffval[t][(T.valptr[t][l] + c) & 255];
            return true;
        }
    }
    return false;
}

__device__ inline uint32_t make_entry(bool ac, uint32_t sym, uint32_t len)
{
    uint32_t s = sym & 15u, inc;
    if (!ac) {
        if (sym > 11u) return 0u;  // no such DC category in baseline
        inc = 1;
    } else if (s == 0) {
        inc = (sym >> 4) == 15u ? 16u : 128u;  // ZRL, otherwise end of block
    } else {
        inc = (sym >> 4) + 1u;
    }
    return ((len + s) << 11) | ((inc - 1u) << 4) | s;
}

// The first level is filled code by code: canonical codes of one table are consecutive when
// left-aligned, so the code of length len with value c owns the 2^(kLutBits-len) entries that
// begin with it.  Entries above the last code of at most kLutBits bits begin longer codes (or
// nothing): each such prefix gets a block of the second-level pool sized for the longest
// code that shares it.
// Expands tables t_lo .. t_hi-1 of the four (all lanes of the workgroup must call).
__device__ inline void build_tables(HuffTables &T, const uint8_t *file, const ImageRec &R, int t_lo = 0,
                                    int t_hi = 4)
{
    const int tid = threadIdx.x;
    if (tid >= t_lo && tid < t_hi) {
        const uint8_t *b = file + R.dht_off[tid];
        int32_t bits[16];
#pragma unroll
        for (int l = 0; l < 16; l++) bits[l] = b[l];
        int32_t code = 0, k = 0;
        T.first[tid][0] = T.count[tid][0] = T.valptr[tid][0] = 0;
#pragma unroll
        for (int l = 1; l <= 16; l++) {
            const int32_t c = bits[l - 1];
            T.first[tid][l] = code;
            T.count[tid][l] = c;
            T.valptr[tid][l] = k;
            code = (code + c) << 1;
            k += c;
        }
        T.sub_used[tid] = kPoolReserved;
    }
    for (int t = t_lo; t < t_hi; t++) {
        const uint32_t nval = min(R.dht_nval[t], 256u);
#pragma unroll
        for (uint32_t i = tid; i < 256u; i += kT) T.huffval[t][i] = i < nval ? file[R.dht_off[t] + 16 + i] : 0;
    }
    for (int i = t_lo * kSubEntries + tid; i < t_hi * kSubEntries; i += kT) T.sub[i] = 0;
    __syncthreads();
    for (int t = t_lo; t < t_hi; t++) {
        // codes of at most kLutBits bits: one lane per code
        const int32_t n_short = min(T.valptr[t][kLutBits] + T.count[t][kLutBits], 256);
        for (int32_t i = tid; i < n_short; i += kT) {
            int l = 1;
            while (l < kLutBits && T.valptr[t][l] + T.count[t][l] <= i) l++;
            const uint32_t c = (uint32_t)(T.first[t][l] + (i - T.valptr[t][l]));
            const uint32_t e = make_entry(t & 1, T.huffval[t][i], (uint32_t)l);
            const uint32_t span = 1u << (kLutBits - l), base = c << (kLutBits - l);
            if (base + span > (1u << kLutBits)) continue;  // not a prefix code; the parser refuses these
            for (uint32_t j = 0; j < span; j++) T.lut[((base + j) << 2) | (uint32_t)t] = (uint16_t)e;
        }
        // the rest of the first level: beginnings of longer codes, or of none
        const uint32_t x_lo = min((uint32_t)(T.first[t][kLutBits] + T.count[t][kLutBits]), 1u << kLutBits);
        for (uint32_t x = x_lo + tid; x < (1u << kLutBits); x += kT) {
            uint32_t e = 0;
            // codes of one length are consecutive: which lengths have a code that begins with x?
            int maxl = 0;
            for (int l = kLutBits + 1; l <= 16; l++) {
                const int32_t c = T.count[t][l];
                if (c == 0) continue;
                const int32_t lo = T.first[t][l] >> (l - kLutBits);
                const int32_t hi = (T.first[t][l] + c - 1) >> (l - kLutBits);
                if ((int32_t)x >= lo && (int32_t)x <= hi) maxl = l;
            }
            if (maxl) {
                const uint32_t nb = (uint32_t)(maxl - kLutBits), size = 1u << nb;
                const uint32_t off = atomicAdd(&T.sub_used[t], size);
                if (off + size <= (uint32_t)kSubEntries) {
                    e = (nb << 8) | off;
                    // leave a note for the second-level pass: which prefix owns these entries
                    for (uint32_t i = 0; i < size; i++)
                        T.sub[t * kSubEntries + off + i] = (uint16_t)((nb << 11) | x);
                } else {
                    e = kPoolSearchRef;
                }
            }
            T.lut[(x << 2) | (uint32_t)t] = (uint16_t)e;
        }
    }
    __syncthreads();
    // second level: entry i of a block with nb extra bits covers prefix:i:anything
    for (int t = t_lo; t < t_hi; t++) {
        const uint32_t used = min(T.sub_used[t], (uint32_t)kSubEntries);
        for (uint32_t i = tid; i < used; i += kT) {
            const uint32_t note = T.sub[t * kSubEntries + i];
            uint32_t e = i == kPoolSearchRef ? kUseLoop : 0u;
            if (note) {
                const uint32_t nb = note >> 11, x = note & ((1u << kLutBits) - 1u);
                const uint32_t off = T.lut[(x << 2) | (uint32_t)t] & 0xFFu;
                const uint32_t peek = (x << (16 - kLutBits)) | ((i - off) << (16 - kLutBits - nb));
                uint32_t len, sym;
                if (canonical_lookup(T, t, peek, kLutBits + 1, kLutBits + (int)nb, &len, &sym))
                    e = make_entry(t & 1, sym, len);
            }
            T.sub[t * kSubEntries + i] = (uint16_t)e;
        }
    }
    __syncthreads();
}

// ---- bit-level decoding ------------------------------------------------------

struct Geometry {
    uint32_t bpm;        // blocks per MCU
    uint32_t n_luma;     // luma blocks per MCU (blocks >= n_luma use the chroma tables)
    uint32_t ri_blocks;  // blocks per restart interval, 0 = none
    uint32_t n_blocks;   // blocks in the image
    // The symbol loops keep the block's place in the MCU as slot = 5 * block, so that one field
    // extract gives the next block's slot (wrapping at the MCU's end) and another whether a
    // block uses the chroma tables:
    uint32_t next_slot;  // bits [slot, slot + 5): slot of the block after the one at slot
    uint32_t chroma_at;  // bits [slot, slot + 3): 4 if the block at slot uses the chroma tables, else 0
                         // (twice the number of its DC table)
    __device__ void set_slots()
    {
        next_slot = chroma_at = 0;
        for (uint32_t b = 0; b < bpm; b++) {
            next_slot |= (5u * ((b + 1u) % bpm)) << (5u * b);
            chroma_at |= (b >= n_luma ? 4u : 0u) << (5u * b);
        }
    }
};
// (an MCU holds at most six blocks, luma 2 x 2 and two chroma: six 5-bit fields fit a word)

__device__ __forceinline__ uint32_t slot_of_block(uint32_t blk) { return 5u * blk; }
__device__ __forceinline__ uint32_t block_of_slot(uint32_t slot) { return (slot * 13u) >> 6; }  // slot / 5 for slot <= 25

__device__ inline uint32_t comp_of_block(const Geometry &g, uint32_t blk_in_mcu)
{
    return blk_in_mcu < g.n_luma ? 0u : blk_in_mcu - g.n_luma + 1u;
}

// first interval start at or after clean byte q (in bits), limit if none
__device__ inline uint32_t boundary_from(const DecodeShared &S, uint32_t q, uint32_t limit_bits)
{
    const uint32_t j = q >> 6;
    if (j >= (uint32_t)kT) return limit_bits;
    unsigned long long m = ((unsigned long long)S.bmask[2 * j + 1] << 32) | S.bmask[2 * j];
    m >>= (q & 63);
    uint32_t r = m ? q + (uint32_t)__builtin_ctzll(m) : S.next_boundary[j + 1];
    r = r > 0x0FFFFFFFu ? limit_bits : r * 8u;
    return r < limit_bits ? r : limit_bits;
}

// Per-lane state of a writing pass.  Only scalar members and no indexing by a run-time
// value: the struct must stay in registers (a private-memory copy would make every
// iteration of the decode loop wait for its coefficient stores).
struct WriteCtx {
    int16_t *coef;         // this image's first block
    uint32_t side_rel;     // coef + side_rel = this image's DC differences, one int16 per block
    uint32_t block;        // absolute index of the block being decoded
    int32_t iv_rem;        // blocks left before a restart boundary has to come (0: it comes next)
    int32_t bad;
};

// The rarest part of a lookup: a table whose second level did not fit its pool.  Out of
// line so that the decode loops stay short.
__device__ __attribute__((noinline)) uint32_t lookup_by_search(const HuffTables &T, uint32_t tsel,
                                                               uint32_t win)
{
    uint32_t len, sym;
    return canonical_lookup(T, (int)tsel, win >> 16, kLutBits + 1, 16, &len, &sym)
               ? make_entry(tsel & 1u, sym, len) : 0u;
}

// Codes longer than the first level covers: e is the first-level entry (not a code entry),
// win = the next 32 bits of the stream, ts2 = twice the table's number.
// Returns the second-level entry: a code entry, 0, or kUseLoop.
__device__ __forceinline__ uint32_t second_level(const HuffTables &T, uint32_t e, uint32_t ts2, uint32_t win)
{
    const uint32_t nbits = e >> 8;
    // the nbits bits after the first kLutBits; none for nbits = 0
    const uint32_t idx = __builtin_amdgcn_ubfe(win, 32u - kLutBits - nbits, nbits);
    return T.sub[(ts2 >> 1) * kSubEntries + (e & 0xFFu) + idx];
}

// First-level entry for the next bits `win` in table ts2 / 2: byte offset (prefix << 3) | ts2.
__device__ __forceinline__ uint32_t first_level(const uint16_t *lut, uint32_t ts2, uint32_t win)
{
    const uint32_t at = ((win >> (32 - kLutBits - 3)) & (((1u << kLutBits) - 1u) << 3)) | ts2;
    return *reinterpret_cast<const uint16_t *>(reinterpret_cast<const char *>(lut) + at);
}

// Word w of the destuffed stream lives at index w + (w >> kPadShift) of DecodeShared::clean in
// the subsequence passes: rows of seventeen words, a subsequence's sixteen and a copy of the
// first word of the next.  A lane that decodes subsequence r (from wherever in it to the first
// symbol boundary at or past its end) uses no word beyond that copy, so all its reads are at
// index w + r with r fixed: one add instead of the row arithmetic, and lanes that are equally
// far into their subsequences still read from different banks.  (The words it merely
// prefetches, up to two further, lie in the next row at the wrong place and are never used.)
__device__ __forceinline__ uint32_t clean_row_of_bit(uint32_t p)
{
    static_assert(kSubseqBytes * 8 == 1 << 9 && kPadShift == 4, "bit >> 9 = subsequence = row");
    return p >> 9;
}

// the 32 stream bits from bit position p on, of the two words that hold them and the next:
// the upper half of the pair shifted left (one instruction less than shifting it right by
// 32 minus the offset)
__device__ __forceinline__ uint32_t window_at(uint32_t hi, uint32_t lo, uint32_t p)
{
    return (uint32_t)(((((unsigned long long)hi << 32) | lo) << (p & 31u)) >> 32);
}

// value of a stored coefficient: appended bits (T.81 F.2.2.4 RECEIVE) and sign extension
// (F.2.2.1 EXTEND); adv = code length + s
__device__ __forceinline__ int32_t coefficient_value(uint32_t win, uint32_t adv, uint32_t s)
{
    // RECEIVE(s) read as a signed field: t < 0 where the first appended bit is 1; 0 for s = 0
    const int32_t t = __builtin_amdgcn_sbfe((int32_t)win, 32u - adv, s);
    // EXTEND: first bit 1: the bits are the value, t + 2^s; first bit 0: 2^s - 1 below them.
    // With m = t >> 31 both are t + ((-2^s) ^ m) + 1.
    return t + (int32_t)((0xFFFFFFFFu << s) ^ (uint32_t)(t >> 31)) + 1;
}

// Decode from packed state `st` until the bit position reaches end_bit.
// limit_bits = end of the staged data.  Returns the end state; *nblk = blocks completed.
// after_boundary: st.p is the first bit of a restart interval (the boundary there is behind
// us, not ahead).
//
// One iteration = one symbol: take the next 32 bits, look them up, (write mode) extract the
// value and store it, advance position and zig-zag index.  The state carried from one symbol
// to the next is the bit position, block-in-MCU and zig-zag index only.  A writing pass
// stores DC *differences*; dc_prefix() turns them into values afterwards.
//
// A lone wave issues a dependent instruction only every eight cycles or so and pays a fetch
// bubble for every taken branch, and a lane that leaves the loop waits for the whole wave to
// leave it.  So there is one loop, kept short and straight, that every lane stays in until
// its span is done; the two rare events are branches off it that return to it: a code longer
// than the first-level table covers, and a symbol that does not fit before the next restart
// boundary or the end of the data (the bits there are padding, or belong to the next
// interval), which is where the lane steps over the boundary.
template <bool kWrite>
__device__ __forceinline__ uint32_t decode_span(const DecodeShared &S, const Geometry &g, uint32_t st,
                                                bool after_boundary, uint32_t end_bit,
                                                uint32_t limit_bits, uint32_t *nblk, WriteCtx *wc)
{
    uint32_t p = st >> 9, slot = slot_of_block((st >> 6) & 7u), zz = st & 63u;
    uint32_t done = 0;
    // write mode: first coefficient of the current block, the image's last coefficient,
    // blocks left in the restart interval
    uint32_t boff = 0, last = 0;
    int32_t iv_rem = 0;
    if (kWrite) {
        boff = wc->block * 64u;
        last = g.n_blocks * 64u - 1u;
        iv_rem = wc->iv_rem;
    }
    // next restart boundary ahead (bit position), limit_bits if none
    uint32_t nb = boundary_from(S, after_boundary ? (p >> 3) + 1u : (p + 7u) >> 3, limit_bits);
    const uint16_t *lut = S.tab.lut;
    // tb: twice the number of the current table (DC luma 0, AC luma 2, DC chroma 4, AC chroma 6)
    const uint32_t ac_bit = 2u;
    uint32_t tb = __builtin_amdgcn_ubfe(g.chroma_at, slot, 3u) | (zz ? ac_bit : 0u);
    // what a writing pass has to refuse is gathered without branches in the loop: bit 6 of
    // over = a coefficient index past its block; sign of late = a symbol where a restart marker
    // had to come; broken = what the rare branches find
    int32_t late = 0, broken = 0;
    uint32_t over = 0;
    // the stream words that hold bit p, the one after, and the one after that, kept in
    // registers: a symbol is shorter than a word, so at most one new word is needed per
    // symbol, and it is fetched one symbol ahead of its use
    uint32_t w = p >> 5;
    const uint32_t *row = S.clean + clean_row_of_bit(p);  // the span lies in one subsequence
    uint32_t hi = row[w], lo = row[w + 1];
    uint32_t ahead = row[w + 2];
    // look a symbol up: its table entry, or the invalid entry for bits that are no code word
    // (an error unless they are the padding before a boundary, which the invalid entry is too
    // long to fit before)
    auto lookup = [&](uint32_t win) {
        uint32_t e = first_level(lut, tb, win);
        if (__builtin_expect((e >> 11) == 0, 0)) {
            e = second_level(S.tab, e, tb, win);
            if (__builtin_expect((e >> 11) == 0, 0)) {
                if (e == kUseLoop) e = lookup_by_search(S.tab, tb >> 1, win);
                if ((e >> 11) == 0) {
                    e = kInvalidEntry;
                    // (a lookup at or past the span's end is the next span's to judge: this
                    // one's row holds only part of those bits)
                    if (kWrite && p < end_bit && p + (kInvalidEntry >> 11) <= nb) broken = 1;
                }
            }
        }
        return e;
    };
    if (p < end_bit) {
        uint32_t win = window_at(hi, lo, p);
        uint32_t e = lookup(win);
        do {
            const uint32_t adv = e >> 11;
            if (__builtin_expect(p + adv > nb, 0)) {
                // the symbol does not fit before the next restart boundary / the end of the data
                if (nb >= limit_bits) {
                    if (kWrite && (slot != 0 || zz != 0 || limit_bits - p >= 8)) broken = 1;
                    p = limit_bits;  // >= end_bit: the lane is done
                } else {
                    if (kWrite) {
                        // a boundary comes between MCUs, behind fewer than eight padding bits,
                        // and after a whole interval (or right where one has just begun)
                        if (slot != 0 || zz != 0 || nb - p >= 8 || g.ri_blocks == 0 ||
                            (iv_rem != 0 && iv_rem != (int32_t)g.ri_blocks))
                            broken = 1;
                        iv_rem = (int32_t)g.ri_blocks;
                    }
                    p = nb;
                    slot = 0;
                    zz = 0;
                    tb = 0;
                    nb = boundary_from(S, (p >> 3) + 1u, limit_bits);
                    w = p >> 5;
                    hi = row[w];
                    lo = row[w + 1];
                    ahead = row[w + 2];
                }
            } else {
                const uint32_t k = zz + ((e >> 4) & 127u);  // index of the symbol's coefficient
                if (kWrite) {
                    // Every symbol stores.  ZRL and EOB carry no appended bits, so their value
                    // is 0, and it lands on a coefficient that they declare to be zero: the
                    // last of ZRL's sixteen, the last of the block for EOB.  A stream that runs
                    // past the image keeps overwriting the image's last coefficient; the block
                    // count then gives it away.
                    // A DC difference goes to the block's entry of the side array (dc_prefix turns
                    // the differences into values and puts those into the blocks).
                    const uint32_t ci = min(boff + min(k, 63u), last);
                    wc->coef[zz == 0 ? wc->side_rel + (ci >> 6) : ci] = (int16_t)coefficient_value(win, adv, e & 15u);
                    over |= k;
                    late |= iv_rem - 1;
                }
                p += adv;
                {
                    const bool moved = (p >> 5) != w;
                    hi = moved ? lo : hi;
                    lo = moved ? ahead : lo;
                    w += moved ? 1u : 0u;
                    ahead = row[w + 2];
                }
                const bool endb = k >= 63u;  // zz = k + 1 reaches 64
                const uint32_t slot1 = __builtin_amdgcn_ubfe(g.next_slot, slot, 5u);
                zz = endb ? 0u : k + 1u;
                slot = endb ? slot1 : slot;
                done += endb ? 1u : 0u;
                tb = endb ? __builtin_amdgcn_ubfe(g.chroma_at, slot1, 3u) : tb | ac_bit;
                if (kWrite) {
                    boff += endb ? 64u : 0u;
                    iv_rem -= endb ? 1 : 0;
                }
            }
            // the next symbol's lookup, issued before the loop test
            win = window_at(hi, lo, p);
            e = lookup(win);
        } while (p < end_bit);
    }
    if (kWrite) wc->bad |= broken | (late < 0 ? 1 : 0) | (int32_t)((over >> 6) & 1u);
    *nblk = done;
    return pack_state(p, block_of_slot(slot), zz);
}

// Zeros over the blocks [lo, hi) of an image whose coefficients begin at coef, in 16-byte units
// first, first + step, ... of the range's eight per block.  Nothing clears the coefficient
// workspace before the decoder runs, and the writing passes store only the coefficients that
// symbols name: the blocks that a pass is about to decode get their zeros from here first, in
// whole 128-byte lines.  Out of line: it runs a few times per chunk and must not add to the
// registers of the symbol loops.
__device__ __attribute__((noinline)) void zero_blocks(int16_t *coef, uint32_t lo, uint32_t hi, uint32_t first,
                                                      uint32_t step)
{
    uint4 *units = reinterpret_cast<uint4 *>(coef);  // eight to a block
    for (uint32_t u = lo * 8u + first; u < hi * 8u; u += step) units[u] = make_uint4(0, 0, 0, 0);
}

// The short-interval pass: one lane decodes one restart interval from its start state to
// end_bit, which is the next restart boundary (or the end of the data), and writes its
// coefficients.  Same symbol loop as decode_span, specialised for what that pass knows: the
// span's end and the next boundary are the same position, so the loop ends where a symbol no
// longer fits and never steps over a boundary; the stream is staged without pad words; and
// the caller's count of the interval's blocks stands in for the running check against
// restart intervals.  Returns the end state (at end_bit if the stream is sound).
__device__ __forceinline__ uint32_t decode_interval(const DecodeShared &S, const Geometry &g, uint32_t st,
                                                    uint32_t end_bit, uint32_t *nblk, WriteCtx *wc)
{
    uint32_t p = st >> 9, slot = slot_of_block((st >> 6) & 7u);
    // Where the next symbol starts counting, as one number: 64 * (block of the image) + zig-zag
    // index.  A symbol's coefficient index is clamped to 63, so one past the coefficient of a
    // symbol that ends its block is the first coefficient of the next block by itself.  The
    // count of completed blocks is how far the block has moved at the end.
    const uint32_t first_block = wc->block;
    uint32_t at = (first_block << 6) | (st & 63u);
    const uint32_t last = g.n_blocks * 64u - 1u;
    const uint16_t *lut = S.tab.lut;
    const uint32_t ac_bit = 2u;  // tb: twice the number of the current table, see decode_span
    uint32_t tb = __builtin_amdgcn_ubfe(g.chroma_at, slot, 3u) | ((st & 63u) ? ac_bit : 0u);
    int32_t broken = 0;
    uint32_t over = 0;
    uint32_t w = p >> 5;
    uint32_t hi = S.clean[w], lo = S.clean[w + 1], ahead = S.clean[w + 2];
    // look a symbol up: its table entry, or the invalid entry for bits that are no code word
    // (an error unless they are the padding before the boundary, which the invalid entry is too
    // long to fit before)
    auto lookup = [&](uint32_t win) {
        uint32_t e = first_level(lut, tb, win);
        if (__builtin_expect((e >> 11) == 0, 0)) {
            e = second_level(S.tab, e, tb, win);
            if (__builtin_expect((e >> 11) == 0, 0)) {
                if (e == kUseLoop) e = lookup_by_search(S.tab, tb >> 1, win);
                if ((e >> 11) == 0) {
                    e = kInvalidEntry;
                    if (p + (kInvalidEntry >> 11) <= end_bit) broken = 1;
                }
            }
        }
        return e;
    };
    uint32_t win = window_at(hi, lo, p);
    uint32_t e = lookup(win);
    // the loop runs while the symbol that was looked up fits before the end: what does not fit
    // is padding, or nothing at all
    while (p + (e >> 11) <= end_bit) {
        const uint32_t adv = e >> 11;
        const uint32_t k = (at & 63u) + ((e >> 4) & 127u);  // index of the symbol's coefficient
        // every symbol stores (see decode_span)
        // (k = 0 is a DC difference: it goes to the side array)
        const uint32_t here = (at & ~63u) | min(k, 63u);
        const uint32_t ci = min(here, last);
        wc->coef[k == 0 ? wc->side_rel + (ci >> 6) : ci] = (int16_t)coefficient_value(win, adv, e & 15u);
        at = here + 1u;
        over |= k;
        p += adv;
        {
            const bool moved = (p >> 5) != w;
            hi = moved ? lo : hi;
            lo = moved ? ahead : lo;
            w += moved ? 1u : 0u;
            ahead = S.clean[w + 2];
        }
        const bool endb = k >= 63u;  // the zig-zag index reaches 64
        const uint32_t slot1 = __builtin_amdgcn_ubfe(g.next_slot, slot, 5u);
        slot = endb ? slot1 : slot;
        tb = endb ? __builtin_amdgcn_ubfe(g.chroma_at, slot1, 3u) : tb | ac_bit;
        win = window_at(hi, lo, p);
        e = lookup(win);
    }
    // the lane must stand between MCUs, fewer than eight (padding) bits before the end
    const uint32_t zz = at & 63u;
    if (slot != 0 || zz != 0 || end_bit - p >= 8) broken = 1;
    else p = end_bit;
    wc->bad |= broken | (int32_t)((over >> 6) & 1u);
    *nblk = (at >> 6) - first_block;
    return pack_state(p, block_of_slot(slot), zz);
}

// DC differences -> DC values (T.81 F.2.2.1) for blocks [lo, hi) of the image, by the whole
// workgroup.  The writing passes leave the differences in the image's side array (one int16 per
// block, so both walks below read a few cache lines instead of one line per block); the values go
// into the blocks.  Each lane takes a contiguous run of blocks, sums its differences per component (a
// sum restarts where a restart interval begins), a segmented scan over the lanes carries the
// running values in, and a second walk writes them.  carry[] = running value of each
// component before block lo; on return, after block hi - 1.  All lanes must call.
// Blocks are read eight at a time so that the loads do not wait for one another.
struct DcWalk {
    uint32_t in_mcu, in_iv;  // position of the block in its MCU and in its restart interval
    __device__ inline void start(const Geometry &g, uint32_t block)
    {
        in_mcu = block % g.bpm;
        in_iv = g.ri_blocks ? block % g.ri_blocks : block;
    }
    // the first block of each component in the first MCU of an interval restarts DC prediction
    __device__ inline bool restarts(const Geometry &g) const
    {
        return in_iv == 0 || (in_iv >= g.n_luma && in_iv < g.bpm);
    }
    __device__ inline uint32_t comp(const Geometry &g) const { return comp_of_block(g, in_mcu); }
    __device__ inline void next(const Geometry &g)
    {
        in_mcu = in_mcu + 1u == g.bpm ? 0u : in_mcu + 1u;
        in_iv++;
        if (g.ri_blocks && in_iv == g.ri_blocks) in_iv = 0;
    }
};

__device__ inline void dc_prefix(DecodeShared &S, const Geometry &g, int16_t *coef, const int16_t *side,
                                 uint32_t lo, uint32_t hi, int32_t carry[3])
{
    __syncthreads();  // the stores of every lane (zeros, coefficients, differences) are done and visible
    const uint32_t n = hi > lo ? hi - lo : 0u;
    const uint32_t per = (n + kT - 1) / kT;
    const uint32_t a = min(lo + threadIdx.x * per, hi), b = min(a + per, hi);
    int32_t s0 = 0, s1 = 0, s2 = 0, r0 = 0, r1 = 0, r2 = 0;
    DcWalk wk;
    wk.start(g, a);
    for (uint32_t i = a; i < b; i += 8) {
        int32_t d[8];
#pragma unroll
        for (uint32_t u = 0; u < 8; u++) d[u] = side[min(i + u, b - 1)];
#pragma unroll
        for (uint32_t u = 0; u < 8; u++) {
            if (i + u < b) {
                const uint32_t c = wk.comp(g);
                const bool rst = wk.restarts(g);
                if (c == 0) { s0 = (rst ? 0 : s0) + d[u]; r0 |= rst; }
                else if (c == 1) { s1 = (rst ? 0 : s1) + d[u]; r1 |= rst; }
                else { s2 = (rst ? 0 : s2) + d[u]; r2 |= rst; }
                wk.next(g);
            }
        }
    }
    int32_t out;
    int32_t c0 = block_seg_excl_scan(s0, r0, carry[0], S.dc_val, S.dc_flag, &out);
    carry[0] = out;
    int32_t c1 = block_seg_excl_scan(s1, r1, carry[1], S.dc_val, S.dc_flag, &out);
    carry[1] = out;
    int32_t c2 = block_seg_excl_scan(s2, r2, carry[2], S.dc_val, S.dc_flag, &out);
    carry[2] = out;
    wk.start(g, a);
    for (uint32_t i = a; i < b; i += 8) {
        int32_t d[8];
#pragma unroll
        for (uint32_t u = 0; u < 8; u++) d[u] = side[min(i + u, b - 1)];
#pragma unroll
        for (uint32_t u = 0; u < 8; u++) {
            if (i + u < b) {
                const uint32_t c = wk.comp(g);
                const bool rst = wk.restarts(g);
                int32_t v;
                if (c == 0) { c0 = (rst ? 0 : c0) + d[u]; v = c0; }
                else if (c == 1) { c1 = (rst ? 0 : c1) + d[u]; v = c1; }
                else { c2 = (rst ? 0 : c2) + d[u]; v = c2; }
                coef[(size_t)(i + u) * 64] = (int16_t)v;
                wk.next(g);
            }
        }
    }
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

// Which raw bytes of one 16-byte piece are entropy-coded data (keep) and which are the
// code byte of an RSTn marker (bound).  prev = the byte before the piece, next = the byte
// after it.  Bytes outside [cs, ce) are neither.  A byte after FF is stuffing or a marker
// code; FF itself is data only before 00.
__device__ inline void classify16(const uint4 v, uint32_t prev, uint32_t nextb, int32_t plo,
                                  int32_t cs, int32_t ce, uint32_t *keep, uint32_t *bound,
                                  uint32_t *last, int32_t *bad)
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t k = 0, b = 0;
#pragma unroll
    for (int i = 0; i < 16; i++) {
        const uint32_t cur = (w[i >> 2] >> (8 * (i & 3))) & 255u;
        const uint32_t nxt = i < 15 ? (w[(i + 1) >> 2] >> (8 * ((i + 1) & 3))) & 255u : nextb;
        const int32_t pos = plo + i;
        const bool inside = pos >= cs && pos < ce;
        const bool kp = cur == 0xFFu ? nxt == 0u : prev != 0xFFu;
        if (inside && kp) k |= 1u << i;
        if (inside && prev == 0xFFu && cur != 0u) {
            if (cur >= 0xD0u && cur <= 0xD7u) b |= 1u << i;
            else if (cur != 0xFFu) *bad = 1;  // a marker that may not occur inside a scan
        }
        prev = cur;
    }
    *keep = k;
    *bound = b;
    *last = prev;
}

}  // namespace

// ---- kernel 1: restart markers per window -----------------------------------
// window w of an image = raw bytes [w*window_bytes, (w+1)*window_bytes) of its
// entropy-coded segment.  cnt = RSTn markers whose FF byte lies in the window,
// first = offset (from the segment start) of the first such FF byte.
// data_end[image] arrives as the length that the host gave the segment (up to the file's last
// EOI marker, which it finds from the file's end) and leaves as the offset of the first EOI
// marker in it: FF D9 cannot occur inside entropy-coded data (T.81 F.1.2.3), so where a file
// goes on after its image (a second image, a preview) the data end there.
// Workgroups from n_windows on do something else: workgroup n_windows + 4 s + t expands
// Huffman table t of image table_rep[s] into slot s of `tables`.
__global__ __launch_bounds__(kDecodeThreads) void scan_restart_markers(
    const uint8_t *__restrict__ bits, const ImageRec *__restrict__ recs, int n_images,
    uint32_t n_windows, uint32_t window_bytes, uint32_t *__restrict__ win_count,
    uint32_t *__restrict__ win_first, uint32_t *__restrict__ data_end, int32_t *__restrict__ status,
    const uint32_t *__restrict__ table_rep, uint4 *__restrict__ tables)
{
    __shared__ uint32_t s_cnt[kT / 64], s_first[kT / 64];
    const uint32_t wg = blockIdx.x;
    if (wg >= n_windows) {
        // four workgroups per slot, one table each, so that the expansion is not the longest
        // thing this kernel does
        __shared__ HuffTables tab;
        const uint32_t slot = (wg - n_windows) >> 2;
        const int t = (int)((wg - n_windows) & 3u);
        const ImageRec &I = recs[table_rep[slot]];
        build_tables(tab, bits + I.file_off, I, t, t + 1);
        const uint32_t *src = reinterpret_cast<const uint32_t *>(&tab);
        uint32_t *dst = reinterpret_cast<uint32_t *>(tables) + (size_t)slot * (sizeof(HuffTables) / 4);
        // the members of table t, as 32-bit words of the struct
        // (its first-level entries lie among the other tables': they go one by one)
        uint16_t *dst_lut = reinterpret_cast<uint16_t *>(dst + offsetof(HuffTables, lut) / 4);
        for (uint32_t i = threadIdx.x; i < (1u << kLutBits); i += kT)
            dst_lut[(i << 2) | (uint32_t)t] = tab.lut[(i << 2) | (uint32_t)t];
        const uint32_t part[6][2] = {
            {(uint32_t)offsetof(HuffTables, sub) + (uint32_t)t * 2u * kSubEntries, 2u * kSubEntries},
            {(uint32_t)offsetof(HuffTables, first) + (uint32_t)t * 68u, 68u},
            {(uint32_t)offsetof(HuffTables, count) + (uint32_t)t * 68u, 68u},
            {(uint32_t)offsetof(HuffTables, valptr) + (uint32_t)t * 68u, 68u},
            {(uint32_t)offsetof(HuffTables, huffval) + (uint32_t)t * 256u, 256u},
            {(uint32_t)offsetof(HuffTables, sub_used) + (uint32_t)t * 4u, 4u}};
#pragma unroll
        for (int m = 0; m < 6; m++)
            for (uint32_t i = threadIdx.x; i < part[m][1] / 4; i += kT)
                dst[part[m][0] / 4 + i] = src[part[m][0] / 4 + i];
        return;
    }
    const int img = find_image(n_images, wg, [&](int i) { return recs[i].window0; });
    const ImageRec &R = recs[img];
    const uint32_t w = wg - R.window0;
    // the per-image verdict starts as the host parser's; the decoder may lower it
    if (w == 0 && threadIdx.x == 0) status[img] = R.status;
    uint32_t cnt = 0, first = kNoMarker, eoi = kNoMarker;
    if (R.status == PREP_OK && w < R.n_windows) {
        const bool count_rst = R.restart_interval != 0;
        const uint8_t *seg = bits + R.file_off + R.entropy_rel;
        const int32_t lo = (int32_t)(w * window_bytes);
        const int32_t hi = (int32_t)min(w * window_bytes + window_bytes, R.entropy_len);
        // 16-byte aligned parts that cover [lo, hi), dealt to the lanes in turn; a part that
        // begins before lo reaches at most 15 bytes back, into the file's headers
        const int32_t a0 = lo - (int32_t)((uintptr_t)(seg + lo) & 15u);
        for (int32_t plo = a0 + 16 * (int32_t)threadIdx.x; plo < hi; plo += 16 * kT) {
            const uint4 v = *reinterpret_cast<const uint4 *>(seg + plo);
            // the byte after the last one of the segment is the EOI marker's FF
            const uint32_t after = load_byte(seg + min(plo + 16, (int32_t)R.entropy_len));
            const uint32_t wv[5] = {v.x, v.y, v.z, v.w, after};
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const uint32_t cur = (wv[i >> 2] >> (8 * (i & 3))) & 255u;
                const uint32_t nxt = (wv[(i + 1) >> 2] >> (8 * ((i + 1) & 3))) & 255u;
                const int32_t pos = plo + i;
                if (cur == 0xFFu && nxt >= 0xD0u && nxt <= 0xD9u && nxt != 0xD8u && pos >= lo && pos < hi) {
                    if (nxt == 0xD9u) {
                        eoi = min(eoi, (uint32_t)pos);
                    } else if (count_rst) {
                        cnt++;
                        first = min(first, (uint32_t)pos);
                    }
                }
            }
        }
        if (eoi != kNoMarker) atomicMin(&data_end[img], eoi);
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
// kHyp: the variant for calls with little data, whose workgroups own a few restart intervals
// each (small windows).  Inside a restart interval the state at a subsequence border is not
// known; what keeps iteration slow there is the block's place in the MCU (which tables come
// next), while bit position and zig-zag index fall into step within a block or two.  So every
// subsequence is decoded once from each place-in-MCU hypothesis by a lane of its own (the chip
// is idle otherwise), and once more from the end states those lanes reached in the subsequence
// before; the true chain then only picks, link by link, the candidate that it equals.
template <bool kHyp>
__global__ __launch_bounds__(kDecodeThreads) void decode_entropy(
    const uint8_t *__restrict__ bits, const ImageRec *__restrict__ recs, int n_images,
    const uint32_t *__restrict__ win_count, const uint32_t *__restrict__ win_first,
    const uint32_t *__restrict__ data_end, int16_t *__restrict__ coef_all, uint32_t side_off,
    int32_t *__restrict__ status, const uint4 *__restrict__ tables, uint32_t hyp_span_bits)
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
    g.n_luma = (uint32_t)(luma_h(R.sampling) * luma_v(R.sampling));
    g.ri_blocks = (uint32_t)R.restart_interval * g.bpm;
    g.set_slots();
    g.n_blocks = R.n_blocks;

    // ---- which part of the stream is ours -------------------------------------
    // window 0 starts at the segment start; window w > 0 starts after the first
    // marker of its window, if it has one, and runs to the first marker of the
    // next window that has one.
    // the entropy-coded data end at the segment's first EOI marker (found by the scan kernel)
    const uint32_t data_len = min(R.entropy_len, data_end[img]);
    uint32_t range_lo = 0, range_hi = data_len, block0 = 0, block_end = R.n_blocks;
    uint32_t marker_base = 0;  // number, within the image, of the first restart marker at or after cs
    bool first_marker_ok = true;
    {
        const uint32_t *wc = win_count + R.window0, *wf = win_first + R.window0;
        uint32_t my_first = w == 0 ? 0u : wf[w];
        if (w != 0 && (my_first == kNoMarker || my_first >= data_len)) return;  // uniform over the workgroup
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
            S.dc_val[tid >> 6] = (int32_t)next_w;
            S.dc_flag[tid >> 6] = (int32_t)next_first;
        }
        __syncthreads();
        before = 0;
        next_w = kNoMarker;
        for (int i = 0; i < kT / 64; i++) {
            before += S.scan_a[i];
            if ((uint32_t)S.dc_val[i] < next_w) {
                next_w = (uint32_t)S.dc_val[i];
                next_first = (uint32_t)S.dc_flag[i];
            }
        }
        __syncthreads();
        if (next_w != kNoMarker && next_first >= data_len) next_w = kNoMarker;  // (a marker of what follows the image)
        if (w != 0) {
            range_lo = my_first + 2;
            block0 = (before + 1) * g.ri_blocks;  // markers before ours + ours = intervals done
            marker_base = before + 1;
            // our marker is number `before` of the image, and markers count modulo 8 from RST0
            // (T.81 E.2.4, B.2.1); the markers inside the run are checked where they are staged
            first_marker_ok = ((load_byte(bits + R.file_off + R.entropy_rel + my_first + 1) ^ before) & 7u) == 0;
        }
        if (next_w != kNoMarker) {
            range_hi = next_first;
            // markers up to and including the first one of window next_w
            uint32_t upto = 0;
            for (uint32_t i = tid; i < next_w; i += kT) upto += wc[i];
            upto = block_sum(upto, S.scan_a);
            block_end = (upto + 1) * g.ri_blocks;
        }
    }
    if (block0 >= R.n_blocks || block_end > R.n_blocks || range_lo > range_hi || !first_marker_ok) {
        if (tid == 0) atomicMin(&status[img], (int32_t)PREP_E_CORRUPT);
        return;
    }

    const uint8_t *file = bits + R.file_off;
    if (R.table_slot != kNoTableSlot) {
        // the tables were expanded once for the batch: copy them
        constexpr uint32_t units = sizeof(HuffTables) / 16;
        uint4 *dst = reinterpret_cast<uint4 *>(&S.tab);
        for (uint32_t i = tid; i < units; i += kT) dst[i] = tables[(size_t)R.table_slot * units + i];
        __syncthreads();
    } else {
        build_tables(S.tab, file, R);
    }

    const uint8_t *seg = file + R.entropy_rel;
    int16_t *coef = coef_all + (size_t)R.coef_block0 * 64;
    // DC differences of this image's blocks: the side array begins side_off elements after the
    // first coefficient of the workspace, one entry per block
    const uint32_t side_rel = side_off + R.coef_block0 - R.coef_block0 * 64u;
    // raw offsets are signed: the aligned span of the first chunk may begin a few bytes
    // before the segment (inside the file's headers)
    const int32_t seg_len = (int32_t)data_len;
    const int32_t rhi = (int32_t)range_hi;
    int32_t cs = (int32_t)range_lo;      // raw offset where the next chunk starts
    uint32_t st0 = pack_state(0, 0, 0);  // true state at the start of the chunk
    uint32_t block_base = block0;
    int32_t dc_carry[3] = {0, 0, 0};
    int32_t bad = 0;

    const uint32_t max_chunks = (range_hi - range_lo) / 64u + 2;
    for (uint32_t iter = 0; iter < max_chunks && cs < rhi; iter++) {
        // ---- stage: destuff raw bytes [cs, ce) into S.clean --------------------------
        // lanes own 64-byte pieces (four 16-byte parts) of the 16-byte aligned span that
        // contains cs
        const int32_t mis = (int32_t)((uintptr_t)(seg + cs) & 15u);
        const int32_t a0 = cs - mis;
        const int32_t ce = min(a0 + (int32_t)kChunkRaw, rhi);
        const bool last = ce == rhi;
        __syncthreads();
        for (int i = tid; i < kMaskWords; i += kT) S.bmask[i] = 0;
        const int32_t my_lo = a0 + tid * 64;  // raw offset of my first byte
        // 16-byte parts are loaded whether or not they still overlap [cs, ce] (what lies
        // outside is not looked at), from an address clamped to the part that holds ce, so
        // that the loads of a piece do not wait for one another.  Such a load is aligned
        // and holds at least one byte of the file, so it stays inside the file's last page.
        const int32_t last_part = a0 + ((ce - a0) & ~15);
        uint4 v[4];
#pragma unroll
        for (int k = 0; k < 4; k++)
            v[k] = *reinterpret_cast<const uint4 *>(seg + min(my_lo + 16 * k, last_part));
        unsigned long long keep = 0, bound = 0;
        {
            // the byte before my piece and the byte after each 16-byte part, for the FF xx
            // pairs that straddle; past the segment comes the FF of the EOI marker
            const uint32_t after = load_byte(seg + min(my_lo + 64, ce));
            uint32_t prev = 0;
            if (my_lo > cs && my_lo <= ce) prev = load_byte(seg + my_lo - 1);
#pragma unroll
            for (int k = 0; k < 4; k++) {
                const int32_t plo = my_lo + 16 * k;
                uint32_t kp = 0, bd = 0;
                // a part is looked at only if it overlaps [cs, ce]: the byte at ce (the FF of
                // the marker that ends the run) is examined, not consumed
                if (plo <= ce) {
                    uint32_t nextb = k < 3 ? (v[(k + 1) & 3].x & 255u) : after;
                    if (!(plo + 16 < seg_len && plo + 16 <= ce)) nextb = 0xFFu;
                    classify16(v[k], prev, nextb, plo, cs, ce, &kp, &bd, &prev, &bad);
                } else {
                    prev = 0;
                }
                keep |= (unsigned long long)kp << (16 * k);
                bound |= (unsigned long long)bd << (16 * k);
            }
        }
        // clean offsets (low half) and boundary ranks (high half) in one scan
        uint32_t totals;
        const uint32_t my_pre = block_excl_scan((uint32_t)__popcll(keep) | ((uint32_t)__popcll(bound) << 16),
                                                S.scan_a, &totals);
        const uint32_t clean_len = totals & 0xFFFFu, nbnd = totals >> 16;
        const uint32_t my_off = my_pre & 0xFFFFu;
        S.keep[tid] = keep;
        S.keep_off[tid] = my_off;
        if (tid == 0) S.keep_off[kT] = clean_len;
        // zeros behind the data: the last word is written byte by byte, and lookups near the
        // end read a few words past it
        // Which of the two passes will decode the chunk is known now.  Intervals 0..n_iv-1 of
        // the chunk end inside it: the first runs from the chunk's start state to the first
        // listed start, interval k > 0 between listed starts k-1 and k, and in the last chunk
        // one more runs to the end of the data.
        const uint32_t n_iv = last ? nbnd + 1 : nbnd;
        // (the variant for small calls finds the states inside restart intervals by hypotheses)
        const bool by_hypotheses = kHyp && g.ri_blocks != 0;
        const bool short_intervals = !by_hypotheses && g.ri_blocks != 0 && n_iv >= 1 &&
                                     nbnd <= (uint32_t)kMaxBoundaries && clean_len <= kShortInterval * (nbnd + 1);
        // the short-interval pass reads the stream without pad words (its lanes start anywhere)
        const uint32_t pad_shift = short_intervals ? 31u : (uint32_t)kPadShift;
        // zeros behind the data: the last word is written byte by byte, and lookups near the
        // end read a few words past it
        {
            // (a run of array entries: in the subsequence passes it takes in the rows' last words,
            // the copies, among them the copy of the data's last, partly written word)
            const uint32_t wd = clean_len >> 2, first = wd + (wd >> pad_shift);
            const uint32_t from = !short_intervals && (wd & 15u) == 0 && wd != 0 ? first - 1u : first;
            if (tid < 14) S.clean[from + (uint32_t)tid] = 0;
        }
        __syncthreads();  // zero fill done before bytes are written
        {
            uint8_t *cb = reinterpret_cast<uint8_t *>(S.clean);
            uint32_t o = my_off, rank = my_pre >> 16;
#pragma unroll
            for (int k = 0; k < 4; k++) {
                const uint32_t kp = (uint32_t)(keep >> (16 * k)) & 0xFFFFu;
                const uint32_t bd = (uint32_t)(bound >> (16 * k)) & 0xFFFFu;
                if ((kp | bd) == 0) continue;
                const uint32_t wv[4] = {v[k].x, v[k].y, v[k].z, v[k].w};
#pragma unroll
                for (int i = 0; i < 16; i++) {
                    if ((bd >> i) & 1u) {
                        // marker number marker_base + rank of the image must be RST((that) mod 8)
                        if ((((wv[i >> 2] >> (8 * (i & 3))) ^ (marker_base + rank)) & 7u) != 0) bad = 1;
                        atomicOr(&S.bmask[o >> 5], 1u << (o & 31));
                        if (rank < (uint32_t)kMaxBoundaries) S.bpos[rank] = (uint16_t)o;
                        // raw offset just after the last marker of the chunk: where a chunk of
                        // whole intervals would resume
                        if (rank + 1 == nbnd) S.bcast[2] = (uint32_t)(my_lo + 16 * k + i + 1);
                        rank++;
                    }
                    if ((kp >> i) & 1u) {
                        const uint32_t wq = o >> 2, at = ((wq + (wq >> pad_shift)) << 2) | ((o & 3u) ^ 3u);
                        const uint8_t byte = (uint8_t)((wv[i >> 2] >> (8 * (i & 3))) & 255u);
                        cb[at] = byte;
                        // the first word of a subsequence is also the last of the row before
                        if (!short_intervals && (wq & 15u) == 0 && wq != 0) cb[at - 4] = byte;
                        o++;
                    }
                }
            }
        }
        __syncthreads();
        {
            // first interval start at or after each lane's subsequence: suffix minimum
            unsigned long long m = ((unsigned long long)S.bmask[2 * tid + 1] << 32) | S.bmask[2 * tid];
            uint32_t mine = m ? (uint32_t)tid * 64u + (uint32_t)__builtin_ctzll(m) : kNoMarker;
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
        WriteCtx wc;
        wc.coef = coef;
        wc.side_rel = side_rel;
        wc.bad = 0;

        // ---- short intervals: one lane per restart interval, one pass -----------------
        // A decoding lane is bound by the latency of its own dependent instructions, and a
        // wave takes as long as its slowest lane whatever the number of busy lanes:
        // consecutive intervals go to consecutive lanes, so that they fill as few waves as
        // possible and the other waves of the workgroup leave their SIMDs to other workgroups.
        if (short_intervals) {
            const uint32_t rem0 = g.ri_blocks - block_base % g.ri_blocks;  // blocks left in interval 0
            {
                // zeros over the blocks of the chunk's intervals: [z_lo, z_hi) of the image (a block
                // that is under way when the chunk begins was begun, and zeroed, in the chunk before)
                const uint32_t z_lo = min(block_base + ((st0 & 63u) ? 1u : 0u), g.n_blocks);
                const uint32_t z_hi = min(min(block_base + rem0 + (n_iv - 1) * g.ri_blocks, block_end), g.n_blocks);
                zero_blocks(coef, z_lo, z_hi, (uint32_t)tid, kT);
                __syncthreads();  // (and only then does any lane store a coefficient)
            }
            for (uint32_t k = (uint32_t)tid; k < n_iv; k += kT) {
                const uint32_t start = k ? pack_state((uint32_t)S.bpos[k - 1] * 8u, 0, 0) : st0;
                const uint32_t end_bit = k < nbnd ? (uint32_t)S.bpos[k] * 8u : limit_bits;
                const uint32_t blk0 = k ? block_base + rem0 + (k - 1) * g.ri_blocks : block_base;
                const uint32_t want = min(k ? g.ri_blocks : rem0, block_end > blk0 ? block_end - blk0 : 0u);
                wc.block = blk0;
                uint32_t got;
                const uint32_t fin = decode_interval(S, g, start, end_bit, &got, &wc);
                // the interval must end on its boundary, between MCUs, with exactly its blocks
                if (got != want || (fin & 511u) != 0 || (fin >> 9) != end_bit) wc.bad = 1;
            }
            bad |= wc.bad;
            {
                // DC values of the blocks whose DC was decoded here (the chunk may begin inside a block)
                const uint32_t dc_lo = block_base + ((st0 & 63u) ? 1u : 0u);
                block_base = min(block_base + rem0 + (n_iv - 1) * g.ri_blocks, block_end);
                dc_prefix(S, g, coef, coef + side_rel, dc_lo, min(block_base, g.n_blocks), dc_carry);
            }
            st0 = pack_state(0, 0, 0);
            dc_carry[0] = dc_carry[1] = dc_carry[2] = 0;
            if (last) { cs = rhi; break; }
            __syncthreads();
            const int32_t next_cs = (int32_t)S.bcast[2];
            if (next_cs <= cs || next_cs > rhi) { bad = 1; cs = rhi; break; }
            cs = next_cs;
            marker_base += nbnd;  // the next chunk starts just after the last marker of this one
            continue;
        }

        // ---- long intervals: speculative subsequences ------------------------------------
        // a chunk that is not the last keeps a tail back so that no symbol straddles its end
        const uint32_t own_bits = last ? limit_bits
                                       : (clean_len > (uint32_t)kChunkTail ? (clean_len - kChunkTail) * 8u : 0u);
        // What a lane takes: a subsequence, or, in the hypothesis passes of the smallest calls,
        // half of one (the passes are shorter, and a chunk of a small window has the lanes for
        // twice the rows); a lane's reads stay inside its subsequence's row either way.
        const uint32_t span_bits = kHyp && by_hypotheses && own_bits <= (uint32_t)kT * hyp_span_bits ? hyp_span_bits : kSubBits;
        const uint32_t nsub = (own_bits + span_bits - 1) / span_bits;  // <= kT
        const bool active = (uint32_t)tid < nsub;
        const uint32_t end_bit = min(((uint32_t)tid + 1u) * span_bits, own_bits);

        uint32_t in_state = tid == 0 ? st0 : pack_state((uint32_t)tid * span_bits, 0, 0);
        uint32_t out_state = in_state, nblk = 0;
        if (by_hypotheses) {
            // ---- the true states by place-in-MCU hypotheses ------------------------------
            // Subsequences [0, first) are settled; x = true state where subsequence `first`
            // begins.  A region is the next kT / H subsequences (H = blocks per MCU), lane
            // tid = j H + h working on subsequence first + j (row j) under hypothesis h.
            //   pass 0: decode from (first bit of the subsequence, block h of an MCU, DC), no
            //           matter where a symbol really begins there; the lanes of row 0 know the
            //           true state and decode from it.  End states -> cand[].
            //   pass 1: decode again from cand[] of the row before: these are the candidates
            //           for the true state at the row's start.  End states -> next[].
            //   link[] of a lane: which candidate of its own row its end state next[] equals.
            //   Lane 0 then follows the links from row to row.  Where the true state is none
            //   of the candidates (the true decoder had not fallen into step with any
            //   hypothesis by the end of the row before), the lanes of that row decode it
            //   once more from the true state, as row 0 did, and the walk goes on from there.
            __shared__ uint16_t hyp_blocks[kT];
            __shared__ uint8_t link[kT], chosen[kT];
            uint32_t *cand = reinterpret_cast<uint32_t *>(S.bpos);  // (the list of interval starts
            uint32_t *next = cand + kT;                             // is of no use to these passes)
            static_assert(sizeof(S.bpos) >= 2 * kT * sizeof(uint32_t), "cand[] and next[] fit");
            constexpr uint32_t kNoLink = 255;
            const uint32_t H = g.bpm, per = (uint32_t)kT / H;
            const uint32_t j = (uint32_t)tid / H, h = (uint32_t)tid - j * H;
            uint32_t first = 0, x = st0;
            for (uint32_t region = 0; region < nsub && first < nsub; region++) {
                const uint32_t cnt = min(per, nsub - first);
                const bool mine = j < cnt;
                const uint32_t s_end = min((first + j + 1u) * span_bits, own_bits);
                // which candidate of my row my end state equals (rows link to themselves: the
                // state where row j + 1 begins is looked up among the ends of row j)
                auto find_link = [&]() {
                    uint32_t hit = kNoLink;
                    for (uint32_t k = 0; k < H; k++)
                        if (cand[j * H + k] == next[tid]) { hit = k; break; }
                    link[tid] = (uint8_t)hit;
                };
                for (int pass = 0; pass < 2; pass++) {
                    const bool run = mine && (pass == 0 || j != 0);
                    if (run) {
                        const uint32_t from = pass == 0 ? (j == 0 ? x : pack_state((first + j) * span_bits, h, 0))
                                                        : cand[(uint32_t)tid - H];
                        uint32_t to = from, nb = 0;
                        // (a state past the subsequence's end: the lane before ran through it)
                        if ((from >> 9) < s_end) to = decode_span<false>(S, g, from, false, s_end, limit_bits, &nb, nullptr);
                        if (pass == 0) cand[tid] = to;
                        if (pass == 1 || j == 0) { next[tid] = to; hyp_blocks[tid] = (uint16_t)nb; }
                    }
                    __syncthreads();
                }
                // (row 0's own candidates are all the true end state: it links to candidate 0)
                if (mine) find_link();
                if (tid == 0) S.bcast[5] = 0;
                __syncthreads();
                // rows [0, walked) are settled; chosen[r] = the lane of row r that decoded from
                // the true state
                for (uint32_t walk = 0; walk < cnt; walk++) {
                    if (tid == 0) {
                        uint32_t r = S.bcast[5], k = 0;  // row r holds the true state in every lane
                        chosen[r] = 0;
                        for (r++; r < cnt; r++) {
                            k = link[(r - 1u) * H + k];
                            if (k == kNoLink) break;
                            chosen[r] = (uint8_t)k;
                        }
                        S.bcast[5] = r;
                    }
                    __syncthreads();
                    const uint32_t r = S.bcast[5];
                    if (r >= cnt) break;
                    // row r begins in a state that is no candidate: decode it from that state
                    if (j == r) {
                        const uint32_t from = next[(r - 1u) * H + chosen[r - 1u]];
                        uint32_t to = from, nb = 0;
                        if ((from >> 9) < s_end) to = decode_span<false>(S, g, from, false, s_end, limit_bits, &nb, nullptr);
                        next[tid] = to;
                        hyp_blocks[tid] = (uint16_t)nb;
                    }
                    __syncthreads();
                    if (j == r) find_link();
                    __syncthreads();
                }
                if ((uint32_t)tid >= first && (uint32_t)tid < first + cnt) {
                    const uint32_t r = (uint32_t)tid - first;
                    in_state = r == 0 ? x : next[(r - 1u) * H + chosen[r - 1u]];
                    out_state = next[r * H + chosen[r]];
                    nblk = hyp_blocks[r * H + chosen[r]];
                    S.state[tid] = out_state;
                }
                x = next[(cnt - 1u) * H + chosen[cnt - 1u]];
                first += cnt;
                __syncthreads();  // cand[], next[] and the rest are free again
            }
            if (!active) S.state[tid] = out_state;
        } else {
        // synchronise: iterate end states to their fixed point
        if (active) out_state = decode_span<false>(S, g, in_state, false, end_bit, limit_bits, &nblk, nullptr);
        S.state[tid] = out_state;
        for (uint32_t round = 0; round <= nsub; round++) {
            __syncthreads();
            int changed = 0;
            const uint32_t prev_state = tid > 0 ? S.state[tid - 1] : st0;
            __syncthreads();
            if (active && tid > 0 && prev_state != in_state) {
                in_state = prev_state;
                uint32_t o = in_state;
                // a predecessor that already ran past my subsequence leaves me nothing to decode
                if ((in_state >> 9) < end_bit) o = decode_span<false>(S, g, in_state, false, end_bit, limit_bits, &nblk, nullptr);
                else nblk = 0;
                if (o != out_state) { out_state = o; changed = 1; }
                S.state[tid] = out_state;
            }
            if (!__syncthreads_or(changed)) break;
        }
        }

        // write: decode once more from the true states
        uint32_t total_blocks;
        const uint32_t my_block = block_base + block_excl_scan(active ? nblk : 0u, S.scan_a, &total_blocks);
        wc.block = my_block;
        // a lane that begins on an MCU boundary where an interval ends must meet the boundary
        // first; lane 0 of a chunk may begin just after one (start of the run, or a boundary
        // consumed at the very end of the previous chunk)
        const bool boundary_due = (in_state & 511u) == 0 && g.ri_blocks != 0 && my_block % g.ri_blocks == 0 &&
                                  my_block < g.n_blocks && tid != 0;
        wc.iv_rem = boundary_due ? 0 : g.ri_blocks ? (int32_t)(g.ri_blocks - my_block % g.ri_blocks) : 0x7FFFFFFF;
        // Nothing has cleared the blocks: every lane stores zeros over the blocks whose first
        // coefficient it will decode (a block that is under way when the lane begins was begun,
        // and zeroed, by an earlier lane or chunk), and only then does any lane store a coefficient.
        if (active && (in_state >> 9) < end_bit) {
            const uint32_t z_lo = my_block + ((in_state & 63u) ? 1u : 0u);
            const uint32_t z_hi = min(my_block + nblk + ((out_state & 63u) ? 1u : 0u), g.n_blocks);
            zero_blocks(coef, z_lo, max(z_lo, z_hi), 0, 1);
        }
        __syncthreads();
        uint32_t final_state = out_state;
        if (active && (in_state >> 9) < end_bit) {
            uint32_t nb2;
            final_state = decode_span<true>(S, g, in_state, false, end_bit, limit_bits, &nb2, &wc);
            if (final_state != out_state || nb2 != nblk) wc.bad = 1;
        }
        bad |= wc.bad;
        __syncthreads();
        if (tid == 0) S.bcast[0] = nsub ? S.state[nsub - 1] : st0;
        __syncthreads();
        const uint32_t fs = S.bcast[0];  // true end state of the chunk
        {
            // DC values of the blocks whose DC was decoded in this chunk: it may begin inside
            // a block (DC decoded earlier) and end inside one (DC decoded here)
            const uint32_t dc_lo = block_base + ((st0 & 63u) ? 1u : 0u);
            const uint32_t dc_hi = block_base + total_blocks + ((fs & 63u) ? 1u : 0u);
            dc_prefix(S, g, coef, coef + side_rel, dc_lo, min(dc_hi, g.n_blocks), dc_carry);
        }

        // carry the true end state into the next chunk
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
        if (tid == 0) S.bcast[1] = S.bcast[3] = 0;
        __syncthreads();
        {
            // restart markers of this chunk that the next chunk will not stage again: those whose
            // interval begins at or before the clean byte the next chunk starts with
            const unsigned long long m = ((unsigned long long)S.bmask[2 * tid + 1] << 32) | S.bmask[2 * tid];
            const uint32_t first = (uint32_t)tid * 64u;
            if (m != 0 && qc >= first)
                atomicAdd(&S.bcast[3], qc - first >= 63u ? (uint32_t)__popcll(m)
                                                         : (uint32_t)__popcll(m & ((2ull << (qc - first)) - 1ull)));
        }
        if (S.keep_off[tid] <= qc && qc < S.keep_off[tid] + (uint32_t)__popcll(S.keep[tid])) {
            unsigned long long m = S.keep[tid];
            const uint32_t skip = qc - S.keep_off[tid];
            for (uint32_t i = 0; i < skip; i++) m &= m - 1;  // drop the lowest set bits
            S.bcast[1] = (uint32_t)(my_lo + (int32_t)__builtin_ctzll(m));
        }
        __syncthreads();
        const int32_t next_cs = (int32_t)S.bcast[1];
        if (next_cs <= cs || next_cs >= rhi) { bad = 1; cs = rhi; break; }  // no progress: refuse to spin
        cs = next_cs;
        st0 = pack_state(pbit & 7u, (fs >> 6) & 7u, fs & 63u);
        marker_base += S.bcast[3];
    }

    // the run must end on an MCU boundary with exactly the blocks it should hold
    if (tid == 0 && (block_base != block_end || (st0 & 511u) != 0)) bad = 1;
    if (__syncthreads_or(bad)) {
        if (tid == 0) atomicMin(&status[img], (int32_t)PREP_E_CORRUPT);
    }
}

size_t huff_tables_bytes() { return sizeof(HuffTables); }
static_assert(sizeof(HuffTables) % 16 == 0, "table slots are copied in 16-byte units");

void launch_scan_restart_markers(const uint8_t *bits, const ImageRec *recs, int n_images,
                                 uint32_t n_windows, uint32_t window_bytes, uint32_t *win_count, uint32_t *win_first,
                                 uint32_t *data_end,
                                 int32_t *status, const uint32_t *table_rep, uint32_t n_tables,
                                 uint8_t *tables, hipStream_t stream)
{
    if (n_windows == 0) return;
    hipLaunchKernelGGL(scan_restart_markers, dim3(n_windows + 4 * n_tables), dim3(kDecodeThreads), 0, stream,
                       bits, recs, n_images, n_windows, window_bytes, win_count, win_first, data_end, status, table_rep,
                       reinterpret_cast<uint4 *>(tables));
}

void launch_decode_entropy(const uint8_t *bits, const ImageRec *recs, int n_images,
                           uint32_t n_windows, const uint32_t *win_count, const uint32_t *win_first,
                           const uint32_t *data_end, int16_t *coef, uint32_t side_off, int32_t *status,
                           const uint8_t *tables, bool small_windows, uint32_t hyp_span_bits, hipStream_t stream)
{
    if (n_windows == 0) return;
    if (small_windows)
        hipLaunchKernelGGL(decode_entropy<true>, dim3(n_windows), dim3(kDecodeThreads), 0, stream, bits, recs,
                           n_images, win_count, win_first, data_end, coef, side_off, status,
                           reinterpret_cast<const uint4 *>(tables), hyp_span_bits);
    else
        hipLaunchKernelGGL(decode_entropy<false>, dim3(n_windows), dim3(kDecodeThreads), 0, stream, bits, recs,
                           n_images, win_count, win_first, data_end, coef, side_off, status,
                           reinterpret_cast<const uint4 *>(tables), hyp_span_bits);
}

}  // namespace prep
