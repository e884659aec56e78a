// Audio preprocessing for gfx950: resample -> log-Mel spectrogram -> per-feature normalize.
//
// The audio compute units of PREBA's DPU (section 2.3 item b; section 4.2, Fig. 11(b), Table 1:
// Resample, Mel spectrogram, Normalize).  The paper names the operations only; the definitions
// are: band-limited interpolation with a Hann-windowed sinc (six zero crossings, cut-off at
// 0.99 of the lower Nyquist rate); frames of n_fft samples every hop samples, centred by
// reflecting the signal at both ends, a periodic Hann window of win_length samples centred in
// the frame, squared magnitude of the DFT; n_mels unit-peak triangles with corners equally
// spaced on m(f) = 2595 log10(1 + f/700) from 0 to half the rate; ln(x + 2^-24); per Mel
// channel and utterance mean, variance (mean squared deviation) and
// (x - mean) / (sqrt(variance) + 1e-5).
//
// Tables (interpolation taps per phase, window, twiddle factors, Mel weights) are computed on
// the host in double precision.  From the input samples to the logarithm everything is double:
// fp64 runs at the rate of unpacked fp32 on this chip, and in float the transform's rounding
// noise (a few 1e-7 of the strongest bin) would be a visible fraction of the weak high bands
// whose logarithm is taken.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <numeric>
#include <vector>

#include "../../include/prep.h"

namespace {

constexpr int kZeroCrossings = 6;
constexpr double kRolloff = 0.99;
constexpr float kLogGuard = 5.9604644775390625e-08f;  // 2^-24
constexpr float kStdGuard = 1e-5f;
constexpr int kFft = 512;                             // the transform the kernel is built for
constexpr int kFrameThreads = 256;                    // four frames per workgroup, one wave each
constexpr int kMaxMels = 128;

struct Utterance {
    uint64_t in_off;    // first input sample
    uint64_t mid_off;   // first resampled sample in the workspace
    uint64_t out_off;   // first output element
    uint32_t in_len, mid_len, frames, pad_;
};

// ---- resample -----------------------------------------------------------------------------
// Output m = a q + r of an utterance (r < q) is sum_j x[a p + first[r] + j] taps[j][r]: the
// taps depend on the phase r only.  Neighbouring lanes have neighbouring phases, so tap j of
// all phases is contiguous.
__global__ __launch_bounds__(256) void resample_kernel(const float *__restrict__ in, const Utterance *__restrict__ utt,
                                                       const uint64_t *__restrict__ mid_start, int n_utt,
                                                       const double *__restrict__ taps, const int32_t *__restrict__ first,
                                                       int p, int q, int n_taps, double *__restrict__ mid,
                                                       uint64_t total)
{
    const uint64_t g = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= total) return;
    // the utterance that holds output g: the last one whose first output does not exceed g
    int lo = 0, hi = n_utt - 1;
    while (lo < hi) {
        const int m = (lo + hi + 1) >> 1;
        if (mid_start[m] <= g) lo = m; else hi = m - 1;
    }
    const Utterance u = utt[lo];
    const uint32_t m = (uint32_t)(g - u.mid_off);
    const uint32_t a = m / (uint32_t)q, r = m - a * (uint32_t)q;
    const int64_t n0 = (int64_t)a * p + first[r];
    const float *x = in + u.in_off;
    const double *t = taps + r;
    double acc = 0.0;
    if (n0 >= 0 && n0 + n_taps <= (int64_t)u.in_len) {
        // every tap lies inside the utterance
        const float *xs = x + n0;
#pragma unroll 4
        for (int j = 0; j < n_taps; j++) acc = fma((double)xs[j], t[(size_t)j * q], acc);
    } else {
        for (int j = 0; j < n_taps; j++) {
            const int64_t n = n0 + j;
            if (n >= 0 && n < (int64_t)u.in_len) acc = fma((double)x[n], t[(size_t)j * q], acc);
        }
    }
    mid[g] = acc;
}

// The same sum with the taps in registers: a thread keeps one phase r for all its outputs (the
// workgroup has a multiple of q threads and steps over whole multiples of q outputs), so its
// taps are loaded once and only the signal is read in the loop.  tile_start[u] = first
// workgroup of utterance u; a workgroup makes kTilesPerWg * blockDim.x consecutive outputs.
constexpr int kMaxTaps = 40;
// A rate pair p : q (reduced) is accepted up to this size of either term; its tap table has q
// rows of at most 2 * 6 / 0.99 * max(p / q, 1) + 2 taps, fewer than 14 * max(p, q) + 2 q entries.
constexpr int kMaxRateTerm = 4096;
constexpr size_t kMaxTapEntries = 16 * (size_t)kMaxRateTerm;
constexpr int kTilesPerWg = 8;

__global__ __launch_bounds__(512) void resample_phase_kernel(
    const float *__restrict__ in, const Utterance *__restrict__ utt, const uint64_t *__restrict__ tile_start,
    int n_utt, const double *__restrict__ taps, const int32_t *__restrict__ first, int p, int q, int n_taps,
    double *__restrict__ mid)
{
    int lo = 0, hi = n_utt - 1;
    while (lo < hi) {
        const int m = (lo + hi + 1) >> 1;
        if (tile_start[m] <= blockIdx.x) lo = m; else hi = m - 1;
    }
    const Utterance u = utt[lo];
    const uint32_t r = threadIdx.x % (uint32_t)q, sub = threadIdx.x / (uint32_t)q;
    const uint32_t per_tile = blockDim.x / (uint32_t)q;            // blocks of q outputs per tile
    double tap[kMaxTaps];
#pragma unroll
    for (int j = 0; j < kMaxTaps; j++) tap[j] = j < n_taps ? taps[(size_t)j * q + r] : 0.0;
    const float *x = in + u.in_off;
    double *y = mid + u.mid_off;
    // a = index of the block of q outputs
    uint32_t a = ((uint32_t)(blockIdx.x - tile_start[lo]) * kTilesPerWg) * per_tile + sub;
    const int32_t f = first[r];
    for (int it = 0; it < kTilesPerWg; it++, a += per_tile) {
        const uint64_t m = (uint64_t)a * (uint32_t)q + r;
        if (m >= u.mid_len) break;
        const int64_t n0 = (int64_t)a * p + f;
        double acc = 0.0;
        if (n0 >= 0 && n0 + kMaxTaps <= (int64_t)u.in_len) {
            const float *xs = x + n0;
#pragma unroll
            for (int j = 0; j < kMaxTaps; j++) acc = fma((double)xs[j], tap[j], acc);
        } else {
#pragma unroll
            for (int j = 0; j < kMaxTaps; j++) {
                const int64_t n = n0 + j;
                if (n >= 0 && n < (int64_t)u.in_len) acc = fma((double)x[n], tap[j], acc);
            }
        }
        y[m] = acc;
    }
}

// ---- frames -> log-Mel --------------------------------------------------------------------
struct MelTable {          // filter m covers bins start[m] .. start[m] + count[m] - 1
    int32_t start[kMaxMels], count[kMaxMels], first_weight[kMaxMels];
};

__device__ __forceinline__ double2 cadd(double2 a, double2 b) { return make_double2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ double2 csub(double2 a, double2 b) { return make_double2(a.x - b.x, a.y - b.y); }
__device__ __forceinline__ double2 cmul(double2 a, double2 b)
{
    return make_double2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
__device__ __forceinline__ double2 times_minus_i(double2 a) { return make_double2(a.y, -a.x); }

// Forward DFT of four values: Y[k] = sum_n y[n] (-i)^(n k)
__device__ __forceinline__ void dft4(const double2 y[4], double2 *Y0, double2 *Y1, double2 *Y2, double2 *Y3)
{
    const double2 s02 = cadd(y[0], y[2]), d02 = csub(y[0], y[2]);
    const double2 s13 = cadd(y[1], y[3]), d13 = times_minus_i(csub(y[1], y[3]));
    *Y0 = cadd(s02, s13);
    *Y2 = csub(s02, s13);
    *Y1 = cadd(d02, d13);
    *Y3 = csub(d02, d13);
}

// Forward DFT of eight values in place, natural order: even outputs from x[n] + x[n+4], odd
// ones from (x[n] - x[n+4]) W^n, W = exp(-2 pi i / 8).
__device__ __forceinline__ void dft8(double2 v[8])
{
    constexpr double h = 0.70710678118654752440;
    double2 e[4], o[4];
#pragma unroll
    for (int n = 0; n < 4; n++) {
        e[n] = cadd(v[n], v[n + 4]);
        o[n] = csub(v[n], v[n + 4]);
    }
    o[1] = make_double2(h * (o[1].x + o[1].y), h * (o[1].y - o[1].x));     // * (1 - i) / sqrt 2
    o[2] = times_minus_i(o[2]);
    o[3] = make_double2(h * (o[3].y - o[3].x), -h * (o[3].x + o[3].y));    // * (-1 - i) / sqrt 2
    dft4(e, &v[0], &v[2], &v[4], &v[6]);
    dft4(o, &v[1], &v[3], &v[5], &v[7]);
}

// LDS index of element i of a frame: one spare element after every eight keeps the eight lanes
// that a 16-byte access serves per cycle on different banks in every pass.
__device__ __forceinline__ int padded(int i) { return i + (i >> 3); }
constexpr int kFramePadded = kFft + kFft / 8;

// One wave per frame; a 512-point transform in three radix-8 passes (self-sorting: pass s reads
// element j + 64 r, multiplies by W512^(r k 512 / (8 Ns)), k = j mod Ns, Ns = 8^s, transforms
// the eight values and writes them Ns apart from (j / Ns) 8 Ns + k), each lane holding eight
// values in registers; the first pass reads the signal itself.  frame_start[u] = first frame of
// utterance u among all frames.  Sample is double for a resampled signal, float where the
// input is framed as it is.
template <typename Sample>
__global__ __launch_bounds__(kFrameThreads) void log_mel_kernel(
    const Sample *__restrict__ mid, const Utterance *__restrict__ utt, const uint64_t *__restrict__ frame_start,
    int n_utt, uint64_t n_frames, int hop, const double *__restrict__ window, const double2 *__restrict__ twiddle,
    MelTable mel, const double *__restrict__ mel_weights, int n_mels, float *__restrict__ out)
{
    __shared__ double2 s_x[kFrameThreads / 64][kFramePadded];
    __shared__ double s_power[kFrameThreads / 64][kFft / 2 + 1];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const uint64_t f = (uint64_t)blockIdx.x * (kFrameThreads / 64) + wave;
    if (f >= n_frames) return;   // no workgroup-wide barrier below: a wave works on its own frame
    int lo = 0, hi = n_utt - 1;
    while (lo < hi) {
        const int m = (lo + hi + 1) >> 1;
        if (frame_start[m] <= f) lo = m; else hi = m - 1;
    }
    const Utterance u = utt[lo];
    const uint32_t t = (uint32_t)(f - frame_start[lo]);
    double2 *x = s_x[wave];
    double2 v[8];
    {
        const Sample *sig = mid + u.mid_off;
        const int64_t len = (int64_t)u.mid_len;
#pragma unroll
        for (int r = 0; r < 8; r++) {
            const int j = lane + 64 * r;
            int64_t s = (int64_t)t * hop + j - kFft / 2;
            if (s < 0) s = -s;                       // reflection about the first sample
            if (s >= len) s = 2 * (len - 1) - s;     // and about the last (len > n_fft / 2)
            v[r] = make_double2((double)sig[s] * window[j], 0.0);
        }
    }
    dft8(v);
#pragma unroll
    for (int r = 0; r < 8; r++) x[padded(lane * 8 + r)] = v[r];
    // the accesses of one wave to LDS complete in order; the fence keeps the compiler from
    // moving loads over the stores
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
    for (int pass = 1; pass < 3; pass++) {
        const int ns = pass == 1 ? 8 : 64;
        const int k = lane & (ns - 1);
#pragma unroll
        for (int r = 0; r < 8; r++) v[r] = x[padded(lane + 64 * r)];
#pragma unroll
        for (int r = 1; r < 8; r++) v[r] = cmul(v[r], twiddle[r * k * (kFft / (8 * ns))]);
        dft8(v);
        if (pass == 1) {
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            const int j0 = (lane >> 3) * 64 + k;
#pragma unroll
            for (int r = 0; r < 8; r++) x[padded(j0 + 8 * r)] = v[r];
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        }
    }
    // after the last pass value r of lane j is bin j + 64 r: bins 0 .. 255, and 256 in lane 0
#pragma unroll
    for (int r = 0; r < 4; r++) s_power[wave][lane + 64 * r] = v[r].x * v[r].x + v[r].y * v[r].y;
    if (lane == 0) s_power[wave][kFft / 2] = v[4].x * v[4].x + v[4].y * v[4].y;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    // The triangles widen with their number, so a lane takes a narrow one and then the wide one
    // that mirrors it (m and n_mels - 1 - m): every busy lane sums about the same number of bins.
    for (int i = lane; i < (n_mels + 1) / 2; i += 64) {
#pragma unroll
        for (int side = 0; side < 2; side++) {
            const int m = side == 0 ? i : n_mels - 1 - i;
            if (side == 1 && m == i) break;  // the middle one of an odd number
            const double *w = mel_weights + mel.first_weight[m];
            const double *pw = s_power[wave] + mel.start[m];
            double acc = 0.0;
            for (int k = 0; k < mel.count[m]; k++) acc = fma(w[k], pw[k], acc);
            out[u.out_off + (uint64_t)m * u.frames + t] = (float)log(acc + (double)kLogGuard);
        }
    }
}

// ---- normalize ----------------------------------------------------------------------------
// One workgroup per (utterance, Mel channel) row: mean, then the mean squared deviation, then
// the normalised values, the row held in registers (up to kRowPerThread * 256 frames) or
// re-read from memory when longer.
constexpr int kRowPerThread = 16;

__device__ __forceinline__ double block_sum_256(double v, double *s)
{
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s[threadIdx.x >> 6] = v;
    __syncthreads();
    return s[0] + s[1] + s[2] + s[3];
}

__global__ __launch_bounds__(256) void normalize_kernel(const Utterance *__restrict__ utt, int n_mels, float *__restrict__ out)
{
    __shared__ double s[4];
    const Utterance u = utt[blockIdx.x / n_mels];
    float *row = out + u.out_off + (uint64_t)(blockIdx.x % n_mels) * u.frames;
    const uint32_t n = u.frames;
    const bool cached = n <= (uint32_t)kRowPerThread * 256u;
    float v[kRowPerThread];
    double sum = 0.0;
    if (cached) {
#pragma unroll
        for (int i = 0; i < kRowPerThread; i++) {
            const uint32_t k = threadIdx.x + 256u * i;
            v[i] = k < n ? row[k] : 0.0f;
            sum += v[i];
        }
    } else {
        for (uint32_t k = threadIdx.x; k < n; k += 256) sum += row[k];
    }
    const double mean = block_sum_256(sum, s) / (double)n;
    double dev = 0.0;
    if (cached) {
#pragma unroll
        for (int i = 0; i < kRowPerThread; i++) {
            const uint32_t k = threadIdx.x + 256u * i;
            const double d = (double)v[i] - mean;
            dev += k < n ? d * d : 0.0;
        }
    } else {
        for (uint32_t k = threadIdx.x; k < n; k += 256) { const double d = (double)row[k] - mean; dev += d * d; }
    }
    const double var = block_sum_256(dev, s) / (double)n;
    const double scale = 1.0 / (sqrt(var) + (double)kStdGuard);
    if (cached) {
#pragma unroll
        for (int i = 0; i < kRowPerThread; i++) {
            const uint32_t k = threadIdx.x + 256u * i;
            if (k < n) row[k] = (float)(((double)v[i] - mean) * scale);
        }
    } else {
        for (uint32_t k = threadIdx.x; k < n; k += 256) row[k] = (float)(((double)row[k] - mean) * scale);
    }
}

double sinc(double u) { return u == 0.0 ? 1.0 : sin(M_PI * u) / (M_PI * u); }

}  // namespace

struct prep_audio {
    prep_audio_config cfg;
    // tables on the device
    double *d_window = nullptr;
    double2 *d_twiddle = nullptr;
    double *d_mel_weights = nullptr;
    MelTable mel;
    // interpolation taps of the two rate pairs seen last, in buffers of the largest size a rate
    // pair can need (reserved in prep_audio_create: a call never allocates or frees)
    struct TapSlot {
        int p = 0, q = 0, n_taps = 0;
        double *d_taps = nullptr;
        int32_t *d_first = nullptr;
        uint64_t used = 0;       // call counter when the slot served last
    } slot[2];
    double *h_taps_pinned = nullptr;   // staging of an upload, free again once `done` has passed
    int32_t *h_first_pinned = nullptr;
    uint64_t calls = 0;
    // per call
    Utterance *h_utt = nullptr, *d_utt = nullptr;
    uint64_t *h_starts = nullptr, *d_starts = nullptr;  // [mid_start n][frame_start n][tile_start n]
    double *d_mid = nullptr;
    hipEvent_t done = nullptr;
    bool pending = false;
    std::vector<double> h_taps;
    std::vector<int32_t> h_first;
};

namespace {

#define AUDIO_TRY(expr)                                   \
    do {                                                  \
        if ((expr) != hipSuccess) {                       \
            (void)hipGetLastError();                      \
            return PREP_E_HIP;                            \
        }                                                 \
    } while (0)

uint64_t resampled_length(uint64_t len, int p, int q) { return (len * (uint64_t)q + (uint64_t)p - 1) / (uint64_t)p; }

// taps[j][r] = h((first[r] + j) / p - r / q) for phase r of p : q (input : output rate, reduced)
void make_taps(int p, int q, std::vector<double> *taps, std::vector<int32_t> *first, int *n_taps)
{
    const double base = kRolloff * std::min(p, q);
    const double reach = kZeroCrossings / base * p;  // in input samples
    int width = 0;
    first->resize((size_t)q);
    std::vector<int> last((size_t)q);
    for (int r = 0; r < q; r++) {
        const double centre = (double)r * p / q;
        (*first)[(size_t)r] = (int32_t)ceil(centre - reach);
        last[(size_t)r] = (int)floor(centre + reach);
        width = std::max(width, last[(size_t)r] - (*first)[(size_t)r] + 1);
    }
    *n_taps = width;
    taps->assign((size_t)q * width, 0.0);
    for (int r = 0; r < q; r++)
        for (int j = 0; j < width; j++) {
            const int n = (*first)[(size_t)r] + j;
            const double uarg = base * ((double)n / p - (double)r / q);
            if (fabs(uarg) < kZeroCrossings && n <= last[(size_t)r]) {
                const double c = cos(M_PI * uarg / (2.0 * kZeroCrossings));
                (*taps)[(size_t)j * q + r] = (base / p) * sinc(uarg) * c * c;
            }
        }
}

}  // namespace

extern "C" {

int64_t prep_audio_frames(const prep_audio_config *cfg, uint64_t samples_in, int32_t rate_in)
{
    if (!cfg || rate_in < 1 || cfg->rate < 1 || cfg->hop < 1) return PREP_E_INVALID_ARG;
    const int g = std::gcd(rate_in, cfg->rate);
    const uint64_t len = resampled_length(samples_in, rate_in / g, cfg->rate / g);
    return (int64_t)(1 + len / (uint64_t)cfg->hop);
}

int prep_audio_create(prep_audio **out, const prep_audio_config *cfg)
{
    if (!out) return PREP_E_INVALID_ARG;
    *out = nullptr;
    if (!cfg || cfg->max_batch < 1 || cfg->rate < 1 || cfg->n_fft != kFft || cfg->win_length < 1 ||
        cfg->win_length > cfg->n_fft || cfg->hop < 1 || cfg->n_mels < 1 || cfg->n_mels > kMaxMels ||
        cfg->max_total_samples < 1)
        return PREP_E_INVALID_ARG;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || cfg->device < 0 || cfg->device >= ndev) {
        (void)hipGetLastError();
        return PREP_E_HIP;
    }
    prep_audio *h = new (std::nothrow) prep_audio;
    if (!h) return PREP_E_NOMEM;
    h->cfg = *cfg;
    // window, twiddle factors, Mel triangles: double precision, rounded once
    std::vector<double> window((size_t)kFft, 0.0);
    const int left = (kFft - cfg->win_length) / 2;
    for (int i = 0; i < cfg->win_length; i++)
        window[(size_t)(left + i)] = 0.5 - 0.5 * cos(2.0 * M_PI * i / cfg->win_length);
    std::vector<double2> tw((size_t)kFft);  // W^k = exp(-2 pi i k / 512), k = 0 .. 511 (r k reaches 7 * 63)
    for (int k = 0; k < kFft; k++)
        tw[(size_t)k] = make_double2(cos(2.0 * M_PI * k / kFft), -sin(2.0 * M_PI * k / kFft));
    std::vector<double> weights;
    {
        auto mel_of = [](double f) { return 2595.0 * log10(1.0 + f / 700.0); };
        auto hz_of = [](double m) { return 700.0 * (pow(10.0, m / 2595.0) - 1.0); };
        const double top = mel_of(cfg->rate / 2.0);
        std::vector<double> corner((size_t)cfg->n_mels + 2);
        for (int i = 0; i < cfg->n_mels + 2; i++) corner[(size_t)i] = hz_of(top * i / (cfg->n_mels + 1));
        for (int m = 0; m < cfg->n_mels; m++) {
            const double lo = corner[(size_t)m], mid = corner[(size_t)m + 1], hi = corner[(size_t)m + 2];
            h->mel.start[m] = 0;
            h->mel.count[m] = 0;
            h->mel.first_weight[m] = (int32_t)weights.size();
            for (int k = 0; k <= kFft / 2; k++) {
                const double f = (double)k * cfg->rate / kFft;
                const double w = std::max(0.0, std::min((f - lo) / (mid - lo), (hi - f) / (hi - mid)));
                if (w > 0.0) {
                    if (h->mel.count[m] == 0) h->mel.start[m] = k;
                    // zeros between positive weights cannot occur in a triangle
                    h->mel.count[m] = k - h->mel.start[m] + 1;
                    weights.push_back(w);
                }
            }
        }
        if (weights.empty()) weights.push_back(0.0);
    }
    const size_t n = (size_t)cfg->max_batch;
    bool ok = hipSetDevice(cfg->device) == hipSuccess;
    ok = ok && hipMalloc((void **)&h->d_window, sizeof(double) * kFft) == hipSuccess;
    ok = ok && hipMalloc((void **)&h->d_twiddle, sizeof(double2) * kFft) == hipSuccess;
    ok = ok && hipMalloc((void **)&h->d_mel_weights, sizeof(double) * weights.size()) == hipSuccess;
    ok = ok && hipMalloc((void **)&h->d_utt, sizeof(Utterance) * n) == hipSuccess;
    ok = ok && hipMalloc((void **)&h->d_starts, sizeof(uint64_t) * 3 * n) == hipSuccess;
    ok = ok && hipHostMalloc((void **)&h->h_utt, sizeof(Utterance) * n, hipHostMallocDefault) == hipSuccess;
    ok = ok && hipHostMalloc((void **)&h->h_starts, sizeof(uint64_t) * 3 * n, hipHostMallocDefault) == hipSuccess;
    // the resampled signal is never longer than max_total_samples scaled by the largest ratio accepted
    ok = ok && hipMalloc((void **)&h->d_mid, sizeof(double) * (cfg->max_total_samples + n)) == hipSuccess;
    for (auto &ts : h->slot) {
        ok = ok && hipMalloc((void **)&ts.d_taps, sizeof(double) * kMaxTapEntries) == hipSuccess;
        ok = ok && hipMalloc((void **)&ts.d_first, sizeof(int32_t) * kMaxRateTerm) == hipSuccess;
    }
    ok = ok && hipHostMalloc((void **)&h->h_taps_pinned, sizeof(double) * kMaxTapEntries, hipHostMallocDefault) == hipSuccess;
    ok = ok && hipHostMalloc((void **)&h->h_first_pinned, sizeof(int32_t) * kMaxRateTerm, hipHostMallocDefault) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&h->done, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipMemcpy(h->d_window, window.data(), sizeof(double) * kFft, hipMemcpyHostToDevice) == hipSuccess;
    ok = ok && hipMemcpy(h->d_twiddle, tw.data(), sizeof(double2) * kFft, hipMemcpyHostToDevice) == hipSuccess;
    ok = ok && hipMemcpy(h->d_mel_weights, weights.data(), sizeof(double) * weights.size(), hipMemcpyHostToDevice) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        prep_audio_destroy(h);
        return PREP_E_NOMEM;
    }
    *out = h;
    return PREP_OK;
}

int prep_audio_destroy(prep_audio *h)
{
    if (!h) return PREP_E_INVALID_ARG;
    (void)hipSetDevice(h->cfg.device);
    if (h->pending) (void)hipEventSynchronize(h->done);
    (void)hipFree(h->d_window);
    (void)hipFree(h->d_twiddle);
    (void)hipFree(h->d_mel_weights);
    (void)hipFree(h->d_utt);
    (void)hipFree(h->d_starts);
    (void)hipFree(h->d_mid);
    for (auto &ts : h->slot) {
        (void)hipFree(ts.d_taps);
        (void)hipFree(ts.d_first);
    }
    if (h->h_taps_pinned) (void)hipHostFree(h->h_taps_pinned);
    if (h->h_first_pinned) (void)hipHostFree(h->h_first_pinned);
    if (h->h_utt) (void)hipHostFree(h->h_utt);
    if (h->h_starts) (void)hipHostFree(h->h_starts);
    if (h->done) (void)hipEventDestroy(h->done);
    delete h;
    return PREP_OK;
}

int prep_audio_features(prep_audio *h, const float *waveforms, const uint64_t *offsets, int32_t n, int32_t rate_in,
                        float *out, uint64_t *out_offsets, void *stream_ptr)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
    if (!h || !waveforms || !offsets || !out || !out_offsets || n < 0 || rate_in < 1) return PREP_E_INVALID_ARG;
    if (n > h->cfg.max_batch) return PREP_E_TOO_LARGE;
    out_offsets[0] = 0;
    if (n == 0) return PREP_OK;
    const int g = std::gcd(rate_in, h->cfg.rate);
    const int p = rate_in / g, q = h->cfg.rate / g;
    if (p > kMaxRateTerm || q > kMaxRateTerm) return PREP_E_INVALID_ARG;  // the tap table has q rows
    AUDIO_TRY(hipSetDevice(h->cfg.device));
    if (h->pending) {  // the pinned records of the call before are still being read
        AUDIO_TRY(hipEventSynchronize(h->done));
        h->pending = false;
    }
    uint64_t mid_total = 0, frames_total = 0, out_total = 0, tiles_total = 0;
    // threads per workgroup of the resampler that keeps its taps in registers: a multiple of q
    const uint32_t phase_threads = q <= 320 ? (uint32_t)q * (uint32_t)std::max(1, 320 / q) : 0u;
    const uint64_t per_wg = (uint64_t)phase_threads * kTilesPerWg;
    for (int32_t i = 0; i < n; i++) {
        if (offsets[i + 1] < offsets[i] || offsets[i + 1] - offsets[i] > 0xFFFFFFFFull) return PREP_E_INVALID_ARG;
        Utterance &u = h->h_utt[i];
        u.in_off = offsets[i];
        u.in_len = (uint32_t)(offsets[i + 1] - offsets[i]);
        const uint64_t len = resampled_length(u.in_len, p, q);
        // centring reflects n_fft / 2 samples at both ends
        if (len <= (uint64_t)kFft / 2 || len > 0x7FFFFFFFull) return PREP_E_INVALID_ARG;
        u.mid_len = (uint32_t)len;
        u.frames = (uint32_t)(1 + len / (uint64_t)h->cfg.hop);
        u.mid_off = mid_total;
        u.out_off = out_total;
        u.pad_ = 0;
        h->h_starts[i] = mid_total;
        h->h_starts[(size_t)n + i] = frames_total;
        h->h_starts[2 * (size_t)n + i] = tiles_total;
        if (per_wg) tiles_total += (len + per_wg - 1) / per_wg;
        mid_total += len;
        frames_total += u.frames;
        out_total += (uint64_t)u.frames * (uint64_t)h->cfg.n_mels;
        out_offsets[i + 1] = out_total;
    }
    if (offsets[n] - offsets[0] > h->cfg.max_total_samples || mid_total > h->cfg.max_total_samples + (uint64_t)n)
        return PREP_E_TOO_LARGE;
    prep_audio::TapSlot *taps = &h->slot[0];
    if (p != q) {
        h->calls++;
        if (!(taps->p == p && taps->q == q)) {
            if (h->slot[1].p == p && h->slot[1].q == q) {
                taps = &h->slot[1];
            } else {
                // a new rate pair: build its taps into the slot that served longest ago and upload
                // them on the caller's stream, ahead of the kernels that read them (the pinned
                // staging is free: the call before has been waited for above; so is the slot)
                if (h->slot[1].used < taps->used) taps = &h->slot[1];
                make_taps(p, q, &h->h_taps, &h->h_first, &taps->n_taps);
                if (h->h_taps.size() > kMaxTapEntries) return PREP_E_TOO_LARGE;
                memcpy(h->h_taps_pinned, h->h_taps.data(), sizeof(double) * h->h_taps.size());
                memcpy(h->h_first_pinned, h->h_first.data(), sizeof(int32_t) * (size_t)q);
                AUDIO_TRY(hipMemcpyAsync(taps->d_taps, h->h_taps_pinned, sizeof(double) * h->h_taps.size(),
                                         hipMemcpyHostToDevice, stream));
                AUDIO_TRY(hipMemcpyAsync(taps->d_first, h->h_first_pinned, sizeof(int32_t) * (size_t)q,
                                         hipMemcpyHostToDevice, stream));
                taps->p = p;
                taps->q = q;
            }
        }
        taps->used = h->calls;
    }
    if (p == q) {
        // same rate: the frames read the input itself; utterance offsets are the input's
        for (int32_t i = 0; i < n; i++) h->h_utt[i].mid_off = h->h_utt[i].in_off;
    }
    AUDIO_TRY(hipMemcpyAsync(h->d_utt, h->h_utt, sizeof(Utterance) * (size_t)n, hipMemcpyHostToDevice, stream));
    AUDIO_TRY(hipMemcpyAsync(h->d_starts, h->h_starts, sizeof(uint64_t) * 3 * (size_t)n, hipMemcpyHostToDevice, stream));
    if (p != q && phase_threads && taps->n_taps <= kMaxTaps && tiles_total <= 0x7FFFFFFFull) {
        hipLaunchKernelGGL(resample_phase_kernel, dim3((unsigned)tiles_total), dim3(phase_threads), 0, stream, waveforms,
                           h->d_utt, h->d_starts + 2 * n, n, taps->d_taps, taps->d_first, p, q, taps->n_taps, h->d_mid);
    } else if (p != q) {
        hipLaunchKernelGGL(resample_kernel, dim3((unsigned)((mid_total + 255) / 256)), dim3(256), 0, stream, waveforms,
                           h->d_utt, h->d_starts, n, taps->d_taps, taps->d_first, p, q, taps->n_taps, h->d_mid, mid_total);
    }
    const dim3 frame_grid((unsigned)((frames_total + 3) / 4));
    if (p == q)
        hipLaunchKernelGGL(log_mel_kernel<float>, frame_grid, dim3(kFrameThreads), 0, stream, waveforms, h->d_utt,
                           h->d_starts + n, n, frames_total, h->cfg.hop, h->d_window, h->d_twiddle, h->mel,
                           h->d_mel_weights, h->cfg.n_mels, out);
    else
        hipLaunchKernelGGL(log_mel_kernel<double>, frame_grid, dim3(kFrameThreads), 0, stream, (const double *)h->d_mid,
                           h->d_utt, h->d_starts + n, n, frames_total, h->cfg.hop, h->d_window, h->d_twiddle, h->mel,
                           h->d_mel_weights, h->cfg.n_mels, out);
    hipLaunchKernelGGL(normalize_kernel, dim3((unsigned)n * (unsigned)h->cfg.n_mels), dim3(256), 0, stream, h->d_utt,
                       h->cfg.n_mels, out);
    AUDIO_TRY(hipGetLastError());
    AUDIO_TRY(hipEventRecord(h->done, stream));
    h->pending = true;
    return PREP_OK;
}

}  // extern "C"
