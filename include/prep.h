/*
 * prep -- batched JPEG -> model-input tensor preprocessing on one AMD Instinct
 * MI355X (gfx950).
 *
 * The library computes the "data preprocessing" stage of an inference server
 * for vision models as PREBA states it (section 2.3, item 1; the Decode,
 * Resize, Crop and Normalize functional units of the image CU in section 4.2,
 * Figure 11(a) and Table 1): every image of a batch is decoded from a JPEG
 * bitstream to RGB, resized, cropped to the model's input size and normalized.
 * The paper fixes nothing below that level; this library reads it as
 *   decode    : ITU-T T.81 baseline sequential DCT, Huffman coded, 8 bit,
 *               1 or 3 components in one interleaved scan, sampling gray /
 *               4:4:4 / 4:2:0 / 4:2:2 / 4:4:0, optional restart intervals; chroma upsampled by
 *               sample replication (or interpolated, PREP_FLAG_SMOOTH_CHROMA); JFIF YCbCr -> RGB; samples and RGB values
 *               rounded half up and clamped to 0..255;
 *   resize    : short side -> resize_short, long side floor(resize_short *
 *               long / short); bilinear, pixel centres at half-integers,
 *               per-axis scale in/out, taps clamped at the border, no
 *               prefilter, no intermediate rounding (PREP_FILTER_BILINEAR), or the
 *               antialiased form of it (PREP_FILTER_ANTIALIAS, see there);
 *   crop      : centre window crop_h x crop_w, origin floor(margin / 2);
 *   normalize : (v / 255 - mean[c]) / std[c];
 *   output    : planar NCHW, RGB channel order, fp32 or fp16; or, without normalize,
 *               the resized crop as interleaved 8-bit RGB (PREP_U8_NHWC).
 *
 * One restriction inside the baseline subset: the two chroma components must name the same
 * Huffman tables (the decoder holds one DC/AC pair for luma and one for chroma; a file that
 * gives Cb and Cr different tables is reported PREP_E_UNSUPPORTED).  A file may go on after
 * its image (a second image, a preview, padding): the host, which does not read the
 * entropy-coded bytes, takes them to run up to the file's last EOI marker, and the GPU ends
 * them at the first FF D9 inside (which cannot occur in entropy-coded data, T.81 F.1.2.3).
 *
 * All entry points are plain C.  "HOST" pointers are ordinary process memory,
 * "DEVICE" pointers are HIP device memory of the handle's GPU.  A handle may be
 * used by one thread and one stream at a time; use several handles for
 * concurrent streams.  Every function returns PREP_OK (0) or a negative
 * PREP_E_* code and never throws, aborts or prints.
 */
#ifndef PREP_H
#define PREP_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    PREP_OK = 0,
    PREP_E_INVALID_ARG = -1, /* null pointer, n out of range, bad params            */
    PREP_E_TOO_LARGE = -2,   /* batch exceeds what prep_create reserved             */
    PREP_E_HIP = -3,         /* a HIP runtime call failed                           */
    PREP_E_UNSUPPORTED = -4, /* per image: valid JPEG outside the supported subset  */
    PREP_E_CORRUPT = -5,     /* per image: stream violates the JPEG syntax          */
    PREP_E_NOMEM = -6        /* host or device allocation failed in prep_create     */
};

/* Output element type and layout.  PREP_F32, PREP_F16: the normalized tensor, planar
 * [n][3][crop_h][crop_w].  PREP_U8_NHWC: Resize and Crop without Normalize (mean and std are
 * not looked at), the resized samples rounded to the nearest integer, halves upwards, as
 * interleaved RGB bytes [n][crop_h][crop_w][3].  The kernels interpolate in fp32: a sample
 * that lies within 2^-12 below a half is taken for the half (rational scales produce exact
 * halves all the time, and fp32 lands on either side of them), so a result may be one level
 * above the exactly rounded one there. */
enum { PREP_F32 = 0, PREP_F16 = 1, PREP_U8_NHWC = 2 };

/* The Resize unit's filter (PREBA section 4.2, Table 1 names the unit, not the filter).
 * PREP_FILTER_BILINEAR: two samples per axis around the output sample's centre (half-pixel
 *   centres, clamped at the border), whatever the scale.
 * PREP_FILTER_ANTIALIAS: where an axis shrinks, the mean of the source samples under a
 *   triangle centred on the output sample and as wide as an output sample (support
 *   in/out source samples each way), the window cut at the image's edge and the weights
 *   scaled to sum 1, which is what image libraries do when they reduce an image; where an
 *   axis grows it is PREP_FILTER_BILINEAR. */
enum { PREP_FILTER_BILINEAR = 0, PREP_FILTER_ANTIALIAS = 1 };
/* prep_config.flags.
 * PREP_FLAG_TABLES_PER_WORKGROUP: expand the Huffman tables in every decoder workgroup
 *   instead of once per distinct table set of the batch (same results; kept for checking
 *   that path).
 * PREP_FLAG_FULL_RGB: convert every MCU of every image to RGB.  Without it only the MCUs
 *   whose pixels the crop window's outputs read (the two taps per axis of the bilinear filter,
 *   the samples under the triangles of the antialiased one) are converted (the output tensor is the
 *   same; the paper's image unit streams decode into resize and crop without keeping a
 *   decoded image either, section 4.2), and prep_debug_last_rgb returns what the workspace
 *   holds outside those MCUs.
 * PREP_FLAG_SMOOTH_CHROMA: a decode variant (flexibility objective of section 4.2).  Subsampled
 *   chroma (4:2:0, 4:2:2, 4:4:0) is brought to full resolution by linear interpolation between
 *   sample centres (a centred triangle: a pixel takes 3/4 of the chroma sample it belongs to and
 *   1/4 of the next one on its side, per subsampled axis; the sample at the image's edge stands
 *   in for a neighbour outside; rounded to the nearest integer, halves upwards) instead of
 *   sample replication.  Reconstruction then takes two kernels and a chroma workspace a third
 *   of the RGB workspace's size; prep_debug_last_region leaves out the outermost chroma sample
 *   of the converted region where that does not end with the image.
 * PREP_FLAG_LARGE_WINDOWS: a call with little entropy-coded data (up to 1.5 MiB, and in
 *   smaller pieces still up to 448 KiB) is normally cut into more and smaller pieces for the
 *   entropy decoder, which then finds the decoder states
 *   inside restart intervals by hypotheses over the block's place in the MCU, so that the
 *   single-input and small-batch latency (a design objective of section 4.2) is not that of
 *   one lane walking a restart interval; with this flag such a call is decoded like a large
 *   one (same results; kept for checking that path on small inputs). */
enum { PREP_FLAG_TABLES_PER_WORKGROUP = 1, PREP_FLAG_FULL_RGB = 2, PREP_FLAG_SMOOTH_CHROMA = 4,
       PREP_FLAG_LARGE_WINDOWS = 8 };
/* luma sampling factors H x V (chroma is 1 x 1): 4:4:4 = 1 x 1, 4:2:0 = 2 x 2, 4:2:2 = 2 x 1,
 * 4:4:0 = 1 x 2; GRAY = one component */
enum { PREP_SAMPLING_444 = 0, PREP_SAMPLING_420 = 1, PREP_SAMPLING_GRAY = 2, PREP_SAMPLING_422 = 3,
       PREP_SAMPLING_440 = 4 };

typedef struct prep_handle prep_handle;

/* Capacity of a handle; all device and pinned host memory is reserved here. */
typedef struct {
    int32_t device;               /* HIP device ordinal                              */
    int32_t max_batch;            /* largest n of one call                           */
    int32_t max_width, max_height; /* largest single image                          */
    uint64_t max_bitstream_bytes; /* largest sum of file sizes of one call           */
    uint64_t max_total_pixels;    /* largest sum of width*height of one call;
                                     0 = max_batch * max_width * max_height         */
    uint32_t flags;               /* 0 or PREP_FLAG_*; other bits must be 0          */
} prep_config;

/* Resize / crop / normalize parameters, the same for every image of a call. */
typedef struct {
    int32_t resize_short;  /* target length of the short side; 0 = keep the size    */
    int32_t crop_h, crop_w;
    int32_t out_dtype;     /* PREP_F32, PREP_F16 or PREP_U8_NHWC                    */
    float mean[3], std[3]; /* on the 0..1 pixel scale, R, G, B                      */
    int32_t filter;        /* PREP_FILTER_BILINEAR or PREP_FILTER_ANTIALIAS         */
} prep_params;

/* What the host marker parser learns about one file (T.81 Annex B). */
typedef struct {
    int32_t status;            /* PREP_OK, PREP_E_UNSUPPORTED or PREP_E_CORRUPT     */
    int32_t width, height;
    int32_t sampling;          /* PREP_SAMPLING_*                                   */
    int32_t mcu_cols, mcu_rows;
    int32_t blocks_per_mcu;    /* 1, 3, 4 or 6                                      */
    int32_t restart_interval;  /* MCUs per restart interval, 0 = none               */
    int32_t n_intervals;       /* restart-interval work descriptors of this image   */
    int32_t reserved;
    uint64_t entropy_offset;   /* first entropy-coded byte, from the file start     */
    uint64_t entropy_bytes;    /* up to, not including, the file's last EOI marker  */
} prep_image_info;

/* One restart-interval work descriptor: the unit of independent entropy
 * decoding (T.81 E.2.4).  The parser knows which MCUs an interval covers; where
 * its bytes begin inside the entropy-coded segment is found on the GPU.       */
typedef struct {
    int32_t image;      /* index into the batch                                     */
    int32_t first_mcu;  /* first MCU of the interval, raster order                  */
    int32_t n_mcu;      /* MCUs in the interval                                     */
    int32_t rst_index;  /* n of the RSTn marker that precedes it, -1 for the first  */
} prep_interval_desc;

/* Reserve a handle's memory on cfg->device.  *out is NULL on failure.         */
int prep_create(prep_handle **out, const prep_config *cfg);

/* Release everything the handle owns (synchronises the device first).         */
int prep_destroy(prep_handle *h);

/*
 * The whole path for one batch (section 2.3 item 1 / section 4.2): parse, copy
 * to the GPU, entropy-decode, reconstruct RGB, resize + crop + normalize.
 *   bitstreams HOST   n files back to back
 *   offsets    HOST   n+1 entries; file i is bytes [offsets[i], offsets[i+1])
 *   out        DEVICE n*3*crop_h*crop_w elements of params->out_dtype, NCHW (NHWC for
 *              PREP_U8_NHWC);
 *              must stay valid until `stream` has run the enqueued work
 *   stream     a hipStream_t (NULL = the default stream)
 * The call copies what it needs from the host buffers before it returns (copies of 1 MiB
 * or more with the help of three threads that the library starts once per process) and
 * returns as soon as the GPU work is enqueued on `stream` (uploads of large
 * batches run on a stream of the handle that `stream` is made to wait for).  Whole-call errors
 * (INVALID_ARG, TOO_LARGE, HIP) enqueue nothing.  A file that cannot be decoded
 * does not fail the call: its status is reported by prep_get_status and its
 * slab of `out` is filled with zeros.
 */
int prep_decode_resize_batch(prep_handle *h, const uint8_t *bitstreams, const uint64_t *offsets,
                             int32_t n, const prep_params *params, void *out, void *stream);

/*
 * Same computation for a batch whose bytes already lie in device memory:
 * `bitstreams_device` (DEVICE) holds the same bytes as `bitstreams` (HOST).  Of
 * the host copy only the headers up to each file's start-of-scan header (a few
 * hundred bytes per file) and the bytes at its end (to find the EOI marker) are
 * read; the entropy-coded data is read on the GPU alone and is not copied.
 * `bitstreams_device` must stay valid until `stream` has run the work.  The
 * kernels read it with aligned 16-byte loads that contain at least one byte of
 * a file, so they stay inside the last page of the buffer whatever its size.
 */
int prep_decode_resize_batch_resident(prep_handle *h, const uint8_t *bitstreams,
                                      const uint8_t *bitstreams_device, const uint64_t *offsets,
                                      int32_t n, const prep_params *params, void *out,
                                      void *stream);

/* Wait for the handle's last call and fetch one status per image (HOST, n
 * entries of the last call): PREP_OK, PREP_E_UNSUPPORTED or PREP_E_CORRUPT.   */
int prep_get_status(prep_handle *h, int32_t *per_image_status, int32_t n);

/* Text for a PREP_* code (static storage).                                    */
const char *prep_strerror(int code);

/* ---- host-only pieces (no GPU needed) ---------------------------------- */

/* The marker/table parser alone (T.81 Annex B): fills info[i] for each file. */
int prep_parse_headers(const uint8_t *bitstreams, const uint64_t *offsets, int32_t n,
                       prep_image_info *info);

/* Restart-interval work descriptors of a parsed batch, image after image.
 * Writes at most cap entries and returns the total number (>= 0).             */
int64_t prep_interval_descriptors(const prep_image_info *info, int32_t n,
                                  prep_interval_desc *desc, int64_t cap);

/* ---- single stages, for checking each against its own definition ---------- */

/*
 * Resize + centre crop + normalize alone (the Resize, Crop and Normalize units
 * of Table 1) on RGB images the caller supplies.
 *   rgb      DEVICE  interleaved 8-bit RGB images; image i starts at byte
 *            rgb_offsets[i], rows are pitches[i] bytes apart
 *   rgb_offsets, widths, heights, pitches   HOST, n entries each
 */
int prep_resize_normalize(prep_handle *h, const uint8_t *rgb, const uint64_t *rgb_offsets,
                          const int32_t *widths, const int32_t *heights, const int32_t *pitches,
                          int32_t n, const prep_params *params, void *out, void *stream);

/*
 * prep_resize_normalize for callers that cannot allocate: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments without a handle (device = HIP device ordinal), same kernels, same
 * results.  The per-image mapping records that the kernels read, which
 * prep_resize_normalize keeps in buffers of its handle, live in a device array
 * of fixed size inside the library (PREP_STATIC_MAX_IMAGES records, 56 KiB per
 * GPU, held until the process ends); the records reach it as kernel arguments.
 * The call makes no hipMalloc, hipFree or other allocating call.
 * n > PREP_STATIC_MAX_IMAGES returns PREP_E_TOO_LARGE and enqueues nothing.
 * Every call on a GPU uses that GPU's one array: calls that may overlap on one
 * GPU (two streams, two threads) race and must be serialised by the caller;
 * calls on one stream are ordered by the stream.
 */
#define PREP_STATIC_MAX_IMAGES 1024
int prep_resize_normalize_static(int32_t device, const uint8_t *rgb, const uint64_t *rgb_offsets,
                                 const int32_t *widths, const int32_t *heights,
                                 const int32_t *pitches, int32_t n, const prep_params *params,
                                 void *out, void *stream);

/*
 * Dequantise + inverse DCT + chroma upsampling + colour conversion (the second
 * half of the Decode unit), then resize/crop/normalize, from coefficients the
 * caller supplies instead of the entropy decoder's: the files' headers give
 * geometry and quantisation tables.
 *   coefficients HOST  for each image in turn, its blocks in scan order, 64
 *                int16 per block in zig-zag order with absolute DC values
 * Unlike the batch calls this one waits for `stream` before it returns (the
 * coefficients are copied from pageable host memory): it is a checking aid.
 */
int prep_reconstruct_from_coefficients(prep_handle *h, const uint8_t *bitstreams,
                                       const uint64_t *offsets, int32_t n,
                                       const int16_t *coefficients, uint64_t n_coefficients,
                                       const prep_params *params, void *out, void *stream);

/* ---- checkpoints of the last call, copied to the host (these synchronise) - */

/* Entropy decoder output of image `image`: blocks in scan order (MCU by MCU;
 * in a 4:2:0 MCU Y00 Y01 Y10 Y11 Cb Cr), 64 int16 per block in zig-zag order,
 * DC values absolute.  `cap` counts int16 entries; returns the number written
 * (blocks*64) or a negative code.                                             */
int64_t prep_debug_last_coefficients(prep_handle *h, int32_t image, int16_t *host_out,
                                     uint64_t cap);

/* Decoded RGB of image `image`: height*width*3 bytes, interleaved, tightly
 * packed.  Returns the number of bytes written or a negative code.  Only the
 * pixels inside the rectangle of prep_debug_last_region are the image's.      */
int64_t prep_debug_last_rgb(prep_handle *h, int32_t image, uint8_t *host_out_hwc, uint64_t cap);

/* The pixels of image `image` that the last call converted to RGB:
 * rect = {x0, y0, x1, y1}, columns x0 <= x < x1 and rows y0 <= y < y1 (HOST,
 * 4 entries).  It is the whole image for a handle created with
 * PREP_FLAG_FULL_RGB, else the MCUs that the crop window's outputs read
 * through the call's resize filter, clipped to the image.  Returns PREP_OK, the image's own status if
 * it was refused, or PREP_E_INVALID_ARG.                                      */
int prep_debug_last_region(prep_handle *h, int32_t image, int32_t rect[4]);

/* Stage timing.  While enabled, every batch call brackets its GPU stages with
 * events on the call's stream (calls that enqueue no decode are not counted).
 * prep_stage_ms waits for the call made `calls_back` timed calls ago (0 = the
 * last one; at most the last 256 are kept) and returns the milliseconds of
 * [0] restart-marker scan (with expanding the batch's Huffman tables), [1] entropy
 * decode, [2] reconstruct RGB, [3] resize/crop/normalize.  prep_set_timing
 * forgets earlier timings.                                                    */
int prep_set_timing(prep_handle *h, int32_t enabled);
int prep_stage_ms(prep_handle *h, int32_t calls_back, float ms[4]);

/* ---- dynamic batching (PREBA section 4.3, "Dynamic Batching System") --------
 *
 * Single-input requests wait in one queue.  A batch is released as soon as
 * batch_max requests wait (Batch_max) or the oldest has waited time_queue
 * (Time_queue, which the paper sets to the consumer's tail latency at the knee
 * divided by the number of consumers); a free consumer then takes the oldest
 * requests waiting at that moment, at most batch_max.
 *
 * prep_policy_* is that rule alone, driven by the caller's clock: host only,
 * no GPU, not thread safe.  Times are integer nanoseconds on any one clock.   */
typedef struct prep_policy prep_policy;

int prep_policy_create(prep_policy **out, int32_t batch_max, int64_t time_queue_ns);
void prep_policy_destroy(prep_policy *p);
/* Request `id` arrives at t_ns (no earlier than the arrival before it). */
int prep_policy_arrive(prep_policy *p, uint64_t id, int64_t t_ns);
/* Earliest time at which a batch is released given no further arrival:
 * INT64_MAX when nothing waits.                                               */
int64_t prep_policy_deadline(const prep_policy *p);
/* A consumer is free at now_ns: if a batch is released by then, writes its
 * ids (HOST, cap >= batch_max entries), oldest first, removes them from the
 * queue and returns their number; else returns 0.  Negative on bad arguments. */
int32_t prep_policy_take(prep_policy *p, int64_t now_ns, uint64_t *ids, int32_t cap);
int32_t prep_policy_pending(const prep_policy *p);

/* prep_server_*: that rule in front of n_consumers handles, each with its own
 * HIP stream and host thread (the paper's vGPUs consuming batches).  Requests
 * are copied on submission; every request's tensor slab [3, crop_h, crop_w]
 * lands in device memory owned by the server.  All calls are thread safe.     */
typedef struct prep_server prep_server;

typedef struct {
    prep_config handle;        /* capacity of each consumer's handle; max_batch is taken from batch_max */
    prep_params params;
    int32_t n_consumers;       /* 1..64                                          */
    int32_t batch_max;         /* 1..65535                                       */
    int64_t time_queue_us;     /* >= 0                                           */
    int32_t max_request_bytes; /* largest file accepted                          */
    int32_t queue_capacity;    /* requests that may wait; more are refused       */
} prep_server_config;

typedef struct {
    uint64_t tag;              /* the caller's tag                               */
    int32_t status;            /* PREP_OK or the image's error                   */
    int32_t batch_size;        /* size of the batch it was served in             */
    int32_t consumer;          /* which consumer served it                       */
    int32_t slot;              /* which of the consumer's output buffers holds it */
    int64_t arrival_ns, start_ns, done_ns; /* steady clock: submitted, batch taken, tensor ready */
    const void *tensor;        /* DEVICE: this request's slab, valid until
                                * prep_server_release                             */
} prep_server_result;

int prep_server_create(prep_server **out, const prep_server_config *cfg);
/* Stops the consumers (requests still waiting are dropped) and frees everything. */
int prep_server_destroy(prep_server *s);
/* Queues one JPEG file (HOST, copied before the call returns).
 * PREP_E_TOO_LARGE: the file is larger than max_request_bytes or the queue is full. */
int prep_server_submit(prep_server *s, const uint8_t *jpeg, uint64_t len, uint64_t tag);
/* Next finished request, in order of completion: 1 and *out filled, 0 after
 * timeout_us without one, negative on bad arguments.  Every result must be
 * given back with prep_server_release: a consumer has three output buffers
 * and reuses one only when all results of the batch it held are released.     */
int prep_server_next(prep_server *s, prep_server_result *out, int64_t timeout_us);
/* The caller is done with the result's tensor.                                */
int prep_server_release(prep_server *s, const prep_server_result *r);
/* The same for several results at once: up to cap finished requests into out
 * (HOST), waiting at most timeout_us for the first; returns their number.     */
int32_t prep_server_next_many(prep_server *s, prep_server_result *out, int32_t cap, int64_t timeout_us);
int prep_server_release_many(prep_server *s, const prep_server_result *r, int32_t n);
/* Copies a finished request's tensor slab (3*crop_h*crop_w elements of the
 * configured dtype) to host_out (HOST); for checks, while the slab is valid.  */
int prep_server_copy_tensor(prep_server *s, const prep_server_result *r, void *host_out);

/* ---- audio path (PREBA section 2.3 item b; section 4.2, Fig. 11(b), Table 1) ----
 *
 * Resample -> log-Mel spectrogram -> per-feature normalize, the three units of
 * the paper's audio compute units.  Definitions: band-limited interpolation
 * with a Hann-windowed sinc (six zero crossings, cut-off at 0.99 of the lower
 * Nyquist rate); frames of n_fft samples every hop samples, frame t centred on
 * sample t*hop of the signal extended by reflection; periodic Hann window of
 * win_length samples centred in the frame; squared magnitude of the DFT;
 * n_mels unit-peak triangles with corners equally spaced on
 * m(f) = 2595 log10(1 + f/700) between 0 and rate/2; ln(x + 2^-24); per Mel
 * channel of an utterance mean, variance (mean squared deviation) and
 * (x - mean) / (sqrt(variance) + 1e-5).                                        */
typedef struct prep_audio prep_audio;

typedef struct {
    int32_t device;
    int32_t max_batch;          /* utterances per call                             */
    int32_t rate;               /* sampling rate the features are computed at      */
    int32_t n_fft;              /* 512                                             */
    int32_t win_length;         /* 1 .. n_fft                                      */
    int32_t hop;                /* >= 1                                            */
    int32_t n_mels;             /* 1 .. 128                                        */
    int32_t reserved;
    uint64_t max_total_samples; /* samples per call, before and after resampling   */
} prep_audio_config;

int prep_audio_create(prep_audio **out, const prep_audio_config *cfg);
int prep_audio_destroy(prep_audio *h);
/* Frames of an utterance of samples_in samples at rate_in: 1 + ceil(samples_in *
 * rate / rate_in) / hop (integer division), or a negative code.                 */
int64_t prep_audio_frames(const prep_audio_config *cfg, uint64_t samples_in, int32_t rate_in);
/* waveforms: DEVICE, float32 mono, n utterances back to back; offsets: HOST,
 * n+1 entries in samples; rate_in: their sampling rate.  out: DEVICE float32;
 * utterance i lands at out_offsets[i] (HOST, n+1 entries, written by the call,
 * in elements) as [n_mels][frames_i], frames innermost.  Every utterance must
 * be longer than n_fft/2 samples after resampling.  Enqueues on `stream` (a
 * hipStream_t, NULL = the default stream) and
 * returns; allocates nothing (the interpolation taps of a new rate pair are built on
 * the host and uploaded on `stream`; the last two pairs are kept).              */
int prep_audio_features(prep_audio *h, const float *waveforms, const uint64_t *offsets, int32_t n,
                        int32_t rate_in, float *out, uint64_t *out_offsets, void *stream);

#ifdef __cplusplus
}
#endif
#endif
