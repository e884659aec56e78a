"""Shared helpers of the parity tests: run a batch through the GPU library's C ABI and
compare every checkpoint with the CPU oracle."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np

import oracle
import synth

MEAN, STD = synth.IMAGENET_MEAN, synth.IMAGENET_STD

# tolerances of the three checkpoints
RGB_MAX_LSB = 1          # decoded RGB: every pixel within 1 LSB ...
RGB_EXACT_FRACTION = 0.999   # ... and at least 99.9 % of all values exact
TENSOR_ABS_TOL = 0.02    # normalized tensor, absolute


def tap_footprint(width, height, resize_short, crop_h, crop_w):
    """(x_lo, y_lo, x_hi, y_hi), inclusive: the source pixels that count in the crop window's
    outputs, from the mapping in exact rational arithmetic (pixel centres at half-integers,
    per-axis scale in/out, taps floor(s) and floor(s) + 1 clamped to the image; the second tap
    has weight zero where s is an integer)."""
    from fractions import Fraction
    ow, oh = oracle.resized_size(width, height, resize_short)
    top, left = (oh - crop_h) // 2, (ow - crop_w) // 2

    def span(size, out_size, first, count):
        s_first = Fraction(2 * first + 1, 2) * Fraction(size, out_size) - Fraction(1, 2)
        s_last = Fraction(2 * (first + count - 1) + 1, 2) * Fraction(size, out_size) - Fraction(1, 2)
        lo = s_first.numerator // s_first.denominator
        hi = s_last.numerator // s_last.denominator + (0 if s_last.denominator == 1 else 1)
        return min(max(lo, 0), size - 1), min(max(hi, 0), size - 1)

    x_lo, x_hi = span(width, ow, left, crop_w)
    y_lo, y_hi = span(height, oh, top, crop_h)
    return x_lo, y_lo, x_hi, y_hi


def window_footprint(width, height, resize_short, crop_h, crop_w):
    """The same for the antialiased filter: the source pixels strictly inside the triangles of
    the crop window's outputs (centre (i + 1/2) * in/out, half-width max(in/out, 1)), in exact
    rational arithmetic."""
    from fractions import Fraction
    import math
    ow, oh = oracle.resized_size(width, height, resize_short)
    top, left = (oh - crop_h) // 2, (ow - crop_w) // 2

    def span(size, out_size, first, count):
        scale = Fraction(size, out_size)
        support = max(scale, Fraction(1))
        c_first = Fraction(2 * first + 1, 2) * scale
        c_last = Fraction(2 * (first + count - 1) + 1, 2) * scale
        lo = math.floor(c_first - support - Fraction(1, 2)) + 1   # j + 1/2 > centre - support
        hi = math.ceil(c_last + support - Fraction(1, 2)) - 1     # j + 1/2 < centre + support
        return min(max(lo, 0), size - 1), min(max(hi, 0), size - 1)

    x_lo, x_hi = span(width, ow, left, crop_w)
    y_lo, y_hi = span(height, oh, top, crop_h)
    return x_lo, y_lo, x_hi, y_hi


def rgb_in_region(rect, got_rgb, ref_rgb, footprint):
    """|got - ref| over the pixels that the library converted (rect = x0, y0, x1, y1), after
    checking that they cover the crop window's taps."""
    x0, y0, x1, y1 = rect
    x_lo, y_lo, x_hi, y_hi = footprint
    assert x0 <= x_lo and x_hi < x1 and y0 <= y_lo and y_hi < y1, (rect, footprint)
    return np.abs(got_rgb[y0:y1, x0:x1].astype(np.int32) - ref_rgb[y0:y1, x0:x1].astype(np.int32))


def oracle_batch(streams, resize_short, crop_h, crop_w, workers=8, antialias=False, smooth_chroma=False):
    """[(coef, rgb, info, tensor float64)] for every stream, computed by the oracle."""
    def one(s):
        coef, rgb, info = oracle.decode(s, smooth_chroma=smooth_chroma)
        ten = oracle.preprocess(rgb, resize_short, crop_h, crop_w, MEAN, STD, antialias)
        return coef, rgb, info, ten
    with ThreadPoolExecutor(workers) as ex:
        return list(ex.map(one, streams))


def run_gpu(pp, streams, resize_short, crop_h, crop_w, out_dtype, resident=False, antialias=False):
    import torch
    from paper_2411_19114_amd.binding import FILTER_ANTIALIAS, FILTER_BILINEAR, make_params
    blob, offsets = synth.pack(streams)
    params = make_params(resize_short, crop_h, crop_w, out_dtype, MEAN, STD,
                         FILTER_ANTIALIAS if antialias else FILTER_BILINEAR)
    dt = torch.float16 if out_dtype == "f16" else torch.float32
    # poison the output so that unwritten elements show
    out = torch.full((len(streams), 3, crop_h, crop_w), 777.0, dtype=dt, device="cuda:0")
    stream = torch.cuda.current_stream()
    if resident:
        dev_bits = torch.from_numpy(blob).to("cuda:0")
        torch.cuda.synchronize()
        pp.decode_resize_batch_resident(blob, dev_bits.data_ptr(), offsets, params, out.data_ptr(),
                                        stream.cuda_stream)
    else:
        pp.decode_resize_batch(blob, offsets, params, out.data_ptr(), stream.cuda_stream)
    status = pp.get_status(len(streams))
    return status, out.float().cpu().numpy().astype(np.float64)


def check_against_oracle(pp, streams, resize_short, crop_h, crop_w, out_dtype, resident=False,
                         check_intermediates=True, antialias=False, smooth_chroma=False):
    """smooth_chroma: pp was created with FLAG_SMOOTH_CHROMA, and the oracle interpolates too."""
    status, got = run_gpu(pp, streams, resize_short, crop_h, crop_w, out_dtype, resident, antialias)
    assert status == [0] * len(streams), status
    ref = oracle_batch(streams, resize_short, crop_h, crop_w, antialias=antialias, smooth_chroma=smooth_chroma)
    footprint = window_footprint if antialias else tap_footprint
    n_values = n_exact = 0
    for i, (coef, rgb, info, ten) in enumerate(ref):
        if check_intermediates:
            mine = pp.debug_last_coefficients(i, coef.shape[0])
            assert np.array_equal(mine, coef), f"image {i}: entropy-decoded coefficients differ"
            d = rgb_in_region(pp.debug_last_region(i), pp.debug_last_rgb(i, info.height, info.width), rgb,
                              footprint(info.width, info.height, resize_short, crop_h, crop_w))
            assert d.max() <= RGB_MAX_LSB, f"image {i}: RGB off by {d.max()} LSB"
            n_values += d.size
            n_exact += int((d == 0).sum())
        err = np.abs(got[i] - ten).max()
        assert err <= TENSOR_ABS_TOL, f"image {i}: tensor off by {err}"
    if check_intermediates:
        assert n_exact >= RGB_EXACT_FRACTION * n_values, f"only {n_exact / n_values:.5f} of RGB exact"
    return got


# ---- damaged streams ------------------------------------------------------------------
DAMAGE_BASES = [(96, 64, oracle.MODE_420, 2, 85), (96, 64, oracle.MODE_420, 0, 90),
                (80, 72, oracle.MODE_444, 0, 92), (120, 90, oracle.MODE_GRAY, 0, 80),
                (200, 160, oracle.MODE_420, 13, 95), (64, 48, oracle.MODE_444, 1, 60),
                (320, 240, oracle.MODE_420, 0, 96)]


def damaged_streams(seed, per_base, n_bases=len(DAMAGE_BASES)):
    """Sound oracle-encoded files whose entropy-coded segment is then damaged at random: bit
    flips, inserted marker bytes, deleted runs, garbage runs, truncation, runs of FF, restart
    markers with a wrong number or two of them swapped.
    Headers stay intact, so every file reaches the decoder kernels."""
    rng = np.random.default_rng(seed)
    out = []
    for k, (w, h, mode, dri, q) in enumerate(DAMAGE_BASES[:n_bases]):
        rgb = synth.gradient_noise_image(np.random.default_rng(50 + k), w, h, 14.0)
        b = oracle.encode(rgb, q, mode, dri, table_mode=k % 2)[0]
        sos = b.index(b"\xff\xda")
        start, end = sos + 2 + int.from_bytes(b[sos + 2:sos + 4], "big"), len(b) - 2
        for _ in range(per_base):
            a = bytearray(b)
            kind = int(rng.integers(0, 7))
            pos = int(rng.integers(start, end))
            marks = [m for m in range(start, end - 1) if b[m] == 0xFF and 0xD0 <= b[m + 1] <= 0xD7]
            if kind == 6 and not marks:
                kind = 0
            if kind == 0:
                for _ in range(int(rng.integers(1, 4))):
                    a[int(rng.integers(start, end))] ^= 1 << int(rng.integers(0, 8))
            elif kind == 1:
                a[pos:pos] = bytes([0xFF, int(rng.choice([0xD0, 0xD3, 0xD7, 0x00, 0xFF, 0xD9, 0xC4]))])
            elif kind == 2:
                del a[pos:pos + int(rng.integers(1, 40))]
            elif kind == 3:
                n = int(rng.integers(1, 64))
                a[pos:pos + n] = rng.integers(0, 256, n, dtype=np.uint8).tobytes()
            elif kind == 4:
                a = a[:pos] + b"\xff\xd9"
            elif kind == 5:
                n = int(rng.integers(1, 30))
                a[pos:pos + n] = b"\xff" * n
            elif len(marks) >= 2 and rng.random() < 0.5:
                m1, m2 = (int(x) for x in rng.choice(len(marks), 2, replace=False))
                a[marks[m1] + 1], a[marks[m2] + 1] = a[marks[m2] + 1], a[marks[m1] + 1]
            else:
                m = marks[int(rng.integers(0, len(marks)))]
                a[m + 1] = 0xD0 + (a[m + 1] - 0xD0 + int(rng.integers(1, 8))) % 8
            out.append(bytes(a))
    return out


def check_damaged(streams, status, coefficients_of, tensor):
    """A damaged stream is either refused (zero slab) or decoded to the oracle's coefficients;
    the kernels never accept what the oracle refuses."""
    refused = 0
    for i, s in enumerate(streams):
        try:
            c0 = oracle.decode(s, want_rgb=False)[0]
        except oracle.OracleError:
            c0 = None
        if status[i] == 0:
            assert c0 is not None, f"stream {i}: accepted, but the oracle refuses it"
            assert np.array_equal(coefficients_of(i, c0.shape[0]), c0), f"stream {i}: coefficients differ"
        else:
            refused += 1
            assert (tensor[i] == 0).all(), f"stream {i}: refused but its slab is not zero"
    return refused
