"""Host logic and kernel indexing, checked without a GPU: the library's sources are compiled
by g++ against a CPU stand-in for HIP (one OS thread per lane, AddressSanitizer and UBSan
on) and run end to end through the C ABI.  The product never uses this build; the GPU
parity tests are the ones marked `gpu`."""
import os

import numpy as np
import pytest

import emul
import helpers
import oracle
import synth
from oracle import MODE_420, MODE_422, MODE_440, MODE_444, MODE_GRAY

MEAN, STD = synth.IMAGENET_MEAN, synth.IMAGENET_STD


def _img(seed, w, h, sigma=12.0):
    return synth.gradient_noise_image(np.random.default_rng(seed), w, h, sigma)


def _check(streams, rs, ch, cw, dt, expect_status=None, flags=0, antialias=False, smooth_chroma=False):
    per, ten = emul.run(streams, rs, ch, cw, dt, MEAN, STD, flags=flags, antialias=antialias)
    footprint = helpers.window_footprint if antialias else helpers.tap_footprint
    for i, s in enumerate(streams):
        status, coef, rgb, rect = per[i]
        if expect_status and expect_status[i] != 0:
            assert status == expect_status[i]
            assert (ten[i] == 0).all()
            continue
        assert status == 0, f"image {i}: status {status}"
        c0, r0, info = oracle.decode(s, smooth_chroma=smooth_chroma)
        assert np.array_equal(coef, c0), f"image {i}: coefficients differ"
        if flags & 2:
            assert rect == (0, 0, info.width, info.height)
        d = helpers.rgb_in_region(rect, rgb.reshape(r0.shape), r0,
                                  footprint(info.width, info.height, rs, ch, cw))
        assert d.max() <= 1 and (d == 0).mean() >= 0.999, f"image {i}: rgb"
        ref = oracle.preprocess(r0, rs, ch, cw, MEAN, STD, antialias)
        assert np.abs(ten[i].astype(np.float64) - ref).max() <= 0.02, f"image {i}: tensor"


# Small inputs are cut into small windows and decoded by the hypothesis passes; flag 8
# (PREP_FLAG_LARGE_WINDOWS) sends them down the paths that large batches take: one lane per
# short restart interval, iterated subsequences for long ones.
BOTH_DECODERS = pytest.mark.parametrize("windows", [0, 8], ids=["small-windows", "large-windows"])


@BOTH_DECODERS
def test_modes_restart_intervals_and_odd_sizes(windows):
    streams = []
    for k, (w, h) in enumerate([(1, 1), (17, 33), (70, 45)]):
        for mode in (MODE_444, MODE_420, MODE_GRAY, MODE_422, MODE_440):
            cols = -(-w // (8 * oracle.MODE_GEOMETRY[mode][0]))
            # (streams without markers take the same way whatever the windows)
            for dri in ((0, 1, cols) if windows else (1, cols)):
                streams.append(oracle.encode(_img(10 + k, w, h), 88, mode, dri, table_mode=k % 2)[0])
    _check(streams, 0, 1, 1, "f32", flags=2 | windows)  # whole images are converted to RGB and compared


def test_tables_whose_codes_are_mostly_sixteen_bits_long():
    # nearly every AC symbol takes the decoder's second-level lookup, and the table's
    # second-level blocks do not all fit their pool, so some take the canonical search
    streams = [oracle.encode(_img(40 + k, 70, 45), 88, mode, dri, table_mode=2)[0]
               for k, (mode, dri) in enumerate([(MODE_420, 0), (MODE_420, 2), (MODE_444, 0), (MODE_GRAY, 3)])]
    _check(streams, 0, 1, 1, "f32", flags=2)


def test_antialiased_resize_reducing_enlarging_and_at_the_edges():
    # reduce by 2.5 and by a non-integer factor, enlarge, keep the size; crop windows that
    # touch the image's edge and ones well inside it (region of interest of the reconstruction)
    streams = [oracle.encode(_img(50, 160, 100), 90, MODE_420, 4)[0],
               oracle.encode(_img(51, 75, 131), 90, MODE_444, 0)[0],
               oracle.encode(_img(52, 97, 64), 90, MODE_GRAY, 0)[0]]
    # (large windows: the decoder's ways are other tests' business, and fewer workgroups run)
    _check(streams, 40, 40, 40, "f32", antialias=True, flags=8)
    _check(streams, 40, 24, 30, "f16", antialias=True, flags=8)
    _check(streams[:2], 150, 120, 150, "f32", antialias=True, flags=8)
    _check(streams[2:], 0, 64, 97, "f32", antialias=True, flags=8)


def test_interpolated_chroma_in_the_crop_region_and_over_whole_images():
    streams = []
    for k, (w, h) in enumerate([(1, 1), (17, 33), (97, 70)]):
        for mode in (MODE_420, MODE_422, MODE_440, MODE_444):
            streams.append(oracle.encode(_img(70 + k, w, h), 90, mode, dri=(0, 2)[k % 2])[0])
    _check(streams, 0, 1, 1, "f32", flags=4 | 2 | 8, smooth_chroma=True)
    _check(streams[8:], 50, 36, 40, "f32", flags=4 | 8, smooth_chroma=True)
    _check(streams[8:11], 0, 70, 97, "f16", flags=4, smooth_chroma=True)


def test_eight_bit_interleaved_output_of_both_filters():
    streams = [oracle.encode(_img(60, 160, 100), 90, MODE_420, 4)[0],
               oracle.encode(_img(61, 75, 131), 90, MODE_444, 0)[0],
               b"not a jpeg"]
    for rs, ch, cw, aa in ((40, 40, 40, False), (40, 33, 38, True), (0, 64, 75, False), (150, 120, 150, True)):
        per, got = emul.run(streams, rs, ch, cw, "u8", MEAN, STD, antialias=aa, flags=8)
        assert [p[0] for p in per][:2] == [0, 0] and per[2][0] != 0
        assert (got[2] == 0).all()    # a failed image's slab is zero-filled
        exact = total = 0
        for i in range(2):
            _, rgb, _ = oracle.decode(streams[i], want_coef=False)
            ref = oracle.resize_crop_u8(rgb, rs, ch, cw, aa).astype(int)
            d = np.abs(got[i].astype(int) - ref)
            # the decoded pixels may be a level off and the rounding may fall the other way
            assert d.max() <= 2, (rs, ch, cw, aa, i, d.max())
            exact += int((d == 0).sum())
            total += d.size
        assert exact >= 0.97 * total, (rs, ch, cw, aa, exact / total)


def test_pillow_streams_of_workloads_1_and_5():
    streams = [synth.make_image(1, 5)[0], synth.make_image(5, 0)[0], synth.make_image(5, 1)[0],
               synth.make_image(5, 2)[0]]
    _check(streams, 256, 224, 224, "f16")


@BOTH_DECODERS
def test_long_intervals_and_many_chunks(windows):
    rgb = _img(20, 480, 320, sigma=25.0)
    streams = [oracle.encode(rgb, 95, MODE_444, 0)[0],        # ~150 KB without markers
               oracle.encode(rgb, 95, MODE_420, 30)[0],       # one interval per MCU row, > 1 KB each
               oracle.encode(rgb, 95, MODE_420, 3)[0],        # short intervals over many windows
               oracle.encode(rgb[:160, :240], 95, MODE_420, 0)[0]]   # no markers, six blocks per MCU, two chunks
    assert len(streams[0]) > 100000 and len(streams[3]) > 20000
    if windows:
        _check(streams, 128, 112, 120, "f32", flags=windows)
    else:
        # small windows make many workgroups, each 256 host threads here: a part of the image
        # does (the window size changes nothing for streams without markers)
        part = rgb[:128, :208]
        _check([oracle.encode(part, 95, MODE_420, 13)[0], oracle.encode(part, 95, MODE_420, 3)[0]],
               64, 56, 60, "f32")


@BOTH_DECODERS
def test_files_that_go_on_after_their_image(windows):
    # a second image (with restart markers of its own) or noise ending in another EOI marker
    # behind a sound file: the entropy-coded data end at the first EOI marker
    rng = np.random.default_rng(77)
    tail_image = oracle.encode(_img(78, 96, 80), 85, MODE_420, 2)[0]
    noise = bytes(rng.integers(0, 256, 300, dtype=np.uint8)).replace(b"\xff\xd9", b"\xff\x00") + b"\xff\xd9"
    streams = []
    for k, (w, h, mode, dri) in enumerate([(120, 90, MODE_420, 4), (77, 65, MODE_444, 0), (136, 96, MODE_420, 9)]):
        sound = oracle.encode(_img(80 + k, w, h, sigma=20.0), 92, mode, dri)[0]
        streams += [sound + tail_image, sound + noise]
    _check(streams, 0, 40, 48, "f32", flags=windows)


def test_broken_streams_are_reported_and_zero_filled():
    good = [oracle.encode(_img(30 + k, 64, 48), 85, MODE_420, 2)[0] for k in range(3)]
    sos = good[0].index(b"\xff\xda")
    i = good[0].index(b"\xff\xd1", sos)
    streams = [good[0], good[1][:len(good[1]) // 2], good[2],
               good[0].replace(b"\xff\xc0", b"\xff\xc2", 1),
               good[0][:i - 1] + good[0][i + 2:],
               good[0][:sos + 30] + bytes(60) + good[0][sos + 90:]]
    _check(streams, 32, 24, 24, "f32", expect_status=[0, -5, 0, -4, -5, -5])


@BOTH_DECODERS
def test_damaged_entropy_data_stays_in_bounds(windows):
    """Random damage to the entropy-coded bytes: the sanitizers see no access out of bounds,
    every kernel loop ends, and each stream is refused or decoded as the oracle decodes it.
    PREP_DAMAGE_FULL=1 runs the larger set that the GPU test of the same name uses."""
    if os.environ.get("PREP_DAMAGE_FULL"):
        streams = helpers.damaged_streams(11, 12) + helpers.damaged_streams(12, 12)
    else:
        streams = helpers.damaged_streams(7, 4, n_bases=4)
    per, ten = emul.run(streams, 32, 24, 24, "f32", MEAN, STD, timeout=3000, flags=windows)
    refused = helpers.check_damaged(streams, [p[0] for p in per], lambda i, nb: per[i][1], ten)
    assert refused >= len(streams) // 2
