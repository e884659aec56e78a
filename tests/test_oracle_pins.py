"""Pins of the CPU oracle against facts that do not come from the oracle itself:
the JPEG standard's printed tables, closed forms, textbook routines (scipy), brute
force, an independent codec (Pillow) and the encode -> decode round trip."""
import io
import itertools

import numpy as np
import pytest

import oracle
from oracle import MODE_420, MODE_422, MODE_440, MODE_444, MODE_GRAY

MEAN = (0.485, 0.456, 0.406)
STD = (0.229, 0.224, 0.225)


def _golden_rows(path):
    out = {}
    rows = []
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        parts = line.split()
        if parts[0][0].isalpha():
            out[parts[0]] = [int(p) for p in parts[1:]]
        else:
            rows.append([int(p) for p in parts])
    return out, rows


def _noise_image(seed, w, h, sigma=20.0):
    rng = np.random.default_rng(seed)
    x = np.arange(w)[None, :, None] / max(w, 1)
    y = np.arange(h)[:, None, None] / max(h, 1)
    base = rng.uniform(60, 190, size=(1, 1, 3)) + 50 * x - 40 * y
    return np.clip(np.rint(base + rng.normal(0, sigma, size=(h, w, 3))), 0, 255).astype(np.uint8)


# ---------------------------------------------------------------- zig-zag

def test_zigzag_matches_figure_a6(golden_dir):
    _, rows = _golden_rows(golden_dir + "/zigzag_order.txt")
    fig = np.array(rows)
    assert fig.shape == (8, 8)
    for k in range(64):
        v, u = oracle.zigzag_pos(k)
        assert fig[v, u] == k


def test_zigzag_structure():
    pos = [oracle.zigzag_pos(k) for k in range(64)]
    assert sorted(pos) == sorted(itertools.product(range(8), range(8)))
    assert pos[0] == (0, 0) and pos[1] == (0, 1) and pos[2] == (1, 0) and pos[63] == (7, 7)
    diag = [v + u for v, u in pos]
    assert diag == sorted(diag)


# ---------------------------------------------------------------- DCT

def test_idct_equals_scipy_orthonormal_idct():
    from scipy.fft import idctn
    rng = np.random.default_rng(1)
    for _ in range(20):
        F = rng.normal(0, 200, size=(8, 8))
        np.testing.assert_allclose(oracle.idct8x8(F), idctn(F, norm="ortho"), atol=1e-9)


def test_fdct_equals_scipy_and_inverts():
    from scipy.fft import dctn
    rng = np.random.default_rng(2)
    f = rng.uniform(-128, 127, size=(8, 8))
    np.testing.assert_allclose(oracle.fdct8x8(f), dctn(f, norm="ortho"), atol=1e-9)
    np.testing.assert_allclose(oracle.idct8x8(oracle.fdct8x8(f)), f, atol=1e-9)


def test_idct_dc_only_is_constant_dc_over_8():
    for dc in (-1024, -17, 0, 4, 12, 1016):
        F = np.zeros((8, 8))
        F[0, 0] = dc
        np.testing.assert_allclose(oracle.idct8x8(F), np.full((8, 8), dc / 8.0), atol=1e-10)


def test_idct_single_coefficient_is_separable_cosine():
    for v, u in ((0, 1), (3, 0), (2, 5), (7, 7)):
        F = np.zeros((8, 8))
        F[v, u] = 100.0
        cu = np.sqrt(0.5) if u == 0 else 1.0
        cv = np.sqrt(0.5) if v == 0 else 1.0
        x = np.arange(8)
        expect = 0.25 * cu * cv * 100.0 * np.outer(np.cos((2 * x + 1) * v * np.pi / 16),
                                                   np.cos((2 * x + 1) * u * np.pi / 16))
        np.testing.assert_allclose(oracle.idct8x8(F), expect, atol=1e-10)


def test_idct_parseval():
    rng = np.random.default_rng(3)
    F = rng.normal(0, 100, size=(8, 8))
    assert abs((oracle.idct8x8(F) ** 2).sum() - (F ** 2).sum()) < 1e-6


def test_idct_is_not_transposed():
    # a horizontal-frequency coefficient F[v=0,u=1] must vary along x (columns) only
    F = np.zeros((8, 8))
    F[0, 1] = 64.0
    f = oracle.idct8x8(F)
    assert np.allclose(f, f[0:1, :]) and not np.allclose(f[:, 0], f[:, 7].mean())
    assert f[0, 0] > 0 > f[0, 7]


# ---------------------------------------------------------------- quantisation tables

def test_quant_tables_match_annex_k(golden_dir):
    g, _ = _golden_rows(golden_dir + "/quant_tables.txt")
    q50 = oracle.quant_table(50, 0)
    assert list(q50[:8]) == g["k1_first_row"]
    assert int(q50.sum()) == g["k1_sum"][0]
    assert list(oracle.quant_table(85, 0)[:8]) == g["q85_first_row"]
    assert list(oracle.quant_table(50, 1)[:8]) == g["k2_first_row"]
    assert oracle.quant_table(100, 0).max() == 1 and oracle.quant_table(1, 1).max() == 255


# ---------------------------------------------------------------- Huffman tables

def _check_prefix_free(code, size):
    words = [format(int(c), "0%db" % int(s)) for c, s in zip(code, size)]
    assert len(set(words)) == len(words)
    for a in words:
        for b in words:
            if a is not b:
                assert not b.startswith(a) or a == b
    return words


def test_canonical_codes_kraft_and_prefix_free():
    bits = np.zeros(17, dtype=np.uint8)
    bits[2], bits[3], bits[4], bits[5] = 1, 3, 2, 3
    code, size = oracle.huff_codes(bits)
    words = _check_prefix_free(code, size)
    assert words[:4] == ["00", "010", "011", "100"]  # consecutive within a length, <<1 between
    assert sum(2.0 ** -int(s) for s in size) < 1.0
    bad = np.zeros(17, dtype=np.uint8)
    bad[1] = 3  # three 1-bit codes do not exist
    with pytest.raises(oracle.OracleError):
        oracle.huff_codes(bad)


def _optimal_cost(freq):
    import heapq
    h = [int(f) for f in freq if f > 0] + [1]  # + reserved code point
    heapq.heapify(h)
    cost = 0
    while len(h) > 1:
        a, b = heapq.heappop(h), heapq.heappop(h)
        cost += a + b
        heapq.heappush(h, a + b)
    return cost


def test_lengths_from_counts_are_optimal_limited_and_reserve_all_ones():
    rng = np.random.default_rng(4)
    for trial in range(6):
        freq = np.zeros(256, dtype=np.int64)
        n = [3, 12, 40, 162, 200, 256][trial]
        idx = rng.choice(256, size=n, replace=False)
        freq[idx] = (rng.pareto(0.7 if trial % 2 else 2.0, size=n) * 50 + 1).astype(np.int64)
        bits, vals = oracle.huff_from_freq(freq)
        assert sorted(vals) == sorted(idx)
        assert bits[1:].sum() == n
        code, size = oracle.huff_codes(bits)
        _check_prefix_free(code, size)
        kraft = sum(2.0 ** -int(s) for s in size)
        assert kraft < 1.0  # strict: one code point of the longest length stays free
        longest = int(size.max())
        assert int(code[-1]) != (1 << longest) - 1  # no all-ones code word
        cost = sum(int(freq[v]) * int(s) for v, s in zip(vals, size))
        if longest < 16:
            # no length limiting happened: the code (with the reserved point, count 1, at the
            # longest length) has the optimal cost, which is unique even if the tree is not
            assert cost + longest == _optimal_cost(freq)
            # and rarer symbols never get shorter codes
            order = np.argsort([-int(freq[v]) for v in vals], kind="stable")
            s_sorted = [int(size[i]) for i in order]
            assert s_sorted == sorted(s_sorted)
        else:
            assert cost + longest >= _optimal_cost(freq)


def test_length_limit_16_is_enforced():
    freq = np.zeros(256, dtype=np.int64)
    for i in range(40):  # Fibonacci-like counts force a very deep tree
        freq[i] = int(1.6 ** i) + 1
    bits, vals = oracle.huff_from_freq(freq)
    assert len(vals) == 40 and bits[1:].sum() == 40
    code, size = oracle.huff_codes(bits)
    assert size.max() == 16
    assert sum(2.0 ** -int(s) for s in size) < 1.0


# ---------------------------------------------------------------- colour

def test_neutral_chroma_gives_gray():
    for y in range(256):
        assert oracle.ycc_to_rgb(y, 128, 128) == (y, y, y)


def test_colour_known_values_and_roundtrip():
    # primaries through the JFIF forward matrix, rounded
    assert oracle.rgb_to_ycc(255, 0, 0) == (76, 85, 255)
    assert oracle.rgb_to_ycc(0, 255, 0) == (150, 44, 21)
    assert oracle.rgb_to_ycc(0, 0, 255) == (29, 255, 107)
    # Cr only: R = Y + 1.402 (Cr-128), B unchanged, G = Y - 0.714136 (Cr-128)
    assert oracle.ycc_to_rgb(100, 128, 178) == (170, 64, 100)
    assert oracle.ycc_to_rgb(100, 178, 128) == (100, 83, 189)
    worst = 0
    for r, g, b in itertools.product(range(0, 256, 15), repeat=3):
        back = oracle.ycc_to_rgb(*oracle.rgb_to_ycc(r, g, b))
        worst = max(worst, max(abs(back[0] - r), abs(back[1] - g), abs(back[2] - b)))
    assert worst <= 2  # 0.5 LSB of each of Y, Cb, Cr amplified by at most 1.772, then rounded


# ---------------------------------------------------------------- entropy coding round trip

SIZES = [(1, 1), (7, 9), (17, 33), (64, 48), (300, 251)]


@pytest.mark.parametrize("mode", [MODE_444, MODE_420, MODE_GRAY, MODE_422, MODE_440])
@pytest.mark.parametrize("size", SIZES)
def test_roundtrip_recovers_quantised_coefficients(mode, size):
    w, h = size
    rgb = _noise_image(100 + w + h + mode, w, h)
    hmax = oracle.MODE_GEOMETRY[mode][0]
    mcu_cols = -(-w // (8 * hmax))
    for dri in (0, 1, mcu_cols, 8):
        for table_mode in (0, 1, 2):
            data, coef = oracle.encode(rgb, quality=90, mode=mode, dri=dri, table_mode=table_mode)
            got, _, info = oracle.decode(data, want_rgb=False)
            assert (info.width, info.height) == (w, h)
            assert info.restart_interval == dri
            assert got.shape == coef.shape
            assert np.array_equal(got, coef)
            nmcu = info.mcu_cols * info.mcu_rows
            n_rst = sum(data.count(bytes([0xFF, 0xD0 + i])) for i in range(8))
            if dri:
                assert n_rst >= (nmcu - 1) // dri  # markers present (data bytes may alias)


def test_roundtrip_extreme_coefficients_and_byte_stuffing():
    # hand-made coefficients: largest magnitudes, long zero runs (ZRL), full blocks,
    # and enough 1-bits that FF bytes (hence stuffed zeros) must occur
    rng = np.random.default_rng(7)
    w, h, mode = 48, 32, MODE_420
    nb = (48 // 16) * (32 // 16) * 6
    coef = np.zeros((nb, 64), dtype=np.int16)
    coef[:, 0] = rng.integers(-1000, 1000, size=nb)
    coef[0, 1:] = 1023
    coef[1, 1:] = -1023
    coef[2, 63] = -1          # 62 zeros then a value: three ZRLs
    coef[3, 17] = 5
    coef[3, 50] = -300
    coef[4, 1:] = rng.integers(-1023, 1024, size=63)
    coef[5:, 1:] = rng.integers(-3, 4, size=(nb - 5, 63))
    q = np.ones(64, dtype=np.uint16)
    for dri in (0, 1, 2):
        for table_mode in (0, 1, 2):
            data = oracle.write_jpeg(coef, w, h, mode, q, q, dri=dri, table_mode=table_mode)
            sos = data.index(b"\xff\xda")
            assert b"\xff\x00" in data[sos:], "no stuffed byte: test lost its point"
            got, _, _ = oracle.decode(data, want_rgb=False)
            assert np.array_equal(got, coef)


def test_all_eob_blocks_and_dc_only_blocks_decode_to_constant_blocks():
    w, h = 32, 24
    q = oracle.quant_table(75, 0)
    nb = 4 * 3
    coef = np.zeros((nb, 64), dtype=np.int16)
    coef[:, 0] = [0, 1, -1, 5, 100, -100, 3, 4, 12, -12, 37, -64]
    data = oracle.write_jpeg(coef, w, h, MODE_GRAY, q, q, dri=0, table_mode=0)
    got, rgb, info = oracle.decode(data)
    assert np.array_equal(got, coef)
    for b in range(nb):
        by, bx = divmod(b, 4)
        block = rgb[by * 8:by * 8 + 8, bx * 8:bx * 8 + 8, 0]
        dcq = int(coef[b, 0]) * int(q[0])
        expect = min(255, max(0, (dcq + 4) // 8 + 128))  # floor(DC*Q/8 + 0.5) + 128
        assert (block == expect).all()
    assert int(q[0]) == 8 and rgb[0, 8, 0] == 129 and rgb[0, 16, 0] == 127


def test_dc_only_ties_round_half_up_for_both_signs():
    # DC*Q = 4 (mod 8) puts the sample exactly half way between two integers:
    # floor(DC*Q/8 + 0.5) must go up for positive and for negative values alike
    q = np.full(64, 4, dtype=np.uint16)          # DC*Q = 4*DC: a tie for every odd DC
    dcs = [1, -1, 3, -3, 9, -9, 35, -35, 101, -101, 7, -7]
    coef = np.zeros((12, 64), dtype=np.int16)
    coef[:, 0] = dcs
    data = oracle.write_jpeg(coef, 32, 24, MODE_GRAY, q, q)
    _, rgb, _ = oracle.decode(data, want_coef=False)
    for b, dc in enumerate(dcs):
        by, bx = divmod(b, 4)
        expect = min(255, max(0, (4 * dc + 4) // 8 + 128))
        assert (rgb[by * 8:by * 8 + 8, bx * 8:bx * 8 + 8] == expect).all(), (dc, expect)
    F = np.zeros((8, 8))
    for dc in (-36.0, 36.0, -4.0, 1020.0):
        F[0, 0] = dc
        assert (oracle.idct8x8(F) == dc / 8.0).all()   # exactly, not approximately


def test_structured_ties_of_dc_plus_one_cosine_term_round_up():
    # only F(0,0) and F(v=0,u=4) non-zero: the definition gives (F00 +- F04)/8 exactly, with
    # the sign of cos((2x+1) pi/4); many of these samples sit exactly half way
    q = np.ones(64, dtype=np.uint16)
    k04 = [k for k in range(64) if oracle.zigzag_pos(k) == (0, 4)][0]
    cases = [(12, 8), (-12, 8), (100, -24), (4, 0), (-44, 16), (36, -8), (-4, 40), (20, 24)]
    coef = np.zeros((len(cases), 64), dtype=np.int16)
    for b, (f00, f04) in enumerate(cases):
        coef[b, 0], coef[b, k04] = f00, f04
    data = oracle.write_jpeg(coef, 8 * len(cases), 8, MODE_GRAY, q, q)
    _, rgb, _ = oracle.decode(data, want_coef=False)
    sign = np.array([1, -1, -1, 1, 1, -1, -1, 1])
    n_ties = 0
    for b, (f00, f04) in enumerate(cases):
        num = f00 + sign * f04                      # sample * 8, exact integers
        expect = np.clip((num + 4) // 8 + 128, 0, 255)   # floor(num/8 + 1/2) + 128
        n_ties += int((num % 8 == 4).sum())
        block = rgb[:, 8 * b:8 * b + 8, 0]
        assert (block == expect[None, :]).all(), (f00, f04)
    assert n_ties >= 16


# ---------------------------------------------------------------- independent codec (Pillow)

def _pil_decode(data):
    from PIL import Image
    return np.asarray(Image.open(io.BytesIO(data)).convert("RGB"))


@pytest.mark.parametrize("mode", [MODE_444, MODE_GRAY])
def test_pillow_decodes_oracle_files_to_nearly_the_same_pixels(mode):
    rgb = _noise_image(11, 83, 61)
    for dri, table_mode in ((0, 0), (3, 1), (0, 2)):
        data, _ = oracle.encode(rgb, quality=92, mode=mode, dri=dri, table_mode=table_mode)
        _, mine, _ = oracle.decode(data, want_coef=False)
        theirs = _pil_decode(data)
        diff = np.abs(mine.astype(int) - theirs.astype(int))
        # libjpeg's integer IDCT may be 1 LSB off per component; colour conversion amplifies
        # a chroma LSB by up to 1.772
        assert diff.max() <= (1 if mode == MODE_GRAY else 3) and diff.mean() < 0.3


def test_lopsided_ac_table_is_the_prefix_code_it_is_meant_to_be():
    # table_mode 2: one AC code of each length 2..15, sixteen bits for the other 148 symbols,
    # EOB among them; Pillow (libjpeg) reads the file to the same pixels as the file with
    # ordinary tables, so the table in the file and the codes in the scan agree
    rgb = _noise_image(12, 64, 48)
    plain, coef = oracle.encode(rgb, quality=90, mode=MODE_420, table_mode=1)
    data, coef2 = oracle.encode(rgb, quality=90, mode=MODE_420, table_mode=2)
    assert np.array_equal(coef, coef2) and len(data) > 2 * len(plain)
    at, seen = 0, 0
    while True:
        at = data.find(b"\xff\xc4", at)
        if at < 0 or at > data.index(b"\xff\xda"):
            break
        tc_th, bits = data[at + 4], list(data[at + 5:at + 21])
        if tc_th >> 4 == 1:
            vals = data[at + 21:at + 21 + sum(bits)]
            assert bits == [0] + [1] * 14 + [148] and len(set(vals)) == 162
            assert vals[-1] == 0x00 and vals[-2] == 0xF0 and vals[0] == 0xFA
            assert sum(b / (1 << (l + 1)) for l, b in enumerate(bits)) < 1.0   # Kraft
            seen += 1
        at += 2
    assert seen == 2
    assert np.array_equal(_pil_decode(data), _pil_decode(plain))


@pytest.mark.parametrize("mode", [MODE_422, MODE_440])
def test_pillow_decodes_oracle_422_and_440_files(mode):
    rgb = _noise_image(15, 90, 70, sigma=3.0)
    data, _ = oracle.encode(rgb, quality=92, mode=mode, dri=4)
    _, mine, info = oracle.decode(data, want_coef=False)
    assert (info.hs[0], info.vs[0], info.blocks_per_mcu) == oracle.MODE_GEOMETRY[mode]
    theirs = _pil_decode(data)  # libjpeg interpolates chroma where this decoder replicates it
    assert np.abs(mine.astype(int) - theirs.astype(int)).mean() < 1.5
    assert np.abs(mine.astype(int) - rgb.astype(int)).mean() < 6.0


@pytest.mark.parametrize("mode", [MODE_422, MODE_440])
def test_chroma_pairs_start_at_even_positions(mode):
    # Colour stripes two pixels wide across the halved axis lose nothing when they start at even
    # positions (each chroma sample covers one stripe) and are smeared when they start at odd
    # ones.  The axis itself is pinned by Pillow, which reads the sampling factors from the
    # frame header (the tests above and below).
    rng = np.random.default_rng(16)
    colours = rng.integers(40, 216, size=(24, 3)).astype(np.uint8)
    stripes = np.repeat(colours, 2, axis=0)                      # 48 lines, 2 alike in a row
    if mode == MODE_422:
        good = np.broadcast_to(stripes[None, :, :], (32, 48, 3)).copy()   # varies along x
        bad = np.roll(good, 1, axis=1)
    else:
        good = np.broadcast_to(stripes[:, None, :], (48, 32, 3)).copy()   # varies along y
        bad = np.roll(good, 1, axis=0)
    one = np.ones(64, dtype=np.uint16)  # no quantisation loss beyond rounding

    def error(rgb):
        coef, info = oracle.forward_blocks(rgb, mode, one, one)
        data = oracle.write_jpeg(coef, info.width, info.height, mode, one, one)
        return np.abs(oracle.decode(data, want_coef=False)[1].astype(int) - rgb.astype(int))

    assert error(good).max() <= 3
    assert error(bad).mean() > 5


def test_pillow_decodes_oracle_420_file():
    rgb = _noise_image(12, 80, 64, sigma=3.0)
    data, _ = oracle.encode(rgb, quality=92, mode=MODE_420, dri=5)
    _, mine, _ = oracle.decode(data, want_coef=False)
    theirs = _pil_decode(data)  # smooth chroma interpolation: close, not equal
    assert np.abs(mine.astype(int) - theirs.astype(int)).mean() < 1.5
    assert np.abs(mine.astype(int) - rgb.astype(int)).mean() < 6.0


# ---------------------------------------------------------------- centred-triangle upsampling

def test_triangle_upsampling_of_an_impulse_has_weights_9_3_3_1():
    plane = np.zeros((5, 6), dtype=np.uint8)
    plane[2, 3] = 160
    out = oracle.upsample_triangle(plane, 2, 2, 12, 10).astype(int)
    # sample (2, 3) lies between rows 4, 5 and columns 6, 7: nine sixteenths there, three
    # sixteenths one step away along an axis, one sixteenth at the diagonal
    expect = np.zeros((10, 12), dtype=int)
    expect[3:7, 5:9] = np.outer([1, 3, 3, 1], [1, 3, 3, 1]) * 10
    assert np.array_equal(out, expect)
    # one axis only: 3/4 and 1/4
    across = oracle.upsample_triangle(plane, 2, 1, 12, 5).astype(int)
    assert across[2, 5:9].tolist() == [40, 120, 120, 40] and across.sum() == 320
    down = oracle.upsample_triangle(plane, 1, 2, 6, 10).astype(int)
    assert down[3:7, 3].tolist() == [40, 120, 120, 40] and down.sum() == 320


def test_triangle_upsampling_reproduces_a_ramp_at_quarter_positions_and_clamps_at_the_edge():
    # samples 16, 24, 32, ... sit at pixel coordinates 0.5, 2.5, 4.5, ...: slope 4 per pixel
    ramp = (16 + 8 * np.arange(9)).astype(np.uint8)
    out = oracle.upsample_triangle(np.tile(ramp, (3, 1)), 2, 1, 18, 3).astype(int)
    x = np.arange(18)
    inside = 16 + 4 * (x - 0.5)
    assert np.array_equal(out[1, 1:17], inside[1:17].astype(int)) and (inside[1:17] % 1 == 0).all()
    assert out[1, 0] == 16 and out[1, 17] == 80      # beyond the first and last sample: the sample
    # an odd width owns ceil(w / 2) samples; the last column is a left-hand one
    odd = oracle.upsample_triangle(np.tile(ramp, (3, 1)), 2, 1, 17, 3).astype(int)
    assert np.array_equal(odd[1], out[1, :17])
    # the same down the rows
    rows = oracle.upsample_triangle(np.tile(ramp[:, None], (1, 4)), 1, 2, 4, 18).astype(int)
    assert np.array_equal(rows[:, 2], out[1])
    # constants stay
    assert (oracle.upsample_triangle(np.full((4, 4), 77, np.uint8), 2, 2, 7, 8) == 77).all()


def test_triangle_upsampling_rounds_halves_up():
    # one sample of 8 among zeros: 72, 24, 8 sixteenths -> 4.5 -> 5, 1.5 -> 2, 0.5 -> 1
    plane = np.zeros((3, 3), dtype=np.uint8)
    plane[1, 1] = 8
    out = oracle.upsample_triangle(plane, 2, 2, 6, 6).astype(int)
    assert out[1:5, 1:5].tolist() == [[1, 2, 2, 1], [2, 5, 5, 2], [2, 5, 5, 2], [1, 2, 2, 1]]
    # 7 sixteenths stay below: a sample of 7 gives 63/16 -> 4, 21/16 -> 1, 7/16 -> 0
    plane[1, 1] = 7
    out = oracle.upsample_triangle(plane, 2, 2, 6, 6).astype(int)
    assert out[1:5, 1:5].tolist() == [[0, 1, 1, 0], [1, 4, 4, 1], [1, 4, 4, 1], [0, 1, 1, 0]]


@pytest.mark.parametrize("mode", [MODE_420, MODE_422, MODE_440])
def test_smooth_chroma_decode_is_what_an_image_library_decodes(mode):
    # an image library interpolates subsampled chroma with the same triangle (its two rounding
    # offsets alternate, and its IDCT is an integer one): on smooth colour the interpolating
    # decoder is within a few levels of it everywhere and much closer than the replicating one
    yy, xx = np.mgrid[0:72, 0:88]
    rgb = np.stack([40 + 2 * xx, 200 - 2 * yy, 60 + xx + yy], axis=-1).astype(np.uint8)
    data, _ = oracle.encode(rgb, quality=95, mode=mode, dri=0)
    theirs = _pil_decode(data).astype(int)
    coef_s, smooth, _ = oracle.decode(data, smooth_chroma=True)
    coef_r, plain, _ = oracle.decode(data)
    assert np.array_equal(coef_s, coef_r)
    d_smooth, d_plain = np.abs(smooth.astype(int) - theirs), np.abs(plain.astype(int) - theirs)
    assert d_smooth.max() <= 3 and d_smooth.mean() < 0.5
    assert d_plain.mean() > 2 * d_smooth.mean()
    # full-resolution chroma and gray have nothing to interpolate
    for m in (MODE_444, MODE_GRAY):
        data, _ = oracle.encode(rgb, quality=90, mode=m, dri=3)
        assert np.array_equal(oracle.decode(data, smooth_chroma=True)[1], oracle.decode(data)[1])


@pytest.mark.parametrize("mode", [MODE_444, MODE_420, MODE_GRAY, MODE_422])
def test_oracle_decodes_pillow_files(mode):
    import synth
    rgb = _noise_image(13, 101, 77, sigma=6.0)
    for kw in (dict(), dict(restart_blocks=4), dict(restart_rows=1, optimize=True)):
        data = synth.encode_jpeg(rgb, 90, mode, **kw)
        _, mine, info = oracle.decode(data, want_coef=False)
        theirs = _pil_decode(data)
        diff = np.abs(mine.astype(int) - theirs.astype(int))
        if mode in (MODE_420, MODE_422):
            assert diff.mean() < 1.5
        else:
            assert diff.max() <= (1 if mode == MODE_GRAY else 3) and diff.mean() < 0.3
        assert (info.restart_interval > 0) == bool(kw.get("restart_blocks") or kw.get("restart_rows"))


def test_gray_file_equals_luma_plane_of_colour_file():
    rgb = _noise_image(14, 40, 40)
    _, coef_c = oracle.encode(rgb, quality=80, mode=MODE_444)
    _, coef_g = oracle.encode(rgb, quality=80, mode=MODE_GRAY)
    assert np.array_equal(coef_c[0::3], coef_g)


# ---------------------------------------------------------------- decoder error paths

def test_decoder_rejects_broken_streams():
    rgb = _noise_image(15, 33, 17)
    data, _ = oracle.encode(rgb, quality=85, mode=MODE_420, dri=2)
    sos = data.index(b"\xff\xda")
    for cut in list(range(0, sos + 14, 3)) + [len(data) // 2, len(data) - 6]:
        with pytest.raises(oracle.OracleError):
            oracle.decode(data[:cut])
    prog = data.replace(b"\xff\xc0", b"\xff\xc2", 1)
    with pytest.raises(oracle.OracleError) as e:
        oracle.decode(prog)
    assert e.value.code == oracle.E_UNSUPPORTED
    # a wrong restart index is corrupt
    i = data.index(b"\xff\xd0", sos)
    bad = data[:i + 1] + b"\xd3" + data[i + 2:]
    with pytest.raises(oracle.OracleError) as e:
        oracle.decode(bad)
    assert e.value.code == oracle.E_CORRUPT


# ---------------------------------------------------------------- resize / crop / normalize

def test_resized_size_rule():
    assert oracle.resized_size(640, 480, 256) == (341, 256)   # floor(256*640/480)
    assert oracle.resized_size(480, 640, 256) == (256, 341)
    assert oracle.resized_size(1920, 1080, 384) == (682, 384)
    assert oracle.resized_size(256, 256, 256) == (256, 256)
    assert oracle.resized_size(300, 200, 0) == (300, 200)


def test_constant_image_stays_constant_and_normalize_closed_form():
    for val, (w, h) in ((0, (50, 40)), (255, (300, 500)), (77, (123, 321))):
        rgb = np.full((h, w, 3), val, dtype=np.uint8)
        out = oracle.preprocess(rgb, 64, 48, 56, MEAN, STD)
        for c in range(3):
            np.testing.assert_allclose(out[c], (val / 255.0 - MEAN[c]) / STD[c], atol=1e-12)


def test_linear_ramp_is_reproduced_at_mapped_coordinates():
    w, h, s, ch, cw = 90, 60, 40, 32, 48
    x = np.arange(w)[None, :]
    y = np.arange(h)[:, None]
    ramp = [(1, 2, 3), (2, 0, 10), (0, 3, 20)]  # a x + b y + c stays inside 0..255
    rgb = np.stack([a * x + b * y + c0 for a, b, c0 in ramp], axis=-1).astype(np.uint8)
    ow, oh = oracle.resized_size(w, h, s)
    assert (ow, oh) == (60, 40)
    out = oracle.preprocess(rgb, s, ch, cw, MEAN, STD)
    top, left = (oh - ch) // 2, (ow - cw) // 2
    assert (top, left) == (4, 6)
    oy = np.arange(ch)[:, None]
    ox = np.arange(cw)[None, :]
    sx = (ox + left + 0.5) * (w / ow) - 0.5
    sy = (oy + top + 0.5) * (h / oh) - 0.5
    inside = (sx >= 0) & (sx <= w - 1) & (sy >= 0) & (sy <= h - 1)
    assert inside.mean() > 0.9
    for c, (a, b, c0) in enumerate(ramp):
        expect = ((a * sx + b * sy + c0) / 255.0 - MEAN[c]) / STD[c]
        np.testing.assert_allclose(out[c][inside], expect[inside], atol=1e-10)


def test_ramp_upscaling_clamps_at_the_border():
    rgb = np.zeros((2, 2, 3), dtype=np.uint8)
    rgb[:, 1] = 100
    out = oracle.preprocess(rgb, 8, 8, 8, (0, 0, 0), (1, 1, 1)) * 255.0
    row = out[0, 3]
    # source x of output x: (x+0.5)/4 - 0.5 -> clamped for x<2 and x>=6, linear between
    np.testing.assert_allclose(row, [0, 0, 12.5, 37.5, 62.5, 87.5, 100, 100], atol=1e-9)
    np.testing.assert_allclose(out[0], out[0][0:1].repeat(8, axis=0), atol=1e-9)


def test_identity_scale_returns_the_cropped_source_pixels():
    rgb = _noise_image(16, 256, 256)
    out = oracle.preprocess(rgb, 256, 224, 224, MEAN, STD)
    for c in range(3):
        expect = (rgb[16:240, 16:240, c] / 255.0 - MEAN[c]) / STD[c]
        np.testing.assert_allclose(out[c], expect, atol=1e-12)
    # no-resize mode with an odd margin: origin floor(margin/2)
    out2 = oracle.preprocess(rgb[:201, :101], 0, 100, 50, MEAN, STD)
    np.testing.assert_allclose(out2[1], (rgb[50:150, 25:75, 1] / 255.0 - MEAN[1]) / STD[1], atol=1e-12)


def test_downscale_by_two_averages_pixel_pairs():
    rng = np.random.default_rng(17)
    rgb = rng.integers(0, 256, size=(40, 40, 3), dtype=np.uint8)
    out = oracle.preprocess(rgb, 20, 20, 20, (0, 0, 0), (1, 1, 1)) * 255.0
    f = rgb.astype(np.float64)
    expect = (f[0::2, 0::2] + f[0::2, 1::2] + f[1::2, 0::2] + f[1::2, 1::2]) / 4.0
    np.testing.assert_allclose(out, expect.transpose(2, 0, 1), atol=1e-9)


# ---------------------------------------------------------------- antialiased resize

def _torch_antialias(rgb, resize_short, crop_h, crop_w):
    import torch
    import torch.nn.functional as F
    h, w, _ = rgb.shape
    ow, oh = oracle.resized_size(w, h, resize_short)
    t = torch.from_numpy(rgb.astype(np.float64)).permute(2, 0, 1)[None]
    r = F.interpolate(t, size=(oh, ow), mode="bilinear", antialias=True, align_corners=False)[0].numpy()
    top, left = (oh - crop_h) // 2, (ow - crop_w) // 2
    r = r[:, top:top + crop_h, left:left + crop_w]
    return (r / 255.0 - np.array(MEAN)[:, None, None]) / np.array(STD)[:, None, None]


@pytest.mark.parametrize("size,resize,crop", [((97, 61), 40, (32, 40)), ((300, 451), 128, (112, 100)),
                                               ((64, 48), 96, (80, 80)), ((201, 77), 64, (64, 150)),
                                               ((37, 500), 31, (300, 31))])
def test_antialiased_resize_against_torch_interpolate(size, resize, crop):
    # a library routine with the same definition (torch's CPU antialiased bilinear), in double
    w, h = size
    rgb = np.random.default_rng(w + h).integers(0, 256, size=(h, w, 3), dtype=np.uint8)
    got = oracle.preprocess(rgb, resize, crop[0], crop[1], MEAN, STD, antialias=True)
    np.testing.assert_allclose(got, _torch_antialias(rgb, resize, *crop), atol=1e-9)


def test_antialiased_resize_against_pillow_within_its_rounding():
    from PIL import Image
    rgb = _noise_image(31, 333, 222, sigma=20.0)
    ow, oh = oracle.resized_size(333, 222, 100)
    theirs = np.asarray(Image.fromarray(rgb).resize((ow, oh), Image.BILINEAR)).astype(np.float64)
    mine = oracle.preprocess(rgb, 100, oh, ow, (0, 0, 0), (1, 1, 1), antialias=True) * 255.0
    # Pillow rounds to 8 bits after each of its two passes
    assert np.abs(mine.transpose(1, 2, 0) - theirs).max() <= 1.0 + 1e-9
    # the plain two-tap resize is a different function on this image
    plain = oracle.preprocess(rgb, 100, oh, ow, (0, 0, 0), (1, 1, 1)) * 255.0
    assert np.abs(plain.transpose(1, 2, 0) - theirs).max() > 8.0


def test_antialiased_reduction_by_two_has_weights_1_3_3_1_over_8():
    rng = np.random.default_rng(32)
    rgb = rng.integers(0, 256, size=(24, 40, 3), dtype=np.uint8)
    out = oracle.preprocess(rgb, 12, 12, 20, (0, 0, 0), (1, 1, 1), antialias=True) * 255.0
    f = rgb.astype(np.float64)
    k = np.array([1.0, 3.0, 3.0, 1.0]) / 8.0
    for y in range(1, 11):
        for x in range(1, 19):
            patch = f[2 * y - 1:2 * y + 3, 2 * x - 1:2 * x + 3]
            np.testing.assert_allclose(out[:, y, x], np.einsum("r,c,rck->k", k, k, patch), atol=1e-9)
    # at the edge the window loses a sample and the other three are scaled up: 3 3 1 over 7
    e = np.array([3.0, 3.0, 1.0]) / 7.0
    np.testing.assert_allclose(out[:, 0, 0], np.einsum("r,c,rck->k", e, e, f[0:3, 0:3]), atol=1e-9)


def test_antialiased_resize_equals_the_plain_one_when_enlarging_and_keeps_constants():
    rgb = _noise_image(33, 50, 40)
    a = oracle.preprocess(rgb, 90, 80, 100, MEAN, STD, antialias=True)
    b = oracle.preprocess(rgb, 90, 80, 100, MEAN, STD)
    np.testing.assert_allclose(a, b, atol=1e-12)
    same = oracle.preprocess(rgb, 0, 30, 30, MEAN, STD, antialias=True)
    np.testing.assert_allclose(same, oracle.preprocess(rgb, 0, 30, 30, MEAN, STD), atol=1e-12)
    flat = np.full((45, 70, 3), 77, dtype=np.uint8)
    out = oracle.preprocess(flat, 20, 20, 20, MEAN, STD, antialias=True)
    for c in range(3):
        np.testing.assert_allclose(out[c], (77 / 255.0 - MEAN[c]) / STD[c], atol=1e-12)


def test_eight_bit_output_is_the_rounded_resized_sample():
    rng = np.random.default_rng(34)
    rgb = rng.integers(0, 256, size=(40, 60, 3), dtype=np.uint8)
    # scale 1: the source pixels themselves, interleaved
    assert np.array_equal(oracle.resize_crop_u8(rgb, 0, 30, 50), rgb[5:35, 5:55])
    # 2:1 with the plain filter: means of four integers, halves upwards
    f = rgb.astype(np.int64)
    s4 = f[0::2, 0::2] + f[0::2, 1::2] + f[1::2, 0::2] + f[1::2, 1::2]
    assert (s4 % 4 == 2).any(), "no half-way mean: the pin lost its point"
    assert np.array_equal(oracle.resize_crop_u8(rgb, 20, 20, 30), (s4 + 2) // 4)
    # 8:1 with the plain filter: the mean of the four pixels around 8 i + 4, halves upwards
    big = rng.integers(0, 256, size=(64, 64, 3), dtype=np.int64)
    m4 = big[3::8, 3::8] + big[3::8, 4::8] + big[4::8, 3::8] + big[4::8, 4::8]
    assert (m4 % 4 == 2).any()
    assert np.array_equal(oracle.resize_crop_u8(big.astype(np.uint8), 8, 8, 8), (m4 + 2) // 4)
    # antialiased: Pillow's own 8-bit result within a level (it rounds after each pass)
    from PIL import Image
    theirs = np.asarray(Image.fromarray(rgb).resize((30, 20), Image.BILINEAR)).astype(int)
    mine = oracle.resize_crop_u8(rgb, 20, 20, 30, antialias=True).astype(int)
    assert np.abs(mine - theirs).max() <= 1 and (mine == theirs).mean() > 0.75


def _exact_resize_u8(rgb, resize_short, crop_h, crop_w, antialias):
    """The resize definitions in exact fractions, rounded half up: the two-tap filter (taps
    floor(s), floor(s) + 1 of s = (i + 1/2) in/out - 1/2, clamped) and the triangle of
    half-width max(in/out, 1) around (i + 1/2) in/out over the window
    [floor(c - support + 1/2), floor(c + support + 1/2)) cut at the edge, weights scaled to sum 1."""
    from fractions import Fraction as F
    import math
    h, w, _ = rgb.shape
    ow, oh = oracle.resized_size(w, h, resize_short)
    top, left = (oh - crop_h) // 2, (ow - crop_w) // 2

    def taps(i, n_in, n_out):
        scale = F(n_in, n_out)
        if not antialias:
            s_ = (i + F(1, 2)) * scale - F(1, 2)
            f = math.floor(s_)
            t = s_ - f
            return [(min(max(f, 0), n_in - 1), 1 - t), (min(max(f + 1, 0), n_in - 1), t)]
        support, c = max(scale, F(1)), (i + F(1, 2)) * scale
        first, end = max(math.floor(c - support + F(1, 2)), 0), min(math.floor(c + support + F(1, 2)), n_in)
        wt = [max(1 - abs(j + F(1, 2) - c) / support, F(0)) for j in range(first, end)]
        return [(j, x / sum(wt)) for j, x in zip(range(first, end), wt)]

    out = np.zeros((crop_h, crop_w, 3), dtype=np.int64)
    halves = 0
    for y in range(crop_h):
        ty = taps(y + top, h, oh)
        for x in range(crop_w):
            tx = taps(x + left, w, ow)
            for c in range(3):
                v = sum(wy * wx * int(rgb[j, i, c]) for j, wy in ty for i, wx in tx)
                halves += (v - math.floor(v)) == F(1, 2)
                out[y, x, c] = math.floor(v + F(1, 2))
    return out, halves


@pytest.mark.parametrize("antialias", [False, True])
def test_eight_bit_output_at_exact_halves_of_rational_scales(antialias):
    # 4 -> 3 (two-tap weights in sixths) and 5 -> 3 (thirds; fifteenths under the triangle), on
    # pixels that are multiples of 3 plus a few others: many samples lie exactly half way between
    # two integers, where a floating-point evaluation falls on either side
    rng = np.random.default_rng(35)
    total = 0
    for (h, w, short, ch, cw) in ((32, 24, 18, 22, 18), (35, 25, 15, 21, 14)):
        rgb = (3 * rng.integers(0, 86, size=(h, w, 3))).astype(np.uint8)
        rgb[::4, ::3] += 1
        want, halves = _exact_resize_u8(rgb, short, ch, cw, antialias)
        total += halves
        assert np.array_equal(oracle.resize_crop_u8(rgb, short, ch, cw, antialias), want)
    assert total >= 20, "too few half-way samples: the pin lost its point"
    # an enlargement (2 -> 3: sixths again), where the triangle filter is the two-tap one
    small = rgb[:6, :8]
    want, _ = _exact_resize_u8(small, 9, 9, 12, antialias)
    assert np.array_equal(oracle.resize_crop_u8(small, 9, 9, 12, antialias), want)


def test_preprocess_rejects_bad_arguments():
    rgb = np.zeros((10, 10, 3), dtype=np.uint8)
    with pytest.raises(oracle.OracleError):
        oracle.preprocess(rgb, 8, 9, 8, MEAN, STD)       # crop larger than resized image
    with pytest.raises(oracle.OracleError):
        oracle.preprocess(rgb, 8, 8, 8, MEAN, (0.2, 0.0, 0.2))


def test_end_to_end_scale_one_ties_rgb_to_tensor():
    rgb = _noise_image(18, 256, 256, sigma=8.0)
    data, _ = oracle.encode(rgb, quality=85, mode=MODE_420, dri=16)
    _, dec, _ = oracle.decode(data, want_coef=False)
    out = oracle.decode_preprocess(data, 256, 224, 224, MEAN, STD)
    for c in range(3):
        np.testing.assert_allclose(out[c], (dec[16:240, 16:240, c] / 255.0 - MEAN[c]) / STD[c],
                                   atol=1e-12)
    assert np.abs(dec.astype(int) - rgb.astype(int)).mean() < 8.0


def test_error_budget_one_lsb_fits_the_tensor_tolerance():
    assert 1.0 / (255.0 * min(STD)) < 0.02
