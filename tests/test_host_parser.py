"""Host-side logic of libprep, no GPU needed: the shared library loads and exports every
symbol the header declares, and the marker/table parser agrees with the oracle's own marker
walk and survives malformed input."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2411_19114_amd as prep
import synth
from oracle import MODE_420, MODE_444, MODE_GRAY

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def built():
    if not os.path.exists(prep.lib_path()):
        prep.build()


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "prep.h")).read()
    declared = set(re.findall(r"\b(prep_[a-z_0-9]+)\s*\(", header))
    assert declared == set(prep.binding.EXPORTS)
    L = ctypes.CDLL(prep.lib_path())
    for name in sorted(declared):
        assert hasattr(L, name), name
    assert prep.strerror(0) == "ok" and "corrupt" in prep.strerror(prep.E_CORRUPT)


def _img(seed, w, h):
    return synth.gradient_noise_image(np.random.default_rng(seed), w, h, 10.0)


def test_parser_agrees_with_the_oracle_marker_walk():
    streams = []
    for k, (w, h) in enumerate([(1, 1), (17, 33), (300, 251), (640, 480)]):
        for mode in (MODE_444, MODE_420, MODE_GRAY):
            for dri in (0, 1, 7):
                streams.append(oracle.encode(_img(k, w, h), 80, mode, dri)[0])
    streams += synth.make_batch(2, 3) + synth.make_batch(5, 3)
    blob, offsets = synth.pack(streams)
    infos = prep.parse_headers(blob, offsets)
    total = 0
    for s, i in zip(streams, infos):
        o = oracle.jpeg_info(s)
        assert i.status == 0
        assert (i.width, i.height, i.mcu_cols, i.mcu_rows) == (o.width, o.height, o.mcu_cols, o.mcu_rows)
        assert i.blocks_per_mcu == o.blocks_per_mcu and i.restart_interval == o.restart_interval
        assert i.sampling == (MODE_GRAY if o.ncomp == 1 else MODE_420 if o.hmax == 2 else MODE_444)
        sos = s.index(b"\xff\xda")
        ns = s[sos + 4]
        assert i.entropy_offset == sos + 2 + 6 + 2 * ns
        assert i.entropy_offset + i.entropy_bytes == len(s) - 2 and s[-2:] == b"\xff\xd9"
        nmcu = o.mcu_cols * o.mcu_rows
        assert i.n_intervals == (-(-nmcu // o.restart_interval) if o.restart_interval else 1)
        total += i.n_intervals
    desc = prep.interval_descriptors(infos)
    assert len(desc) == total
    # descriptors tile each image's MCUs in order, RST index counts modulo 8
    k = 0
    for n, i in enumerate(infos):
        nmcu, ri, m, j = i.mcu_cols * i.mcu_rows, i.restart_interval or i.mcu_cols * i.mcu_rows, 0, 0
        while m < nmcu:
            d = desc[k]
            assert (d.image, d.first_mcu, d.n_mcu) == (n, m, min(ri, nmcu - m))
            assert d.rst_index == (-1 if j == 0 else (j - 1) % 8)
            m += ri; j += 1; k += 1


def test_parser_rejects_what_it_does_not_support():
    good = oracle.encode(_img(9, 40, 24), 80, MODE_420, 3)[0]

    def status(data):
        blob, off = synth.pack([data])
        return prep.parse_headers(blob, off)[0].status

    assert status(good) == 0
    assert status(good.replace(b"\xff\xc0", b"\xff\xc2", 1)) == prep.E_UNSUPPORTED   # progressive
    assert status(good.replace(b"\xff\xc0", b"\xff\xc9", 1)) == prep.E_UNSUPPORTED   # arithmetic
    sof = good.index(b"\xff\xc0")
    assert status(good[:sof + 4] + b"\x0c" + good[sof + 5:]) == prep.E_UNSUPPORTED   # 12 bit
    assert status(good[:sof + 11] + b"\x41" + good[sof + 12:]) == prep.E_UNSUPPORTED  # luma 4 x 1
    assert status(good[:sof + 14] + b"\x21" + good[sof + 15:]) == prep.E_UNSUPPORTED  # chroma 2 x 1
    assert status(good[:-2]) == prep.E_CORRUPT                                       # no EOI
    assert status(b"\x00" + good[1:]) == prep.E_CORRUPT                              # no SOI
    dht = good.index(b"\xff\xc4")
    assert status(good[:dht] + good[dht + 2 + (good[dht + 2] << 8 | good[dht + 3]):]) == prep.E_CORRUPT
    dqt = good.index(b"\xff\xdb")
    assert status(good[:dqt + 5] + b"\x00" + good[dqt + 6:]) == prep.E_CORRUPT       # zero quantiser
    # a Huffman table that uses the whole code space (an all-ones code word) is refused
    full = bytearray(good)
    bits = bytes([0, 4] + [0] * 14)            # four 2-bit codes: 00 01 10 11
    assert full[dht + 4] == 0x00
    seg_len = 2 + 1 + 16 + 4
    new_dht = b"\xff\xc4" + bytes([0, seg_len, 0x00]) + bits + bytes([0, 1, 2, 3])
    old_len = (good[dht + 2] << 8) | good[dht + 3]
    assert status(bytes(full[:dht]) + new_dht + bytes(full[dht + 2 + old_len:])) == prep.E_CORRUPT


def test_parser_survives_truncation_and_noise_everywhere():
    rng = np.random.default_rng(3)
    good = synth.make_image(2, 0)[0]
    sos = good.index(b"\xff\xda")
    cases = [good[:n] for n in range(0, sos + 20)]
    for _ in range(300):
        b = bytearray(good[:sos + 64])
        for _ in range(int(rng.integers(1, 6))):
            b[int(rng.integers(0, len(b)))] = int(rng.integers(0, 256))
        cases.append(bytes(b) + good[sos + 64:])
    blob, offsets = synth.pack(cases)
    infos = prep.parse_headers(blob, offsets)
    assert len(infos) == len(cases)
    for c, i in zip(cases, infos):
        assert i.status in (0, prep.E_CORRUPT, prep.E_UNSUPPORTED)
        if i.status == 0:
            assert 1 <= i.width <= 65535 and 1 <= i.height <= 65535
            assert i.entropy_offset + i.entropy_bytes + 2 <= len(c)
    assert all(i.status != 0 for i in infos[:sos + 14])   # every truncated header fails
