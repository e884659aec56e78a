"""ctypes binding of the CPU oracle (``liboracle.so``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
``cpu_baseline`` leg of the benchmark.  The GPU library and its Python binding
never import this package.  Every function is a thin wrapper that marshals numpy
arrays; the arithmetic lives in the C sources next to this file.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SOURCES = ["transforms.c", "huffman.c", "jpeg_encode.c", "jpeg_decode.c"]
LIB_PATH = os.path.join(_HERE, "liboracle.so")

MODE_444, MODE_420, MODE_GRAY, MODE_422, MODE_440 = 0, 1, 2, 3, 4
# luma sampling factors (horizontal, vertical) and blocks per MCU of each mode
MODE_GEOMETRY = {MODE_444: (1, 1, 3), MODE_420: (2, 2, 6), MODE_GRAY: (1, 1, 1), MODE_422: (2, 1, 4),
                 MODE_440: (1, 2, 4)}
OK, E_ARG, E_CORRUPT, E_UNSUPPORTED = 0, -1, -2, -3


def build(force=True):
    """Compile the oracle with gcc (plain C11, -O2)."""
    if not force and os.path.exists(LIB_PATH):
        return LIB_PATH
    cmd = ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", LIB_PATH]
    cmd += [os.path.join(_HERE, s) for s in _SOURCES] + ["-lm"]
    subprocess.run(cmd, check=True)
    return LIB_PATH


class Info(C.Structure):
    _fields_ = [
        ("width", C.c_int32), ("height", C.c_int32), ("ncomp", C.c_int32),
        ("hs", C.c_int32 * 3), ("vs", C.c_int32 * 3),
        ("hmax", C.c_int32), ("vmax", C.c_int32),
        ("mcu_cols", C.c_int32), ("mcu_rows", C.c_int32),
        ("blocks_per_mcu", C.c_int32), ("restart_interval", C.c_int32),
        ("nblocks", C.c_int64), ("entropy_bytes", C.c_int64),
        ("symbols", C.c_int64), ("coded_bits", C.c_int64),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        L = C.CDLL(LIB_PATH)
        u8p, i16p, u16p, dp = (C.POINTER(C.c_uint8), C.POINTER(C.c_int16),
                               C.POINTER(C.c_uint16), C.POINTER(C.c_double))
        L.oracle_zigzag_pos.argtypes = [C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)]
        L.oracle_zigzag_pos.restype = None
        L.oracle_idct8x8.argtypes = [dp, dp]
        L.oracle_idct8x8.restype = None
        L.oracle_fdct8x8.argtypes = [dp, dp]
        L.oracle_fdct8x8.restype = None
        L.oracle_ycc_to_rgb.argtypes = [C.c_int, C.c_int, C.c_int, u8p]
        L.oracle_ycc_to_rgb.restype = None
        L.oracle_rgb_to_ycc.argtypes = [C.c_int, C.c_int, C.c_int, u8p]
        L.oracle_rgb_to_ycc.restype = None
        L.oracle_huff_codes.argtypes = [u8p, u16p, u8p]
        L.oracle_huff_codes.restype = C.c_int
        L.oracle_huff_from_freq.argtypes = [C.POINTER(C.c_int64), u8p, u8p]
        L.oracle_huff_from_freq.restype = C.c_int
        L.oracle_quant_table.argtypes = [C.c_int, C.c_int, u16p]
        L.oracle_quant_table.restype = None
        L.oracle_forward_blocks.argtypes = [u8p, C.c_int, C.c_int, C.c_int, u16p, u16p,
                                            i16p, C.c_size_t, C.POINTER(Info)]
        L.oracle_forward_blocks.restype = C.c_int
        L.oracle_write_jpeg.argtypes = [i16p, C.c_int, C.c_int, C.c_int, u16p, u16p,
                                        C.c_int, C.c_int, u8p, C.c_size_t]
        L.oracle_write_jpeg.restype = C.c_int64
        L.oracle_jpeg_info.argtypes = [u8p, C.c_size_t, C.POINTER(Info)]
        L.oracle_jpeg_info.restype = C.c_int
        L.oracle_jpeg_decode.argtypes = [u8p, C.c_size_t, i16p, C.c_size_t, u8p, C.c_size_t,
                                         C.POINTER(Info)]
        L.oracle_jpeg_decode.restype = C.c_int
        L.oracle_jpeg_decode_smooth.argtypes = L.oracle_jpeg_decode.argtypes
        L.oracle_jpeg_decode_smooth.restype = C.c_int
        L.oracle_upsample_triangle.argtypes = [u8p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                               C.c_int, C.c_int, u8p]
        L.oracle_upsample_triangle.restype = C.c_int
        L.oracle_resized_size.argtypes = [C.c_int, C.c_int, C.c_int,
                                          C.POINTER(C.c_int), C.POINTER(C.c_int)]
        L.oracle_resized_size.restype = None
        L.oracle_preprocess.argtypes = [u8p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                        dp, dp, dp]
        L.oracle_preprocess.restype = C.c_int
        L.oracle_preprocess_antialias.argtypes = L.oracle_preprocess.argtypes
        L.oracle_preprocess_antialias.restype = C.c_int
        L.oracle_resize_crop_u8.argtypes = [u8p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, u8p]
        L.oracle_resize_crop_u8.restype = C.c_int
        _lib = L
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what}: oracle error {code}")
        self.code = code


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def _bytes_arr(data):
    return np.frombuffer(bytes(data), dtype=np.uint8) if not isinstance(data, np.ndarray) \
        else np.ascontiguousarray(data, dtype=np.uint8)


def zigzag_pos(k):
    v, u = C.c_int(), C.c_int()
    lib().oracle_zigzag_pos(k, C.byref(v), C.byref(u))
    return v.value, u.value


def idct8x8(F):
    F = np.ascontiguousarray(F, dtype=np.float64).reshape(64)
    f = np.empty(64, dtype=np.float64)
    lib().oracle_idct8x8(_p(F, C.c_double), _p(f, C.c_double))
    return f.reshape(8, 8)


def fdct8x8(f):
    f = np.ascontiguousarray(f, dtype=np.float64).reshape(64)
    F = np.empty(64, dtype=np.float64)
    lib().oracle_fdct8x8(_p(f, C.c_double), _p(F, C.c_double))
    return F.reshape(8, 8)


def ycc_to_rgb(y, cb, cr):
    out = (C.c_uint8 * 3)()
    lib().oracle_ycc_to_rgb(int(y), int(cb), int(cr), out)
    return tuple(out)


def rgb_to_ycc(r, g, b):
    out = (C.c_uint8 * 3)()
    lib().oracle_rgb_to_ycc(int(r), int(g), int(b), out)
    return tuple(out)


def huff_codes(bits17):
    bits = np.ascontiguousarray(bits17, dtype=np.uint8)
    assert bits.size == 17
    code = np.zeros(256, dtype=np.uint16)
    size = np.zeros(256, dtype=np.uint8)
    n = lib().oracle_huff_codes(_p(bits, C.c_uint8), _p(code, C.c_uint16), _p(size, C.c_uint8))
    if n < 0:
        raise OracleError(n, "huff_codes")
    return code[:n].copy(), size[:n].copy()


def huff_from_freq(freq256):
    freq = np.ascontiguousarray(freq256, dtype=np.int64)
    assert freq.size == 256
    bits = np.zeros(17, dtype=np.uint8)
    vals = np.zeros(256, dtype=np.uint8)
    n = lib().oracle_huff_from_freq(_p(freq, C.c_int64), _p(bits, C.c_uint8), _p(vals, C.c_uint8))
    if n < 0:
        raise OracleError(n, "huff_from_freq")
    return bits, vals[:n].copy()


def quant_table(quality, chroma):
    q = np.zeros(64, dtype=np.uint16)
    lib().oracle_quant_table(int(quality), int(bool(chroma)), _p(q, C.c_uint16))
    return q


def forward_blocks(rgb, mode, qluma, qchroma):
    """RGB8 HWC image -> (coefficients [nblocks,64] int16 zig-zag, Info)."""
    rgb = np.ascontiguousarray(rgb, dtype=np.uint8)
    h, w, _ = rgb.shape
    qluma = np.ascontiguousarray(qluma, dtype=np.uint16)
    qchroma = np.ascontiguousarray(qchroma, dtype=np.uint16)
    hmax, vmax, bpm = MODE_GEOMETRY[mode]
    nb = -(-w // (8 * hmax)) * -(-h // (8 * vmax)) * bpm
    coef = np.zeros((nb, 64), dtype=np.int16)
    info = Info()
    rc = lib().oracle_forward_blocks(_p(rgb, C.c_uint8), w, h, mode, _p(qluma, C.c_uint16),
                                     _p(qchroma, C.c_uint16), _p(coef, C.c_int16), coef.size,
                                     C.byref(info))
    if rc:
        raise OracleError(rc, "forward_blocks")
    assert info.nblocks == nb
    return coef, info


def write_jpeg(coef, w, h, mode, qluma, qchroma, dri=0, table_mode=0):
    """Quantised coefficients -> bytes of a baseline JPEG file."""
    coef = np.ascontiguousarray(coef, dtype=np.int16)
    qluma = np.ascontiguousarray(qluma, dtype=np.uint16)
    qchroma = np.ascontiguousarray(qchroma, dtype=np.uint16)
    cap = 4096 + coef.size * 4 + (coef.size // 64) * 8
    out = np.empty(cap, dtype=np.uint8)
    n = lib().oracle_write_jpeg(_p(coef, C.c_int16), w, h, mode, _p(qluma, C.c_uint16),
                                _p(qchroma, C.c_uint16), int(dri), int(table_mode),
                                _p(out, C.c_uint8), cap)
    if n < 0:
        raise OracleError(int(n), "write_jpeg")
    return out[:n].tobytes()


def encode(rgb, quality=90, mode=MODE_420, dri=0, table_mode=0):
    """RGB8 HWC image -> (jpeg bytes, coefficients the encoder coded)."""
    ql, qc = quant_table(quality, 0), quant_table(quality, 1)
    coef, info = forward_blocks(rgb, mode, ql, qc)
    data = write_jpeg(coef, info.width, info.height, mode, ql, qc, dri, table_mode)
    return data, coef


def jpeg_info(data):
    a = _bytes_arr(data)
    info = Info()
    rc = lib().oracle_jpeg_info(_p(a, C.c_uint8), a.size, C.byref(info))
    if rc:
        raise OracleError(rc, "jpeg_info")
    return info


def upsample_triangle(plane, fx, fy, w, h):
    """Subsampled plane [ch, cw] uint8 -> [h, w] by the centred triangle (oracle_upsample_triangle)."""
    plane = np.ascontiguousarray(plane, dtype=np.uint8)
    ch, cw = plane.shape
    out = np.empty((h, w), dtype=np.uint8)
    rc = lib().oracle_upsample_triangle(_p(plane, C.c_uint8), cw, cw, ch, fx, fy, w, h, _p(out, C.c_uint8))
    if rc:
        raise OracleError(rc, "upsample_triangle")
    return out


def decode(data, want_coef=True, want_rgb=True, smooth_chroma=False):
    """JPEG bytes -> (coefficients [nblocks,64] or None, rgb [H,W,3] or None, Info).

    smooth_chroma: subsampled chroma is interpolated (centred triangle) instead of replicated."""
    a = _bytes_arr(data)
    info = jpeg_info(a)
    coef = np.zeros((info.nblocks, 64), dtype=np.int16) if want_coef else None
    rgb = np.zeros((info.height, info.width, 3), dtype=np.uint8) if want_rgb else None
    fn = lib().oracle_jpeg_decode_smooth if smooth_chroma else lib().oracle_jpeg_decode
    rc = fn(
        _p(a, C.c_uint8), a.size,
        _p(coef, C.c_int16) if want_coef else None, coef.size if want_coef else 0,
        _p(rgb, C.c_uint8) if want_rgb else None, rgb.size if want_rgb else 0,
        C.byref(info))
    if rc:
        raise OracleError(rc, "decode")
    return coef, rgb, info


def resized_size(w, h, s):
    ow, oh = C.c_int(), C.c_int()
    lib().oracle_resized_size(w, h, s, C.byref(ow), C.byref(oh))
    return ow.value, oh.value


def preprocess(rgb, resize_short, crop_h, crop_w, mean, std, antialias=False):
    """RGB8 HWC -> float64 [3, crop_h, crop_w] (resize, centre crop, normalize).

    antialias: the resize averages under a triangle as wide as an output sample where the
    image shrinks (oracle_preprocess_antialias) instead of reading two samples per axis."""
    rgb = np.ascontiguousarray(rgb, dtype=np.uint8)
    h, w, _ = rgb.shape
    mean = np.ascontiguousarray(mean, dtype=np.float64)
    std = np.ascontiguousarray(std, dtype=np.float64)
    out = np.empty((3, crop_h, crop_w), dtype=np.float64)
    fn = lib().oracle_preprocess_antialias if antialias else lib().oracle_preprocess
    rc = fn(_p(rgb, C.c_uint8), w, h, int(resize_short), crop_h, crop_w,
            _p(mean, C.c_double), _p(std, C.c_double), _p(out, C.c_double))
    if rc:
        raise OracleError(rc, "preprocess")
    return out


def resize_crop_u8(rgb, resize_short, crop_h, crop_w, antialias=False):
    """RGB8 HWC -> RGB8 [crop_h, crop_w, 3]: resize and centre crop, rounded to 8 bits."""
    rgb = np.ascontiguousarray(rgb, dtype=np.uint8)
    h, w, _ = rgb.shape
    out = np.empty((crop_h, crop_w, 3), dtype=np.uint8)
    rc = lib().oracle_resize_crop_u8(_p(rgb, C.c_uint8), w, h, int(resize_short), crop_h, crop_w,
                                     int(bool(antialias)), _p(out, C.c_uint8))
    if rc:
        raise OracleError(rc, "resize_crop_u8")
    return out


def decode_preprocess(data, resize_short, crop_h, crop_w, mean, std, antialias=False):
    """Whole path for one image: JPEG bytes -> float64 tensor [3, crop_h, crop_w]."""
    _, rgb, _ = decode(data, want_coef=False, want_rgb=True)
    return preprocess(rgb, resize_short, crop_h, crop_w, mean, std, antialias)
