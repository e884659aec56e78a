"""ctypes marshalling for libprep.so.  Same names as the C ABI, no arithmetic."""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_HERE, "csrc")
_SOURCES = ["entropy.hip", "reconstruct.hip", "resize.hip", "static_entry.hip", "api.cpp", "parser.cpp", "batcher.cpp", "audio.hip"]

OK, E_INVALID_ARG, E_TOO_LARGE, E_HIP, E_UNSUPPORTED, E_CORRUPT, E_NOMEM = 0, -1, -2, -3, -4, -5, -6
F32, F16, U8_NHWC = 0, 1, 2
FLAG_TABLES_PER_WORKGROUP = 1
FLAG_FULL_RGB = 2
FLAG_SMOOTH_CHROMA = 4
FLAG_LARGE_WINDOWS = 8
FILTER_BILINEAR, FILTER_ANTIALIAS = 0, 1


def lib_path():
    return os.path.join(_HERE, "libprep.so")


def build(verbose=False):
    """Compile the HIP library for gfx950 with hipcc (cross-compiles without a GPU)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    # -falign-loops: the entropy decoder's symbol loops run as lone waves that pay for every
    # instruction fetch; where their headers fall in a fetch line moved its time by 3 %
    cmd = [hipcc, "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared", "-pthread",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-falign-loops=32",
           "-o", lib_path()] + [os.path.join(_CSRC, s) for s in _SOURCES]
    r = subprocess.run(cmd, capture_output=not verbose, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + (r.stderr or ""))
    return lib_path()


class PrepError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what}: {strerror(code)} ({code})")
        self.code = code


class Config(C.Structure):
    _fields_ = [("device", C.c_int32), ("max_batch", C.c_int32), ("max_width", C.c_int32),
                ("max_height", C.c_int32), ("max_bitstream_bytes", C.c_uint64),
                ("max_total_pixels", C.c_uint64), ("flags", C.c_uint32)]


class Params(C.Structure):
    _fields_ = [("resize_short", C.c_int32), ("crop_h", C.c_int32), ("crop_w", C.c_int32),
                ("out_dtype", C.c_int32), ("mean", C.c_float * 3), ("std", C.c_float * 3),
                ("filter", C.c_int32)]


class AudioConfig(C.Structure):
    _fields_ = [("device", C.c_int32), ("max_batch", C.c_int32), ("rate", C.c_int32), ("n_fft", C.c_int32),
                ("win_length", C.c_int32), ("hop", C.c_int32), ("n_mels", C.c_int32), ("reserved", C.c_int32),
                ("max_total_samples", C.c_uint64)]


class ServerConfig(C.Structure):
    _fields_ = [("handle", Config), ("params", Params), ("n_consumers", C.c_int32), ("batch_max", C.c_int32),
                ("time_queue_us", C.c_int64), ("max_request_bytes", C.c_int32), ("queue_capacity", C.c_int32)]


class ServerResult(C.Structure):
    _fields_ = [("tag", C.c_uint64), ("status", C.c_int32), ("batch_size", C.c_int32), ("consumer", C.c_int32),
                ("slot", C.c_int32), ("arrival_ns", C.c_int64), ("start_ns", C.c_int64),
                ("done_ns", C.c_int64), ("tensor", C.c_void_p)]


class ImageInfo(C.Structure):
    _fields_ = [("status", C.c_int32), ("width", C.c_int32), ("height", C.c_int32),
                ("sampling", C.c_int32), ("mcu_cols", C.c_int32), ("mcu_rows", C.c_int32),
                ("blocks_per_mcu", C.c_int32), ("restart_interval", C.c_int32),
                ("n_intervals", C.c_int32), ("reserved", C.c_int32),
                ("entropy_offset", C.c_uint64), ("entropy_bytes", C.c_uint64)]


class IntervalDesc(C.Structure):
    _fields_ = [("image", C.c_int32), ("first_mcu", C.c_int32), ("n_mcu", C.c_int32),
                ("rst_index", C.c_int32)]


EXPORTS = [
    "prep_create", "prep_destroy", "prep_decode_resize_batch", "prep_decode_resize_batch_resident",
    "prep_get_status", "prep_strerror", "prep_parse_headers", "prep_interval_descriptors",
    "prep_resize_normalize", "prep_resize_normalize_static", "prep_reconstruct_from_coefficients", "prep_debug_last_coefficients",
    "prep_debug_last_rgb", "prep_debug_last_region", "prep_stage_ms", "prep_set_timing",
    "prep_policy_create", "prep_policy_destroy", "prep_policy_arrive", "prep_policy_deadline",
    "prep_policy_take", "prep_policy_pending", "prep_server_create", "prep_server_destroy",
    "prep_server_submit", "prep_server_next", "prep_server_release", "prep_server_next_many",
    "prep_server_release_many", "prep_server_copy_tensor",
    "prep_audio_create", "prep_audio_destroy", "prep_audio_frames", "prep_audio_features",
]

_lib = None


def lib():
    """Load libprep.so; there is no fallback when it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(lib_path()):
            raise RuntimeError(f"{lib_path()} is not built: run __graft_entry__.build() "
                               "(hipcc --offload-arch=gfx950)")
        # PyTorch ships its own HIP runtime under the same soname; it must be the one
        # this process uses, so it is loaded first and libprep binds to it.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(lib_path())
        vp, u8p, u64p, i32p = C.c_void_p, C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(C.c_int32)
        L.prep_create.argtypes = [C.POINTER(vp), C.POINTER(Config)]
        L.prep_destroy.argtypes = [vp]
        L.prep_decode_resize_batch.argtypes = [vp, u8p, u64p, C.c_int32, C.POINTER(Params), vp, vp]
        L.prep_decode_resize_batch_resident.argtypes = [vp, u8p, vp, u64p, C.c_int32,
                                                        C.POINTER(Params), vp, vp]
        L.prep_get_status.argtypes = [vp, i32p, C.c_int32]
        L.prep_strerror.argtypes = [C.c_int]
        L.prep_strerror.restype = C.c_char_p
        L.prep_parse_headers.argtypes = [u8p, u64p, C.c_int32, C.POINTER(ImageInfo)]
        L.prep_interval_descriptors.argtypes = [C.POINTER(ImageInfo), C.c_int32,
                                                C.POINTER(IntervalDesc), C.c_int64]
        L.prep_interval_descriptors.restype = C.c_int64
        L.prep_resize_normalize.argtypes = [vp, vp, u64p, i32p, i32p, i32p, C.c_int32,
                                            C.POINTER(Params), vp, vp]
        L.prep_resize_normalize_static.argtypes = [C.c_int32, vp, u64p, i32p, i32p, i32p, C.c_int32,
                                                   C.POINTER(Params), vp, vp]
        L.prep_reconstruct_from_coefficients.argtypes = [vp, u8p, u64p, C.c_int32, vp, C.c_uint64,
                                                         C.POINTER(Params), vp, vp]
        L.prep_debug_last_coefficients.argtypes = [vp, C.c_int32, vp, C.c_uint64]
        L.prep_debug_last_coefficients.restype = C.c_int64
        L.prep_debug_last_rgb.argtypes = [vp, C.c_int32, vp, C.c_uint64]
        L.prep_debug_last_rgb.restype = C.c_int64
        L.prep_debug_last_region.argtypes = [vp, C.c_int32, C.POINTER(C.c_int32)]
        L.prep_stage_ms.argtypes = [vp, C.c_int32, C.POINTER(C.c_float)]
        L.prep_set_timing.argtypes = [vp, C.c_int32]
        L.prep_policy_create.argtypes = [C.POINTER(vp), C.c_int32, C.c_int64]
        L.prep_policy_destroy.argtypes = [vp]
        L.prep_policy_destroy.restype = None
        L.prep_policy_arrive.argtypes = [vp, C.c_uint64, C.c_int64]
        L.prep_policy_deadline.argtypes = [vp]
        L.prep_policy_deadline.restype = C.c_int64
        L.prep_policy_take.argtypes = [vp, C.c_int64, C.POINTER(C.c_uint64), C.c_int32]
        L.prep_policy_pending.argtypes = [vp]
        L.prep_server_create.argtypes = [C.POINTER(vp), C.POINTER(ServerConfig)]
        L.prep_server_destroy.argtypes = [vp]
        L.prep_server_submit.argtypes = [vp, vp, C.c_uint64, C.c_uint64]
        L.prep_server_next.argtypes = [vp, C.POINTER(ServerResult), C.c_int64]
        L.prep_server_copy_tensor.argtypes = [vp, C.POINTER(ServerResult), vp]
        L.prep_server_release.argtypes = [vp, C.POINTER(ServerResult)]
        L.prep_server_next_many.argtypes = [vp, C.POINTER(ServerResult), C.c_int32, C.c_int64]
        L.prep_server_release_many.argtypes = [vp, C.POINTER(ServerResult), C.c_int32]
        L.prep_audio_create.argtypes = [C.POINTER(vp), C.POINTER(AudioConfig)]
        L.prep_audio_destroy.argtypes = [vp]
        L.prep_audio_frames.argtypes = [C.POINTER(AudioConfig), C.c_uint64, C.c_int32]
        L.prep_audio_frames.restype = C.c_int64
        L.prep_audio_features.argtypes = [vp, vp, u64p, C.c_int32, C.c_int32, vp, u64p, vp]
        _lib = L
    return _lib


def strerror(code):
    return lib().prep_strerror(int(code)).decode()


def _check(rc, what):
    if rc != OK:
        raise PrepError(rc, what)


def _u8(a):
    a = np.ascontiguousarray(a, dtype=np.uint8)
    return a, a.ctypes.data


def _u64(a):
    a = np.ascontiguousarray(a, dtype=np.uint64)
    return a, a.ctypes.data_as(C.POINTER(C.c_uint64))


def make_params(resize_short, crop_h, crop_w, out_dtype, mean, std, filter=FILTER_BILINEAR):
    p = Params()
    p.resize_short, p.crop_h, p.crop_w = int(resize_short), int(crop_h), int(crop_w)
    p.out_dtype = {"f32": F32, "f16": F16, "u8": U8_NHWC}.get(out_dtype, out_dtype)
    p.filter = int(filter)
    p.mean[:] = [float(m) for m in mean]
    p.std[:] = [float(s) for s in std]
    return p


def parse_headers(bitstreams, offsets):
    """prep_parse_headers: host marker parser only -> list of ImageInfo."""
    b, bp = _u8(bitstreams)
    o, op = _u64(offsets)
    n = len(o) - 1
    info = (ImageInfo * max(n, 1))()
    _check(lib().prep_parse_headers(bp, op, n, info), "prep_parse_headers")
    return list(info)[:n]


def interval_descriptors(infos):
    """prep_interval_descriptors -> list of IntervalDesc."""
    n = len(infos)
    arr = (ImageInfo * max(n, 1))(*infos)
    total = lib().prep_interval_descriptors(arr, n, None, 0)
    if total < 0:
        raise PrepError(int(total), "prep_interval_descriptors")
    desc = (IntervalDesc * max(total, 1))()
    lib().prep_interval_descriptors(arr, n, desc, total)
    return list(desc)[:total]


def resize_normalize_static(device, rgb_ptr, rgb_offsets, widths, heights, pitches, params, out_ptr,
                            stream=0):
    """prep_resize_normalize_static: the resize stage without a handle, allocating nothing."""
    o, op = _u64(rgb_offsets)
    w = np.ascontiguousarray(widths, dtype=np.int32)
    h = np.ascontiguousarray(heights, dtype=np.int32)
    p = np.ascontiguousarray(pitches, dtype=np.int32)
    i32p = C.POINTER(C.c_int32)
    _check(lib().prep_resize_normalize_static(
        int(device), C.c_void_p(rgb_ptr), op, w.ctypes.data_as(i32p), h.ctypes.data_as(i32p),
        p.ctypes.data_as(i32p), len(w), C.byref(params), C.c_void_p(out_ptr), C.c_void_p(stream)),
        "prep_resize_normalize_static")


class Preprocessor:
    """Owns one prep_handle.  Device pointers are plain integers (tensor.data_ptr())."""

    def __init__(self, device=0, max_batch=256, max_width=640, max_height=640,
                 max_bitstream_bytes=64 << 20, max_total_pixels=0, flags=0):
        self._h = C.c_void_p()
        cfg = Config(device, max_batch, max_width, max_height, max_bitstream_bytes,
                     max_total_pixels, flags)
        _check(lib().prep_create(C.byref(self._h), C.byref(cfg)), "prep_create")

    def close(self):
        if self._h:
            lib().prep_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def decode_resize_batch(self, bitstreams, offsets, params, out_ptr, stream=0):
        b, bp = _u8(bitstreams)
        o, op = _u64(offsets)
        _check(lib().prep_decode_resize_batch(self._h, bp, op, len(o) - 1, C.byref(params),
                                              C.c_void_p(out_ptr), C.c_void_p(stream)),
               "prep_decode_resize_batch")

    def decode_resize_batch_resident(self, bitstreams, bitstreams_device_ptr, offsets, params,
                                     out_ptr, stream=0):
        b, bp = _u8(bitstreams)
        o, op = _u64(offsets)
        _check(lib().prep_decode_resize_batch_resident(
            self._h, bp, C.c_void_p(bitstreams_device_ptr), op, len(o) - 1, C.byref(params),
            C.c_void_p(out_ptr), C.c_void_p(stream)), "prep_decode_resize_batch_resident")

    def get_status(self, n):
        st = (C.c_int32 * max(n, 1))()
        _check(lib().prep_get_status(self._h, st, n), "prep_get_status")
        return list(st)[:n]

    def resize_normalize(self, rgb_ptr, rgb_offsets, widths, heights, pitches, params, out_ptr,
                         stream=0):
        o, op = _u64(rgb_offsets)
        w = np.ascontiguousarray(widths, dtype=np.int32)
        h = np.ascontiguousarray(heights, dtype=np.int32)
        p = np.ascontiguousarray(pitches, dtype=np.int32)
        i32p = C.POINTER(C.c_int32)
        _check(lib().prep_resize_normalize(
            self._h, C.c_void_p(rgb_ptr), op, w.ctypes.data_as(i32p), h.ctypes.data_as(i32p),
            p.ctypes.data_as(i32p), len(w), C.byref(params), C.c_void_p(out_ptr),
            C.c_void_p(stream)), "prep_resize_normalize")

    def reconstruct_from_coefficients(self, bitstreams, offsets, coefficients, params, out_ptr,
                                      stream=0):
        b, bp = _u8(bitstreams)
        o, op = _u64(offsets)
        c = np.ascontiguousarray(coefficients, dtype=np.int16)
        _check(lib().prep_reconstruct_from_coefficients(
            self._h, bp, op, len(o) - 1, c.ctypes.data, c.size, C.byref(params),
            C.c_void_p(out_ptr), C.c_void_p(stream)), "prep_reconstruct_from_coefficients")

    def debug_last_coefficients(self, image, n_blocks):
        out = np.empty((n_blocks, 64), dtype=np.int16)
        n = lib().prep_debug_last_coefficients(self._h, image, out.ctypes.data, out.size)
        if n < 0:
            raise PrepError(int(n), "prep_debug_last_coefficients")
        assert n == out.size
        return out

    def debug_last_rgb(self, image, height, width):
        out = np.empty((height, width, 3), dtype=np.uint8)
        n = lib().prep_debug_last_rgb(self._h, image, out.ctypes.data, out.size)
        if n < 0:
            raise PrepError(int(n), "prep_debug_last_rgb")
        assert n == out.size
        return out

    def debug_last_region(self, image):
        """(x0, y0, x1, y1): the pixels of the image that the last call converted to RGB."""
        rect = (C.c_int32 * 4)()
        _check(lib().prep_debug_last_region(self._h, image, rect), "prep_debug_last_region")
        return tuple(rect)

    def set_timing(self, enabled):
        _check(lib().prep_set_timing(self._h, int(bool(enabled))), "prep_set_timing")

    def stage_ms(self, calls_back=0):
        ms = (C.c_float * 4)()
        _check(lib().prep_stage_ms(self._h, calls_back, ms), "prep_stage_ms")
        return list(ms)


class BatchPolicy:
    """The batching rule alone (prep_policy_*), driven by the caller's clock."""

    def __init__(self, batch_max, time_queue_ns):
        self._p = C.c_void_p()
        _check(lib().prep_policy_create(C.byref(self._p), int(batch_max), int(time_queue_ns)), "prep_policy_create")
        self._ids = (C.c_uint64 * int(batch_max))()

    def arrive(self, request_id, t_ns):
        _check(lib().prep_policy_arrive(self._p, int(request_id), int(t_ns)), "prep_policy_arrive")

    def deadline(self):
        return int(lib().prep_policy_deadline(self._p))

    def take(self, now_ns):
        n = lib().prep_policy_take(self._p, int(now_ns), self._ids, len(self._ids))
        if n < 0:
            raise PrepError(int(n), "prep_policy_take")
        return [int(self._ids[i]) for i in range(n)]

    def pending(self):
        return int(lib().prep_policy_pending(self._p))

    def close(self):
        if self._p:
            lib().prep_policy_destroy(self._p)
            self._p = C.c_void_p()


class Server:
    """prep_server_*: the batching rule in front of n_consumers handles and streams."""

    def __init__(self, n_consumers, batch_max, time_queue_us, params, max_width, max_height,
                 max_request_bytes, queue_capacity=4096, device=0, flags=0):
        cfg = ServerConfig()
        cfg.handle = Config(device, batch_max, max_width, max_height, batch_max * max_request_bytes,
                            0, flags)
        cfg.params = params
        cfg.n_consumers, cfg.batch_max, cfg.time_queue_us = int(n_consumers), int(batch_max), int(time_queue_us)
        cfg.max_request_bytes, cfg.queue_capacity = int(max_request_bytes), int(queue_capacity)
        if params.out_dtype == U8_NHWC:
            self._shape, self._dtype = (params.crop_h, params.crop_w, 3), np.uint8
        else:
            self._shape = (3, params.crop_h, params.crop_w)
            self._dtype = np.float16 if params.out_dtype == F16 else np.float32
        self._s = C.c_void_p()
        _check(lib().prep_server_create(C.byref(self._s), C.byref(cfg)), "prep_server_create")

    def submit(self, jpeg, tag):
        a, p = _u8(np.frombuffer(jpeg, dtype=np.uint8) if isinstance(jpeg, (bytes, bytearray)) else jpeg)
        return int(lib().prep_server_submit(self._s, p, a.size, int(tag)))

    def next(self, timeout_us=1000000):
        r = ServerResult()
        got = lib().prep_server_next(self._s, C.byref(r), int(timeout_us))
        if got < 0:
            raise PrepError(int(got), "prep_server_next")
        return r if got else None

    def next_many(self, results, timeout_us=1000000):
        """Fills `results` (a ctypes array of ServerResult) with finished requests; returns how many."""
        n = lib().prep_server_next_many(self._s, results, len(results), int(timeout_us))
        if n < 0:
            raise PrepError(int(n), "prep_server_next_many")
        return int(n)

    def release_many(self, results, n):
        _check(lib().prep_server_release_many(self._s, results, int(n)), "prep_server_release_many")

    def release(self, result):
        """The caller is done with the result's tensor (every result must be released)."""
        _check(lib().prep_server_release(self._s, C.byref(result)), "prep_server_release")

    def copy_tensor(self, result):
        out = np.empty(self._shape, dtype=self._dtype)
        _check(lib().prep_server_copy_tensor(self._s, C.byref(result), out.ctypes.data), "prep_server_copy_tensor")
        return out

    def close(self):
        if self._s:
            lib().prep_server_destroy(self._s)
            self._s = C.c_void_p()


class AudioPreprocessor:
    """prep_audio_*: resample -> log-Mel spectrogram -> per-feature normalize on the GPU."""

    def __init__(self, max_batch, max_total_samples, rate=16000, n_fft=512, win_length=400, hop=160, n_mels=80,
                 device=0):
        self.cfg = AudioConfig(device, max_batch, rate, n_fft, win_length, hop, n_mels, 0, max_total_samples)
        self._h = C.c_void_p()
        _check(lib().prep_audio_create(C.byref(self._h), C.byref(self.cfg)), "prep_audio_create")

    def frames(self, samples_in, rate_in):
        return int(lib().prep_audio_frames(C.byref(self.cfg), int(samples_in), int(rate_in)))

    def features(self, waveforms_ptr, offsets, rate_in, out_ptr, stream=0):
        """Enqueues the batch; returns the output offsets (elements) of the utterances."""
        o, op = _u64(offsets)
        out_offsets = np.zeros(len(o), dtype=np.uint64)
        _check(lib().prep_audio_features(self._h, C.c_void_p(waveforms_ptr), op, len(o) - 1, int(rate_in),
                                         C.c_void_p(out_ptr), out_offsets.ctypes.data_as(C.POINTER(C.c_uint64)),
                                         C.c_void_p(stream)), "prep_audio_features")
        return out_offsets

    def close(self):
        if self._h:
            lib().prep_audio_destroy(self._h)
            self._h = C.c_void_p()
