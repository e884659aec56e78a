"""Build and run the CPU build of libprep (kernels compiled by g++ against the HIP
stand-in in tests/hip_emulation, one OS thread per lane, AddressSanitizer on).
It checks host logic and kernel indexing without a GPU; it is not the product."""
import os
import struct
import subprocess
import tempfile

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EMU = os.path.join(ROOT, "tests", "hip_emulation")
CSRC = os.path.join(ROOT, "paper_2411_19114_amd", "csrc")
BINARY = os.environ.get("PREP_EMUL_BIN", os.path.join(EMU, "prep_emul"))
KERNELS = ["entropy.hip", "reconstruct.hip", "resize.hip", "api.cpp", "parser.cpp"]


def build(force=False):
    srcs = [os.path.join(CSRC, k) for k in KERNELS] + \
           [os.path.join(EMU, "emul_runtime.cpp"), os.path.join(EMU, "emul_main.cpp")]
    deps = srcs + [os.path.join(CSRC, x) for x in ("kernels.h", "parser.h", "prep_internal.h")] + \
        [os.path.join(ROOT, "include", "prep.h"), os.path.join(EMU, "hip", "hip_runtime.h")]
    if not force and os.path.exists(BINARY) and \
            os.path.getmtime(BINARY) >= max(os.path.getmtime(d) for d in deps):
        return BINARY
    cmd = ["g++", "-std=c++20", "-O1", "-g", "-pthread", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-I", EMU, "-x", "c++"] + srcs + ["-o", BINARY]
    subprocess.run(cmd, check=True)
    return BINARY


def run(streams, resize_short, crop_h, crop_w, out_dtype, mean, std, timeout=600, flags=0, antialias=False):
    """-> list of (status, coef [nb,64] or None, rgb flat or None, rect), tensor [n,3,ch,cw];
    rect = (x0, y0, x1, y1), the pixels of the image that were converted to RGB."""
    build()
    n = len(streams)
    offsets = np.zeros(n + 1, dtype=np.uint64)
    np.cumsum([len(s) for s in streams], out=offsets[1:])
    f16 = out_dtype == "f16"
    code = {"f32": 0, "f16": 1, "u8": 2}[out_dtype]
    with tempfile.TemporaryDirectory() as d:
        fin, fout = os.path.join(d, "in.bin"), os.path.join(d, "out.bin")
        with open(fin, "wb") as f:
            f.write(struct.pack("<5i", n, resize_short, crop_h, crop_w, code))
            f.write(struct.pack("<6f", *mean, *std))
            f.write(offsets.tobytes())
            f.write(b"".join(streams))
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", PREP_EMUL_FLAGS=str(int(flags)),
                   PREP_EMUL_FILTER="1" if antialias else "0")
        r = subprocess.run([BINARY, fin, fout], capture_output=True, text=True, timeout=timeout,
                           env=env)
        if os.environ.get("PREP_EMUL_VERBOSE") and r.stderr:
            print(r.stderr[-6000:])
        if r.returncode != 0:
            raise RuntimeError(f"prep_emul exit {r.returncode}\n{r.stderr[-4000:]}")
        blob = open(fout, "rb").read()
    pos = 0
    per_image = []
    for _ in range(n):
        status, = struct.unpack_from("<i", blob, pos); pos += 4
        nc, = struct.unpack_from("<q", blob, pos); pos += 8
        coef = np.frombuffer(blob, dtype=np.int16, count=nc, offset=pos).reshape(-1, 64) if nc else None
        pos += 2 * nc
        rect = struct.unpack_from("<4i", blob, pos); pos += 16
        nr, = struct.unpack_from("<q", blob, pos); pos += 8
        rgb = np.frombuffer(blob, dtype=np.uint8, count=nr, offset=pos) if nr else None
        pos += nr
        per_image.append((status, coef, rgb, rect))
    if out_dtype == "u8":
        return per_image, np.frombuffer(blob, dtype=np.uint8, offset=pos).reshape(n, crop_h, crop_w, 3)
    dt = np.float16 if f16 else np.float32
    tensor = np.frombuffer(blob, dtype=dt, offset=pos).reshape(n, 3, crop_h, crop_w)
    return per_image, tensor
