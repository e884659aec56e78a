"""Seeded synthetic inputs for the JPEG -> tensor preprocessing path.

This module only *produces inputs*: RGB images drawn from numpy's seeded
generator, compressed to baseline JPEG by an independent third-party encoder
(Pillow / libjpeg).  It holds none of the decode / resize / normalize
arithmetic and imports neither the GPU library nor the CPU oracle, so both
sides can be fed the very same bytes.

The five workloads stand in for the photographs of the ImageNet validation set
used in PREBA's evaluation (section 5, "Benchmarks"): a few-hundred-pixel photo
size range, full-HD frames, and photo-like entropy (2-3 bit/pixel) from additive
Gaussian noise on smooth content.
"""
import hashlib
import io

import numpy as np

MODE_444, MODE_420, MODE_GRAY, MODE_422 = 0, 1, 2, 3

IMAGENET_MEAN = (0.485, 0.456, 0.406)
IMAGENET_STD = (0.229, 0.224, 0.225)


def image_seed(config, index):
    return 1000 * config + index


def gradient_noise_image(rng, w, h, sigma=8.0):
    """Per channel a + bx*x/W + by*y/H plus i.i.d. N(0, sigma^2), rounded and clipped."""
    x = np.arange(w, dtype=np.float64)[None, :] / w
    y = np.arange(h, dtype=np.float64)[:, None] / h
    img = np.empty((h, w, 3), dtype=np.float64)
    for c in range(3):
        a = rng.uniform(48.0, 208.0)
        bx = rng.uniform(-48.0, 48.0)
        by = rng.uniform(-48.0, 48.0)
        img[:, :, c] = a + bx * x + by * y
    img += rng.normal(0.0, sigma, size=img.shape)
    return np.clip(np.rint(img), 0, 255).astype(np.uint8)


def shapes_image(rng, w, h, sigma=6.0):
    """Random background, 5-15 filled rectangles / ellipses, Gaussian blur, noise."""
    from scipy.ndimage import gaussian_filter1d
    img = np.empty((h, w, 3), dtype=np.float64)
    img[:] = rng.uniform(0.0, 255.0, size=3)
    yy, xx = np.ogrid[0:h, 0:w]
    for _ in range(int(rng.integers(5, 16))):
        colour = rng.uniform(0.0, 255.0, size=3)
        cx, cy = rng.uniform(0, w), rng.uniform(0, h)
        rx, ry = rng.uniform(0.05, 0.35) * w, rng.uniform(0.05, 0.35) * h
        if rng.random() < 0.5:
            mask = (np.abs(xx - cx) <= rx) & (np.abs(yy - cy) <= ry)
        else:
            mask = ((xx - cx) / rx) ** 2 + ((yy - cy) / ry) ** 2 <= 1.0
        img[mask] = colour
    blur = rng.uniform(1.0, 3.0)
    img = gaussian_filter1d(img, blur, axis=0, mode="nearest")
    img = gaussian_filter1d(img, blur, axis=1, mode="nearest")
    img += rng.normal(0.0, sigma, size=img.shape)
    return np.clip(np.rint(img), 0, 255).astype(np.uint8)


def encode_jpeg(rgb, quality, mode, restart_blocks=0, restart_rows=0, optimize=False):
    """Baseline JPEG bytes of an RGB8 image via Pillow (libjpeg): standard Annex-K
    Huffman tables unless ``optimize`` (then per-image tables)."""
    from PIL import Image
    im = Image.fromarray(rgb, "RGB")
    kw = dict(quality=int(quality), optimize=bool(optimize), progressive=False)
    if restart_blocks:
        kw["restart_marker_blocks"] = int(restart_blocks)
    if restart_rows:
        kw["restart_marker_rows"] = int(restart_rows)
    if mode == MODE_GRAY:
        im = im.convert("L")
    else:
        kw["subsampling"] = {MODE_444: 0, MODE_422: 1, MODE_420: 2}[mode]
    buf = io.BytesIO()
    im.save(buf, "JPEG", **kw)
    return buf.getvalue()


# name -> recipe.  Sizes: fixed (w, h) or ranges; "restart": ("rows", n) | ("blocks", n) | None
CONFIGS = {
    1: dict(n=64, size=(256, 256), content="gradient", sigma=8.0, quality=85, modes=(MODE_420,),
            restart=("rows", 1), resize_short=256, crop=224, out_dtype="f32"),
    2: dict(n=256, size=((300, 640), (250, 500)), content="shapes", sigma=6.0, quality=90,
            modes=(MODE_420,), restart=("blocks", 8), resize_short=256, crop=224,
            out_dtype="f16"),
    4: dict(n=64, size=(1920, 1080), content="shapes", sigma=6.0, quality=95, modes=(MODE_420,),
            restart=("rows", 1), resize_short=384, crop=384, out_dtype="f16"),
    5: dict(n=512, size=(256, 256), content="gradient", sigma=8.0, quality=(50, 95),
            modes=(MODE_444, MODE_420, MODE_GRAY), restart=None, resize_short=256, crop=224,
            out_dtype="f16"),
}
# workload 3 draws its batches of 8 from a pool of workload-1 images
CONFIGS[3] = dict(CONFIGS[1], n=512)


def make_image(config, index):
    """(jpeg bytes, rgb source image) of image ``index`` of workload ``config``."""
    r = CONFIGS[config]
    # workload 3 shares workload 1's distribution but not its seeds
    rng = np.random.default_rng(image_seed(config, index))
    size = r["size"]
    if isinstance(size[0], tuple):
        w = int(rng.integers(size[0][0], size[0][1] + 1))
        h = int(rng.integers(size[1][0], size[1][1] + 1))
    else:
        w, h = size
    rgb = (gradient_noise_image if r["content"] == "gradient" else shapes_image)(
        rng, w, h, r["sigma"])
    q = r["quality"]
    if isinstance(q, tuple):
        q = int(rng.integers(q[0], q[1] + 1))
    mode = r["modes"][index % len(r["modes"])]
    kw = {}
    if r["restart"]:
        kw["restart_" + r["restart"][0]] = r["restart"][1]
    # every eighth image carries Huffman tables optimised for itself
    data = encode_jpeg(rgb, q, mode, optimize=(index % 8 == 5), **kw)
    return data, rgb


def make_batch(config, n=None, first=0):
    """List of JPEG byte strings for images first..first+n-1 of a workload."""
    n = CONFIGS[config]["n"] if n is None else n
    return [make_image(config, first + i)[0] for i in range(n)]


def params_of(config):
    r = CONFIGS[config]
    return dict(resize_short=r["resize_short"], crop_h=r["crop"], crop_w=r["crop"],
                out_dtype=r["out_dtype"], mean=IMAGENET_MEAN, std=IMAGENET_STD)


def pack(streams):
    """Concatenate byte strings -> (uint8 array, uint64 offsets of length n+1)."""
    offsets = np.zeros(len(streams) + 1, dtype=np.uint64)
    np.cumsum([len(s) for s in streams], out=offsets[1:])
    blob = np.frombuffer(b"".join(streams), dtype=np.uint8).copy()
    return blob, offsets


def sha256_of(streams):
    h = hashlib.sha256()
    for s in streams:
        h.update(s)
    return h.hexdigest()
