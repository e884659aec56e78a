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


def oracle_batch(streams, resize_short, crop_h, crop_w, workers=8):
    """[(coef, rgb, info, tensor float64)] for every stream, computed by the oracle."""
    def one(s):
        coef, rgb, info = oracle.decode(s)
        ten = oracle.preprocess(rgb, resize_short, crop_h, crop_w, MEAN, STD)
        return coef, rgb, info, ten
    with ThreadPoolExecutor(workers) as ex:
        return list(ex.map(one, streams))


def run_gpu(pp, streams, resize_short, crop_h, crop_w, out_dtype, resident=False):
    import torch
    from paper_2411_19114_amd.binding import make_params
    blob, offsets = synth.pack(streams)
    params = make_params(resize_short, crop_h, crop_w, out_dtype, MEAN, STD)
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
                         check_intermediates=True):
    status, got = run_gpu(pp, streams, resize_short, crop_h, crop_w, out_dtype, resident)
    assert status == [0] * len(streams), status
    ref = oracle_batch(streams, resize_short, crop_h, crop_w)
    n_values = n_exact = 0
    for i, (coef, rgb, info, ten) in enumerate(ref):
        if check_intermediates:
            mine = pp.debug_last_coefficients(i, coef.shape[0])
            assert np.array_equal(mine, coef), f"image {i}: entropy-decoded coefficients differ"
            d = np.abs(pp.debug_last_rgb(i, info.height, info.width).astype(np.int32) - rgb.astype(np.int32))
            assert d.max() <= RGB_MAX_LSB, f"image {i}: RGB off by {d.max()} LSB"
            n_values += d.size
            n_exact += int((d == 0).sum())
        err = np.abs(got[i] - ten).max()
        assert err <= TENSOR_ABS_TOL, f"image {i}: tensor off by {err}"
    if check_intermediates:
        assert n_exact >= RGB_EXACT_FRACTION * n_values, f"only {n_exact / n_values:.5f} of RGB exact"
    return got
