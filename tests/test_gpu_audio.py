"""Parity of the GPU audio path (prep_audio_*, through the C ABI) with the numpy oracle:
normalised log-Mel features within FEATURE_TOL.  The kernels compute in double from the float32
samples to the logarithm and store float32 features: what remains is the rounding of a
log-Mel value of magnitude up to about 20 to float32 (1e-6) divided by a standard deviation
of order one, and the order of summation."""
import numpy as np
import pytest

from oracle import audio

pytestmark = pytest.mark.gpu

FEATURE_TOL = 2e-5


def speech_like(seed, rate, seconds):
    """Seeded stand-in for an utterance: a few drifting harmonics under a slow envelope plus
    low-pass noise, peak about 0.5."""
    rng = np.random.default_rng(seed)
    n = int(rate * seconds)
    t = np.arange(n) / rate
    f0 = 110.0 + 60.0 * rng.random() + 20.0 * np.sin(2 * np.pi * (0.7 + rng.random()) * t)
    phase = 2 * np.pi * np.cumsum(f0) / rate
    x = sum(rng.random() / (h ** 0.8) * np.sin(h * phase + rng.random() * 6.28) for h in range(1, 24))
    envelope = 0.55 + 0.45 * np.sin(2 * np.pi * 3.1 * t + rng.random() * 6.28)
    noise = np.convolve(rng.standard_normal(n + 15), np.hanning(16) / 8.0, mode="valid")
    x = x * envelope + 0.6 * noise
    return (0.5 * x / np.abs(x).max()).astype(np.float32)


@pytest.fixture(scope="module")
def prep():
    import paper_2411_19114_amd as p
    return p


def run(ap, waves, rate_in):
    import torch
    offsets = np.zeros(len(waves) + 1, dtype=np.uint64)
    np.cumsum([len(w) for w in waves], out=offsets[1:])
    dev = torch.from_numpy(np.concatenate(waves)).to("cuda:0")
    total = sum(ap.cfg.n_mels * ap.frames(len(w), rate_in) for w in waves)
    out = torch.full((total,), 777.0, dtype=torch.float32, device="cuda:0")
    oo = ap.features(dev.data_ptr(), offsets, rate_in, out.data_ptr(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    flat = out.cpu().numpy()
    assert int(oo[-1]) == total
    return [flat[int(oo[i]):int(oo[i + 1])].reshape(ap.cfg.n_mels, -1) for i in range(len(waves))]


@pytest.mark.parametrize("rate_in", [44100, 48000, 22050, 16000, 8000])
def test_features_match_the_oracle(prep, rate_in):
    waves = [speech_like(10 * rate_in % 997 + k, rate_in, sec) for k, sec in enumerate((0.9, 2.3, 1.0, 0.35, 3.1))]
    ap = prep.AudioPreprocessor(max_batch=8, max_total_samples=sum(len(w) for w in waves) * 3)
    try:
        got = run(ap, waves, rate_in)
        for w, g in zip(waves, got):
            ref = audio.preprocess(w.astype(np.float64), rate_in)
            assert g.shape == ref.shape
            assert np.isfinite(g).all()
            assert np.abs(g - ref).max() <= FEATURE_TOL
        # a second call on the same handle, other lengths, same rate pair
        again = run(ap, waves[::-1][:3], rate_in)
        for g, h in zip(again, got[::-1][:3]):
            assert np.array_equal(g, h)
    finally:
        ap.close()


def test_other_frame_parameters_and_many_short_utterances(prep):
    rate_in = 32000
    waves = [speech_like(300 + k, rate_in, 0.05 + 0.03 * k) for k in range(24)]
    ap = prep.AudioPreprocessor(max_batch=32, max_total_samples=400000, rate=16000, win_length=512, hop=128, n_mels=64)
    try:
        for w, g in zip(waves, run(ap, waves, rate_in)):
            ref = audio.preprocess(w.astype(np.float64), rate_in, rate=16000, win_length=512, hop=128, n_mels=64)
            assert g.shape == ref.shape and np.abs(g - ref).max() <= FEATURE_TOL
    finally:
        ap.close()


def test_long_utterance_rows_longer_than_the_register_cache(prep):
    rate = 16000
    w = speech_like(7, rate, 45.0)               # 4501 frames > 4096
    ap = prep.AudioPreprocessor(max_batch=1, max_total_samples=len(w))
    try:
        g, = run(ap, [w], rate)
        ref = audio.preprocess(w.astype(np.float64), rate)
        assert g.shape == ref.shape == (80, 4501)
        assert np.abs(g - ref).max() <= FEATURE_TOL
    finally:
        ap.close()


def test_argument_errors(prep):
    import torch
    ap = prep.AudioPreprocessor(max_batch=2, max_total_samples=20000)
    try:
        x = torch.zeros(20000, device="cuda:0")
        out = torch.zeros(80 * 200, device="cuda:0")
        ok = np.array([0, 4000, 8000], dtype=np.uint64)
        ap.features(x.data_ptr(), ok, 16000, out.data_ptr())
        torch.cuda.synchronize()
        with pytest.raises(prep.PrepError):      # an utterance of 200 samples cannot be centred
            ap.features(x.data_ptr(), np.array([0, 200], dtype=np.uint64), 16000, out.data_ptr())
        with pytest.raises(prep.PrepError):      # three utterances, max_batch two
            ap.features(x.data_ptr(), np.array([0, 3000, 6000, 9000], dtype=np.uint64), 16000, out.data_ptr())
        with pytest.raises(prep.PrepError):      # more samples than reserved
            ap.features(x.data_ptr(), np.array([0, 30000], dtype=np.uint64), 16000, out.data_ptr())
    finally:
        ap.close()
    with pytest.raises(prep.PrepError):
        prep.AudioPreprocessor(max_batch=1, max_total_samples=1000, n_fft=1024)
