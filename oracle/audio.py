"""CPU oracle (test infrastructure): the audio preprocessing path of PREBA (section 2.3 item
b and Fig. 4(b): resampling, Fourier transform, Mel filters; section 4.2, Fig. 11(b) and
Table 1: the Resample, Mel spectrogram and Normalize units) in plain numpy, float64.

The paper names the operations and nothing else.  The definitions taken here (listed as
readings in the design notes):
  resample      band-limited interpolation with a Hann-windowed sinc, six zero crossings wide,
                cut-off at 0.99 of the lower Nyquist rate
  spectrogram   frames of n_fft samples every hop samples, the signal extended by reflection
                so that frame t is centred on sample t * hop; periodic Hann window of win_length
                samples centred in the frame; squared magnitude of the DFT, bins 0 .. n_fft/2
  Mel filters   n_mels triangles whose corners are equally spaced on the scale
                m(f) = 2595 log10(1 + f / 700) between f_min and f_max, unit peak
  logarithm     ln(value + 2^-24)
  normalize     per Mel channel over the frames of one utterance: mean, variance (the mean of
                the squared deviations), then (x - mean) / (sqrt(variance) + 1e-5); the
                three sub-steps of the paper's Normalize unit (section 4.2)

Only tests and the benchmark's comparison leg may import this module.
"""
from math import gcd

import numpy as np

ZERO_CROSSINGS = 6
ROLLOFF = 0.99
LOG_GUARD = 2.0 ** -24
STD_GUARD = 1e-5


def resample(x, rate_in, rate_out):
    """y[m] = sum_n x[n] h(n / rate_in - m / rate_out), m = 0 .. ceil(len * rate_out / rate_in) - 1,
    h(t) = (B / rate_in) sinc(B t) cos^2(pi B t / (2 W)) for |B t| < W, else 0,
    B = ROLLOFF * min(rate_in, rate_out), W = ZERO_CROSSINGS, sinc(u) = sin(pi u) / (pi u)."""
    x = np.asarray(x, dtype=np.float64)
    g = gcd(int(rate_in), int(rate_out))
    p, q = int(rate_in) // g, int(rate_out) // g      # only the ratio matters
    if p == q:
        return x.copy()
    base = ROLLOFF * min(p, q)
    n_out = -(-len(x) * q // p)
    reach = ZERO_CROSSINGS / base                     # half width of h in time (units: 1 = p samples in)
    y = np.zeros(n_out)
    for m in range(n_out):
        centre = m / q                                # time of output m
        lo = int(np.ceil((centre - reach) * p))
        hi = int(np.floor((centre + reach) * p))
        n = np.arange(max(lo, 0), min(hi, len(x) - 1) + 1)
        u = base * (n / p - centre)
        inside = np.abs(u) < ZERO_CROSSINGS
        h = (base / p) * np.sinc(u) * np.cos(np.pi * u / (2 * ZERO_CROSSINGS)) ** 2 * inside
        y[m] = np.dot(x[n], h)
    return y


def hann_periodic(n):
    return 0.5 - 0.5 * np.cos(2.0 * np.pi * np.arange(n) / n)


def power_spectrogram(x, n_fft, win_length, hop):
    """[n_fft/2 + 1, 1 + len // hop]: |DFT|^2 of the windowed frames."""
    x = np.asarray(x, dtype=np.float64)
    half = n_fft // 2
    assert len(x) > half, "reflection needs more than n_fft/2 samples"
    padded = np.concatenate([x[half:0:-1], x, x[-2:-half - 2:-1]])
    window = np.zeros(n_fft)
    left = (n_fft - win_length) // 2
    window[left:left + win_length] = hann_periodic(win_length)
    n_frames = 1 + len(x) // hop
    out = np.empty((half + 1, n_frames))
    for t in range(n_frames):
        frame = padded[t * hop:t * hop + n_fft] * window
        out[:, t] = np.abs(np.fft.rfft(frame)) ** 2
    return out


def mel_of_hz(f):
    return 2595.0 * np.log10(1.0 + np.asarray(f, dtype=np.float64) / 700.0)


def hz_of_mel(m):
    return 700.0 * (10.0 ** (np.asarray(m, dtype=np.float64) / 2595.0) - 1.0)


def mel_filters(n_mels, n_fft, rate, f_min=0.0, f_max=None):
    """[n_mels, n_fft/2 + 1] triangular weights with unit peak."""
    f_max = rate / 2.0 if f_max is None else f_max
    corners = hz_of_mel(np.linspace(mel_of_hz(f_min), mel_of_hz(f_max), n_mels + 2))
    bins = np.arange(n_fft // 2 + 1) * rate / n_fft
    fb = np.zeros((n_mels, len(bins)))
    for m in range(n_mels):
        lo, mid, hi = corners[m], corners[m + 1], corners[m + 2]
        up = (bins - lo) / (mid - lo)
        down = (hi - bins) / (hi - mid)
        fb[m] = np.maximum(0.0, np.minimum(up, down))
    return fb


def log_mel(x, rate, n_fft=512, win_length=400, hop=160, n_mels=80):
    """[n_mels, frames]: ln(Mel filters applied to the power spectrogram + 2^-24)."""
    return np.log(mel_filters(n_mels, n_fft, rate) @ power_spectrogram(x, n_fft, win_length, hop) + LOG_GUARD)


def normalize_features(f):
    """Per row (Mel channel): mean over the frames, variance as the mean squared deviation,
    then (x - mean) / (sqrt(variance) + STD_GUARD)."""
    f = np.asarray(f, dtype=np.float64)
    mean = f.mean(axis=1, keepdims=True)
    var = ((f - mean) ** 2).mean(axis=1, keepdims=True)
    return (f - mean) / (np.sqrt(var) + STD_GUARD)


def preprocess(x, rate_in, rate=16000, n_fft=512, win_length=400, hop=160, n_mels=80):
    """Whole path for one utterance: resample -> log-Mel spectrogram -> normalize."""
    return normalize_features(log_mel(resample(x, rate_in, rate), rate, n_fft, win_length, hop, n_mels))
