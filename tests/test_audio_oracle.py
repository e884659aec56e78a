"""Pins of the audio oracle (oracle/audio.py): what the definitions fix without running them
(tones, impulses, Parseval, the brute-force DFT, partition of unity of the Mel triangles,
moments after normalisation) and an independent resampler on band-limited signals."""
import numpy as np
import pytest
from scipy import signal

from oracle import audio


def _tone(freq, rate, n, phase=0.3):
    return np.sin(2 * np.pi * freq * np.arange(n) / rate + phase)


@pytest.mark.parametrize("rates", [(44100, 16000), (48000, 16000), (22050, 16000), (8000, 16000), (16000, 22050)])
def test_resampling_keeps_a_tone_below_the_cut_off(rates):
    rin, rout = rates
    x = _tone(440.0, rin, rin // 4)
    y = audio.resample(x, rin, rout)
    assert len(y) == -(-len(x) * rout // rin)
    want = _tone(440.0, rout, len(y))
    edge = 200
    assert np.abs(y[edge:-edge] - want[edge:-edge]).max() < 2e-3


def test_resampling_removes_what_the_new_rate_cannot_carry():
    x = _tone(12000.0, 44100, 11025)            # above the 8 kHz Nyquist of the output
    y = audio.resample(x, 44100, 16000)
    assert np.abs(y[200:-200]).max() < 10 ** (-40 / 20)
    z = audio.resample(_tone(5000.0, 44100, 11025), 44100, 16000)   # well below: kept
    assert np.abs(z[200:-200]).max() > 0.97


def test_resampling_special_cases():
    x = np.random.default_rng(1).standard_normal(500)
    assert np.array_equal(audio.resample(x, 16000, 16000), x)
    assert np.array_equal(audio.resample(x, 32000, 32000), x)
    c = audio.resample(np.ones(3000), 44100, 16000)
    assert np.abs(c[100:-100] - 1.0).max() < 2e-3                # unit gain at 0 Hz
    # linear in the signal
    a, b = x, np.roll(x, 7)
    assert np.allclose(audio.resample(2 * a - 3 * b, 48000, 16000),
                       2 * audio.resample(a, 48000, 16000) - 3 * audio.resample(b, 48000, 16000))


def _series_sin_cos(x, terms=40):
    """sin and cos of the exact rational x by their power series in exact rational arithmetic."""
    from fractions import Fraction
    s, c, t = Fraction(0), Fraction(0), Fraction(1)
    for k in range(terms):
        if k % 2 == 0:
            c += t if k % 4 == 0 else -t
        else:
            s += t if k % 4 == 1 else -t
        t = t * x / (k + 1)
    return s, c


@pytest.mark.parametrize("rates,n0", [((44100, 16000), 300), ((8000, 16000), 40), ((48000, 16000), 123)])
def test_resampling_an_impulse_gives_the_kernel_itself(rates, n0):
    # a unit impulse at input sample n0 comes out as h(n0 / rate_in - m / rate_out): evaluated
    # here in exact rational arithmetic (power series of sin and cos, pi to 40 digits), so the
    # band edge, the gain, the time alignment of the two grids and the extent of the window
    # are all held to rounding error
    from fractions import Fraction
    rin, rout = rates
    pi = Fraction("3.1415926535897932384626433832795028841972")
    x = np.zeros(2 * n0 + 1)
    x[n0] = 1.0
    y = audio.resample(x, rin, rout)
    band = Fraction(99, 100) * min(rin, rout)      # 0.99 of the lower rate
    zeros = 6                                        # zero crossings kept each side
    worst, inside = 0.0, 0
    for m in range(len(y)):
        u = band * (Fraction(n0, rin) - Fraction(m, rout))
        if abs(u) >= zeros:
            assert y[m] == 0.0
            continue
        inside += 1
        if u == 0:
            sinc = Fraction(1)
        else:
            # reduce pi u to within pi of zero: sin(a + k pi) = (-1)^k sin(a)
            k = round(u)
            sn, _ = _series_sin_cos(pi * (u - k))
            sinc = (-sn if k % 2 else sn) / (pi * u)
        _, cw = _series_sin_cos(pi * u / (2 * zeros))
        want = band / rin * sinc * cw * cw
        worst = max(worst, abs(y[m] - float(want)))
    assert worst < 1e-12
    # the window spans 2 * 6 / (0.99 min(rate)) seconds of output samples
    assert abs(inside - 2 * zeros * rout / float(band)) <= 1


def test_resampling_agrees_with_a_polyphase_resampler_on_band_limited_noise():
    rng = np.random.default_rng(2)
    spec = np.zeros(2049, dtype=complex)
    spec[5:300] = rng.standard_normal(295) + 1j * rng.standard_normal(295)   # < 3.3 kHz of 22.05 kHz
    x = np.fft.irfft(spec)
    x /= np.abs(x).max()
    mine = audio.resample(x, 44100, 16000)
    theirs = signal.resample_poly(x, 160, 441, window=("kaiser", 12.0))
    n = min(len(mine), len(theirs))
    assert np.abs(mine[300:n - 300] - theirs[300:n - 300]).max() < 5e-3


def test_frames_are_centred_and_reflected():
    n_fft, win, hop = 64, 48, 16
    x = np.zeros(400)
    x[5 * hop] = 1.0
    p = audio.power_spectrogram(x, n_fft, win, hop)
    assert p.shape == (n_fft // 2 + 1, 1 + len(x) // hop)
    # an impulse at the centre of frame 5 meets the window's peak (1): a flat unit spectrum
    assert np.allclose(p[:, 5], 1.0)
    assert np.all(p[:, 5] >= p[:, 4]) and np.all(p[:, 5] >= p[:, 6])
    # frame 0 sees the reflection of the signal's start
    y = np.arange(1.0, 101.0)
    first = np.pad(y, n_fft // 2, mode="reflect")[:n_fft]
    w = np.zeros(n_fft)
    w[8:56] = audio.hann_periodic(48)
    assert np.allclose(audio.power_spectrogram(y, n_fft, win, hop)[:, 0], np.abs(np.fft.rfft(first * w)) ** 2)


def test_spectrum_is_the_dft_by_brute_force_and_obeys_parseval():
    rng = np.random.default_rng(3)
    n_fft, win, hop = 32, 32, 8
    x = rng.standard_normal(200)
    p = audio.power_spectrogram(x, n_fft, win, hop)
    padded = np.pad(x, n_fft // 2, mode="reflect")
    t = 7
    frame = padded[t * hop:t * hop + n_fft] * audio.hann_periodic(n_fft)
    k = np.arange(n_fft // 2 + 1)[:, None]
    n = np.arange(n_fft)[None, :]
    dft = (frame[None, :] * np.exp(-2j * np.pi * k * n / n_fft)).sum(axis=1)
    assert np.allclose(p[:, t], np.abs(dft) ** 2)
    # Parseval: bins 1 .. n/2-1 stand for two conjugate bins each
    total = p[0, t] + p[-1, t] + 2 * p[1:-1, t].sum()
    assert np.isclose(total, n_fft * (frame ** 2).sum())


def test_a_tone_on_a_bin_peaks_there():
    rate, n_fft = 16000, 512
    k = 37
    p = audio.power_spectrogram(_tone(k * rate / n_fft, rate, 4000), n_fft, 400, 160)
    assert (p[:, 3:-3].argmax(axis=0) == k).all()


def test_mel_scale_and_triangles():
    assert abs(audio.mel_of_hz(1000.0) - 1000.0) < 0.05           # the scale's anchor: 1000 Hz ~ 1000 mel
    f = np.array([0.0, 123.0, 4000.0, 7999.0])
    assert np.allclose(audio.hz_of_mel(audio.mel_of_hz(f)), f)
    fb = audio.mel_filters(80, 512, 16000)
    assert fb.shape == (80, 257) and fb.min() >= 0.0 and fb.max() <= 1.0
    corners = audio.hz_of_mel(np.linspace(0.0, audio.mel_of_hz(8000.0), 82))
    bins = np.arange(257) * 16000 / 512
    inside = (bins >= corners[1]) & (bins <= corners[80])
    # between the first and the last peak the triangles add up to one
    assert np.allclose(fb[:, inside].sum(axis=0), 1.0)
    # triangle m is zero outside its corners and peaks between them
    for m in (0, 17, 79):
        outside = (bins <= corners[m]) | (bins >= corners[m + 2])
        assert np.all(fb[m, outside] == 0.0)
        assert abs(bins[fb[m].argmax()] - corners[m + 1]) <= 16000 / 512
    # centres are equally spaced in mel
    assert np.allclose(np.diff(audio.mel_of_hz(corners)), audio.mel_of_hz(8000.0) / 81)


def test_log_guard_and_normalisation():
    silent = audio.log_mel(np.zeros(2000), 16000)
    assert np.allclose(silent, np.log(2.0 ** -24))
    rng = np.random.default_rng(4)
    f = rng.standard_normal((5, 300)) * np.array([[1.0], [10.0], [0.1], [3.0], [0.0]]) + 7.0
    g = audio.normalize_features(f)
    assert np.allclose(g.mean(axis=1), 0.0, atol=1e-12)
    assert np.allclose(g[:4].std(axis=1), 1.0, atol=2e-4)          # population moments, guard 1e-5
    assert np.all(g[4] == 0.0)                                     # a constant channel
    # (x - mean) / (std + guard) written out for one element
    assert np.isclose(g[1, 5], (f[1, 5] - f[1].mean()) / (np.sqrt(((f[1] - f[1].mean()) ** 2).mean()) + 1e-5))


def test_whole_path_shape_and_level_invariance():
    x = np.random.default_rng(5).standard_normal(22050)
    a = audio.preprocess(x, 22050)
    assert a.shape == (80, 1 + 16000 // 160)
    # scaling the waveform shifts every log-Mel value by the same amount, which the
    # normalisation removes
    b = audio.preprocess(4.0 * x, 22050)
    assert np.abs(a - b).max() < 1e-3
