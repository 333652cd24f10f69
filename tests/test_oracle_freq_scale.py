"""Pins for the re-spaced (linear / log) frequency axis of the STFT oracle (CPU only).

Checked against the values the paper prints for its worked example, numpy's FFT where the
re-spaced bins fall on integer multiples of s/N, closed forms of a windowed tone, and a
complex exponential sum written out here.
"""
import os

import numpy as np
import pytest

import oracle
from paper_1912_12055_amd import signals

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "freq_scale_linear.txt")


def _rows():
    out = []
    for line in open(GOLDEN):
        line = line.strip()
        if line and not line.startswith("#"):
            out.append([float(v) for v in line.split()])
    return out


def test_linear_sigma_matches_the_papers_worked_example():
    for k, sigma, f, stol, ftol in _rows():
        got = oracle.freq_sigma(oracle.FREQ_LINEAR, int(k), 50.0, 6000.0, 1025, 2048, 44100)
        assert abs(got - sigma) <= stol, (k, got, sigma)
        assert abs(got * 44100 / 2048 - f) <= ftol, (k, got * 44100 / 2048, f)
    # resolution improves from 21.53 Hz to 5.8 Hz
    step = oracle.freq_sigma(1, 1, 50.0, 6000.0, 1025, 2048, 44100) - oracle.freq_sigma(1, 0, 50.0, 6000.0, 1025, 2048, 44100)
    assert abs(step * 44100 / 2048 - 5.8) < 0.05


def test_log_sigma_is_geometric_between_the_two_frequencies():
    N, s, mu, fs, fe = 2048, 22050, 200, 55.0, 7040.0  # seven octaves
    sig = np.array([oracle.freq_sigma(oracle.FREQ_LOG, k, fs, fe, mu, N, s) for k in range(mu + 1)])
    assert abs(sig[0] * s / N - fs) < 1e-9
    assert abs(sig[mu] * s / N - fe) < 1e-8  # the bin just past the last one lands on f_e
    ratio = sig[1:] / sig[:-1]
    assert np.allclose(ratio, 2.0 ** (7.0 / mu), rtol=1e-12)
    # bin mu/7 is exactly one octave above the first
    assert mu % 7 != 0 or abs(sig[mu // 7] / sig[0] - 2.0) < 1e-12
    assert abs(sig[100] / sig[0] - 2.0 ** 3.5) < 1e-11


def test_plain_scale_is_identity():
    assert oracle.freq_sigma(oracle.FREQ_DFT, 37, 50.0, 6000.0, 1025, 2048, 44100) == 37.0


def test_integer_sigma_reduces_to_numpy_fft():
    # f_s = 0, f_e = s/2 and mu = N/2 bins put sigma(k) on the integers 0..N/2-1
    N, hop, s = 256, 64, 8000
    x = signals.batch(1, B=2, L=1500)
    sig = np.array([oracle.freq_sigma(oracle.FREQ_LINEAR, k, 0.0, s / 2, N // 2, N, s) for k in range(N // 2)])
    assert np.allclose(sig, np.arange(N // 2), atol=1e-12)
    re, im = oracle.stft_sigma_complex(x, sig, n_fft=N, hop=hop)
    w = 0.5 - 0.5 * np.cos(2 * np.pi * np.arange(N) / N)
    for b in range(2):
        xp = np.pad(x[b].astype(np.float64), N // 2, mode="reflect")
        T = 1 + (xp.size - N) // hop
        assert re.shape[2] == T
        for t in range(T):
            F = np.fft.rfft(xp[t * hop:t * hop + N] * w)
            assert np.allclose(re[b, :, t], F.real[:N // 2], atol=1e-9)
            assert np.allclose(im[b, :, t], F.imag[:N // 2], atol=1e-9)
    # and the scaled spectrogram built from the same parameters is that DFT's magnitude
    mag = oracle.stft_scaled(x, sr=s, n_fft=N, hop=hop, scale=oracle.FREQ_LINEAR, fmin=0.0, fmax=s / 2, freq_bins=N // 2)
    ref = oracle.stft(x, n_fft=N, hop=hop)
    assert np.allclose(mag, ref[:, :N // 2, :], atol=1e-9)


def test_non_integer_sigma_matches_complex_exponential_sum():
    N, hop = 128, 32
    rng = np.random.default_rng(5)
    x = rng.standard_normal((1, 700)).astype(np.float32)
    sig = np.array([0.0, 0.37, 2.5, 17.123, 63.9])
    re, im = oracle.stft_sigma_complex(x, sig, n_fft=N, hop=hop, window=oracle.WIN_RECT, center=False)
    n = np.arange(N)
    for t in range(re.shape[2]):
        seg = x[0, t * hop:t * hop + N].astype(np.float64)
        for i, sg in enumerate(sig):
            z = np.sum(seg * np.exp(-2j * np.pi * sg * n / N))
            assert abs(re[0, i, t] - z.real) < 1e-10 and abs(im[0, i, t] - z.imag) < 1e-10


@pytest.mark.parametrize("scale", [oracle.FREQ_LINEAR, oracle.FREQ_LOG])
def test_tone_at_a_bins_frequency_peaks_in_that_bin_with_half_the_window_sum(scale):
    # a tone placed exactly on bin k's (non-integer) frequency: |X| at that bin is A/2 * sum(w),
    # up to the leakage of the mirror-image component, and no other bin is larger
    N, hop, s, mu, fs, fe = 2048, 512, 22050, 300, 200.0, 4000.0
    A = 0.7
    for k in (17, 150, 288):
        f = oracle.freq_sigma(scale, k, fs, fe, mu, N, s) * s / N
        x = signals.tone(12000, s, f, amp=A)[None, :]
        out = oracle.stft_scaled(x, sr=s, n_fft=N, hop=hop, scale=scale, fmin=fs, fmax=fe, freq_bins=mu)
        mid = out[0, :, 6:-6]  # frames that see no reflected samples
        assert np.all(mid.argmax(axis=0) == k)
        assert np.allclose(mid[k], A / 2 * N / 2, rtol=2e-3)


def test_scaled_rejects_bad_ranges():
    x = signals.batch(1, B=1, L=3000)
    with pytest.raises(oracle.OracleError):
        oracle.stft_scaled(x, scale=oracle.FREQ_LOG, fmin=0.0, fmax=4000.0, freq_bins=64)
    with pytest.raises(oracle.OracleError):
        oracle.stft_scaled(x, scale=oracle.FREQ_LINEAR, fmin=500.0, fmax=400.0, freq_bins=64)
