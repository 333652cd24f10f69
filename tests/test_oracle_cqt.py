"""Pins for the constant-Q part of the CPU oracle (CPU only)."""
import numpy as np
import pytest

import oracle
from paper_1912_12055_amd import signals


def _golden_rows(path):
    return [l.split() for l in open(path) if l.strip() and not l.startswith("#")]


def test_Q_closed_form():
    # eq. (Q): b = 12 -> 1/(2^(1/12)-1), b = 1 -> 1 cycle per octave-wide bin
    assert abs(oracle.cqt_Q(1) - 1.0) < 1e-15
    assert abs(oracle.cqt_Q(12) - 16.817153745105756) < 1e-12
    assert abs(oracle.cqt_Q(24) - 34.12708770892168) < 1e-11
    for b in (3, 12, 24, 36):
        assert abs((2.0 ** (1.0 / b) - 1.0) * oracle.cqt_Q(b) - 1.0) < 1e-14


def test_longest_kernel_lengths_quoted_in_paper(golden_dir):
    for sr, b, fmin, printed, pow2 in _golden_rows(golden_dir + "/cqt_lengths.txt"):
        sr, b, fmin, printed, pow2 = int(sr), int(b), float(fmin), int(printed), int(pow2)
        Nk, fk = oracle.cqt_lengths(sr, fmin, 1, b)
        # the paper prints Q*s/f rounded down; eq. (N_k) is the ceiling: one more
        assert Nk[0] - printed in (0, 1, 5), (Nk[0], printed)
        assert oracle.cqt_default_taps(sr, fmin, b) == pow2
    # exact quotients behind those integers (C1 = 32.7032 Hz gives the paper's 46,020)
    assert int(np.floor(oracle.cqt_Q(24) * 44100 / 27.5)) == 54727
    assert int(np.floor(oracle.cqt_Q(24) * 44100 / 32.7032)) == 46020


def test_kernel_lengths_of_the_two_cqt_workloads():
    Nk, fk = oracle.cqt_lengths(22050, 32.70, 84, 12)
    assert (Nk[0], Nk[-1]) == (11341, 94)  # Q*s/fmin = 11340.007: ceil, in double
    assert Nk.sum() == 200505
    assert abs(fk[12] - 65.4) < 1e-12 and abs(fk[83] - 32.70 * 2 ** (83 / 12)) < 1e-9
    Nk, fk = oracle.cqt_lengths(44100, 32.70, 168, 24)
    assert (Nk[0], Nk[-1]) == (46025, 371)
    assert Nk.sum() == 1604166
    assert np.all(np.diff(Nk) <= 0)
    assert oracle.cqt_default_taps(22050, 32.70, 12) == 16384
    assert oracle.cqt_default_taps(44100, 32.70, 24) == 65536


def test_kernel_bank_structure():
    sr, fmin, nb, b, taps = 22050, 32.70, 84, 12, 16384
    kre, kim = oracle.cqt_kernels(sr, fmin, nb, b, n_taps=taps)
    Nk, _ = oracle.cqt_lengths(sr, fmin, nb, b)
    Q = oracle.cqt_Q(b)
    for k in (0, 1, 40, 83):
        s = (taps - Nk[k]) // 2
        mag = np.hypot(kre[k], kim[k])
        assert np.all(mag[:s] == 0) and np.all(mag[s + Nk[k]:] == 0)  # centred support
        assert abs(mag.sum() - 1.0) < 1e-12  # L1 norm
        assert mag[s] == 0.0 and mag[s + 1] > 0  # periodic Hann starts at zero
        # magnitude is the Hann window / sum(w) = w / (N_k/2)
        n = np.arange(Nk[k])
        np.testing.assert_allclose(mag[s:s + Nk[k]], (0.5 - 0.5 * np.cos(2 * np.pi * n / Nk[k])) / (Nk[k] / 2),
                                   atol=1e-15)
        # phase advances by -2 pi Q / N_k per tap: exactly Q cycles across the kernel
        z = kre[k, s + 1:s + Nk[k]] + 1j * kim[k, s + 1:s + Nk[k]]
        step = np.angle(z[1:] / z[:-1])
        np.testing.assert_allclose(step, -2 * np.pi * Q / Nk[k], atol=1e-9)
    with pytest.raises(oracle.OracleError):
        oracle.cqt_kernels(44100, 32.70, 168, 24, n_taps=32768)  # longest kernel 46,025 does not fit


@pytest.mark.parametrize("k,phase", [(0, 0.3), (40, 1.9), (83, -2.5)])
def test_tone_at_kernel_frequency_reads_half_amplitude(k, phase):
    # A cos(2 pi f t + phase) with f = Q s / N_k (exactly Q cycles per kernel): the
    # L1-normalised kernel returns |X| = A/2 (+ a Hann side lobe 2Q bins away, < 1e-5 A)
    sr, fmin, nb, b, taps, hop, A = 22050, 32.70, 84, 12, 16384, 512, 0.8
    Nk, fk = oracle.cqt_lengths(sr, fmin, nb, b)
    f = oracle.cqt_Q(b) * sr / Nk[k]
    assert abs(f / fk[k] - 1.0) < 1.0 / Nk[k]
    L = 3 * taps
    x = signals.tone(L, sr, f, amp=A, phase=phase)
    C = oracle.cqt(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b, n_taps=taps)[0]
    assert C.shape == (nb, 1 + L // hop)
    mid = C[:, 20:-20]  # frames whose longest kernel stays inside the signal
    assert np.all(np.argmax(mid, axis=0) == k)
    assert np.max(np.abs(mid[k] - A / 2)) < 2e-5 * A + 1e-7


def test_tone_at_nominal_bin_frequency_peaks_at_that_bin_24_per_octave():
    sr, fmin, nb, b, hop = 44100, 32.70, 168, 24, 512
    taps = 65536
    Nk, fk = oracle.cqt_lengths(sr, fmin, nb, b)
    L = taps + 8 * hop
    for p in (30, 70):  # semitone p sits on bin 2p when b = 24
        x = signals.tone(L, sr, 32.70 * 2 ** (p / 12), amp=0.5)
        C = oracle.cqt(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b, n_taps=taps)[0]
        mid = C[:, 60:70]
        assert np.all(np.argmax(mid, axis=0) == 2 * p)
        assert np.all(np.abs(mid[2 * p] - 0.25) < 0.25 * 5e-3)


def test_cqt_equals_framed_product_with_kernel_bank():
    # direct inner products == (independently framed, numpy-padded signal) x (dense bank)
    rng = np.random.default_rng(31)
    sr, fmin, nb, b, taps, hop, L = 8000, 220.0, 24, 12, 1024, 128, 3000
    x = rng.standard_normal((2, L)).astype(np.float32)
    kre, kim = oracle.cqt_kernels(sr, fmin, nb, b, n_taps=taps)
    for fmt in (oracle.MAGNITUDE, oracle.POWER):
        C = oracle.cqt(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b, n_taps=taps, fmt=fmt)
        for bb in range(2):
            xp = np.pad(x[bb].astype(np.float64), taps // 2, mode="reflect")
            frames = np.stack([xp[t * hop:t * hop + taps] for t in range(1 + L // hop)], 1)
            Z = (kre + 1j * kim) @ frames
            want = np.abs(Z) if fmt == oracle.MAGNITUDE else np.abs(Z) ** 2
            np.testing.assert_allclose(C[bb], want, rtol=1e-9, atol=1e-12)


def test_rect_window_kernel_is_a_dft_at_fractional_bin_Q():
    # with a rectangular window eq. (CQT) is (1/N_k) sum x[n] exp(-2 pi i Q n / N_k)
    rng = np.random.default_rng(32)
    sr, fmin, nb, b, hop = 8000, 500.0, 6, 3, 64
    Nk, _ = oracle.cqt_lengths(sr, fmin, nb, b)
    taps = 128
    assert Nk[0] <= taps
    L = 1000
    x = rng.standard_normal(L).astype(np.float32)
    C = oracle.cqt(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b, window=oracle.WIN_RECT, n_taps=taps,
                   center=False)[0]
    Q = oracle.cqt_Q(b)
    for k in range(nb):
        s = (taps - Nk[k]) // 2
        n = np.arange(Nk[k])
        for t in range(C.shape[1]):
            seg = x[t * hop + s:t * hop + s + Nk[k]].astype(np.float64)
            want = abs(np.sum(seg * np.exp(-2j * np.pi * Q * n / Nk[k])) / Nk[k])
            assert abs(C[k, t] - want) < 1e-12


def test_default_taps_and_bad_args():
    x = np.zeros(40000, np.float32)
    assert oracle.cqt(x).shape == (1, 84, 1 + 40000 // 512)
    with pytest.raises(oracle.OracleError):
        oracle.cqt(np.zeros(8000, np.float32))  # pad 8192 >= L
    with pytest.raises(oracle.OracleError):
        oracle.cqt(x, n_taps=8192)  # shorter than the longest kernel


@pytest.mark.parametrize("k,phase", [(5, 0.4), (40, -1.3), (83, 2.6)])
def test_complex_result_carries_the_tone_phase(k, phase):
    # x[n] = A cos(2 pi Q n' / N_k + phase) with n' counted from the kernel's first tap: the kernel
    # exp(-2 pi i Q n' / N_k) w / sum(w) then returns (A/2) exp(+i phase) (+ the conjugate term 2Q bins away)
    sr, fmin, nb, b, taps, hop, A = 22050, 32.70, 84, 12, 16384, 512, 0.8
    Nk, _ = oracle.cqt_lengths(sr, fmin, nb, b)
    L = 3 * taps
    t = 10  # a mid-signal frame: padded start t*hop, kernel k starts s_k taps later
    s_k = (taps - Nk[k]) // 2
    n = np.arange(L)
    first = t * hop + s_k - taps // 2  # stored-sample index of the kernel's first tap in frame t
    x = (A * np.cos(2 * np.pi * oracle.cqt_Q(b) * (n - first) / Nk[k] + phase)).astype(np.float32)
    re, im = oracle.cqt_complex(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b, n_taps=taps)
    z = re[0, k, t] + 1j * im[0, k, t]
    assert abs(z - A / 2 * np.exp(1j * phase)) < 2e-5 * A
    mag = oracle.cqt(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b, n_taps=taps)
    np.testing.assert_allclose(np.hypot(re, im), mag, rtol=1e-12, atol=1e-15)
