"""Pins for the oracle's constant-Q transforms with frequency-domain kernels (CPU only): the one-rate
transform and, at the end, the recursive-downsampling form built on it.

Sec. III-C, "CQT using neural networks": eqs. (Parseval), (CQT1992), Figs. 4 and 5.  The pins do
not re-run the oracle's own steps: frames are cut here with numpy's padding, spectra are taken
with explicit O(N^2) sums or numpy's FFT on those frames, and the time-domain CQT the result is
compared with is the separately pinned direct-inner-product oracle.
"""
import numpy as np
import pytest
import scipy.signal

import oracle
from paper_1912_12055_amd import signals


def _frames(x, n_fft, hop):
    xp = np.pad(x.astype(np.float64), n_fft // 2, mode="reflect")
    T = 1 + x.size // hop
    return np.stack([xp[t * hop:t * hop + n_fft] for t in range(T)])


def test_spectral_kernels_peak_at_the_bin_frequency_with_unit_height():
    # Fig. 4 set-up: A3 (220 Hz) upwards, 12 bins per octave, 8 kHz.  Kernel q is a windowed complex
    # exponential of frequency Q s / N_q, L1-normalised: its spectrum peaks at DFT bin f N / s, with
    # height sum(w)/sum(w) = 1 where that bin is an integer and >= 0.84 (Hann main lobe half a bin
    # off) elsewhere, and is negligible in the half of the spectrum that is dropped.
    sr, fmin, nb, b = 8000, 220.0, 49, 12
    N = oracle.cqt_default_taps(sr, fmin, b)
    Nk, fk = oracle.cqt_lengths(sr, fmin, nb, b)
    Y = oracle.cqt1992_spectral_kernels(sr, fmin, nb, b)
    assert Y.shape == (nb, N // 2 + 1)
    Q = oracle.cqt_Q(b)
    for q in range(nb):
        mag = np.abs(Y[q])
        k_peak = int(np.argmax(mag))
        k_true = Q * N / Nk[q]  # the kernel's frequency in DFT bins
        assert abs(k_peak - k_true) <= 0.5 + 1e-9
        # resolution ratio: one bin of the kernel's own length-N_q DFT = N / N_q bins here
        assert 0.84 < mag[k_peak] <= 1.0 + 1e-12
    # the full spectrum, for the dropped half
    kre, kim = oracle.cqt_kernels(sr, fmin, nb, b, n_taps=N)
    full = np.fft.fft(kre - 1j * kim, axis=1)
    # (for kernels in the lower half of the band; the Hann side lobes of those close to the Nyquist
    # frequency reach across it)
    low = fk < sr / 4
    assert low.sum() >= 36
    assert np.abs(full[low, N // 2 + 1:]).max() < 1e-3
    np.testing.assert_allclose(np.conj(full[:, :N // 2 + 1]), Y, atol=1e-14)


def test_tiny_case_against_explicit_sums():
    # brute force, no FFT anywhere: N = 64 taps, 5 bins; X[k] and B[k] by their defining sums
    sr, fmin, nb, b, N, hop = 1000, 100.0, 5, 3, 64, 16
    assert oracle.cqt_default_taps(sr, fmin, b) == N
    x = signals.batch(3, B=1, L=150)[0]
    Nk, _ = oracle.cqt_lengths(sr, fmin, nb, b)
    Q = oracle.cqt_Q(b)
    fr = _frames(x, N, hop)
    n = np.arange(N)
    want = np.zeros((nb, fr.shape[0]))
    for q in range(nb):
        s = (N - Nk[q]) // 2
        m = np.arange(Nk[q])
        w = 0.5 - 0.5 * np.cos(2 * np.pi * m / Nk[q])
        kc = np.zeros(N, dtype=complex)  # conj of eq. (CQT)'s kernel, centred
        kc[s:s + Nk[q]] = w / w.sum() * np.exp(+2j * np.pi * Q * m / Nk[q])
        for t in range(fr.shape[0]):
            acc = 0.0
            for k in range(N // 2 + 1):
                e = np.exp(-2j * np.pi * k * n / N)
                acc += np.sum(fr[t] * e) * np.conj(np.sum(kc * e))
            want[q, t] = abs(acc) / N
    got = oracle.cqt1992(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b)[0]
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-13)


@pytest.mark.parametrize("sr,fmin,nb,b,hop,small", [(22050, 220.0, 36, 12, 256, 2e-4), (8000, 110.0, 30, 6, 128, 5e-3)])
def test_differs_from_the_time_domain_cqt_by_the_dropped_half_only(sr, fmin, nb, b, hop, small):
    # Parseval over all N bins is exact, so  X_time - X_1992 = (1/N) sum_{k > N/2} X[k] conj(B[k]).
    # Checked as complex numbers per (bin, frame) against numpy's FFT of frames cut here -- and the
    # remainder must be small, or "approximated CQT" would not describe it (it grows as Q falls and
    # as the top bin nears the Nyquist frequency: second case, Q = 8.2, top bin at 0.78 Nyquist).
    N = oracle.cqt_default_taps(sr, fmin, b)
    x = signals.batch(3, B=1, L=3 * N + 77)[0]
    fr = _frames(x, N, hop)
    X = np.fft.fft(fr, axis=1)  # [T, N]
    kre, kim = oracle.cqt_kernels(sr, fmin, nb, b, n_taps=N)
    Bq = np.fft.fft(kre - 1j * kim, axis=1)  # [nb, N]
    kept = (X[:, :N // 2 + 1] @ np.conj(Bq[:, :N // 2 + 1]).T).T / N  # [nb, T]
    dropped = (X[:, N // 2 + 1:] @ np.conj(Bq[:, N // 2 + 1:]).T).T / N
    got = oracle.cqt1992(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b)[0]
    time_domain = oracle.cqt(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b)[0]
    peak = time_domain.max()
    np.testing.assert_allclose(got, np.abs(kept), atol=1e-12 * peak)
    # the complex output is that kept sum itself (rows 2q = Re, 2q+1 = Im), the phase output its argument
    cplx = oracle.cqt1992(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b, fmt=oracle.COMPLEX)[0]
    np.testing.assert_allclose(cplx[0::2] + 1j * cplx[1::2], kept, atol=1e-12 * peak)
    tre, tim = oracle.cqt_complex(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b)
    np.testing.assert_allclose(tre[0] + 1j * tim[0], kept + dropped, atol=1e-11 * peak)
    ph = oracle.cqt1992(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b, fmt=oracle.PHASE)[0]
    strong = np.abs(kept) > 1e-3 * peak
    assert np.abs(np.angle(np.exp(1j * ph) * np.exp(-1j * np.angle(kept))))[strong].max() < 1e-9
    np.testing.assert_allclose(time_domain, np.abs(kept + dropped), atol=1e-11 * peak)
    assert np.abs(dropped).max() < small * peak
    assert np.abs(got - time_domain).max() < small * peak


def test_tone_reads_half_its_amplitude():
    # a tone of exactly Q cycles per kernel (f = Q s / N_q): |X_cq| = A/2 in mid-signal frames
    sr, fmin, nb, b, hop, A = 22050, 220.0, 36, 12, 256, 0.6
    N = oracle.cqt_default_taps(sr, fmin, b)
    Nk, _ = oracle.cqt_lengths(sr, fmin, nb, b)
    for q in (0, 17, 35):
        f = oracle.cqt_Q(b) * sr / Nk[q]
        x = signals.tone(4 * N, sr, f, amp=A, phase=0.7 + q)
        C = oracle.cqt1992(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b)[0]
        mid = C[:, C.shape[1] // 2]
        assert int(np.argmax(mid)) == q
        assert abs(mid[q] - A / 2) < 1e-4 * A


def test_formats_and_frame_count():
    sr, fmin, nb, b, hop = 8000, 220.0, 13, 12, 64
    N = oracle.cqt_default_taps(sr, fmin, b)
    x = signals.batch(3, B=2, L=2 * N + 5)
    mag = oracle.cqt1992(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b)
    assert mag.shape == (2, nb, 1 + x.shape[1] // hop)
    pw = oracle.cqt1992(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b, fmt=oracle.POWER)
    lg = oracle.cqt1992(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b, fmt=oracle.LOG)
    np.testing.assert_allclose(pw, mag ** 2, rtol=1e-12)
    np.testing.assert_allclose(lg, np.log(np.maximum(pw, oracle.LOG_FLOOR)), rtol=1e-12)
    # a larger n_fft pads the kernels (and the waveform) further: the time-domain CQT with as many taps
    big = oracle.cqt1992(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b, n_fft=2 * N)
    ref = oracle.cqt(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b, n_taps=2 * N)
    assert big.shape == mag.shape
    assert np.abs(big - ref).max() < 2e-4 * ref.max()


# ---------------------------------------------------------------------------------------
# recursive downsampling with frequency-domain kernels (the paper's CQT2010 layer)
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("sr,hop,fmin,nb,b,fir", [(22050, 512, 32.70, 84, 12, 257), (16000, 64, 220.0, 29, 12, 63),
                                                  (44100, 128, 523.25, 72, 24, 257)])
def test_cqt2010_octave_by_octave_against_scipy_downsampling_and_the_one_rate_transform(sr, hop, fmin, nb, b, fir):
    # octave a of the result = the (pinned) one-rate transform with frequency-domain kernels of the
    # waveform downsampled a times here with SciPy, for that octave's bins at sr / 2^a, hop / 2^a
    L = 22050
    x = signals.batch(3, B=1, L=L)[0]
    N = oracle.cqt2010_default_taps(sr, fmin, nb, b)
    got = oracle.cqt2010(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b, fir_taps=fir)[0]
    T = 1 + L // hop
    assert got.shape == (nb, T)
    gotc = oracle.cqt2010(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b, fir_taps=fir, fmt=oracle.COMPLEX)[0]
    assert gotc.shape == (2 * nb, T)
    np.testing.assert_allclose(np.hypot(gotc[0::2], gotc[1::2]), got, atol=1e-12)
    gotp = oracle.cqt2010(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b, fir_taps=fir, fmt=oracle.PHASE)[0]
    assert np.array_equal(gotp, np.arctan2(gotc[1::2], gotc[0::2]))
    h = scipy.signal.firwin(fir, 0.5)
    xa = x.astype(np.float64)
    n_oct = (nb + b - 1) // b
    for a in range(n_oct):
        hi = nb - a * b
        lo = max(hi - b, 0)
        # the one-rate oracle takes float32 input: the comparison carries that rounding (6e-8)
        ref = oracle.cqt1992(xa.astype(np.float32), sr=sr, hop=hop >> a, fmin=fmin * 2.0 ** ((lo + a * b) / b),
                             n_bins=hi - lo, bins_per_octave=b, n_fft=N)[0]
        assert np.abs(got[lo:hi] - ref[:, :T]).max() < 5e-7 * max(ref.max(), 1e-3)
        # and before the magnitude: rows 2q / 2q+1 of the complex format against the one-rate transform's
        refc = oracle.cqt1992(xa.astype(np.float32), sr=sr, hop=hop >> a, fmin=fmin * 2.0 ** ((lo + a * b) / b),
                              n_bins=hi - lo, bins_per_octave=b, n_fft=N, fmt=oracle.COMPLEX)[0]
        assert np.abs(gotc[2 * lo:2 * hi] - refc[:, :T]).max() < 5e-7 * max(ref.max(), 1e-3)
        xa = scipy.signal.convolve(np.pad(xa, fir // 2, mode="reflect"), h, mode="valid")[::2]


def test_cqt2010_agrees_with_its_time_domain_twin_up_to_the_dropped_half():
    x = signals.batch(3, B=2, L=22050)
    a = oracle.cqt2010(x)
    c = oracle.cqt2010v2(x)
    assert a.shape == c.shape == (2, 84, 44)
    for o in range(7):
        sl = slice(84 - 12 * (o + 1), 84 - 12 * o)
        assert np.abs(a[:, sl] - c[:, sl]).max() < 5e-4 * c[:, sl].max()


def test_cqt2010_tone_reads_half_its_amplitude_in_every_octave():
    sr, hop, fmin, nb, b, A = 22050, 512, 32.70, 84, 12, 0.5
    L = 6 * 22050
    for k in (3, 40, 80):
        a = (nb - 1 - k) // b
        Nk = int(np.ceil(oracle.cqt_Q(b) * sr / (fmin * 2.0 ** ((k + a * b) / b))))
        f = oracle.cqt_Q(b) * (sr / 2 ** a) / Nk  # Q cycles per kernel at the octave's rate
        x = signals.tone(L, sr, f, amp=A, phase=0.4 + k)
        C = oracle.cqt2010(x, sr=sr, hop=hop, fmin=fmin, n_bins=nb, bins_per_octave=b)[0]
        mid = C[:, C.shape[1] // 2]
        assert int(np.argmax(mid)) == k
        assert abs(mid[k] - A / 2) < 4e-3 * A  # filter ripple of the octaves above (3e-3) included
