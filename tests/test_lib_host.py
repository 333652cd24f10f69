"""Host-side checks of the HIP library that need no GPU: the C ABI loads and exports what
include/nna.h declares, argument checking, and the kernel banks a host-only plan (device -1)
builds, compared with the oracle's independently built banks."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_1912_12055_amd import binding as nb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _status(fn, *a, **k):
    try:
        fn(*a, **k)
    except nb.NnaError as e:
        return e.status
    return nb.NNA_OK


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "nna.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(nna_[a-z0-9_]+)\s*\(", header))
    assert declared == set(nb.EXPORTS)
    L = ctypes.CDLL(nb.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name


def test_status_strings_and_last_error():
    assert nb.nna_status_str(0) == "ok"
    assert _status(nb.nna_plan_stft, n_fft=2047, device=-1) == nb.NNA_ERR_INVALID_ARG
    assert "n_fft" in nb.nna_last_error()


def test_plan_argument_checking():
    assert _status(nb.nna_plan_stft, n_fft=6, device=-1) == nb.NNA_ERR_INVALID_ARG
    assert _status(nb.nna_plan_stft, hop=0, device=-1) == nb.NNA_ERR_INVALID_ARG
    assert _status(nb.nna_plan_stft, win=7, device=-1) == nb.NNA_ERR_INVALID_ARG
    assert _status(nb.nna_plan_stft, fmt=5, device=-1) == nb.NNA_ERR_INVALID_ARG
    assert _status(nb.nna_plan_stft, device=-2) == nb.NNA_ERR_INVALID_ARG
    assert _status(nb.nna_plan_mel, fmax=12000.0, device=-1) == nb.NNA_ERR_INVALID_ARG  # above sr/2
    assert _status(nb.nna_plan_mel, fmin=500.0, fmax=400.0, device=-1) == nb.NNA_ERR_INVALID_ARG
    assert _status(nb.nna_plan_mel, power=3.0, device=-1) == nb.NNA_ERR_INVALID_ARG
    assert _status(nb.nna_plan_mel, n_mels=0, device=-1) == nb.NNA_ERR_INVALID_ARG
    assert _status(nb.nna_plan_cqt, fmin=0.0, device=-1) == nb.NNA_ERR_INVALID_ARG
    assert _status(nb.nna_plan_cqt, n_taps=8192, device=-1) == nb.NNA_ERR_INVALID_ARG  # < longest kernel 11,341
    assert _status(nb.nna_plan_cqt, n_taps=16385, device=-1) == nb.NNA_ERR_INVALID_ARG  # odd
    assert _status(nb.nna_plan_cqt, n_bins=120, device=-1) == nb.NNA_ERR_INVALID_ARG  # top bin above Nyquist
    # the 1,770-waveform CQT workload: 32,768 taps cannot hold the 46,025-tap kernel; 65,536 can
    assert _status(nb.nna_plan_cqt, sr=44100, n_bins=168, bins_per_octave=24, n_taps=32768, device=-1) \
        == nb.NNA_ERR_INVALID_ARG
    assert "46025" in nb.nna_last_error()


def test_no_gpu_means_an_error_not_a_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    assert _status(nb.nna_plan_stft, device=0) == nb.NNA_ERR_HIP


def test_host_only_plan_cannot_run():
    p = nb.nna_plan_stft(n_fft=64, hop=16, device=-1)
    rc = nb.lib().nna_stft(p.handle, 16, 1, 1000, 16, None)  # dummy non-null pointers, never touched
    assert rc == nb.NNA_ERR_UNSUPPORTED
    assert nb.lib().nna_stft(p.handle, None, 1, 1000, 16, None) == nb.NNA_ERR_INVALID_ARG
    assert nb.lib().nna_mel(p.handle, 16, 1, 1000, 16, None) == nb.NNA_ERR_INVALID_ARG  # wrong plan kind
    assert nb.lib().nna_cqt(p.handle, 16, 1, 1000, 16, None) == nb.NNA_ERR_INVALID_ARG


@pytest.mark.parametrize("L,K,hop,center", [(22050, 2048, 512, True), (110250, 2048, 512, True),
                                             (176400, 2048, 512, True), (5000, 512, 100, False), (600, 512, 64, True)])
def test_out_shape_matches_oracle_frame_count(L, K, hop, center):
    p = nb.nna_plan_stft(n_fft=K, hop=hop, center=center, device=-1)
    bins, frames = nb.nna_out_shape(p, 3, L)
    assert bins == K // 2 + 1
    assert frames == oracle.num_frames(L, K, hop, center)


def test_out_shape_rejects_short_signals():
    p = nb.nna_plan_stft(n_fft=2048, hop=512, device=-1)
    assert _status(nb.nna_out_shape, p, 1, 1024) == nb.NNA_ERR_SHAPE  # needs L > pad
    assert nb.nna_out_shape(p, 1, 1025) == (1025, 3)
    assert _status(nb.nna_out_shape, p, 0, 4096) == nb.NNA_ERR_SHAPE
    q = nb.nna_plan_stft(n_fft=2048, hop=512, center=False, device=-1)
    assert _status(nb.nna_out_shape, q, 1, 2047) == nb.NNA_ERR_SHAPE
    assert nb.nna_out_shape(q, 1, 2048) == (1025, 1)


@pytest.mark.parametrize("n_fft,hop,win", [(2048, 512, nb.NNA_WIN_HANN), (256, 64, nb.NNA_WIN_HANN),
                                           (256, 64, nb.NNA_WIN_HAMMING), (512, 128, nb.NNA_WIN_BLACKMAN),
                                            (96, 25, nb.NNA_WIN_HANN), (200, 50, nb.NNA_WIN_RECT),
                                            (130, 130, nb.NNA_WIN_HANN)])
def test_stft_bank_is_windowed_dft_kernels(n_fft, hop, win):
    # eq. (DFT2) with the window folded in, rebuilt here with numpy; the library's bank has
    # gone through its tile permutation and back
    p = nb.nna_plan_stft(n_fft=n_fft, hop=hop, win=win, device=-1)
    bank = nb.nna_plan_bank(p)
    F = n_fft // 2 + 1
    assert bank.shape == (2 * F, n_fft)
    n = np.arange(n_fft)
    w = oracle.window(win, n_fft)
    k = np.arange(F)[:, None]
    re = w * np.cos(2 * np.pi * ((k * n) % n_fft) / n_fft)
    im = -w * np.sin(2 * np.pi * ((k * n) % n_fft) / n_fft)
    im[0] = 0.0
    im[-1] = 0.0  # sin(pi n) is identically zero: the library stores exact zeros
    np.testing.assert_allclose(bank[0::2], re, atol=1e-7)
    np.testing.assert_allclose(bank[1::2], im, atol=1e-7)
    info = p.info()
    assert info["kind"] == nb.NNA_KIND_STFT and info["out_bins"] == F
    assert info["algorithmic_flops_per_frame"] == 2.0 * n_fft * n_fft  # the direct contraction of eq. (DFT2)
    J = n_fft // hop if n_fft % hop == 0 else 0
    if J >= 4 and J % 2 == 0 and hop % 32 == 0:
        # folded frames (x[n] +- x[N-n] against the kernels' first halves): N/2 taps for the N rows of bins
        # 0 .. N/2-1 (padded to whole 64-bin row tiles), and bin N/2 by itself
        rows = -(-(n_fft // 2) // 64) * 128
        if n_fft % 256 == 0 and hop % 2 == 0:
            # split once more by tap parity: the rows of the bins below N/4 only, and bin N/4 (two real sums) by itself
            assert info["executed_flops_per_frame"] == 2.0 * (n_fft // 2) * (rows // 2) + 4.0 * n_fft
        else:
            assert info["executed_flops_per_frame"] == 2.0 * (n_fft // 2) * rows + 2.0 * n_fft
    else:
        assert info["executed_flops_per_frame"] >= info["algorithmic_flops_per_frame"]
    # a trainable or complex-output plan keeps the direct contraction
    pc = nb.nna_plan_stft(n_fft=n_fft, hop=hop, win=win, fmt=nb.NNA_OUT_COMPLEX, device=-1)
    assert pc.info()["executed_flops_per_frame"] >= 2.0 * n_fft * n_fft


@pytest.mark.parametrize("scale,sr,n_fft,hop,fmin,fmax,bins", [
    (nb.NNA_FREQ_LINEAR, 44100, 2048, 512, 50.0, 6000.0, 1025),   # the worked example of Sec. II-B
    (nb.NNA_FREQ_LINEAR, 22050, 256, 64, 0.0, 11025.0, 128),
    (nb.NNA_FREQ_LOG, 22050, 512, 100, 55.0, 7040.0, 84),
    (nb.NNA_FREQ_LOG, 16000, 96, 25, 100.0, 8000.0, 7),
])
def test_scaled_stft_bank_is_eq_dft3(scale, sr, n_fft, hop, fmin, fmax, bins):
    p = nb.nna_plan_stft_scaled(sr=sr, n_fft=n_fft, hop=hop, freq_scale=scale, fmin=fmin, fmax=fmax, freq_bins=bins,
                                device=-1)
    sig = nb.nna_plan_sigma(p)
    want = np.array([oracle.freq_sigma(scale, k, fmin, fmax, bins, n_fft, sr) for k in range(bins)])
    np.testing.assert_allclose(sig, want, rtol=1e-13, atol=1e-13)
    bank = nb.nna_plan_bank(p)
    assert bank.shape == (2 * bins, n_fft)
    n = np.arange(n_fft)
    w = oracle.window(nb.NNA_WIN_HANN, n_fft)
    np.testing.assert_allclose(bank[0::2], w * np.cos(2 * np.pi * want[:, None] * n / n_fft), atol=2e-7)
    np.testing.assert_allclose(bank[1::2], -w * np.sin(2 * np.pi * want[:, None] * n / n_fft), atol=2e-7)
    info = p.info()
    assert info["kind"] == nb.NNA_KIND_STFT and info["out_bins"] == bins
    assert nb.nna_out_shape(p, 3, 5 * n_fft)[0] == bins
    assert info["algorithmic_flops_per_frame"] == 4.0 * n_fft * bins
    assert info["executed_flops_per_frame"] >= info["algorithmic_flops_per_frame"]


def test_scaled_stft_argument_checking():
    f = nb.nna_plan_stft_scaled
    assert _status(f, freq_scale=0, device=-1) == nb.NNA_ERR_INVALID_ARG
    assert _status(f, freq_scale=nb.NNA_FREQ_LOG, fmin=0.0, device=-1) == nb.NNA_ERR_INVALID_ARG
    assert _status(f, fmin=500.0, fmax=400.0, device=-1) == nb.NNA_ERR_INVALID_ARG
    assert _status(f, fmax=12000.0, device=-1) == nb.NNA_ERR_INVALID_ARG  # above sr/2
    assert _status(f, freq_bins=-1, device=-1) == nb.NNA_ERR_INVALID_ARG
    assert _status(f, freq_bins=20000, device=-1) == nb.NNA_ERR_INVALID_ARG
    assert f(freq_bins=0, device=-1).info()["out_bins"] == 1025  # default: n_fft/2 + 1 bins
    # sigma of a plain plan is the bin index; other kinds have none
    np.testing.assert_array_equal(nb.nna_plan_sigma(nb.nna_plan_stft(n_fft=64, hop=16, device=-1)), np.arange(33.0))
    assert _status(nb.nna_plan_sigma, nb.nna_plan_mel(device=-1)) == nb.NNA_ERR_INVALID_ARG


@pytest.mark.parametrize("sr,n_fft,n_mels,fmin,fmax,scale,norm", [
    (22050, 2048, 128, 0.0, 0.0, nb.NNA_MEL_SLANEY, True),
    (44100, 2048, 128, 0.0, 22050.0, nb.NNA_MEL_SLANEY, True),
    (1000, 128, 4, 0.0, 500.0, nb.NNA_MEL_HTK, False),
    (16000, 512, 200, 50.0, 7000.0, nb.NNA_MEL_HTK, True),
])
def test_mel_weights_match_oracle_filterbank(sr, n_fft, n_mels, fmin, fmax, scale, norm):
    p = nb.nna_plan_mel(sr=sr, n_fft=n_fft, hop=n_fft // 4, n_mels=n_mels, fmin=fmin, fmax=fmax, scale=scale,
                        norm_area=norm, device=-1)
    W = nb.nna_plan_mel_weights(p)
    Wo, _ = oracle.mel_filterbank(sr, n_fft, n_mels, fmin, fmax, scale, norm)
    assert W.shape == Wo.shape
    np.testing.assert_allclose(W, Wo, atol=2e-7 * Wo.max(), rtol=2e-6)
    assert p.info()["out_bins"] == n_mels


@pytest.mark.parametrize("sr,hop,fmin,nbins,bpo,taps", [
    (22050, 512, 32.70, 84, 12, 16384),   # config 3
    (8000, 128, 220.0, 24, 12, 1024),
    (8000, 100, 220.0, 30, 12, 1000),     # hop does not divide the taps: non-overlapping LDS mode
    (8000, 48, 300.0, 13, 6, 0),          # default taps, hop not a multiple of 16
    (44100, 441, 32.70, 26, 24, 0),       # non-overlapping mode with 46,025-tap kernels (65,536 taps): 2,878 chunks
])
def test_cqt_bank_matches_oracle_kernels(sr, hop, fmin, nbins, bpo, taps):
    p = nb.nna_plan_cqt(sr=sr, hop=hop, fmin=fmin, n_bins=nbins, bins_per_octave=bpo, n_taps=taps, device=-1)
    bank = nb.nna_plan_bank(p)
    kre, kim = oracle.cqt_kernels(sr, fmin, nbins, bpo, n_taps=taps)
    assert bank.shape == (2 * nbins, kre.shape[1])
    scale = np.abs(kre).max(axis=1, keepdims=True)
    assert np.max(np.abs(bank[0::2] - kre) / scale) < 1e-7
    assert np.max(np.abs(bank[1::2] - kim) / scale) < 1e-7
    Nk, _ = oracle.cqt_lengths(sr, fmin, nbins, bpo)
    np.testing.assert_array_equal(nb.nna_plan_cqt_lengths(p), Nk)
    info = p.info()
    assert info["algorithmic_flops_per_frame"] == 4.0 * Nk.sum()
    # (12 bins per octave or fewer: whichever kernel runs multiplies more than the taps of the direct form)
    assert info["executed_flops_per_frame"] >= info["algorithmic_flops_per_frame"]


def test_cqt_plans_fold_their_kernels_where_it_pays():
    # 24 bins per octave and kernels of many hops: the kernels are folded about their centres, and the plan
    # multiplies less than the direct form's 4 sum N_k -- but never less than half of it
    kw = dict(sr=44100, hop=512, fmin=32.70, n_bins=168, bins_per_octave=24, n_taps=0, device=-1)
    info = nb.nna_plan_cqt(**kw).info()
    assert 0.5 * info["algorithmic_flops_per_frame"] < info["executed_flops_per_frame"] < 0.8 * info["algorithmic_flops_per_frame"]
    # a window that does not vanish at n = 0 has no mirror partner for that tap: direct kernel
    ham = nb.nna_plan_cqt(win=nb.NNA_WIN_HAMMING, **kw).info()
    assert ham["executed_flops_per_frame"] >= ham["algorithmic_flops_per_frame"]
    # a hop that does not divide half the taps, kernels shorter than eight hops: direct kernel
    for odd in (dict(kw, hop=441), dict(kw, fmin=2000.0, n_bins=24)):
        i = nb.nna_plan_cqt(**odd).info()
        assert i["executed_flops_per_frame"] >= i["algorithmic_flops_per_frame"]


def test_cqt_workload_5_plan_facts():
    p = nb.nna_plan_cqt(sr=44100, hop=512, fmin=32.70, n_bins=168, bins_per_octave=24, n_taps=0, device=-1)
    info = p.info()
    assert info["taps"] == 65536 and info["bank_rows"] == 336
    Nk = nb.nna_plan_cqt_lengths(p)
    assert (Nk[0], Nk[-1], Nk.sum()) == (46025, 371, 1604166)
    # zero-tap skipping and the fold: executed work stays below the taps of the direct form
    assert info["executed_flops_per_frame"] < info["algorithmic_flops_per_frame"]


@pytest.mark.parametrize("sr,hop,fmin,n_bins,bpo,fir", [(22050, 512, 32.70, 84, 12, 0), (16000, 64, 220.0, 29, 12, 63),
                                                       (44100, 512, 32.70, 168, 24, 257)])
def test_cqt2010v2_plan_parts(sr, hop, fmin, n_bins, bpo, fir):
    p = nb.nna_plan_cqt2010v2(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, fir_taps=fir, device=-1)
    info = p.info()
    n_taps = oracle.cqt2010_default_taps(sr, fmin, n_bins, bpo)
    assert info["kind"] == nb.NNA_KIND_CQT2010V2 and info["out_bins"] == n_bins and info["taps"] == n_taps
    # the filter: 64 shifted copies of the window-method half-band design
    h = oracle.lowpass_fir(fir or oracle.FIR_TAPS, 0.5)
    bank = nb.nna_plan_bank(nb.nna_plan_part(p, -1))
    assert bank.shape[0] == 64
    for r in range(64):
        want = np.zeros(bank.shape[1])
        want[2 * r:2 * r + h.size] = h
        np.testing.assert_allclose(bank[r], want, atol=3e-8)
    # octave a: the kernels of its bins, one factor 2^a up the frequency axis, at the original rate
    n_oct = -(-n_bins // bpo)
    for a in range(n_oct):
        hi = n_bins - a * bpo
        lo = max(0, hi - bpo)
        part = nb.nna_plan_part(p, a)
        kre, kim = oracle.cqt_kernels(sr, fmin * 2.0 ** ((lo + a * bpo) / bpo), hi - lo, bpo, n_taps=n_taps)
        got = nb.nna_plan_bank(part)
        assert got.shape == (2 * (hi - lo), n_taps)
        np.testing.assert_allclose(got[0::2], kre, atol=2e-9)
        np.testing.assert_allclose(got[1::2], kim, atol=2e-9)
    assert _status(nb.nna_plan_part, p, n_oct) == nb.NNA_ERR_INVALID_ARG
    assert nb.nna_out_shape(p, 3, 400 * hop + 5) == (n_bins, 401)


def test_cqt2010v2_argument_checking():
    f = nb.nna_plan_cqt2010v2
    assert _status(f, hop=100, device=-1) == nb.NNA_ERR_INVALID_ARG       # 7 octaves need hop % 64 == 0
    assert _status(f, fir_taps=256, device=-1) == nb.NNA_ERR_INVALID_ARG  # even: no integer delay
    assert _status(f, n_bins=120, device=-1) == nb.NNA_ERR_INVALID_ARG    # top bin above Nyquist
    assert _status(f, n_taps=128, device=-1) == nb.NNA_ERR_INVALID_ARG    # shorter than the top octave's longest kernel
    p = f(device=-1)
    assert _status(nb.nna_out_shape, p, 1, 4000) == nb.NNA_ERR_SHAPE      # deepest octave: 63 samples <= 128
    assert _status(nb.nna_plan_bank, p) == nb.NNA_ERR_INVALID_ARG         # several banks: ask for a part
    assert _status(nb.nna_plan_part, nb.nna_plan_cqt(device=-1), 0) == nb.NNA_ERR_INVALID_ARG
    single = f(fmin=1000.0, n_bins=12, sr=16000, device=-1)
    assert _status(nb.nna_plan_part, single, -1) == nb.NNA_ERR_INVALID_ARG  # one octave: no filter
    assert nb.nna_cqt2010v2_workspace(single, 4, 9000) == 0
    assert nb.nna_cqt2010v2_workspace(p, 4, 22050) >= 4 * 4 * (11025 + 5513)


@pytest.mark.parametrize("sr,hop,fmin,n_bins,bpo,n_fft", [(22050, 256, 220.0, 36, 12, 0), (8000, 64, 110.0, 60, 12, 4096),
                                                          (1000, 16, 100.0, 5, 3, 0)])
def test_cqt1992_plan_holds_the_dft_bank_and_the_oracles_spectral_kernels(sr, hop, fmin, n_bins, bpo, n_fft):
    p = nb.nna_plan_cqt1992(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, n_fft=n_fft, device=-1)
    info = p.info()
    N = n_fft or oracle.cqt_default_taps(sr, fmin, bpo)
    assert (info["kind"], info["taps"], info["out_bins"], info["bank_rows"]) == (nb.NNA_KIND_CQT1992, N, n_bins, N + 2)
    np.testing.assert_array_equal(nb.nna_plan_cqt_lengths(p), oracle.cqt_lengths(sr, fmin, n_bins, bpo)[0])
    # stage 2: Y / n_fft, float32-rounded
    want = oracle.cqt1992_spectral_kernels(sr, fmin, n_bins, bpo, n_fft=N) / N
    got = nb.nna_plan_spectral_kernels(p)
    assert got.shape == want.shape
    np.testing.assert_allclose(got, want, atol=2e-7 * np.abs(want).max())
    # stage 1: the un-windowed DFT kernels of eq. (DFT2)
    bank = nb.nna_plan_bank(p)
    n = np.arange(N)
    for k in (0, 1, N // 4 + 1, N // 2):
        np.testing.assert_allclose(bank[2 * k], np.cos(2 * np.pi * k * n / N), atol=1e-6)
        np.testing.assert_allclose(bank[2 * k + 1], -np.sin(2 * np.pi * k * n / N), atol=1e-6)
    assert nb.nna_out_shape(p, 3, 5 * N) == (n_bins, 1 + 5 * N // hop)
    assert info["algorithmic_flops_per_frame"] == 2.0 * N * N + 8.0 * n_bins * (N // 2 + 1)


def test_cqt1992_argument_checking():
    kw = dict(sr=22050, hop=256, fmin=220.0, n_bins=36, bins_per_octave=12, device=-1)
    assert _status(nb.nna_plan_cqt1992, **kw) == nb.NNA_OK
    assert _status(nb.nna_plan_cqt1992, n_fft=1024, **kw) == nb.NNA_ERR_INVALID_ARG  # longest kernel: 1,686 taps
    assert "longest kernel" in nb.nna_last_error()
    assert _status(nb.nna_plan_cqt1992, n_fft=3000, **kw) == nb.NNA_ERR_INVALID_ARG  # not a power of two
    assert _status(nb.nna_plan_cqt1992, n_fft=1 << 17, **kw) == nb.NNA_ERR_UNSUPPORTED
    assert _status(nb.nna_plan_cqt1992, **{**kw, "n_bins": 80}) == nb.NNA_ERR_INVALID_ARG  # top bin above sr/2
    p = nb.nna_plan_cqt(sr=22050, hop=256, fmin=220.0, n_bins=36, device=-1)
    assert _status(nb.nna_plan_spectral_kernels, p) == nb.NNA_ERR_INVALID_ARG


@pytest.mark.parametrize("sr,hop,fmin,n_bins,bpo,fir", [(22050, 512, 32.70, 84, 12, 0), (16000, 64, 220.0, 29, 12, 63)])
def test_cqt2010_plan_parts(sr, hop, fmin, n_bins, bpo, fir):
    p = nb.nna_plan_cqt2010(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, fir_taps=fir, device=-1)
    info = p.info()
    N = oracle.cqt2010_default_taps(sr, fmin, n_bins, bpo)
    assert (info["kind"], info["taps"], info["out_bins"]) == (nb.NNA_KIND_CQT2010, N, n_bins)
    n_oct = (n_bins + bpo - 1) // bpo
    L = 22050
    assert nb.nna_out_shape(p, 2, L) == (n_bins, 1 + L // hop)
    assert nb.nna_cqt2010v2_workspace(p, 2, L) == nb.nna_cqt2010v2_workspace(
        nb.nna_plan_cqt2010v2(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, fir_taps=fir, device=-1), 2, L)
    flops = 0.0
    for a in range(n_oct):
        hi = n_bins - a * bpo
        lo = max(hi - bpo, 0)
        sub = nb.nna_plan_part(p, a)
        si = sub.info()
        assert (si["kind"], si["taps"], si["out_bins"]) == (nb.NNA_KIND_CQT1992, N, hi - lo)
        # the octave's spectral kernels: those of the one-rate transform for its bins' frequencies x 2^a
        want = oracle.cqt1992_spectral_kernels(sr, fmin * 2.0 ** ((lo + a * bpo) / bpo), hi - lo, bpo, n_fft=N) / N
        got = nb.nna_plan_spectral_kernels(sub)
        np.testing.assert_allclose(got, want, atol=2e-7 * np.abs(want).max())
        flops += si["algorithmic_flops_per_frame"]
    if n_oct > 1:
        fir_plan = nb.nna_plan_part(p, -1)
        flops += sum((hop >> (a + 1)) / 64 * fir_plan.info()["algorithmic_flops_per_frame"] for a in range(n_oct - 1))
    assert abs(info["algorithmic_flops_per_frame"] - flops) < 1e-6 * flops
    assert _status(nb.nna_plan_bank, p) == nb.NNA_ERR_INVALID_ARG


def test_cqt2010_argument_checking():
    kw = dict(sr=22050, fmin=32.70, n_bins=84, bins_per_octave=12, device=-1)
    assert _status(nb.nna_plan_cqt2010, hop=512, **kw) == nb.NNA_OK
    assert _status(nb.nna_plan_cqt2010, hop=96, **kw) == nb.NNA_ERR_INVALID_ARG  # 7 octaves need hop % 64 == 0
    assert _status(nb.nna_plan_cqt2010, hop=512, n_fft=128, **kw) == nb.NNA_ERR_INVALID_ARG  # top octave: 178 taps
    assert _status(nb.nna_plan_cqt2010, hop=512, n_fft=300, **kw) == nb.NNA_ERR_INVALID_ARG  # not a power of two
    assert _status(nb.nna_plan_cqt2010, hop=512, fir_taps=64, **kw) == nb.NNA_ERR_INVALID_ARG


def test_complex_and_phase_formats_shapes_and_where_they_exist():
    p = nb.nna_plan_stft(n_fft=256, hop=64, fmt=nb.NNA_OUT_COMPLEX, device=-1)
    assert nb.nna_out_shape(p, 2, 1000) == (2 * 129, 16) and p.info()["out_bins"] == 258
    p = nb.nna_plan_stft(n_fft=256, hop=64, fmt=nb.NNA_OUT_PHASE, device=-1)
    assert nb.nna_out_shape(p, 2, 1000) == (129, 16)
    p = nb.nna_plan_stft_scaled(n_fft=256, hop=64, fmt=nb.NNA_OUT_COMPLEX, freq_bins=40, device=-1)
    assert nb.nna_out_shape(p, 1, 1000) == (80, 16)
    p = nb.nna_plan_cqt(sr=8000, hop=64, fmin=220.0, n_bins=24, fmt=nb.NNA_OUT_COMPLEX, device=-1)
    assert nb.nna_out_shape(p, 1, 4000)[0] == 48 and nb.nna_plan_cqt_lengths(p).size == 24
    # all four constant-Q transforms have them (the output_format argument of the paper's CQT layers) ...
    for fn, kw in ((nb.nna_plan_cqt2010v2, {}), (nb.nna_plan_cqt2010, {}), (nb.nna_plan_cqt1992, dict(fmin=220.0, n_bins=24))):
        p = fn(fmt=nb.NNA_OUT_COMPLEX, device=-1, **kw)
        n_bins = kw.get("n_bins", 84)
        assert nb.nna_out_shape(p, 2, 44100) == (2 * n_bins, 1 + 44100 // 512) and p.info()["out_bins"] == 2 * n_bins
        assert nb.nna_out_shape(fn(fmt=nb.NNA_OUT_PHASE, device=-1, **kw), 2, 44100)[0] == n_bins
    # ... float16 plans do not (a Mel plan has no output format at all)
    assert _status(nb.nna_plan_stft_prec, fmt=nb.NNA_OUT_COMPLEX, precision=nb.NNA_PREC_F16, device=-1) == nb.NNA_ERR_UNSUPPORTED
    assert _status(nb.nna_plan_stft, fmt=5, device=-1) == nb.NNA_ERR_INVALID_ARG


def test_bench_refuses_more_than_one_gpu_and_has_no_cpu_fallback():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and not r.stdout.strip()
    import torch
    if not torch.cuda.is_available():
        r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True)
        assert r.returncode != 0 and "no CPU fallback" in r.stderr and not r.stdout.strip()


def test_waveforms_shorter_than_four_samples_are_refused():
    # a 4-tap constant-Q bank pads by 2, so L = 3 would have a mirror image; the loader's 16-byte windows
    # need four stored samples
    p = nb.nna_plan_cqt(sr=10, hop=1, fmin=4.0, n_bins=1, bins_per_octave=1, device=-1)
    assert p.info()["taps"] == 4
    with pytest.raises(nb.NnaError) as e:
        nb.nna_out_shape(p, 1, 3)
    assert e.value.status == nb.NNA_ERR_SHAPE
    assert nb.nna_out_shape(p, 1, 4) == (1, 5)
