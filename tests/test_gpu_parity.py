"""GPU parity: the HIP library (through its C ABI binding) against the float64 CPU oracle,
element by element on the same seeded inputs.

Bar (floating point): per waveform, max |gpu - oracle| <= 1e-3 * max |oracle| -- the
tolerance the benchmark spec states -- and the kernels accumulate in float32 from float32-rounded
banks, so the observed error is expected near 1e-6.
"""
import sys

import numpy as np
import pytest

import oracle
from paper_1912_12055_amd import signals
from tile_sample import sampled_waveforms

pytestmark = pytest.mark.gpu

TOL = 1e-3


@pytest.fixture(scope="module")
def nb():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (there is no CPU fallback)")
    from paper_1912_12055_amd import binding
    binding.lib()
    return binding


def _say(msg):
    print(f"[case] {msg}", file=sys.stderr, flush=True)


def _dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")


def _rel_err(got, ref):
    """max over waveforms of max|got-ref| / max|ref| (each output's own peak)."""
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got))
    worst = 0.0
    for b in range(ref.shape[0]):
        peak = np.abs(ref[b]).max()
        err = np.abs(got[b] - ref[b]).max()
        worst = max(worst, err / peak if peak > 0 else err)
    return worst


def _rand(B, L, seed):
    rng = np.random.default_rng(seed)
    return (0.5 * rng.standard_normal((B, L))).astype(np.float32)


# ---------------------------------------------------------------------------------------
# STFT
# ---------------------------------------------------------------------------------------
STFT_CASES = [
    # name, B, L, n_fft, hop, window, center, fmt
    ("one tile, one waveform", 1, 8000, 256, 64, 0, True, 0),
    ("several tiles, ragged tail, tiles span waveforms", 5, 30000, 256, 64, 0, True, 0),
    ("many short waveforms per tile", 37, 700, 256, 64, 0, True, 1),
    ("single-frame waveforms (T=1)", 9, 40, 64, 64, 0, True, 0),
    ("hop does not divide n_fft", 3, 5000, 96, 25, 0, True, 0),
    ("hop not a multiple of 32", 2, 6000, 240, 48, 0, False, 0),
    ("no centring, rect window", 2, 9000, 512, 128, 1, False, 1),
    ("L not a multiple of 4 (unaligned rows)", 3, 22050, 512, 128, 0, True, 0),
    ("n_fft not a multiple of 128", 2, 7000, 200, 50, 0, True, 0),
    ("n_fft = 4096, hop 512 (8 shifts)", 2, 40000, 4096, 512, 0, True, 0),
    ("32 hop-shifts", 2, 20000, 1024, 32, 0, True, 0),
    ("log output", 2, 9000, 256, 64, 0, True, 2),
    ("Hamming window", 2, 9000, 256, 64, 2, True, 0),
    ("Blackman window, power", 3, 12000, 512, 128, 3, True, 1),
    # n_fft a multiple of 128 but not of 256: folded once, not split by tap parity (the plan's executed flops say which)
    ("folded once: n_fft 384, six shifts", 3, 9000, 384, 64, 0, True, 0),
    ("split: three row tiles below N/4, hop 96", 3, 9000, 768, 96, 0, True, 1),
    ("split: Hamming window (w[0] != 0), no centring", 2, 9000, 512, 64, 2, False, 0),
]


@pytest.mark.parametrize("case", STFT_CASES, ids=[c[0] for c in STFT_CASES])
def test_stft_parity_small(nb, case):
    name, B, L, n_fft, hop, win, center, fmt = case
    _say(f"stft {name}: B={B} L={L} n_fft={n_fft} hop={hop} win={win} center={center} fmt={fmt}")
    x = _rand(B, L, 100 + n_fft + hop)
    plan = nb.nna_plan_stft(n_fft=n_fft, hop=hop, win=win, center=center, fmt=fmt, device=0)
    got = nb.nna_stft(plan, _dev(x)).cpu().numpy()
    ref = oracle.stft(x, n_fft=n_fft, hop=hop, window=win, center=center, fmt=fmt)
    if fmt == 2:
        # log compression: compare where the power is above -60 dB of the peak, absolutely
        pw = oracle.stft(x, n_fft=n_fft, hop=hop, window=win, center=center, fmt=1)
        sel = pw > 1e-6 * pw.max()
        assert np.abs(got - ref)[sel].max() < 2e-3
    else:
        assert _rel_err(got, ref) < TOL
        assert _rel_err(got, ref) < 2e-5  # what float32 accumulation actually delivers


def test_stft_device_bank_equals_host_bank(nb):
    _say("stft bank read-back")
    host = nb.nna_plan_bank(nb.nna_plan_stft(n_fft=512, hop=128, device=-1))
    dev = nb.nna_plan_bank(nb.nna_plan_stft(n_fft=512, hop=128, device=0))
    np.testing.assert_array_equal(host, dev)


def test_stft_config1_full(nb):
    wl = signals.WORKLOADS[1]
    _say("stft config 1 (4 x 22050 @ 22050 Hz, n_fft 2048, hop 512)")
    x = signals.batch(1)
    plan = nb.nna_plan_stft(sr=wl["sr"], n_fft=2048, hop=512, device=0)
    got = nb.nna_stft(plan, _dev(x)).cpu().numpy()
    assert got.shape == (4, 1025, 44)
    ref = oracle.stft(x, n_fft=2048, hop=512)
    e = _rel_err(got, ref)
    _say(f"  rel err {e:.3e}")
    assert e < TOL


def test_stft_tone_closed_form_on_gpu(nb):
    # tone on bin k0: |X[k0]| = A * sum(w) / 2 = 512 A (the closed form that pins the oracle)
    _say("stft closed form tone")
    N, k0, A = 2048, 300, 0.25
    x = (A * np.cos(2 * np.pi * k0 * np.arange(4 * N) / N + 0.4)).astype(np.float32)[None]
    plan = nb.nna_plan_stft(n_fft=N, hop=512, center=False, device=0)
    got = nb.nna_stft(plan, _dev(x)).cpu().numpy()[0]
    assert np.all(np.argmax(got, axis=0) == k0)
    assert np.max(np.abs(got[k0] - 512.0 * A)) < 1e-3 * 512.0 * A


SCALED_CASES = [
    # name, B, L, sr, n_fft, hop, scale, fmin, fmax, bins, center, fmt
    ("linear axis, bins not a multiple of the row tile", 3, 9000, 22050, 256, 64, 1, 50.0, 6000.0, 100, True, 0),
    ("linear axis, one partial row tile", 2, 5000, 16000, 128, 32, 1, 0.0, 8000.0, 7, True, 1),
    ("log axis, seven octaves", 4, 12000, 22050, 512, 128, 2, 55.0, 7040.0, 84, True, 0),
    ("log axis, hop does not divide n_fft, log output", 2, 7000, 22050, 240, 50, 2, 100.0, 9000.0, 129, False, 2),
    ("more bins than n_fft/2+1", 2, 6000, 22050, 128, 32, 1, 20.0, 11000.0, 300, True, 0),
]


@pytest.mark.parametrize("case", SCALED_CASES, ids=[c[0] for c in SCALED_CASES])
def test_scaled_stft_parity_small(nb, case):
    name, B, L, sr, n_fft, hop, scale, fmin, fmax, bins, center, fmt = case
    _say(f"scaled stft {name}: B={B} L={L} n_fft={n_fft} hop={hop} scale={scale} bins={bins} fmt={fmt}")
    x = _rand(B, L, 900 + bins)
    plan = nb.nna_plan_stft_scaled(sr=sr, n_fft=n_fft, hop=hop, center=center, fmt=fmt, freq_scale=scale, fmin=fmin,
                                   fmax=fmax, freq_bins=bins, device=0)
    got = nb.nna_stft(plan, _dev(x)).cpu().numpy()
    ref = oracle.stft_scaled(x, sr=sr, n_fft=n_fft, hop=hop, center=center, scale=scale, fmin=fmin, fmax=fmax,
                             freq_bins=bins, fmt=fmt)
    e = _rel_err(got, ref)
    _say(f"  rel err {e:.3e}")
    assert e < TOL


def test_scaled_stft_worked_example_full(nb):
    # the linear axis of Sec. II-B (50..6000 Hz, 1,025 bins, n_fft 2048 @ 44.1 kHz) on workload-4 waveforms
    _say("scaled stft, worked example of Sec. II-B on 3 x 176400 samples")
    x = signals.batch(4, [0, 885, 1769])
    plan = nb.nna_plan_stft_scaled(sr=44100, n_fft=2048, hop=512, freq_scale=nb.NNA_FREQ_LINEAR, fmin=50.0,
                                   fmax=6000.0, freq_bins=1025, device=0)
    got = nb.nna_stft(plan, _dev(x)).cpu().numpy()
    assert got.shape == (3, 1025, 345)
    ref = oracle.stft_scaled(x, sr=44100, n_fft=2048, hop=512, scale=oracle.FREQ_LINEAR, fmin=50.0, fmax=6000.0,
                             freq_bins=1025)
    e = _rel_err(got, ref)
    _say(f"  rel err {e:.3e}")
    assert e < TOL


def test_stft_rejects_bad_shapes(nb):
    import torch
    plan = nb.nna_plan_stft(n_fft=2048, hop=512, device=0)
    with pytest.raises(nb.NnaError) as e:
        nb.nna_stft(plan, torch.zeros((2, 1024), device="cuda:0"))
    assert e.value.status == nb.NNA_ERR_SHAPE
    mel = nb.nna_plan_mel(device=0)
    x = torch.zeros((1, 4096), device="cuda:0")
    out = torch.empty((1, 1025, 9), device="cuda:0")
    assert nb.lib().nna_stft(mel.handle, x.data_ptr(), 1, 4096, out.data_ptr(), None) == nb.NNA_ERR_INVALID_ARG


def test_size_limits_are_errors_not_launches(nb):
    # empty batches and sizes beyond the kernels' 32-bit sample / frame indices are refused before anything
    # is enqueued (the pointers are never touched: small buffers stand in for the impossible ones)
    import torch
    L_ = nb.lib()
    x = torch.zeros((1, 4096), device="cuda:0")
    out = torch.empty((1, 1025, 9), device="cuda:0")
    for plan, fn in ((nb.nna_plan_stft(device=0), L_.nna_stft), (nb.nna_plan_mel(device=0), L_.nna_mel),
                     (nb.nna_plan_cqt(sr=8000, hop=128, fmin=220.0, n_bins=24, n_taps=1024, device=0), L_.nna_cqt)):
        for B, L in ((0, 4096), (-3, 4096), (1 << 41, 4096), (1, (1 << 31) + 8), (1 << 31, 1 << 20)):
            assert fn(plan.handle, x.data_ptr(), B, L, out.data_ptr(), None) == nb.NNA_ERR_SHAPE, (B, L)
            assert nb.nna_last_error()
        assert fn(plan.handle, None, 1, 4096, out.data_ptr(), None) == nb.NNA_ERR_INVALID_ARG
        assert fn(plan.handle, x.data_ptr(), 1, 4096, None, None) == nb.NNA_ERR_INVALID_ARG
    torch.cuda.synchronize()


def _phase_err(got, ref_re, ref_im):
    """largest phase difference (modulo 2 pi) over the bins whose magnitude is above 1e-3 of the peak: below
    that the float32 rounding of (Re, Im) turns into an arbitrary angle"""
    mag = np.hypot(ref_re, ref_im)
    keep = mag > 1e-3 * mag.max()
    d = np.angle(np.exp(1j * (np.asarray(got, dtype=np.float64) - np.arctan2(ref_im, ref_re))))
    return np.abs(d[keep]).max()


COMPLEX_STFT_CASES = [
    # name, B, L, n_fft, hop, window, center
    ("several tiles, ragged tail, tiles span waveforms", 5, 30000, 256, 64, 0, True),
    ("no centring, rect window", 2, 9000, 512, 128, 1, False),
    ("hop does not divide n_fft", 3, 5000, 96, 25, 0, True),
    ("n_fft = 2048, hop 512", 2, 20000, 2048, 512, 0, True),
    ("32 hop-shifts: the 192-row tile of the one-workgroup-per-CU build, tiles span waveforms", 3, 14000, 2048, 64, 0, True),
]


@pytest.mark.parametrize("case", COMPLEX_STFT_CASES, ids=[c[0] for c in COMPLEX_STFT_CASES])
def test_stft_complex_and_phase_output(nb, case):
    name, B, L, n_fft, hop, win, center = case
    _say(f"stft complex/phase {name}: B={B} L={L} n_fft={n_fft} hop={hop} win={win} center={center}")
    x = _rand(B, L, 4000 + n_fft)
    re, im = oracle.stft_complex(x, n_fft=n_fft, hop=hop, window=win, center=center)
    plan = nb.nna_plan_stft(n_fft=n_fft, hop=hop, win=win, center=center, fmt=nb.NNA_OUT_COMPLEX, device=0)
    got = nb.nna_stft(plan, _dev(x)).cpu().numpy()
    e = _rel_err(got, oracle.interleave(re, im))
    assert not got[:, 1].any() and not got[:, -1].any()  # Im of bins 0 and N/2
    plan = nb.nna_plan_stft(n_fft=n_fft, hop=hop, win=win, center=center, fmt=nb.NNA_OUT_PHASE, device=0)
    ph = nb.nna_stft(plan, _dev(x)).cpu().numpy()
    assert ph.shape == re.shape and np.abs(ph).max() <= np.pi + 1e-6
    ep = _phase_err(ph[:, 1:-1], re[:, 1:-1], im[:, 1:-1])
    # bins 0 and N/2 are real: phase 0 or +-pi by the sign of Re
    for k in (0, -1):
        strong = np.abs(re[:, k]) > 1e-3 * np.abs(re).max()
        want_pi = re[:, k] < 0
        assert np.all((np.abs(ph[:, k]) > 3.0)[strong] == want_pi[strong])
    _say(f"  complex rel err {e:.3e}, phase err {ep:.3e} rad")
    assert e < TOL and e < 5e-5 and ep < 1e-3


def test_scaled_stft_complex_output(nb):
    _say("scaled stft complex")
    x = _rand(3, 9000, 4100)
    sig = np.array([oracle.freq_sigma(oracle.FREQ_LOG, k, 100.0, 3500.0, 37, 512, 8000) for k in range(37)])
    re, im = oracle.stft_sigma_complex(x, sig, n_fft=512, hop=128)
    plan = nb.nna_plan_stft_scaled(sr=8000, n_fft=512, hop=128, fmt=nb.NNA_OUT_COMPLEX, freq_scale=nb.NNA_FREQ_LOG,
                                   fmin=100.0, fmax=3500.0, freq_bins=37, device=0)
    e = _rel_err(nb.nna_stft(plan, _dev(x)).cpu().numpy(), oracle.interleave(re, im))
    _say(f"  rel err {e:.3e}")
    assert e < TOL and e < 5e-5


# ---------------------------------------------------------------------------------------
# Mel
# ---------------------------------------------------------------------------------------
MEL_CASES = [
    # name, B, L, sr, n_fft, hop, n_mels, fmin, fmax, scale, norm, power
    ("slaney 40 mels", 3, 12000, 16000, 512, 128, 40, 0.0, 0.0, 0, True, 2.0),
    ("htk magnitude", 2, 9000, 8000, 256, 64, 20, 100.0, 3500.0, 1, False, 1.0),
    ("128 mels, ragged", 5, 30000, 22050, 1024, 256, 128, 0.0, 0.0, 0, True, 2.0),
    ("200 mels (two passes)", 2, 20000, 22050, 2048, 512, 200, 30.0, 9000.0, 0, True, 2.0),
    ("fig. 2 set-up", 1, 1000, 1000, 128, 32, 4, 0.0, 500.0, 1, False, 2.0),
    ("hop does not divide n_fft", 2, 8000, 16000, 400, 160, 64, 0.0, 0.0, 0, True, 2.0),
    # the launch split by tap parity: row tiles of 32 bins below N/4, filters met through bins and through partners
    ("split: n_fft 384 (three row tiles), six shifts", 3, 9000, 16000, 384, 64, 30, 0.0, 0.0, 0, True, 2.0),
    ("split: filters below bin N/4 only", 2, 9000, 16000, 512, 128, 24, 50.0, 1500.0, 0, True, 2.0),
    ("split: filters above bin N/4 only (partners)", 2, 9000, 16000, 512, 128, 24, 5000.0, 8000.0, 1, True, 1.0),
    ("split: 300 mels in three band-limited passes, n_fft 4096", 2, 30000, 44100, 4096, 512, 300, 0.0, 0.0, 0, True, 2.0),
]


@pytest.mark.parametrize("case", MEL_CASES, ids=[c[0] for c in MEL_CASES])
def test_mel_parity_small(nb, case):
    name, B, L, sr, n_fft, hop, n_mels, fmin, fmax, scale, norm, power = case
    _say(f"mel {name}: B={B} L={L} sr={sr} n_fft={n_fft} hop={hop} n_mels={n_mels}")
    x = _rand(B, L, 200 + n_mels)
    plan = nb.nna_plan_mel(sr=sr, n_fft=n_fft, hop=hop, n_mels=n_mels, fmin=fmin, fmax=fmax, scale=scale,
                           norm_area=norm, power=power, device=0)
    got = nb.nna_mel(plan, _dev(x)).cpu().numpy()
    ref = oracle.mel(x, sr=sr, n_fft=n_fft, hop=hop, n_mels=n_mels, fmin=fmin, fmax=fmax, scale=scale,
                     norm_area=norm, power=power)
    e = _rel_err(got, ref)
    _say(f"  rel err {e:.3e}")
    assert e < TOL and e < 5e-5


def test_mel_device_weights_equal_host_weights(nb):
    _say("mel weight read-back")
    host = nb.nna_plan_mel_weights(nb.nna_plan_mel(n_mels=200, device=-1))
    dev = nb.nna_plan_mel_weights(nb.nna_plan_mel(n_mels=200, device=0))
    np.testing.assert_array_equal(host, dev)


def test_mel_config2_full(nb):
    wl = signals.WORKLOADS[2]
    _say("mel config 2 (64 x 110250 @ 22050 Hz, 128 mels)")
    x = signals.batch(2)
    plan = nb.nna_plan_mel(sr=wl["sr"], n_fft=2048, hop=512, n_mels=128, fmin=0.0, fmax=11025.0, device=0)
    got = nb.nna_mel(plan, _dev(x)).cpu().numpy()
    assert got.shape == (64, 128, 216)
    ref = oracle.mel(x, sr=wl["sr"], n_fft=2048, hop=512, n_mels=128, fmin=0.0, fmax=11025.0)
    e = _rel_err(got, ref)
    _say(f"  rel err {e:.3e}")
    assert e < TOL


# ---------------------------------------------------------------------------------------
# CQT
# ---------------------------------------------------------------------------------------
CQT_CASES = [
    # name, B, L, sr, hop, fmin, n_bins, bpo, n_taps, win, center, fmt
    ("24 bins, 1024 taps", 2, 6000, 8000, 128, 220.0, 24, 12, 1024, 0, True, 0),
    ("ragged, tiles span waveforms", 7, 5000, 8000, 64, 220.0, 30, 12, 1024, 0, True, 1),
    ("odd bin count, default taps", 2, 9000, 8000, 128, 300.0, 13, 6, 0, 0, True, 0),
    ("hop does not divide taps", 2, 6000, 8000, 100, 220.0, 30, 12, 1000, 0, True, 0),
    ("hop not a multiple of 16", 2, 6000, 8000, 48, 300.0, 13, 6, 0, 0, False, 0),
    ("rect window, no centring", 2, 7000, 8000, 128, 500.0, 6, 3, 128, 1, False, 0),
    ("short waveforms, many per tile", 40, 1100, 8000, 128, 220.0, 24, 12, 1024, 0, True, 0),
    ("36 bins per octave", 2, 30000, 22050, 256, 110.0, 100, 36, 0, 0, True, 0),
    ("Hamming-windowed kernels", 2, 6000, 8000, 128, 220.0, 24, 12, 1024, 2, True, 0),
    ("Blackman-windowed kernels", 2, 6000, 8000, 128, 220.0, 24, 12, 1024, 3, True, 0),
    # a hop that divides the 16-tap chunk (deep octaves of a downsampling plan): rows step by one hop, shifts by 16 taps
    ("hop 8 (two LDS rows per 16-tap shift)", 3, 3000, 8000, 8, 500.0, 20, 12, 512, 0, True, 0),
    ("hop 4, short kernels", 2, 1500, 8000, 4, 1000.0, 12, 12, 256, 0, True, 1),
    ("hop 8, tiles span waveforms, no centring", 9, 700, 8000, 8, 700.0, 14, 12, 256, 1, False, 0),
    # hop 441 does not divide 65,536 taps: one chunk per 16 taps of a 46,025-tap kernel, 2,878 chunk
    # descriptors per work item -- more than the kernel keeps in LDS at a time (ring of 512)
    ("46,025-tap kernels whose frames do not overlap in LDS", 2, 40000, 44100, 441, 32.70, 30, 24, 0, 0, True, 0),
    ("the same, chunk count just past one ring refill", 1, 9000, 44100, 441, 130.0, 6, 24, 0, 0, True, 1),
]


@pytest.mark.parametrize("case", CQT_CASES, ids=[c[0] for c in CQT_CASES])
def test_cqt_parity_small(nb, case):
    name, B, L, sr, hop, fmin, n_bins, bpo, taps, win, center, fmt = case
    _say(f"cqt {name}: B={B} L={L} sr={sr} hop={hop} bins={n_bins}/{bpo} taps={taps}")
    x = _rand(B, L, 300 + n_bins)
    plan = nb.nna_plan_cqt(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, win=win, center=center,
                           n_taps=taps, fmt=fmt, device=0)
    got = nb.nna_cqt(plan, _dev(x)).cpu().numpy()
    ref = oracle.cqt(x, sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, window=win, center=center,
                     n_taps=taps, fmt=fmt)
    e = _rel_err(got, ref)
    _say(f"  rel err {e:.3e}")
    assert e < TOL and e < 5e-5


@pytest.mark.parametrize("case", [CQT_CASES[1], CQT_CASES[2], CQT_CASES[3], CQT_CASES[6]], ids=lambda c: c[0])
def test_cqt_complex_and_phase_output(nb, case):
    name, B, L, sr, hop, fmin, n_bins, bpo, taps, win, center, _ = case
    _say(f"cqt complex/phase {name}: B={B} L={L} sr={sr} hop={hop} bins={n_bins}/{bpo} taps={taps}")
    x = _rand(B, L, 300 + n_bins)
    kw = dict(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, center=center, n_taps=taps)
    re, im = oracle.cqt_complex(x, window=win, **kw)
    got = nb.nna_cqt(nb.nna_plan_cqt(win=win, fmt=nb.NNA_OUT_COMPLEX, device=0, **kw), _dev(x)).cpu().numpy()
    e = _rel_err(got, oracle.interleave(re, im))
    ph = nb.nna_cqt(nb.nna_plan_cqt(win=win, fmt=nb.NNA_OUT_PHASE, device=0, **kw), _dev(x)).cpu().numpy()
    ep = _phase_err(ph, re, im)
    _say(f"  complex rel err {e:.3e}, phase err {ep:.3e} rad")
    assert e < TOL and e < 5e-5 and ep < 1e-3


# Plans whose kernels run folded about their centres (many bins per octave, kernels of eight hops or more): the
# blocks of the folded bank hold bins of one length parity, tiles come in pairs (behind / in front of the frame
# centre), and the epilogue turns the two sums back by the kernels' common phase.
CQT_FOLD_CASES = [
    # name, B, L, sr, hop, fmin, n_bins, bpo, win, center, fmt
    # (lengths that are no multiples of four: the mirrored samples at the waveform's ends straddle the loader's windows)
    ("36 per octave, 64 hop-shifts, tiles span waveforms", 3, 9002, 8000, 32, 200.0, 60, 36, 0, True, 0),
    ("Blackman kernels, no centring, power", 2, 9000, 8000, 32, 200.0, 60, 36, 3, False, 1),
    ("48 per octave, ragged batch, no centring", 5, 4000, 8000, 64, 300.0, 33, 48, 0, False, 0),
    ("waveforms of 36 frames, eight to a tile", 20, 4501, 16000, 128, 100.0, 40, 24, 0, True, 2),
]


def _fold_plan(nb, case, fmt=None, trainable=False):
    name, B, L, sr, hop, fmin, n_bins, bpo, win, center, f = case
    plan = nb.nna_plan_cqt(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, win=win, center=center,
                           n_taps=0, fmt=f if fmt is None else fmt, device=0)
    return nb.nna_plan_trainable(plan) if trainable else plan


@pytest.mark.parametrize("case", CQT_FOLD_CASES, ids=[c[0] for c in CQT_FOLD_CASES])
def test_cqt_folded_kernels_parity(nb, case):
    name, B, L, sr, hop, fmin, n_bins, bpo, win, center, fmt = case
    _say(f"cqt folded {name}: B={B} L={L} sr={sr} hop={hop} bins={n_bins}/{bpo}")
    x = _rand(B, L, 700 + n_bins)
    plan = _fold_plan(nb, case)
    info = plan.info()
    # the plan does run the folded kernel: it multiplies less than the direct form's 4 sum N_k
    assert info["executed_flops_per_frame"] < info["algorithmic_flops_per_frame"]
    got = nb.nna_cqt(plan, _dev(x)).cpu().numpy()
    ref = oracle.cqt(x, sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, window=win, center=center,
                     n_taps=0, fmt=fmt)
    e = _rel_err(got, ref)
    _say(f"  rel err {e:.3e}")
    assert e < TOL and e < 5e-5


@pytest.mark.parametrize("case", [CQT_FOLD_CASES[0], CQT_FOLD_CASES[2], CQT_FOLD_CASES[3]], ids=lambda c: c[0])
def test_cqt_folded_kernels_complex_and_phase_output(nb, case):
    name, B, L, sr, hop, fmin, n_bins, bpo, win, center, _ = case
    _say(f"cqt folded complex/phase {name}")
    x = _rand(B, L, 700 + n_bins)
    re, im = oracle.cqt_complex(x, sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, window=win,
                                center=center, n_taps=0)
    got = nb.nna_cqt(_fold_plan(nb, case, fmt=nb.NNA_OUT_COMPLEX), _dev(x)).cpu().numpy()
    e = _rel_err(got, oracle.interleave(re, im))
    ph = nb.nna_cqt(_fold_plan(nb, case, fmt=nb.NNA_OUT_PHASE), _dev(x)).cpu().numpy()
    ep = _phase_err(ph, re, im)
    _say(f"  complex rel err {e:.3e}, phase err {ep:.3e} rad")
    assert e < TOL and e < 5e-5 and ep < 1e-3


def test_cqt_folded_and_direct_kernels_agree(nb):
    # the same plan made trainable keeps its kernels as free parameters and runs the direct kernel
    case = CQT_FOLD_CASES[0]
    _say("cqt folded against direct kernel")
    x = _dev(_rand(case[1], case[2], 77))
    folded, direct = _fold_plan(nb, case, fmt=nb.NNA_OUT_COMPLEX), _fold_plan(nb, case, fmt=nb.NNA_OUT_COMPLEX, trainable=True)
    assert folded.info()["executed_flops_per_frame"] < 0.75 * direct.info()["executed_flops_per_frame"]
    a, b = nb.nna_cqt(folded, x).cpu().numpy(), nb.nna_cqt(direct, x).cpu().numpy()
    e = float(np.max(np.abs(a - b)) / np.max(np.abs(b)))
    _say(f"  rel diff {e:.3e}")
    assert e < 2e-5


def test_cqt_device_bank_equals_host_bank(nb):
    _say("cqt bank read-back")
    kw = dict(sr=8000, hop=128, fmin=220.0, n_bins=24, bins_per_octave=12, n_taps=1024)
    host = nb.nna_plan_bank(nb.nna_plan_cqt(device=-1, **kw))
    dev = nb.nna_plan_bank(nb.nna_plan_cqt(device=0, **kw))
    np.testing.assert_array_equal(host, dev)


def test_cqt_config3_full(nb):
    wl = signals.WORKLOADS[3]
    _say("cqt config 3 (16 x 220500 @ 22050 Hz, 84 bins, 16384 taps)")
    x = signals.batch(3)
    plan = nb.nna_plan_cqt(sr=wl["sr"], hop=512, fmin=32.70, n_bins=84, bins_per_octave=12, n_taps=16384, device=0)
    got = nb.nna_cqt(plan, _dev(x)).cpu().numpy()
    assert got.shape == (16, 84, 431)
    ref = oracle.cqt(x, sr=wl["sr"], hop=512, fmin=32.70, n_bins=84, bins_per_octave=12, n_taps=16384)
    e = _rel_err(got, ref)
    _say(f"  rel err {e:.3e}")
    assert e < TOL


def test_cqt_tone_closed_form_on_gpu(nb):
    # a tone with exactly Q cycles per kernel reads A/2 (the closed form that pins the oracle)
    _say("cqt closed form tone")
    sr, fmin, nbins, bpo, taps, A, k = 22050, 32.70, 84, 12, 16384, 0.6, 40
    Nk, _ = oracle.cqt_lengths(sr, fmin, nbins, bpo)
    x = signals.tone(3 * taps, sr, oracle.cqt_Q(bpo) * sr / Nk[k], amp=A, phase=0.9)[None]
    plan = nb.nna_plan_cqt(sr=sr, hop=512, fmin=fmin, n_bins=nbins, bins_per_octave=bpo, n_taps=taps, device=0)
    got = nb.nna_cqt(plan, _dev(x)).cpu().numpy()[0][:, 20:-20]
    assert np.all(np.argmax(got, axis=0) == k)
    assert np.max(np.abs(got[k] - A / 2)) < 1e-3 * A / 2


# ---------------------------------------------------------------------------------------
# STFT with float16 operands (float32 accumulation): same bar, 1e-3 of the peak
# ---------------------------------------------------------------------------------------
STFT16_CASES = [
    # name, B, L, n_fft, hop, window, center, fmt
    ("one tile, one waveform", 1, 8000, 256, 64, 0, True, 0),
    ("several tiles, ragged tail, tiles span waveforms", 5, 30000, 256, 64, 0, True, 0),
    ("many short waveforms per tile, power", 37, 700, 256, 64, 0, True, 1),
    ("single-frame waveforms (T=1)", 9, 40, 64, 64, 0, True, 0),
    ("hop = n_fft / 2, rect window, no centring", 2, 9000, 512, 256, 1, False, 1),
    ("L not a multiple of 4 (unaligned rows), log", 3, 22050, 512, 128, 0, True, 2),
    ("row tiles: 1,025 bins", 2, 12000, 2048, 512, 0, True, 0),
    ("32 hop-shifts", 2, 9000, 1024, 32, 0, True, 0),
    ("8 hop-shifts, three row tiles", 4, 20000, 768, 96, 0, True, 0),
]


@pytest.mark.parametrize("case", STFT16_CASES, ids=[c[0] for c in STFT16_CASES])
def test_stft_f16_parity_small(nb, case):
    name, B, L, n_fft, hop, win, center, fmt = case
    _say(f"stft f16 {name}: B={B} L={L} n_fft={n_fft} hop={hop} win={win} center={center} fmt={fmt}")
    x = _rand(B, L, 1600 + n_fft + hop)
    plan = nb.nna_plan_stft_prec(n_fft=n_fft, hop=hop, win=win, center=center, fmt=fmt, precision=nb.NNA_PREC_F16,
                                 device=0)
    got = nb.nna_stft(plan, _dev(x)).cpu().numpy()
    ref = oracle.stft(x, n_fft=n_fft, hop=hop, window=win, center=center, fmt=fmt)
    if fmt == 2:
        # ln amplifies the error of small powers without bound: compare the magnitudes it encodes
        got, ref = np.exp(0.5 * got.astype(np.float64)), np.exp(0.5 * ref)
    e = _rel_err(got, ref)
    _say(f"  rel err {e:.3e}")
    assert e < TOL


def test_stft_f16_unsupported_shapes(nb):
    for n_fft, hop in ((96, 25), (240, 48), (2048, 16)):
        with pytest.raises(nb.NnaError) as e:
            nb.nna_plan_stft_prec(n_fft=n_fft, hop=hop, precision=nb.NNA_PREC_F16, device=0)
        assert e.value.status == nb.NNA_ERR_UNSUPPORTED


# ---------------------------------------------------------------------------------------
# CQT by recursive downsampling
# ---------------------------------------------------------------------------------------
CQT2010_CASES = [
    # name, B, L, sr, hop, fmin, n_bins, bpo, n_taps, fir_taps, fmt
    ("defaults: 7 octaves of 12 bins", 2, 22050, 22050, 512, 32.70, 84, 12, 0, 0, 0),
    ("partial lowest octave, short filter", 3, 6000, 16000, 64, 220.0, 29, 12, 0, 63, 0),
    ("single octave: no filter, no workspace", 2, 9000, 16000, 128, 1000.0, 12, 12, 0, 0, 1),
    ("odd lengths at every octave (scalar stores, unaligned rows)", 2, 22051, 22050, 256, 65.41, 48, 12, 0, 129, 0),
    ("many short waveforms per tile, log output", 37, 3000, 16000, 32, 500.0, 16, 4, 0, 31, 2),
    ("24 bins per octave, explicit taps", 2, 30000, 44100, 128, 523.25, 72, 24, 2048, 257, 0),
]


@pytest.mark.parametrize("case", CQT2010_CASES, ids=[c[0] for c in CQT2010_CASES])
def test_cqt2010v2_parity_small(nb, case):
    name, B, L, sr, hop, fmin, n_bins, bpo, n_taps, fir_taps, fmt = case
    _say(f"cqt2010v2 {name}: B={B} L={L} sr={sr} hop={hop} bins={n_bins}/{bpo} taps={n_taps} fir={fir_taps} fmt={fmt}")
    x = _rand(B, L, 2010 + n_bins)
    plan = nb.nna_plan_cqt2010v2(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, n_taps=n_taps,
                                 fir_taps=fir_taps, fmt=fmt, device=0)
    got = nb.nna_cqt2010v2(plan, _dev(x)).cpu().numpy()
    ref = oracle.cqt2010v2(x, sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, n_taps=n_taps,
                           fir_taps=fir_taps or oracle.FIR_TAPS, fmt=fmt)
    e = _rel_err(got, ref)
    # every octave against its own peak too: the low octaves of noise are much weaker than the top
    n_oct = -(-n_bins // bpo)
    for a in range(n_oct):
        hi = n_bins - a * bpo
        lo = max(0, hi - bpo)
        e = max(e, _rel_err(got[:, lo:hi], ref[:, lo:hi]))
    _say(f"  rel err {e:.3e}")
    assert e < TOL


def _octave_complex_errs(got_c, got_ph, re, im, n_bins, bpo):
    """complex-format error (every octave against its own peak too) and phase error per octave (the octaves of one
    signal differ by orders of magnitude: each is judged on its own strong bins)"""
    ref = oracle.interleave(re, im)
    e, ep = _rel_err(got_c, ref), 0.0
    for a in range(-(-n_bins // bpo)):
        hi = n_bins - a * bpo
        lo = max(0, hi - bpo)
        e = max(e, _rel_err(got_c[:, 2 * lo:2 * hi], ref[:, 2 * lo:2 * hi]))
        ep = max(ep, _phase_err(got_ph[:, lo:hi], re[:, lo:hi], im[:, lo:hi]))
    return e, ep


@pytest.mark.parametrize("case", [CQT2010_CASES[0], CQT2010_CASES[1], CQT2010_CASES[3], CQT2010_CASES[4]], ids=lambda c: c[0])
def test_cqt2010v2_complex_and_phase_output(nb, case):
    name, B, L, sr, hop, fmin, n_bins, bpo, n_taps, fir_taps, _ = case
    _say(f"cqt2010v2 complex/phase {name}: B={B} L={L} sr={sr} hop={hop} bins={n_bins}/{bpo} fir={fir_taps}")
    x = _rand(B, L, 2010 + n_bins)
    kw = dict(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, n_taps=n_taps)
    re, im = oracle.cqt2010v2_complex(x, fir_taps=fir_taps or oracle.FIR_TAPS, **kw)
    pc = nb.nna_plan_cqt2010v2(fir_taps=fir_taps, fmt=nb.NNA_OUT_COMPLEX, device=0, **kw)
    assert nb.nna_out_shape(pc, B, L) == (2 * n_bins, 1 + L // hop)
    got = _poisoned(B, 2 * n_bins, 1 + L // hop)
    nb.nna_cqt2010v2(pc, _dev(x), out=got)
    got = got.cpu().numpy()
    assert np.isfinite(got).all()
    ph = nb.nna_cqt2010v2(nb.nna_plan_cqt2010v2(fir_taps=fir_taps, fmt=nb.NNA_OUT_PHASE, device=0, **kw), _dev(x)).cpu().numpy()
    assert ph.shape == (B, n_bins, 1 + L // hop)
    e, ep = _octave_complex_errs(got, ph, re, im, n_bins, bpo)
    _say(f"  complex rel err {e:.3e}, phase err {ep:.3e} rad")
    assert e < TOL and ep < 1e-3


def test_cqt2010v2_tone_closed_form_on_gpu(nb):
    # a tone on bin k reads A/2 in whichever octave k falls (filter ripple and kernel detuning: 1 %)
    _say("cqt2010v2 closed form tones")
    sr, A = 22050, 0.6
    _, fk = oracle.cqt_lengths(sr, 32.70, 84, 12)
    ks = [3, 30, 50, 71, 83]
    x = np.stack([signals.tone(22050, sr, fk[k], amp=A) for k in ks])
    plan = nb.nna_plan_cqt2010v2(sr=sr, device=0)
    got = nb.nna_cqt2010v2(plan, _dev(x)).cpu().numpy()
    for i, k in enumerate(ks):
        mid = got[i, :, 15:30]
        assert np.all(mid.argmax(axis=0) == k)
        assert np.allclose(mid[k], A / 2, rtol=1e-2)


def test_cqt2010v2_workspace_and_shape_checks(nb):
    import torch
    plan = nb.nna_plan_cqt2010v2(sr=22050, device=0)
    x = torch.zeros((2, 22050), device="cuda:0")
    need = nb.nna_cqt2010v2_workspace(plan, 2, 22050)
    assert need >= 4 * 2 * (11025 + 5513)
    with pytest.raises(nb.NnaError) as e:
        nb.nna_cqt2010v2(plan, x, workspace=torch.empty(need - 256, dtype=torch.uint8, device="cuda:0"))
    assert e.value.status == nb.NNA_ERR_INVALID_ARG
    with pytest.raises(nb.NnaError) as e:
        nb.nna_cqt2010v2(plan, torch.zeros((2, 4000), device="cuda:0"))  # the deepest octave would have 63 samples
    assert e.value.status == nb.NNA_ERR_SHAPE
    with pytest.raises(nb.NnaError):
        nb.nna_cqt(plan, x)  # wrong entry point for this plan
    # a caller-owned workspace is enough, and is reusable
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    a = nb.nna_cqt2010v2(plan, x + 0.25, workspace=ws)
    b = nb.nna_cqt2010v2(plan, x + 0.25, workspace=ws)
    assert torch.equal(a, b)


def test_cqt2010v2_one_plan_two_host_threads_two_streams(nb):
    """The octave loop forks onto streams the plan owns and joins them again; calls on one plan from two host
    threads, each on a stream and with a workspace of its own, must give what the calls give one after the other."""
    import threading
    import torch
    _say("cqt2010v2: one plan, two host threads on two streams")
    plan = nb.nna_plan_cqt2010v2(sr=22050, hop=256, fmin=110.0, n_bins=48, bins_per_octave=12, device=0)
    B, L = 6, 30000
    xs = [_dev(_rand(B, L, 4100 + i)) for i in range(2)]
    need = nb.nna_cqt2010v2_workspace(plan, B, L)
    expect = [nb.nna_cqt2010v2(plan, x) for x in xs]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(device="cuda:0") for _ in range(2)]
    wss = [torch.empty(need, dtype=torch.uint8, device="cuda:0") for _ in range(2)]
    outs = [torch.full_like(e, float("nan")) for e in expect]
    torch.cuda.synchronize()
    errors = []

    def work(i):
        try:
            for _ in range(20):
                nb.nna_cqt2010v2(plan, xs[i], out=outs[i], workspace=wss[i], stream=streams[i].cuda_stream)
        except Exception as e:  # noqa: BLE001 -- reported by the asserting thread
            errors.append(e)

    threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for got, want in zip(outs, expect):
        assert torch.equal(got, want)


# ---------------------------------------------------------------------------------------
# CQT with frequency-domain kernels (un-windowed STFT x spectral kernels, one kernel)
# ---------------------------------------------------------------------------------------
CQT1992_CASES = [
    # name, B, L, sr, hop, fmin, n_bins, bpo, n_fft, win, center, fmt
    ("36 bins, 2048 taps, one pass", 2, 9000, 22050, 256, 220.0, 36, 12, 0, 0, True, 0),
    ("70 bins: one pass of six 32-row blocks, ragged, tiles span waveforms", 5, 9000, 8000, 64, 55.0, 70, 12, 0, 0, True, 0),
    ("100 bins: two passes of four blocks", 3, 9000, 16000, 64, 200.0, 100, 24, 0, 0, True, 0),
    ("odd bin count, power output, padded n_fft", 2, 12000, 8000, 128, 300.0, 13, 6, 1024, 0, True, 1),
    ("hop does not divide n_fft", 2, 6000, 8000, 100, 220.0, 30, 12, 1024, 0, True, 0),
    ("rect kernels, no centring, log output", 2, 7000, 8000, 128, 500.0, 6, 3, 128, 1, False, 2),
    ("short waveforms, many per tile", 40, 1100, 8000, 128, 220.0, 24, 12, 1024, 0, True, 0),
    ("150 bins: two passes of six blocks, 4096 taps", 2, 20000, 22050, 512, 110.0, 150, 24, 0, 0, True, 0),
    ("8192 taps, 16 hop-shifts", 1, 30000, 22050, 512, 65.41, 40, 12, 0, 0, True, 0),
]


@pytest.mark.parametrize("case", CQT1992_CASES, ids=[c[0] for c in CQT1992_CASES])
def test_cqt1992_parity_small(nb, case):
    name, B, L, sr, hop, fmin, n_bins, bpo, n_fft, win, center, fmt = case
    _say(f"cqt1992 {name}: B={B} L={L} sr={sr} hop={hop} bins={n_bins}/{bpo} n_fft={n_fft}")
    x = _rand(B, L, 700 + n_bins)
    plan = nb.nna_plan_cqt1992(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, win=win,
                               center=center, n_fft=n_fft, fmt=fmt, device=0)
    got = nb.nna_cqt1992(plan, _dev(x)).cpu().numpy()
    ref = oracle.cqt1992(x, sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, window=win, center=center,
                         n_fft=n_fft, fmt=fmt)
    if fmt == 2:
        # log output: compare where the power is above -60 dB of the peak (below, float32 rounding of a
        # near-zero power is amplified without bound by the logarithm)
        pw = oracle.cqt1992(x, sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, window=win,
                            center=center, n_fft=n_fft, fmt=1)
        keep = pw > 1e-6 * pw.max()
        e = np.abs(got - ref)[keep].max()
    else:
        e = _rel_err(got, ref)
    _say(f"  rel err {e:.3e}")
    assert e < TOL and e < 5e-5


@pytest.mark.parametrize("case", [CQT1992_CASES[1], CQT1992_CASES[2], CQT1992_CASES[3], CQT1992_CASES[7]], ids=lambda c: c[0])
def test_cqt1992_complex_and_phase_output(nb, case):
    name, B, L, sr, hop, fmin, n_bins, bpo, n_fft, win, center, _ = case
    _say(f"cqt1992 complex/phase {name}: B={B} L={L} sr={sr} hop={hop} bins={n_bins}/{bpo} n_fft={n_fft}")
    x = _rand(B, L, 700 + n_bins)
    kw = dict(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, center=center, n_fft=n_fft)
    ref = oracle.cqt1992(x, window=win, fmt=oracle.COMPLEX, **kw)
    pc = nb.nna_plan_cqt1992(win=win, fmt=nb.NNA_OUT_COMPLEX, device=0, **kw)
    got = _poisoned(*ref.shape)
    nb.nna_cqt1992(pc, _dev(x), out=got)
    got = got.cpu().numpy()
    assert np.isfinite(got).all()
    e = _rel_err(got, ref)
    ph = nb.nna_cqt1992(nb.nna_plan_cqt1992(win=win, fmt=nb.NNA_OUT_PHASE, device=0, **kw), _dev(x)).cpu().numpy()
    ep = _phase_err(ph, ref[:, 0::2], ref[:, 1::2])
    _say(f"  complex rel err {e:.3e}, phase err {ep:.3e} rad")
    assert e < TOL and e < 5e-5 and ep < 1e-3


def test_cqt1992_device_kernels_equal_host_kernels(nb):
    _say("cqt1992 spectral kernels and DFT bank read-back")
    kw = dict(sr=8000, hop=64, fmin=55.0, n_bins=70, bins_per_octave=12)
    host, dev = nb.nna_plan_cqt1992(device=-1, **kw), nb.nna_plan_cqt1992(device=0, **kw)
    np.testing.assert_array_equal(nb.nna_plan_spectral_kernels(host), nb.nna_plan_spectral_kernels(dev))
    np.testing.assert_array_equal(nb.nna_plan_bank(host), nb.nna_plan_bank(dev))


def test_cqt1992_tone_closed_form_and_time_domain_cqt_on_gpu(nb):
    # a tone of exactly Q cycles per kernel reads A/2; and the whole output stays within the dropped
    # half's share (1e-4 of the peak for this set-up) of the time-domain kernels' result
    _say("cqt1992 tone closed form")
    sr, fmin, n_bins, bpo, hop, A = 22050, 220.0, 36, 12, 256, 0.6
    Nk, _ = oracle.cqt_lengths(sr, fmin, n_bins, bpo)
    q = 17
    f = oracle.cqt_Q(bpo) * sr / Nk[q]
    x = signals.tone(4 * 2048, sr, f, amp=A, phase=1.1)[None, :]
    kw = dict(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, device=0)
    got = nb.nna_cqt1992(nb.nna_plan_cqt1992(**kw), _dev(x)).cpu().numpy()[0]
    mid = got[:, got.shape[1] // 2]
    assert int(np.argmax(mid)) == q and abs(mid[q] - A / 2) < 1e-4 * A
    time_domain = nb.nna_cqt(nb.nna_plan_cqt(**kw), _dev(x)).cpu().numpy()[0]
    assert np.abs(got - time_domain).max() < 2e-4 * time_domain.max()


def test_cqt1992_rejects_wrong_plan_and_short_input(nb):
    _say("cqt1992 error paths")
    plan = nb.nna_plan_cqt1992(sr=8000, hop=64, fmin=220.0, n_bins=24, device=0)
    with pytest.raises(nb.NnaError) as ei:
        nb.nna_cqt1992(plan, _dev(_rand(1, 400, 1)))  # L <= n_fft / 2
    assert ei.value.status == nb.NNA_ERR_SHAPE
    with pytest.raises(nb.NnaError) as ei:
        nb.nna_cqt(plan, _dev(_rand(1, 4000, 1)))
    assert ei.value.status == nb.NNA_ERR_INVALID_ARG


@pytest.mark.parametrize("case", CQT2010_CASES, ids=[c[0] for c in CQT2010_CASES])
def test_cqt2010_parity_small(nb, case):
    # the same shapes as the time-domain flavour (its n_taps, where given, is a power of two and serves as n_fft)
    name, B, L, sr, hop, fmin, n_bins, bpo, n_fft, fir_taps, fmt = case
    _say(f"cqt2010 {name}: B={B} L={L} sr={sr} hop={hop} bins={n_bins}/{bpo} n_fft={n_fft} fir={fir_taps} fmt={fmt}")
    x = _rand(B, L, 2010 + n_bins)
    plan = nb.nna_plan_cqt2010(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, n_fft=n_fft,
                               fir_taps=fir_taps, fmt=fmt, device=0)
    got = nb.nna_cqt2010(plan, _dev(x)).cpu().numpy()
    kw = dict(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, n_fft=n_fft,
              fir_taps=fir_taps or oracle.FIR_TAPS)
    ref = oracle.cqt2010(x, fmt=fmt, **kw)
    if fmt == 2:
        # log output: compare the magnitudes it encodes (ln amplifies the error of small powers without bound)
        got, ref = np.exp(0.5 * got.astype(np.float64)), np.exp(0.5 * ref)
    e = _rel_err(got, ref)
    n_oct = -(-n_bins // bpo)
    for a in range(n_oct):  # every octave against its own peak too
        hi = n_bins - a * bpo
        lo = max(0, hi - bpo)
        e = max(e, _rel_err(got[:, lo:hi], ref[:, lo:hi]))
    _say(f"  rel err {e:.3e}")
    assert e < TOL


@pytest.mark.parametrize("case", [CQT2010_CASES[0], CQT2010_CASES[1], CQT2010_CASES[3], CQT2010_CASES[4]], ids=lambda c: c[0])
def test_cqt2010_complex_and_phase_output(nb, case):
    name, B, L, sr, hop, fmin, n_bins, bpo, n_fft, fir_taps, _ = case
    _say(f"cqt2010 complex/phase {name}: B={B} L={L} sr={sr} hop={hop} bins={n_bins}/{bpo} fir={fir_taps}")
    x = _rand(B, L, 2010 + n_bins)
    kw = dict(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, n_fft=n_fft)
    ref = oracle.cqt2010(x, fir_taps=fir_taps or oracle.FIR_TAPS, fmt=oracle.COMPLEX, **kw)
    re, im = ref[:, 0::2], ref[:, 1::2]
    got = _poisoned(*ref.shape)
    nb.nna_cqt2010(nb.nna_plan_cqt2010(fir_taps=fir_taps, fmt=nb.NNA_OUT_COMPLEX, device=0, **kw), _dev(x), out=got)
    got = got.cpu().numpy()
    assert np.isfinite(got).all()
    ph = nb.nna_cqt2010(nb.nna_plan_cqt2010(fir_taps=fir_taps, fmt=nb.NNA_OUT_PHASE, device=0, **kw), _dev(x)).cpu().numpy()
    e, ep = _octave_complex_errs(got, ph, re, im, n_bins, bpo)
    _say(f"  complex rel err {e:.3e}, phase err {ep:.3e} rad")
    assert e < TOL and ep < 1e-3


def test_cqt2010_tone_closed_form_and_wrong_entry_point_on_gpu(nb):
    _say("cqt2010 closed form tones")
    sr, A = 22050, 0.6
    _, fk = oracle.cqt_lengths(sr, 32.70, 84, 12)
    ks = [3, 30, 50, 71, 83]
    x = _dev(np.stack([signals.tone(22050, sr, fk[k], amp=A) for k in ks]))
    plan = nb.nna_plan_cqt2010(sr=sr, device=0)
    got = nb.nna_cqt2010(plan, x).cpu().numpy()
    for i, k in enumerate(ks):
        mid = got[i, :, 15:30]
        assert np.all(mid.argmax(axis=0) == k)
        assert np.allclose(mid[k], A / 2, rtol=1e-2)
    with pytest.raises(nb.NnaError) as e:
        nb.nna_cqt2010v2(plan, x)
    assert e.value.status == nb.NNA_ERR_INVALID_ARG
    with pytest.raises(nb.NnaError) as e:
        nb.nna_cqt2010(plan, x[:, :4000].contiguous())  # the deepest octave would have 63 samples
    assert e.value.status == nb.NNA_ERR_SHAPE


# ---------------------------------------------------------------------------------------
# The two 1,770-waveform workloads at full size, in the launch configuration the bench times.
# Every output (and workspace) starts out as NaN, so an element no workgroup writes stays NaN and fails
# the finiteness check over all 1,770 waveforms; the oracle checks whole waveforms chosen from the kernel's
# own tile walk (tests/tile_sample.py): every XCD's range, a group boundary and the partial last group.
# ---------------------------------------------------------------------------------------
SAMPLED = sampled_waveforms(1770, 345)


def _full_batch(cfg_id):
    import torch
    wl = signals.WORKLOADS[cfg_id]
    x = torch.empty((wl["B"], wl["L"]), dtype=torch.float32, device="cuda:0")
    step = 128
    for s in range(0, wl["B"], step):
        idx = list(range(s, min(wl["B"], s + step)))
        x[s:s + len(idx)] = torch.from_numpy(signals.batch(cfg_id, idx)).to("cuda:0")
    return x


def _poisoned(*shape):
    import torch
    return torch.full(shape, float("nan"), dtype=torch.float32, device="cuda:0")


def _poisoned_bytes(n):
    import torch
    return torch.full(((max(n, 16) + 3) // 4,), float("nan"), dtype=torch.float32, device="cuda:0").view(torch.uint8)


@pytest.fixture(scope="module")
def batch4():
    return _full_batch(4)


def test_sample_covers_every_xcd_range():
    # 4,771 tiles of 128 frames, 597 per XCD: each XCD's range holds at least three sampled waveforms
    assert len(SAMPLED) >= 24 + 5 and SAMPLED[0] == 0 and SAMPLED[-1] == 1769
    n_ft = -(-1770 * 345 // 128)
    per = -(-n_ft // 8)
    for xcd in range(8):
        lo, hi = xcd * per * 128 // 345, min(1769, (min(n_ft, (xcd + 1) * per) * 128 - 1) // 345)
        assert sum(lo <= b <= hi for b in SAMPLED) >= 3, (xcd, lo, hi)


def test_stft_config4_full_sampled(nb, batch4):
    import torch
    _say(f"stft config 4 (1770 x 176400 @ 44100 Hz), {len(SAMPLED)} sampled waveforms")
    plan = nb.nna_plan_stft(sr=44100, n_fft=2048, hop=512, device=0)
    out = nb.nna_stft(plan, batch4, out=_poisoned(1770, 1025, 345))
    torch.cuda.synchronize()
    assert torch.isfinite(out).all() and (out >= 0).all()  # every element was written
    xs = signals.batch(4, SAMPLED)
    ref = oracle.stft(xs, n_fft=2048, hop=512)
    got = out[SAMPLED].cpu().numpy()
    e = _rel_err(got, ref)
    _say(f"  rel err {e:.3e}")
    assert e < TOL
    # every waveform, no oracle needed: the batch cut into three launches of other sizes (other tile walks:
    # 1,595 / 1,591 / 1,588 tiles instead of 4,771) gives the same bits
    for lo, hi in ((0, 590), (590, 1180), (1180, 1770)):
        part = nb.nna_stft(plan, batch4[lo:hi], out=_poisoned(hi - lo, 1025, 345))
        assert torch.equal(part, out[lo:hi]), (lo, hi)


def test_mel_config4_full_sampled(nb, batch4):
    import torch
    _say(f"mel config 4 (1770 x 176400 @ 44100 Hz, 128 mels), {len(SAMPLED)} sampled waveforms")
    plan = nb.nna_plan_mel(sr=44100, n_fft=2048, hop=512, n_mels=128, fmin=0.0, fmax=22050.0, device=0)
    out = nb.nna_mel(plan, batch4, out=_poisoned(1770, 128, 345))
    torch.cuda.synchronize()
    assert torch.isfinite(out).all() and (out >= 0).all()
    xs = signals.batch(4, SAMPLED)
    ref = oracle.mel(xs, sr=44100, n_fft=2048, hop=512, n_mels=128, fmin=0.0, fmax=22050.0)
    e = _rel_err(out[SAMPLED].cpu().numpy(), ref)
    _say(f"  rel err {e:.3e}")
    assert e < TOL
    for lo, hi in ((0, 590), (590, 1770)):
        part = nb.nna_mel(plan, batch4[lo:hi], out=_poisoned(hi - lo, 128, 345))
        assert torch.equal(part, out[lo:hi]), (lo, hi)
    # the same batch through the launch that also writes the power spectrogram (the direct contraction, where
    # nna_mel folds its frames: the two agree to rounding, not bit for bit), and the spectrogram the oracle's
    # STFT gives
    _say("mel + spectrogram in one launch, config 4")
    mel2, spec = nb.nna_mel_with_stft(plan, batch4, out=_poisoned(1770, 128, 345), spec=_poisoned(1770, 1025, 345))
    torch.cuda.synchronize()
    assert torch.isfinite(mel2).all() and torch.isfinite(spec).all()
    assert float((mel2 - out).abs().max()) < 2e-5 * float(out.max())
    e = _rel_err(mel2[SAMPLED].cpu().numpy(), ref)
    _say(f"  mel rel err {e:.3e}")
    assert e < TOL
    e = _rel_err(spec[SAMPLED].cpu().numpy(), oracle.stft(xs, n_fft=2048, hop=512, fmt=oracle.POWER))
    _say(f"  spectrogram rel err {e:.3e}")
    assert e < TOL


def test_cqt_config5_full_sampled(nb):
    import torch
    _say(f"cqt config 5 (1770 x 176400 @ 44100 Hz, 168 bins, 65536 taps), {len(SAMPLED)} sampled waveforms")
    x = _full_batch(5)
    plan = nb.nna_plan_cqt(sr=44100, hop=512, fmin=32.70, n_bins=168, bins_per_octave=24, n_taps=0, device=0)
    assert plan.info()["taps"] == 65536
    out = nb.nna_cqt(plan, x, out=_poisoned(1770, 168, 345))
    torch.cuda.synchronize()
    assert torch.isfinite(out).all() and (out >= 0).all()
    xs = signals.batch(5, SAMPLED)
    ref = oracle.cqt(xs, sr=44100, hop=512, fmin=32.70, n_bins=168, bins_per_octave=24, n_taps=65536)
    e = _rel_err(out[SAMPLED].cpu().numpy(), ref)
    _say(f"  rel err {e:.3e}")
    assert e < TOL
    for lo, hi in ((0, 590), (590, 1770)):
        part = nb.nna_cqt(plan, x[lo:hi], out=_poisoned(hi - lo, 168, 345))
        assert torch.equal(part, out[lo:hi]), (lo, hi)


def test_cqt2010v2_config5_full_sampled(nb):
    import torch
    _say(f"cqt2010v2 on config 5's batch (1770 x 176400 @ 44100 Hz, 168 bins, 24 / octave), {len(SAMPLED)} sampled waveforms")
    x = _full_batch(5)
    plan = nb.nna_plan_cqt2010v2(sr=44100, hop=512, fmin=32.70, n_bins=168, bins_per_octave=24, device=0)
    ws = _poisoned_bytes(nb.nna_cqt2010v2_workspace(plan, 1770, 176400))
    out = nb.nna_cqt2010v2(plan, x, out=_poisoned(1770, 168, 345), workspace=ws)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all() and (out >= 0).all()
    xs = signals.batch(5, SAMPLED)
    ref = oracle.cqt2010v2(xs, sr=44100, hop=512, fmin=32.70, n_bins=168, bins_per_octave=24)
    got = out[SAMPLED].cpu().numpy()
    e = _rel_err(got, ref)
    for a in range(7):
        e = max(e, _rel_err(got[:, 168 - 24 * (a + 1):168 - 24 * a], ref[:, 168 - 24 * (a + 1):168 - 24 * a]))
    _say(f"  rel err {e:.3e}")
    assert e < TOL


def test_stft_f16_config4_full_sampled(nb, batch4):
    import torch
    _say(f"stft f16 config 4 (1770 x 176400 @ 44100 Hz), {len(SAMPLED)} sampled waveforms")
    plan = nb.nna_plan_stft_prec(sr=44100, n_fft=2048, hop=512, precision=nb.NNA_PREC_F16, device=0)
    out = nb.nna_stft(plan, batch4, out=_poisoned(1770, 1025, 345))
    torch.cuda.synchronize()
    assert torch.isfinite(out).all() and (out >= 0).all()
    xs = signals.batch(4, SAMPLED)
    ref = oracle.stft(xs, n_fft=2048, hop=512)
    e = _rel_err(out[SAMPLED].cpu().numpy(), ref)
    _say(f"  rel err {e:.3e}")
    assert e < TOL


# ---------------------------------------------------------------------------------------
# One waveform as long as the library accepts (sample indices just below 2^31): frames sampled at
# the start, across the signal and at the mirrored end, each against the oracle run on a slice.
# ---------------------------------------------------------------------------------------
def _check_long_signal(nb, plan, run, oracle_fn, K, hop, L, x):
    import torch
    T = 1 + L // hop
    bins = nb.nna_out_shape(plan, 1, L)[0]
    out = run(plan, x, out=_poisoned(1, bins, T))  # NaN wherever no workgroup writes
    torch.cuda.synchronize()
    assert out.shape[0] == 1 and out.shape[2] == T
    for lo in range(0, bins, 128):  # in slices: the comparison's temporaries stay small
        assert torch.isfinite(out[:, lo:lo + 128]).all()
    worst = 0.0
    span = 8 * K  # samples per slice, a multiple of hop
    # the first frames (left mirror), slices inside, the last frames (right mirror)
    head = x[0, :span].cpu().numpy()[None, :]
    ref = oracle_fn(head, True)[0]
    n = (span - K) // hop  # frames of the slice that do not reach past its right end
    worst = max(worst, np.abs(out[0, :, :n].cpu().numpy() - ref[:, :n]).max() / ref.max())
    for frac in (0.13, 0.5, 0.77, 0.999):
        t0 = int(frac * (T - 2 * span // hop))
        s0 = t0 * hop - K // 2  # frame t0 starts here in the un-padded signal
        sl = x[0, s0:s0 + span].cpu().numpy()[None, :]
        ref = oracle_fn(sl, False)[0]  # frame j of the slice = frame t0 + j
        got = out[0, :, t0:t0 + ref.shape[1]].cpu().numpy()
        worst = max(worst, np.abs(got - ref).max() / ref.max())
    s0 = (L - span) // hop * hop  # a slice that ends where the signal ends, starting on a frame boundary
    tail = x[0, s0:].cpu().numpy()[None, :]
    ref = oracle_fn(tail, True)[0]
    skip = (K // 2 + hop - 1) // hop  # its first frames see its own artificial left mirror
    got = out[0, :, s0 // hop + skip:].cpu().numpy()
    assert got.shape[1] == ref.shape[1] - skip
    worst = max(worst, np.abs(got - ref[:, skip:]).max() / ref.max())
    return worst


def test_stft_longest_accepted_waveform(nb):
    import torch
    n_fft, hop = 2048, 512
    L = ((1 << 31) - 1 - 4 * n_fft - 64) // 4 * 4  # the largest multiple of 4 the library takes
    _say(f"stft, one waveform of {L} samples")
    x = (torch.rand((1, L), device="cuda:0") - 0.5)
    plan = nb.nna_plan_stft(n_fft=n_fft, hop=hop, device=0)
    e = _check_long_signal(nb, plan, nb.nna_stft, lambda s, c: oracle.stft(s, n_fft=n_fft, hop=hop, center=c), n_fft, hop, L, x)
    _say(f"  rel err {e:.3e}")
    assert e < TOL
    # eight samples more are refused (nothing is launched, the pointers are not touched)
    assert nb.lib().nna_stft(plan.handle, x.data_ptr(), 1, L + 8, x.data_ptr(), None) == nb.NNA_ERR_SHAPE


def test_cqt_longest_accepted_waveform(nb):
    import torch
    sr, hop, fmin, n_bins, taps = 8000, 128, 220.0, 24, 1024
    L = ((1 << 31) - 1 - 4 * taps - 64) // 4 * 4
    _say(f"cqt, one waveform of {L} samples")
    x = (torch.rand((1, L), device="cuda:0") - 0.5)
    plan = nb.nna_plan_cqt(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, n_taps=taps, device=0)
    e = _check_long_signal(nb, plan, nb.nna_cqt,
                           lambda s, c: oracle.cqt(s, sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, n_taps=taps, center=c),
                           taps, hop, L, x)
    _say(f"  rel err {e:.3e}")
    assert e < TOL


# ---- the paper's own validation inputs (Sec. IV-B) ------------------------------------------------
def test_sweeps_impulses_and_a_chromatic_scale_through_every_layer(nb):
    # the paper compares its layers with a reference implementation on sine sweeps, an impulse tone and
    # a piano scale; here the same kinds of input go through every layer against the oracle, per signal
    _say("validation signals (linear sweep, log sweep, impulses, chromatic scale) through all layers")
    sr = 22050
    x = signals.validation_signals(L=22050, sr=sr)
    xd = _dev(x)
    cq = dict(sr=sr, hop=256, fmin=110.0, n_bins=72, bins_per_octave=12)
    layers = [
        ("stft", nb.nna_stft(nb.nna_plan_stft(sr=sr, n_fft=1024, hop=256, device=0), xd),
         oracle.stft(x, n_fft=1024, hop=256)),
        ("log-frequency stft", nb.nna_stft(nb.nna_plan_stft_scaled(sr=sr, n_fft=1024, hop=256, freq_scale=nb.NNA_FREQ_LOG,
                                                                   fmin=60.0, fmax=8000.0, freq_bins=256, device=0), xd),
         oracle.stft_scaled(x, sr=sr, n_fft=1024, hop=256, scale=oracle.FREQ_LOG, fmin=60.0, fmax=8000.0, freq_bins=256)),
        ("mel", nb.nna_mel(nb.nna_plan_mel(sr=sr, n_fft=1024, hop=256, n_mels=96, device=0), xd),
         oracle.mel(x, sr=sr, n_fft=1024, hop=256, n_mels=96)),
        ("cqt1992v2", nb.nna_cqt(nb.nna_plan_cqt(device=0, **cq), xd), oracle.cqt(x, **cq)),
        ("cqt2010v2", nb.nna_cqt2010v2(nb.nna_plan_cqt2010v2(device=0, **cq), xd), oracle.cqt2010v2(x, **cq)),
        ("cqt1992", nb.nna_cqt1992(nb.nna_plan_cqt1992(device=0, **cq), xd), oracle.cqt1992(x, **cq)),
        ("cqt2010", nb.nna_cqt2010(nb.nna_plan_cqt2010(device=0, **cq), xd), oracle.cqt2010(x, **cq)),
    ]
    for name, got, ref in layers:
        got = got.cpu().numpy().astype(np.float64)
        assert got.shape == ref.shape, name
        errs = [np.abs(got[b] - ref[b]).max() / np.abs(ref[b]).max() for b in range(ref.shape[0])]
        _say(f"  {name}: " + ", ".join(f"{e:.2e}" for e in errs))
        assert max(errs) < TOL, (name, errs)


# ---- Mel and its spectrogram from one launch --------------------------------------------------------
MEL_STFT_CASES = [
    # name, B, L, sr, n_fft, hop, n_mels, fmin, fmax, power
    ("power, 128 mels", 3, 20000, 22050, 2048, 512, 128, 0.0, 0.0, 2.0),
    ("magnitude, filters that stop below Nyquist (upper row tiles untouched by them)", 2, 9000, 22050, 1024, 256, 40, 100.0, 3000.0, 1.0),
    ("more than 128 mels: two passes", 2, 12000, 22050, 2048, 512, 200, 0.0, 0.0, 2.0),
    ("many short waveforms, ragged tiles", 37, 1500, 8000, 256, 64, 20, 0.0, 0.0, 2.0),
]


@pytest.mark.parametrize("case", MEL_STFT_CASES, ids=[c[0] for c in MEL_STFT_CASES])
def test_mel_with_stft_parity(nb, case):
    name, B, L, sr, n_fft, hop, n_mels, fmin, fmax, power = case
    _say(f"mel + spectrogram in one launch: {name}")
    x = signals.batch(2, B=B, L=L, sr=sr)
    plan = nb.nna_plan_mel(sr=sr, n_fft=n_fft, hop=hop, n_mels=n_mels, fmin=fmin, fmax=fmax, power=power, device=0)
    mel, spec = nb.nna_mel_with_stft(plan, _dev(x))
    ref_mel = oracle.mel(x, sr=sr, n_fft=n_fft, hop=hop, n_mels=n_mels, fmin=fmin, fmax=fmax, power=power)
    ref_spec = oracle.stft(x, n_fft=n_fft, hop=hop, fmt=oracle.POWER if power == 2.0 else oracle.MAGNITUDE)
    e_m, e_s = _rel_err(mel.cpu().numpy(), ref_mel), _rel_err(spec.cpu().numpy(), ref_spec)
    _say(f"  mel {e_m:.2e}, spectrogram {e_s:.2e}")
    assert e_m < TOL and e_s < TOL
    # the Mel output is the one nna_mel writes (to rounding: nna_mel may run the folded contraction)
    assert _rel_err(nb.nna_mel(plan, _dev(x)).cpu().numpy(), ref_mel) < TOL
    assert np.abs(mel.cpu().numpy() - nb.nna_mel(plan, _dev(x)).cpu().numpy()).max() < 2e-5 * ref_mel.max()
    with pytest.raises(nb.NnaError):
        nb.nna_mel_with_stft(nb.nna_plan_stft(n_fft=n_fft, hop=hop, device=0), _dev(x))
