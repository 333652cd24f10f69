"""Seeded random configurations of every transform against the oracle (GPU).

The hand-picked cases of the other files aim at known tile edges; these draw sizes the authors did
not think of: odd lengths, hops that divide nothing, batch sizes around the tile boundaries, every
window and output format.  Each draw is reproducible from its seed (printed before the launch).
Bar: 1e-3 of each waveform's output peak, as everywhere."""
import sys

import numpy as np
import pytest

import oracle

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


def _err(got, ref):
    got = got.cpu().numpy().astype(np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got))
    worst = 0.0
    for b in range(ref.shape[0]):
        peak = np.abs(ref[b]).max()
        worst = max(worst, np.abs(got[b] - ref[b]).max() / (peak if peak > 0 else 1.0))
    return worst


def _wave(rng, B, L):
    # a few sinusoids plus noise, amplitudes that differ from waveform to waveform
    t = np.arange(L)
    x = 0.1 * rng.standard_normal((B, L))
    for b in range(B):
        for _ in range(3):
            x[b] += rng.uniform(0.05, 0.5) * np.sin(2 * np.pi * rng.uniform(0.001, 0.45) * t + rng.uniform(0, 6.28))
    return x.astype(np.float32)


@pytest.mark.parametrize("seed", range(24))
def test_random_stft_and_mel(nb, seed):
    rng = np.random.default_rng([7, seed])
    n_fft = int(rng.choice([32, 64, 96, 100, 128, 200, 256, 384, 500, 512, 1000, 1024, 2048]))
    hop = int(rng.choice([d for d in (1, 3, 8, 16, 25, 32, 50, 64, 100, 128, 160, 256, 512) if d <= n_fft]))
    center = bool(rng.integers(0, 2))
    win = int(rng.integers(0, 4))
    fmt = int(rng.integers(0, 5))
    B = int(rng.choice([1, 2, 3, 5, 17, 33]))
    T_want = int(rng.choice([1, 2, 7, 31, 64, 129, 300]))
    L = (T_want - 1) * hop + int(rng.integers(0, hop)) + (n_fft // 2 + 1 if center else n_fft)
    L = min(L, 60000 // B * 4 + n_fft)
    _say(f"random stft seed={seed}: n_fft={n_fft} hop={hop} center={center} win={win} fmt={fmt} B={B} L={L}")
    x = _wave(rng, B, L)
    got = nb.nna_stft(nb.nna_plan_stft(n_fft=n_fft, hop=hop, win=win, center=center, fmt=fmt, device=0), _dev(x))
    if fmt <= 2:
        ref = oracle.stft(x, n_fft=n_fft, hop=hop, window=win, center=center, fmt=fmt)
    else:
        re, im = oracle.stft_complex(x, n_fft=n_fft, hop=hop, window=win, center=center)
        ref = oracle.interleave(re, im) if fmt == 3 else None
    if fmt == 2:    # log: compare where the power is well above the floor
        pw = oracle.stft(x, n_fft=n_fft, hop=hop, window=win, center=center, fmt=oracle.POWER)
        keep = pw > 1e-6 * pw.max()
        assert np.abs(got.cpu().numpy()[keep] - ref[keep]).max() < 1e-2
    elif fmt == 4:  # phase: compare where the magnitude is not tiny, modulo 2 pi
        mag = np.hypot(re, im)
        keep = mag > 1e-3 * mag.max()
        d = got.cpu().numpy().astype(np.float64) - np.arctan2(im, re)
        d = np.abs((d + np.pi) % (2 * np.pi) - np.pi)
        assert d[keep].max() < 1e-2
    else:
        assert _err(got, ref) < TOL
    # Mel on the same draw (needs at least a few bins per filter)
    if n_fft >= 128:
        n_mels = int(rng.choice([8, 20, 40, 64, 128, 150]))
        n_mels = min(n_mels, n_fft // 8)
        power = float(rng.choice([1.0, 2.0]))
        htk = bool(rng.integers(0, 2))
        sr = int(rng.choice([8000, 16000, 22050, 44100]))
        fmax = float(rng.choice([0.0, 0.4 * sr]))
        _say(f"  mel: sr={sr} n_mels={n_mels} power={power} htk={htk} fmax={fmax}")
        plan = nb.nna_plan_mel(sr=sr, n_fft=n_fft, hop=hop, win=win, center=center, n_mels=n_mels, fmax=fmax,
                               scale=nb.NNA_MEL_HTK if htk else nb.NNA_MEL_SLANEY, power=power, device=0)
        ref = oracle.mel(x, sr=sr, n_fft=n_fft, hop=hop, window=win, center=center, n_mels=n_mels, fmax=fmax,
                         scale=oracle.MEL_HTK if htk else oracle.MEL_SLANEY, power=power)
        assert _err(nb.nna_mel(plan, _dev(x)), ref) < TOL
        mel2, spec = nb.nna_mel_with_stft(plan, _dev(x))
        assert _err(mel2, ref) < TOL
        assert _err(spec, oracle.stft(x, n_fft=n_fft, hop=hop, window=win, center=center,
                                      fmt=oracle.POWER if power == 2.0 else oracle.MAGNITUDE)) < TOL


@pytest.mark.parametrize("seed", range(16))
def test_random_cqt_layers(nb, seed):
    rng = np.random.default_rng([11, seed])
    sr = int(rng.choice([8000, 16000, 22050]))
    bpo = int(rng.choice([6, 12, 19, 24]))
    n_oct = int(rng.integers(1, 5))
    n_bins = int(n_oct * bpo - rng.integers(0, bpo // 2))
    top = 0.45 * sr / 2.0 ** (1.0 / bpo)
    fmin = float(top / 2.0 ** ((n_bins - 1) / bpo) * rng.uniform(0.5, 1.0))
    hop = int(rng.choice([16, 32, 64, 128, 256]))           # multiples of 2^(octaves - 1)
    win = int(rng.integers(0, 4))
    B = int(rng.choice([1, 2, 5]))
    taps = oracle.cqt_default_taps(sr, fmin, bpo)
    L = taps // 2 + 1 + int(rng.integers(200, 4000))
    L = max(L, 600)
    cfg = dict(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo)
    _say(f"random cqt seed={seed}: {cfg} win={win} B={B} L={L} taps={taps}")
    x = _wave(rng, B, L)
    xd = _dev(x)
    assert _err(nb.nna_cqt(nb.nna_plan_cqt(win=win, device=0, **cfg), xd), oracle.cqt(x, window=win, **cfg)) < TOL
    assert _err(nb.nna_cqt1992(nb.nna_plan_cqt1992(win=win, device=0, **cfg), xd), oracle.cqt1992(x, window=win, **cfg)) < TOL
    # the documented length rule of the downsampling layers: every octave longer than its padding, all
    # but the lowest at least one frame of the filter stage (384 samples for the default 257 taps)
    n_oct = -(-n_bins // bpo)
    taps_top = oracle.cqt2010_default_taps(sr, fmin, n_bins, bpo)
    lens = [L]
    for _ in range(n_oct - 1):
        lens.append((lens[-1] + 1) // 2)
    fits = all(l > taps_top // 2 for l in lens) and all(l >= 384 for l in lens[:-1])
    if not fits:
        _say(f"  downsampling layers: octave lengths {lens} are refused")
        with pytest.raises(nb.NnaError) as e:
            nb.nna_cqt2010v2(nb.nna_plan_cqt2010v2(win=win, device=0, **cfg), xd)
        assert e.value.status == nb.NNA_ERR_SHAPE
    else:
        ref = oracle.cqt2010v2(x, window=win, **cfg)
        assert _err(nb.nna_cqt2010v2(nb.nna_plan_cqt2010v2(win=win, device=0, **cfg), xd), ref) < TOL
        assert _err(nb.nna_cqt2010(nb.nna_plan_cqt2010(win=win, device=0, **cfg), xd), oracle.cqt2010(x, window=win, **cfg)) < TOL


@pytest.mark.parametrize("seed", range(12))
def test_random_cqt_many_bins_per_octave(nb, seed):
    # the region where nna_cqt folds its kernels about their centres: many bins per octave, kernels of many hops,
    # windows that vanish at n = 0 (Hann, Blackman); every output format
    rng = np.random.default_rng([17, seed])
    sr = int(rng.choice([8000, 16000, 22050]))
    bpo = int(rng.choice([24, 30, 36, 48]))
    n_bins = int(rng.integers(bpo + bpo // 2, 3 * bpo))
    top = float(rng.uniform(0.25, 0.45)) * sr / 2.0 ** (1.0 / bpo)
    fmin = float(top / 2.0 ** ((n_bins - 1) / bpo))
    hop = int(rng.choice([16, 32, 64, 128]))
    win = int(rng.choice([0, 3]))
    center = bool(rng.integers(0, 2))
    fmt = int(rng.integers(0, 3))
    B = int(rng.choice([1, 3, 6]))
    taps = oracle.cqt_default_taps(sr, fmin, bpo)
    L = taps + int(rng.integers(1, 3000))
    cfg = dict(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo, center=center)
    plan = nb.nna_plan_cqt(win=win, fmt=fmt, device=0, **cfg)
    info = plan.info()
    folded = info["executed_flops_per_frame"] < info["algorithmic_flops_per_frame"]
    _say(f"random cqt, many bins per octave, seed={seed}: {cfg} win={win} fmt={fmt} B={B} L={L} taps={taps} folded={folded}")
    x = _wave(rng, B, L)
    xd = _dev(x)
    assert _err(nb.nna_cqt(plan, xd), oracle.cqt(x, window=win, fmt=fmt, **cfg)) < TOL
    re, im = oracle.cqt_complex(x, window=win, **cfg)
    got = nb.nna_cqt(nb.nna_plan_cqt(win=win, fmt=nb.NNA_OUT_COMPLEX, device=0, **cfg), xd)
    assert _err(got, oracle.interleave(re, im)) < TOL


@pytest.mark.parametrize("seed", range(10))
def test_random_backward(nb, seed):
    import torch
    rng = np.random.default_rng([13, seed])
    n_fft = int(rng.choice([64, 96, 128, 200, 256, 512]))
    hop = int(rng.choice([d for d in (8, 16, 25, 32, 64, 128) if d <= n_fft]))
    center = bool(rng.integers(0, 2))
    fmt = int(rng.integers(0, 5))
    B = int(rng.choice([1, 3, 9]))
    L = n_fft + int(rng.integers(1, 40)) * hop + int(rng.integers(0, hop))
    _say(f"random backward seed={seed}: n_fft={n_fft} hop={hop} center={center} fmt={fmt} B={B} L={L}")
    x = _wave(rng, B, L)
    plan = nb.nna_plan_trainable(nb.nna_plan_stft(n_fft=n_fft, hop=hop, center=center, fmt=fmt, device=0))
    W = nb.nna_plan_get_bank(plan).cpu().numpy()
    W = (W * (1.0 + 0.1 * rng.standard_normal(W.shape))).astype(np.float32)
    nb.nna_plan_set_bank(plan, _dev(W))
    W = nb.nna_plan_get_bank(plan).cpu().numpy()            # rows 1 and 2F-1 read back as zero
    out_shape = oracle.stft_bank(x, W, hop=hop, center=center, fmt=fmt).shape
    gout = rng.standard_normal(out_shape).astype(np.float32)
    ref_gw, ref_gx = oracle.stft_dft_bank_backward(x, W, gout, hop=hop, center=center, fmt=fmt)
    gw, gx = nb.nna_stft_backward(plan, _dev(x), _dev(gout))
    torch.cuda.synchronize()
    for got, ref, name in ((gw, ref_gw, "bank"), (gx, ref_gx, "waveform")):
        got = got.cpu().numpy().astype(np.float64)
        e = np.abs(got - ref).max() / np.abs(ref).max()
        assert e < (1e-2 if fmt in (2, 4) else TOL), (name, e)


@pytest.mark.parametrize("seed", range(12))
def test_random_cqt_and_mel_backward(nb, seed):
    import torch
    rng = np.random.default_rng([17, seed])
    # constant-Q layer with trainable kernels
    sr = int(rng.choice([8000, 16000]))
    bpo = int(rng.choice([6, 12, 17]))
    n_bins = int(rng.integers(3, 4 * bpo))
    top = 0.4 * sr
    fmin = float(top / 2.0 ** ((n_bins - 1) / bpo) * rng.uniform(0.6, 1.0))
    hop = int(rng.choice([4, 16, 25, 32, 64, 100, 128, 256]))
    center = bool(rng.integers(0, 2))
    fmt = int(rng.integers(0, 5))
    taps = oracle.cqt_default_taps(sr, fmin, bpo)
    if rng.integers(0, 2):
        Nk, _ = oracle.cqt_lengths(sr, fmin, n_bins, bpo)
        taps = int(Nk[0]) + int(Nk[0]) % 2 + 2 * int(rng.integers(0, 40))   # ragged, even, >= the longest kernel
    B = int(rng.choice([1, 2, 6]))
    L = (taps // 2 + 1 if center else taps) + int(rng.integers(0, 30)) * hop + int(rng.integers(0, hop))
    _say(f"random cqt backward seed={seed}: sr={sr} fmin={fmin:.1f} bins={n_bins} bpo={bpo} hop={hop} taps={taps} "
         f"center={center} fmt={fmt} B={B} L={L}")
    x = _wave(rng, B, L)
    plan = nb.nna_plan_trainable(nb.nna_plan_cqt(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo,
                                                 n_taps=taps, center=center, fmt=fmt, device=0))
    _, mask = oracle.cqt_bank(sr, fmin, n_bins, bpo, n_taps=taps)
    W = nb.nna_plan_get_bank(plan).cpu().numpy()
    W = np.where(mask, W * (1.0 + 0.1 * rng.standard_normal(W.shape)), 0).astype(np.float32)
    nb.nna_plan_set_bank(plan, _dev(W))
    gout = rng.standard_normal(oracle.stft_bank(x, W, hop=hop, center=center, fmt=fmt).shape).astype(np.float32)
    ref_gw, ref_gx = oracle.cqt_bank_backward(x, W, mask, gout, hop=hop, center=center, fmt=fmt)
    gw, gx = nb.nna_cqt_backward(plan, _dev(x), _dev(gout))
    torch.cuda.synchronize()
    tol = 1e-2 if fmt in (2, 4) else TOL   # log and phase divide by the power: ill-conditioned where it is small
    for got, ref, name in ((gw, ref_gw, "bank"), (gx, ref_gx, "waveform")):
        got = got.cpu().numpy().astype(np.float64)
        assert np.all(np.isfinite(got))
        e = np.abs(got - ref).max() / np.abs(ref).max()
        assert e < tol, (name, e)
    assert not gw.cpu().numpy()[~mask].any()

    # Mel layer with both stages trainable
    n_fft = int(rng.choice([128, 200, 256, 512]))
    hop = int(rng.choice([d for d in (16, 25, 32, 64, 128) if d <= n_fft]))
    n_mels = int(rng.choice([8, 20, 40]))
    n_mels = min(n_mels, n_fft // 8)
    power = float(rng.choice([1.0, 2.0]))
    L = n_fft + int(rng.integers(1, 30)) * hop + int(rng.integers(0, hop))
    _say(f"  mel backward: n_fft={n_fft} hop={hop} n_mels={n_mels} power={power} B={B} L={L}")
    x = _wave(rng, B, L)
    plan = nb.nna_plan_trainable(nb.nna_plan_mel(sr=sr, n_fft=n_fft, hop=hop, n_mels=n_mels, power=power, device=0))
    W = nb.nna_plan_get_bank(plan).cpu().numpy()
    Wm = nb.nna_plan_get_mel_weights(plan).cpu().numpy()
    Wm = (Wm + 0.05 * Wm.max() * rng.random(Wm.shape)).astype(np.float32)   # dense, no longer triangles
    nb.nna_plan_set_mel_weights(plan, _dev(Wm))
    gout = rng.standard_normal(oracle.mel_bank(x, W, Wm, hop=hop, power=power).shape).astype(np.float32)
    ref = oracle.mel_bank_backward(x, W, Wm, gout, hop=hop, power=power)
    ref[1][1] = 0.0
    ref[1][-1] = 0.0
    got = nb.nna_mel_backward(plan, _dev(x), _dev(gout))
    torch.cuda.synchronize()
    for g, r, name in zip(got, ref, ("filterbank", "bank", "waveform")):
        g = g.cpu().numpy().astype(np.float64)
        e = np.abs(g - r).max() / np.abs(r).max()
        assert np.all(np.isfinite(g)) and e < TOL, (name, e)


def _peak(got, ref):
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / np.abs(ref).max())


@pytest.mark.parametrize("seed", range(10))
def test_random_downsampling_and_spectral_backward(nb, seed):
    """Backward passes of the three other constant-Q layers (downsampling with time-domain kernels; frequency-domain
    kernels at one rate and downsampling) on configurations nobody hand-picked."""
    import torch
    rng = np.random.default_rng([19, seed])
    sr = int(rng.choice([8000, 16000, 22050]))
    bpo = int(rng.choice([4, 6, 12]))
    n_oct = int(rng.integers(1, 4))
    n_bins = int(n_oct * bpo - rng.integers(0, max(1, bpo // 2)))
    top = float(rng.uniform(0.06, 0.4)) * sr / 2.0 ** (1.0 / bpo)   # low tops: top-octave kernels of up to ~2,000 taps
    fmin = float(top / 2.0 ** ((n_bins - 1) / bpo) * rng.uniform(0.6, 1.0))
    hop = int(rng.choice([16, 32, 64, 128]))                 # multiples of 2^(octaves - 1)
    fir = int(rng.choice([31, 63, 127]))
    fmt = int(rng.choice([0, 1, 3]))                         # magnitude, power, complex (log / phase: ill-conditioned)
    B = int(rng.choice([1, 2, 5]))
    n_oct = -(-n_bins // bpo)
    taps_top = oracle.cqt2010_default_taps(sr, fmin, n_bins, bpo)
    frame = (fir + 126 + 127) // 128 * 128                   # the filter stage's frame (see nna_cqt2010v2)
    L = max(taps_top // 2 + 2, frame) * 2 ** (n_oct - 1) + int(rng.integers(100, 3000))
    _say(f"random downsampling / spectral backward seed={seed}: sr={sr} fmin={fmin:.1f} bins={n_bins}/{bpo} hop={hop} "
         f"fir={fir} fmt={fmt} B={B} L={L}")
    x = _wave(rng, B, L)
    kw = dict(hop=hop, n_bins=n_bins, bins_per_octave=bpo, fir_taps=fir, fmt=fmt)

    # time-domain kernels, downsampling
    plan = nb.nna_plan_trainable(nb.nna_plan_cqt2010v2(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo,
                                                       fir_taps=fir, fmt=fmt, device=0))
    _, mask = oracle.cqt2010v2_bank(sr, fmin, n_bins, bpo)
    W = nb.nna_plan_get_bank(plan).cpu().numpy()
    W = np.where(mask, W * (1.0 + 0.2 * rng.standard_normal(W.shape)), 0).astype(np.float32)
    nb.nna_plan_set_bank(plan, _dev(W))
    gout = rng.standard_normal(oracle.cqt2010v2_bank_forward(x, W, **kw).shape).astype(np.float32)
    ref_gw, ref_gx = oracle.cqt2010v2_bank_backward(x, W, mask, gout, **kw)
    gw, gx = nb.nna_cqt2010v2_backward(plan, _dev(x), _dev(gout))
    torch.cuda.synchronize()
    gw = gw.cpu().numpy()
    assert np.isfinite(gw).all() and not gw[~mask].any()
    assert _peak(gw, ref_gw) < TOL and _peak(gx.cpu().numpy(), ref_gx) < TOL

    # frequency-domain kernels, downsampling
    plan = nb.nna_plan_trainable(nb.nna_plan_cqt2010(sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bpo,
                                                     fir_taps=fir, fmt=fmt, device=0))
    Wd = nb.nna_plan_get_bank(plan).cpu().numpy()
    Y = nb.nna_plan_get_spectral_kernels(plan).cpu().numpy()
    dmask = oracle.dft_bank_parameter_mask(Wd.shape[1])
    Wd = np.where(dmask, Wd * (1.0 + 0.1 * rng.standard_normal(Wd.shape)), 0).astype(np.float32)
    Y = (Y * (1.0 + 0.2 * rng.standard_normal(Y.shape))).astype(np.float32)
    nb.nna_plan_set_bank(plan, _dev(Wd))
    nb.nna_plan_set_spectral_kernels(plan, _dev(Y))
    gout = rng.standard_normal(oracle.cqt2010_bank_forward(x, Wd, Y, **kw).shape).astype(np.float32)
    ref = oracle.cqt2010_bank_backward(x, Wd, Y, gout, **kw)
    got = nb.nna_cqt2010_backward(plan, _dev(x), _dev(gout))
    torch.cuda.synchronize()
    for g, r, name in zip(got, ref, ("spectral kernels", "bank", "waveform")):
        g = g.cpu().numpy()
        assert np.isfinite(g).all() and _peak(g, r) < TOL, (name, _peak(g, r))

    # frequency-domain kernels, one rate (its n_fft holds the longest kernel: keep that one short)
    bins1 = min(n_bins, 2 * bpo)
    fmin1 = float(top / 2.0 ** ((bins1 - 1) / bpo))
    hop1 = int(rng.choice([32, 64, 100, 128]))
    center = bool(rng.integers(0, 2))
    plan = nb.nna_plan_trainable(nb.nna_plan_cqt1992(sr=sr, hop=hop1, fmin=fmin1, n_bins=bins1, bins_per_octave=bpo,
                                                     center=center, fmt=fmt, device=0))
    Wd = nb.nna_plan_get_bank(plan).cpu().numpy()
    Y = nb.nna_plan_get_spectral_kernels(plan).cpu().numpy()
    n_fft = Wd.shape[1]
    dmask = oracle.dft_bank_parameter_mask(n_fft)
    Wd = np.where(dmask, Wd * (1.0 + 0.1 * rng.standard_normal(Wd.shape)), 0).astype(np.float32)
    Y = (Y * (1.0 + 0.2 * rng.standard_normal(Y.shape))).astype(np.float32)
    nb.nna_plan_set_bank(plan, _dev(Wd))
    nb.nna_plan_set_spectral_kernels(plan, _dev(Y))
    L1 = (n_fft // 2 + 1 if center else n_fft) + int(rng.integers(0, 20)) * hop1 + int(rng.integers(0, hop1))
    x1 = _wave(rng, B, L1)
    _say(f"  one rate: bins={bins1} fmin={fmin1:.1f} hop={hop1} n_fft={n_fft} center={center} L={L1}")
    gout = rng.standard_normal(oracle.cqt1992_bank_forward(x1, Wd, Y, hop=hop1, center=center, fmt=fmt).shape).astype(np.float32)
    ref = oracle.cqt1992_bank_backward(x1, Wd, Y, gout, hop=hop1, center=center, fmt=fmt)
    got = nb.nna_cqt1992_backward(plan, _dev(x1), _dev(gout))
    torch.cuda.synchronize()
    for g, r, name in zip(got, ref, ("spectral kernels", "bank", "waveform")):
        g = g.cpu().numpy()
        assert np.isfinite(g).all() and _peak(g, r) < TOL, (name, _peak(g, r))
