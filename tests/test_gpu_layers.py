"""The nn.Module layers (the paper's API names and defaults) on the GPU: forward against the oracle,
autograd through the trainable layers against the oracle's gradients, and a few optimiser steps."""
import sys

import numpy as np
import pytest

import oracle
from paper_1912_12055_amd import signals

pytestmark = pytest.mark.gpu
TOL = 1e-3


@pytest.fixture(scope="module")
def layers():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (there is no CPU fallback)")
    from paper_1912_12055_amd import layers as L
    return L


def _say(msg):
    print(f"[case] {msg}", file=sys.stderr, flush=True)


def _err(got, ref):
    got = got.detach().cpu().numpy().astype(np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    return np.abs(got - ref).max() / np.abs(ref).max()


def test_layers_with_the_papers_defaults_match_the_oracle(layers):
    import torch
    _say("layers: forward with default arguments")
    x = signals.batch(1, B=2, L=22050)
    xd = torch.from_numpy(x).cuda()
    assert _err(layers.STFT()(xd), oracle.stft(x)) < TOL
    assert _err(layers.STFT(freq_scale="log", freq_bins=200, fmin=50, fmax=6000)(xd),
                oracle.stft_scaled(x, scale=oracle.FREQ_LOG, fmin=50.0, fmax=6000.0, freq_bins=200)) < TOL
    assert _err(layers.MelSpectrogram()(xd), oracle.mel(x)) < TOL
    assert _err(layers.MelSpectrogram(htk=True, n_mels=40, fmax=8000.0, norm=None)(xd),
                oracle.mel(x, n_mels=40, fmax=8000.0, scale=oracle.MEL_HTK, norm_area=False)) < TOL
    assert _err(layers.CQT1992v2()(xd), oracle.cqt(x)) < TOL
    assert _err(layers.CQT2010v2()(xd), oracle.cqt2010v2(x)) < TOL
    assert _err(layers.CQT2010()(xd), oracle.cqt2010(x)) < TOL
    assert _err(layers.CQT1992(n_bins=36)(xd), oracle.cqt1992(x, fmin=220.0, n_bins=36)) < TOL
    re, im = oracle.cqt_complex(x)
    assert _err(layers.CQT1992v2(output_format="Complex")(xd), oracle.interleave(re, im)) < TOL
    assert layers.STFT()(xd[0]).shape == (1, 1025, 44)  # a single waveform
    mel, spec = layers.MelSpectrogram()(xd, return_spectrogram=True)
    assert _err(mel, oracle.mel(x)) < TOL and _err(spec, oracle.stft(x, fmt=oracle.POWER)) < TOL
    with pytest.raises(NotImplementedError):
        layers.CQT2010v2(trainable=True)
    with pytest.raises(ValueError):
        layers.STFT(pad_mode="constant")


def test_autograd_through_the_trainable_stft_layer(layers):
    import torch
    _say("layers: autograd through STFT(trainable=True)")
    x = signals.batch(1, B=3, L=6000)
    layer = layers.STFT(n_fft=256, hop_length=64, trainable=True)
    xd = torch.from_numpy(x).cuda().requires_grad_(True)
    out = layer(xd)
    gout = np.random.default_rng(1).standard_normal(tuple(out.shape)).astype(np.float32)
    (out * torch.from_numpy(gout).cuda()).sum().backward()
    W = layer.wsin_wcos.detach().cpu().numpy().astype(np.float64)
    ref_gw, ref_gx = oracle.stft_bank_backward(x, W, gout, hop=64)
    assert _err(layer.wsin_wcos.grad, ref_gw) < TOL and _err(xd.grad, ref_gx) < TOL


def test_optimiser_steps_tune_the_kernels_and_the_filterbank(layers):
    # Sec. IV-C in miniature: a small n_fft, kernels and filters tuned by gradient descent towards a target
    import torch
    _say("layers: optimiser steps on STFT kernels and Mel filters")
    torch.manual_seed(0)
    x = torch.from_numpy(signals.batch(1, B=8, L=4000)).cuda()
    stft = layers.STFT(n_fft=64, hop_length=16, trainable=True, output_format="Power")
    target = 0.25 * stft(x).detach()
    opt = torch.optim.Adam(stft.parameters(), lr=0.02)
    losses = []
    for _ in range(6):
        opt.zero_grad()
        loss = ((stft(x) - target) ** 2).mean()
        loss.backward()
        opt.step()
        losses.append(float(loss.detach()))
    _say(f"  stft loss {losses[0]:.4e} -> {losses[-1]:.4e}")
    assert losses[-1] < 0.8 * losses[0] and all(b < a for a, b in zip(losses, losses[1:]))
    # the forward uses the updated kernels: what the library holds is what the parameter holds
    from paper_1912_12055_amd import binding as nb
    stft(x)
    assert torch.equal(nb.nna_plan_get_bank(stft.plan)[2:-2], stft.wsin_wcos.detach()[2:-2])

    mel = layers.MelSpectrogram(sr=8000, n_fft=256, hop_length=64, n_mels=20, trainable_mel=True)
    assert mel.mel_basis.requires_grad and not mel.wsin_wcos.requires_grad
    target = 0.5 * mel(x).detach()
    opt = torch.optim.Adam([mel.mel_basis], lr=1e-4)
    losses = []
    for _ in range(6):
        opt.zero_grad()
        loss = ((mel(x) - target) ** 2).mean()
        loss.backward()
        opt.step()
        losses.append(float(loss.detach()))
    _say(f"  mel loss {losses[0]:.4e} -> {losses[-1]:.4e}")
    assert losses[-1] < 0.8 * losses[0] and mel.wsin_wcos.grad is None


def test_autograd_and_an_optimiser_on_the_trainable_cqt_layer(layers):
    import torch
    _say("layers: CQT1992v2(trainable=True)")
    cfg = dict(sr=8000, fmin=220.0, n_bins=30, bins_per_octave=12)
    layer = layers.CQT1992v2(hop_length=64, trainable=True, **cfg)
    x = signals.batch(3, B=3, L=5000, sr=8000)
    xd = torch.from_numpy(x).cuda().requires_grad_(True)
    out = layer(xd)
    gout = np.random.default_rng(2).standard_normal(tuple(out.shape)).astype(np.float32)
    (out * torch.from_numpy(gout).cuda()).sum().backward()
    W = layer.cqt_kernels.detach().cpu().numpy().astype(np.float64)
    _, mask = oracle.cqt_bank(**cfg)
    ref_gw, ref_gx = oracle.cqt_bank_backward(x, W, mask, gout, hop=64)
    assert _err(layer.cqt_kernels.grad, ref_gw) < TOL and _err(xd.grad, ref_gx) < TOL
    # a few optimiser steps towards a scaled copy of the initial transform; the zeros that centre the kernels stay zeros
    target = 0.5 * layer(xd.detach()).detach()
    opt = torch.optim.Adam(layer.parameters(), lr=1e-4)
    losses = []
    for _ in range(6):
        opt.zero_grad()
        loss = ((layer(xd.detach()) - target) ** 2).mean()
        loss.backward()
        opt.step()
        losses.append(float(loss.detach()))
    _say(f"  cqt loss {losses[0]:.4e} -> {losses[-1]:.4e}")
    assert losses[-1] < 0.8 * losses[0]
    layer(xd.detach())
    from paper_1912_12055_amd import binding as nb
    assert not nb.nna_plan_get_bank(layer.plan).cpu().numpy()[~mask].any()


def test_replaced_parameter_storage_reaches_the_library_and_frozen_layers_refuse_gradients(layers):
    import torch
    from paper_1912_12055_amd import binding as nb
    _say("layers: param.data swap, and a waveform that asks for a gradient from a layer without one")
    x = torch.from_numpy(signals.batch(1, B=2, L=3000)).cuda()
    stft = layers.STFT(n_fft=64, hop_length=16, trainable=True)
    before = stft(x).detach().clone()
    # swapping the storage leaves Tensor._version alone: the layer must still upload the new kernels
    stft.wsin_wcos.data = 0.5 * stft.wsin_wcos.data.clone()
    after = stft(x).detach()
    assert torch.allclose(after, 0.5 * before, rtol=1e-5, atol=1e-7)
    assert torch.equal(nb.nna_plan_get_bank(stft.plan)[2:-2], stft.wsin_wcos.detach()[2:-2])
    xg = x.clone().requires_grad_(True)
    for layer in (layers.STFT(n_fft=64, hop_length=16), layers.MelSpectrogram(sr=8000, n_fft=256, hop_length=64, n_mels=20),
                  layers.CQT1992v2(sr=8000, hop_length=64, fmin=220.0, n_bins=24),
                  layers.CQT2010v2(sr=8000, hop_length=64, fmin=220.0, n_bins=24)):
        with pytest.raises(RuntimeError):
            layer(xg)
        with torch.no_grad():
            layer(xg)
    with pytest.raises(ValueError):
        layers.CQT1992v2(sr=8000, fmin=220.0, fmax=2000.0)
