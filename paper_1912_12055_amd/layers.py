"""The paper's layers as ``torch.nn.Module`` wrappers over the C ABI binding.

Names, arguments and defaults follow the "nnAudio API" paragraphs of Sec. III (STFT, MelSpectrogram,
CQT1992, CQT2010, CQT1992v2, CQT2010v2).  Argument marshalling only: every transform -- and, for the
trainable layers of Sec. IV-C, every gradient -- is computed by the HIP library; PyTorch supplies the
tensors, the parameter objects and the autograd graph the calls are hooked into.

Input ``x``: float32 CUDA tensor ``[B, L]`` (or ``[L]``); output ``[B, bins, T]``.
"""
from __future__ import annotations

import torch

from . import binding as nb

_WINDOWS = {"hann": nb.NNA_WIN_HANN, "hamming": nb.NNA_WIN_HAMMING, "blackman": nb.NNA_WIN_BLACKMAN,
            "ones": nb.NNA_WIN_RECT, "rect": nb.NNA_WIN_RECT, "boxcar": nb.NNA_WIN_RECT}
_FORMATS = {"magnitude": nb.NNA_OUT_MAGNITUDE, "power": nb.NNA_OUT_POWER, "log": nb.NNA_OUT_LOG,
            "complex": nb.NNA_OUT_COMPLEX, "phase": nb.NNA_OUT_PHASE}


def _window(name):
    try:
        return _WINDOWS[str(name).lower()]
    except KeyError:
        raise ValueError(f"window {name!r}: one of {sorted(_WINDOWS)}") from None


def _format(name):
    try:
        return _FORMATS[str(name).lower()]
    except KeyError:
        raise ValueError(f"output_format {name!r}: one of {sorted(_FORMATS)}") from None


def _check_pad(center, pad_mode):
    if center and pad_mode != "reflect":
        raise ValueError("pad_mode: only 'reflect' is implemented")


def _device_index(device):
    d = torch.device(device)
    if d.type != "cuda":
        raise ValueError("the library runs on the GPU only: device must be a CUDA device")
    return 0 if d.index is None else d.index


def _as_batch(x):
    if x.dim() == 1:
        x = x[None, :]
    return x.contiguous().float()


def _no_grad_input(x):
    """Input of a layer whose call has no derivative: a waveform that asks for a gradient would silently get none."""
    if torch.is_grad_enabled() and x.requires_grad:
        raise RuntimeError("this layer is not differentiable with respect to its input: build it with "
                           "trainable=True (STFT, MelSpectrogram, CQT1992v2) or detach the waveform")
    return _as_batch(x)


class _StftFn(torch.autograd.Function):
    """nna_stft with nna_stft_backward as its derivative (kernels W and waveform x)."""

    @staticmethod
    def forward(ctx, x, W, layer):
        ctx.layer = layer
        ctx.save_for_backward(x)
        return nb.nna_stft(layer.plan, x)

    @staticmethod
    def backward(ctx, gout):
        (x,) = ctx.saved_tensors
        need_x, need_w = ctx.needs_input_grad[0], ctx.needs_input_grad[1]
        gw, gx = nb.nna_stft_backward(ctx.layer.plan, x, gout.contiguous(), want_gw=need_w, want_gx=need_x)
        return gx, gw, None


class _MelFn(torch.autograd.Function):
    """nna_mel with nna_mel_backward as its derivative (filterbank, kernels and waveform)."""

    @staticmethod
    def forward(ctx, x, W, Wmel, layer):
        ctx.layer = layer
        ctx.save_for_backward(x)
        return nb.nna_mel(layer.plan, x)

    @staticmethod
    def backward(ctx, gout):
        (x,) = ctx.saved_tensors
        need_x, need_w, need_m = ctx.needs_input_grad[:3]
        gm, gw, gx = nb.nna_mel_backward(ctx.layer.plan, x, gout.contiguous(), want_gmelw=need_m, want_gw=need_w,
                                         want_gx=need_x)
        return gx, gw, gm, None


class _Trainable(torch.nn.Module):
    """Keeps the library's copy of a parameter in step with the ``nn.Parameter`` an optimiser updates."""

    def _sync(self, param, setter, tag):
        # Tensor._version counts in-place updates (optimiser steps, load_state_dict, manual edits)
        # alone misses `param.data = ...` and a replaced Parameter object: the storage and the object count too
        key = (param._version, param.data_ptr(), id(param))
        if getattr(self, "_seen_" + tag, None) != key:
            setter(self.plan, param.detach())
            setattr(self, "_seen_" + tag, key)


class STFT(_Trainable):
    """Sec. III-A.  ``freq_scale`` 'no' (bins k sr / n_fft), 'linear' or 'log' (Sec. II-B, with fmin, fmax,
    freq_bins).  ``trainable=True`` makes the Fourier kernels ``self.wsin_wcos`` [2 F, n_fft] a parameter
    (rows 2k / 2k+1 = real / imaginary kernel of bin k)."""

    def __init__(self, n_fft=2048, freq_bins=None, hop_length=512, window="hann", freq_scale="no", center=True,
                 pad_mode="reflect", fmin=50, fmax=6000, sr=22050, trainable=False, output_format="Magnitude",
                 device="cuda:0"):
        super().__init__()
        _check_pad(center, pad_mode)
        dev = _device_index(device)
        fmt, win = _format(output_format), _window(window)
        if freq_scale == "no":
            if freq_bins not in (None, n_fft // 2 + 1):
                raise ValueError("freq_scale='no' has n_fft/2 + 1 bins; choose 'linear' or 'log' for another count")
            self.plan = nb.nna_plan_stft(sr=sr, n_fft=n_fft, hop=hop_length, win=win, center=center, fmt=fmt, device=dev)
        elif freq_scale in ("linear", "log"):
            scale = nb.NNA_FREQ_LINEAR if freq_scale == "linear" else nb.NNA_FREQ_LOG
            self.plan = nb.nna_plan_stft_scaled(sr=sr, n_fft=n_fft, hop=hop_length, win=win, center=center, fmt=fmt,
                                                freq_scale=scale, fmin=fmin, fmax=fmax, freq_bins=freq_bins or 0,
                                                device=dev)
        else:
            raise ValueError("freq_scale: 'no', 'linear' or 'log'")
        self.trainable = bool(trainable)
        if self.trainable:
            nb.nna_plan_trainable(self.plan)
            self.wsin_wcos = torch.nn.Parameter(nb.nna_plan_get_bank(self.plan))

    def forward(self, x):
        if not self.trainable:
            return nb.nna_stft(self.plan, _no_grad_input(x))
        x = _as_batch(x)
        self._sync(self.wsin_wcos, nb.nna_plan_set_bank, "bank")
        return _StftFn.apply(x, self.wsin_wcos, self)


class MelSpectrogram(_Trainable):
    """Sec. III-B.  ``norm=1`` is the area normalisation of the filters, ``htk`` picks the mel scale;
    ``trainable_mel`` / ``trainable_STFT`` make ``self.mel_basis`` [n_mels, F] / ``self.wsin_wcos`` [2 F, n_fft]
    parameters."""

    def __init__(self, sr=22050, n_fft=2048, n_mels=128, hop_length=512, window="hann", center=True,
                 pad_mode="reflect", htk=False, fmin=0.0, fmax=None, norm=1, trainable_mel=False, trainable_STFT=False,
                 power=2.0, device="cuda:0"):
        super().__init__()
        _check_pad(center, pad_mode)
        self.plan = nb.nna_plan_mel(sr=sr, n_fft=n_fft, hop=hop_length, win=_window(window), center=center,
                                    n_mels=n_mels, fmin=fmin, fmax=fmax or 0.0,
                                    scale=nb.NNA_MEL_HTK if htk else nb.NNA_MEL_SLANEY, norm_area=bool(norm),
                                    power=power, device=_device_index(device))
        self.trainable = bool(trainable_mel or trainable_STFT)
        if self.trainable:
            nb.nna_plan_trainable(self.plan)
            self.mel_basis = torch.nn.Parameter(nb.nna_plan_get_mel_weights(self.plan), requires_grad=bool(trainable_mel))
            self.wsin_wcos = torch.nn.Parameter(nb.nna_plan_get_bank(self.plan), requires_grad=bool(trainable_STFT))

    def forward(self, x, return_spectrogram=False):
        """``return_spectrogram=True`` returns (mel, |X|^power) from the one launch (not differentiable)."""
        x = _as_batch(x)
        if self.trainable:
            self._sync(self.wsin_wcos, nb.nna_plan_set_bank, "bank")
            self._sync(self.mel_basis, nb.nna_plan_set_mel_weights, "mel")
        if return_spectrogram:
            return nb.nna_mel_with_stft(self.plan, x.detach())
        if not self.trainable:
            return nb.nna_mel(self.plan, _no_grad_input(x))
        self._sync(self.wsin_wcos, nb.nna_plan_set_bank, "bank")
        self._sync(self.mel_basis, nb.nna_plan_set_mel_weights, "mel")
        return _MelFn.apply(x, self.wsin_wcos, self.mel_basis, self)


def _cqt_bins(sr, fmin, fmax, n_bins, bins_per_octave):
    # the library's plans take the number of bins; these wrappers do no arithmetic of the method
    if fmax is not None:
        raise ValueError("fmax: give n_bins instead (the top bin is fmin * 2^((n_bins - 1) / bins_per_octave))")
    return n_bins


class _CqtFn(torch.autograd.Function):
    """nna_cqt with nna_cqt_backward as its derivative (kernels W and waveform x)."""

    @staticmethod
    def forward(ctx, x, W, layer):
        ctx.layer = layer
        ctx.save_for_backward(x)
        return nb.nna_cqt(layer.plan, x)

    @staticmethod
    def backward(ctx, gout):
        (x,) = ctx.saved_tensors
        need_x, need_w = ctx.needs_input_grad[0], ctx.needs_input_grad[1]
        gw, gx = nb.nna_cqt_backward(ctx.layer.plan, x, gout.contiguous(), want_gw=need_w, want_gx=need_x)
        return gx, gw, None


class _Cqt(_Trainable):
    def __init__(self, trainable):
        super().__init__()
        if trainable:
            raise NotImplementedError("this wrapper hooks only CQT1992v2 into autograd; the other constant-Q layers train through "
                                      "binding.nna_cqt2010v2_backward / nna_cqt1992_backward / nna_cqt2010_backward")


class CQT1992v2(_Cqt):
    """Sec. III-C "CQT with time domain kernels": one rate, full-length kernels (the paper's default CQT).
    ``trainable=True`` makes the kernels ``self.cqt_kernels`` [2 n_bins, n_taps] a parameter (rows 2k / 2k+1 =
    real / imaginary part of bin k's kernel; the taps outside a kernel's own length stay zero)."""

    def __init__(self, sr=22050, hop_length=512, fmin=32.70, fmax=None, n_bins=84, bins_per_octave=12, norm=1,
                 window="hann", center=True, pad_mode="reflect", trainable=False, output_format="Magnitude",
                 device="cuda:0"):
        super().__init__(False)
        _check_pad(center, pad_mode)
        if norm != 1:
            raise ValueError("norm: only the L1 normalisation (1) is implemented")
        self.plan = nb.nna_plan_cqt(sr=sr, hop=hop_length, fmin=fmin, n_bins=_cqt_bins(sr, fmin, fmax, n_bins, bins_per_octave),
                                    bins_per_octave=bins_per_octave, win=_window(window), center=center,
                                    fmt=_format(output_format), device=_device_index(device))
        self.trainable = bool(trainable)
        if self.trainable:
            nb.nna_plan_trainable(self.plan)
            self.cqt_kernels = torch.nn.Parameter(nb.nna_plan_get_bank(self.plan))

    def forward(self, x):
        if not self.trainable:
            return nb.nna_cqt(self.plan, _no_grad_input(x))
        x = _as_batch(x)
        self._sync(self.cqt_kernels, nb.nna_plan_set_bank, "bank")
        return _CqtFn.apply(x, self.cqt_kernels, self)


class CQT1992(_Cqt):
    """Sec. III-C "CQT using neural networks": STFT times frequency-domain kernels."""

    def __init__(self, sr=22050, hop_length=512, fmin=220, fmax=None, n_bins=84, bins_per_octave=12, norm=1,
                 window="hann", center=True, pad_mode="reflect", trainable=False, output_format="Magnitude",
                 device="cuda:0"):
        super().__init__(trainable)
        _check_pad(center, pad_mode)
        self.plan = nb.nna_plan_cqt1992(sr=sr, hop=hop_length, fmin=fmin,
                                        n_bins=_cqt_bins(sr, fmin, fmax, n_bins, bins_per_octave),
                                        bins_per_octave=bins_per_octave, win=_window(window), center=center,
                                        fmt=_format(output_format), device=_device_index(device))

    def forward(self, x):
        return nb.nna_cqt1992(self.plan, _no_grad_input(x))


class _Cqt2010(_Cqt):
    _plan_fn = None
    _run_fn = None

    def __init__(self, sr=22050, hop_length=512, fmin=32.70, fmax=None, n_bins=84, bins_per_octave=12, norm=True,
                 basis_norm=1, window="hann", pad_mode="reflect", earlydownsample=False, trainable=False,
                 output_format="Magnitude", device="cuda:0"):
        super().__init__(trainable)
        _check_pad(True, pad_mode)
        if earlydownsample:
            raise NotImplementedError("early downsampling is not implemented")
        self.plan = type(self)._plan_fn(sr=sr, hop=hop_length, fmin=fmin,
                                        n_bins=_cqt_bins(sr, fmin, fmax, n_bins, bins_per_octave),
                                        bins_per_octave=bins_per_octave, win=_window(window),
                                        fmt=_format(output_format), device=_device_index(device))
        self._workspace = None

    def forward(self, x):
        x = _no_grad_input(x)
        need = nb.nna_cqt2010v2_workspace(self.plan, x.shape[0], x.shape[1])
        if self._workspace is None or self._workspace.numel() < need or self._workspace.device != x.device:
            self._workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
        return type(self)._run_fn(self.plan, x, workspace=self._workspace)


class CQT2010v2(_Cqt2010):
    """Sec. III-C: recursive downsampling with time-domain kernels."""
    _plan_fn = staticmethod(nb.nna_plan_cqt2010v2)
    _run_fn = staticmethod(nb.nna_cqt2010v2)


class CQT2010(_Cqt2010):
    """Sec. III-C "Constant-Q transform (2010 version)": recursive downsampling, frequency-domain kernels."""
    _plan_fn = staticmethod(nb.nna_plan_cqt2010)
    _run_fn = staticmethod(nb.nna_cqt2010)


# The constant-Q layer the paper recommends (fastest on a GPU, best output: Sec. IV-A, IV-B) under the plain name.
CQT = CQT1992v2
