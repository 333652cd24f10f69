"""Thin ctypes binding of the C ABI in include/nna.h.

Argument marshalling only: every step of the transforms runs in the HIP library.
PyTorch supplies device memory and streams.  There is no fallback: if libnna.so is
missing the import of this module's functions raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnna.so")

NNA_OK = 0
NNA_ERR_INVALID_ARG, NNA_ERR_UNSUPPORTED, NNA_ERR_SHAPE, NNA_ERR_ALLOC, NNA_ERR_HIP = 1, 2, 3, 4, 5
NNA_OUT_MAGNITUDE, NNA_OUT_POWER, NNA_OUT_LOG, NNA_OUT_COMPLEX, NNA_OUT_PHASE = 0, 1, 2, 3, 4
NNA_WIN_HANN, NNA_WIN_RECT, NNA_WIN_HAMMING, NNA_WIN_BLACKMAN = 0, 1, 2, 3
NNA_MEL_SLANEY, NNA_MEL_HTK = 0, 1
NNA_FREQ_LINEAR, NNA_FREQ_LOG = 1, 2
NNA_PREC_F32, NNA_PREC_F16 = 0, 1
NNA_KIND_STFT, NNA_KIND_MEL, NNA_KIND_CQT, NNA_KIND_CQT2010V2, NNA_KIND_CQT1992, NNA_KIND_CQT2010 = 0, 1, 2, 3, 4, 5

# every symbol include/nna.h declares
EXPORTS = [
    "nna_plan_stft", "nna_plan_stft_prec", "nna_plan_stft_scaled", "nna_plan_mel", "nna_plan_cqt", "nna_plan_cqt2010v2", "nna_out_shape", "nna_stft", "nna_mel", "nna_cqt",
    "nna_plan_bank", "nna_plan_mel_weights", "nna_plan_info", "nna_plan_cqt_lengths", "nna_plan_sigma", "nna_cqt2010v2_workspace",
    "nna_cqt2010v2", "nna_plan_part", "nna_plan_cqt1992", "nna_cqt1992", "nna_plan_spectral_kernels",
    "nna_plan_cqt2010", "nna_cqt2010",
    "nna_plan_get_mel_weights", "nna_plan_set_mel_weights", "nna_mel_backward_workspace", "nna_mel_backward",
    "nna_plan_trainable", "nna_plan_get_bank", "nna_plan_set_bank", "nna_stft_backward_workspace", "nna_stft_backward",
    "nna_cqt_backward_workspace", "nna_cqt_backward", "nna_mel_with_stft", "nna_cqt2010v2_static",
    "nna_cqt2010v2_backward_workspace", "nna_cqt2010v2_backward",
    "nna_plan_get_spectral_kernels", "nna_plan_set_spectral_kernels", "nna_cqt1992_backward_workspace", "nna_cqt1992_backward",
    "nna_cqt2010_backward_workspace", "nna_cqt2010_backward",
    "nna_plan_destroy",
    "nna_status_str", "nna_last_error",
]

_c = ctypes
_LL = _c.c_longlong
_VP = _c.c_void_p
_lib = None


class NnaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"nna status {status}: {message}")
        self.status = status
        self.message = message


def lib():
    """Load libnna.so (built in-tree by build.py / __graft_entry__.build())."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_1912_12055_amd.build` "
                "(there is no CPU fallback)")
        # PyTorch ships a HIP runtime of its own.  Loading it first makes the library's dependency on
        # the runtime resolve to that copy, so the process holds one runtime; loaded the other way
        # round, the second copy finds no device.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = _c.CDLL(LIB_PATH)
        PP = _c.POINTER(_VP)
        L.nna_plan_stft.argtypes = [PP, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_int]
        L.nna_plan_stft_prec.argtypes = [PP, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_int,
                                         _c.c_int]
        L.nna_plan_stft_scaled.argtypes = [PP, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_int,
                                           _c.c_double, _c.c_double, _c.c_int, _c.c_int]
        L.nna_plan_mel.argtypes = [PP, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_double,
                                   _c.c_double, _c.c_int, _c.c_int, _c.c_double, _c.c_int]
        L.nna_plan_cqt.argtypes = [PP, _c.c_int, _c.c_int, _c.c_double, _c.c_int, _c.c_int, _c.c_int, _c.c_int,
                                   _c.c_int, _c.c_int, _c.c_int]
        L.nna_plan_cqt2010v2.argtypes = [PP, _c.c_int, _c.c_int, _c.c_double, _c.c_int, _c.c_int, _c.c_int, _c.c_int,
                                         _c.c_int, _c.c_int, _c.c_int]
        L.nna_plan_cqt1992.argtypes = [PP, _c.c_int, _c.c_int, _c.c_double, _c.c_int, _c.c_int, _c.c_int, _c.c_int,
                                       _c.c_int, _c.c_int, _c.c_int]
        L.nna_plan_spectral_kernels.argtypes = [_VP, _c.POINTER(_c.c_double), _c.c_size_t]
        L.nna_cqt2010v2_workspace.argtypes = [_VP, _LL, _LL, _c.POINTER(_c.c_size_t)]
        L.nna_cqt2010v2.argtypes = [_VP, _VP, _LL, _LL, _VP, _VP, _c.c_size_t, _VP]
        L.nna_cqt2010.argtypes = [_VP, _VP, _LL, _LL, _VP, _VP, _c.c_size_t, _VP]
        L.nna_plan_cqt2010.argtypes = [PP, _c.c_int, _c.c_int, _c.c_double, _c.c_int, _c.c_int, _c.c_int, _c.c_int,
                                       _c.c_int, _c.c_int, _c.c_int]
        L.nna_plan_part.argtypes = [_VP, _c.c_int, PP]
        L.nna_plan_get_mel_weights.argtypes = [_VP, _VP, _VP]
        L.nna_plan_set_mel_weights.argtypes = [_VP, _VP, _VP]
        L.nna_mel_backward_workspace.argtypes = [_VP, _LL, _LL, _c.POINTER(_c.c_size_t)]
        L.nna_mel_backward.argtypes = [_VP, _VP, _LL, _LL, _VP, _VP, _VP, _VP, _VP, _c.c_size_t, _VP]
        L.nna_plan_trainable.argtypes = [_VP]
        L.nna_plan_get_bank.argtypes = [_VP, _VP, _VP]
        L.nna_plan_set_bank.argtypes = [_VP, _VP, _VP]
        L.nna_stft_backward_workspace.argtypes = [_VP, _LL, _LL, _c.POINTER(_c.c_size_t)]
        L.nna_stft_backward.argtypes = [_VP, _VP, _LL, _LL, _VP, _VP, _VP, _VP, _c.c_size_t, _VP]
        L.nna_cqt_backward_workspace.argtypes = [_VP, _LL, _LL, _c.POINTER(_c.c_size_t)]
        L.nna_cqt_backward.argtypes = [_VP, _VP, _LL, _LL, _VP, _VP, _VP, _VP, _c.c_size_t, _VP]
        L.nna_cqt2010v2_backward_workspace.argtypes = [_VP, _LL, _LL, _c.POINTER(_c.c_size_t)]
        L.nna_cqt2010v2_backward.argtypes = [_VP, _VP, _LL, _LL, _VP, _VP, _VP, _VP, _c.c_size_t, _VP]
        L.nna_plan_get_spectral_kernels.argtypes = [_VP, _VP, _VP]
        L.nna_plan_set_spectral_kernels.argtypes = [_VP, _VP, _VP]
        for name in ("nna_cqt1992", "nna_cqt2010"):
            getattr(L, name + "_backward_workspace").argtypes = [_VP, _LL, _LL, _c.POINTER(_c.c_size_t)]
            getattr(L, name + "_backward").argtypes = [_VP, _VP, _LL, _LL, _VP, _VP, _VP, _VP, _VP, _c.c_size_t, _VP]
        L.nna_mel_with_stft.argtypes = [_VP, _VP, _LL, _LL, _VP, _VP, _VP]
        L.nna_out_shape.argtypes = [_VP, _LL, _LL, _c.POINTER(_LL), _c.POINTER(_LL)]
        for name in ("nna_stft", "nna_mel", "nna_cqt", "nna_cqt1992", "nna_cqt2010v2_static"):
            getattr(L, name).argtypes = [_VP, _VP, _LL, _LL, _VP, _VP]
        L.nna_plan_bank.argtypes = [_VP, _c.POINTER(_c.c_double), _c.c_size_t]
        L.nna_plan_mel_weights.argtypes = [_VP, _c.POINTER(_c.c_double), _c.c_size_t]
        L.nna_plan_info.argtypes = [_VP, _c.POINTER(_c.c_int), _c.POINTER(_LL), _c.POINTER(_LL), _c.POINTER(_LL),
                                    _c.POINTER(_c.c_double), _c.POINTER(_c.c_double)]
        L.nna_plan_cqt_lengths.argtypes = [_VP, _c.POINTER(_LL), _c.c_size_t]
        L.nna_plan_sigma.argtypes = [_VP, _c.POINTER(_c.c_double), _c.c_size_t]
        L.nna_plan_destroy.argtypes = [_VP]
        L.nna_plan_destroy.restype = None
        L.nna_status_str.argtypes = [_c.c_int]
        L.nna_status_str.restype = _c.c_char_p
        L.nna_last_error.restype = _c.c_char_p
        for name in EXPORTS:
            if name not in ("nna_plan_destroy", "nna_status_str", "nna_last_error"):
                getattr(L, name).restype = _c.c_int
        _lib = L
    return _lib


def nna_last_error() -> str:
    return lib().nna_last_error().decode()


def nna_status_str(status: int) -> str:
    return lib().nna_status_str(status).decode()


def _check(status: int):
    if status != NNA_OK:
        raise NnaError(status, nna_last_error() or nna_status_str(status))


class Plan:
    """Owns one nna_plan*; destroyed with the object."""

    def __init__(self, handle: int, device: int, owner=None):
        self.handle = handle
        self.device = device
        self.owner = owner  # a part of another plan: that plan owns the handle (and is kept alive here)

    def __del__(self):
        h, self.handle = getattr(self, "handle", None), None
        if h and _lib is not None and getattr(self, "owner", None) is None:
            _lib.nna_plan_destroy(h)

    def info(self) -> dict:
        kind = _c.c_int()
        rows, taps, bins = _LL(), _LL(), _LL()
        ex, alg = _c.c_double(), _c.c_double()
        _check(lib().nna_plan_info(self.handle, kind, rows, taps, bins, ex, alg))
        return dict(kind=kind.value, bank_rows=rows.value, taps=taps.value, out_bins=bins.value,
                    executed_flops_per_frame=ex.value, algorithmic_flops_per_frame=alg.value)


def _new_plan(fn, args, device):
    h = _VP()
    _check(fn(_c.byref(h), *args, device))
    return Plan(h.value, device)


def nna_plan_stft(sr=22050, n_fft=2048, hop=512, win=NNA_WIN_HANN, center=True, fmt=NNA_OUT_MAGNITUDE,
                  device=0) -> Plan:
    return _new_plan(lib().nna_plan_stft, (sr, n_fft, hop, win, int(center), fmt), device)


def nna_plan_stft_prec(sr=22050, n_fft=2048, hop=512, win=NNA_WIN_HANN, center=True, fmt=NNA_OUT_MAGNITUDE,
                       precision=NNA_PREC_F16, device=0) -> Plan:
    return _new_plan(lib().nna_plan_stft_prec, (sr, n_fft, hop, win, int(center), fmt, precision), device)


def nna_plan_stft_scaled(sr=22050, n_fft=2048, hop=512, win=NNA_WIN_HANN, center=True, fmt=NNA_OUT_MAGNITUDE,
                         freq_scale=NNA_FREQ_LINEAR, fmin=50.0, fmax=6000.0, freq_bins=0, device=0) -> Plan:
    return _new_plan(lib().nna_plan_stft_scaled,
                     (sr, n_fft, hop, win, int(center), fmt, freq_scale, float(fmin), float(fmax), freq_bins), device)


def nna_plan_mel(sr=22050, n_fft=2048, hop=512, win=NNA_WIN_HANN, center=True, n_mels=128, fmin=0.0, fmax=0.0,
                 scale=NNA_MEL_SLANEY, norm_area=True, power=2.0, device=0) -> Plan:
    return _new_plan(lib().nna_plan_mel,
                     (sr, n_fft, hop, win, int(center), n_mels, float(fmin), float(fmax), scale, int(norm_area),
                      float(power)), device)


def nna_plan_cqt(sr=22050, hop=512, fmin=32.70, n_bins=84, bins_per_octave=12, win=NNA_WIN_HANN, center=True,
                 n_taps=0, fmt=NNA_OUT_MAGNITUDE, device=0) -> Plan:
    return _new_plan(lib().nna_plan_cqt,
                     (sr, hop, float(fmin), n_bins, bins_per_octave, win, int(center), n_taps, fmt), device)


def nna_plan_cqt2010v2(sr=22050, hop=512, fmin=32.70, n_bins=84, bins_per_octave=12, win=NNA_WIN_HANN, n_taps=0,
                       fir_taps=0, fmt=NNA_OUT_MAGNITUDE, device=0) -> Plan:
    return _new_plan(lib().nna_plan_cqt2010v2,
                     (sr, hop, float(fmin), n_bins, bins_per_octave, win, n_taps, fir_taps, fmt), device)


def nna_plan_cqt1992(sr=22050, hop=512, fmin=32.70, n_bins=84, bins_per_octave=12, win=NNA_WIN_HANN, center=True,
                     n_fft=0, fmt=NNA_OUT_MAGNITUDE, device=0) -> Plan:
    plan = _new_plan(lib().nna_plan_cqt1992,
                     (sr, hop, float(fmin), n_bins, bins_per_octave, win, int(center), n_fft, fmt), device)
    plan.spectral_rows = 2 * n_bins  # rows of the spectral kernels as a tensor: (Re, Im) per constant-Q bin
    return plan


def nna_plan_spectral_kernels(plan: Plan) -> np.ndarray:
    """Complex [n_bins, n_fft/2+1]: the spectral kernels of a plan from nna_plan_cqt1992, divided by n_fft."""
    i = plan.info()
    # (a complex-format plan reports two output rows per bin; the constructor wrapper recorded the real count)
    out = np.empty((getattr(plan, "spectral_rows", 2 * i["out_bins"]), i["taps"] // 2 + 1), dtype=np.float64)
    _check(lib().nna_plan_spectral_kernels(plan.handle, out.ctypes.data_as(_c.POINTER(_c.c_double)), out.size))
    return out[0::2] + 1j * out[1::2]


def nna_plan_cqt2010(sr=22050, hop=512, fmin=32.70, n_bins=84, bins_per_octave=12, win=NNA_WIN_HANN, n_fft=0,
                     fir_taps=0, fmt=NNA_OUT_MAGNITUDE, device=0) -> Plan:
    plan = _new_plan(lib().nna_plan_cqt2010,
                     (sr, hop, float(fmin), n_bins, bins_per_octave, win, n_fft, fir_taps, fmt), device)
    plan.spectral_rows = 2 * min(n_bins, bins_per_octave)  # the top octave's kernels serve every octave
    return plan


def nna_plan_part(plan: Plan, index: int) -> Plan:
    """Octave `index` (0 = top) of a downsampling CQT plan, or its filter bank for index -1."""
    h = _VP()
    _check(lib().nna_plan_part(plan.handle, index, _c.byref(h)))
    return Plan(h.value, plan.device, owner=plan)


def nna_cqt2010v2_workspace(plan: Plan, B: int, L: int) -> int:
    n = _c.c_size_t()
    _check(lib().nna_cqt2010v2_workspace(plan.handle, B, L, _c.byref(n)))
    return n.value


def nna_out_shape(plan: Plan, B: int, L: int):
    nb, nf = _LL(), _LL()
    _check(lib().nna_out_shape(plan.handle, B, L, nb, nf))
    return nb.value, nf.value


def nna_plan_bank(plan: Plan) -> np.ndarray:
    i = plan.info()
    out = np.empty((i["bank_rows"], i["taps"]), dtype=np.float64)
    _check(lib().nna_plan_bank(plan.handle, out.ctypes.data_as(_c.POINTER(_c.c_double)), out.size))
    return out


def nna_plan_mel_weights(plan: Plan) -> np.ndarray:
    i = plan.info()
    out = np.empty((i["out_bins"], i["bank_rows"] // 2), dtype=np.float64)
    _check(lib().nna_plan_mel_weights(plan.handle, out.ctypes.data_as(_c.POINTER(_c.c_double)), out.size))
    return out


def nna_plan_cqt_lengths(plan: Plan) -> np.ndarray:
    i = plan.info()
    # (out_bins counts (Re, Im) row pairs twice for a complex-output CQT plan; the plan's bank has 2 rows per bin)
    out = np.empty(i["out_bins"] if i["kind"] == NNA_KIND_CQT1992 else i["bank_rows"] // 2, dtype=np.int64)
    _check(lib().nna_plan_cqt_lengths(plan.handle, out.ctypes.data_as(_c.POINTER(_LL)), out.size))
    return out


def nna_plan_sigma(plan: Plan) -> np.ndarray:
    i = plan.info()
    out = np.empty(i["bank_rows"] // 2, dtype=np.float64)
    _check(lib().nna_plan_sigma(plan.handle, out.ctypes.data_as(_c.POINTER(_c.c_double)), out.size))
    return out


def _run(fn, plan: Plan, x, out, stream):
    import torch

    if not (isinstance(x, torch.Tensor) and x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()):
        raise TypeError("x must be a contiguous float32 CUDA tensor [B, L]")
    if x.dim() != 2:
        raise TypeError("x must be [B, L]")
    if x.device.index != plan.device:
        raise ValueError("x lives on a different device than the plan")
    B, L = x.shape
    bins, frames = nna_out_shape(plan, B, L)
    if out is None:
        out = torch.empty((B, bins, frames), dtype=torch.float32, device=x.device)
    elif not (out.is_cuda and out.dtype == torch.float32 and out.is_contiguous()
              and tuple(out.shape) == (B, bins, frames) and out.device == x.device):
        raise TypeError(f"out must be a contiguous float32 CUDA tensor of shape {(B, bins, frames)}")
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    _check(fn(plan.handle, x.data_ptr(), B, L, out.data_ptr(), stream))
    return out


def _run_octaves(cfn, plan: Plan, x, out, workspace, stream):
    import torch

    if not (isinstance(x, torch.Tensor) and x.is_cuda and x.dim() == 2):
        raise TypeError("x must be a contiguous float32 CUDA tensor [B, L]")
    need = nna_cqt2010v2_workspace(plan, x.shape[0], x.shape[1])
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    elif not (workspace.is_cuda and workspace.is_contiguous() and workspace.device == x.device):
        raise TypeError("workspace must be a contiguous CUDA tensor on x's device")
    ws_bytes = workspace.numel() * workspace.element_size()

    def fn(handle, xp, B, L, op, st):
        return cfn(handle, xp, B, L, op, workspace.data_ptr(), ws_bytes, st)

    return _run(fn, plan, x, out, stream)


def nna_cqt2010v2(plan: Plan, x, out=None, workspace=None, stream=None):
    """out[B, n_bins, T] = constant-Q spectrogram of x[B, L] by recursive downsampling.  `workspace`: a CUDA
    tensor of at least nna_cqt2010v2_workspace(plan, B, L) bytes (one is made here if None)."""
    return _run_octaves(lib().nna_cqt2010v2, plan, x, out, workspace, stream)


NNA_STATIC_SCRATCH_BYTES = 64 << 20


def nna_cqt2010v2_static(plan: Plan, x, out=None, stream=None):
    """nna_cqt2010v2 with the library's own static workspace: the call allocates nothing (pass `out`)."""
    return _run(lib().nna_cqt2010v2_static, plan, x, out, stream)


def nna_cqt2010(plan: Plan, x, out=None, workspace=None, stream=None):
    """As nna_cqt2010v2, for a plan from nna_plan_cqt2010 (frequency-domain kernels per octave)."""
    return _run_octaves(lib().nna_cqt2010, plan, x, out, workspace, stream)


def nna_stft(plan: Plan, x, out=None, stream=None):
    """out[B, F, T] = STFT of x[B, L] (device tensors; asynchronous on `stream`); F = n_fft/2+1, or freq_bins
    for a plan from nna_plan_stft_scaled."""
    return _run(lib().nna_stft, plan, x, out, stream)


def nna_mel(plan: Plan, x, out=None, stream=None):
    """out[B, n_mels, T] = Mel spectrogram of x[B, L]."""
    return _run(lib().nna_mel, plan, x, out, stream)


def nna_mel_with_stft(plan: Plan, x, out=None, spec=None, stream=None):
    """(mel[B, n_mels, T], spec[B, n_fft/2+1, T]) from one contraction: the Mel spectrogram and the |X|^power
    spectrogram its filterbank is applied to."""
    import torch

    F = plan.info()["bank_rows"] // 2
    cfn = lib().nna_mel_with_stft
    holder = {}

    def fn(handle, xp, B, L, op, st):
        T = nna_out_shape(plan, B, L)[1]
        sp = spec
        if sp is None:
            sp = torch.empty((B, F, T), dtype=torch.float32, device=x.device)
        elif not (sp.is_cuda and sp.dtype == torch.float32 and sp.is_contiguous() and tuple(sp.shape) == (B, F, T)
                  and sp.device == x.device):
            raise TypeError(f"spec must be a contiguous float32 CUDA tensor of shape {(B, F, T)}")
        holder["spec"] = sp
        return cfn(handle, xp, B, L, op, sp.data_ptr(), st)

    mel = _run(fn, plan, x, out, stream)
    return mel, holder["spec"]


def nna_cqt1992(plan: Plan, x, out=None, stream=None):
    """out[B, n_bins, T] = constant-Q spectrogram of x[B, L] with frequency-domain kernels."""
    return _run(lib().nna_cqt1992, plan, x, out, stream)


def nna_cqt(plan: Plan, x, out=None, stream=None):
    """out[B, n_bins, T] = constant-Q spectrogram of x[B, L]."""
    return _run(lib().nna_cqt, plan, x, out, stream)


# ---- trainable Fourier kernels -------------------------------------------------------------------
def nna_plan_trainable(plan: Plan) -> Plan:
    _check(lib().nna_plan_trainable(plan.handle))
    return plan


def _bank_shape(plan: Plan):
    i = plan.info()
    return (i["bank_rows"], i["taps"])


def _stream_of(t, stream):
    import torch

    return torch.cuda.current_stream(t.device).cuda_stream if stream is None else stream


def nna_plan_get_bank(plan: Plan, out=None, stream=None):
    """W[2F, K]: the plan's kernel bank as a float32 CUDA tensor (logical layout)."""
    import torch

    shape = _bank_shape(plan)
    if out is None:
        out = torch.empty(shape, dtype=torch.float32, device=f"cuda:{plan.device}")
    elif not (out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and tuple(out.shape) == shape):
        raise TypeError(f"out must be a contiguous float32 CUDA tensor of shape {shape}")
    _check(lib().nna_plan_get_bank(plan.handle, out.data_ptr(), _stream_of(out, stream)))
    return out


def nna_plan_set_bank(plan: Plan, W, stream=None):
    shape = _bank_shape(plan)
    if not (W.is_cuda and W.dtype.is_floating_point and W.element_size() == 4 and W.is_contiguous()
            and tuple(W.shape) == shape and W.device.index == plan.device):
        raise TypeError(f"W must be a contiguous float32 CUDA tensor of shape {shape} on the plan's device")
    _check(lib().nna_plan_set_bank(plan.handle, W.data_ptr(), _stream_of(W, stream)))


def nna_stft_backward_workspace(plan: Plan, B: int, L: int) -> int:
    n = _c.c_size_t()
    _check(lib().nna_stft_backward_workspace(plan.handle, B, L, _c.byref(n)))
    return n.value


def nna_stft_backward(plan: Plan, x, gout, want_gw=True, want_gx=True, workspace=None, stream=None):
    """(gW[2F, K] or None, gx[B, L] or None) = gradients of a loss through nna_stft(plan, x), given
    gout[B, F, T] = dLoss/dout.  `workspace`: a CUDA tensor of nna_stft_backward_workspace bytes (made here if None)."""
    import torch

    if not (isinstance(x, torch.Tensor) and x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and x.dim() == 2):
        raise TypeError("x must be a contiguous float32 CUDA tensor [B, L]")
    B, L = x.shape
    bins, frames = nna_out_shape(plan, B, L)
    if not (gout.is_cuda and gout.dtype == torch.float32 and gout.is_contiguous()
            and tuple(gout.shape) == (B, bins, frames) and gout.device == x.device):
        raise TypeError(f"gout must be a contiguous float32 CUDA tensor of shape {(B, bins, frames)}")
    need = nna_stft_backward_workspace(plan, B, L)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    gw = torch.empty(_bank_shape(plan), dtype=torch.float32, device=x.device) if want_gw else None
    gx = torch.empty_like(x) if want_gx else None
    _check(lib().nna_stft_backward(plan.handle, x.data_ptr(), B, L, gout.data_ptr(),
                                   gw.data_ptr() if want_gw else None, gx.data_ptr() if want_gx else None,
                                   workspace.data_ptr(), ws_bytes, _stream_of(x, stream)))
    return gw, gx


def nna_cqt_backward_workspace(plan: Plan, B: int, L: int) -> int:
    n = _c.c_size_t()
    _check(lib().nna_cqt_backward_workspace(plan.handle, B, L, _c.byref(n)))
    return n.value


def nna_cqt_backward(plan: Plan, x, gout, want_gw=True, want_gx=True, workspace=None, stream=None):
    """(gW[2 n_bins, n_taps] or None, gx[B, L] or None) = gradients of a loss through nna_cqt(plan, x), given
    gout = dLoss/dout.  `workspace`: a CUDA tensor of nna_cqt_backward_workspace bytes (made here if None)."""
    import torch

    if not (isinstance(x, torch.Tensor) and x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and x.dim() == 2):
        raise TypeError("x must be a contiguous float32 CUDA tensor [B, L]")
    B, L = x.shape
    bins, frames = nna_out_shape(plan, B, L)
    if not (gout.is_cuda and gout.dtype == torch.float32 and gout.is_contiguous()
            and tuple(gout.shape) == (B, bins, frames) and gout.device == x.device):
        raise TypeError(f"gout must be a contiguous float32 CUDA tensor of shape {(B, bins, frames)}")
    need = nna_cqt_backward_workspace(plan, B, L)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    gw = torch.empty(_bank_shape(plan), dtype=torch.float32, device=x.device) if want_gw else None
    gx = torch.empty_like(x) if want_gx else None
    _check(lib().nna_cqt_backward(plan.handle, x.data_ptr(), B, L, gout.data_ptr(),
                                  gw.data_ptr() if want_gw else None, gx.data_ptr() if want_gx else None,
                                  workspace.data_ptr(), ws_bytes, _stream_of(x, stream)))
    return gw, gx


def nna_cqt2010v2_backward_workspace(plan: Plan, B: int, L: int) -> int:
    n = _c.c_size_t()
    _check(lib().nna_cqt2010v2_backward_workspace(plan.handle, B, L, _c.byref(n)))
    return n.value


def nna_cqt2010v2_backward(plan: Plan, x, gout, want_gw=True, want_gx=True, workspace=None, stream=None):
    """(gW[2 n_top, n_taps] or None, gx[B, L] or None) = gradients of a loss through nna_cqt2010v2(plan, x), given
    gout = dLoss/dout.  `workspace`: a CUDA tensor of nna_cqt2010v2_backward_workspace bytes (made here if None)."""
    import torch

    if not (isinstance(x, torch.Tensor) and x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and x.dim() == 2):
        raise TypeError("x must be a contiguous float32 CUDA tensor [B, L]")
    B, L = x.shape
    bins, frames = nna_out_shape(plan, B, L)
    if not (gout.is_cuda and gout.dtype == torch.float32 and gout.is_contiguous()
            and tuple(gout.shape) == (B, bins, frames) and gout.device == x.device):
        raise TypeError(f"gout must be a contiguous float32 CUDA tensor of shape {(B, bins, frames)}")
    need = nna_cqt2010v2_backward_workspace(plan, B, L)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    gw = torch.empty(_bank_shape(plan), dtype=torch.float32, device=x.device) if want_gw else None
    gx = torch.empty_like(x) if want_gx else None
    _check(lib().nna_cqt2010v2_backward(plan.handle, x.data_ptr(), B, L, gout.data_ptr(),
                                        gw.data_ptr() if want_gw else None, gx.data_ptr() if want_gx else None,
                                        workspace.data_ptr(), ws_bytes, _stream_of(x, stream)))
    return gw, gx


def _spectral_shapes(plan: Plan):
    """(shape of the spectral kernels Ysk, shape of the STFT stage's bank) of a plan with frequency-domain kernels"""
    i = (nna_plan_part(plan, 0) if plan.info()["kind"] == NNA_KIND_CQT2010 else plan).info()
    return (plan.spectral_rows, i["bank_rows"] // 2), (i["bank_rows"], i["taps"])


def nna_plan_get_spectral_kernels(plan: Plan, out=None, stream=None):
    """Ysk[2 n_bins, F]: the spectral kernels of a trainable plan from nna_plan_cqt1992 / nna_plan_cqt2010."""
    import torch

    shape = _spectral_shapes(plan)[0]
    if out is None:
        out = torch.empty(shape, dtype=torch.float32, device=f"cuda:{plan.device}")
    elif not (out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and tuple(out.shape) == shape):
        raise TypeError(f"out must be a contiguous float32 CUDA tensor of shape {shape}")
    _check(lib().nna_plan_get_spectral_kernels(plan.handle, out.data_ptr(), _stream_of(out, stream)))
    return out


def nna_plan_set_spectral_kernels(plan: Plan, Y, stream=None):
    shape = _spectral_shapes(plan)[0]
    if not (Y.is_cuda and Y.dtype.is_floating_point and Y.element_size() == 4 and Y.is_contiguous()
            and tuple(Y.shape) == shape and Y.device.index == plan.device):
        raise TypeError(f"Y must be a contiguous float32 CUDA tensor of shape {shape} on the plan's device")
    _check(lib().nna_plan_set_spectral_kernels(plan.handle, Y.data_ptr(), _stream_of(Y, stream)))


def _spectral_backward(name, plan, x, gout, want_gy, want_gw, want_gx, workspace, stream):
    import torch

    if not (isinstance(x, torch.Tensor) and x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and x.dim() == 2):
        raise TypeError("x must be a contiguous float32 CUDA tensor [B, L]")
    B, L = x.shape
    bins, frames = nna_out_shape(plan, B, L)
    if not (gout.is_cuda and gout.dtype == torch.float32 and gout.is_contiguous()
            and tuple(gout.shape) == (B, bins, frames) and gout.device == x.device):
        raise TypeError(f"gout must be a contiguous float32 CUDA tensor of shape {(B, bins, frames)}")
    n = _c.c_size_t()
    _check(getattr(lib(), name + "_backward_workspace")(plan.handle, B, L, _c.byref(n)))
    if workspace is None:
        workspace = torch.empty(n.value, dtype=torch.uint8, device=x.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    y_shape, w_shape = _spectral_shapes(plan)
    gy = torch.empty(y_shape, dtype=torch.float32, device=x.device) if want_gy else None
    gw = torch.empty(w_shape, dtype=torch.float32, device=x.device) if want_gw else None
    gx = torch.empty_like(x) if want_gx else None
    _check(getattr(lib(), name + "_backward")(plan.handle, x.data_ptr(), B, L, gout.data_ptr(),
                                              gy.data_ptr() if want_gy else None, gw.data_ptr() if want_gw else None,
                                              gx.data_ptr() if want_gx else None, workspace.data_ptr(), ws_bytes,
                                              _stream_of(x, stream)))
    return gy, gw, gx


def nna_cqt1992_backward_workspace(plan: Plan, B: int, L: int) -> int:
    n = _c.c_size_t()
    _check(lib().nna_cqt1992_backward_workspace(plan.handle, B, L, _c.byref(n)))
    return n.value


def nna_cqt2010_backward_workspace(plan: Plan, B: int, L: int) -> int:
    n = _c.c_size_t()
    _check(lib().nna_cqt2010_backward_workspace(plan.handle, B, L, _c.byref(n)))
    return n.value


def nna_cqt1992_backward(plan: Plan, x, gout, want_gy=True, want_gw=True, want_gx=True, workspace=None, stream=None):
    """(gYsk[2 n_bins, F], gW[2F, n_fft], gx[B, L]; None where not wanted) = gradients of a loss through
    nna_cqt1992(plan, x), given gout = dLoss/dout."""
    return _spectral_backward("nna_cqt1992", plan, x, gout, want_gy, want_gw, want_gx, workspace, stream)


def nna_cqt2010_backward(plan: Plan, x, gout, want_gy=True, want_gw=True, want_gx=True, workspace=None, stream=None):
    """As nna_cqt1992_backward, through nna_cqt2010(plan, x): the top octave's kernels are the weights of every octave."""
    return _spectral_backward("nna_cqt2010", plan, x, gout, want_gy, want_gw, want_gx, workspace, stream)


def _mel_shape(plan: Plan):
    i = plan.info()
    return (i["out_bins"], i["bank_rows"] // 2)


def nna_plan_get_mel_weights(plan: Plan, stream=None):
    """Wmel[n_mels, F]: the filterbank of a trainable Mel plan as a float32 CUDA tensor."""
    import torch

    out = torch.empty(_mel_shape(plan), dtype=torch.float32, device=f"cuda:{plan.device}")
    _check(lib().nna_plan_get_mel_weights(plan.handle, out.data_ptr(), _stream_of(out, stream)))
    return out


def nna_plan_set_mel_weights(plan: Plan, W, stream=None):
    shape = _mel_shape(plan)
    if not (W.is_cuda and W.element_size() == 4 and W.dtype.is_floating_point and W.is_contiguous()
            and tuple(W.shape) == shape and W.device.index == plan.device):
        raise TypeError(f"W must be a contiguous float32 CUDA tensor of shape {shape} on the plan's device")
    _check(lib().nna_plan_set_mel_weights(plan.handle, W.data_ptr(), _stream_of(W, stream)))


def nna_mel_backward_workspace(plan: Plan, B: int, L: int) -> int:
    n = _c.c_size_t()
    _check(lib().nna_mel_backward_workspace(plan.handle, B, L, _c.byref(n)))
    return n.value


def nna_mel_backward(plan: Plan, x, gout, want_gmelw=True, want_gw=True, want_gx=True, workspace=None, stream=None):
    """(gWmel[n_mels, F], gW[2F, K], gx[B, L]) (None where not wanted) = gradients of a loss through
    nna_mel(plan, x), given gout[B, n_mels, T] = dLoss/dout."""
    import torch

    if not (isinstance(x, torch.Tensor) and x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and x.dim() == 2):
        raise TypeError("x must be a contiguous float32 CUDA tensor [B, L]")
    B, L = x.shape
    bins, frames = nna_out_shape(plan, B, L)
    if not (gout.is_cuda and gout.dtype == torch.float32 and gout.is_contiguous()
            and tuple(gout.shape) == (B, bins, frames) and gout.device == x.device):
        raise TypeError(f"gout must be a contiguous float32 CUDA tensor of shape {(B, bins, frames)}")
    need = nna_mel_backward_workspace(plan, B, L)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    gm = torch.empty(_mel_shape(plan), dtype=torch.float32, device=x.device) if want_gmelw else None
    gw = torch.empty(_bank_shape(plan), dtype=torch.float32, device=x.device) if want_gw else None
    gx = torch.empty_like(x) if want_gx else None
    _check(lib().nna_mel_backward(plan.handle, x.data_ptr(), B, L, gout.data_ptr(),
                                  gm.data_ptr() if want_gmelw else None, gw.data_ptr() if want_gw else None,
                                  gx.data_ptr() if want_gx else None, workspace.data_ptr(), ws_bytes,
                                  _stream_of(x, stream)))
    return gm, gw, gx
