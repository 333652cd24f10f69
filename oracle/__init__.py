"""float64 CPU oracle for the spectrogram transforms of arXiv 1912.12055.

TEST INFRASTRUCTURE ONLY.  This package wraps ``nna_oracle.c`` (plain C, naive
loops, double precision) through ctypes.  Only ``tests/``, the smoke check and
the bench's ``cpu_baseline`` leg may import it; the GPU library never does and
shares no code with it.  Function names follow the C file; every array is
row-major with the frame axis fastest: ``[B, bins, T]``.

Two transforms are written here in numpy rather than in the C file, as compositions of its
pinned parts and numpy's FFT / matrix product: ``cqt1992`` (constant-Q transform with
frequency-domain kernels) and ``cqt2010`` (the same per octave of a recursive downsampling).
Parity status: ``cqt1992_spectral_kernels`` / ``cqt1992`` pinned (explicit O(N^2) sums on a tiny
case, numpy's FFT of frames cut independently, the exact dropped-half difference from the
time-domain CQT, tone magnitude A/2); ``cqt2010`` pinned (octave by octave against ``cqt1992`` on
SciPy-downsampled signals, its time-domain twin, tones A/2 in every octave); their complex and phase
outputs pinned (the kept-half sum as a complex number; rows of the complex format octave by octave);
``cqt2010v2_complex`` (the octave loop over the C file's ``cqt_complex`` and ``downsample2``) pinned
(modulus = the C routine's magnitude; a tone's closed-form phase in the lower octaves).

Also in numpy: the layers with their kernels as weights and the gradients through them (Sec. IV-C).
Parity status: ``stft_bank`` pinned (equals the windowed-DFT oracle for a bank written out from eq. (DFT2));
``stft_bank_backward`` pinned (central differences of that forward in float64, one-frame closed forms);
``mel_bank`` / ``mel_bank_backward`` pinned (the Mel oracle for the initial weights; central differences);
``cqt_bank`` pinned (``stft_bank`` with it equals the constant-Q oracle, real and imaginary parts; supports
equal the kernel lengths); ``cqt_bank_backward`` pinned (central differences inside the supports, exact
zeros outside); ``dft_bank_parameter_mask`` / ``stft_dft_bank_backward`` pinned (the masked rows are exactly
the rows of eq. (DFT2)'s bank, written out in the test, that are zero for every tap; the unmasked gradient
there is already zero for the magnitude-type outputs); ``downsample2_transpose`` pinned (adjoint identity
against the SciPy-pinned ``downsample2``, matrix rows on a tiny case); ``cqt2010v2_bank`` /
``cqt2010v2_bank_forward`` pinned (equal the downsampling-CQT oracle, all five output formats);
``cqt2010v2_bank_backward`` pinned (central differences of that forward for kernel taps of shared and
partial-octave rows and for waveform samples at the mirrored ends and inside); ``cqt1992_weights`` /
``cqt1992_bank_forward`` and ``cqt2010_weights`` / ``cqt2010_bank_forward`` pinned (equal the ``cqt1992`` /
``cqt2010`` oracles; the DFT bank equals eq. (DFT2) written out in the test); ``cqt1992_bank_backward`` /
``cqt2010_bank_backward`` pinned (central differences for spectral-kernel entries, DFT-bank taps and waveform
samples).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nna_oracle.c")
_LIB = os.path.join(_HERE, "libnna_oracle.so")

MAGNITUDE, POWER, LOG = 0, 1, 2
COMPLEX, PHASE = 3, 4  # the transform before the magnitude: (Re, Im) row pairs [B, 2 bins, T]; atan2(Im, Re)
WIN_HANN, WIN_RECT, WIN_HAMMING, WIN_BLACKMAN = 0, 1, 2, 3
MEL_SLANEY, MEL_HTK = 0, 1
FREQ_DFT, FREQ_LINEAR, FREQ_LOG = 0, 1, 2
LOG_FLOOR = 1e-10


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math: the summation order is the C file's)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None
_LL = ctypes.c_longlong
_D = ctypes.c_double
_I = ctypes.c_int
_PF = ctypes.POINTER(ctypes.c_float)
_PD = ctypes.POINTER(ctypes.c_double)
_PLL = ctypes.POINTER(ctypes.c_longlong)


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.orc_threads.restype = _I
        L.orc_reflect_index.restype = _LL
        L.orc_reflect_index.argtypes = [_LL, _LL]
        L.orc_num_frames.restype = _LL
        L.orc_num_frames.argtypes = [_LL, _LL, _LL, _I]
        L.orc_window.argtypes = [_I, _LL, _PD]
        L.orc_stft_complex.argtypes = [_PF, _LL, _LL, _I, _I, _I, _I, _PD, _PD]
        L.orc_stft.argtypes = [_PF, _LL, _LL, _I, _I, _I, _I, _I, _PD]
        L.orc_freq_sigma.restype = _D
        L.orc_freq_sigma.argtypes = [_I, _LL, _D, _D, _LL, _LL, _D]
        L.orc_stft_sigma_complex.argtypes = [_PF, _LL, _LL, _I, _I, _I, _I, _LL, _PD, _PD, _PD]
        L.orc_stft_scaled.argtypes = [_PF, _LL, _LL, _I, _I, _I, _I, _I, _I, _D, _D, _LL, _I, _PD]
        L.orc_hz_to_mel.restype = _D
        L.orc_hz_to_mel.argtypes = [_D, _I]
        L.orc_mel_to_hz.restype = _D
        L.orc_mel_to_hz.argtypes = [_D, _I]
        L.orc_mel_filterbank.argtypes = [_I, _I, _I, _D, _D, _I, _I, _PD, _PD]
        L.orc_mel.argtypes = [_PF, _LL, _LL, _I, _I, _I, _I, _I, _I, _D, _D, _I, _I, _D, _PD]
        L.orc_cqt_Q.restype = _D
        L.orc_cqt_Q.argtypes = [_I]
        L.orc_cqt_lengths.argtypes = [_I, _D, _I, _I, _PLL, _PD]
        L.orc_cqt_default_taps.restype = _LL
        L.orc_cqt_default_taps.argtypes = [_I, _D, _I]
        L.orc_cqt_kernels.argtypes = [_I, _D, _I, _I, _I, _LL, _PD, _PD]
        L.orc_cqt.argtypes = [_PF, _LL, _LL, _I, _I, _D, _I, _I, _I, _I, _LL, _I, _PD]
        L.orc_cqt_complex.argtypes = [_PF, _LL, _LL, _I, _I, _D, _I, _I, _I, _I, _LL, _PD, _PD]
        L.orc_lowpass_fir.argtypes = [_I, _D, _PD]
        L.orc_downsample2.argtypes = [_PD, _LL, _PD, _I, _PD]
        L.orc_cqt2010_default_taps.restype = _LL
        L.orc_cqt2010_default_taps.argtypes = [_I, _D, _I, _I]
        L.orc_cqt2010v2.argtypes = [_PF, _LL, _LL, _I, _I, _D, _I, _I, _I, _LL, _I, _I, _PD]
        _lib = L
    return _lib


class OracleError(ValueError):
    pass


def _check(rc, what):
    if rc != 0:
        raise OracleError(f"{what}: oracle returned {rc} ({'invalid argument' if rc == 1 else 'out of memory'})")


def _x(x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    if x.ndim == 1:
        x = x[None, :]
    if x.ndim != 2:
        raise OracleError("x must be [B, L]")
    return x


def _pf(a):
    return a.ctypes.data_as(_PF)


def _pd(a):
    return a.ctypes.data_as(_PD)


def threads() -> int:
    return int(lib().orc_threads())


def reflect_index(j: int, L: int) -> int:
    return int(lib().orc_reflect_index(j, L))


def num_frames(L: int, N: int, hop: int, center: bool = True) -> int:
    return int(lib().orc_num_frames(L, N, hop, int(center)))


def window(kind: int, N: int) -> np.ndarray:
    w = np.empty(N, dtype=np.float64)
    _check(lib().orc_window(kind, N, _pd(w)), "window")
    return w


_window_values = window  # (most functions below have an argument of that name)


def stft_complex(x, n_fft=2048, hop=512, window=WIN_HANN, center=True):
    x = _x(x)
    B, L = x.shape
    T = num_frames(L, n_fft, hop, center)
    if T < 1:
        raise OracleError("signal too short")
    re = np.empty((B, n_fft // 2 + 1, T), dtype=np.float64)
    im = np.empty_like(re)
    _check(lib().orc_stft_complex(_pf(x), B, L, n_fft, hop, window, int(center), _pd(re), _pd(im)), "stft_complex")
    return re, im


def stft(x, n_fft=2048, hop=512, window=WIN_HANN, center=True, fmt=MAGNITUDE):
    x = _x(x)
    B, L = x.shape
    T = num_frames(L, n_fft, hop, center)
    if T < 1:
        raise OracleError("signal too short")
    out = np.empty((B, n_fft // 2 + 1, T), dtype=np.float64)
    _check(lib().orc_stft(_pf(x), B, L, n_fft, hop, window, int(center), fmt, _pd(out)), "stft")
    return out


def freq_sigma(scale, k, fmin, fmax, freq_bins, n_fft, sr) -> float:
    return float(lib().orc_freq_sigma(scale, k, fmin, fmax, freq_bins, n_fft, float(sr)))


def stft_sigma_complex(x, sigma, n_fft=2048, hop=512, window=WIN_HANN, center=True):
    x = _x(x)
    B, L = x.shape
    sigma = np.ascontiguousarray(sigma, dtype=np.float64)
    T = num_frames(L, n_fft, hop, center)
    if T < 1:
        raise OracleError("signal too short")
    re = np.empty((B, sigma.size, T), dtype=np.float64)
    im = np.empty_like(re)
    _check(lib().orc_stft_sigma_complex(_pf(x), B, L, n_fft, hop, window, int(center), sigma.size, _pd(sigma),
                                        _pd(re), _pd(im)), "stft_sigma_complex")
    return re, im


def stft_scaled(x, sr=22050, n_fft=2048, hop=512, window=WIN_HANN, center=True, scale=FREQ_LINEAR, fmin=50.0,
                fmax=6000.0, freq_bins=0, fmt=MAGNITUDE):
    x = _x(x)
    B, L = x.shape
    if freq_bins <= 0:
        freq_bins = n_fft // 2 + 1
    T = num_frames(L, n_fft, hop, center)
    if T < 1:
        raise OracleError("signal too short")
    out = np.empty((B, freq_bins, T), dtype=np.float64)
    _check(lib().orc_stft_scaled(_pf(x), B, L, sr, n_fft, hop, window, int(center), scale, fmin, fmax, freq_bins,
                                 fmt, _pd(out)), "stft_scaled")
    return out


def hz_to_mel(f: float, scale=MEL_SLANEY) -> float:
    return float(lib().orc_hz_to_mel(f, scale))


def mel_to_hz(m: float, scale=MEL_SLANEY) -> float:
    return float(lib().orc_mel_to_hz(m, scale))


def mel_filterbank(sr, n_fft, n_mels, fmin=0.0, fmax=0.0, scale=MEL_SLANEY, norm_area=True):
    W = np.empty((n_mels, n_fft // 2 + 1), dtype=np.float64)
    edges = np.empty(n_mels + 2, dtype=np.float64)
    _check(lib().orc_mel_filterbank(sr, n_fft, n_mels, fmin, fmax, scale, int(norm_area), _pd(W), _pd(edges)),
           "mel_filterbank")
    return W, edges


def mel(x, sr=22050, n_fft=2048, hop=512, window=WIN_HANN, center=True, n_mels=128, fmin=0.0, fmax=0.0,
        scale=MEL_SLANEY, norm_area=True, power=2.0):
    x = _x(x)
    B, L = x.shape
    T = num_frames(L, n_fft, hop, center)
    if T < 1:
        raise OracleError("signal too short")
    out = np.empty((B, n_mels, T), dtype=np.float64)
    _check(lib().orc_mel(_pf(x), B, L, sr, n_fft, hop, window, int(center), n_mels, fmin, fmax, scale,
                         int(norm_area), float(power), _pd(out)), "mel")
    return out


def cqt_Q(bins_per_octave: int) -> float:
    return float(lib().orc_cqt_Q(bins_per_octave))


def cqt_lengths(sr, fmin, n_bins, bins_per_octave):
    Nk = np.empty(n_bins, dtype=np.int64)
    fk = np.empty(n_bins, dtype=np.float64)
    _check(lib().orc_cqt_lengths(sr, fmin, n_bins, bins_per_octave, Nk.ctypes.data_as(_PLL), _pd(fk)), "cqt_lengths")
    return Nk, fk


def cqt_default_taps(sr, fmin, bins_per_octave) -> int:
    return int(lib().orc_cqt_default_taps(sr, fmin, bins_per_octave))


def cqt_kernels(sr, fmin, n_bins, bins_per_octave, window=WIN_HANN, n_taps=0):
    if n_taps <= 0:
        n_taps = cqt_default_taps(sr, fmin, bins_per_octave)
    kre = np.empty((n_bins, n_taps), dtype=np.float64)
    kim = np.empty_like(kre)
    _check(lib().orc_cqt_kernels(sr, fmin, n_bins, bins_per_octave, window, n_taps, _pd(kre), _pd(kim)), "cqt_kernels")
    return kre, kim


def cqt(x, sr=22050, hop=512, fmin=32.70, n_bins=84, bins_per_octave=12, window=WIN_HANN, center=True,
        n_taps=0, fmt=MAGNITUDE):
    x = _x(x)
    B, L = x.shape
    if n_taps <= 0:
        n_taps = cqt_default_taps(sr, fmin, bins_per_octave)
    T = num_frames(L, n_taps, hop, center)
    if T < 1:
        raise OracleError("signal too short")
    out = np.empty((B, n_bins, T), dtype=np.float64)
    _check(lib().orc_cqt(_pf(x), B, L, sr, hop, fmin, n_bins, bins_per_octave, window, int(center), n_taps, fmt,
                         _pd(out)), "cqt")
    return out


def cqt_complex(x, sr=22050, hop=512, fmin=32.70, n_bins=84, bins_per_octave=12, window=WIN_HANN, center=True,
                n_taps=0):
    """(re, im) of the constant-Q transform, each [B, n_bins, T]."""
    x = _x(x)
    B, L = x.shape
    if n_taps <= 0:
        n_taps = cqt_default_taps(sr, fmin, bins_per_octave)
    T = num_frames(L, n_taps, hop, center)
    if T < 1:
        raise OracleError("signal too short")
    re = np.empty((B, n_bins, T), dtype=np.float64)
    im = np.empty_like(re)
    _check(lib().orc_cqt_complex(_pf(x), B, L, sr, hop, fmin, n_bins, bins_per_octave, window, int(center), n_taps,
                                 _pd(re), _pd(im)), "cqt_complex")
    return re, im


FIR_TAPS = 257


def lowpass_fir(n_taps=FIR_TAPS, cutoff=0.5) -> np.ndarray:
    h = np.empty(n_taps, dtype=np.float64)
    _check(lib().orc_lowpass_fir(n_taps, float(cutoff), _pd(h)), "lowpass_fir")
    return h


def downsample2(x, h) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    h = np.ascontiguousarray(h, dtype=np.float64)
    y = np.empty((x.size + 1) // 2, dtype=np.float64)
    _check(lib().orc_downsample2(_pd(x), x.size, _pd(h), h.size, _pd(y)), "downsample2")
    return y


def cqt2010_default_taps(sr, fmin, n_bins, bins_per_octave) -> int:
    return int(lib().orc_cqt2010_default_taps(sr, fmin, n_bins, bins_per_octave))


def cqt2010v2(x, sr=22050, hop=512, fmin=32.70, n_bins=84, bins_per_octave=12, window=WIN_HANN, n_taps=0,
              fir_taps=FIR_TAPS, fmt=MAGNITUDE):
    x = _x(x)
    B, L = x.shape
    if fmt in (COMPLEX, PHASE):
        re, im = cqt2010v2_complex(x, sr=sr, hop=hop, fmin=fmin, n_bins=n_bins, bins_per_octave=bins_per_octave,
                                   window=window, n_taps=n_taps, fir_taps=fir_taps)
        return apply_complex_format(re, im, fmt)
    out = np.empty((B, n_bins, 1 + L // hop), dtype=np.float64)
    _check(lib().orc_cqt2010v2(_pf(x), B, L, sr, hop, fmin, n_bins, bins_per_octave, window, n_taps, fir_taps, fmt,
                               _pd(out)), "cqt2010v2")
    return out


def cqt2010v2_complex(x, sr=22050, hop=512, fmin=32.70, n_bins=84, bins_per_octave=12, window=WIN_HANN, n_taps=0,
                      fir_taps=FIR_TAPS):
    """(re, im) of the downsampling CQT with time-domain kernels before the magnitude is taken (the
    ``output_format`` argument of the paper's CQT layers, Sec. III-C), each [B, n_bins, 1 + L // hop].
    Sec. III-C "Downsampling" in its own order, per waveform: octave a = 0 (top), 1, ... is the complex
    one-rate transform (``cqt_complex``: eqs. (Q), (N_k), (CQT)) of the waveform downsampled a times, with
    hop / 2^a and the kernels of the octave's bins at frequencies times 2^a -- the readings of
    ``orc_cqt2010v2``, whose magnitude this function's modulus must reproduce (pinned); then
    ``downsample2``.
    """
    x = _x(x)
    B, L = x.shape
    b = bins_per_octave
    n_oct = (n_bins + b - 1) // b
    if hop % (1 << (n_oct - 1)):
        raise OracleError("hop must be a multiple of 2^(octaves-1)")
    if n_taps <= 0:
        n_taps = cqt2010_default_taps(sr, fmin, n_bins, b)
    h = lowpass_fir(fir_taps, 0.5)
    T = 1 + L // hop
    re = np.empty((B, n_bins, T), dtype=np.float64)
    im = np.empty_like(re)
    for bi in range(B):
        xa = x[bi].astype(np.float64)
        for a in range(n_oct):
            hi = n_bins - a * b
            lo = max(hi - b, 0)
            # the C routines take float32 waveforms: the downsampled signal is rounded (6e-8 relative)
            r, i = cqt_complex(xa.astype(np.float32), sr=sr, hop=hop >> a, fmin=fmin * 2.0 ** (float(lo + a * b) / float(b)),
                               n_bins=hi - lo, bins_per_octave=b, window=window, center=True, n_taps=n_taps)
            re[bi, lo:hi, :] = r[0, :, :T]
            im[bi, lo:hi, :] = i[0, :, :T]
            if a + 1 < n_oct:
                xa = downsample2(xa, h)
    return re, im


def apply_complex_format(re, im, fmt):
    """The output formats of the paper's layers from the transform's real and imaginary parts:
    magnitude, power, log power, the interleaved (Re, Im) rows, or the phase atan2(Im, Re)."""
    if fmt == COMPLEX:
        return interleave(re, im)
    if fmt == PHASE:
        return np.arctan2(im, re)
    pw = re ** 2 + im ** 2
    if fmt == MAGNITUDE:
        return np.sqrt(pw)
    if fmt == POWER:
        return pw
    if fmt == LOG:
        return np.log(np.maximum(pw, LOG_FLOOR))
    raise OracleError("unknown output format")


def cqt1992_spectral_kernels(sr, fmin, n_bins, bins_per_octave, window=WIN_HANN, n_fft=0):
    """Frequency-domain constant-Q kernels Y[k_cq, k], k = 0..n_fft/2 (Sec. III-C, "CQT using neural
    networks", eq. (CQT1992), Fig. 4 right): each time-domain kernel of ``cqt_kernels`` (centred in
    n_fft taps) taken to the frequency domain by an FFT, of which the half k <= n_fft/2 is kept.

    Reading: eq. (Parseval) as printed has neither a conjugate nor an index reversal, which a product of
    two complex spectra needs.  The identity used is  sum_n a[n] kappa[n] = (1/N) sum_k A[k] conj(B[k])
    with B = DFT(conj(kappa)); kappa = w exp(-2 pi i Q n / N_k) / sum(w) is the kernel of eq. (CQT), so
    conj(kappa) has a positive frequency and B lives in the kept half.  Returned: Y = conj(B).
    """
    if n_fft <= 0:
        n_fft = cqt_default_taps(sr, fmin, bins_per_octave)
    kre, kim = cqt_kernels(sr, fmin, n_bins, bins_per_octave, window=window, n_taps=n_fft)
    B = np.fft.fft(kre - 1j * kim, axis=1)
    return np.conj(B[:, :n_fft // 2 + 1])


def cqt1992(x, sr=22050, hop=512, fmin=32.70, n_bins=84, bins_per_octave=12, window=WIN_HANN, center=True,
            n_fft=0, fmt=MAGNITUDE):
    """Constant-Q spectrogram with frequency-domain kernels (Sec. III-C, eq. (CQT1992), Fig. 5), in the
    paper's order: (1) the un-windowed STFT of the waveform with n_fft = the kernels' padded length
    (the CQT window lives in the kernels), bins 0..n_fft/2; (2) every time step multiplied with the
    spectral kernels, X_cq[k_cq, t] = (1/n_fft) sum_k X_t[k] Y[k_cq, k]; (3) element-wise magnitude.
    The sum runs over the kept half of the spectrum only, which makes this the approximation of the
    time-domain CQT that the paper says it is.  out: [B, n_bins, T].
    """
    x = _x(x)
    if n_fft <= 0:
        n_fft = cqt_default_taps(sr, fmin, bins_per_octave)
    Y = cqt1992_spectral_kernels(sr, fmin, n_bins, bins_per_octave, window=window, n_fft=n_fft)
    re, im = stft_complex(x, n_fft=n_fft, hop=hop, window=WIN_RECT, center=center)
    X = re + 1j * im                                    # [B, F, T]
    Xcq = np.einsum("qk,bkt->bqt", Y, X) / float(n_fft)  # [B, n_bins, T]
    return apply_complex_format(Xcq.real, Xcq.imag, fmt)


def cqt2010(x, sr=22050, hop=512, fmin=32.70, n_bins=84, bins_per_octave=12, window=WIN_HANN, n_fft=0,
            fir_taps=FIR_TAPS, fmt=MAGNITUDE):
    """Constant-Q spectrogram by recursive downsampling with frequency-domain kernels (Sec. III-C,
    "Constant-Q transform (2010 version)", Fig. CQT2010), in the paper's order.  For octave a = 0 (top),
    1, ...: the un-windowed STFT (n_fft = the padded length of the top octave's kernels, hop / 2^a) of
    the waveform downsampled a times is multiplied with the octave's spectral kernels exactly as in
    ``cqt1992``; then the waveform is low-pass filtered and every second sample kept (``downsample2``).
    Octaves, bins per octave, kernel lengths, filter, frame positions and the absence of any
    per-octave scaling are the readings of ``orc_cqt2010v2``; only the kernels' domain differs.
    out: [B, n_bins, 1 + L // hop], lowest frequency first.
    """
    x = _x(x)
    B, L = x.shape
    b = bins_per_octave
    n_oct = (n_bins + b - 1) // b
    if hop % (1 << (n_oct - 1)):
        raise OracleError("hop must be a multiple of 2^(octaves-1)")
    N = int(n_fft) if n_fft > 0 else cqt2010_default_taps(sr, fmin, n_bins, b)
    Q = cqt_Q(b)
    h = lowpass_fir(fir_taps, 0.5)
    T = 1 + L // hop
    F = N // 2 + 1
    n = np.arange(N)
    dft = np.exp(-2j * np.pi * np.outer(n, np.arange(F)) / N)  # eq. (DFT2), no window: [N, F]
    out = np.empty((B, n_bins, T), dtype=np.complex128)
    for bi in range(B):
        xa = x[bi].astype(np.float64)
        for a in range(n_oct):
            hi = n_bins - a * b
            lo = max(hi - b, 0)
            hop_a = hop >> a
            La = xa.size
            if La <= N // 2:
                raise OracleError("signal too short for this many octaves")
            # this octave's kernels (eq. (CQT) for the bins' frequencies times 2^a), centred in N taps
            kap = np.zeros((hi - lo, N), dtype=np.complex128)
            for k in range(lo, hi):
                f = fmin * 2.0 ** (float(k + a * b) / float(b))
                Nk = int(np.ceil(Q * float(sr) / f))
                if Nk > N:
                    raise OracleError("n_fft is shorter than the octave's longest kernel")
                m = np.arange(Nk)
                w = _window_values(window, Nk)
                s = (N - Nk) // 2
                kap[k - lo, s:s + Nk] = w / w.sum() * np.exp(-2j * np.pi * Q * m / Nk)
            Y = np.conj(np.fft.fft(np.conj(kap), axis=1))[:, :F]
            # frames of the mirrored waveform, frame t centred on sample t * hop_a
            idx = (np.arange(T)[:, None] * hop_a + n[None, :]) - N // 2
            idx = np.where(idx < 0, -idx, idx)
            idx = np.where(idx >= La, 2 * (La - 1) - idx, idx)
            X = xa[idx] @ dft                       # [T, F]
            Xcq = (X @ Y.T) / float(N)               # [T, bins of the octave]
            out[bi, lo:hi, :] = Xcq.T
            if a + 1 < n_oct:
                xa = downsample2(xa, h)
    return apply_complex_format(out.real, out.imag, fmt)


# ---------------------------------------------------------------------------------------
# Trainable Fourier kernels (Sec. IV-C, "Trainable Transformation Kernels"): the STFT layer with an
# arbitrary kernel bank, and the gradients of a scalar loss through it.
# ---------------------------------------------------------------------------------------
def _frame_index(L, K, hop, center):
    """[T, K] index of the stored sample behind tap n of frame t (mirror reflection when centred)."""
    T = num_frames(L, K, hop, center)
    if T < 1:
        raise OracleError("signal too short")
    pad = K // 2 if center else 0
    idx = np.arange(T)[:, None] * hop + np.arange(K)[None, :] - pad
    idx = np.where(idx < 0, -idx, idx)
    idx = np.where(idx >= L, 2 * (L - 1) - idx, idx)
    return idx


def interleave(re, im):
    """[B, 2 bins, T] with row 2k = re[:, k], row 2k+1 = im[:, k]: the layout of the complex output format."""
    out = np.empty((re.shape[0], 2 * re.shape[1], re.shape[2]), dtype=np.float64)
    out[:, 0::2] = re
    out[:, 1::2] = im
    return out


def stft_bank(x, W, hop=512, center=True, fmt=MAGNITUDE):
    """The STFT layer with a given kernel bank (Sec. III-A with the kernels as weights, Sec. IV-C):
    W[2F, K], row 2k = real-part kernel and row 2k+1 = imaginary-part kernel of bin k (window folded
    in, as eq. (DFT2) initialises them).  C[b, r, t] = sum_n W[r, n] xp_b[t hop + n] (the strided
    convolution of Sec. III-A with its kernel flip folded away), out[b, k, t] = the format applied to
    C[b, 2k, t]^2 + C[b, 2k+1, t]^2.  out: [B, F, T]."""
    x = _x(x).astype(np.float64)
    W = np.ascontiguousarray(W, dtype=np.float64)
    K = W.shape[1]
    idx = _frame_index(x.shape[1], K, hop, center)
    out = []
    for b in range(x.shape[0]):
        C = x[b][idx] @ W.T                      # [T, 2F]
        if fmt == COMPLEX:
            out.append(C.T)
        elif fmt == PHASE:
            out.append(np.arctan2(C[:, 1::2], C[:, 0::2]).T)
        else:
            out.append((C[:, 0::2] ** 2 + C[:, 1::2] ** 2).T)   # [F, T]
    pw = np.stack(out)
    if fmt in (COMPLEX, PHASE):
        return pw
    if fmt == MAGNITUDE:
        return np.sqrt(pw)
    if fmt == POWER:
        return pw
    if fmt == LOG:
        return np.log(np.maximum(pw, LOG_FLOOR))
    raise OracleError("unknown output format")


def stft_bank_backward(x, W, gout, hop=512, center=True, fmt=MAGNITUDE):
    """Gradients of a scalar loss through ``stft_bank`` by the chain rule, given gout = dLoss/dout
    [B, F, T]: returns (gW [2F, K], gx [B, L]).

    With P = Re^2 + Im^2:  magnitude: d out/d Re = Re / sqrt(P) (0 where P = 0);  power: 2 Re;
    log: 2 Re / P where P exceeds the floor, else 0 -- and likewise for Im;  complex (gout [B, 2F, T]):
    the output is C itself;  phase: d atan2(Im, Re) = (Re dIm - Im dRe) / P.  G[b, r, t] = dLoss/dC.
    gW[r, n] = sum_{b,t} G[b, r, t] xp_b[t hop + n];   gx_b[j] = sum over all (t, n) whose padded
    sample t hop + n mirrors onto j of sum_r W[r, n] G[b, r, t] (the transposed strided convolution,
    with the reflection padding folded back)."""
    return stft_bank_backward_f64(_x(x).astype(np.float64), W, gout, hop=hop, center=center, fmt=fmt)


def stft_bank_backward_f64(x, W, gout, hop=512, center=True, fmt=MAGNITUDE):
    """``stft_bank_backward`` on float64 waveforms as given (the layer functions round their input to
    float32, the precision the GPU path receives it in; the octaves of a downsampling CQT stay float64)."""
    x = np.atleast_2d(np.asarray(x, dtype=np.float64))
    W = np.ascontiguousarray(W, dtype=np.float64)
    gout = np.ascontiguousarray(gout, dtype=np.float64)
    B, L = x.shape
    K = W.shape[1]
    idx = _frame_index(L, K, hop, center)
    gW = np.zeros_like(W)
    gx = np.zeros_like(x)
    for b in range(B):
        X = x[b][idx]                            # [T, K]
        C = X @ W.T                              # [T, 2F]
        re, im = C[:, 0::2], C[:, 1::2]
        pw = re ** 2 + im ** 2
        g = gout[b].T                            # [T, F]  ([T, 2F] for the complex format)
        if fmt == COMPLEX:
            G = g
            gW += G.T @ X
            np.add.at(gx[b], idx, G @ W)
            continue
        if fmt == PHASE:
            s = np.where(pw > 0, g / np.where(pw > 0, pw, 1.0), 0.0)
            G = np.empty_like(C)
            G[:, 0::2] = -s * im
            G[:, 1::2] = s * re
            gW += G.T @ X
            np.add.at(gx[b], idx, G @ W)
            continue
        if fmt == MAGNITUDE:
            s = np.where(pw > 0, g / np.sqrt(np.where(pw > 0, pw, 1.0)), 0.0)
        elif fmt == POWER:
            s = 2.0 * g
        elif fmt == LOG:
            s = np.where(pw > LOG_FLOOR, 2.0 * g / np.where(pw > LOG_FLOOR, pw, 1.0), 0.0)
        else:
            raise OracleError("unknown output format")
        G = np.empty_like(C)
        G[:, 0::2] = s * re
        G[:, 1::2] = s * im
        gW += G.T @ X
        np.add.at(gx[b], idx, G @ W)
    return gW, gx


def dft_bank_parameter_mask(n_fft: int) -> np.ndarray:
    """Which entries of the STFT layer's weight W[2F, K] (F = n_fft/2 + 1, K = n_fft) are parameters
    when the layer is initialised from eq. (DFT2): everything except rows 1 and 2F-1, the sine kernels
    of bins 0 and n_fft/2.  Those two are sin(0 n) and sin(pi n), identically zero for integer n, so the
    layer has no kernel there to train (Sec. IV-C trains the kernels eq. (DFT2) gives it): they stay
    zero, and their gradient is reported as zero.  [2F, K] bool."""
    F = n_fft // 2 + 1
    mask = np.ones((2 * F, n_fft), dtype=bool)
    mask[1] = False
    mask[2 * F - 1] = False
    return mask


def stft_dft_bank_backward(x, W, gout, hop=512, center=True, fmt=MAGNITUDE):
    """``stft_bank_backward`` for a bank that started as eq. (DFT2)'s kernels: the gradient of the two
    structurally zero sine rows (``dft_bank_parameter_mask``) is dropped.  (gW, gx)."""
    gW, gx = stft_bank_backward(x, W, gout, hop=hop, center=center, fmt=fmt)
    return np.where(dft_bank_parameter_mask(np.asarray(W).shape[1]), gW, 0.0), gx


def mel_bank(x, W, Wmel, hop=512, center=True, power=2.0):
    """The Mel-spectrogram layer with given weights (Sec. III-B, Fig. 3, with both stages as weights,
    Sec. IV-C): the STFT layer of ``stft_bank`` with kernel bank W[2F, K], then the fully connected
    layer Wmel[n_mels, F] applied per time step to |X|^power (power 1 or 2).  out: [B, n_mels, T]."""
    fmt = POWER if power == 2.0 else MAGNITUDE
    P = stft_bank(x, W, hop=hop, center=center, fmt=fmt)           # [B, F, T]
    return np.einsum("mk,bkt->bmt", np.asarray(Wmel, dtype=np.float64), P)


def mel_bank_backward(x, W, Wmel, gout, hop=512, center=True, power=2.0, dft_rows=False):
    """Gradients of a scalar loss through ``mel_bank`` given gout = dLoss/dout [B, n_mels, T]:
    (gWmel [n_mels, F], gW [2F, K], gx [B, L]).  dft_rows: the bank started as eq. (DFT2)'s kernels, so
    the two structurally zero sine rows are not parameters (``dft_bank_parameter_mask``).  gWmel[m, k] = sum_{b,t} gout[b, m, t] P[b, k, t];
    the gradient reaching the STFT layer's output is gP[b, k, t] = sum_m Wmel[m, k] gout[b, m, t],
    which ``stft_bank_backward`` carries on to the kernel bank and the waveform."""
    fmt = POWER if power == 2.0 else MAGNITUDE
    Wmel = np.asarray(Wmel, dtype=np.float64)
    gout = np.asarray(gout, dtype=np.float64)
    P = stft_bank(x, W, hop=hop, center=center, fmt=fmt)
    gWmel = np.einsum("bmt,bkt->mk", gout, P)
    gP = np.einsum("mk,bmt->bkt", Wmel, gout)
    gW, gx = stft_bank_backward(x, W, gP, hop=hop, center=center, fmt=fmt)
    if dft_rows:
        gW = np.where(dft_bank_parameter_mask(np.asarray(W).shape[1]), gW, 0.0)
    return gWmel, gW, gx


def cqt_bank(sr=22050, fmin=32.70, n_bins=84, bins_per_octave=12, window=WIN_HANN, n_taps=0):
    """The constant-Q kernels of Sec. III-C ("CQT with time domain kernels") as the weight of a
    convolution layer (Sec. IV-C): W[2 n_bins, n_taps], row 2k / 2k+1 = real / imaginary part of the
    kernel w_k[n] exp(-2 pi i Q n / N_k) / sum(w_k) that eq. (CQT) multiplies the signal with, so that
    ``stft_bank(x, W)`` is eq. (CQT) for every frame; and the support mask
    [2 n_bins, n_taps] (True on taps s_k .. s_k + N_k - 1 of bin k's rows: the window's extent,
    whether or not the window value there is zero)."""
    kre, kim = cqt_kernels(sr, fmin, n_bins, bins_per_octave, window, n_taps)
    taps = kre.shape[1]
    Nk, _ = cqt_lengths(sr, fmin, n_bins, bins_per_octave)
    W = np.empty((2 * n_bins, taps), dtype=np.float64)
    W[0::2] = kre
    W[1::2] = kim
    mask = np.zeros(W.shape, dtype=bool)
    for k in range(n_bins):
        s = (taps - int(Nk[k])) // 2
        mask[2 * k:2 * k + 2, s:s + int(Nk[k])] = True
    return W, mask


def cqt_bank_backward(x, W, mask, gout, hop=512, center=True, fmt=MAGNITUDE):
    """Gradients through the constant-Q layer with kernel bank W (``stft_bank`` with W from
    ``cqt_bank``): the chain rule of ``stft_bank_backward``; the taps outside ``mask`` are the zeros
    that centre each kernel, not parameters, so their gradient is dropped.  (gW, gx)."""
    gW, gx = stft_bank_backward(x, W, gout, hop=hop, center=center, fmt=fmt)
    return np.where(mask, gW, 0.0), gx


# ---------------------------------------------------------------------------------------
# Trainable kernels of the downsampling CQT with time-domain kernels (the `trainable` argument of the
# paper's CQT2010v2 layer, Sec. III-C / IV-C): one kernel bank -- the top octave's -- is the weight every
# octave convolves its downsampled waveform with, so its gradient is the sum over the octaves and the
# waveform's gradient flows back up through the transposed decimation steps.
# ---------------------------------------------------------------------------------------
def cqt2010v2_bank(sr=22050, fmin=32.70, n_bins=84, bins_per_octave=12, window=WIN_HANN, n_taps=0):
    """The weight of the downsampling CQT layer: the top octave's kernels, W[2 n_top, n_taps] with
    n_top = min(bins_per_octave, n_bins) (``cqt_bank`` for the bins n_bins - n_top .. n_bins - 1), and
    their support mask.  Octave a uses rows of the same W (its bins sit one factor 2^a lower, its
    waveform is downsampled a times); a partial lowest octave uses the rows of the upper bins only."""
    b = bins_per_octave
    n_top = min(b, n_bins)
    if n_taps <= 0:
        n_taps = cqt2010_default_taps(sr, fmin, n_bins, b)
    return cqt_bank(sr, fmin * 2.0 ** (float(n_bins - n_top) / float(b)), n_top, b, window, n_taps)


def downsample2_transpose(g, h, L):
    """Transpose of ``downsample2`` as a linear map R^L -> R^ceil(L/2): y[m] = sum_i h[i] x~[2m + i - half]
    with x~ the mirror extension, so out[j] collects h[i] g[m] from every (m, i) whose sample
    2m + i - half mirrors onto j.  g: [ceil(L/2)] -> [L]."""
    g = np.ascontiguousarray(g, dtype=np.float64)
    h = np.ascontiguousarray(h, dtype=np.float64)
    half = h.size // 2
    if half > L - 1:
        raise OracleError("signal shorter than the filter's half length")
    idx = 2 * np.arange(g.size)[:, None] + np.arange(h.size)[None, :] - half
    idx = np.where(idx < 0, -idx, idx)
    idx = np.where(idx >= L, 2 * (L - 1) - idx, idx)
    out = np.zeros(L, dtype=np.float64)
    np.add.at(out, idx, g[:, None] * h[None, :])
    return out


def _cqt2010v2_octaves(n_bins, b):
    """[(a, lo, hi, first row of W)] for the octaves a = 0 (top), 1, ...: bins [lo, hi) of the output."""
    n_top = min(b, n_bins)
    out = []
    for a in range((n_bins + b - 1) // b):
        hi = n_bins - a * b
        lo = max(hi - b, 0)
        out.append((a, lo, hi, 2 * (n_top - (hi - lo))))
    return out


def cqt2010v2_bank_forward(x, W, hop=512, n_bins=84, bins_per_octave=12, fir_taps=FIR_TAPS, fmt=MAGNITUDE):
    """The downsampling CQT layer with the given weight W (from ``cqt2010v2_bank``): Sec. III-C
    "Downsampling" with ``stft_bank`` as each octave's convolution.  Float64 throughout.
    out: [B, n_bins, 1 + L // hop] ([B, 2 n_bins, T] for the complex format)."""
    x = np.atleast_2d(np.asarray(x, dtype=np.float64))
    W = np.asarray(W, dtype=np.float64)
    B, L = x.shape
    T = 1 + L // hop
    h = lowpass_fir(fir_taps, 0.5)
    rpb = 2 if fmt == COMPLEX else 1
    out = np.empty((B, rpb * n_bins, T), dtype=np.float64)
    for bi in range(B):
        xa = x[bi]
        for a, lo, hi, r0 in _cqt2010v2_octaves(n_bins, bins_per_octave):
            o = _stft_bank64(xa, W[r0:r0 + 2 * (hi - lo)], hop >> a, fmt)
            out[bi, rpb * lo:rpb * hi, :] = o[:, :T]
            if lo > 0:
                xa = downsample2(xa, h)
    return out


def _stft_bank64(xa, W, hop, fmt):
    """``stft_bank`` for one float64 waveform (that function rounds its input to float32 first)."""
    idx = _frame_index(xa.size, W.shape[1], hop, True)
    C = xa[idx] @ W.T
    if fmt == COMPLEX:
        return C.T
    if fmt == PHASE:
        return np.arctan2(C[:, 1::2], C[:, 0::2]).T
    pw = (C[:, 0::2] ** 2 + C[:, 1::2] ** 2).T
    if fmt == MAGNITUDE:
        return np.sqrt(pw)
    if fmt == POWER:
        return pw
    if fmt == LOG:
        return np.log(np.maximum(pw, LOG_FLOOR))
    raise OracleError("unknown output format")


def cqt2010v2_bank_backward(x, W, mask, gout, hop=512, n_bins=84, bins_per_octave=12, fir_taps=FIR_TAPS, fmt=MAGNITUDE):
    """Gradients of a scalar loss through ``cqt2010v2_bank_forward`` given gout = dLoss/dout: (gW, gx).
    Chain rule, octave by octave from the lowest up: octave a's convolution gives the gradient of its
    rows of W and of its waveform x_a (``stft_bank_backward``; frames past 1 + L // hop are not part of
    the output, their gradient is zero); x_a also feeds octave a + 1 through ``downsample2``, whose
    transpose carries that octave's waveform gradient back.  gW sums over the octaves and the batch;
    taps outside ``mask`` are structure, not parameters."""
    x = np.atleast_2d(np.asarray(x, dtype=np.float64))
    W = np.asarray(W, dtype=np.float64)
    gout = np.asarray(gout, dtype=np.float64)
    B, L = x.shape
    T = 1 + L // hop
    h = lowpass_fir(fir_taps, 0.5)
    rpb = 2 if fmt == COMPLEX else 1
    octs = _cqt2010v2_octaves(n_bins, bins_per_octave)
    gW = np.zeros_like(W)
    gx = np.zeros_like(x)
    for bi in range(B):
        xs = [x[bi]]
        for _ in octs[1:]:
            xs.append(downsample2(xs[-1], h))
        g_below = None  # gradient of x_{a+1}
        for a, lo, hi, r0 in reversed(octs):
            Wa = W[r0:r0 + 2 * (hi - lo)]
            Ta = num_frames(xs[a].size, W.shape[1], hop >> a, True)
            ga = np.zeros((1, rpb * (hi - lo), Ta), dtype=np.float64)
            ga[0, :, :T] = gout[bi, rpb * lo:rpb * hi, :]
            gWa, gxa = _stft_bank_backward64(xs[a], Wa, ga[0], hop >> a, fmt)
            gW[r0:r0 + 2 * (hi - lo)] += gWa
            if g_below is not None:
                gxa = gxa + downsample2_transpose(g_below, h, xs[a].size)
            g_below = gxa
        gx[bi] = g_below
    return np.where(mask, gW, 0.0), gx


def _stft_bank_backward64(xa, W, g, hop, fmt):
    """``stft_bank_backward`` for one float64 waveform: g [F, T] ([2F, T] complex) -> (gW, gx)."""
    gW, gx = stft_bank_backward_f64(xa[None], W, g[None], hop=hop, center=True, fmt=fmt)
    return gW, gx[0]


# ---------------------------------------------------------------------------------------
# Trainable kernels of the CQT layers with frequency-domain kernels (Sec. III-C "CQT using neural networks",
# eq. (CQT1992), Fig. 5, with both stages' kernels as weights, Sec. IV-C): the un-windowed STFT layer's bank W and
# the spectral kernels Y.
# ---------------------------------------------------------------------------------------
def cqt1992_weights(sr=22050, fmin=220.0, n_bins=84, bins_per_octave=12, window=WIN_HANN, n_fft=0):
    """(W, Ysk): W[2F, n_fft] = eq. (DFT2)'s kernels without a window (row 2k = cos, row 2k+1 = -sin of 2 pi k n /
    n_fft, F = n_fft/2 + 1), the weight of the layer's STFT stage; Ysk[2 n_bins, F] = the spectral kernels of
    ``cqt1992_spectral_kernels`` divided by n_fft, row 2q = real part, row 2q+1 = imaginary part -- the weight of
    its second stage, X_cq[q, t] = sum_k X_t[k] (Ysk[2q, k] + i Ysk[2q+1, k])."""
    if n_fft <= 0:
        n_fft = cqt_default_taps(sr, fmin, bins_per_octave)
    F = n_fft // 2 + 1
    n = np.arange(n_fft)
    W = np.empty((2 * F, n_fft), dtype=np.float64)
    for k in range(F):
        # (k n) mod n_fft keeps the argument small: the table is exact to the last bit or two for large n_fft
        ang = 2.0 * np.pi * ((k * n) % n_fft) / float(n_fft)
        W[2 * k] = np.cos(ang)
        W[2 * k + 1] = -np.sin(ang)
    W[1] = 0.0           # sin(0 n) and sin(pi n): identically zero
    W[2 * F - 1] = 0.0
    Y = cqt1992_spectral_kernels(sr, fmin, n_bins, bins_per_octave, window=window, n_fft=n_fft) / float(n_fft)
    Ysk = np.empty((2 * n_bins, F), dtype=np.float64)
    Ysk[0::2] = Y.real
    Ysk[1::2] = Y.imag
    return W, Ysk


def _cqt1992_bank_forward64(xa, W, Ysk, hop, center, fmt):
    """One float64 waveform through both stages: (output [rows, T], X [T, F] complex, V [T, n_bins] complex)."""
    idx = _frame_index(xa.size, W.shape[1], hop, center)
    C = xa[idx] @ W.T                                  # [T, 2F]
    X = C[:, 0::2] + 1j * C[:, 1::2]
    Y = Ysk[0::2] + 1j * Ysk[1::2]
    V = X @ Y.T                                        # [T, n_bins]
    out = apply_complex_format(V.real.T[None], V.imag.T[None], fmt)[0]
    return out, X, V


def cqt1992_bank_forward(x, W, Ysk, hop=512, center=True, fmt=MAGNITUDE):
    """The CQT layer with frequency-domain kernels for given weights: the STFT layer ``stft_bank`` (complex output)
    with bank W, then every time step multiplied with the spectral kernels, then the output format.
    out: [B, n_bins, T] ([B, 2 n_bins, T] complex)."""
    x = _x(x).astype(np.float64)
    return np.stack([_cqt1992_bank_forward64(xb, np.asarray(W, dtype=np.float64), np.asarray(Ysk, dtype=np.float64),
                                             hop, center, fmt)[0] for xb in x])


def _complex_format_gradient(V, g, fmt):
    """dLoss/dRe V, dLoss/dIm V (each [T, n_bins]) from g = dLoss/dout for one waveform ([n_bins, T], or [2 n_bins, T]
    for the complex format): the output formats' derivatives as in ``stft_bank_backward``."""
    re, im = V.real, V.imag
    pw = re ** 2 + im ** 2
    g = g.T
    if fmt == COMPLEX:
        return g[:, 0::2], g[:, 1::2]
    if fmt == PHASE:
        s = np.where(pw > 0, g / np.where(pw > 0, pw, 1.0), 0.0)
        return -s * im, s * re
    if fmt == MAGNITUDE:
        s = np.where(pw > 0, g / np.sqrt(np.where(pw > 0, pw, 1.0)), 0.0)
    elif fmt == POWER:
        s = 2.0 * g
    elif fmt == LOG:
        s = np.where(pw > LOG_FLOOR, 2.0 * g / np.where(pw > LOG_FLOOR, pw, 1.0), 0.0)
    else:
        raise OracleError("unknown output format")
    return s * re, s * im


def _cqt1992_bank_backward64(xa, W, Ysk, g, hop, center, fmt):
    """One float64 waveform: (gYsk, gW, gx) given g = dLoss/dout of that waveform."""
    _, X, V = _cqt1992_bank_forward64(xa, W, Ysk, hop, center, fmt)
    gVr, gVi = _complex_format_gradient(V, g, fmt)
    Yr, Yi = Ysk[0::2], Ysk[1::2]
    # V_re = sum_k (Yr X_re - Yi X_im),  V_im = sum_k (Yr X_im + Yi X_re)
    gYsk = np.empty_like(Ysk)
    gYsk[0::2] = gVr.T @ X.real + gVi.T @ X.imag
    gYsk[1::2] = -gVr.T @ X.imag + gVi.T @ X.real
    gXr = gVr @ Yr + gVi @ Yi                          # [T, F]
    gXi = -gVr @ Yi + gVi @ Yr
    gC = np.empty((2 * Yr.shape[1], gXr.shape[0]), dtype=np.float64)
    gC[0::2] = gXr.T
    gC[1::2] = gXi.T
    gW, gx = stft_bank_backward_f64(xa[None], W, gC[None], hop=hop, center=center, fmt=COMPLEX)
    return gYsk, gW, gx[0]


def cqt1992_bank_backward(x, W, Ysk, gout, hop=512, center=True, fmt=MAGNITUDE):
    """Gradients of a scalar loss through ``cqt1992_bank_forward`` given gout = dLoss/dout:
    (gYsk [2 n_bins, F], gW [2F, n_fft], gx [B, L]).  Chain rule through the output format, the complex product
    with the spectral kernels and the STFT layer (``stft_bank_backward``); the two identically zero sine rows of
    the DFT bank are not parameters (``dft_bank_parameter_mask``)."""
    x = _x(x).astype(np.float64)
    W = np.asarray(W, dtype=np.float64)
    Ysk = np.asarray(Ysk, dtype=np.float64)
    gout = np.asarray(gout, dtype=np.float64)
    gY, gW, gx = np.zeros_like(Ysk), np.zeros_like(W), np.zeros_like(x)
    for b in range(x.shape[0]):
        a, w, gx[b] = _cqt1992_bank_backward64(x[b], W, Ysk, gout[b], hop, center, fmt)
        gY += a
        gW += w
    return gY, np.where(dft_bank_parameter_mask(W.shape[1]), gW, 0.0), gx


def cqt2010_weights(sr=22050, fmin=32.70, n_bins=84, bins_per_octave=12, window=WIN_HANN, n_fft=0):
    """The weights of the downsampling CQT layer with frequency-domain kernels: ``cqt1992_weights`` for the top
    octave's bins, shared by every octave (a partial lowest octave uses the rows of the upper bins)."""
    b = bins_per_octave
    n_top = min(b, n_bins)
    if n_fft <= 0:
        n_fft = cqt2010_default_taps(sr, fmin, n_bins, b)
    return cqt1992_weights(sr, fmin * 2.0 ** (float(n_bins - n_top) / float(b)), n_top, b, window, n_fft)


def cqt2010_bank_forward(x, W, Ysk, hop=512, n_bins=84, bins_per_octave=12, fir_taps=FIR_TAPS, fmt=MAGNITUDE):
    """``cqt2010`` as a layer with the given weights: per octave ``cqt1992_bank_forward`` (hop / 2^a, always
    centred) on the waveform downsampled a times.  Float64 throughout."""
    x = np.atleast_2d(np.asarray(x, dtype=np.float64))
    W = np.asarray(W, dtype=np.float64)
    Ysk = np.asarray(Ysk, dtype=np.float64)
    B, L = x.shape
    T = 1 + L // hop
    h = lowpass_fir(fir_taps, 0.5)
    rpb = 2 if fmt == COMPLEX else 1
    out = np.empty((B, rpb * n_bins, T), dtype=np.float64)
    for bi in range(B):
        xa = x[bi]
        for a, lo, hi, r0 in _cqt2010v2_octaves(n_bins, bins_per_octave):
            o = _cqt1992_bank_forward64(xa, W, Ysk[r0:r0 + 2 * (hi - lo)], hop >> a, True, fmt)[0]
            out[bi, rpb * lo:rpb * hi, :] = o[:, :T]
            if lo > 0:
                xa = downsample2(xa, h)
    return out


def cqt2010_bank_backward(x, W, Ysk, gout, hop=512, n_bins=84, bins_per_octave=12, fir_taps=FIR_TAPS, fmt=MAGNITUDE):
    """(gYsk, gW, gx) through ``cqt2010_bank_forward``: per octave ``cqt1992_bank_backward``'s chain, summed over
    the octaves for the shared weights; the waveform gradient climbs through ``downsample2_transpose``."""
    x = np.atleast_2d(np.asarray(x, dtype=np.float64))
    W = np.asarray(W, dtype=np.float64)
    Ysk = np.asarray(Ysk, dtype=np.float64)
    gout = np.asarray(gout, dtype=np.float64)
    B, L = x.shape
    T = 1 + L // hop
    h = lowpass_fir(fir_taps, 0.5)
    rpb = 2 if fmt == COMPLEX else 1
    octs = _cqt2010v2_octaves(n_bins, bins_per_octave)
    gY, gW, gx = np.zeros_like(Ysk), np.zeros_like(W), np.zeros_like(x)
    for bi in range(B):
        xs = [x[bi]]
        for _ in octs[1:]:
            xs.append(downsample2(xs[-1], h))
        g_below = None
        for a, lo, hi, r0 in reversed(octs):
            Ta = num_frames(xs[a].size, W.shape[1], hop >> a, True)
            ga = np.zeros((rpb * (hi - lo), Ta), dtype=np.float64)
            ga[:, :T] = gout[bi, rpb * lo:rpb * hi, :]
            gYa, gWa, gxa = _cqt1992_bank_backward64(xs[a], W, Ysk[r0:r0 + 2 * (hi - lo)], ga, hop >> a, True, fmt)
            gY[r0:r0 + 2 * (hi - lo)] += gYa
            gW += gWa
            if g_below is not None:
                gxa = gxa + downsample2_transpose(g_below, h, xs[a].size)
            g_below = gxa
        gx[bi] = g_below
    return gY, np.where(dft_bank_parameter_mask(W.shape[1]), gW, 0.0), gx
