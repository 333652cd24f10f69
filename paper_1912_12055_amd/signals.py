"""Seeded synthetic waveforms shared by the tests, the smoke check and the bench.

This module holds input generation only -- none of the transforms' arithmetic --
so that the CPU oracle and the GPU library can be fed identical float32 arrays
without sharing any code of their own.

Every waveform ``b`` of workload ``cfg_id`` is drawn from its own generator
``numpy.random.default_rng([1912, cfg_id, b])``: any subset of a batch can be
regenerated without the rest.  The two content recipes stand in for the audio
clips the paper times its transforms on (Sec. IV-A: 1,770 mono clips at
44.1 kHz); only their shape is taken from there, the content is synthetic.

  sinusoid mix  3 sinusoids, frequency U(50, 5000) Hz, amplitude U(0.1, 0.3),
                phase U(0, 2 pi), plus Gaussian noise of variance 0.01
  tone mix      3 tones at semitone pitches p ~ randint(0, 84) above 32.70 Hz
                (f = 32.70 * 2^(p/12)), same amplitudes, phases and noise
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import numpy as np

SEED = 1912
NOISE_SIGMA = 0.1  # "N(0, 0.01)" read as variance 0.01

# The five workloads: name, transform, batch, length, sample rate, content recipe.
WORKLOADS = {
    1: dict(name="stft_4x1s_22k", transform="stft", B=4, L=22050, sr=22050, kind="sinusoid"),
    2: dict(name="mel_64x5s_22k", transform="mel", B=64, L=110250, sr=22050, kind="sinusoid"),
    3: dict(name="cqt_16x10s_22k", transform="cqt", B=16, L=220500, sr=22050, kind="tone"),
    4: dict(name="stftmel_1770x4s_44k", transform="mel", B=1770, L=176400, sr=44100, kind="sinusoid"),
    5: dict(name="cqt_1770x4s_44k", transform="cqt", B=1770, L=176400, sr=44100, kind="tone"),
}


def waveform(cfg_id: int, b: int, L: int, sr: int, kind: str) -> np.ndarray:
    """One float32 waveform of length L (see module docstring for the recipes)."""
    rng = np.random.default_rng([SEED, cfg_id, b])
    t = np.arange(L, dtype=np.float64) / float(sr)
    x = np.zeros(L, dtype=np.float64)
    for _ in range(3):
        if kind == "sinusoid":
            f = rng.uniform(50.0, 5000.0)
        elif kind == "tone":
            f = 32.70 * 2.0 ** (int(rng.integers(0, 84)) / 12.0)
        else:
            raise ValueError(f"unknown content kind {kind!r}")
        a = rng.uniform(0.1, 0.3)
        ph = rng.uniform(0.0, 2.0 * np.pi)
        x += a * np.sin(2.0 * np.pi * f * t + ph)
    x += rng.normal(0.0, NOISE_SIGMA, size=L)
    return x.astype(np.float32)


def batch(cfg_id: int, indices=None, B=None, L=None, sr=None, kind=None, workers: int = 8) -> np.ndarray:
    """float32 [len(indices), L]: waveforms `indices` (default: all B) of workload cfg_id.

    B / L / sr / kind default to the workload's own; passing them lets a test use
    the same recipe at a reduced size."""
    wl = WORKLOADS[cfg_id]
    B = wl["B"] if B is None else B
    L = wl["L"] if L is None else L
    sr = wl["sr"] if sr is None else sr
    kind = wl["kind"] if kind is None else kind
    idx = list(range(B)) if indices is None else [int(i) for i in indices]
    out = np.empty((len(idx), L), dtype=np.float32)

    def fill(i):
        out[i] = waveform(cfg_id, idx[i], L, sr, kind)

    if len(idx) <= 4 or workers <= 1:
        for i in range(len(idx)):
            fill(i)
    else:
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(fill, range(len(idx))))
    return out


# Extra test signals (the families the paper checks its outputs on, Sec. IV-B).

def linear_sweep(L: int, sr: int, f0: float, f1: float, amp: float = 0.5) -> np.ndarray:
    t = np.arange(L, dtype=np.float64) / sr
    dur = L / sr
    phase = 2.0 * np.pi * (f0 * t + 0.5 * (f1 - f0) * t * t / dur)
    return (amp * np.sin(phase)).astype(np.float32)


def log_sweep(L: int, sr: int, f0: float, f1: float, amp: float = 0.5) -> np.ndarray:
    t = np.arange(L, dtype=np.float64) / sr
    dur = L / sr
    k = np.log(f1 / f0) / dur
    phase = 2.0 * np.pi * f0 * (np.exp(k * t) - 1.0) / k
    return (amp * np.sin(phase)).astype(np.float32)


def impulse(L: int, at: int, amp: float = 1.0) -> np.ndarray:
    x = np.zeros(L, dtype=np.float32)
    x[at] = amp
    return x


def tone(L: int, sr: float, f: float, amp: float = 1.0, phase: float = 0.0) -> np.ndarray:
    t = np.arange(L, dtype=np.float64) / sr
    return (amp * np.cos(2.0 * np.pi * f * t + phase)).astype(np.float32)


def validation_signals(L: int = 22050, sr: int = 22050) -> np.ndarray:
    """float32 [4, L]: the kinds of input the paper checks its output on (Sec. IV-B) -- a linear sine
    sweep, a logarithmic sine sweep, an impulse train, and, standing in for the recorded piano scale, a
    chromatic scale of decaying harmonic tones.  Deterministic; generation only."""
    t = np.arange(L, dtype=np.float64) / float(sr)
    dur = L / float(sr)
    f0, f1 = 50.0, 0.45 * sr
    lin = np.sin(2.0 * np.pi * (f0 * t + 0.5 * (f1 - f0) / dur * t * t))
    k = np.log(f1 / f0) / dur
    log = np.sin(2.0 * np.pi * f0 * (np.exp(k * t) - 1.0) / k)
    imp = np.zeros(L)
    imp[L // 8::L // 4] = 1.0
    scale = np.zeros(L)
    n_notes = 12
    seg = L // n_notes
    for i in range(n_notes):
        f = 220.0 * 2.0 ** (i / 12.0)
        tt = t[:seg]
        note = sum(np.sin(2.0 * np.pi * f * h * tt) / h for h in (1, 2, 3, 4) if f * h < 0.5 * sr)
        scale[i * seg:(i + 1) * seg] = 0.25 * note * np.exp(-3.0 * tt)
    return np.stack([0.5 * lin, 0.5 * log, imp, scale]).astype(np.float32)
