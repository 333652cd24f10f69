#!/usr/bin/env python3
"""Throughput of the spectrogram hot path on one MI355X.

One step = one pass of the whole path over the 1,770-waveform workloads: nna_stft and
nna_mel on 1,770 x 176,400 samples @ 44.1 kHz (n_fft 2048, hop 512, 128 mels) and nna_cqt on
1,770 x 176,400 samples @ 44.1 kHz (168 bins, 24 per octave, 65,536 taps).  Inputs are
seeded synthetic waveforms already resident in HBM; plans (kernel banks) are built before
timing, as the paper excludes initialisation from its timings (Sec. IV-A).

Prints one JSON line: whole-job GSamples/s (input samples consumed by the three transforms
per second), per-transform figures, the MFMA roofline of the dominant kernel measured with
HIP events on the launch stream, and the float64 CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3  # MI355X dense fp32 matrix peak
PEAK_F16_MFMA_TFLOPS = 2500.0  # MI355X dense fp16 / bf16 matrix peak
PEAK_HBM_GBS = 8000.0
# the kernel each transform of the step launches (names as rocprofv3 prints them)
KERNELS = {"stft": "stft_fold_kernel<0, 2, true, true>", "mel": "stft_fold_kernel<1, 4, true, true>", "cqt": "cqt_fold_kernel"}


def _read_traffic():
    """HBM bytes per launch of each kernel from the committed rocprofv3 counter summary, if any."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_1770x176400.json.txt")
    try:
        return json.load(open(path))
    except Exception:
        return {}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--batch", type=int, default=1770, help="waveforms per transform (default: the full workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy, so that a rocprofv3 --pmc run of this command "
                         "holds a kernel of known HBM traffic to scale FETCH_SIZE / WRITE_SIZE by")
    ap.add_argument("--only", choices=["stft", "mel", "cqt"], default=None,
                    help="time a single transform (profiling aid); the JSON line then covers that one only")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the transforms timed beside the headline step (linear-frequency STFT, downsampling CQT)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (waveforms are independent, so more GPUs would "
              "just shard the batch); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_1912_12055_amd import binding as nb
    from paper_1912_12055_amd import signals

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU fallback", file=sys.stderr)
        return 2
    nb.lib()
    dev = torch.device("cuda:0")
    B, L, sr = args.batch, 176400, 44100

    def resident(cfg_id):
        x = torch.empty((B, L), dtype=torch.float32, device=dev)
        for s in range(0, B, 256):
            idx = list(range(s, min(B, s + 256)))
            x[s:s + len(idx)] = torch.from_numpy(signals.batch(cfg_id, idx, workers=16)).to(dev)
        return x

    t0 = time.time()
    x4 = resident(4)
    x5 = resident(5)
    t_gen = time.time() - t0

    t0 = time.time()
    p_stft = nb.nna_plan_stft(sr=sr, n_fft=2048, hop=512, device=0)
    p_mel = nb.nna_plan_mel(sr=sr, n_fft=2048, hop=512, n_mels=128, fmin=0.0, fmax=22050.0, device=0)
    p_cqt = nb.nna_plan_cqt(sr=sr, hop=512, fmin=32.70, n_bins=168, bins_per_octave=24, n_taps=0, device=0)
    t_plan = time.time() - t0

    T = 1 + L // 512
    o_stft = torch.empty((B, 1025, T), dtype=torch.float32, device=dev)
    o_mel = torch.empty((B, 128, T), dtype=torch.float32, device=dev)
    o_cqt = torch.empty((B, 168, T), dtype=torch.float32, device=dev)

    legs = {
        "stft": (lambda: nb.nna_stft(p_stft, x4, o_stft), p_stft, o_stft),
        "mel": (lambda: nb.nna_mel(p_mel, x4, o_mel), p_mel, o_mel),
        "cqt": (lambda: nb.nna_cqt(p_cqt, x5, o_cqt), p_cqt, o_cqt),
    }
    names = [args.only] if args.only else ["stft", "mel", "cqt"]

    def step(events=None):
        for n in names:
            if events is not None:
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                legs[n][0]()
                b.record()
                events[n].append((a, b))
            else:
                legs[n][0]()

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)  # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = {n: [] for n in names}
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_per_step = 1e3 * wall / args.steps
    samples_per_step = len(names) * B * L
    value = samples_per_step / (wall / args.steps) / 1e9

    traffic = _read_traffic()
    per = {}
    for n in names:
        ms = float(np.mean([a.elapsed_time(b) for a, b in events[n]]))
        info = legs[n][1].info()
        frames = B * T
        alg = info["algorithmic_flops_per_frame"] * frames
        exe = info["executed_flops_per_frame"] * frames
        out_bytes = legs[n][2].numel() * 4
        # STFT and Mel run the folded contraction (x[n] +- x[N-n] against the first halves of the kernels of
        # eq. (DFT2)): N^2 + 2N flop per frame where the direct form needs 2 N^2.  Their roofline numerator is
        # what the kernel executes (the matrix-instruction counter confirms it), never the direct form's count;
        # that one is quoted beside it as `direct_form_equivalent_tflops`.  The plain STFT halves once more (the
        # folded taps summed by parity give bin k and bin N/2 - k from the kernels of k < N/4): N^2 / 2 + 4N.
        # The CQT runs its kernels folded about their centres (2 sum N_k flop per frame where the direct form needs
        # 4 sum N_k); its 16-row blocks hold bins of one length parity, and what the launch executes is the
        # longest kernel of each block for all 16 rows (`executed`), about 1.5 x the taps inside the kernels
        # themselves (`mfma_frac_useful`).
        folded = exe < alg
        split = folded and exe < 0.3 * alg  # the plain STFT is split once more by tap parity: N^2 / 2 + 4N
        cq_fold = n == "cqt" and folded
        useful = exe if folded else alg
        strict = alg / 2 if cq_fold else useful  # multiply-adds the method itself needs in the form that runs
        per[n] = {
            "ms": round(ms, 4),
            "gsamples_per_s": round(B * L / ms / 1e6, 4),
            "frames_per_s": round(frames / ms * 1e3, 1),
            "contraction": ("kernels folded about their centres, 2 sum N_k flop per frame inside the kernels" if cq_fold
                            else "folded frame split by tap parity, N^2 / 2 + 4N flop per frame" if split
                            else "folded frame, N^2 + 2N flop per frame" if folded else "direct"),
            "algorithmic_tflops": round(useful / ms / 1e9, 3),
            "executed_tflops": round(exe / ms / 1e9, 3),
            "mfma_frac": round(useful / ms / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4),
            "mfma_frac_executed": round(exe / ms / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4),
            "mfma_frac_useful": round(strict / ms / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4),
            "direct_form_equivalent_tflops": round(alg / ms / 1e9, 3) if folded else None,
            "algorithmic_gb": round((B * L * 4 + out_bytes) / 1e9, 4),
            "hbm_frac": round((B * L * 4 + out_bytes) / ms / 1e6 / PEAK_HBM_GBS, 5),
            "hbm_traffic_bytes": traffic.get(n),
        }
    dom = max(names, key=lambda n: per[n]["ms"])
    roofline = {
        "kernel": KERNELS[dom],
        "bound": "mfma",
        "achieved": per[dom]["algorithmic_tflops"],
        "peak": PEAK_FP32_MFMA_TFLOPS,
        "unit": "TFLOP/s",
        "frac": per[dom]["mfma_frac"],
        "frac_useful": per[dom]["mfma_frac_useful"],
        "traffic": traffic.get(dom),
    }
    # the kernel of the step that sits furthest below its roof, by the strictest count: the multiply-adds the form
    # that runs needs (for the folded CQT the taps inside the kernels, not the zeros its blocks multiply as well)
    low = min(names, key=lambda n: per[n]["mfma_frac_useful"])
    roofline_min = {"kernel": KERNELS[low], "frac": per[low]["mfma_frac_useful"],
                    "frac_executed": per[low]["mfma_frac_executed"]}

    # Timed beside the step, never part of `value`: the same batch through the STFT on the linear
    # frequency axis of Sec. II-B's worked example, through the downsampling CQT (Sec. III-C) and through
    # the STFT with float16 operands; and the CQT with frequency-domain kernels on a smaller batch.
    # the waveforms the cpu_baseline leg will run the oracle on: keep the GPU's results for them, so that
    # the oracle's outputs are compared with them afterwards (outside every timed region)
    n_cpu = min(B, 96)
    cpu_idx = sorted({int(i) for i in np.linspace(0, B - 1, n_cpu)})
    gpu_sample = {}
    if not args.no_cpu_baseline:
        for n in names:
            legs[n][0]()
        torch.cuda.synchronize()
        gpu_sample = {n: legs[n][2][cpu_idx].cpu().numpy() for n in names}

    extras = None
    if not args.no_extras and not args.only:
        extras = {}
        del o_stft, o_mel
        p_lin = nb.nna_plan_stft_scaled(sr=sr, n_fft=2048, hop=512, freq_scale=nb.NNA_FREQ_LINEAR, fmin=50.0,
                                        fmax=6000.0, freq_bins=1025, device=0)
        p_2010 = nb.nna_plan_cqt2010v2(sr=sr, hop=512, fmin=32.70, n_bins=168, bins_per_octave=24, device=0)
        o_lin = torch.empty((B, 1025, T), dtype=torch.float32, device=dev)
        ws = torch.empty(max(16, nb.nna_cqt2010v2_workspace(p_2010, B, L)), dtype=torch.uint8, device=dev)
        p_h = nb.nna_plan_stft_prec(sr=sr, n_fft=2048, hop=512, precision=nb.NNA_PREC_F16, device=0)
        # the CQT with frequency-domain kernels costs an STFT of n_fft = 16,384 per 64 bins: timed on the
        # smaller CQT workload's waveforms (220,500 samples @ 22,050 Hz, 84 bins, 12 per octave), 152 of
        # them, which makes 1,024 workgroups (two per compute unit, twice over)
        B3 = 152
        x3 = torch.from_numpy(signals.batch(3, list(range(B3)), workers=16)).to(dev)
        p_1992 = nb.nna_plan_cqt1992(sr=22050, hop=512, fmin=32.70, n_bins=84, bins_per_octave=12, device=0)
        o_1992 = torch.empty((B3, 84, 1 + 220500 // 512), dtype=torch.float32, device=dev)
        p_2010f = nb.nna_plan_cqt2010(sr=sr, hop=512, fmin=32.70, n_bins=168, bins_per_octave=24, device=0)
        full = (B * L, B * T)
        for name, fn, plan, (n_samples, n_frames) in (
                ("stft_linear_axis", lambda: nb.nna_stft(p_lin, x4, o_lin), p_lin, full),
                ("cqt2010v2", lambda: nb.nna_cqt2010v2(p_2010, x5, o_cqt, workspace=ws), p_2010, full),
                ("cqt2010", lambda: nb.nna_cqt2010(p_2010f, x5, o_cqt, workspace=ws), p_2010f, full),
                ("stft_f16_operands", lambda: nb.nna_stft(p_h, x4, o_lin), p_h, full),
                ("cqt1992_152x220500", lambda: nb.nna_cqt1992(p_1992, x3, o_1992), p_1992, (B3 * 220500, B3 * 431))):
            for _ in range(max(1, args.warmup)):
                fn()
            ev = []
            for _ in range(args.steps):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                fn()
                b.record()
                ev.append((a, b))
            torch.cuda.synchronize()
            ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
            info = plan.info()
            extras[name] = {
                "ms": round(ms, 4),
                "gsamples_per_s": round(n_samples / ms / 1e6, 4),
                "algorithmic_tflops": round(info["algorithmic_flops_per_frame"] * n_frames / ms / 1e9, 3),
                "executed_tflops": round(info["executed_flops_per_frame"] * n_frames / ms / 1e9, 3),
                "mfma_frac": round(info["algorithmic_flops_per_frame"] * n_frames / ms / 1e9
                                   / (PEAK_F16_MFMA_TFLOPS if name == "stft_f16_operands" else PEAK_FP32_MFMA_TFLOPS), 4),
                "mfma_peak_tflops": PEAK_F16_MFMA_TFLOPS if name == "stft_f16_operands" else PEAK_FP32_MFMA_TFLOPS,
            }
        # The paper's own timing parameters (Sec. IV-A): n_fft 4096 / hop 512 STFT, 512 Mel filters on it, and the
        # 24-bins-per-octave CQT, on 1,770 clips of 80,000 samples at 44.1 kHz -- the shape of its MAPS excerpts
        # with synthetic content (the first 80,000 samples of the same waveforms).
        Lp, Tp = 80000, 1 + 80000 // 512
        x4p = x4[:, :Lp].contiguous()
        x5p = x5[:, :Lp].contiguous()
        p_s4 = nb.nna_plan_stft(sr=sr, n_fft=4096, hop=512, device=0)
        p_m4 = nb.nna_plan_mel(sr=sr, n_fft=4096, hop=512, n_mels=512, fmin=0.0, fmax=22050.0, device=0)
        p_c4 = nb.nna_plan_cqt(sr=sr, hop=512, fmin=32.70, n_bins=168, bins_per_octave=24, n_taps=0, device=0)
        o_s4 = torch.empty((B, 2049, Tp), dtype=torch.float32, device=dev)
        o_m4 = torch.empty((B, 512, Tp), dtype=torch.float32, device=dev)
        o_c4 = torch.empty((B, 168, Tp), dtype=torch.float32, device=dev)
        paper = {}
        for name, fn, plan, out_t, xin, cfg in (
                ("stft_n4096", lambda: nb.nna_stft(p_s4, x4p, o_s4), p_s4, o_s4, x4p, 4),
                ("mel_n4096_512mels", lambda: nb.nna_mel(p_m4, x4p, o_m4), p_m4, o_m4, x4p, 4),
                ("cqt_168bins", lambda: nb.nna_cqt(p_c4, x5p, o_c4), p_c4, o_c4, x5p, 5)):
            for _ in range(max(1, args.warmup)):
                fn()
            ev = []
            for _ in range(args.steps):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                fn()
                b.record()
                ev.append((a, b))
            torch.cuda.synchronize()
            ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
            info = plan.info()
            exe, alg = info["executed_flops_per_frame"] * B * Tp, info["algorithmic_flops_per_frame"] * B * Tp
            paper[name] = {
                "ms": round(ms, 4),
                "gsamples_per_s": round(B * Lp / ms / 1e6, 4),
                "executed_tflops": round(exe / ms / 1e9, 3),
                "mfma_frac": round(min(exe, alg) / ms / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4),
                "mfma_frac_executed": round(exe / ms / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4),
                "sample": (out_t, xin, cfg),
            }
        extras["paper_parameters_1770x80000"] = paper
        del x4p, x5p
        # Mel and the power spectrogram it is computed from, both written by one launch (one contraction)
        p_mel2 = nb.nna_plan_mel(sr=sr, n_fft=2048, hop=512, n_mels=128, fmin=0.0, fmax=22050.0, device=0)
        o_mel2 = torch.empty((B, 128, T), dtype=torch.float32, device=dev)
        for _ in range(max(1, args.warmup)):
            nb.nna_mel_with_stft(p_mel2, x4, o_mel2, o_lin)
        ev = []
        for _ in range(args.steps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            nb.nna_mel_with_stft(p_mel2, x4, o_mel2, o_lin)
            b.record()
            ev.append((a, b))
        torch.cuda.synchronize()
        ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
        # the launch runs the folded contraction split by tap parity: the fraction of the peak is of the flops it
        # executes; the direct form's count is quoted beside it
        info2 = p_mel2.info()
        alg = info2["algorithmic_flops_per_frame"] * B * T
        exe = info2["executed_flops_per_frame"] * B * T
        extras["mel_with_stft"] = {
            "ms": round(ms, 4),
            "gsamples_per_s": round(B * L / ms / 1e6, 4),
            "direct_form_tflops": round(alg / ms / 1e9, 3),
            "executed_tflops": round(exe / ms / 1e9, 3),
            "mfma_frac": round(exe / ms / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4),
            "mfma_peak_tflops": PEAK_FP32_MFMA_TFLOPS,
        }
        del o_lin, ws, x3, o_1992, o_mel2, p_mel2
        # backward pass of the STFT layer (trainable kernels): dLoss/dW and dLoss/dx for the same batch.
        # Algorithmic work: the forward contraction again (2 N^2 per frame) + the bank gradient (2 N^2)
        # + the waveform gradient (2 N^2) = 6 N^2 flop per frame.
        p_tr = nb.nna_plan_trainable(nb.nna_plan_stft(sr=sr, n_fft=2048, hop=512, device=0))
        gout = torch.ones((B, 1025, T), dtype=torch.float32, device=dev)
        ws_bw = torch.empty(nb.nna_stft_backward_workspace(p_tr, B, L), dtype=torch.uint8, device=dev)
        for _ in range(max(1, args.warmup)):
            nb.nna_stft_backward(p_tr, x4, gout, workspace=ws_bw)
        ev = []
        for _ in range(args.steps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            nb.nna_stft_backward(p_tr, x4, gout, workspace=ws_bw)
            b.record()
            ev.append((a, b))
        torch.cuda.synchronize()
        ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
        alg = 3 * p_tr.info()["algorithmic_flops_per_frame"] * B * T
        extras["stft_backward"] = {
            "ms": round(ms, 4),
            "gsamples_per_s": round(B * L / ms / 1e6, 4),
            "algorithmic_tflops": round(alg / ms / 1e9, 3),
            "mfma_frac": round(alg / ms / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4),
            "mfma_peak_tflops": PEAK_FP32_MFMA_TFLOPS,
        }
        del gout, ws_bw, p_tr
        # backward pass of the Mel layer (filterbank, kernel-bank and waveform gradients): the three
        # contractions above plus the Mel stage's two small ones (2 n_mels F flop per frame each)
        p_trm = nb.nna_plan_trainable(nb.nna_plan_mel(sr=sr, n_fft=2048, hop=512, n_mels=128, fmin=0.0, fmax=22050.0, device=0))
        gmel = torch.ones((B, 128, T), dtype=torch.float32, device=dev)
        ws_bw = torch.empty(nb.nna_mel_backward_workspace(p_trm, B, L), dtype=torch.uint8, device=dev)
        for _ in range(max(1, args.warmup)):
            nb.nna_mel_backward(p_trm, x4, gmel, workspace=ws_bw)
        ev = []
        for _ in range(args.steps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            nb.nna_mel_backward(p_trm, x4, gmel, workspace=ws_bw)
            b.record()
            ev.append((a, b))
        torch.cuda.synchronize()
        ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
        alg = (3 * 2.0 * 2048 * 2048 + 2 * 2.0 * 128 * 1025) * B * T
        extras["mel_backward"] = {
            "ms": round(ms, 4),
            "gsamples_per_s": round(B * L / ms / 1e6, 4),
            "algorithmic_tflops": round(alg / ms / 1e9, 3),
            "mfma_frac": round(alg / ms / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4),
            "mfma_peak_tflops": PEAK_FP32_MFMA_TFLOPS,
        }
        del gmel, ws_bw, p_trm
        # backward pass of the constant-Q layer with trainable time-domain kernels: the forward contraction
        # again, the bank gradient and the waveform gradient, 4 sum(N_k) flop per frame each
        p_trc = nb.nna_plan_trainable(nb.nna_plan_cqt(sr=sr, hop=512, fmin=32.70, n_bins=168, bins_per_octave=24,
                                                      n_taps=65536, device=0))
        gcq = torch.ones((B, 168, T), dtype=torch.float32, device=dev)
        ws_bw = torch.empty(nb.nna_cqt_backward_workspace(p_trc, B, L), dtype=torch.uint8, device=dev)
        for _ in range(max(1, args.warmup)):
            nb.nna_cqt_backward(p_trc, x5, gcq, workspace=ws_bw)
        ev = []
        for _ in range(args.steps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            nb.nna_cqt_backward(p_trc, x5, gcq, workspace=ws_bw)
            b.record()
            ev.append((a, b))
        torch.cuda.synchronize()
        ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
        alg = 3 * p_trc.info()["algorithmic_flops_per_frame"] * B * T
        extras["cqt_backward"] = {
            "ms": round(ms, 4),
            "gsamples_per_s": round(B * L / ms / 1e6, 4),
            "algorithmic_tflops": round(alg / ms / 1e9, 3),
            "mfma_frac": round(alg / ms / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4),
            "mfma_peak_tflops": PEAK_FP32_MFMA_TFLOPS,
        }
        del ws_bw, p_trc
        # backward pass of the downsampling CQT with trainable time-domain kernels (7 octaves sharing the top octave's
        # kernels; the waveform gradient climbs through the transposed decimation steps); flops as for its forward
        # pass (nna_plan_info), three times: forward again, kernel gradient, waveform gradient
        p_trv = nb.nna_plan_trainable(nb.nna_plan_cqt2010v2(sr=sr, hop=512, fmin=32.70, n_bins=168, bins_per_octave=24, device=0))
        ws_bw = torch.empty(nb.nna_cqt2010v2_backward_workspace(p_trv, B, L), dtype=torch.uint8, device=dev)
        for _ in range(max(1, args.warmup)):
            nb.nna_cqt2010v2_backward(p_trv, x5, gcq, workspace=ws_bw)
        ev = []
        for _ in range(args.steps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            nb.nna_cqt2010v2_backward(p_trv, x5, gcq, workspace=ws_bw)
            b.record()
            ev.append((a, b))
        torch.cuda.synchronize()
        ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
        alg = 3 * p_trv.info()["algorithmic_flops_per_frame"] * B * T
        extras["cqt2010v2_backward"] = {
            "ms": round(ms, 4),
            "gsamples_per_s": round(B * L / ms / 1e6, 4),
            "algorithmic_tflops": round(alg / ms / 1e9, 3),
            "mfma_frac": round(alg / ms / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4),
            "mfma_peak_tflops": PEAK_FP32_MFMA_TFLOPS,
        }
        del ws_bw, p_trv
        # backward pass of the downsampling CQT with trainable frequency-domain kernels (both stages' kernels are
        # weights: the DFT bank of the un-windowed STFT and the spectral kernels); flops: its forward pass three times
        p_trf = nb.nna_plan_trainable(nb.nna_plan_cqt2010(sr=sr, hop=512, fmin=32.70, n_bins=168, bins_per_octave=24, device=0))
        ws_bw = torch.empty(nb.nna_cqt2010_backward_workspace(p_trf, B, L), dtype=torch.uint8, device=dev)
        for _ in range(max(1, args.warmup)):
            nb.nna_cqt2010_backward(p_trf, x5, gcq, workspace=ws_bw)
        ev = []
        for _ in range(args.steps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            nb.nna_cqt2010_backward(p_trf, x5, gcq, workspace=ws_bw)
            b.record()
            ev.append((a, b))
        torch.cuda.synchronize()
        ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
        alg = 3 * p_trf.info()["algorithmic_flops_per_frame"] * B * T
        extras["cqt2010_backward"] = {
            "ms": round(ms, 4),
            "gsamples_per_s": round(B * L / ms / 1e6, 4),
            "algorithmic_tflops": round(alg / ms / 1e9, 3),
            "mfma_frac": round(alg / ms / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4),
            "mfma_peak_tflops": PEAK_FP32_MFMA_TFLOPS,
        }
        del gcq, ws_bw, p_trf
        # backward pass of the one-rate CQT with trainable frequency-domain kernels, on the 152-waveform batch of its
        # forward figure above (84 bins, n_fft 16,384)
        x92 = torch.from_numpy(signals.batch(3, list(range(152)), workers=16)).to(dev)
        p_tr92 = nb.nna_plan_trainable(nb.nna_plan_cqt1992(sr=22050, hop=512, fmin=32.70, n_bins=84, bins_per_octave=12, device=0))
        B92, L92 = x92.shape
        T92 = 1 + L92 // 512
        g92 = torch.ones((B92, 84, T92), dtype=torch.float32, device=dev)
        ws_bw = torch.empty(nb.nna_cqt1992_backward_workspace(p_tr92, B92, L92), dtype=torch.uint8, device=dev)
        for _ in range(max(1, args.warmup)):
            nb.nna_cqt1992_backward(p_tr92, x92, g92, workspace=ws_bw)
        ev = []
        for _ in range(args.steps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            nb.nna_cqt1992_backward(p_tr92, x92, g92, workspace=ws_bw)
            b.record()
            ev.append((a, b))
        torch.cuda.synchronize()
        ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
        alg = 3 * p_tr92.info()["algorithmic_flops_per_frame"] * B92 * T92
        extras["cqt1992_backward_152x220500"] = {
            "ms": round(ms, 4),
            "gsamples_per_s": round(B92 * L92 / ms / 1e6, 4),
            "algorithmic_tflops": round(alg / ms / 1e9, 3),
            "mfma_frac": round(alg / ms / 1e9 / PEAK_FP32_MFMA_TFLOPS, 4),
            "mfma_peak_tflops": PEAK_FP32_MFMA_TFLOPS,
        }
        del x92, g92, ws_bw, p_tr92

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        idx = cpu_idx
        n_cpu = len(idx)
        xs4 = signals.batch(4, idx)
        xs5 = signals.batch(5, idx)
        ref = {}
        t0 = time.perf_counter()
        done = 0
        if "stft" in names:
            ref["stft"] = oracle.stft(xs4, n_fft=2048, hop=512)
            done += 1
        if "mel" in names:
            ref["mel"] = oracle.mel(xs4, sr=sr, n_fft=2048, hop=512, n_mels=128, fmin=0.0, fmax=22050.0)
            done += 1
        if "cqt" in names:
            ref["cqt"] = oracle.cqt(xs5, sr=sr, hop=512, fmin=32.70, n_bins=168, bins_per_octave=24, n_taps=65536)
            done += 1
        t_cpu = time.perf_counter() - t0
        # parity of this very run: per waveform max |gpu - oracle| / max |oracle|, the worst over the sample
        for n in names:
            got = gpu_sample[n].astype(np.float64)
            per[n]["max_rel_err"] = float(max(
                np.abs(got[i] - ref[n][i]).max() / np.abs(ref[n][i]).max() for i in range(n_cpu)))
            per[n]["max_rel_err_waveforms"] = n_cpu
        cpu = {
            "value": round(done * n_cpu * L / t_cpu / 1e9, 6),
            "unit": "GSamples/s",
            "cores": oracle.threads(),
            "kind": "oracle",
            "sample": f"{n_cpu} of the {B} waveforms (evenly spaced indices) through the same {done} transforms, "
                      f"{t_cpu:.1f} s of float64 oracle time",
        }

    if extras and "paper_parameters_1770x80000" in extras:
        paper = extras["paper_parameters_1770x80000"]
        if not args.no_cpu_baseline:
            import oracle
            pidx = [0, B // 2, B - 1]
            for name, entry in paper.items():
                out_t, xin, cfg = entry["sample"]
                xs = signals.batch(cfg, pidx)[:, :80000]
                if name == "stft_n4096":
                    ref = oracle.stft(xs, n_fft=4096, hop=512)
                elif name == "mel_n4096_512mels":
                    ref = oracle.mel(xs, sr=sr, n_fft=4096, hop=512, n_mels=512, fmin=0.0, fmax=22050.0)
                else:
                    ref = oracle.cqt(xs, sr=sr, hop=512, fmin=32.70, n_bins=168, bins_per_octave=24, n_taps=65536)
                got = out_t[pidx].cpu().numpy().astype(np.float64)
                entry["max_rel_err"] = float(max(np.abs(got[i] - ref[i]).max() / np.abs(ref[i]).max() for i in range(len(pidx))))
        for entry in paper.values():
            entry.pop("sample", None)

    line = {
        "metric": "GSamples/s per transform (STFT/Mel/CQT) + % of MFMA roofline, 1 MI355X",
        "value": round(value, 4),
        "unit": "GSamples/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": "1,770 waveforms x 176,400 samples @ 44.1 kHz through " + "+".join(names)
                        + " (STFT/Mel: n_fft 2048, hop 512, 128 mels; CQT: 168 bins, 24/octave, 65,536 taps)",
            "batch": B, "samples_per_waveform": L, "frames_per_waveform": T,
            "value_definition": "input samples consumed by the timed transforms per second, whole step",
        },
        "per_transform": per,
        "roofline": roofline,
        "roofline_min": roofline_min,
        "cpu_baseline": cpu,
        "extras": extras,
        "setup_s": {"input_generation": round(t_gen, 2), "plans": round(t_plan, 2)},
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
