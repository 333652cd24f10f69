"""The transform calls allocate nothing and never synchronise, so a caller may record them into a HIP
graph.  Each entry point is captured once and replayed several times with new input written into the
same buffers and eager work between the replays; every replay must reproduce the eager result."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


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


def test_forward_and_backward_calls_replay_from_a_graph(nb):
    import torch
    _say("graph capture and replay of stft / mel / cqt / cqt2010v2 / cqt2010 / stft_backward / cqt_backward")
    dev = "cuda:0"
    B, L = 6, 30000
    gen = torch.Generator(device=dev).manual_seed(5)
    x = 0.3 * torch.randn((B, L), device=dev, generator=gen)
    p_stft = nb.nna_plan_trainable(nb.nna_plan_stft(n_fft=512, hop=128, device=0))
    p_mel = nb.nna_plan_mel(n_fft=512, hop=128, n_mels=40, device=0)
    p_cqt = nb.nna_plan_trainable(nb.nna_plan_cqt(sr=16000, hop=128, fmin=110.0, n_bins=48, device=0))
    # 24 bins per octave, 8,192-tap kernels: the plan folds its kernels about their centres (another kernel)
    p_cqf = nb.nna_plan_cqt(sr=16000, hop=128, fmin=100.0, n_bins=40, bins_per_octave=24, device=0)
    assert p_cqf.info()["executed_flops_per_frame"] < p_cqf.info()["algorithmic_flops_per_frame"]
    p_v2 = nb.nna_plan_cqt2010v2(sr=16000, hop=128, fmin=110.0, n_bins=48, device=0)
    p_fd = nb.nna_plan_cqt2010(sr=16000, hop=128, fmin=110.0, n_bins=48, device=0)
    outs = {k: torch.empty((B,) + nb.nna_out_shape(p, B, L), device=dev)
            for k, p in (("stft", p_stft), ("mel", p_mel), ("cqt", p_cqt), ("cqf", p_cqf), ("v2", p_v2), ("fd", p_fd))}
    outs["mel2"] = torch.empty_like(outs["mel"])
    outs["spec"] = torch.empty_like(outs["stft"])
    ws_v2 = torch.empty(max(16, nb.nna_cqt2010v2_workspace(p_v2, B, L)), dtype=torch.uint8, device=dev)
    ws_fd = torch.empty(max(16, nb.nna_cqt2010v2_workspace(p_fd, B, L)), dtype=torch.uint8, device=dev)
    ws_bw = torch.empty(nb.nna_stft_backward_workspace(p_stft, B, L), dtype=torch.uint8, device=dev)
    gout = torch.randn(outs["stft"].shape, device=dev, generator=gen)
    gw = torch.empty((2 * 257, 512), device=dev)
    gx = torch.empty_like(x)
    ws_cq = torch.empty(nb.nna_cqt_backward_workspace(p_cqt, B, L), dtype=torch.uint8, device=dev)
    gout_cq = torch.randn(outs["cqt"].shape, device=dev, generator=gen)
    gw_cq = torch.empty(nb._bank_shape(p_cqt), device=dev)
    gx_cq = torch.empty_like(x)
    L_ = nb.lib()

    def run_all():
        nb.nna_stft(p_stft, x, outs["stft"])
        nb.nna_mel(p_mel, x, outs["mel"])
        nb.nna_mel_with_stft(p_mel, x, outs["mel2"], outs["spec"])
        nb.nna_cqt(p_cqt, x, outs["cqt"])
        nb.nna_cqt(p_cqf, x, outs["cqf"])
        nb.nna_cqt2010v2(p_v2, x, outs["v2"], workspace=ws_v2)
        nb.nna_cqt2010(p_fd, x, outs["fd"], workspace=ws_fd)
        st = torch.cuda.current_stream().cuda_stream
        nb._check(L_.nna_stft_backward(p_stft.handle, x.data_ptr(), B, L, gout.data_ptr(), gw.data_ptr(), gx.data_ptr(),
                                       ws_bw.data_ptr(), ws_bw.numel(), st))
        nb._check(L_.nna_cqt_backward(p_cqt.handle, x.data_ptr(), B, L, gout_cq.data_ptr(), gw_cq.data_ptr(),
                                      gx_cq.data_ptr(), ws_cq.data_ptr(), ws_cq.numel(), st))

    run_all()  # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run_all()
    for rep in range(3):
        x.copy_(0.3 * torch.randn((B, L), device=dev, generator=gen))  # eager work between replays
        gout.copy_(torch.randn(gout.shape, device=dev, generator=gen))
        for o in outs.values():
            o.fill_(-1.0)
        gout_cq.copy_(torch.randn(gout_cq.shape, device=dev, generator=gen))
        for g_ in (gw, gx, gw_cq, gx_cq):
            g_.fill_(-1.0)
        graph.replay()
        torch.cuda.synchronize()
        got = {k: v.clone() for k, v in outs.items()}
        got_gw, got_gx, got_gw_cq, got_gx_cq = gw.clone(), gx.clone(), gw_cq.clone(), gx_cq.clone()
        run_all()  # the eager result for the same input
        torch.cuda.synchronize()
        for k in outs:
            assert torch.equal(got[k], outs[k]), (rep, k)
        # the gradients are summed with float atomics: equal up to the order of the additions
        for a, b, name in ((got_gw, gw, "gw"), (got_gx, gx, "gx"), (got_gw_cq, gw_cq, "gw cqt"), (got_gx_cq, gx_cq, "gx cqt")):
            err = float((a - b).abs().max() / b.abs().max())
            assert err < 1e-5, (rep, name, err)
