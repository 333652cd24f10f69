"""The entry point that allocates nothing: nna_cqt2010v2_static runs the downsampling constant-Q
transform with the library's own static device workspace.  Its output must equal nna_cqt2010v2's (the same
kernels on the same data: bit for bit) on two calls in a row that share the workspace, the second with a
smaller batch; a batch whose workspace exceeds the static one is refused.
"""
import sys

import numpy as np
import pytest

from paper_1912_12055_amd import signals

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


def test_static_workspace_entry_point_matches_the_workspace_one(nb):
    import torch
    kw = dict(sr=22050, hop=512, fmin=32.70, n_bins=84, bins_per_octave=12)
    plan = nb.nna_plan_cqt2010v2(device=0, **kw)
    first = True
    # two calls in a row on the same GPU, the second smaller in both dimensions (its downsampled waveforms
    # land on top of the first call's left-overs)
    for B, L in ((24, 120000), (5, 50001)):
        _say(f"nna_cqt2010v2_static B={B} L={L}")
        x = torch.from_numpy(signals.batch(3, B=B, L=L)).to("cuda:0")
        need = nb.nna_cqt2010v2_workspace(plan, B, L)
        assert 0 < need <= nb.NNA_STATIC_SCRATCH_BYTES
        T = 1 + L // 512
        ref = nb.nna_cqt2010v2(plan, x, out=torch.full((B, 84, T), float("nan"), device="cuda:0"))
        out = torch.full((B, 84, T), float("nan"), device="cuda:0")
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        rc = nb.lib().nna_cqt2010v2_static(plan.handle, x.data_ptr(), B, L, out.data_ptr(),
                                           torch.cuda.current_stream().cuda_stream)
        assert rc == nb.NNA_OK, nb.nna_last_error()
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before  # no device memory taken or returned by the call
        assert torch.isfinite(out).all()
        assert torch.equal(out, ref), (B, L, first)
        first = False


def test_static_workspace_entry_point_through_the_binding_and_its_limit(nb):
    import torch
    plan = nb.nna_plan_cqt2010v2(sr=22050, hop=512, fmin=32.70, n_bins=84, bins_per_octave=12, device=0)
    x = torch.from_numpy(signals.batch(3, B=3, L=70000)).to("cuda:0")
    assert torch.equal(nb.nna_cqt2010v2_static(plan, x), nb.nna_cqt2010v2(plan, x))
    # about 3 B L bytes of workspace: 200 x 120,000 samples need 72 MB, more than the static 64 MiB
    B, L = 200, 120000
    assert nb.nna_cqt2010v2_workspace(plan, B, L) > nb.NNA_STATIC_SCRATCH_BYTES
    big = torch.zeros((B, L), device="cuda:0")
    out = torch.zeros((B, 84, 1 + L // 512), device="cuda:0")
    rc = nb.lib().nna_cqt2010v2_static(plan.handle, big.data_ptr(), B, L, out.data_ptr(), None)
    assert rc == nb.NNA_ERR_SHAPE and "NNA_STATIC_SCRATCH_BYTES" in nb.nna_last_error()
    assert not out.any()  # nothing was launched
    # wrong plan kinds and host-only plans are refused too
    other = nb.nna_plan_cqt2010(sr=22050, hop=512, fmin=32.70, n_bins=84, bins_per_octave=12, device=0)
    with pytest.raises(nb.NnaError) as e:
        nb.nna_cqt2010v2_static(other, x)
    assert e.value.status == nb.NNA_ERR_INVALID_ARG
