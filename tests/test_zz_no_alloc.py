"""mggcn_softmax_ce_static -- the entry point for callers that cannot allocate -- against
mggcn_softmax_ce (same kernels: the results must be the same bits) and against the oracle, on two
calls in a row, the second on a smaller input (the built-in buffer keeps the first call's partials)."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


def test_softmax_ce_static_matches_the_workspace_form(ref):
    import torch

    import paper_2110_08688_amd as mg

    mg.binding.lib()
    dev = torch.device("cuda:0")
    loss_s = torch.empty(1, dtype=torch.float32, device=dev)
    for n, C, ld in ((300_000, 41, 48), (1_237, 8, 8), (70_001, 600, 600), (5, 3, 16)):
        print(f"[softmax_ce_static] n={n} C={C} ld={ld}", flush=True)
        Z = wl.normal_f32(900 + C, 1, (n, ld)) * 3.0
        y = wl.labels_i32(900 + C, 2, n, C)
        Zd, yd = torch.from_numpy(Z).to(dev), torch.from_numpy(y).to(dev)
        # reference form first (it allocates its workspace and its outputs)
        loss_w, d_w = mg.mggcn_softmax_ce(Zd[:, :C].clone(), yd)
        d_s = torch.full((n, ld), 7.0, device=dev)
        torch.cuda.synchronize()
        zin, dout = Zd[:, :C], d_s[:, :C]
        before = torch.cuda.memory_stats()["allocation.all.allocated"]  # allocations made so far, cumulative
        mg.mggcn_softmax_ce_static(zin, yd, loss_s, dlogits=dout)
        torch.cuda.synchronize()
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before, "the call went through torch's allocator"
        assert loss_s.item() == loss_w.item()
        assert torch.equal(d_s[:, :C], d_w)
        assert bool((d_s[:, C:] == 7.0).all()), "padding columns must stay untouched"
        r_loss, r_d = ref.softmax_ce(Z[:, :C].astype(np.float64), y)
        assert abs(loss_s.item() - r_loss) <= 1e-5 * abs(r_loss)
        got = d_s[:, :C].cpu().numpy().astype(np.float64)
        err = np.abs(got - r_d).max(axis=1) / np.abs(r_d).max(axis=1)
        assert err.max() <= 1e-4
        # in place, as the epoch uses it
        Zi = Zd.clone()
        mg.mggcn_softmax_ce_static(Zi[:, :C], yd, loss_s)
        assert torch.equal(Zi[:, :C], d_w) and loss_s.item() == loss_w.item()


def test_softmax_ce_static_argument_errors():
    import torch

    import paper_2110_08688_amd as mg

    dev = torch.device("cuda:0")
    Z = torch.zeros((4, 8), device=dev)
    y = torch.zeros(4, dtype=torch.int32, device=dev)
    loss = torch.empty(1, device=dev)
    L = mg.binding.lib()
    assert L.mggcn_softmax_ce_static(0, 8, Z.data_ptr(), 8, y.data_ptr(), loss.data_ptr(), Z.data_ptr(), 8, None) == mg.binding.E_INVALID_ARG
    assert L.mggcn_softmax_ce_static(4, 8, Z.data_ptr(), 4, y.data_ptr(), loss.data_ptr(), Z.data_ptr(), 8, None) == mg.binding.E_INVALID_ARG
    assert L.mggcn_softmax_ce_static(4, 8, None, 8, y.data_ptr(), loss.data_ptr(), Z.data_ptr(), 8, None) == mg.binding.E_INVALID_ARG
    assert L.mggcn_softmax_ce_static((1 << 40) + 1, 8, Z.data_ptr(), 8, y.data_ptr(), loss.data_ptr(), Z.data_ptr(), 8,
                                     None) == mg.binding.E_UNSUPPORTED
    assert b"mggcn_softmax_ce_static" in L.mggcn_last_error()
