"""The selection entry point that allocates nothing (ws_synapse_select_static: its scratch is a fixed array in
the library's device image) against ws_synapse_select on a caller-owned workspace: same landmarks, bit for
bit, on two calls in a row, the second with a smaller input (the array keeps the first call's contents, so
whatever must start at zero has to be cleared by the call itself).  Both kernels are covered: bf16 heads that
stay on chip, and fp32 heads that stream through the array's slabs."""
import numpy as np
import pytest

from paper_2601_01298_amd import synthetic as syn
from _util import to_device

pytestmark = pytest.mark.gpu


def both_ways(ws, torch, K, rho, k, alpha):
    H = K.shape[0]
    ref, ref_score = ws.ws_synapse_select(K, rho, k, alpha, want_score=True)
    idx = torch.full((H, k), -7, dtype=torch.int32, device="cuda")
    score = torch.zeros((H, k), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    allocations = lambda: torch.cuda.memory_stats()["allocation.all.allocated"]     # a count: frees do not move it
    before = allocations()
    ws.ws_synapse_select_static(K, rho, k, alpha, idx, score_out=score)
    assert not ws.ws_synapse_select_failed(None)
    assert allocations() == before                             # nothing came from torch's allocator either
    assert int(idx.min()) >= 0
    assert torch.equal(idx, ref), "landmarks differ between the two entry points"
    assert torch.equal(score, ref_score)
    return idx


def test_select_static_matches_select_on_two_calls_in_a_row():
    import torch
    from paper_2601_01298_amd import binding as ws
    ws.lib()
    # on-chip kernel: 40 heads of 4096 keys, then 5 heads of 1000 keys (fewer slots in use, ragged last block)
    w = syn.small_variant(syn.WORKLOADS[2], H=40, Hq=40, L=4096, k=82)
    Kh = np.stack([syn.cloud(w, h, syn.TENSOR_K) for h in range(w.H)])
    K = to_device(Kh, w.dtype)
    rho = ws.ws_synapse_density(K, [float(syn.bandwidth(Kh[h])) for h in range(w.H)])
    assert ws.ws_synapse_select_plan("auto", ws.WS_BF16, w.H, w.L, w.d).resident
    first = both_ways(ws, torch, K, rho, w.k, w.alpha)
    K2 = K[:5, :1000].contiguous()
    rho2 = ws.ws_synapse_density(K2, [float(syn.bandwidth(Kh[h, :1000])) for h in range(5)])
    both_ways(ws, torch, K2, rho2, 20, w.alpha)
    again = both_ways(ws, torch, K, rho, w.k, w.alpha)         # and back: the first result, from a used array
    assert torch.equal(first, again)

    # streaming kernel (fp32 keys): 3 heads of 2000 keys, then 1 head of 512
    w1 = syn.small_variant(syn.WORKLOADS[1], H=3, Hq=3, L=2000, k=40)
    Kf = np.stack([syn.cloud(w1, h, syn.TENSOR_K) for h in range(w1.H)])
    Kd = to_device(Kf, w1.dtype)
    rhof = ws.ws_synapse_density(Kd, [float(syn.bandwidth(Kf[h])) for h in range(w1.H)])
    assert not ws.ws_synapse_select_plan("auto", ws.WS_F32, w1.H, w1.L, w1.d).resident
    both_ways(ws, torch, Kd, rhof, w1.k, w1.alpha)
    K3 = Kd[:1, :512].contiguous()
    rho3 = ws.ws_synapse_density(K3, [float(syn.bandwidth(Kf[0, :512]))])
    both_ways(ws, torch, K3, rho3, 10, 1.0)

    # a size beyond the fixed array is refused before anything runs
    big = torch.zeros((1, 600_000, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(ws.WsError) as e:
        ws.ws_synapse_select_static(big, torch.ones((1, 600_000), device="cuda"), 4, 0.5,
                                    torch.empty((1, 4), dtype=torch.int32, device="cuda"))
    assert e.value.status == ws.WS_ERR_TOO_LARGE


def test_select_static_on_a_wide_instance():
    """A head that needs 128 workgroups (whole dies per head, four slots polled per lane) through the fixed array:
    the same picks as with a caller-owned workspace, then a narrow shape on the used array."""
    import torch
    from paper_2601_01298_amd import binding as ws
    ws.lib()
    torch.manual_seed(5)
    H, L, d, k = 2, 131072, 128, 48
    plan = ws.ws_synapse_select_plan("auto", ws.WS_BF16, H, L, d)
    assert plan.resident and plan.workgroups_per_head == 128
    K = torch.randn((H, L, d), device="cuda").to(torch.bfloat16)
    rho = torch.rand((H, L), device="cuda") * 0.9 + 0.05
    both_ways(ws, torch, K, rho, k, 0.5)
    K2 = K[:1, :5000].contiguous()
    both_ways(ws, torch, K2, rho[:1, :5000].contiguous(), 30, 0.25)
