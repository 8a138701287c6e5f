"""The library allocates nothing, never synchronises the host and clears its own scratch with kernels, so a
whole pass of the hot path can be captured in a HIP graph.  The graph is replayed several times, with the
inputs overwritten in place and eager work in between, and every replay must equal the eager result."""
import numpy as np
import pytest

from paper_2601_01298_amd import synthetic as syn
from _util import to_device

pytestmark = pytest.mark.gpu


def test_hot_path_under_graph_capture():
    import torch
    from paper_2601_01298_amd import binding as ws
    ws.lib()
    w = syn.small_variant(syn.WORKLOADS[2], H=24, Hq=24, L=2048, k=41, N=50)
    dt = ws.WS_BF16
    dev = torch.device("cuda")
    K = torch.empty((w.H, w.L, w.d), dtype=torch.bfloat16, device=dev)
    V = torch.empty_like(K)
    Q = to_device(syn.queries(w), w.dtype)
    rho = torch.empty((w.H, w.L), dtype=torch.float32, device=dev)
    idx = torch.empty((w.H, w.k), dtype=torch.int32, device=dev)
    Ks = torch.empty((w.H, w.k, w.d), dtype=torch.bfloat16, device=dev)
    Vs = torch.empty_like(Ks)
    O = torch.empty((w.N, w.Hq, w.d), dtype=torch.float32, device=dev)
    O1 = torch.empty_like(O)              # the one-pass form (rows read from the cache by index)
    wd = torch.empty(ws.ws_synapse_workspace_bytes(ws.WS_OP_DENSITY, dt, w.H, w.L, w.d), dtype=torch.uint8, device=dev)
    wsel = torch.empty(ws.ws_synapse_workspace_bytes(ws.WS_OP_SELECT, dt, w.H, w.L, w.d, w.k), dtype=torch.uint8, device=dev)
    sigma = [3.0] * w.H          # host values are baked into the captured launches: the same for every data set

    def run():
        ws.ws_synapse_density(K, sigma, rho=rho, workspace=wd)
        ws.ws_synapse_select(K, rho, w.k, w.alpha, idx=idx, workspace=wsel, check=False)
        ws.ws_synapse_gather(K, V, idx, Ks=Ks, Vs=Vs)
        ws.ws_synapse_attend(Q, Ks, Vs, O=O)
        ws.ws_synapse_attend_indexed(Q, K, V, idx, O=O1)

    def load(seed):
        Kh = np.stack([syn.cloud(w, h, syn.TENSOR_K, seed) for h in range(w.H)])
        Vh = np.stack([syn.cloud(w, h, syn.TENSOR_V, seed) for h in range(w.H)])
        K.copy_(to_device(Kh, w.dtype))
        V.copy_(to_device(Vh, w.dtype))

    load(syn.BASE_SEED)
    run()                                   # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for rep, seed in enumerate([syn.BASE_SEED, syn.BASE_SEED + 7, syn.BASE_SEED + 8, syn.BASE_SEED]):
        load(seed)
        run()                               # eager reference on the same buffers
        torch.cuda.synchronize()
        ref = (rho.clone(), idx.clone(), Ks.clone(), Vs.clone(), O.clone(), O1.clone())
        assert torch.equal(O, O1)
        for t in (rho, idx, Ks, Vs, O, O1):
            t.zero_()                       # eager work between replays; wipes the outputs
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert int(idx.min()) >= 0 and not ws.ws_synapse_select_failed(wsel)
        for name, a, b in zip(("rho", "idx", "Ks", "Vs", "O", "O (one pass)"), (rho, idx, Ks, Vs, O, O1), ref):
            assert torch.equal(a, b), f"replay {rep}: {name} differs from the eager run"
