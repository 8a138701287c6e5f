"""Two HIP streams, two synapse buffers (Warp-Cortex Sec. 4: the main stream pushes a new synapse while the side
agents keep reading the one they have).  Every call takes a stream and allocates nothing, so a producer stream
can refresh the density for appended rows, re-select and gather into the BACK buffer while a consumer stream
runs the agents' attention over the FRONT buffer; the buffers then swap.  Results must equal those of the same
calls made one after the other on one stream."""
import numpy as np
import pytest

from paper_2601_01298_amd import synthetic as syn
from _util import to_device

pytestmark = pytest.mark.gpu


def test_producer_and_consumer_streams_with_two_synapse_buffers():
    import torch
    from paper_2601_01298_amd import binding as ws
    ws.lib()
    w = syn.small_variant(syn.WORKLOADS[2], H=16, Hq=16, L=3000, k=60, N=100)
    dt = ws.WS_BF16
    dev = torch.device("cuda")
    steps, m = 4, 2                              # the context grows by m rows per producer step
    Lcap = w.L + steps * m
    wfull = syn.small_variant(w, L=Lcap)
    Kall = to_device(np.stack([syn.cloud(wfull, h, syn.TENSOR_K) for h in range(w.H)]), w.dtype)
    Vall = to_device(np.stack([syn.cloud(wfull, h, syn.TENSOR_V) for h in range(w.H)]), w.dtype)
    Q = to_device(syn.queries(w), w.dtype)
    sigma = [3.0] * w.H

    def buffers():
        return (torch.empty((w.H, w.k, w.d), dtype=torch.bfloat16, device=dev),
                torch.empty((w.H, w.k, w.d), dtype=torch.bfloat16, device=dev))

    def produce(L, rho_prev, Ks, Vs, wsel, wapp, stream):
        """density refresh for the rows appended since the last call, selection, gather into (Ks, Vs)"""
        K = Kall[:, :L].contiguous()
        V = Vall[:, :L].contiguous()
        if rho_prev is None:
            wd = torch.empty(ws.ws_synapse_workspace_bytes(ws.WS_OP_DENSITY, dt, w.H, L, w.d), dtype=torch.uint8, device=dev)
            rho = ws.ws_synapse_density(K, sigma, workspace=wd, stream=stream)
        else:
            rho = torch.empty((w.H, L), dtype=torch.float32, device=dev)
            ws.ws_synapse_density_append(K, m, sigma, rho_prev, rho_new=rho, workspace=wapp, stream=stream)
        idx = torch.empty((w.H, w.k), dtype=torch.int32, device=dev)
        ws.ws_synapse_select(K, rho, w.k, w.alpha, idx=idx, workspace=wsel, stream=stream, check=False)
        ws.ws_synapse_gather(K, V, idx, Ks=Ks, Vs=Vs, stream=stream)
        return rho, idx

    wsel = torch.empty(ws.ws_synapse_workspace_bytes(ws.WS_OP_SELECT, dt, w.H, Lcap, w.d, w.k), dtype=torch.uint8, device=dev)
    wapp = torch.empty(ws.ws_synapse_workspace_bytes(ws.WS_OP_DENSITY_APPEND, dt, w.H, Lcap, w.d, m), dtype=torch.uint8,
                       device=dev)

    # ---- reference: everything in order on the current stream
    ref_O, ref_idx = [], []
    rho = None
    Ks, Vs = buffers()
    for s in range(steps + 1):
        rho, idx = produce(w.L + s * m, rho, Ks, Vs, wsel, wapp, None)
        ref_idx.append(idx.clone())
        ref_O.append(ws.ws_synapse_attend(Q, Ks, Vs).clone())
    torch.cuda.synchronize()

    # ---- two streams, two buffers
    prod, cons = torch.cuda.Stream(), torch.cuda.Stream()
    front, back = buffers(), buffers()
    got_O, got_idx = [], []
    with torch.cuda.stream(prod):
        rho, idx = produce(w.L, None, front[0], front[1], wsel, wapp, prod)
    got_idx.append(idx)
    ready = torch.cuda.Event()
    ready.record(prod)
    for s in range(1, steps + 1):
        # agents read the front buffer on their stream ...
        cons.wait_event(ready)
        with torch.cuda.stream(cons):
            O = torch.empty((w.N, w.Hq, w.d), dtype=torch.float32, device=dev)
            ws.ws_synapse_attend(Q, front[0], front[1], O=O, stream=cons)
        got_O.append(O)
        read_done = torch.cuda.Event()
        read_done.record(cons)
        # ... while the producer fills the back buffer for the grown context
        with torch.cuda.stream(prod):
            rho, idx = produce(w.L + s * m, rho, back[0], back[1], wsel, wapp, prod)
        got_idx.append(idx)
        ready = torch.cuda.Event()
        ready.record(prod)
        # the buffer the agents have just read becomes the next back buffer once they are through with it
        prod.wait_event(read_done)
        front, back = back, front
    cons.wait_event(ready)
    with torch.cuda.stream(cons):
        O = torch.empty((w.N, w.Hq, w.d), dtype=torch.float32, device=dev)
        ws.ws_synapse_attend(Q, front[0], front[1], O=O, stream=cons)
    got_O.append(O)
    torch.cuda.synchronize()

    assert not ws.ws_synapse_select_failed(wsel)      # the flag block at the head of the selection workspace
    for s in range(steps + 1):
        assert int(got_idx[s].min()) >= 0
        assert torch.equal(got_idx[s], ref_idx[s]), f"step {s}: landmarks differ between the two schedules"
        assert torch.equal(got_O[s], ref_O[s]), f"step {s}: attention output differs between the two schedules"
