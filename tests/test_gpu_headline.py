"""Headline workload at FULL size (24 layers x 16 KV heads -> H = 384, L = 32768, d = 64, k = 655,
N = 100 agents, bf16), in the launch configuration bench.py times.  A float64 density of all 384
heads is beyond a test, so: attention and gather are compared with the oracle on all heads; the
density on sampled rows of all heads and on every key of 102 heads; the 655 picks of every head
are compared with the oracle's (102 heads through the whole chain from the oracle's own density,
the other 282 with the oracle fed the library's density); properties that hold at any size are
checked on all heads."""
import numpy as np
import pytest

from paper_2601_01298_amd import synthetic as syn
from _util import TIE_TOL, attn_rel_err, check_indices

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(900)
def test_headline_full_size(oracle, say):
    import torch
    from concurrent.futures import ThreadPoolExecutor
    from paper_2601_01298_amd import binding as ws
    ws.lib()
    w = syn.WORKLOADS[3]
    sigma = np.empty(w.H, dtype=np.float32)

    def fill(tensor):
        out = np.empty((w.H, w.L, w.d), dtype=np.uint16)

        def one(h):
            x = syn.cloud(w, h, tensor)
            if tensor == syn.TENSOR_K:
                sigma[h] = syn.bandwidth(x)
            out[h] = syn.bf16_bits(x)

        with ThreadPoolExecutor(max_workers=16) as ex:
            list(ex.map(one, range(w.H)))
        return torch.from_numpy(out).view(torch.bfloat16).cuda()

    K, V = fill(syn.TENSOR_K), fill(syn.TENSOR_V)
    Qh = syn.queries(w)
    Q = torch.from_numpy(Qh).to(torch.bfloat16).cuda()
    say(f"inputs resident: K,V {tuple(K.shape)} bf16, Q {tuple(Q.shape)}")

    rho = ws.ws_synapse_density(K, [float(s) for s in sigma])
    idx, score = ws.ws_synapse_select(K, rho, w.k, w.alpha, want_score=True)
    Ks, Vs = ws.ws_synapse_gather(K, V, idx)
    O = ws.ws_synapse_attend(Q, Ks, Vs)
    # the one-pass form reads the same rows from the cache and must give the same bits
    assert torch.equal(ws.ws_synapse_attend_indexed(Q, K, V, idx).view(torch.int32), O.view(torch.int32))
    torch.cuda.synchronize()
    say("GPU path done")

    # ---- properties on ALL heads
    assert float(rho.min()) >= (1.0 / w.L) * (1 - 1e-5) and float(rho.max()) <= 1.0 + 1e-5
    assert int(idx.min()) >= 0 and int(idx.max()) < w.L
    srt = torch.sort(idx, dim=1).values
    assert bool((srt[:, 1:] != srt[:, :-1]).all()), "a head chose the same key twice"
    # first pick is the lowest-density key of its head (alpha < 1): lowest index among the minima
    first = idx[:, 0].long()
    rmin = rho.min(dim=1).values
    assert bool((rho.gather(1, first[:, None])[:, 0] == rmin).all())
    assert bool((score > 0).all()) and bool((score <= 1.0 + 1e-6).all())
    # gather is a bit copy on all heads
    ref_Ks = torch.gather(K.view(torch.int16), 1, idx.long()[:, :, None].expand(-1, -1, w.d))
    assert bool((ref_Ks == Ks.view(torch.int16)).all())
    ref_Vs = torch.gather(V.view(torch.int16), 1, idx.long()[:, :, None].expand(-1, -1, w.d))
    assert bool((ref_Vs == Vs.view(torch.int16)).all())
    assert bool(torch.isfinite(O).all())
    # attention on ALL heads against the oracle, as a stage on identical inputs: the rows are the input keys' rows at the
    # chosen positions (bit copies, just checked), the oracle's attention is cheap at k rows per head.  (Whether the
    # positions are the right ones is the business of the full-chain comparison below, which feeds the oracle's own
    # density and picks forward.)
    Ks_h, Vs_h, O_h = Ks.float().cpu().numpy(), Vs.float().cpu().numpy(), O.cpu().numpy()
    worst_att = 0.0
    for h0 in range(0, w.H, 16):
        O_ref = oracle.attend(Qh[:, h0:h0 + 16], Ks_h[h0:h0 + 16], Vs_h[h0:h0 + 16])
        worst_att = max(worst_att, attn_rel_err(O_h[:, h0:h0 + 16], O_ref))
    say(f"attention, all {w.H} heads: max rel err {worst_att:.2e}")
    assert worst_att <= 2e-3

    # ---- oracle on sampled rows: density of 8 rows in every head, 16 in 55 of them (two per layer and the corners)
    rng = np.random.default_rng(2026)
    worst = 0.0
    row_heads = sorted({0, 1, 95, 191, 192, 300, 382, 383} | {16 * l + (7 * l + 2) % 16 for l in range(24)}
                       | {16 * l + (3 * l + 11) % 16 for l in range(24)})
    rho_h = rho.cpu().numpy()
    for h in range(w.H):
        Kh = K[h].float().cpu().numpy()
        if h in row_heads:
            assert np.array_equal(Kh, syn.cloud(w, h, syn.TENSOR_K))          # same bits as the generator's
        nrows = 15 if h in row_heads else 7
        rows = np.concatenate([rng.integers(0, w.L, nrows), idx[h, :1].cpu().numpy()]).astype(np.int32)
        ref = oracle.density_rows(Kh, float(sigma[h]), rows)
        worst = max(worst, float(np.abs(rho_h[h][rows] / ref - 1).max()))
    say(f"density, sampled rows of all {w.H} heads (16 in {len(row_heads)} of them, 8 in the others): max rel err {worst:.2e}")
    assert worst <= 5e-5

    # ---- oracle on sampled heads: full chain (first and last head, first and last head of a layer, and four heads of
    # every one of the 24 layers: about a hundred of the 384, two seconds of float64 density each)
    forks_total, ties_total = 0, 0
    chain_heads = sorted({0, 383, 137, 15, 16, 200, 287, 368}
                         | {16 * l + (5 * l + 3 + 4 * j) % 16 for l in range(24) for j in range(4)})
    for h in chain_heads:
        Kh = K[h].float().cpu().numpy()
        Vh = V[h].float().cpu().numpy()
        rho_ref = oracle.density(Kh, float(sigma[h]))
        err = float(np.abs(rho[h].cpu().numpy() / rho_ref - 1).max())
        ref, _, gap = oracle.select(Kh, rho_ref, w.k, w.alpha)
        forks = check_indices(oracle, Kh, rho_ref, w.k, w.alpha, idx[h].cpu().numpy(), ref)
        ks, vs = oracle.gather(Kh, Vh, idx[h].cpu().numpy())
        assert np.array_equal(Ks[h].float().cpu().numpy(), ks) and np.array_equal(Vs[h].float().cpu().numpy(), vs)
        O_ref = oracle.attend(Qh[:, h:h + 1], ks[None], vs[None])
        aerr = attn_rel_err(O[:, h:h + 1].cpu().numpy(), O_ref)
        say(f"head {h}: density rel err {err:.2e}; oracle steps under tie tolerance {(gap < TIE_TOL).sum()}, "
              f"forks {forks}; attention rel err {aerr:.2e}")
        assert err <= 5e-5 and aerr <= 2e-3
        forks_total += forks
        ties_total += int((gap < TIE_TOL).sum())
    say(f"headline, {len(chain_heads)} heads through the whole chain: {ties_total} near-tie steps survived, "
          f"{forks_total} near-tie forks")

    # ---- every other head: the selection as a stage on identical inputs.  The oracle is fed the library's own density
    # (fp32, widened exactly), so all 655 picks of each head are compared with the oracle's under the same near-tie
    # protocol; the density those picks rest on was checked above on sampled rows of the same heads.
    idx_h = idx.cpu().numpy()
    rest = [h for h in range(w.H) if h not in set(chain_heads)]
    forks_rest, ties_rest, exact_rest = 0, 0, 0
    for i, h in enumerate(rest):
        Kh = K[h].float().cpu().numpy()
        rho64 = rho_h[h].astype(np.float64)
        ref, _, gap = oracle.select(Kh, rho64, w.k, w.alpha)
        forks = check_indices(oracle, Kh, rho64, w.k, w.alpha, idx_h[h], ref)
        forks_rest += forks
        exact_rest += int(forks == 0)
        ties_rest += int((gap < TIE_TOL).sum())
        if (i + 1) % 64 == 0:
            say(f"  selection on the library's density: {i + 1} of {len(rest)} heads compared")
    say(f"headline, selection of the other {len(rest)} heads on the library's density: {exact_rest} heads bit-equal, "
        f"{ties_rest} near-tie steps survived, {forks_rest} near-tie forks")

    # ---- the steps next to the hot path at the same full size
    # attention mass: all 24 layers in one call; oracle on 3 whole layers, sum rule on all
    G, Hl = w.layers, w.H // w.layers
    Qm_h = syn.main_query(w)
    Qm = torch.from_numpy(Qm_h).to(torch.bfloat16).cuda()
    A = ws.ws_synapse_attention_mass(K, Qm, G, as_density=False)
    tot = A.view(G, Hl, w.L)[:, 0].double().sum(dim=1).cpu().numpy()
    assert np.abs(tot - Hl).max() < 1e-3 * Hl, "attention mass of a layer must sum to its number of query heads"
    worst = 0.0
    for grp in [0, 11, 23]:
        Kg = K[grp * Hl:(grp + 1) * Hl].float().cpu().numpy()
        ref = oracle.attention_mass(Kg, Qm_h[grp * Hl:(grp + 1) * Hl])
        got = A[grp * Hl].double().cpu().numpy()
        big = ref > 1e-12 * ref.max()
        worst = max(worst, float(np.abs(got[big] / ref[big] - 1).max()))
    say(f"attention mass, 3 of {G} layers: max rel err {worst:.2e}")
    assert worst <= 1e-4

    # density refresh: the last 3 rows of every head treated as just appended; oracle on sampled rows
    m = 3
    sig = [float(s) for s in sigma]
    rho_old = ws.ws_synapse_density(K[:, :w.L - m].contiguous(), sig)
    rho_new = ws.ws_synapse_density_append(K, m, sig, rho_old)
    diff = float((rho_new / rho - 1).abs().max())
    say(f"density refresh (m={m}) vs full density on all {w.H} heads: max rel diff {diff:.2e}")
    assert diff <= 1e-4                                   # two GPU paths, each within 5e-5 of the oracle
    worst = 0.0
    for h in [0, 200, 383]:
        Kh = K[h].float().cpu().numpy()
        rows = np.concatenate([rng.integers(0, w.L - m, 13), np.arange(w.L - m, w.L)]).astype(np.int32)
        ref = oracle.density_rows(Kh, sig[h], rows)
        worst = max(worst, float(np.abs(rho_new[h].cpu().numpy()[rows] / ref - 1).max()))
    say(f"density refresh, 3 heads x 16 rows (new rows included): max rel err {worst:.2e}")
    assert worst <= 5e-5
