"""CPU pins of the oracle (oracle/ws_oracle.c) against things other than itself:
closed forms, library routines, brute force on tiny inputs and invariants.  Each
pin is chosen so that a plausible slip in the oracle (dropped term, wrong sign,
wrong index, transposed operand, wrong normalisation) fails at least one."""
import itertools
import math
import os

import numpy as np
import pytest
from scipy.spatial.distance import cdist
from scipy.special import logsumexp

from paper_2601_01298_amd import synthetic as syn

GOLD = os.path.join(os.path.dirname(__file__), "golden", "closed_forms.txt")


def golden(name):
    for line in open(GOLD):
        if line.startswith("#") or "|" not in line:
            continue
        key, vals, _ = [p.strip() for p in line.split("|", 2)]
        if key == name:
            return np.array([float(v) for v in vals.split()])
    raise KeyError(name)


def small_cloud(L, d, seed, ncomp=3):
    rng = np.random.default_rng(seed)
    c = 2.0 * rng.standard_normal((ncomp, d))
    return c[rng.integers(0, ncomp, L)] + 0.5 * rng.standard_normal((L, d))


# ------------------------------------------------------------------ density
def test_density_two_point_closed_form(oracle):
    K = np.array([[0.0, 0.0], [3.0, 4.0]])
    rho = oracle.density(K, math.sqrt(12.5))
    assert np.allclose(rho, golden("density_two_points")[0], rtol=0, atol=1e-15)
    r2, s2 = 7.3, 1.9          # generic radius and bandwidth
    K = np.array([[1.0, -2.0, 0.5], [1.0 + math.sqrt(r2), -2.0, 0.5]])
    assert np.allclose(oracle.density(K, math.sqrt(s2)), (1 + math.exp(-r2 / (2 * s2))) / 2, rtol=1e-14)


def test_density_three_collinear(oracle):
    K = np.array([[0.0], [1.0], [3.0]])
    assert np.allclose(oracle.density(K, math.sqrt(0.5)), golden("density_three_collinear"), rtol=1e-12)


def test_density_limits(oracle):
    K = np.tile(np.array([[0.3, -1.2, 4.0]]), (7, 1))
    assert np.array_equal(oracle.density(K, 0.7), np.ones(7))
    K = small_cloud(40, 5, 1)
    assert np.allclose(oracle.density(K, 1e6), 1.0, rtol=1e-9)
    # sigma -> 0: only exact duplicates contribute -> multiplicity / L
    K = np.array([[0.0, 0.0], [5.0, 5.0], [0.0, 0.0], [9.0, -3.0], [0.0, 0.0]])
    assert np.allclose(oracle.density(K, 1e-3), np.array([3, 1, 3, 1, 3]) / 5.0, rtol=0, atol=1e-300)


def test_density_matches_logsumexp(oracle):
    for L, d, seed, sig in [(64, 8, 2, 1.3), (200, 64, 3, 4.0), (33, 1, 4, 0.2)]:
        K = small_cloud(L, d, seed)
        ref = np.exp(logsumexp(-cdist(K, K, "sqeuclidean") / (2 * sig * sig), axis=1) - math.log(L))
        got = oracle.density(K, sig)
        assert np.allclose(got, ref, rtol=1e-12)
        assert np.all(got >= 1.0 / L - 1e-15) and np.all(got <= 1.0 + 1e-15)


def test_density_invariances(oracle):
    K = small_cloud(50, 6, 5)
    sig = 1.1
    base = oracle.density(K, sig)
    assert np.allclose(oracle.density(K + 17.5, sig), base, rtol=1e-10)
    Qm, _ = np.linalg.qr(np.random.default_rng(6).standard_normal((6, 6)))
    assert np.allclose(oracle.density(K @ Qm, sig), base, rtol=1e-10)
    perm = np.random.default_rng(7).permutation(50)
    assert np.allclose(oracle.density(K[perm], sig), base[perm], rtol=1e-12)
    # scaling points and bandwidth together changes nothing
    assert np.allclose(oracle.density(3.0 * K, 3.0 * sig), base, rtol=1e-12)


def test_density_rows_equals_full(oracle):
    K = small_cloud(120, 16, 8)
    rows = [0, 5, 119, 64]
    assert np.array_equal(oracle.density_rows(K, 0.9, rows), oracle.density(K, 0.9)[rows])


def test_inverse_density(oracle):
    rho = np.array([0.5, 0.25, 0.75, 0.25, 1.0])
    u = oracle.inverse_density(rho)
    assert np.array_equal(u, np.array([0.5, 1.0, 1.0 / 3.0, 1.0, 0.25]))
    K = small_cloud(80, 4, 9)
    rho = oracle.density(K, 0.8)
    u = oracle.inverse_density(rho)
    assert u.max() == 1.0 and u[np.argmin(rho)] == 1.0 and np.all(u > 0)


# ---------------------------------------------------------------- selection
def scores_from_definition(K, u, chosen, alpha):
    """Score of every point from the definition: D_i is the minimum over ALL
    chosen landmarks of the Euclidean distance (no running array)."""
    L = K.shape[0]
    free = [i for i in range(L) if i not in chosen]
    if not chosen:
        c = np.ones(L)
    else:
        D = np.array([min(math.sqrt(((K[i] - K[s]) ** 2).sum()) for s in chosen) for i in range(L)])
        dmax = max(D[i] for i in free)
        c = D / dmax if dmax > 0 else np.zeros(L)
    return alpha * c + (1 - alpha) * u, free


@pytest.mark.parametrize("alpha", [0.0, 0.25, 0.5, 1.0])
@pytest.mark.parametrize("L,d,k,seed", [(24, 3, 24, 11), (64, 8, 20, 12), (40, 2, 13, 13)])
def test_select_each_pick_maximises_score(oracle, alpha, L, d, k, seed):
    K = small_cloud(L, d, seed)
    rho = oracle.density(K, 0.9)
    u = rho.min() / rho
    idx, score, gap = oracle.select(K, rho, k, alpha)
    assert len(set(idx.tolist())) == k
    chosen = []
    for t in range(k):
        if t == 0 and alpha == 1.0:
            assert idx[0] == 0
        else:
            sc, free = scores_from_definition(K, u, chosen, alpha)
            best = max(sc[i] for i in free)
            winners = [i for i in free if sc[i] == best]
            assert idx[t] == winners[0], (t, idx[t], winners)
            assert score[t] == pytest.approx(best, rel=1e-13)
            rest = sorted((sc[i] for i in free if i != idx[t]), reverse=True)
            if rest:
                assert gap[t] == pytest.approx((best - rest[0]) / abs(best), rel=1e-9, abs=1e-15)
            else:
                assert gap[t] == np.inf
        chosen.append(int(idx[t]))
    if k == L:
        assert sorted(idx.tolist()) == list(range(L))


def gonzalez(K, k):
    D = np.full(K.shape[0], np.inf)
    order, radii, s = [], [], 0
    for _ in range(k):
        order.append(s)
        D = np.minimum(D, np.sqrt(((K - K[s]) ** 2).sum(1)))
        D[order] = -1.0
        s = int(np.argmax(D))          # numpy argmax returns the first maximum
        radii.append(D[s])
    return order, radii


def test_select_alpha1_is_farthest_point_traversal(oracle):
    for L, d, k, seed in [(200, 16, 40, 21), (64, 2, 64, 22)]:
        K = small_cloud(L, d, seed)
        rho = oracle.density(K, 1.0)
        idx, _, _ = oracle.select(K, rho, k, 1.0)
        order, radii = gonzalez(K, k)
        assert idx.tolist() == order
        r = np.array(radii[:-1])
        assert np.all(np.diff(r) <= 1e-12)         # covering radius never grows


def test_select_alpha1_two_approximation(oracle):
    K = small_cloud(12, 2, 23, ncomp=4)
    rho = oracle.density(K, 1.0)
    full = cdist(K, K)
    for k in (2, 3, 4):
        idx, _, _ = oracle.select(K, rho, k, 1.0)
        greedy_r = full[:, idx].min(1).max()
        opt = min(full[:, list(c)].min(1).max() for c in itertools.combinations(range(12), k))
        assert greedy_r <= 2.0 * opt + 1e-12


def test_select_alpha0_is_sorted_density(oracle):
    K = small_cloud(150, 5, 24)
    rho = oracle.density(K, 0.7)
    rho[17] = rho[90]                      # plant an exact tie: lower index first
    idx, _, _ = oracle.select(K, rho, 30, 0.0)
    assert idx.tolist() == np.argsort(rho, kind="stable")[:30].tolist()


def test_select_exact_tie_example(oracle):
    K = np.array([[0.0], [3.0], [7.0], [10.0], [5.0]])
    idx, _, gap = oracle.select(K, np.ones(5), 5, 1.0)
    assert idx.tolist() == golden("fps_exact_tie").astype(int).tolist()
    assert gap[3] == 0.0


def test_select_hybrid_hand_example(oracle):
    K = np.array([[0.0], [1.0], [3.0]])
    rho = oracle.density(K, math.sqrt(0.5))
    assert np.allclose(oracle.inverse_density(rho), golden("hybrid_u"), rtol=1e-12)
    idx, score, _ = oracle.select(K, rho, 3, 0.5)
    assert idx.tolist() == golden("hybrid_picks").astype(int).tolist()
    assert score[1] == pytest.approx(0.8722357186487468, rel=1e-12)


def test_select_duplicates_zero_radius(oracle):
    # all remaining points coincide with landmarks -> coverage term 0, pick by u then index
    K = np.array([[0.0, 0.0]] * 3 + [[1.0, 1.0]] * 3)
    rho = np.array([0.5, 0.4, 0.6, 0.3, 0.35, 0.3])
    idx, _, _ = oracle.select(K, rho, 6, 0.5)
    assert sorted(idx.tolist()) == list(range(6))
    assert idx[0] == 3                     # lowest density, lowest index among ties
    # after {3, one of 0..2} are chosen every D is 0: the rest follow u, lowest index first
    assert idx.tolist()[2:] == sorted(set(range(6)) - set(idx[:2].tolist()),
                                      key=lambda i: (-rho.min() / rho[i], i))


def test_select_verify_mode(oracle):
    K = small_cloud(300, 8, 25)
    rho = oracle.density(K, 0.8)
    idx, _, _ = oracle.select(K, rho, 25, 0.5)
    forks, pick, deficit = oracle.select_verify(K, rho, 25, 0.5, idx)
    assert forks == 0 and pick.tolist() == idx.tolist() and not deficit.any()
    bad = idx.copy()
    others = [i for i in range(300) if i not in set(idx.tolist())]
    bad[10] = others[0]
    forks, pick, deficit = oracle.select_verify(K, rho, 25, 0.5, bad)
    assert forks >= 1 and pick[10] == idx[10] and deficit[10] > 0
    assert pick[:10].tolist() == idx[:10].tolist()
    rep = idx.copy()
    rep[5] = rep[2]
    assert oracle.select_verify(K, rho, 25, 0.5, rep)[0] == -2


def verify_from_definition(K, u, alpha, cand):
    """What verify mode must report, from the definition alone: at step t the landmarks are the
    CANDIDATE's first t entries; the pick is the lowest index among the exact maxima of the score,
    the deficit (best - score[cand[t]]) / |best| (0 where the candidate is that pick)."""
    picks, deficits, chosen = [], [], []
    for t, c in enumerate(cand):
        if t == 0 and alpha == 1.0:
            best_i, best, sc_c = 0, alpha, alpha
        else:
            sc, free = scores_from_definition(K, u, chosen, alpha)
            best = max(sc[i] for i in free)
            best_i = [i for i in free if sc[i] == best][0]
            sc_c = sc[c]
        picks.append(best_i)
        deficits.append(0.0 if best_i == c else (best - sc_c) / abs(best))
        chosen.append(int(c))
    return picks, deficits


def verify_cases(select, alpha):
    """A small cloud and candidate chains that leave the greedy chain in different ways: the step's
    runner-up, a mid-ranked point, another first landmark, the last step, and two forks in one
    chain.  `select(K, rho, k, alpha)` returns the greedy chain the candidates start from."""
    L, k = 60, 14
    K = small_cloud(L, 4, 26)
    rho = np.exp(logsumexp(-cdist(K, K, "sqeuclidean") / (2 * 0.9 * 0.9), axis=1)) / L
    u = rho.min() / rho
    idx = select(K, rho, k, alpha)

    def ranked(chosen):                       # free points, best score first (lowest index on ties)
        sc, free = scores_from_definition(K, u, chosen, alpha)
        return sorted(free, key=lambda i: (-sc[i], i))

    cands = []
    for t_fork, rank in [(3, 1), (7, len(idx)), (0, 1), (0, 5), (k - 1, 1)]:
        cand = idx.tolist()[:t_fork]
        order = ranked(cand) if not (t_fork == 0 and alpha == 1.0) else list(range(L))
        cand.append(order[min(rank, len(order) - 1)])
        while len(cand) < k:                  # continue greedily along the candidate's own prefix
            cand.append(ranked(cand)[0])
        cands.append(cand)
    cand = cands[0][:9]                       # a second fork, mid-ranked ...
    cand.append(ranked(cand)[20])
    while len(cand) < k:
        cand.append(ranked(cand)[1])          # ... and the runner-up at every later step
    cands.append(cand)
    return K, rho, u, k, cands


def verify_mismatches(verify, K, rho, u, k, alpha, cands):
    """Number of candidates on which `verify` (returning forks, picks, deficits) departs from the
    definition in any pick, any deficit (1e-12) or the fork count."""
    wrong = 0
    for cand in cands:
        want_pick, want_def = verify_from_definition(K, u, alpha, cand)
        forks, pick, deficit = verify(K, rho, k, alpha, np.array(cand, dtype=np.int32))
        ok = (list(pick) == want_pick and np.allclose(deficit, want_def, rtol=1e-12, atol=1e-15)
              and forks == sum(1 for a, b in zip(cand, want_pick) if a != b))
        wrong += not ok
    return wrong


@pytest.mark.parametrize("alpha", [0.0, 0.25, 0.5, 1.0])
def test_select_verify_values_along_candidate_prefix(oracle, alpha):
    """Pick and deficit of every step, also after a fork, against the definition."""
    K, rho, u, k, cands = verify_cases(lambda *a: oracle.select(*a)[0], alpha)
    assert verify_mismatches(oracle.select_verify, K, rho, u, k, alpha, cands) == 0
    for n, cand in enumerate(cands):
        want_pick, want_def = verify_from_definition(K, u, alpha, cand)
        assert want_pick != cand
        if not (alpha == 1.0 and n in (2, 3)):     # (a first landmark other than 0 at alpha = 1 costs nothing)
            assert max(want_def) > 1e-3       # the planted forks are real deficits, not rounding


MUTANTS = [   # (text in ws_oracle.c, replacement): slips a verify mode could plausibly contain
    ("(t1 - sc) / fabs(t1)", "(t1 - t2) / fabs(t1)"),            # deficit against the runner-up
    ("(t1 - sc) / fabs(t1)", "(t1 - sc) / fabs(sc)"),            # another denominator
    ("absorb_landmark(K, L, d, c, D, chosen);", "absorb_landmark(K, L, d, s, D, chosen);"),  # oracle's prefix
    ("if (i == probe) *probe_score = s;", "if (i == probe) *probe_score = c;"),   # coverage term for the score
]


@pytest.mark.parametrize("mutant", range(len(MUTANTS)))
def test_select_verify_pins_catch_planted_mistakes(oracle, tmp_path, mutant):
    """The value pins above must fail on a verify mode with a planted slip.  The slip is planted in
    a private copy of the oracle's source, compiled here on the CPU."""
    import ctypes
    import subprocess
    old, new = MUTANTS[mutant]
    src = open(os.path.join(os.path.dirname(oracle.__file__), "ws_oracle.c")).read()
    assert src.count(old) == 1
    cfile, so = tmp_path / "mutant.c", tmp_path / "libmutant.so"
    cfile.write_text(src.replace(old, new))
    subprocess.run(["gcc", "-O1", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC", "-o", str(so), str(cfile), "-lm"],
                   check=True)
    lib = ctypes.CDLL(str(so))
    dp, ip = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)
    lib.wso_select_verify.argtypes = [dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double, ip, ip, dp]
    lib.wso_select_verify.restype = ctypes.c_int

    def verify(K, rho, k, alpha, cand):
        K = np.ascontiguousarray(K, dtype=np.float64)
        rho = np.ascontiguousarray(rho, dtype=np.float64)
        pick, deficit = np.zeros(k, dtype=np.int32), np.zeros(k)
        forks = lib.wso_select_verify(K.ctypes.data_as(dp), rho.ctypes.data_as(dp), K.shape[0], K.shape[1], k, alpha,
                                      cand.ctypes.data_as(ip), pick.ctypes.data_as(ip), deficit.ctypes.data_as(dp))
        return forks, pick.tolist(), deficit

    wrong = 0
    for alpha in (0.25, 0.5):
        K, rho, u, k, cands = verify_cases(lambda *a: oracle.select(*a)[0], alpha)
        wrong += verify_mismatches(verify, K, rho, u, k, alpha, cands)
    assert wrong > 0, f"mutant {old!r} -> {new!r} passes the verify pins"


def test_select_verify_exact_tie_and_zero_radius(oracle):
    # exact tie (integer coordinates, alpha = 1): 4th pick ties between indices 1 and 2; taking the
    # higher index is a fork with deficit exactly 0, and the steps after it still follow its prefix
    K = np.array([[0.0], [3.0], [7.0], [10.0], [5.0]])
    rho = np.ones(5)
    forks, pick, deficit = oracle.select_verify(K, rho, 5, 1.0, np.array([0, 3, 4, 2, 1], dtype=np.int32))
    assert forks == 1 and pick.tolist() == [0, 3, 4, 1, 1] and deficit.tolist() == [0.0] * 5
    # a wrong first landmark at alpha = 1 (every score equals alpha there): deficit 0, pick 0
    forks, pick, deficit = oracle.select_verify(K, rho, 3, 1.0, np.array([2, 0, 3], dtype=np.int32))
    want_pick, want_def = verify_from_definition(K, rho.min() / rho, 1.0, [2, 0, 3])
    assert pick.tolist() == want_pick and np.allclose(deficit, want_def, atol=1e-15) and forks == 2
    # density only (alpha = 0): best score 1 at the minimum-density point; candidate with u = 0.5
    K = np.array([[0.0], [1.0], [2.0], [3.0]])
    rho = np.array([0.2, 0.1, 0.4, 0.1])
    forks, pick, deficit = oracle.select_verify(K, rho, 3, 0.0, np.array([0, 3, 1], dtype=np.int32))
    assert forks == 2 and pick.tolist() == [1, 1, 1] and np.allclose(deficit, [0.5, 0.0, 0.0], atol=1e-15)


# ------------------------------------------------------------------- gather
def test_gather_is_bit_copy(oracle):
    rng = np.random.default_rng(31)
    K = rng.integers(0, 2 ** 16, size=(100, 64), dtype=np.uint16)
    V = rng.integers(0, 2 ** 16, size=(100, 64), dtype=np.uint16)
    idx = rng.permutation(100)[:17].astype(np.int32)
    Ks, Vs = oracle.gather(K, V, idx)
    assert np.array_equal(Ks, K[idx]) and np.array_equal(Vs, V[idx])


# ---------------------------------------------------------------- attention
def dense_attention(Q, K, V, g):
    N, Hq, d = Q.shape
    O = np.empty_like(Q)
    for n in range(N):
        for q in range(Hq):
            z = K[q // g] @ Q[n, q] / math.sqrt(d)
            p = np.exp(z - z.max())
            O[n, q] = (p / p.sum()) @ V[q // g]
    return O


def test_attend_full_selection_equals_dense_attention(oracle):
    rng = np.random.default_rng(41)
    H, L, d, N = 2, 48, 8, 3
    K = np.stack([small_cloud(L, d, 42 + h) for h in range(H)])
    V = rng.standard_normal((H, L, d))
    Q = rng.standard_normal((N, 2 * H, d))
    Ks, Vs = np.empty_like(K), np.empty_like(V)
    for h in range(H):
        rho = oracle.density(K[h], 1.0)
        idx, _, _ = oracle.select(K[h], rho, L, 0.5)          # k = L: a permutation
        Ks[h], Vs[h] = oracle.gather(K[h], V[h], idx)
    got = oracle.attend(Q, Ks, Vs)
    assert np.allclose(got, dense_attention(Q, K, V, g=2), rtol=1e-12, atol=1e-14)


def test_attend_special_cases(oracle):
    rng = np.random.default_rng(43)
    Ks = rng.standard_normal((3, 9, 16))
    Vs = rng.standard_normal((3, 9, 16))
    Q = rng.standard_normal((5, 3, 16))
    assert np.allclose(oracle.attend(Q, Ks[:, :1], Vs[:, :1]), np.broadcast_to(Vs[:, 0], (5, 3, 16)))
    assert np.allclose(oracle.attend(np.zeros_like(Q), Ks, Vs), np.broadcast_to(Vs.mean(1), (5, 3, 16)))
    O = oracle.attend(Q, Ks, Vs)
    assert np.all(O <= Vs.max(1)[None] + 1e-12) and np.all(O >= Vs.min(1)[None] - 1e-12)
    # a constant added to every logit changes nothing: extra key coordinate 5, query coordinate 1
    Ks2 = np.concatenate([Ks, np.full((3, 9, 1), 5.0)], axis=2)
    Q2 = np.concatenate([Q, np.ones((5, 3, 1))], axis=2)
    Vs2 = np.concatenate([Vs, np.zeros((3, 9, 1))], axis=2)
    O2 = oracle.attend(Q2, Ks2, Vs2, scale=1.0 / math.sqrt(16))
    assert np.allclose(O2[..., :16], O, rtol=1e-12, atol=1e-14)
    # permuting landmark rows changes nothing
    perm = rng.permutation(9)
    assert np.allclose(oracle.attend(Q, Ks[:, perm], Vs[:, perm]), O, rtol=1e-12, atol=1e-14)


def test_attend_matches_library_sdpa(oracle):
    import torch
    rng = np.random.default_rng(44)
    Hkv, g, k, d, N = 2, 4, 37, 32, 6
    Ks = rng.standard_normal((Hkv, k, d))
    Vs = rng.standard_normal((Hkv, k, d))
    Q = rng.standard_normal((N, Hkv * g, d))
    q = torch.from_numpy(Q).permute(1, 0, 2)                       # [Hq,N,d]
    kk = torch.from_numpy(Ks).repeat_interleave(g, dim=0)          # [Hq,k,d]
    vv = torch.from_numpy(Vs).repeat_interleave(g, dim=0)
    ref = torch.nn.functional.scaled_dot_product_attention(q, kk, vv).permute(1, 0, 2).numpy()
    assert np.allclose(oracle.attend(Q, Ks, Vs), ref, rtol=1e-12, atol=1e-14)


# -------------------------------------------------------- input generators
def test_generators_are_seeded_and_on_grid():
    w = syn.small_variant(syn.WORKLOADS[2], L=256)
    a = syn.cloud(w, 3, syn.TENSOR_K)
    b = syn.cloud(w, 3, syn.TENSOR_K)
    assert np.array_equal(a, b) and a.dtype == np.float32 and a.shape == (256, 64)
    assert not np.array_equal(a, syn.cloud(w, 4, syn.TENSOR_K))
    assert not np.array_equal(a, syn.cloud(w, 3, syn.TENSOR_V))
    assert not np.array_equal(a, syn.cloud(w, 3, syn.TENSOR_K, seed=syn.BASE_SEED + 1))
    assert np.array_equal(syn.round_to_bf16(a), a)                 # already bf16 values
    assert np.all((a.view(np.uint32) & 0xFFFF) == 0)
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -9], dtype=np.float32)
    assert syn.round_to_bf16(x).tolist() == [1.0, 1.0 + 2.0 ** -6, 1.0]   # ties to even
    for cfg in (1, 4, 5):
        w = syn.small_variant(syn.WORKLOADS[cfg], L=128)
        assert syn.cloud(w, 0, syn.TENSOR_K).shape == (128, w.d)
    assert syn.queries(syn.WORKLOADS[1]).shape == (4, 1, 64)
    K = syn.cloud(syn.WORKLOADS[1], 0, syn.TENSOR_K)
    s = syn.bandwidth(K)
    assert s.dtype == np.float32 and abs(float(s) ** 2 - K.astype(np.float64).var(0).sum() / 16) < 1e-5
