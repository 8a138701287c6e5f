"""CPU pins of the oracle functions for the steps next to the hot path (attention-mass density
proxy, validation gate, RoPE rotation of injected rows) against closed forms, library routines and
invariants -- never against the oracle's own formula retyped."""
import math
import os

import numpy as np
import pytest
from scipy.special import softmax


GOLD = os.path.join(os.path.dirname(__file__), "golden", "closed_forms.txt")


def golden(name):
    for line in open(GOLD):
        if line.startswith("#") or "|" not in line:
            continue
        key, vals, _ = [p.strip() for p in line.split("|", 2)]
        if key == name:
            return np.array([float(v) for v in vals.split()])
    raise KeyError(name)


def rng_arr(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


# ------------------------------------------------------------------ attention mass
def test_mass_two_token_closed_form(oracle):
    # one head, d = 1: logits (0, ln 3) -> softmax (1/4, 3/4)
    A = oracle.attention_mass(np.array([[[0.0], [1.0]]]), np.array([[math.log(3.0)]]), scale=1.0)
    assert np.allclose(A, golden("mass_two_tokens"), rtol=1e-15)
    # default scale is 1/sqrt(d): d = 4, q.k = 2 ln 3 -> same logits after scaling
    K = np.zeros((1, 2, 4))
    K[0, 1, :] = 1.0
    q = np.full((1, 4), 0.5 * math.log(3.0))
    assert np.allclose(oracle.attention_mass(K, q), [0.25, 0.75], rtol=1e-14)


def test_mass_sums_and_uniform_query(oracle):
    K = rng_arr(1, 3, 50, 8)
    Q = rng_arr(2, 6, 8)
    A = oracle.attention_mass(K, Q)
    assert abs(A.sum() - 6.0) < 1e-12 and (A > 0).all()
    assert np.allclose(oracle.attention_mass(K, np.zeros((6, 8))), 6.0 / 50.0, rtol=1e-14)


def test_mass_matches_library_softmax_with_grouped_heads(oracle):
    Hkv, g, L, d = 3, 2, 37, 16
    K = rng_arr(3, Hkv, L, d)
    Q = 2.0 * rng_arr(4, Hkv * g, d)
    ref = np.zeros(L)
    for q in range(Hkv * g):
        ref += softmax(K[q // g] @ Q[q] / math.sqrt(d))
    assert np.allclose(oracle.attention_mass(K, Q), ref, rtol=1e-12)
    # the same through explicitly repeated KV heads (pins the contiguous-group mapping)
    assert np.allclose(oracle.attention_mass(np.repeat(K, g, axis=0), Q), ref, rtol=1e-12)
    # an interleaved mapping (q mod Hkv) gives something else on these inputs
    wrong = sum(softmax(K[q % Hkv] @ Q[q] / math.sqrt(d)) for q in range(Hkv * g))
    assert not np.allclose(wrong, ref, rtol=1e-3)


def test_mass_invariances(oracle):
    K = rng_arr(5, 2, 64, 8)
    Q = rng_arr(6, 2, 8)
    A = oracle.attention_mass(K, Q)
    # a common shift of every key moves each head's logits by a constant
    assert np.allclose(oracle.attention_mass(K + rng_arr(7, 1, 1, 8), Q), A, rtol=1e-10)
    # permuting tokens permutes A
    p = np.random.default_rng(8).permutation(64)
    assert np.allclose(oracle.attention_mass(K[:, p], Q), A[p], rtol=1e-12)
    # huge logits do not overflow
    big = oracle.attention_mass(1e3 * K, 1e3 * Q)
    assert np.isfinite(big).all() and abs(big.sum() - 2.0) < 1e-9


def test_mass_as_inverse_density(oracle):
    A = np.array([0.5, 2.0, 0.25, 0.0, 1.0])
    rho = oracle.mass_to_density(A)
    assert np.array_equal(rho[[0, 1, 2, 4]], 1.0 / A[[0, 1, 2, 4]]) and math.isclose(rho[3], 1e30, rel_tol=1e-15)
    u = oracle.inverse_density(rho)
    assert np.allclose(u[[0, 1, 2, 4]], A[[0, 1, 2, 4]] / 2.0, rtol=1e-15) and u[3] < 1e-29
    # density-only selection (alpha = 0) then takes tokens by descending attention mass
    K = rng_arr(9, 5, 3)
    idx, _, _ = oracle.select(K, rho, 4, 0.0)
    assert list(idx) == [1, 4, 0, 2]


# ------------------------------------------------------------------ validation gate
def test_gate_hand_values(oracle):
    h = np.array([1.0, 0.0])
    T = np.array([[3.0, 4.0], [1.0, 2.0], [-2.0, 0.0], [0.0, 5.0], [0.0, 0.0], [7.0, 0.0]])
    score, acc = oracle.gate(h, T, 0.5)
    assert np.allclose(score, golden("gate_cosines"), rtol=1e-15, atol=1e-300)
    assert list(acc) == [1, 0, 0, 0, 0, 1]
    # the threshold itself passes (only score < theta is rejected)
    _, acc = oracle.gate(h, T[:1], 0.6)
    assert acc[0] == 1
    _, acc = oracle.gate(h, T[:1], np.nextafter(0.6, 1.0))
    assert acc[0] == 0


def test_gate_matches_library_and_scale_invariance(oracle):
    from sklearn.metrics.pairwise import cosine_similarity
    h = rng_arr(10, 896)
    T = rng_arr(11, 40, 896) + 0.4 * h
    score, acc = oracle.gate(h, T, 0.3)
    ref = cosine_similarity(T, h[None])[:, 0]
    assert np.allclose(score, ref, rtol=1e-12)
    assert np.array_equal(acc, (ref >= 0.3).astype(np.int32))
    s2, _ = oracle.gate(7.5 * h, 0.01 * T, 0.3)
    assert np.allclose(s2, score, rtol=1e-12)
    assert (np.abs(score) <= 1 + 1e-15).all()


# ------------------------------------------------------------------ RoPE of injected rows
def test_rope_hand_values(oracle):
    # d = 2: one pair, frequency base^0 = 1 -> rotation by p radians
    y = oracle.rope(np.array([[1.0, 0.0], [0.0, 1.0]]), [1, 2], base=10000.0)
    assert np.allclose(y, [[math.cos(1), math.sin(1)], [-math.sin(2), math.cos(2)]], rtol=1e-15)
    # d = 4, base = 100: pair (1, 3) turns at 100^(-2/4) = 0.1 rad per position; pair (0, 2) at 1
    x = np.array([[0.0, 1.0, 0.0, 0.0]])
    y = oracle.rope(x, [7], base=100.0)
    assert np.allclose(y, [[0.0, math.cos(0.7), 0.0, math.sin(0.7)]], rtol=1e-14, atol=1e-300)
    assert np.allclose(y[0], golden("rope_d4_base100"), rtol=1e-14, atol=1e-300)
    x = np.array([[2.0, 0.0, 0.0, 0.0]])
    y = oracle.rope(x, [3], base=100.0)
    assert np.allclose(y, [[2 * math.cos(3), 0.0, 2 * math.sin(3), 0.0]], rtol=1e-14, atol=1e-300)


def test_rope_matches_complex_rotation(oracle):
    m, d, base = 9, 64, 1.0e6
    X = rng_arr(12, m, d)
    pos = np.array([0, 1, 5, 100, 4095, 32768, 131071, 1000000, 77], dtype=np.int32)
    freq = base ** (-np.arange(d // 2) / (d / 2))
    zc = (X[:, :d // 2] + 1j * X[:, d // 2:]) * np.exp(1j * pos[:, None] * freq[None, :])
    ref = np.concatenate([zc.real, zc.imag], axis=1)
    assert np.allclose(oracle.rope(X, pos, base), ref, rtol=1e-9, atol=1e-9)
    assert np.array_equal(oracle.rope(X[:1], [0], base), X[:1])       # position 0 is the identity


def test_rope_group_properties(oracle):
    d, base = 32, 10000.0
    q = rng_arr(13, 1, d)
    k = rng_arr(14, 1, d)
    # rotations compose additively and preserve the norm of every pair
    a = oracle.rope(oracle.rope(q, [11], base), [30], base)
    assert np.allclose(a, oracle.rope(q, [41], base), rtol=1e-12, atol=1e-12)
    y = oracle.rope(q, [123], base)
    assert np.allclose(y[:, :d // 2] ** 2 + y[:, d // 2:] ** 2, q[:, :d // 2] ** 2 + q[:, d // 2:] ** 2, rtol=1e-12)
    # the score of a rotated query against a rotated key depends on the position difference only
    s1 = (oracle.rope(q, [500], base) @ oracle.rope(k, [460], base).T).item()
    s2 = (oracle.rope(q, [40], base) @ k.T).item()
    assert abs(s1 - s2) < 1e-10


# ------------------------------------------------------------------ growing context
def test_density_of_grown_cloud_differs_by_one_kernel_column(oracle):
    """What an incremental refresh relies on: L*rho are plain kernel sums, so appending a key adds
    exactly its kernel column to the old keys' sums and its own column sum (self term 1) as a new entry."""
    from scipy.spatial.distance import cdist
    K = rng_arr(15, 41, 6)
    sigma = 1.3
    old = 40 * oracle.density(K[:40], sigma)
    new = 41 * oracle.density(K, sigma)
    col = np.exp(-cdist(K, K[40:41], "sqeuclidean")[:, 0] / (2 * sigma * sigma))
    assert np.allclose(new[:40] - old, col[:40], rtol=1e-10, atol=1e-13)
    assert np.isclose(new[40], col.sum(), rtol=1e-13) and col[40] == 1.0
