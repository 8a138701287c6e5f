"""Helpers shared by the GPU parity tests: moving generated inputs to the device, the
near-tie rejection rule, and the step-granular index check."""
import numpy as np

from paper_2601_01298_amd import synthetic as syn

TIE_TOL = 1e-5          # relative gap below which the oracle's top two scores count as a near-tie


def to_device(x: np.ndarray, dtype: str):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)       # exact: the generator already rounded to the bf16 grid
    return t.cuda()


def accepted_head(oracle, w, head, alpha=None, max_tries=20):
    """Generate head `head` of workload `w`, bumping the seed until the oracle's greedy chain has
    no step whose top two scores are within TIE_TOL.  Returns a dict and the rejection count."""
    alpha = w.alpha if alpha is None else alpha
    for attempt in range(max_tries):
        seed = syn.BASE_SEED + attempt
        K = syn.cloud(w, head, syn.TENSOR_K, seed)
        sigma = syn.bandwidth(K)
        rho = oracle.density(K, float(sigma))
        idx, score, gap = oracle.select(K, rho, w.k, alpha)
        if gap.min() >= TIE_TOL:
            V = syn.cloud(w, head, syn.TENSOR_V, seed)
            return dict(K=K, V=V, sigma=sigma, rho=rho, idx=idx, score=score, gap=gap, seed=seed), attempt
    raise RuntimeError("no tie-free input found")


def check_indices(oracle, K, rho_ref, k, alpha, idx_gpu, idx_ref):
    """Bit-exact match, or -- for long chains where the oracle itself has sub-TIE_TOL steps --
    every differing pick must be a near-tie fork under its own prefix.  Returns the fork count."""
    idx_gpu = np.asarray(idx_gpu, dtype=np.int32)
    if np.array_equal(idx_gpu, idx_ref):
        return 0
    forks, pick, deficit = oracle.select_verify(K, rho_ref, k, alpha, idx_gpu)
    assert forks >= 0, "GPU index list repeats an index or is out of range"
    bad = np.nonzero(deficit > TIE_TOL)[0]
    assert bad.size == 0, (f"pick {bad[0]}: GPU chose {idx_gpu[bad[0]]}, oracle {pick[bad[0]]}, "
                           f"relative deficit {deficit[bad[0]]:.3e} > {TIE_TOL}")
    return int(forks)


def attn_rel_err(O_gpu: np.ndarray, O_ref: np.ndarray) -> float:
    """max over (agent, query head) of |O_gpu - O_ref|_inf / |O_ref|_inf."""
    num = np.abs(O_gpu.astype(np.float64) - O_ref).max(axis=-1)
    den = np.abs(O_ref).max(axis=-1)
    return float((num / den).max())
