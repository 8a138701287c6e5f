"""Writes the oracle's full-size density of the long-context configuration (8 KV heads, d = 128,
L = 131072, bf16 keys), to tests/golden/long_context_density_h{0..7}.npz.

The greedy chain of a head needs the density of all L keys, and the float64 oracle needs several
minutes of CPU time per head for it at this size (L^2 d = 2.2e12 multiply-adds), too long to sit
inside a GPU test.  This script calls ONLY the oracle (oracle/ws_oracle.py) and the seeded input
generator; nothing comes from the HIP path.  Each file holds rho (float64 [L]), the bandwidth that
was used (the float32 of the sigma^2 = tr(Cov)/16 recipe), and a checksum of the generated key bits
so that a test can tell when the generator no longer produces the same cloud.

Run from the repository root:  python tests/golden/make_long_context_density.py [head ...]
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import ws_oracle as oracle                      # noqa: E402
from paper_2601_01298_amd import synthetic as syn           # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))


def key_checksum(K: np.ndarray) -> int:
    bits = syn.bf16_bits(K).astype(np.uint64)
    weights = (np.arange(bits.size, dtype=np.uint64) % np.uint64(65521)) + np.uint64(1)
    return int((bits.ravel() * weights).sum(dtype=np.uint64))


def main():
    heads = [int(a) for a in sys.argv[1:]] or list(range(8))
    w = syn.WORKLOADS[5]
    oracle.build()
    for h in heads:
        K = syn.cloud(w, h, syn.TENSOR_K)
        sigma = syn.bandwidth(K)
        t = time.time()
        rho = oracle.density(K, float(sigma))
        out = os.path.join(HERE, f"long_context_density_h{h}.npz")
        np.savez(out, rho=rho, sigma=np.float32(sigma), key_checksum=np.uint64(key_checksum(K)),
                 L=np.int64(w.L), d=np.int64(w.d))
        print(f"head {h}: {time.time() - t:.0f} s, rho in [{rho.min():.3e}, {rho.max():.3e}] -> {out}", flush=True)


if __name__ == "__main__":
    main()
