#!/usr/bin/env python3
"""Writes tests/golden/oracle_digests.txt: SHA-256 digests of what the CPU oracle produces for a few small seeded
cases (messages, fitted levels, step-size scalars).  Calls only oracle/ and the seeded input generators.  The digests
pin nothing to the paper; they make any later change to the oracle's arithmetic visible, so that such a change has to
be made on purpose (and justified against the paper where it is committed)."""
from __future__ import annotations

import hashlib
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2505_14371_amd import workloads  # noqa: E402


def digest(*arrays) -> str:
    h = hashlib.sha256()
    for a in arrays:
        h.update(np.ascontiguousarray(a).tobytes())
    return h.hexdigest()


def cases():
    w = workloads.mini("txl", max_layer=20000, max_layers=6)
    L = len(w.sizes)
    K = 2
    g = [[workloads.node_numpy(w, k, t) for k in range(K)] for t in (1, 2)]
    for scope, name in ((0, "layer"), (1, "vector"), (2, "bucket")):
        for S in (4, 8, 17):
            uni = (np.arange(S, dtype=np.float64) / (S - 1)).astype(np.float32)
            flat = [g[0][k][l] for k in range(K) for l in range(L)]
            lev, _, pooled, _ = oracle.fit_levels(w.sizes, [l % 2 for l in range(L)], [S, S], K, flat, [uni, uni], scope=scope)
            yield f"fit {name} S={S}", digest(*lev, pooled)
            lev_l = [lev[l % 2] for l in range(L)]
            m1, ss, d1, _ = oracle.quantize(w.sizes, [S] * L, lev_l, g[0][0], w.seed, 1, 0, scope=scope)
            m2, _, d2, _ = oracle.quantize(w.sizes, [S] * L, lev_l, g[1][0], w.seed, 2, 0, msg_prev=m1, scope=scope)
            yield f"quantize {name} S={S}", digest(m1, m2, np.array([d1, d2]), ss)
            mean = oracle.dequant_aggregate(w.sizes, [S] * L, [m1, m2], scope=scope)
            yield f"aggregate {name} S={S}", digest(*mean)
    acc, eta = oracle.step_size([1.5, 2.25, 0.125], 0.75)
    e2, g2 = oracle.alt_step_size(12.5, 3.25, 0.2)
    yield "step sizes", digest(np.array([acc]), np.array([eta, e2, g2], dtype=np.float32))


def main() -> int:
    out = os.path.join(HERE, "oracle_digests.txt")
    with open(out, "w") as f:
        f.write("# written by tests/golden/make_oracle_digests.py (oracle outputs only; see its docstring)\n")
        for name, d in cases():
            f.write(f"{d}  {name}\n")
    print("wrote", out)
    return 0


if __name__ == "__main__":
    sys.exit(main())
