"""Writes tests/golden/tiny_case.txt from the CPU oracle alone (run: python tests/golden/make_golden.py).

The paper prints no worked numeric example for the attention path, so this fixture is a
regression guard for the oracle's arithmetic, not a paper value: the oracle itself is
pinned by the identities and closed forms in tests/test_oracle_pins.py.
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))


def tiny_case(oracle):
    """Two ragged sequences, 4 query heads on 2 KV heads, d = 8, M_k = 3, M_v = 2, K = 4."""
    rng = np.random.Generator(np.random.PCG64(20250618))
    lens = np.array([5, 3])
    cu = np.array([0, 5, 8], np.int32)
    q = rng.standard_normal((2, 4, 8))
    kcb = rng.standard_normal((2, 3, 4, 8))
    vcb = rng.standard_normal((2, 2, 4, 8))
    kc = np.concatenate([rng.integers(0, 4, (2, L, 3)).astype(np.uint8).reshape(-1) for L in lens])
    vc = np.concatenate([rng.integers(0, 4, (2, L, 2)).astype(np.uint8).reshape(-1) for L in lens])
    return oracle.decode_attn(q, kc, vc, kcb, vcb, cu, (lens - 1).astype(np.int32), rope_base=500000.0)


if __name__ == "__main__":
    sys.path.insert(0, ROOT)
    import oracle

    out = tiny_case(oracle)
    np.savetxt(os.path.join(HERE, "tiny_case.txt"), out.reshape(-1, 8), fmt="%.17e",
               header="oracle.decode_attn on tiny_case() of make_golden.py; rows = (b, h), cols = d")
