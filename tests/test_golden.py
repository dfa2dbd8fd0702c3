"""The oracle against the hand-derived worked example stored under tests/golden/."""
import os
from fractions import Fraction

import numpy as np
import torch

from oracle import paged_attention_oracle as oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "power_of_two_weights.txt")


def read_expected():
    rows = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            rows[int(parts[0])] = [float(Fraction(x)) for x in parts[1:]]
    return np.array([rows[0], rows[1]], dtype=np.float64)


def test_power_of_two_weights_example():
    L, D, page = 18, 4, 16
    kd = np.zeros((L, D), dtype=np.float32)
    vd = np.zeros((L, D), dtype=np.float32)
    for t in range(L):
        kd[t] = [t % 3, -(t % 2), 0, 0]
        vd[t] = [t, 1, -t, t * (17 - t)]
    # physical pages 2 (tokens 0..15) and 0 (tokens 16, 17); page 1 and the dead slots hold NaN
    kp = np.full((3, 1, page, D), np.nan, dtype=np.float32)
    vp = np.full((3, 1, page, D), np.nan, dtype=np.float32)
    kp[2, 0], vp[2, 0] = kd[:16], vd[:16]
    kp[0, 0, :2], vp[0, 0, :2] = kd[16:], vd[16:]
    bt = np.array([[2, 0]], dtype=np.int32)
    q = np.array([[[1, 0, 0, 0], [0, 2, 0, 0]]], dtype=np.float32)
    to_bf16 = lambda a: torch.from_numpy(a).to(torch.bfloat16)   # every value above is exact in bf16
    scale = float(np.float32(np.log(2.0)))
    out = oracle.paged_decode_attn(to_bf16(q), to_bf16(kp), to_bf16(vp), bt,
                                   np.array([L], dtype=np.int32), scale)
    np.testing.assert_allclose(out[0], read_expected(), rtol=1e-6, atol=0)
