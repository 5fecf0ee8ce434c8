"""Writes tests/golden/oracle_digests.json from the CPU oracle alone.

Run from the repository root:  python tests/golden/make_golden.py
It calls only oracle/ and the seeded input generator (never the HIP library).
"""
import hashlib
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import oracle as orc                      # noqa: E402
from paper_2510_27656_amd import workloads as wlmod   # noqa: E402


def digest(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def compute():
    wl = wlmod.WORKLOADS["tiny"]
    inp = wlmod.make_inputs(wl)
    N, E, K, H = wl.n_ranks, wl.n_experts, wl.top_k, wl.hidden
    lay = orc.layout(N, E, K, inp.num_tokens, inp.indices)
    stride = int(lay.expert_off[:, -1].max())
    Y = np.zeros((N, stride, H), np.uint16)
    for d in range(N):
        rows = orc.dispatch_rank(d, N, E, K, inp.num_tokens, inp.indices, inp.x)
        Y[d, :rows.shape[0]] = rows
    out = orc.combine(N, E, K, inp.num_tokens, inp.indices, lay.slot, inp.weights, Y, stride, H)
    return {
        "workload": "tiny (2 ranks x 4 experts, 16 tokens/rank, hidden 256, top-2, seed 0)",
        "inputs": {"x": digest(inp.x), "indices": digest(inp.indices),
                   "weights": digest(inp.weights)},
        "C": lay.C.tolist(),
        "M": lay.M.tolist(),
        "expert_off": lay.expert_off.tolist(),
        "slot": digest(lay.slot),
        "expert_rows": digest(Y),
        "combined": digest(out),
    }


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_digests.json")
    json.dump(compute(), open(path, "w"), indent=1)
    print("wrote", path)
