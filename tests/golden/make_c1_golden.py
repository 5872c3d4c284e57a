"""Writes tests/golden/c1_tiny_oracle.json from the CPU oracle alone (never from the HIP path).

The paper prints no worked numerical example of an MoE layer, so this digest only guards the
oracle against drift; the pins in tests/test_oracle_pins.py are what tie it to the definitions.
Run: python tests/golden/make_c1_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2509_07379_amd import synth as S  # noqa: E402

w = S.WORKLOADS["c1_tiny"]
r = oracle.moe_layer(S.activations(w), S.router_weight(w),
                     [S.expert_blob(w, 0, e) for e in range(w.E)], w.k)
out = dict(counts=r["counts"].tolist(), ids_first8=r["ids"][:8].tolist(),
           out_bits_first=r["out"][:2, :8].tolist(),
           out_bits_sum=int(r["out"].astype(np.uint64).sum()))
with open(os.path.join(os.path.dirname(__file__), "c1_tiny_oracle.json"), "w") as f:
    json.dump(out, f, indent=1)
print(out)
