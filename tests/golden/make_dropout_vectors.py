"""Writes dropout_mask_vectors.json from the oracle (and nothing else).

The test-suite checks these stored masks against an independent big-integer
re-implementation of the generator, which is what pins them; the file keeps a
fixed record of the generator's output for a few keys.  Generator definition:
SplitMix64 finaliser keyed by (seed, step, worker, layer), counter = element
index; see the comment above ``oracle_dropout_mask``.
Run:  python tests/golden/make_dropout_vectors.py
"""
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
from oracle import ops  # noqa: E402

cases = []
for seed, step, worker, layer, p in [(0, 0, 0, 0, 0.5), (3003, 19, 3, 21, 0.5), (2**64 - 1, 2**64 - 1, 2**32 - 1, 2**32 - 1, 0.5),
                                     (42, 1, 0, 14, 0.1)]:
    m = ops.dropout_mask(96, seed, step, worker, layer, p)
    cases.append({"seed": seed, "step": step, "worker": worker, "layer": layer, "p": p,
                  "mask": "".join(str(int(b)) for b in m)})
with open(os.path.join(HERE, "dropout_mask_vectors.json"), "w") as f:
    json.dump({"generator": "splitmix64-finaliser, see oracle/asgd_oracle.c", "cases": cases}, f, indent=1)
