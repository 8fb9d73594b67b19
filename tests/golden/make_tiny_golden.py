"""Writes tests/golden/tiny_tp1_rollout.json from the CPU oracle alone.

The paper prints no worked numeric example of the decode step, so this file is
a regression pin of the oracle on the tiny configuration (3 sequences, 4 greedy
steps), not a paper value.  Run:  python tests/golden/make_tiny_golden.py
"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import pat_inputs as pi  # noqa: E402
from oracle import Oracle  # noqa: E402
from test_oracle_pins import _tiny_decoder  # noqa: E402

N_SEQ, STEPS = 3, 4
dec, _, _, _ = _tiny_decoder(Oracle("f64"), pi.CONFIGS["tiny_tp1"]["shard"], n_seq=N_SEQ, steps=STEPS)
tokens, rows = [], []
for _ in range(STEPS):
    logits, nxt, _ = dec.step()
    tokens.append([int(t) for t in nxt])
    rows.append([float(v) for v in logits[0, :8]])
out = dict(source="oracle/pat_oracle.c (float64), pat_inputs seeds 0x5EED0001..3", n_seq=N_SEQ, steps=STEPS,
           tokens=tokens, logits_row0_first8=rows)
with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_tp1_rollout.json"), "w") as f:
    json.dump(out, f, indent=1)
print("wrote", tokens)
