"""Writes tests/golden/cfg1_oracle.json: the oracle's own output on benchmark
configuration 1 (tiny fp32), kept as a drift alarm for the oracle.  The paper
prints no worked numeric example, so no stored value here is the paper's.
Calls only oracle/ and the seeded input generator.

    python tests/golden/make_golden.py
"""
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
from paper_2602_22732_amd import synth  # noqa: E402

w = synth.workload(1)
W, X = synth.make_weights(w), synth.make_context(w)
sid, lp, _ = oracle.Oracle(weights=W, **w.model_kwargs()).decode_batch(X, None, w.beam, oracle.MODE_PLAIN)
with open(os.path.join(HERE, "cfg1_oracle.json"), "w") as f:
    json.dump({"source": "oracle.decode_batch(MODE_PLAIN) on synth.workload(1); written by tests/golden/make_golden.py",
               "sid": sid.tolist(), "logprob": [[float("%.12g" % v) for v in row] for row in lp]}, f)
print("wrote cfg1_oracle.json", sid.shape)
