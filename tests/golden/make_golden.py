"""Writes tests/golden/config1_oracle.json from the CPU oracle only (run from the repo root).

The paper prints no worked numeric example of Alg. 1-4, so this file is a regression pin of
the oracle on workload 1 (B=1, N=64, 4 nodes x 32 cores, seed 0), not a value from the paper."""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import gen                     # noqa: E402
from oracle import orc         # noqa: E402

p = gen.make_config(1)
o = orc.assign(p)
out = dict(node=[int(x) for x in o["node"]], units=[int(x) for x in o["units"]],
           act_us=[int(x) for x in o["act_us"]],
           score_sum_mod64=int(orc.score(p).astype(np.uint64).sum()))
json.dump(out, open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "config1_oracle.json"), "w"))
