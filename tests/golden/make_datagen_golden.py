"""Writes tests/golden/datagen_first8.json: the first draws / indices / labels of workloads 1-3.
Calls only datagen/ (integer-exact input recipes); run once, the file is then frozen."""
import json
import os
import sys
import numpy as np
sys.path.insert(0, os.path.join(os.path.dirname(__file__), "..", ".."))
from datagen import CounterRNG, make_workload  # noqa: E402

out = {}
for cfg in (1, 2, 3):
    wl = make_workload(cfg)
    out[str(cfg)] = dict(raw_stream1=[int(v) for v in CounterRNG(wl.seed).raw(1, 8)],
                         train_batch0=wl.train_batch(0)[:8].tolist(), y_train=wl.y_train[:8].tolist(),
                         y_meta=wl.y_meta[:8].tolist(), flipped_idx=np.nonzero(wl.flipped)[0][:8].tolist())
json.dump(out, open(os.path.join(os.path.dirname(__file__), "datagen_first8.json"), "w"), indent=1)
