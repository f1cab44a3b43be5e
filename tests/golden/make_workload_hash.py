"""Writes tests/golden/workload_cfg0_seed1234.sha256: a digest of the workload-0
input arrays (CSR, hotness order, first seed batch, 16 feature rows) made by
paper_2310_00837_amd.workload alone.  Run from the repo root."""
import hashlib
import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from paper_2310_00837_amd import workload as W  # noqa: E402

g = W.make_graph(W.spec(0), 1234, "cpu")
h = hashlib.sha256()
for t in (g.offsets, g.indices, g.order, W.seed_batch(W.spec(0), g, 0)):
    h.update(t.numpy().tobytes())
h.update(W.feature_rows(1234, torch.arange(16), 64, torch.float32).numpy().tobytes())
out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "workload_cfg0_seed1234.sha256")
with open(out, "w") as fh:
    fh.write(h.hexdigest() + "  workload 0, seed 1234\n")
print(h.hexdigest())
