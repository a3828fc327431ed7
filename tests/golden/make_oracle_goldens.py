"""Writes tests/golden/<cfg>_oracle.json: what the CPU oracle returns for a named configuration at full size.

Calls only the oracle and the seeded input generators (never the HIP path).  The GPU parity test
`tests/test_gpu_configs.py` compares `rama_solve` with these stored values for the configurations the
oracle needs minutes for (cfg4: 2.5e7 edges, cfg5: 9.8e7 edges; single thread, up to ~25 GB of host memory).

    python tests/golden/make_oracle_goldens.py cfg4 cfg5

Stored per configuration: sizes, SHA-256 of the input arrays (so that a test can tell a different input
from a different result), primal cost (eq. 2 of the paper on the input costs), lower bound (eq. 5 after
message passing on the original graph), rounds, clusters, conflicted cycles per length and edges after
triangulation in the first round, edges of the last contracted graph, SHA-256 of the int32 label array
(label = smallest node of the cluster), every `label_stride`-th label, oracle seconds and threads.
"""
import hashlib
import json
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2109_01838_amd import inputs  # noqa: E402

LABEL_SAMPLES = 512


def sha(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def golden(name):
    g = inputs.make(name)
    n = g["n_nodes"]
    t0 = time.time()
    r = oracle.Oracle("f32").solve(n, g["i"], g["j"], g["c"])
    sec = time.time() - t0
    stride = max(1, n // LABEL_SAMPLES)
    return dict(
        config=name, instance=g["name"], n_nodes=int(n), n_edges=int(g["i"].size),
        input_sha256=dict(i=sha(g["i"]), j=sha(g["j"]), c=sha(g["c"])),
        params="rama_params_default: cycles <=5 then <=3, k = 10 then 5, tau 0, forest_ratio 0.1",
        primal=r["primal"], lower_bound=r["lower_bound"], rounds=r["rounds"], n_clusters=r["n_clusters"],
        n_cycles_first=r["n_cycles_first"], n_edges_aug_first=r["n_edges_aug_first"],
        n_edges_final=r["n_edges_final"], labels_sha256=sha(r["labels"].astype("<i4")),
        label_stride=stride, label_samples=[int(x) for x in r["labels"][::stride]],
        oracle_seconds=round(sec, 1), oracle_threads=1, oracle_precision="f32",
    )


if __name__ == "__main__":
    for name in sys.argv[1:] or ["cfg4", "cfg5"]:
        out = golden(name)
        path = os.path.join(HERE, f"{name}_oracle.json")
        with open(path, "w") as f:
            json.dump(out, f, indent=1)
            f.write("\n")
        print(name, {k: out[k] for k in ("primal", "lower_bound", "rounds", "n_clusters", "oracle_seconds")},
              flush=True)
