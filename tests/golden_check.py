"""Comparison of a GPU solve with the oracle's stored result for a named configuration
(tests/golden/<cfg>_oracle.json, written by tests/golden/make_oracle_goldens.py from the oracle alone)."""
import hashlib
import json
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def sha(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def load(name):
    with open(os.path.join(HERE, "golden", f"{name}_oracle.json")) as f:
        return json.load(f)


def check_against_golden(name, g, got):
    """g: the instance (host arrays), got: what Rama.solve returned.  Returns whether the labels are identical."""
    want = load(name)
    # the stored result belongs to exactly this input
    assert g["n_nodes"] == want["n_nodes"] and g["i"].size == want["n_edges"]
    for k in ("i", "j", "c"):
        assert sha(g[k]) == want["input_sha256"][k], f"input array {k} differs from the one the oracle solved"
    labels = got["labels"].cpu().numpy().astype("<i4")
    same = sha(labels) == want["labels_sha256"]
    # end-to-end tolerances: primal within 0.5 %, lower bound within 1e-4 relative; integer counts equal
    assert abs(got["lower_bound"] - want["lower_bound"]) <= 1e-4 * abs(want["lower_bound"]), (got["lower_bound"], want["lower_bound"])
    assert abs(got["primal"] - want["primal"]) <= 5e-3 * abs(want["primal"]), (got["primal"], want["primal"])
    assert got["n_cycles_first"] == want["n_cycles_first"]
    assert got["n_edges_aug_first"] == want["n_edges_aug_first"]
    assert got["lower_bound"] <= got["primal"]
    stride = want["label_stride"]
    sample_same = np.array_equal(labels[::stride], np.asarray(want["label_samples"], dtype="<i4"))
    print(name, "labels identical to the oracle's:", same, "(sampled labels identical:", sample_same, ")",
          "rounds", got["rounds"], want["rounds"], "clusters", got["n_clusters"], want["n_clusters"],
          "primal", got["primal"], want["primal"], "lb", got["lower_bound"], want["lower_bound"], flush=True)
    if same:
        assert got["rounds"] == want["rounds"] and got["n_clusters"] == want["n_clusters"]
        assert got["n_edges_final"] == want["n_edges_final"]
    return same
