"""Writes tests/golden/oracle_digest.json: SHA-256 digests of what the CPU
oracle produces on a small graph made with integer arithmetic only.

Calls only oracle/ and the input generator.  The values are the oracle's own
(the paper prints none for this path): the file guards against unnoticed
changes of the oracle or of the readings it encodes, it is not a pin.

    python tests/golden/make_oracle_digest.py
"""
import hashlib
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle                                   # noqa: E402
from paper_2509_05207_amd import synth          # noqa: E402

PARAMS = dict(n=2000, deg_lo=0, deg_hi=60, graph_seed=5, n_train=450, batch_size=64, fanout=[7, 4, 3],
              s0=42, worker=2, epoch=1, K=120)


def inputs():
    p = PARAMS
    indptr, indices = synth.integer_graph(p["n"], p["deg_lo"], p["deg_hi"], p["graph_seed"])
    train = np.arange(0, p["n"], 4, dtype=np.int32)[: p["n_train"]]
    is_local = (np.arange(p["n"]) % 3 == 0).astype(np.uint8)
    return indptr, indices, train, is_local


def digests():
    p = PARAMS
    indptr, indices, train, is_local = inputs()
    s = oracle.Schedule(indptr, indices, train, p["batch_size"], p["fanout"], p["s0"], p["worker"], p["epoch"])
    h = lambda a: hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()   # noqa: E731
    out = {"graph": h(indptr) + h(indices), "n_batches": int(s.n_batches)}
    for hop in range(s.L + 1):
        ids, off = s.frontier(hop)
        out[f"frontier{hop}"] = h(ids) + h(off)
    for hop in range(s.L):
        so, nb = s.samples(hop)
        out[f"samples{hop}"] = h(so) + h(nb)
    freq = oracle.frequency([s], p["n"])
    ids, slot = oracle.top_hot(freq, is_local, p["K"])
    out["freq"] = h(freq)
    out["cache_ids"] = h(ids)
    out["slot_of"] = h(slot)
    out["batch_seed_0"] = int(oracle.batch_seed(p["s0"], p["worker"], p["epoch"], 0))
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_digest.json")
    with open(path, "w") as fh:
        json.dump({"params": PARAMS, "digests": digests()}, fh, indent=1)
    print("wrote", path)
