"""Writes tests/golden/workload_digest.txt: SHA-256 of the config-1 inputs drawn by the
seeded generators, so that a drift of the generators is caught.  Calls workloads/ only."""
import hashlib
import os
import sys

import numpy as np
import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
import workloads as wl


def digests():
    cfg = wl.CONFIGS[0]
    ids, gates = wl.make_routing(cfg, 0)
    X, dOut = wl.make_tokens(cfg, 0)
    Wg, Wu, Wd = wl.make_weights(cfg)
    out = {"ids": hashlib.sha256(np.ascontiguousarray(ids).tobytes()).hexdigest()}
    for name, t in (("X", X), ("dOut", dOut), ("Wg", Wg), ("Wu", Wu), ("Wd", Wd)):
        out[name] = hashlib.sha256(t.contiguous().view(torch.int16).numpy().tobytes()).hexdigest()
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "workload_digest.txt")
    with open(path, "w") as f:
        f.write("# SHA-256 of config-1 (tiny) inputs; written by write_workload_digest.py\n")
        for k, v in digests().items():
            f.write(f"{k} {v}\n")
    print(open(path).read())
