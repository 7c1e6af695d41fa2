"""Test glue: turn a generated workload into the plain lists the oracle takes."""
import numpy as np


def cache_lists(w, upto_event=None):
    ks, vs = [], []
    for i, e in enumerate(w.events):
        if upto_event is not None and i >= upto_event:
            break
        if e.kind == "append":
            ks.append(e.k.astype(np.float64))
            vs.append(e.v.astype(np.float64))
    return ks, vs


def attend_events(w):
    return [(i, e) for i, e in enumerate(w.events) if e.kind == "attend"]


def read_golden(path):
    """'key v v v' lines, '#' comments; a 'mask' line starts a 0/1 matrix."""
    out, mask, in_mask = {"call": []}, [], False
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if in_mask:
                mask.append([int(x) for x in line.split()])
                continue
            key, *vals = line.split()
            if key == "mask":
                in_mask = True
            elif key == "call":
                out["call"].append(dict(v.split("=") for v in vals))
            else:
                out[key] = vals
    if mask:
        out["mask"] = np.asarray(mask, dtype=bool)
    return out
