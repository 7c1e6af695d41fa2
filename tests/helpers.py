"""Test glue: turn a generated workload into the plain lists the oracle takes."""
import numpy as np


def cache_lists(w, upto_event=None):
    ks, vs = [], []
    for i, e in enumerate(w.events):
        if upto_event is not None and i >= upto_event:
            break
        if e.kind == "append":
            ks.append(e.k)      # float32 holding exactly representable values; the
            vs.append(e.v)      # oracle widens what it gathers to fp64
        elif e.kind == "extend":                    # one more token for each listed message
            for j, m in enumerate(e.msgs):
                ks[m] = np.concatenate([ks[m], e.k[j:j + 1]], axis=0)
                vs[m] = np.concatenate([vs[m], e.v[j:j + 1]], axis=0)
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


def oracle_for_event(w, ev_index, rows_per_call=None, calls_subset=None):
    """Oracle outputs for the attend event at w.events[ev_index].

    rows_per_call: None (all rows) or a function n_q -> list of row indices.
    calls_subset: None (all calls) or a list of call indices.
    Returns a list of (call_index, row_indices, out, lse)."""
    from oracle import choreo_oracle as orc
    ks, vs = cache_lists(w, upto_event=ev_index)
    ev = w.events[ev_index]
    offs = np.concatenate([[0], np.cumsum([c.n_q for c in ev.calls])]).astype(int)
    res = []
    for ci, c in enumerate(ev.calls):
        if calls_subset is not None and ci not in calls_subset:
            continue
        rows = list(range(c.n_q)) if rows_per_call is None else list(rows_per_call(c.n_q))
        o, l = orc.attend_call(ks, vs, c.sel, c.self_msg, c.self_start, c.n_q, c.q_pos,
                               ev.q[offs[ci]:offs[ci + 1]], w.rope_theta, rows=rows)
        res.append((ci, np.asarray(rows, dtype=int) + offs[ci], o, l))
    return res
