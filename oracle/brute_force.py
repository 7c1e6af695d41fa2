"""Scalar brute-force check of the oracle (TEST INFRASTRUCTURE, tiny inputs only).

A second, independent evaluation of choreographed attention written with
Python loops and complex arithmetic: a RoPE pair (x_i, x_{i+D/2}) is the
complex number x_i + 1j*x_{i+D/2}, and placing a token at position p
multiplies it by exp(1j * p * theta^(-2i/D)) (Sec. 2.4 "Position Updates":
rotation by an angle proportional to the position).  The score of a query
against a key is then Re(sum_i q_i * conj(k_i)), which depends on the two
positions only through their difference (Sec. 2.2, assumption 3).

Visibility follows Sec. 2.4 "Dynamic Masking": every token of every listed
parent, plus the new message's tokens up to the query's own token.

It shares nothing with ``choreo_oracle`` beyond the meaning of its arguments.
"""
from __future__ import annotations

import cmath
import math

POS_AUTO = -(2 ** 31)


def attend_call_brute(msgs_k, msgs_v, sel, self_msg, self_start, n_q, q_pos, q, theta, scale=None):
    """Nested-list / ndarray inputs as in the oracle; returns nested lists
    out[r][h][d], lse[r][h]."""
    H_kv = len(msgs_k[0][0])
    D = len(msgs_k[0][0][0])
    H_q = len(q[0]) if n_q else 0
    g = H_q // H_kv if H_q else 1
    half = D // 2
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    w = [theta ** (-2.0 * i / D) for i in range(half)]

    # walk the list: (message, token, position, is_self)
    toks = []
    nxt = 0
    for (m, s) in sel:
        if s == POS_AUTO:
            s = nxt
        L = len(msgs_k[m])
        for t in range(L):
            toks.append((m, t, s + t, False))
        nxt = s + L
    s_self = nxt if self_start == POS_AUTO else self_start
    L_self = len(msgs_k[self_msg]) if self_msg >= 0 else 0
    for t in range(L_self):
        toks.append((self_msg, t, s_self + t, True))

    out = [[[0.0] * D for _ in range(H_q)] for _ in range(n_q)]
    lse = [[-math.inf] * H_q for _ in range(n_q)]
    for r in range(n_q):
        own = (L_self - n_q + r) if self_msg >= 0 else r
        p_r = int(q_pos[r]) if q_pos is not None else s_self + own
        for h in range(H_q):
            kh = h // g
            qc = [complex(q[r][h][i], q[r][h][i + half]) * cmath.exp(1j * p_r * w[i])
                  for i in range(half)]
            scores, vals = [], []
            for (m, t, p, is_self) in toks:
                if is_self and t > own:
                    continue
                acc = 0.0
                for i in range(half):
                    kc = complex(msgs_k[m][t][kh][i], msgs_k[m][t][kh][i + half]) \
                        * cmath.exp(1j * p * w[i])
                    acc += (qc[i] * kc.conjugate()).real
                scores.append(scale * acc)
                vals.append(msgs_v[m][t][kh])
            if not scores:
                continue
            mx = max(scores)
            e = [math.exp(s - mx) for s in scores]
            den = sum(e)
            for d in range(D):
                out[r][h][d] = sum(e[j] * float(vals[j][d]) for j in range(len(e))) / den
            lse[r][h] = mx + math.log(den)
    return out, lse
