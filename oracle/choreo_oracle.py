"""CPU oracle for choreographed attention (TEST INFRASTRUCTURE, not product).

A plain, dense, fp64 statement of what the attention step of Prompt
Choreography computes.  Only tests, the smoke check and the benchmark's CPU
baseline leg may import this module; it shares no code with the HIP path.

What is computed, and where the paper fixes it:

* A call names parent messages and the position each one starts at; the new
  message's tokens see every token of every parent and the earlier tokens of
  their own message, nothing else in the cache (Sec. 2.3 ``prefill`` /
  ``decode``; Sec. 2.4 "Dynamic Masking"; Fig. 2).
* Position enters only through RoPE: token ``i`` of a message placed at
  offset ``o`` sits at logical position ``o + i`` (Sec. 2.4, the ``(m, j)``
  pair), and moving a token rotates its key by an angle proportional to the
  move (Sec. 2.4 "Position Updates").  The oracle therefore takes unrotated
  keys and rotates each gathered copy at its assigned position.
* An omitted offset means "right after the end of the preceding parent"
  (Sec. 2.3).
* Several calls may be batched; each sees exactly what it lists (Sec. 2.4
  "Parallel API Calls").

Readings taken where the paper is silent (pairing convention of RoPE, softmax
scale, self-visibility of a token, what an omitted *first* offset means ...)
are listed in the repository's design notes; each is marked "reading" below.

Every function here is pinned by tests that do not call it to produce their
own expectation: brute force with complex arithmetic, reduction to a library
causal attention, shift / permutation invariance, closed forms, hand-written
tables; the gradient (attend_call_backward) by central differences of the forward
oracle and by closed forms.  Agreement with the authors' implementation on real model activations
is "parity unpinned": that code and its weights are not available.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np

POS_AUTO = -(2 ** 31)


# ---------------------------------------------------------------------------
# cache layout rule (an interface fact shared with the library's header: messages
# are appended in order, ids are 0,1,2..., each starts at the next slot that is
# a multiple of `align` after the previous message's reserved span; Sec. 2.4,
# append-only cache with a message -> span map)
# ---------------------------------------------------------------------------
def slot_starts(reserves: Sequence[int], align: int) -> List[int]:
    starts, nxt = [], 0
    for r in reserves:
        starts.append(nxt)
        nxt = ((nxt + int(r) + align - 1) // align) * align
    return starts


class SlotModel:
    """The same layout rule with messages that can be given back (an interface fact of the
    library's header): a new message takes the lowest freed span that holds its reserve rounded
    up to `align`, else the end of the used region; adjacent freed spans merge; a span freed at
    the end of the used region shrinks it.  Plain bookkeeping over a list of (start, size)."""

    def __init__(self, align: int):
        self.align, self.end, self.free, self.span = align, 0, [], {}

    def append(self, msg_id: int, reserve: int) -> int:
        need = ((int(reserve) + self.align - 1) // self.align) * self.align
        for i, (st, sz) in enumerate(self.free):
            if sz >= need:
                if sz == need:
                    del self.free[i]
                else:
                    self.free[i] = (st + need, sz - need)
                self.span[msg_id] = (st, need)
                return st
        st = self.end
        self.end += need
        self.span[msg_id] = (st, need)
        return st

    def release(self, msg_id: int) -> None:
        st, sz = self.span.pop(msg_id)
        spans = sorted(self.free + [(st, sz)])
        merged = []
        for a, n in spans:
            if merged and merged[-1][0] + merged[-1][1] == a:
                merged[-1] = (merged[-1][0], merged[-1][1] + n)
            else:
                merged.append((a, n))
        if merged and merged[-1][0] + merged[-1][1] == self.end:
            self.end = merged.pop()[0]
        self.free = merged


# ---------------------------------------------------------------------------
# default offsets (Sec. 2.3: an omitted offset is the position right after the
# end of the preceding parent).  Reading: "preceding" = the previous list entry;
# an omitted first offset is 0; an omitted new-message offset is right after the
# last list entry (0 for an empty list).
# ---------------------------------------------------------------------------
def resolve_positions(sel: Sequence[Tuple[int, int]], lengths: Sequence[int],
                      self_start: int) -> Tuple[List[Tuple[int, int]], int]:
    out = []
    nxt = 0
    for (m, s) in sel:
        s = nxt if s == POS_AUTO else int(s)
        out.append((int(m), s))
        nxt = s + int(lengths[m])
    s_self = nxt if self_start == POS_AUTO else int(self_start)
    return out, s_self


def query_positions(n_q: int, self_len: int, s_self: int,
                    q_pos: Optional[np.ndarray]) -> np.ndarray:
    """Row r is the (self_len - n_q + r)-th token of the new message (reading:
    rows align with the LAST n_q tokens, which covers prefill, chunked prefill and
    one-token decode); its position is offset + token index (Sec. 2.4) unless the
    caller states positions explicitly."""
    if q_pos is not None:
        return np.asarray(q_pos, dtype=np.int64)
    return s_self + (self_len - n_q) + np.arange(n_q, dtype=np.int64)


# ---------------------------------------------------------------------------
# gather table and position map: parents in LIST order, token by token, then the
# new message (Sec. 2.3 / 2.4: the i-th token of a message at offset o has
# position o + i)
# ---------------------------------------------------------------------------
def assemble(sel: Sequence[Tuple[int, int]], self_msg: int, s_self: int,
             lengths: Sequence[int], starts: Sequence[int]):
    """Returns kv_slot[int32 N], kv_pos[int32 N], n_parent_tokens."""
    slot, pos = [], []
    for (m, s) in sel:
        for t in range(int(lengths[m])):
            slot.append(starts[m] + t)
            pos.append(s + t)
    n_parent = len(slot)
    if self_msg >= 0:
        for t in range(int(lengths[self_msg])):
            slot.append(starts[self_msg] + t)
            pos.append(s_self + t)
    return (np.asarray(slot, dtype=np.int32), np.asarray(pos, dtype=np.int32), n_parent)


# ---------------------------------------------------------------------------
# RoPE (Sec. 2.2 assumption 3 and Sec. 2.4 "Position Updates").  Reading: pair
# (i, i + D/2) turns by angle pos * theta^(-2i/D), counter-clockwise.
# ---------------------------------------------------------------------------
def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """x: [n, ..., D] fp64, pos: [n] integers.  Rotates along the last axis."""
    x = np.asarray(x, dtype=np.float64)
    D = x.shape[-1]
    half = D // 2
    freq = float(theta) ** (-2.0 * np.arange(half, dtype=np.float64) / D)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * freq[None, :]          # [n, D/2]
    shape = (x.shape[0],) + (1,) * (x.ndim - 2) + (half,)
    c, s = np.cos(ang).reshape(shape), np.sin(ang).reshape(shape)
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, lo * s + hi * c], axis=-1)


# ---------------------------------------------------------------------------
# visibility (Sec. 2.4 "Dynamic Masking", Fig. 2): all parent tokens, and own
# tokens up to and including the row's own token (reading: a token sees itself).
# Position never masks.
# ---------------------------------------------------------------------------
def visibility(n_q: int, n_parent: int, self_len: int) -> np.ndarray:
    vis = np.zeros((n_q, n_parent + self_len), dtype=bool)
    vis[:, :n_parent] = True
    for r in range(n_q):
        last = self_len - n_q + r
        vis[r, n_parent:n_parent + last + 1] = True
    return vis


def batch_mask(n_cache_tokens: int, token_msg: np.ndarray, calls_parents: Sequence[Sequence[int]],
               new_msgs: Sequence[int], new_token_index: Sequence[np.ndarray]) -> np.ndarray:
    """Boolean mask over the WHOLE physical cache for a batch of parallel calls, as
    in Fig. 2: row = a new token, column = a cached token (new tokens included).
    token_msg[c] is the message id stored beside cached token c (the `m` of the
    (m, j) pair, Sec. 2.4); token index within its message is counted in physical
    order.  Used only for structural tests."""
    idx_in_msg = np.zeros(n_cache_tokens, dtype=np.int64)
    seen = {}
    for c in range(n_cache_tokens):
        m = int(token_msg[c])
        idx_in_msg[c] = seen.get(m, 0)
        seen[m] = idx_in_msg[c] + 1
    rows = []
    for parents, m_new, toks in zip(calls_parents, new_msgs, new_token_index):
        for t in toks:
            row = np.zeros(n_cache_tokens, dtype=bool)
            for c in range(n_cache_tokens):
                m = int(token_msg[c])
                if m in parents:
                    row[c] = True
                elif m == m_new and idx_in_msg[c] <= t:
                    row[c] = True
            rows.append(row)
    return np.asarray(rows)


# ---------------------------------------------------------------------------
# one call
# ---------------------------------------------------------------------------
def attend_call(msgs_k: Sequence[np.ndarray], msgs_v: Sequence[np.ndarray],
                sel: Sequence[Tuple[int, int]], self_msg: int, self_start: int,
                n_q: int, q_pos: Optional[np.ndarray], q: np.ndarray,
                theta: float, scale: Optional[float] = None,
                rows: Optional[Sequence[int]] = None):
    """msgs_k[m], msgs_v[m]: [L_m, H_kv, D] unrotated.  q: [n_q, H_q, D].
    Returns (out [n_rows, H_q, D], lse [n_rows, H_q]) in fp64 for the requested
    rows (all by default).  Empty visible set -> zeros and -inf."""
    lengths = [int(k.shape[0]) for k in msgs_k]
    sel_r, s_self = resolve_positions(sel, lengths, self_start)
    self_len = lengths[self_msg] if self_msg >= 0 else 0
    starts = slot_starts(lengths, 1)            # dense ids: only used to index `flat` below
    kv_slot, kv_pos, n_parent = assemble(sel_r, self_msg, s_self, lengths, starts)
    H_kv, D = msgs_k[0].shape[1], msgs_k[0].shape[2]
    H_q = q.shape[1]
    g = H_q // H_kv
    if scale is None:
        scale = 1.0 / np.sqrt(D)                # reading: standard 1/sqrt(d)

    # materialise the assembled sequence explicitly
    N = kv_slot.shape[0]
    Kc = np.empty((N, H_kv, D), dtype=np.float64)
    Vc = np.empty((N, H_kv, D), dtype=np.float64)
    at = 0
    for (m, _s) in sel_r:
        L = lengths[m]
        Kc[at:at + L] = msgs_k[m]
        Vc[at:at + L] = msgs_v[m]
        at += L
    if self_msg >= 0:
        Kc[at:at + self_len] = msgs_k[self_msg]
        Vc[at:at + self_len] = msgs_v[self_msg]
    Kr = rope(Kc, kv_pos, theta)

    p_rows = query_positions(n_q, self_len if self_msg >= 0 else n_q, s_self, q_pos)
    Qr = rope(np.asarray(q, dtype=np.float64), p_rows, theta)
    vis = visibility(n_q, n_parent, self_len)

    if rows is None:
        rows = range(n_q)
    rows = list(rows)
    out = np.zeros((len(rows), H_q, D), dtype=np.float64)
    lse = np.full((len(rows), H_q), -np.inf, dtype=np.float64)
    if N == 0 or not rows:
        return out, lse
    for h in range(H_q):
        kh = h // g
        S = scale * (Qr[rows, h, :] @ Kr[:, kh, :].T)            # [n_rows, N]
        S = np.where(vis[rows], S, -np.inf)
        mx = S.max(axis=1, keepdims=True)
        ok = np.isfinite(mx[:, 0])
        mx = np.where(np.isfinite(mx), mx, 0.0)
        P = np.exp(S - mx)
        den = P.sum(axis=1, keepdims=True)
        with np.errstate(divide="ignore", invalid="ignore"):
            o = (P @ Vc[:, kh, :]) / den
            l = mx[:, 0] + np.log(den[:, 0])
        out[:, h, :] = np.where(ok[:, None], o, 0.0)
        lse[:, h] = np.where(ok, l, -np.inf)
    return out, lse


# ---------------------------------------------------------------------------
# a batch of parallel calls (Sec. 2.4 "Parallel API Calls"): each call is
# independent and sees exactly what it lists; outputs are packed in call order.
# ---------------------------------------------------------------------------
def attend(msgs_k, msgs_v, calls, q, theta, scale=None):
    outs, lses, at = [], [], 0
    for c in calls:
        o, l = attend_call(msgs_k, msgs_v, c.sel, c.self_msg, c.self_start, c.n_q, c.q_pos,
                           q[at:at + c.n_q], theta, scale)
        outs.append(o)
        lses.append(l)
        at += c.n_q
    H_q, D = q.shape[1], q.shape[2]
    if not outs:
        return np.zeros((0, H_q, D)), np.zeros((0, H_q))
    return np.concatenate(outs, axis=0), np.concatenate(lses, axis=0)


def tables_for_call(call, lengths: Sequence[int], reserves: Sequence[int], align: int):
    """Canonical gather table / position map of one call under the cache layout
    rule with slot alignment `align` (bit-exact target for the library)."""
    sel_r, s_self = resolve_positions(call.sel, lengths, call.self_start)
    starts = slot_starts(reserves, align)
    kv_slot, kv_pos, _ = assemble(sel_r, call.self_msg, s_self, lengths, starts)
    return kv_slot, kv_pos


# ---------------------------------------------------------------------------
# merging attention over two disjoint key sets from (out, lse) pairs; the
# textbook log-sum-exp combination, used to check split attention.
# ---------------------------------------------------------------------------
def merge_partials(outs: Sequence[np.ndarray], lses: Sequence[np.ndarray]):
    lses = np.stack(lses)                                   # [S, ...]
    outs = np.stack(outs)                                   # [S, ..., D]
    mx = lses.max(axis=0)
    safe = np.where(np.isfinite(mx), mx, 0.0)
    w = np.exp(lses - safe)                                 # -inf -> 0
    den = w.sum(axis=0)
    with np.errstate(divide="ignore", invalid="ignore"):
        o = (w[..., None] * outs).sum(axis=0) / den[..., None]
        l = safe + np.log(den)
    ok = den > 0
    return np.where(ok[..., None], o, 0.0), np.where(ok, l, -np.inf)


# ---------------------------------------------------------------------------
# gradient of one call (Sec. 2.4: during fine-tuning a position update is applied
# non-destructively so that gradients flow through it to the cached keys; the
# gradient with respect to the UNROTATED keys, the values and the queries is what a
# training graph needs).  The chain rule of attend_call written out step by step on
# the same dense matrices: for the scalar  sum(out * d_out),
#   dV_c = P^T dO,  dP = dO V_c^T,  dS = P * (dP - rowsum(dO * O)),
#   dQr = scale dS Kr,  dKr = scale dS^T Qr,
# a rotation's transpose is the rotation by the opposite angle, and a token gathered
# several times (by several list entries, or by parent and new message both) collects
# the sum of its copies' gradients.
# ---------------------------------------------------------------------------
def attend_call_backward(msgs_k: Sequence[np.ndarray], msgs_v: Sequence[np.ndarray],
                         sel: Sequence[Tuple[int, int]], self_msg: int, self_start: int,
                         n_q: int, q_pos: Optional[np.ndarray], q: np.ndarray, d_out: np.ndarray,
                         theta: float, scale: Optional[float] = None):
    """Returns (d_q [n_q, H_q, D], d_k, d_v) with d_k[m], d_v[m]: [L_m, H_kv, D] for every
    message (zeros where the call does not read it), all fp64."""
    lengths = [int(k.shape[0]) for k in msgs_k]
    sel_r, s_self = resolve_positions(sel, lengths, self_start)
    self_len = lengths[self_msg] if self_msg >= 0 else 0
    starts = slot_starts(lengths, 1)
    kv_slot, kv_pos, n_parent = assemble(sel_r, self_msg, s_self, lengths, starts)
    H_kv, D = msgs_k[0].shape[1], msgs_k[0].shape[2]
    H_q = q.shape[1]
    g = H_q // H_kv
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    d_k = [np.zeros((L, H_kv, D)) for L in lengths]
    d_v = [np.zeros((L, H_kv, D)) for L in lengths]
    d_q = np.zeros((n_q, H_q, D))
    N = kv_slot.shape[0]
    if N == 0:
        return d_q, d_k, d_v
    entries = list(sel_r) + ([(self_msg, s_self)] if self_msg >= 0 else [])
    Kc = np.concatenate([np.asarray(msgs_k[m], dtype=np.float64) for m, _ in entries], axis=0)
    Vc = np.concatenate([np.asarray(msgs_v[m], dtype=np.float64) for m, _ in entries], axis=0)
    Kr = rope(Kc, kv_pos, theta)
    p_rows = query_positions(n_q, self_len if self_msg >= 0 else n_q, s_self, q_pos)
    Qr = rope(np.asarray(q, dtype=np.float64), p_rows, theta)
    vis = visibility(n_q, n_parent, self_len)
    dO = np.asarray(d_out, dtype=np.float64)
    dQr = np.zeros_like(Qr)
    dKr = np.zeros_like(Kr)
    dVc = np.zeros_like(Vc)
    for h in range(H_q):
        kh = h // g
        S = np.where(vis, scale * (Qr[:, h, :] @ Kr[:, kh, :].T), -np.inf)
        mx = S.max(axis=1, keepdims=True)
        ok = np.isfinite(mx[:, 0])
        P = np.exp(S - np.where(np.isfinite(mx), mx, 0.0))
        den = P.sum(axis=1, keepdims=True)
        with np.errstate(divide="ignore", invalid="ignore"):
            P = np.where(ok[:, None], P / den, 0.0)          # a row that sees nothing contributes nothing
        O = P @ Vc[:, kh, :]
        dVc[:, kh, :] += P.T @ dO[:, h, :]
        dP = dO[:, h, :] @ Vc[:, kh, :].T
        dS = P * (dP - (dO[:, h, :] * O).sum(axis=1, keepdims=True))
        dQr[:, h, :] = scale * (dS @ Kr[:, kh, :])
        dKr[:, kh, :] += scale * (dS.T @ Qr[:, h, :])
    d_q = rope(dQr, -np.asarray(p_rows), theta)
    dKc = rope(dKr, -np.asarray(kv_pos), theta)
    at = 0
    for m, _ in entries:
        L = lengths[m]
        d_k[m] += dKc[at:at + L]
        d_v[m] += dVc[at:at + L]
        at += L
    return d_q, d_k, d_v
