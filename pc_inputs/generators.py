"""Seeded workload generators (plain data only, no method arithmetic).

Every generator returns a :class:`Workload`: model shape, dtype name, RoPE
base, and an ordered list of events.  An ``append`` event carries one
message's unrotated K and V (``float32`` arrays whose values are exactly
representable in the workload dtype); an ``extend`` event carries one more token
for each of a list of messages (decode tails growing in step); an ``attend``
event carries a batch of calls and the packed query rows.  Random numbers come from
``numpy.random.default_rng(seed)`` and are drawn in the order the code reads.

The five named workloads mirror the *shapes* of the multi-agent workflows the
paper evaluates (shared system prompt, branches read by all voters, agents
re-reading each other's rounds, overlapped parents); they stand in for the
benchmark the paper ran on, none of whose items appear here.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

POS_AUTO = -(2 ** 31)  # "place right after the preceding list entry"


@dataclass
class Call:
    sel: List[Tuple[int, int]]            # (msg_id, start_pos) in list order
    self_msg: int = -1                    # id of the already appended new message, or -1
    self_start: int = POS_AUTO
    n_q: int = 0                          # query rows, aligned with the last n_q self tokens
    q_pos: Optional[np.ndarray] = None    # int32[n_q] or None (= self_start + token index)


@dataclass
class Event:
    kind: str                             # "append" | "extend" | "attend"
    k: Optional[np.ndarray] = None        # append: [L, H_kv, D] float32; extend: [n_msgs, H_kv, D]
    v: Optional[np.ndarray] = None
    msgs: Optional[List[int]] = None      # extend: message i of the list gets token row i
    reserve: int = 0                      # append: slots to reserve (0 = len)
    calls: Optional[List[Call]] = None    # attend
    q: Optional[np.ndarray] = None        # attend: [sum n_q, H_q, D] float32


@dataclass
class Workload:
    name: str
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str                            # "f32" | "bf16"
    rope_theta: float
    events: List[Event] = field(default_factory=list)

    @property
    def n_messages(self) -> int:
        return sum(1 for e in self.events if e.kind == "append")

    def message_lengths(self, upto_event: Optional[int] = None) -> List[int]:
        """Token counts after the first `upto_event` events (all events if None)."""
        lens: List[int] = []
        for i, e in enumerate(self.events):
            if upto_event is not None and i >= upto_event:
                break
            if e.kind == "append":
                lens.append(int(e.k.shape[0]))
            elif e.kind == "extend":
                for m in e.msgs:
                    lens[m] += 1
        return lens

    def message_reserves(self) -> List[int]:
        return [int(max(e.reserve, e.k.shape[0])) for e in self.events if e.kind == "append"]


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); returns float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + bias) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return r.view(np.float32)


def _normal(rng: np.random.Generator, shape: Sequence[int], dtype: str) -> np.ndarray:
    x = rng.standard_normal(size=tuple(shape), dtype=np.float32)
    return round_to_bf16(x) if dtype == "bf16" else x


def _append(w: Workload, rng, length: int, reserve: int = 0) -> int:
    k = _normal(rng, (length, w.n_kv_heads, w.head_dim), w.dtype)
    v = _normal(rng, (length, w.n_kv_heads, w.head_dim), w.dtype)
    w.events.append(Event("append", k=k, v=v, reserve=reserve))
    return w.n_messages - 1


def _extend(w: Workload, rng, msgs: List[int]) -> None:
    k = _normal(rng, (len(msgs), w.n_kv_heads, w.head_dim), w.dtype)
    v = _normal(rng, (len(msgs), w.n_kv_heads, w.head_dim), w.dtype)
    w.events.append(Event("extend", k=k, v=v, msgs=list(msgs)))


def _attend(w: Workload, rng, calls: List[Call]) -> None:
    total_q = sum(c.n_q for c in calls)
    q = _normal(rng, (total_q, w.n_q_heads, w.head_dim), w.dtype)
    w.events.append(Event("attend", calls=calls, q=q))


# --------------------------------------------------------------------------
# config 1: tiny fp32, one call, shuffled list, one gap of 10, one overlap of 8
# --------------------------------------------------------------------------
def tiny_fp32(seed: int = 1) -> Workload:
    rng = np.random.default_rng(seed)
    w = Workload("tiny_fp32", 4, 2, 64, "f32", 10000.0)
    lens = [int(x) for x in rng.integers(16, 65, size=8)]
    for L in lens:
        _append(w, rng, L)
    new_id = _append(w, rng, 32)
    a, b, c, d = [int(x) for x in rng.permutation(8)[:4]]
    s_a = 0
    s_b = s_a + lens[a] + 10
    s_c = s_b + lens[b] - 8
    s_d = s_c + lens[c]
    placed = [(a, s_a), (b, s_b), (c, s_c), (d, s_d)]
    order = rng.permutation(4)
    sel = [placed[int(i)] for i in order]
    self_start = s_d + lens[d]
    q_pos = (self_start + np.arange(32)).astype(np.int32)
    _attend(w, rng, [Call(sel, new_id, self_start, 32, q_pos)])
    return w


# --------------------------------------------------------------------------
# config 2: single-call prefill, 8B-shaped attention, bf16
# --------------------------------------------------------------------------
def single_prefill(seed: int = 2, n_msgs: int = 256, len_lo: int = 64, len_hi: int = 1024,
                   n_sel: int = 16, n_new: int = 512, n_q_heads: int = 32, n_kv_heads: int = 8,
                   head_dim: int = 128, dtype: str = "bf16") -> Workload:
    rng = np.random.default_rng(seed)
    w = Workload("single_prefill", n_q_heads, n_kv_heads, head_dim, dtype, 500000.0)
    lens = [int(x) for x in rng.integers(len_lo, len_hi + 1, size=n_msgs)]
    for L in lens:
        _append(w, rng, L)
    new_id = _append(w, rng, n_new)
    chosen = [int(x) for x in rng.permutation(n_msgs)[:n_sel]]
    sel = []
    s = int(rng.integers(0, 65))
    for m in chosen:
        sel.append((m, s))
        s = s + lens[m] + int(rng.integers(0, 129))
    _attend(w, rng, [Call(sel, new_id, s, n_new, None)])
    return w


# --------------------------------------------------------------------------
# config 3: parallel decode, shared system message + 8 pool messages + own tail
# --------------------------------------------------------------------------
def parallel_decode(seed: int = 3, n_calls: int = 64, sys_len: int = 2048, n_pool: int = 512,
                    len_lo: int = 128, len_hi: int = 512, n_sel: int = 8, tail_len: int = 64,
                    n_q_heads: int = 32, n_kv_heads: int = 8, head_dim: int = 128,
                    dtype: str = "bf16") -> Workload:
    rng = np.random.default_rng(seed)
    w = Workload("parallel_decode", n_q_heads, n_kv_heads, head_dim, dtype, 500000.0)
    _append(w, rng, sys_len)
    lens = {0: sys_len}
    pool = []
    for L in rng.integers(len_lo, len_hi + 1, size=n_pool):
        m = _append(w, rng, int(L))
        lens[m] = int(L)
        pool.append(m)
    tails = [_append(w, rng, tail_len, reserve=tail_len) for _ in range(n_calls)]
    calls = []
    for c in range(n_calls):
        picks = [pool[int(i)] for i in rng.permutation(n_pool)[:n_sel]]
        sel = [(0, 0)]
        s = sys_len
        for m in picks:
            s += int(rng.integers(0, 33))
            sel.append((m, s))
            s += lens[m]
        calls.append(Call(sel, tails[c], s, 1, None))
    _attend(w, rng, calls)
    return w


# --------------------------------------------------------------------------
# config 4: multi-agent rounds, append and prefill interleaved
# --------------------------------------------------------------------------
def multi_agent_rounds(seed: int = 4, n_agents: int = 8, n_rounds: int = 6, msg_len: int = 256,
                       n_q_heads: int = 32, n_kv_heads: int = 8, head_dim: int = 128,
                       dtype: str = "bf16") -> Workload:
    rng = np.random.default_rng(seed)
    w = Workload("multi_agent_rounds", n_q_heads, n_kv_heads, head_dim, dtype, 500000.0)
    ids = [[-1] * n_agents for _ in range(n_rounds)]      # ids[r][a]
    for r in range(n_rounds):
        for a in range(n_agents):
            ids[r][a] = _append(w, rng, msg_len)
        calls = []
        for a in range(n_agents):
            others = [ids[rr][aa] for rr in range(r) for aa in range(n_agents) if aa != a]
            perm = rng.permutation(len(others)) if others else []
            sel = [(others[int(i)], POS_AUTO) for i in perm]
            sel += [(ids[rr][a], POS_AUTO) for rr in range(r)]
            calls.append(Call(sel, ids[r][a], POS_AUTO, msg_len, None))
        _attend(w, rng, calls)
    return w


# --------------------------------------------------------------------------
# The attention work a prefix-caching baseline does for the same rounds (Sec. 3.1 "A
# Baseline Approach", Sec. 5 "Performance"): an agent's prompt keeps its own earlier
# prompt as a cached prefix, but the messages the OTHER agents wrote in the last round
# are new text in it and are encoded again, followed by its own new message.  So in
# round r agent a appends one chunk of (n_agents - 1) * msg_len re-encoded tokens plus
# msg_len new ones (round 0: only its own msg_len) and all of them are causal query rows
# over the agent's private prefix.  Only shapes matter here; values are random.
# --------------------------------------------------------------------------
def prefix_cache_baseline_rounds(seed: int = 7, n_agents: int = 8, n_rounds: int = 6, msg_len: int = 256,
                                 n_q_heads: int = 32, n_kv_heads: int = 8, head_dim: int = 128,
                                 dtype: str = "bf16") -> Workload:
    rng = np.random.default_rng(seed)
    w = Workload("prefix_cache_baseline_rounds", n_q_heads, n_kv_heads, head_dim, dtype, 500000.0)
    chunks = [[] for _ in range(n_agents)]                 # message ids of each agent's private prompt
    for r in range(n_rounds):
        n_new = msg_len if r == 0 else n_agents * msg_len
        new_ids = [_append(w, rng, n_new) for _ in range(n_agents)]
        calls = [Call([(m, POS_AUTO) for m in chunks[a]], new_ids[a], POS_AUTO, n_new, None) for a in range(n_agents)]
        _attend(w, rng, calls)
        for a in range(n_agents):
            chunks[a].append(new_ids[a])
    return w


# --------------------------------------------------------------------------
# config 5: long-context 70B-shaped, 32 decode calls + one causal prefill
# --------------------------------------------------------------------------
def long_context(seed: int = 5, n_msgs: int = 512, len_lo: int = 64, len_hi: int = 256,
                 target_tokens: int = 65536, n_decode: int = 32, n_prefill_q: int = 2048,
                 n_q_heads: int = 64, n_kv_heads: int = 8, head_dim: int = 128,
                 dtype: str = "bf16") -> Workload:
    rng = np.random.default_rng(seed)
    w = Workload("long_context", n_q_heads, n_kv_heads, head_dim, dtype, 500000.0)
    lens = [int(x) for x in rng.integers(len_lo, len_hi + 1, size=n_msgs)]
    for L in lens:
        _append(w, rng, L)
    tails = [_append(w, rng, 1, reserve=1) for _ in range(n_decode)]
    new_id = _append(w, rng, n_prefill_q) if n_prefill_q > 0 else -1
    calls = []
    for c in range(n_decode + (1 if n_prefill_q > 0 else 0)):
        perm = rng.permutation(n_msgs)
        sel, s, tot = [], 0, 0
        for i in perm:
            m = int(i)
            sel.append((m, s))
            tot += lens[m]
            if tot >= target_tokens:
                s += lens[m]
                break
            s += lens[m] - int(rng.integers(0, 33))
        else:
            s = sel[-1][1] + lens[sel[-1][0]]
        if c < n_decode:
            calls.append(Call(sel, tails[c], s, 1, None))
        else:
            calls.append(Call(sel, new_id, s, n_prefill_q, None))
    _attend(w, rng, calls)
    return w


# --------------------------------------------------------------------------
# parallel decode loop: the calls of config 3, but the tails start short and every
# step adds one token to each tail before the calls attend again (the decode phase
# of a workflow: Sec. 2.4, tails of parallel calls growing in step)
# --------------------------------------------------------------------------
def decode_loop(seed: int = 6, n_calls: int = 64, n_steps: int = 63, sys_len: int = 2048, n_pool: int = 512,
                len_lo: int = 128, len_hi: int = 512, n_sel: int = 8, tail0: int = 1,
                n_q_heads: int = 32, n_kv_heads: int = 8, head_dim: int = 128,
                dtype: str = "bf16") -> Workload:
    rng = np.random.default_rng(seed)
    w = Workload("decode_loop", n_q_heads, n_kv_heads, head_dim, dtype, 500000.0)
    _append(w, rng, sys_len)
    lens = {0: sys_len}
    pool = []
    for L in rng.integers(len_lo, len_hi + 1, size=n_pool):
        m = _append(w, rng, int(L))
        lens[m] = int(L)
        pool.append(m)
    tails = [_append(w, rng, tail0, reserve=tail0 + n_steps) for _ in range(n_calls)]
    layouts = []
    for c in range(n_calls):
        chosen = [pool[int(i)] for i in rng.permutation(n_pool)[:n_sel]]
        sel = [(0, 0)]
        s = sys_len
        for m in chosen:
            s += int(rng.integers(0, 33))
            sel.append((m, s))
            s += lens[m]
        layouts.append((sel, s))
    for step in range(n_steps + 1):
        if step > 0:
            _extend(w, rng, tails)
        _attend(w, rng, [Call(sel, tails[c], s, 1, None) for c, (sel, s) in enumerate(layouts)])
    return w


# --------------------------------------------------------------------------
# small randomised cases for parity tests: ragged lengths, repeats, AUTO and
# negative positions, explicit q_pos, calls without self or without parents
# --------------------------------------------------------------------------
def small_random(seed: int, dtype: str = "bf16", n_q_heads: int = 8, n_kv_heads: int = 2,
                 head_dim: int = 128, n_msgs: int = 12, len_lo: int = 1, len_hi: int = 150,
                 n_calls: int = 6, max_q: int = 70, theta: float = 10000.0) -> Workload:
    rng = np.random.default_rng(seed)
    w = Workload(f"small_random_{seed}", n_q_heads, n_kv_heads, head_dim, dtype, theta)
    lens = [int(x) for x in rng.integers(len_lo, len_hi + 1, size=n_msgs)]
    for L in lens:
        _append(w, rng, L, reserve=int(L + rng.integers(0, 40)) if rng.random() < 0.3 else 0)
    calls = []
    for c in range(n_calls):
        kind = c % 6
        n_sel = int(rng.integers(0, 7)) if kind != 3 else 0
        sel = []
        for _ in range(n_sel):
            m = int(rng.integers(0, n_msgs))                       # repeats allowed
            r = rng.random()
            if r < 0.3:
                s = POS_AUTO
            else:
                s = int(rng.integers(-3000, 70000))
            sel.append((m, s))
        if kind == 4:                                              # parents only, no self
            n_q = int(rng.integers(1, max_q + 1))
            q_pos = rng.integers(-100, 70000, size=n_q).astype(np.int32)
            if not sel:
                sel = [(int(rng.integers(0, n_msgs)), POS_AUTO)]
            calls.append(Call(sel, -1, POS_AUTO, n_q, q_pos))
            continue
        m_self = int(rng.integers(0, n_msgs))
        L = lens[m_self]
        if kind == 1:
            n_q = 1                                                # decode
        elif kind == 2:
            n_q = L                                                # full prefill
        else:
            n_q = int(rng.integers(1, min(L, max_q) + 1))          # chunked prefill
        n_q = min(n_q, L)
        self_start = POS_AUTO if rng.random() < 0.5 else int(rng.integers(-500, 70000))
        q_pos = None
        if kind == 5:
            q_pos = rng.integers(0, 70000, size=n_q).astype(np.int32)
        calls.append(Call(sel, m_self, self_start, n_q, q_pos))
    _attend(w, rng, calls)
    return w


_NAMED = {
    "tiny_fp32": tiny_fp32,
    "single_prefill": single_prefill,
    "parallel_decode": parallel_decode,
    "multi_agent_rounds": multi_agent_rounds,
    "long_context": long_context,
}


def make_workload(name: str, **kw) -> Workload:
    return _NAMED[name](**kw)
