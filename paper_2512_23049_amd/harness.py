"""Drives a generated workload through the C ABI on the GPU (tests, bench, smoke).

Uses torch for device tensors and the current stream only; every step of the
method runs inside libpc.so.
"""
from __future__ import annotations

import numpy as np
import torch

from .binding import PC_BF16, PC_F32, Cache, marshal_calls


def torch_dtype(name: str):
    return torch.bfloat16 if name == "bf16" else torch.float32


def to_device(x: np.ndarray, dtype_name: str, device="cuda:0") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x)).to(device=device, dtype=torch_dtype(dtype_name))


def make_cache(w, slack_tokens: int = 0, extra_messages: int = 0, **kw) -> Cache:
    reserves = w.message_reserves()
    cap = sum(((r + 31) // 32) * 32 for r in reserves) + 32 + slack_tokens
    return Cache(w.n_q_heads, w.n_kv_heads, w.head_dim, PC_BF16 if w.dtype == "bf16" else PC_F32,
                 w.rope_theta, cap, max(len(reserves), 1) + 8 + extra_messages, **kw)


class DeviceWorkload:
    """All tensors of a workload resident on the GPU, calls marshalled once."""

    def __init__(self, w, device="cuda:0"):
        self.w = w
        self.steps = []
        for e in w.events:
            if e.kind == "append":
                self.steps.append(("append", to_device(e.k, w.dtype, device), to_device(e.v, w.dtype, device),
                                   int(e.k.shape[0]), int(e.reserve)))
            elif e.kind == "extend":
                self.steps.append(("extend", to_device(e.k, w.dtype, device), to_device(e.v, w.dtype, device),
                                   list(e.msgs)))
            else:
                q = to_device(e.q, w.dtype, device)
                out = torch.empty_like(q)
                lse = torch.empty(q.shape[:2], dtype=torch.float32, device=device)
                self.steps.append(("attend", e.calls, marshal_calls(e.calls), q, out, lse))

    def run(self, cache: Cache, stream: int = 0, want_lse: bool = True, batch_appends: bool = False,
            fused_steps: bool = False):
        """One pass over all events; returns the list of (out, lse) of the attend events.
        batch_appends: consecutive append events go through one pc_append_messages call.
        fused_steps: an extend event followed by an attend event goes through one pc_decode_step call."""
        res = []
        pending = []
        held = None                                       # an extend step waiting for its attend

        def flush():
            if pending:
                cache.append_messages([p[1].data_ptr() for p in pending], [p[2].data_ptr() for p in pending],
                                      [p[3] for p in pending], [p[4] for p in pending], stream)
                pending.clear()
        for s in self.steps:
            if s[0] == "append" and held is not None:
                cache.append_tokens_batch(held[3], held[1].data_ptr(), held[2].data_ptr(), stream)
                held = None
            if s[0] == "append" and batch_appends:
                pending.append(s)
                continue
            flush()
            if s[0] == "append":
                cache.append_message(s[1].data_ptr(), s[2].data_ptr(), s[3], s[4], stream)
            elif s[0] == "extend":
                if held is not None:
                    cache.append_tokens_batch(held[3], held[1].data_ptr(), held[2].data_ptr(), stream)
                    held = None
                if fused_steps:
                    held = s
                else:
                    cache.append_tokens_batch(s[3], s[1].data_ptr(), s[2].data_ptr(), stream)
            else:
                _, calls, m, q, out, lse = s
                if held is not None:
                    cache.decode_step(held[3], held[1].data_ptr(), held[2].data_ptr(), calls, q.data_ptr(), out.data_ptr(),
                                      lse.data_ptr() if want_lse else 0, stream, m)
                    held = None
                else:
                    cache.attend(calls, q.data_ptr(), out.data_ptr(), lse.data_ptr() if want_lse else 0, stream, m)
                res.append((out, lse))
        flush()
        if held is not None:
            cache.append_tokens_batch(held[3], held[1].data_ptr(), held[2].data_ptr(), stream)
        return res

    def run_attends_only(self, cache: Cache, stream: int = 0, want_lse: bool = False):
        for s in self.steps:
            if s[0] == "attend":
                _, calls, m, q, out, lse = s
                cache.attend(calls, q.data_ptr(), out.data_ptr(), lse.data_ptr() if want_lse else 0, stream, m)
