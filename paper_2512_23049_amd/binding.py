"""ctypes binding of libpc.so: argument marshalling only.

Function names match include/pc.h.  Tensors are passed as raw device pointers
(``tensor.data_ptr()``); PyTorch is used by callers for device memory and
streams only.  Loading fails loudly if the library has not been built
(``python -m paper_2512_23049_amd.build``): there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpc.so")

PC_OK = 0
PC_ERR_INVALID_ARG, PC_ERR_BAD_MSG_ID, PC_ERR_NO_SPACE, PC_ERR_SHAPE, PC_ERR_HIP = -1, -2, -3, -4, -5
PC_F32, PC_BF16 = 0, 1
PC_POS_AUTO = -(2 ** 31)
PC_SLOT_ALIGN = 32
PC_FLAG_HOST_ONLY = 1
PC_FLAG_GROW_EXTENTS = 2
PC_N_KERNEL_CLASSES = 9
KERNEL_CLASSES = ("append", "plan", "prefill", "decode", "merge", "attend_f32", "expand", "reposition", "gather")


class pc_config(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("dtype", C.c_int32), ("rope_theta", C.c_float), ("softmax_scale", C.c_float),
                ("capacity_tokens", C.c_int64), ("max_messages", C.c_int32),
                ("max_position", C.c_int32), ("flags", C.c_uint32),
                ("arena", C.c_void_p), ("arena_bytes", C.c_size_t)]


class pc_sel(C.Structure):
    _fields_ = [("msg_id", C.c_int32), ("start_pos", C.c_int32)]


class pc_call(C.Structure):
    _fields_ = [("sel", C.POINTER(pc_sel)), ("n_sel", C.c_int32), ("self_msg", C.c_int32),
                ("self_start", C.c_int32), ("n_q", C.c_int32), ("q_pos", C.POINTER(C.c_int32))]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2512_23049_amd.build` (no fallback exists)")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.pc_cache_storage_bytes.restype = C.c_size_t
        L.pc_cache_storage_bytes.argtypes = [C.POINTER(pc_config)]
        L.pc_cache_create.restype = i32
        L.pc_cache_create.argtypes = [C.POINTER(pc_config), C.POINTER(vp)]
        L.pc_cache_destroy.restype = i32
        L.pc_cache_destroy.argtypes = [vp]
        L.pc_last_error.restype = C.c_char_p
        L.pc_last_error.argtypes = [vp]
        L.pc_append_message.restype = i32
        L.pc_append_message.argtypes = [vp, vp, vp, i32, i32, C.POINTER(i32), vp]
        L.pc_append_messages.restype = i32
        L.pc_append_messages.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(vp), C.POINTER(i32), C.POINTER(i32),
                                         C.POINTER(i32), vp]
        L.pc_append_tokens.restype = i32
        L.pc_append_tokens.argtypes = [vp, i32, vp, vp, i32, vp]
        L.pc_append_tokens_batch.restype = i32
        L.pc_append_tokens_batch.argtypes = [vp, C.POINTER(i32), i32, vp, vp, vp]
        L.pc_attend.restype = i32
        L.pc_attend.argtypes = [vp, C.POINTER(pc_call), i32, vp, vp, vp, vp]
        L.pc_decode_step.restype = i32
        L.pc_decode_step.argtypes = [vp, C.POINTER(i32), i32, vp, vp, C.POINTER(pc_call), i32, vp, vp, vp, vp]
        L.pc_attend_static.restype = i32
        L.pc_attend_static.argtypes = [vp, C.POINTER(pc_call), i32, vp, vp, vp, vp]
        L.pc_build_tables.restype = i32
        L.pc_build_tables.argtypes = [vp, C.POINTER(pc_call), vp, vp, i64, C.POINTER(i64), vp]
        L.pc_resolve_call.restype = i32
        L.pc_resolve_call.argtypes = [vp, C.POINTER(pc_call), C.POINTER(i32), C.POINTER(i32), C.POINTER(i64)]
        L.pc_message_info.restype = i32
        L.pc_message_info.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i64), C.POINTER(i32)]
        L.pc_message_extents.restype = i32
        L.pc_message_extents.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i64), C.POINTER(i32), i32]
        L.pc_message_free.restype = i32
        L.pc_message_free.argtypes = [vp, i32]
        L.pc_message_base.restype = i32
        L.pc_message_base.argtypes = [vp, i32, C.POINTER(i32)]
        L.pc_reposition.restype = i32
        L.pc_reposition.argtypes = [vp, i32, i32, vp]
        L.pc_reposition_batch.restype = i32
        L.pc_reposition_batch.argtypes = [vp, C.POINTER(i32), C.POINTER(i32), i32, vp]
        L.pc_cache_info.restype = i32
        L.pc_cache_info.argtypes = [vp, C.POINTER(i32), C.POINTER(i64), C.POINTER(i64)]
        L.pc_profile_enable.restype = i32
        L.pc_profile_enable.argtypes = [vp, i32]
        L.pc_profile_read.restype = i32
        L.pc_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64), i32]
        L.pc_set_tuning.restype = i32
        L.pc_set_tuning.argtypes = [vp, i32, i32]
        L.pc_message_swap_bytes.restype = i64
        L.pc_message_swap_bytes.argtypes = [vp, i32]
        L.pc_message_swap_out.restype = i32
        L.pc_message_swap_out.argtypes = [vp, i32, vp, vp]
        L.pc_message_swap_in.restype = i32
        L.pc_message_swap_in.argtypes = [vp, i32, vp, vp]
        L.pc_attend_backward.restype = i32
        L.pc_attend_backward.argtypes = [vp, C.POINTER(pc_call), i32, vp, vp, vp, vp, vp, vp, vp]
        L.pc_grad_keys_finalize.restype = i32
        L.pc_grad_keys_finalize.argtypes = [vp, vp, vp]
        L.pc_set_decode_sharing.restype = i32
        L.pc_set_decode_sharing.argtypes = [vp, i32]
        L.pc_set_key_gather.restype = i32
        L.pc_set_key_gather.argtypes = [vp, i32]
        _lib = L
    return _lib


class PcError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"pc error {code}: {msg}")
        self.code = code


def marshal_calls(calls: Sequence):
    """calls: objects with .sel [(msg, start)], .self_msg, .self_start, .n_q, .q_pos.
    Returns (ctypes array of pc_call, keep-alive list)."""
    arr = (pc_call * max(len(calls), 1))()
    keep = []
    for i, c in enumerate(calls):
        n = len(c.sel)
        sel = (pc_sel * max(n, 1))()
        for e, (m, s) in enumerate(c.sel):
            sel[e].msg_id, sel[e].start_pos = int(m), int(s)
        keep.append(sel)
        arr[i].sel = C.cast(sel, C.POINTER(pc_sel))
        arr[i].n_sel = n
        arr[i].self_msg = int(c.self_msg)
        arr[i].self_start = int(c.self_start)
        arr[i].n_q = int(c.n_q)
        if c.q_pos is not None:
            qp = (C.c_int32 * len(c.q_pos))(*[int(x) for x in c.q_pos])
            keep.append(qp)
            arr[i].q_pos = C.cast(qp, C.POINTER(C.c_int32))
        else:
            arr[i].q_pos = None
    return arr, keep


class Cache:
    """Thin owner of a pc_cache handle; every method is one C call."""

    def __init__(self, n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: int, rope_theta: float,
                 capacity_tokens: int, max_messages: int, max_position: int = 0,
                 softmax_scale: float = 0.0, flags: int = 0, arena: int = 0, arena_bytes: int = 0):
        self.cfg = pc_config(n_q_heads, n_kv_heads, head_dim, dtype, rope_theta, softmax_scale,
                             capacity_tokens, max_messages, max_position, flags,
                             arena or None, arena_bytes)
        self.h = C.c_void_p()
        rc = lib().pc_cache_create(C.byref(self.cfg), C.byref(self.h))
        if rc != PC_OK:
            self.h = None
            raise PcError(rc, "pc_cache_create failed")

    def _check(self, rc: int):
        if rc != PC_OK:
            raise PcError(rc, lib().pc_last_error(self.h).decode())

    def close(self):
        if self.h:
            lib().pc_cache_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def append_message(self, k_ptr: int, v_ptr: int, length: int, reserve: int = 0, stream: int = 0) -> int:
        mid = C.c_int32(-1)
        self._check(lib().pc_append_message(self.h, k_ptr, v_ptr, length, reserve, C.byref(mid), stream or None))
        return mid.value

    def attend(self, calls, q_ptr: int, out_ptr: int, lse_ptr: int = 0, stream: int = 0, marshalled=None):
        arr, keep = marshalled if marshalled is not None else marshal_calls(calls)
        self._check(lib().pc_attend(self.h, arr, len(calls), q_ptr or None, out_ptr or None,
                                    lse_ptr or None, stream or None))

    def decode_step(self, msg_ids, k_ptr: int, v_ptr: int, calls, q_ptr: int, out_ptr: int, lse_ptr: int = 0,
                    stream: int = 0, marshalled=None):
        """One token for each of msg_ids, then the batch of calls, in one library call."""
        ids = (C.c_int32 * max(len(msg_ids), 1))(*[int(m) for m in msg_ids])
        arr, keep = marshalled if marshalled is not None else marshal_calls(calls)
        self._check(lib().pc_decode_step(self.h, ids, len(msg_ids), k_ptr or None, v_ptr or None, arr, len(calls),
                                         q_ptr or None, out_ptr or None, lse_ptr or None, stream or None))

    def attend_static(self, calls, q_ptr: int, out_ptr: int, lse_ptr: int = 0, stream: int = 0, marshalled=None):
        arr, keep = marshalled if marshalled is not None else marshal_calls(calls)
        self._check(lib().pc_attend_static(self.h, arr, len(calls), q_ptr or None, out_ptr or None,
                                           lse_ptr or None, stream or None))

    def build_tables(self, call, kv_slot_ptr: int, kv_pos_ptr: int, cap: int, stream: int = 0) -> int:
        arr, keep = marshal_calls([call])
        n = C.c_int64(0)
        self._check(lib().pc_build_tables(self.h, arr, kv_slot_ptr or None, kv_pos_ptr or None, cap,
                                          C.byref(n), stream or None))
        return n.value

    def resolve_call(self, call):
        arr, keep = marshal_calls([call])
        starts = (C.c_int32 * max(len(call.sel), 1))()
        s_self, n = C.c_int32(0), C.c_int64(0)
        self._check(lib().pc_resolve_call(self.h, arr, starts, C.byref(s_self), C.byref(n)))
        return [starts[i] for i in range(len(call.sel))], s_self.value, n.value

    def message_info(self, msg_id: int):
        ln, st, rs = C.c_int32(0), C.c_int64(0), C.c_int32(0)
        self._check(lib().pc_message_info(self.h, msg_id, C.byref(ln), C.byref(st), C.byref(rs)))
        return ln.value, st.value, rs.value

    def append_messages(self, k_ptrs, v_ptrs, lengths, reserves=None, stream: int = 0):
        n = len(lengths)
        ka = (C.c_void_p * max(n, 1))(*[int(p) if p else None for p in k_ptrs])
        va = (C.c_void_p * max(n, 1))(*[int(p) if p else None for p in v_ptrs])
        la = (C.c_int32 * max(n, 1))(*[int(x) for x in lengths])
        ra = (C.c_int32 * max(n, 1))(*[int(x) for x in (reserves or [0] * n)])
        ids = (C.c_int32 * max(n, 1))()
        self._check(lib().pc_append_messages(self.h, n, ka, va, la, ra, ids, stream))
        return [ids[i] for i in range(n)]

    def append_tokens(self, msg_id: int, k_ptr: int, v_ptr: int, n: int, stream: int = 0):
        self._check(lib().pc_append_tokens(self.h, msg_id, k_ptr, v_ptr, n, stream))

    def append_tokens_batch(self, msg_ids, k_ptr: int, v_ptr: int, stream: int = 0):
        arr = (C.c_int32 * max(len(msg_ids), 1))(*[int(m) for m in msg_ids])
        self._check(lib().pc_append_tokens_batch(self.h, arr, len(msg_ids), k_ptr, v_ptr, stream))

    def message_free(self, msg_id: int):
        self._check(lib().pc_message_free(self.h, msg_id))

    def message_base(self, msg_id: int) -> int:
        b = C.c_int32(0)
        self._check(lib().pc_message_base(self.h, msg_id, C.byref(b)))
        return b.value

    def reposition(self, msg_id: int, new_base: int, stream: int = 0):
        self._check(lib().pc_reposition(self.h, msg_id, new_base, stream))

    def reposition_batch(self, msg_ids, new_bases, stream: int = 0):
        n = len(msg_ids)
        ids = (C.c_int32 * max(n, 1))(*[int(m) for m in msg_ids])
        bases = (C.c_int32 * max(n, 1))(*[int(b) for b in new_bases])
        self._check(lib().pc_reposition_batch(self.h, ids, bases, n, stream))

    def cache_info(self):
        n, used, cap = C.c_int32(0), C.c_int64(0), C.c_int64(0)
        self._check(lib().pc_cache_info(self.h, C.byref(n), C.byref(used), C.byref(cap)))
        return n.value, used.value, cap.value

    def profile_enable(self, on: bool):
        self._check(lib().pc_profile_enable(self.h, 1 if on else 0))

    def profile_read(self, reset: bool = True):
        ms = (C.c_double * PC_N_KERNEL_CLASSES)()
        n = (C.c_int64 * PC_N_KERNEL_CLASSES)()
        self._check(lib().pc_profile_read(self.h, ms, n, 1 if reset else 0))
        return {KERNEL_CLASSES[i]: (ms[i], n[i]) for i in range(PC_N_KERNEL_CLASSES)}

    def set_tuning(self, decode_tiles_per_split: int = 0, prefill_tiles_per_split: int = 0):
        self._check(lib().pc_set_tuning(self.h, decode_tiles_per_split, prefill_tiles_per_split))

    def message_swap_bytes(self, msg: int) -> int:
        n = lib().pc_message_swap_bytes(self.h, msg)
        if n < 0:
            self._check(int(n))
        return int(n)

    def message_swap_out(self, msg: int, blob_ptr: int, stream: int = 0):
        self._check(lib().pc_message_swap_out(self.h, msg, blob_ptr or None, stream or None))

    def message_swap_in(self, msg: int, blob_ptr: int, stream: int = 0):
        self._check(lib().pc_message_swap_in(self.h, msg, blob_ptr or None, stream or None))

    def attend_backward(self, calls, q_ptr: int, lse_ptr: int, d_out_ptr: int, d_q_ptr: int, d_k_ptr: int, d_v_ptr: int,
                        stream: int = 0):
        arr, keep = marshal_calls(calls)
        self._check(lib().pc_attend_backward(self.h, arr, len(calls), q_ptr or None, lse_ptr or None, d_out_ptr or None,
                                             d_q_ptr or None, d_k_ptr or None, d_v_ptr or None, stream or None))

    def grad_keys_finalize(self, d_k_ptr: int, stream: int = 0):
        self._check(lib().pc_grad_keys_finalize(self.h, d_k_ptr or None, stream or None))

    def message_extents(self, msg: int, cap: int = 64):
        """[(slot_start, len), ...] of the message's extents in token order."""
        n = C.c_int32(0)
        starts, lens = (C.c_int64 * cap)(), (C.c_int32 * cap)()
        self._check(lib().pc_message_extents(self.h, msg, C.byref(n), starts, lens, cap))
        return [(int(starts[i]), int(lens[i])) for i in range(min(cap, n.value))]

    def set_key_gather(self, mode: int = 0):
        """0: prefill calls with enough rows read keys from a copy turned to their positions; 1: never; 2: always."""
        self._check(lib().pc_set_key_gather(self.h, mode))

    def set_decode_sharing(self, mode: int = 0):
        """0: shared walk when a group's calls overlap enough; 1: never; 2: whenever the shape allows."""
        self._check(lib().pc_set_decode_sharing(self.h, mode))
