"""CPU-side tests of the C-ABI library: it loads, exports every symbol the header
declares, and its host logic (allocator, validation, offset resolution) agrees with the
oracle's statement of the same rules.  Uses host-only caches: no GPU call is made."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import choreo_oracle as orc
from pc_inputs import POS_AUTO, Call, small_random

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def pc():
    import paper_2512_23049_amd as m
    if not os.path.exists(m.binding.LIB_PATH):
        from paper_2512_23049_amd import build
        build.build()
    return m


def host_cache(pc, **kw):
    args = dict(n_q_heads=8, n_kv_heads=2, head_dim=128, dtype=pc.PC_BF16, rope_theta=1e4,
                capacity_tokens=4096, max_messages=64, flags=pc.PC_FLAG_HOST_ONLY)
    args.update(kw)
    return pc.Cache(**args)


def test_every_declared_symbol_is_exported(pc):
    hdr = open(os.path.join(ROOT, "include", "pc.h")).read()
    names = set(re.findall(r"\b(pc_[a-z_]+)\s*\(", hdr))
    assert {"pc_cache_create", "pc_append_message", "pc_attend", "pc_build_tables"} <= names
    lib = ctypes.CDLL(pc.binding.LIB_PATH)
    for n in sorted(names):
        assert hasattr(lib, n), n


def test_header_constants_match_binding(pc):
    hdr = open(os.path.join(ROOT, "include", "pc.h")).read()
    assert int(re.search(r"#define PC_SLOT_ALIGN (\d+)", hdr).group(1)) == pc.PC_SLOT_ALIGN
    for name in ("PC_ERR_INVALID_ARG", "PC_ERR_BAD_MSG_ID", "PC_ERR_NO_SPACE", "PC_ERR_SHAPE", "PC_ERR_HIP"):
        assert int(re.search(r"#define %s\s+\((-\d+)\)" % name, hdr).group(1)) == getattr(pc, name)


def test_ids_are_sequential_and_slots_follow_the_layout_rule(pc):
    c = host_cache(pc)
    lens = [3, 32, 33, 1, 64, 100]
    reserves = [0, 0, 40, 70, 0, 0]
    ids = [c.append_message(0, 0, L, r) for L, r in zip(lens, reserves)]
    assert ids == list(range(len(lens)))
    eff = [max(L, r) for L, r in zip(lens, reserves)]
    exp = orc.slot_starts(eff, pc.PC_SLOT_ALIGN)
    for i, (L, r) in enumerate(zip(lens, eff)):
        assert c.message_info(i) == (L, exp[i], r)
    n, used, cap = c.cache_info()
    assert n == len(lens) and cap == 4096 and used % pc.PC_SLOT_ALIGN == 0 and used >= exp[-1] + 100


def test_capacity_and_table_limits(pc):
    c = host_cache(pc, capacity_tokens=100, max_messages=3)
    _, _, cap = c.cache_info()
    assert cap == 128                                     # rounded up to the slot alignment
    c.append_message(0, 0, 64)
    with pytest.raises(pc.PcError) as ei:
        c.append_message(0, 0, 65)                        # slots [64, 129) > 128
    assert ei.value.code == pc.PC_ERR_NO_SPACE
    c.append_message(0, 0, 10)
    c.append_message(0, 0, 10)
    with pytest.raises(pc.PcError) as ei:
        c.append_message(0, 0, 1)
    assert ei.value.code == pc.PC_ERR_NO_SPACE
    with pytest.raises(pc.PcError) as ei:
        c.append_message(0, 0, 0)
    assert ei.value.code == pc.PC_ERR_INVALID_ARG


def test_bad_configurations_are_rejected(pc):
    for kw in (dict(n_q_heads=6, n_kv_heads=4), dict(head_dim=96), dict(dtype=7), dict(capacity_tokens=0),
               dict(max_messages=0), dict(rope_theta=0.0), dict(dtype=pc.PC_BF16, head_dim=64)):
        with pytest.raises(pc.PcError):
            host_cache(pc, **kw)
    # the device path refuses to work without a GPU instead of falling back
    import torch
    if not torch.cuda.is_available():
        with pytest.raises(pc.PcError) as ei:
            pc.Cache(8, 2, 128, pc.PC_BF16, 1e4, 1024, 8)
        assert ei.value.code == pc.PC_ERR_HIP


def test_offset_resolution_matches_the_oracle_rule(pc):
    rng = np.random.default_rng(0)
    c = host_cache(pc)
    lens = [int(x) for x in rng.integers(1, 90, size=12)]
    for L in lens:
        c.append_message(0, 0, L)
    for trial in range(50):
        n_sel = int(rng.integers(0, 7))
        sel = [(int(rng.integers(0, 12)), POS_AUTO if rng.random() < 0.4 else int(rng.integers(-500, 500)))
               for _ in range(n_sel)]
        m_self = int(rng.integers(0, 12)) if rng.random() < 0.7 else -1
        s_self = POS_AUTO if rng.random() < 0.5 else int(rng.integers(-500, 500))
        call = Call(sel, m_self, s_self, 1, None)
        starts, got_self, n_kv = c.resolve_call(call)
        exp_sel, exp_self = orc.resolve_positions(sel, lens, s_self)
        assert starts == [s for _, s in exp_sel]
        assert got_self == exp_self
        assert n_kv == sum(lens[m] for m, _ in sel) + (lens[m_self] if m_self >= 0 else 0)
        assert c.build_tables(call, 0, 0, 0) == n_kv     # host-only: count only


def test_call_validation(pc):
    c = host_cache(pc, max_position=1000)
    c.append_message(0, 0, 10)
    c.append_message(0, 0, 20)
    bad = [
        (Call([(2, 0)], -1, 0, 1, None), pc.PC_ERR_BAD_MSG_ID),
        (Call([(-1, 0)], -1, 0, 1, None), pc.PC_ERR_BAD_MSG_ID),
        (Call([], 5, 0, 1, None), pc.PC_ERR_BAD_MSG_ID),
        (Call([], -2, 0, 1, None), pc.PC_ERR_BAD_MSG_ID),
        (Call([], 0, 0, 11, None), pc.PC_ERR_SHAPE),            # more rows than own tokens
        (Call([], 0, 0, 0, None), pc.PC_ERR_INVALID_ARG),
        (Call([(1, 990)], -1, 0, 1, None), pc.PC_ERR_INVALID_ARG),   # 990 + 19 > 1000
        (Call([(1, -1001)], -1, 0, 1, None), pc.PC_ERR_INVALID_ARG),
        (Call([], 0, 995, 1, None), pc.PC_ERR_INVALID_ARG),
        (Call([], -1, 0, 1, np.array([1001], dtype=np.int32)), pc.PC_ERR_INVALID_ARG),
    ]
    for call, code in bad:
        with pytest.raises(pc.PcError) as ei:
            c.resolve_call(call)
        assert ei.value.code == code, (call, ei.value)
        with pytest.raises(pc.PcError) as ei:
            c.attend([call], 0, 0)
        assert ei.value.code == code
    # legal corner cases: same message twice, new message also a parent, parent after the query
    c.resolve_call(Call([(1, 0), (1, 0), (0, 900)], 0, 5, 10, None))
    c.attend([Call([(1, 0)], 0, POS_AUTO, 3, None)], 0, 0)          # host-only: validates and plans only
    c.attend([], 0, 0)


def test_host_plan_accepts_the_generated_workloads(pc):
    w = small_random(77, n_q_heads=8, n_kv_heads=2)
    c = host_cache(pc)
    for e in w.events:
        if e.kind == "append":
            c.append_message(0, 0, int(e.k.shape[0]), int(e.reserve))
        else:
            c.attend(e.calls, 0, 0)
            lens, res = w.message_lengths(), w.message_reserves()
            for call in e.calls:
                slot, pos = orc.tables_for_call(call, lens, res, pc.PC_SLOT_ALIGN)
                assert c.build_tables(call, 0, 0, 0) == slot.shape[0]


def test_reposition_bookkeeping_on_a_host_only_cache(pc):
    c = host_cache(pc, max_position=500)
    a = c.append_message(0, 0, 40)
    b = c.append_message(0, 0, 7)
    assert c.message_base(a) == 0 and c.message_base(b) == 0
    c.reposition(a, 123)
    c.reposition(b, -500)
    assert c.message_base(a) == 123 and c.message_base(b) == -500
    # a move changes neither the span nor what a call resolves to
    assert c.message_info(a)[:2] == (40, 0)
    starts, s_self, n = c.resolve_call(Call([(a, POS_AUTO), (b, POS_AUTO)], -1, 0, 1, np.array([0], dtype=np.int32)))
    assert starts == [0, 40] and n == 47
    with pytest.raises(pc.PcError) as ei:
        c.reposition(a, 501)
    assert ei.value.code == pc.PC_ERR_INVALID_ARG
    with pytest.raises(pc.PcError) as ei:
        c.reposition(9, 0)
    assert ei.value.code == pc.PC_ERR_BAD_MSG_ID


def test_free_and_reuse_follow_the_slot_model(pc):
    rng = np.random.default_rng(7)
    c = host_cache(pc, capacity_tokens=1 << 16, max_messages=400)
    model = orc.SlotModel(pc.PC_SLOT_ALIGN)
    live = []
    for step in range(300):
        if live and rng.random() < 0.4:
            m = live.pop(int(rng.integers(0, len(live))))
            c.message_free(m)
            model.release(m)
            with pytest.raises(pc.PcError) as ei:
                c.message_info(m)
            assert ei.value.code == pc.PC_ERR_BAD_MSG_ID
        else:
            L = int(rng.integers(1, 200))
            r = int(rng.integers(0, 260))
            m = c.append_message(0, 0, L, r)
            assert c.message_info(m)[1] == model.append(m, max(L, r))
            live.append(m)
        assert c.cache_info()[1] == model.end
    # a freed id is unknown everywhere, and is not handed out again
    dead = [m for m in range(c.cache_info()[0]) if m not in live][0]
    for fn in (lambda: c.message_free(dead), lambda: c.reposition(dead, 0), lambda: c.append_tokens(dead, 0, 0, 1),
               lambda: c.resolve_call(Call([(dead, 0)], -1, 0, 1, None)),
               lambda: c.resolve_call(Call([], dead, 0, 1, None))):
        with pytest.raises(pc.PcError) as ei:
            fn()
        assert ei.value.code == pc.PC_ERR_BAD_MSG_ID
    assert c.append_message(0, 0, 1) == c.cache_info()[0] - 1


def test_growing_messages_on_a_host_only_cache(pc):
    c = host_cache(pc)
    a = c.append_message(0, 0, 3, 10)
    b = c.append_message(0, 0, 1, 4)
    c.append_tokens(a, 0, 0, 7)
    c.append_tokens_batch([b], 0, 0)
    assert c.message_info(a)[0] == 10 and c.message_info(b)[0] == 2
    with pytest.raises(pc.PcError) as ei:
        c.append_tokens_batch([a, b], 0, 0)                  # a is full: nothing may change
    assert ei.value.code == pc.PC_ERR_NO_SPACE
    assert c.message_info(b)[0] == 2
    starts, s_self, n = c.resolve_call(Call([(a, POS_AUTO)], b, POS_AUTO, 2, None))
    assert starts == [0] and s_self == 10 and n == 12


def test_batched_append_is_all_or_nothing_and_follows_the_slot_model(pc):
    c = host_cache(pc, capacity_tokens=1024, max_messages=10)
    model = orc.SlotModel(pc.PC_SLOT_ALIGN)
    ids = c.append_messages([0, 0, 0], [0, 0, 0], [40, 3, 100], [0, 64, 0])
    assert ids == [0, 1, 2]
    for m, r in zip(ids, [40, 64, 100]):
        assert c.message_info(m)[1] == model.append(m, r)
    c.message_free(1); model.release(1)
    before = c.cache_info()
    with pytest.raises(pc.PcError) as ei:                 # the third one does not fit: nothing happens
        c.append_messages([0, 0, 0], [0, 0, 0], [10, 20, 900])
    assert ei.value.code == pc.PC_ERR_NO_SPACE
    with pytest.raises(pc.PcError) as ei:
        c.append_messages([0, 0], [0, 0], [10, 0])
    assert ei.value.code == pc.PC_ERR_INVALID_ARG
    assert c.cache_info() == before
    ids = c.append_messages([0, 0], [0, 0], [33, 200])    # 33 -> 64 slots: the freed span; 200: the end
    assert ids == [3, 4]
    assert [c.message_info(m)[1] for m in ids] == [model.append(3, 33), model.append(4, 200)]
    with pytest.raises(pc.PcError) as ei:                 # 5 live ids + 6 > max_messages
        c.append_messages([0] * 6, [0] * 6, [1] * 6)
    assert ei.value.code == pc.PC_ERR_NO_SPACE
    assert c.append_messages([], [], []) == []


def test_swap_bookkeeping_on_a_host_only_cache(pc):
    # swap-out frees the span exactly as a free does, swap-in takes slots by the allocation rule and the
    # message is what it was (id, length, reserve, stored base); in between the id is unknown elsewhere
    c = host_cache(pc, capacity_tokens=1024, max_messages=64)
    model = orc.SlotModel(pc.PC_SLOT_ALIGN)
    ids = []
    for L, r in ((40, 0), (10, 70), (33, 0), (5, 0)):
        m = c.append_message(0, 0, L, r)
        assert c.message_info(m)[1] == model.append(m, max(L, r))
        ids.append(m)
    a, b, cc, d = ids
    c.reposition(b, 123)
    per_slot = 2 * 2 * 64 * 4                                  # K and V, 2 KV heads, D 64, fp32 (host_cache's shape)
    assert c.message_swap_bytes(b) == 96 * per_slot            # reserve 70 -> 96 slots
    c.message_swap_out(b, 0)
    model.release(b)
    assert c.message_swap_bytes(b) == 96 * per_slot
    for fn in (lambda: c.message_info(b), lambda: c.message_swap_out(b, 0), lambda: c.message_free(b),
               lambda: c.reposition(b, 0), lambda: c.append_tokens(b, 0, 0, 1),
               lambda: c.resolve_call(Call([(b, 0)], -1, 0, 1, None))):
        with pytest.raises(pc.PcError) as ei:
            fn()
        assert ei.value.code == pc.PC_ERR_BAD_MSG_ID
    with pytest.raises(pc.PcError) as ei:
        c.message_swap_in(a, 0)                                # a live message cannot be swapped in
    assert ei.value.code == pc.PC_ERR_BAD_MSG_ID
    e = c.append_message(0, 0, 20)                             # takes the head of b's old span
    assert c.message_info(e)[1] == model.append(e, 20)
    c.message_swap_in(b, 0)                                    # 96 slots: what is left of the hole is too small
    assert c.message_info(b)[1] == model.append(b, 70)
    assert c.message_info(b)[0] == 10 and c.message_base(b) == 123
    assert c.cache_info()[1] == model.end
    c.append_tokens(b, 0, 0, 60)                               # the reserve came back with it
    assert c.message_info(b)[0] == 70
    # no room: nothing changes and the message stays swapped out
    c.message_swap_out(cc, 0)
    model.release(cc)
    big = c.append_message(0, 0, 1024 - model.end)             # fills the cache to the end
    model.append(big, 1024 - (model.end))
    f2 = c.append_message(0, 0, 70)                            # and of the hole (cc's span merged with b's leftover: 128) 32 stay
    assert c.message_info(f2)[1] == model.append(f2, 70)
    with pytest.raises(pc.PcError) as ei:
        c.message_swap_in(cc, 0)
    assert ei.value.code == pc.PC_ERR_NO_SPACE
    assert c.message_swap_bytes(cc) == 64 * per_slot
    c.message_free(f2)
    model.release(f2)
    c.message_swap_in(cc, 0)
    assert c.message_info(cc)[1] == model.append(cc, 33)


def test_gradient_entry_points_validate_like_attend(pc):
    for kw in (dict(), dict(dtype=pc.PC_F32, head_dim=64)):       # bf16 and fp32 caches (host-only: validation and planning)
        f = host_cache(pc, **kw)
        a = f.append_message(0, 0, 5)
        f.attend_backward([Call([(a, 0)], -1, 0, 1, None)], 0, 0, 0, 0, 0, 0)
        f.grad_keys_finalize(0)
        with pytest.raises(pc.PcError) as ei:
            f.attend_backward([Call([(a + 1, 0)], -1, 0, 1, None)], 0, 0, 0, 0, 0, 0)
        assert ei.value.code == pc.PC_ERR_BAD_MSG_ID


def test_probe_entries_reject_bad_arguments_before_touching_the_device(pc):
    from paper_2512_23049_amd import probe
    hdr = open(os.path.join(ROOT, "include", "pc_probe.h")).read()
    names = set(re.findall(r"\b(pc_probe_[a-z0-9_]+)\s*\(", hdr))
    assert names == {"pc_probe_mfma_bf16", "pc_probe_hbm_read"}
    lib = probe.lib()
    for n in names:
        assert hasattr(lib, n), n
    out = ctypes.c_double(0.0)
    one = ctypes.c_void_p(4096)            # never dereferenced: every call below fails its argument checks
    INVALID, SHAPE = -1, -4
    assert lib.pc_probe_mfma_bf16(None, 16384, 16, 2, 1, one, ctypes.byref(out), None) == INVALID
    assert lib.pc_probe_mfma_bf16(one, 16383, 16, 2, 1, one, ctypes.byref(out), None) == SHAPE
    assert lib.pc_probe_mfma_bf16(one, 16384, 0, 2, 1, one, ctypes.byref(out), None) == INVALID
    assert lib.pc_probe_mfma_bf16(one, 16384, 16, 3, 1, one, ctypes.byref(out), None) == INVALID
    assert lib.pc_probe_hbm_read(None, 1 << 20, 1, one, ctypes.byref(out), None) == INVALID
    assert lib.pc_probe_hbm_read(one, 24, 1, one, ctypes.byref(out), None) == SHAPE
    assert lib.pc_probe_hbm_read(ctypes.c_void_p(4100), 1 << 20, 1, one, ctypes.byref(out), None) == SHAPE
    assert lib.pc_probe_hbm_read(one, 1 << 20, 0, one, ctypes.byref(out), None) == INVALID
    assert out.value == 0.0


def test_random_walk_over_growing_freed_swapped_and_moved_messages(pc):
    """Messages that grow into further extents (PC_FLAG_GROW_EXTENTS), are freed, swapped out and in and moved,
    in random order on a host-only cache, against a model written from the header's rules: every extent is a span
    of the slot model under a row of its own; a further extent holds what the call still brings for the message
    and at least the message's first reserve (and a tile); a free or a swap-out gives every span back; a swap-in
    takes a span per extent in token order; a position update moves every extent's stored base."""
    rng = np.random.default_rng(123)
    flags = pc.PC_FLAG_HOST_ONLY | pc.PC_FLAG_GROW_EXTENTS
    c = host_cache(pc, capacity_tokens=1 << 17, max_messages=4000, flags=flags)
    model = orc.SlotModel(pc.PC_SLOT_ALIGN)
    ext, base, out = {}, {}, {}          # message -> [[row, len, reserve], ...];  stored base;  swapped-out messages
    rows = [0]                           # next row of the message table

    def new_row():
        rows[0] += 1
        return rows[0] - 1

    def grow(m, n, pending):
        """n tokens for message m; pending collects the extents to allocate, in the order the tokens come."""
        e = ext[m]
        for left in range(n, 0, -1):
            if e[-1][1] == e[-1][2]:
                res = max(left, pc.PC_SLOT_ALIGN, e[0][2])
                e.append([None, 0, res])
                pending.append((m, len(e) - 1))
            e[-1][1] += 1

    def commit(pending):
        for m, i in pending:
            row = new_row()
            ext[m][i][0] = row
            model.append(row, ext[m][i][2])

    for step in range(1500):
        live = sorted(ext)
        op = rng.random()
        if op < 0.25 or not live:
            L, r = int(rng.integers(1, 120)), int(rng.integers(0, 150))
            m = c.append_message(0, 0, L, r)
            row = new_row()
            assert m == row
            model.append(row, max(L, r))
            ext[m], base[m] = [[row, L, max(L, r)]], 0
        elif op < 0.50:
            m = live[int(rng.integers(0, len(live)))]
            n = int(rng.integers(1, 90))
            c.append_tokens(m, 0, 0, n)
            pending = []
            grow(m, n, pending)
            commit(pending)
        elif op < 0.65:
            k = int(rng.integers(1, min(6, len(live)) + 1))
            ms = [live[i] for i in rng.permutation(len(live))[:k]]
            c.append_tokens_batch(ms, 0, 0)
            pending = []
            for m in ms:
                grow(m, 1, pending)
            commit(pending)
        elif op < 0.75:
            m = live[int(rng.integers(0, len(live)))]
            c.message_free(m)
            for row, _, _ in ext.pop(m):
                model.release(row)
            base.pop(m)
        elif op < 0.85:
            m = live[int(rng.integers(0, len(live)))]
            c.message_swap_out(m, 0)
            for row, _, _ in ext[m]:
                model.release(row)
            out[m] = (ext.pop(m), base.pop(m))
        elif op < 0.93 and out:
            m = sorted(out)[int(rng.integers(0, len(out)))]
            c.message_swap_in(m, 0)
            e, b = out.pop(m)
            for rec in e:
                model.append(rec[0], rec[2])
            ext[m], base[m] = e, b
        else:
            m = live[int(rng.integers(0, len(live)))]
            nb = int(rng.integers(-5000, 5000))
            c.reposition(m, nb)
            base[m] = nb
        # the library and the model agree on everything a caller can see
        assert c.cache_info()[1] == model.end, step
        for m in (sorted(ext)[-3:] + sorted(ext)[:2]):
            e = ext[m]
            assert c.message_extents(m) == [(model.span[row][0], ln) for row, ln, _ in e], (step, m)
            assert c.message_info(m) == (sum(ln for _, ln, _ in e), model.span[e[0][0]][0], sum(r for _, _, r in e)), (step, m)
            assert c.message_base(m) == base[m]
        for m in list(out)[:2]:
            with pytest.raises(pc.PcError) as ei:
                c.message_info(m)
            assert ei.value.code == pc.PC_ERR_BAD_MSG_ID
    # at the end: every live message, in full
    for m, e in ext.items():
        assert c.message_extents(m, cap=256) == [(model.span[row][0], ln) for row, ln, _ in e]
    assert len(ext) > 20 and max(len(e) for e in ext.values()) >= 3
    # to a call a message of several extents is one sequence of tokens: omitted offsets and the gathered
    # length follow the oracle's rule on the messages' total lengths
    live = sorted(ext)
    lengths = {m: sum(ln for _, ln, _ in e) for m, e in ext.items()}
    for _ in range(40):
        sel = [(live[int(rng.integers(0, len(live)))], POS_AUTO if rng.random() < 0.5 else int(rng.integers(-900, 900)))
               for _ in range(int(rng.integers(0, 6)))]
        m_self = live[int(rng.integers(0, len(live)))]
        s_self = POS_AUTO if rng.random() < 0.5 else int(rng.integers(-900, 900))
        want_sel, want_self = orc.resolve_positions(sel, lengths, s_self)
        starts, got_self, n_kv = c.resolve_call(Call(sel, m_self, s_self, 1, None))
        assert starts == [s for _, s in want_sel] and got_self == want_self
        assert n_kv == sum(lengths[m] for m, _ in sel) + lengths[m_self]
