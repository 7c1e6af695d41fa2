"""Pins for the CPU oracle: everything here checks it against something other
than itself (closed forms, brute force, a library attention, invariants,
hand-written tables).  No GPU needed."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import brute_force as bf
from oracle import choreo_oracle as orc
from pc_inputs import POS_AUTO, Call, small_random, tiny_fp32
from tests.helpers import cache_lists, read_golden

RNG = np.random.default_rng(1234)


def _rand_cache(rng, lens, H_kv, D):
    ks = [rng.standard_normal((L, H_kv, D)) for L in lens]
    vs = [rng.standard_normal((L, H_kv, D)) for L in lens]
    return ks, vs


# ---------------------------------------------------------------- RoPE itself
def test_rope_quarter_turn_closed_form():
    # D = 2: one pair, frequency theta^0 = 1; position pi/2 is not an integer, so
    # use theta-independent integer position and compare with cos/sin of 1 rad.
    x = np.array([[1.0, 0.0]])
    y = orc.rope(x, np.array([1]), 10000.0)
    assert np.allclose(y, [[math.cos(1.0), math.sin(1.0)]], atol=1e-15)
    x = np.array([[0.0, 1.0]])
    y = orc.rope(x, np.array([1]), 10000.0)
    assert np.allclose(y, [[-math.sin(1.0), math.cos(1.0)]], atol=1e-15)


def test_rope_pairing_and_frequencies_d4():
    # D = 4, base 10000: pairs are (0,2) and (1,3); frequencies 1 and 10000^(-1/2) = 0.01
    p = 7
    y = orc.rope(np.array([[1.0, 0.0, 0.0, 0.0]]), np.array([p]), 10000.0)
    assert np.allclose(y, [[math.cos(7.0), 0.0, math.sin(7.0), 0.0]], atol=1e-15)
    y = orc.rope(np.array([[0.0, 1.0, 0.0, 0.0]]), np.array([p]), 10000.0)
    assert np.allclose(y, [[0.0, math.cos(0.07), 0.0, math.sin(0.07)]], atol=1e-15)


def test_rope_group_properties():
    x = RNG.standard_normal((5, 3, 16))
    p = np.array([0, 3, -17, 4000, 65535])
    y = orc.rope(x, p, 5e5)
    assert np.allclose(y[0], x[0], atol=0)                                   # R(0) = I
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)
    z = orc.rope(orc.rope(x, p, 5e5), np.array([5, -3, 17, 96, 1]), 5e5)      # R(a)R(b) = R(a+b)
    assert np.allclose(z, orc.rope(x, p + np.array([5, -3, 17, 96, 1]), 5e5), atol=1e-9)


def test_rope_scores_depend_on_position_difference_only():
    q = RNG.standard_normal((1, 32))
    k = RNG.standard_normal((1, 32))
    ref = (orc.rope(q, np.array([40]), 1e4) * orc.rope(k, np.array([17]), 1e4)).sum()
    for c in (-40, 5, 1000):
        got = (orc.rope(q, np.array([40 + c]), 1e4) * orc.rope(k, np.array([17 + c]), 1e4)).sum()
        assert abs(got - ref) < 1e-10


def test_delta_rotation_identity():
    # <R(p)q, R(s+t)k> == <R(p-s)q, R(t)k>: the identity behind storing keys rotated
    # at their in-message index and turning the query per parent instead.
    q = RNG.standard_normal((1, 64))
    k = RNG.standard_normal((1, 64))
    p, s, t = 5000, 1234, 77
    lhs = (orc.rope(q, np.array([p]), 5e5) * orc.rope(k, np.array([s + t]), 5e5)).sum()
    rhs = (orc.rope(q, np.array([p - s]), 5e5) * orc.rope(k, np.array([t]), 5e5)).sum()
    assert abs(lhs - rhs) < 1e-10


def test_position_updates_compose():
    # Sec. 2.4 "Position Updates": a cached key already turned to position a is moved to
    # position b by one more rotation of (b - a); moves compose and a move back restores it.
    k = RNG.standard_normal((7, 2, 64))
    t = np.arange(7)
    at_a = orc.rope(k, 40 + t, 1e4)
    moved = orc.rope(at_a, np.full(7, 1000 - 40), 1e4)
    assert np.abs(moved - orc.rope(k, 1000 + t, 1e4)).max() < 1e-10
    back = orc.rope(moved, np.full(7, -(1000 - 40)), 1e4)
    assert np.abs(back - at_a).max() < 1e-10
    # a rotation keeps every (i, i + D/2) pair's length: the textbook property of a plane rotation
    n0 = k[..., :32] ** 2 + k[..., 32:] ** 2
    n1 = moved[..., :32] ** 2 + moved[..., 32:] ** 2
    assert np.abs(n0 - n1).max() < 1e-10


def test_slot_model_hand_worked_sequence():
    # hand-worked with align 32: A(40)->[0,64) B(10)->[64,96) C(100)->[96,224) D(32)->[224,256)
    m = orc.SlotModel(32)
    assert [m.append(i, r) for i, r in enumerate([40, 10, 100, 32])] == [0, 64, 96, 224]
    m.release(1)                                   # free [64,96)
    assert m.append(4, 33) == 256                  # needs 64: the hole is too small, goes to the end -> [256,320)
    assert m.append(5, 32) == 64                   # fits the hole exactly
    m.release(0); m.release(5)                     # [0,64) + [64,96) merge into [0,96)
    assert m.free == [(0, 96)]
    assert m.append(6, 70) == 0                    # takes 96 of it
    m.release(4)                                   # the last span: the used region shrinks to 256
    assert m.end == 256 and m.free == []
    m.release(3)                                   # now D is last: shrinks to 224
    assert m.end == 224
    m.release(2)                                   # C too: 96
    assert m.end == 96 and m.free == []
    assert m.append(7, 1) == 96
    # without any release the model is the bump rule
    m2 = orc.SlotModel(32)
    rs = [3, 64, 65, 1, 200]
    assert [m2.append(i, r) for i, r in enumerate(rs)] == orc.slot_starts(rs, 32)


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_brute_force_agrees_on_tiny_inputs(seed):
    rng = np.random.default_rng(seed)
    H_kv, g, D = 2, 2, 8
    lens = [3, 1, 5, 4, 2]
    ks, vs = _rand_cache(rng, lens, H_kv, D)
    cases = [
        # gaps, overlap, repeat, AUTO, self listed as a parent too
        Call([(2, 7), (0, POS_AUTO), (2, 5), (1, -4)], 3, POS_AUTO, 3, None),
        Call([(4, 100), (3, 90)], 3, 20, 4, None),
        Call([], 2, POS_AUTO, 5, None),
        Call([(0, 0), (1, 0)], -1, POS_AUTO, 2, np.array([9, 2], dtype=np.int32)),
        Call([(1, 3)], 4, 1000, 1, np.array([-6], dtype=np.int32)),
    ]
    for c in cases:
        q = rng.standard_normal((c.n_q, H_kv * g, D))
        o, l = orc.attend_call(ks, vs, c.sel, c.self_msg, c.self_start, c.n_q, c.q_pos, q, 100.0)
        ob, lb = bf.attend_call_brute(ks, vs, c.sel, c.self_msg, c.self_start, c.n_q, c.q_pos,
                                      q, 100.0)
        assert np.allclose(o, np.asarray(ob), atol=1e-12, rtol=0)
        assert np.allclose(l, np.asarray(lb), atol=1e-12, rtol=0)


# ------------------------------------------- reduction to prefix-cache attention
def _torch_rope_complex(x, pos, theta):
    """Standard RoPE through complex multiplication (independent of the oracle's
    real-arithmetic form)."""
    D = x.shape[-1]
    half = D // 2
    freq = torch.tensor([theta ** (-2.0 * i / D) for i in range(half)], dtype=torch.float64)
    ang = pos.to(torch.float64)[:, None] * freq[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)                     # [T, half]
    xc = torch.complex(x[..., :half], x[..., half:])
    yc = xc * rot[:, None, :]
    return torch.cat([yc.real, yc.imag], dim=-1)


@pytest.mark.parametrize("theta", [1e4, 5e5])
def test_in_order_contiguous_selection_is_ordinary_causal_attention(theta):
    rng = np.random.default_rng(7)
    H_kv, g, D = 2, 3, 16
    lens = [5, 9, 1, 12, 6]                       # last message is the new one
    T = sum(lens)
    ks, vs = _rand_cache(rng, lens, H_kv, D)
    n_q = lens[-1]
    q_new = rng.standard_normal((n_q, H_kv * g, D))
    sel, s = [], 0
    for m in range(len(lens) - 1):
        sel.append((m, s))
        s += lens[m]
    o, _ = orc.attend_call(ks, vs, sel, len(lens) - 1, s, n_q, None, q_new, theta)
    # default offsets give the same thing
    o2, _ = orc.attend_call(ks, vs, [(m, POS_AUTO) for m in range(len(lens) - 1)],
                            len(lens) - 1, POS_AUTO, n_q, None, q_new, theta)
    assert np.allclose(o, o2, atol=1e-13)

    K = torch.from_numpy(np.concatenate(ks))      # [T, H_kv, D]
    V = torch.from_numpy(np.concatenate(vs))
    Q = torch.zeros((T, H_kv * g, D), dtype=torch.float64)
    Q[T - n_q:] = torch.from_numpy(q_new)
    pos = torch.arange(T)
    Kr = _torch_rope_complex(K, pos, theta).repeat_interleave(g, dim=1)
    Qr = _torch_rope_complex(Q, pos, theta)
    Vr = V.repeat_interleave(g, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(
        Qr.permute(1, 0, 2)[None], Kr.permute(1, 0, 2)[None], Vr.permute(1, 0, 2)[None],
        is_causal=True)[0].permute(1, 0, 2)[T - n_q:]
    assert np.allclose(o, ref.numpy(), atol=1e-12)


# ------------------------------------------------------------------ invariants
def _random_call_case(seed):
    rng = np.random.default_rng(seed)
    H_kv, g, D = 2, 2, 32
    lens = [int(x) for x in rng.integers(1, 20, size=7)]
    ks, vs = _rand_cache(rng, lens, H_kv, D)
    sel = [(int(rng.integers(0, 6)), int(rng.integers(0, 300))) for _ in range(5)]
    n_q = min(4, lens[6])
    q = rng.standard_normal((n_q, H_kv * g, D))
    return ks, vs, lens, sel, 6, 450, n_q, q


@pytest.mark.parametrize("shift", [-1000, -1, 13, 40000])
def test_shift_invariance(shift):
    ks, vs, lens, sel, m_self, s_self, n_q, q = _random_call_case(11)
    o, l = orc.attend_call(ks, vs, sel, m_self, s_self, n_q, None, q, 5e5)
    sel2 = [(m, s + shift) for m, s in sel]
    o2, l2 = orc.attend_call(ks, vs, sel2, m_self, s_self + shift, n_q, None, q, 5e5)
    assert np.allclose(o, o2, atol=1e-10, rtol=0)
    assert np.allclose(l, l2, atol=1e-10, rtol=0)
    starts = orc.slot_starts(lens, 8)
    a = orc.assemble(sel, m_self, s_self, lens, starts)
    b = orc.assemble(sel2, m_self, s_self + shift, lens, starts)
    assert np.array_equal(a[0], b[0])
    assert np.array_equal(a[1] + shift, b[1])
    # explicit q_pos shifted too
    qp = (s_self + lens[m_self] - n_q + np.arange(n_q)).astype(np.int32)
    o3, _ = orc.attend_call(ks, vs, sel2, m_self, s_self + shift, n_q, qp + shift, q, 5e5)
    assert np.allclose(o, o3, atol=1e-10, rtol=0)


def test_permutation_invariance():
    ks, vs, lens, sel, m_self, s_self, n_q, q = _random_call_case(12)
    o, l = orc.attend_call(ks, vs, sel, m_self, s_self, n_q, None, q, 1e4)
    perm = [3, 0, 4, 2, 1]
    sel2 = [sel[i] for i in perm]
    o2, l2 = orc.attend_call(ks, vs, sel2, m_self, s_self, n_q, None, q, 1e4)
    assert np.allclose(o, o2, atol=1e-12, rtol=0)
    assert np.allclose(l, l2, atol=1e-12, rtol=0)
    starts = orc.slot_starts(lens, 4)
    slot, pos, npar = orc.assemble(sel, m_self, s_self, lens, starts)
    slot2, pos2, _ = orc.assemble(sel2, m_self, s_self, lens, starts)
    # the table is the same permutation of whole segments
    segs, at = [], 0
    for m, _s in sel:
        segs.append((slot[at:at + lens[m]], pos[at:at + lens[m]]))
        at += lens[m]
    exp_slot = np.concatenate([segs[i][0] for i in perm] + [slot[npar:]])
    exp_pos = np.concatenate([segs[i][1] for i in perm] + [pos[npar:]])
    assert np.array_equal(slot2, exp_slot) and np.array_equal(pos2, exp_pos)


def test_all_positions_zero_is_textbook_softmax_attention():
    rng = np.random.default_rng(3)
    H, D = 2, 8
    ks, vs = _rand_cache(rng, [4, 6], H, D)
    q = rng.standard_normal((3, H, D))
    zero = np.zeros(3, dtype=np.int32)
    # parents only, every token at position 0 (message placed at -t is impossible, so
    # use single-token messages instead)
    ks1 = [k[i:i + 1] for k in ks for i in range(k.shape[0])]
    vs1 = [v[i:i + 1] for v in vs for i in range(v.shape[0])]
    sel = [(i, 0) for i in range(len(ks1))]
    o, l = orc.attend_call(ks1, vs1, sel, -1, 0, 3, zero, q, 1e4)
    K = np.concatenate(ks1)
    V = np.concatenate(vs1)
    for h in range(H):
        S = q[:, h] @ K[:, h].T / math.sqrt(D)
        P = np.exp(S - S.max(1, keepdims=True))
        P /= P.sum(1, keepdims=True)
        assert np.allclose(o[:, h], P @ V[:, h], atol=1e-13)
        assert np.allclose(l[:, h], np.log(np.exp(S).sum(1)), atol=1e-12)


def test_constant_values_and_closed_forms():
    rng = np.random.default_rng(4)
    H, D = 1, 4
    ks, vs = _rand_cache(rng, [5, 3], H, D)
    vconst = [np.full_like(v, 2.5) for v in vs]
    q = rng.standard_normal((2, 2, D))
    o, _ = orc.attend_call(ks, vconst, [(0, 3), (1, 50)], -1, 0, 2, np.array([60, 61]), q, 1e4)
    assert np.allclose(o, 2.5, atol=1e-13)
    # one visible key -> its value row
    o, l = orc.attend_call(ks, vs, [], 1, 10, 1, None, q[:1], 1e4)       # decode row sees 3 own
    o1, _ = orc.attend_call([ks[0][:1]], [vs[0][:1]], [(0, 5)], -1, 0, 1, np.array([9]), q[:1], 1e4)
    assert np.allclose(o1[0, 0], vs[0][0, 0], atol=1e-14)
    # two identical keys at the same position -> mean of the two value rows
    k2 = [ks[0][:1], ks[0][:1]]
    v2 = [vs[0][:1], vs[0][1:2]]
    o2, _ = orc.attend_call(k2, v2, [(0, 5), (1, 5)], -1, 0, 1, np.array([9]), q[:1], 1e4)
    assert np.allclose(o2[0, 0], 0.5 * (vs[0][0, 0] + vs[0][1, 0]), atol=1e-14)


def test_listing_every_entry_twice_keeps_output_and_adds_ln2():
    ks, vs, lens, sel, m_self, s_self, n_q, q = _random_call_case(13)
    o, l = orc.attend_call(ks, vs, sel, -1, s_self, n_q, np.arange(n_q) + 500, q, 1e4)
    o2, l2 = orc.attend_call(ks, vs, sel + sel, -1, s_self, n_q, np.arange(n_q) + 500, q, 1e4)
    assert np.allclose(o, o2, atol=1e-12)
    assert np.allclose(l2, l + math.log(2.0), atol=1e-12)


def test_union_equals_lse_merge_of_parts():
    ks, vs, lens, sel, m_self, s_self, n_q, q = _random_call_case(14)
    qp = np.arange(n_q) + 700
    o, l = orc.attend_call(ks, vs, sel, -1, 0, n_q, qp, q, 5e5)
    oa, la = orc.attend_call(ks, vs, sel[:2], -1, 0, n_q, qp, q, 5e5)
    ob, lb = orc.attend_call(ks, vs, sel[2:], -1, 0, n_q, qp, q, 5e5)
    # textbook combination written out here, not through the oracle's helper
    m = np.maximum(la, lb)
    wa, wb = np.exp(la - m), np.exp(lb - m)
    exp_o = (wa[..., None] * oa + wb[..., None] * ob) / (wa + wb)[..., None]
    assert np.allclose(o, exp_o, atol=1e-12)
    assert np.allclose(l, m + np.log(wa + wb), atol=1e-12)
    mo, ml = orc.merge_partials([oa, ob], [la, lb])
    assert np.allclose(mo, o, atol=1e-12) and np.allclose(ml, l, atol=1e-12)
    # an empty part merges as a no-op
    oe, le = orc.attend_call(ks, vs, [], -1, 0, n_q, qp, q, 5e5)
    assert np.all(oe == 0) and np.all(np.isneginf(le))
    mo, ml = orc.merge_partials([o, oe], [l, le])
    assert np.allclose(mo, o, atol=0) and np.allclose(ml, l, atol=0)


def test_decode_row_equals_last_prefill_row():
    ks, vs, lens, sel, m_self, s_self, n_q, q = _random_call_case(15)
    L = lens[m_self]
    qfull = np.random.default_rng(5).standard_normal((L, q.shape[1], q.shape[2]))
    o, l = orc.attend_call(ks, vs, sel, m_self, s_self, L, None, qfull, 1e4)
    o1, l1 = orc.attend_call(ks, vs, sel, m_self, s_self, 1, None, qfull[-1:], 1e4)
    assert np.allclose(o[-1], o1[0], atol=1e-13) and np.allclose(l[-1], l1[0], atol=1e-13)
    # first prefill row sees the parents and only its own token
    of, _ = orc.attend_call(ks + [ks[m_self][:1]], vs + [vs[m_self][:1]], sel, len(ks), s_self,
                            1, None, qfull[:1], 1e4)
    assert np.allclose(o[0], of[0], atol=1e-13)


def test_gqa_equals_mha_with_repeated_kv_heads():
    rng = np.random.default_rng(6)
    H_kv, g, D = 2, 4, 8
    ks, vs = _rand_cache(rng, [6, 5, 4], H_kv, D)
    q = rng.standard_normal((4, H_kv * g, D))
    o, l = orc.attend_call(ks, vs, [(1, 9), (0, 2)], 2, 30, 4, None, q, 1e4)
    kr = [np.repeat(k, g, axis=1) for k in ks]
    vr = [np.repeat(v, g, axis=1) for v in vs]
    o2, l2 = orc.attend_call(kr, vr, [(1, 9), (0, 2)], 2, 30, 4, None, q, 1e4)
    assert np.allclose(o, o2, atol=1e-13) and np.allclose(l, l2, atol=1e-13)


def test_parent_placed_after_the_query_is_still_visible():
    rng = np.random.default_rng(8)
    ks, vs = _rand_cache(rng, [3, 2], 1, 4)
    q = rng.standard_normal((1, 1, 4))
    o_far, _ = orc.attend_call(ks, vs, [(0, 1000)], 1, 0, 1, None, q, 1e4)
    o_none, _ = orc.attend_call(ks, vs, [], 1, 0, 1, None, q, 1e4)
    assert not np.allclose(o_far, o_none)


# -------------------------------------------------------------- tables & masks
def test_handwritten_tables(golden_dir):
    g = read_golden(os.path.join(golden_dir, "tables_three_messages.txt"))
    align = int(g["align"][0])
    lens = [int(x) for x in g["lengths"]]

    def ent(s):
        m, p = s.split(":")
        return int(m), (POS_AUTO if p == "AUTO" else int(p))
    sel = [ent(s) for s in g["sel"]]
    m_self, s_self = ent(g["self"][0])
    call = Call(sel, m_self, s_self, 1, None)
    slot, pos = orc.tables_for_call(call, lens, lens, align)
    assert slot.dtype == np.int32 and pos.dtype == np.int32
    assert slot.tolist() == [int(x) for x in g["kv_slot"]]
    assert pos.tolist() == [int(x) for x in g["kv_pos"]]


def test_slot_layout_rule():
    assert orc.slot_starts([3, 5, 2, 4], 4) == [0, 4, 12, 16]
    assert orc.slot_starts([32, 1, 33, 64], 32) == [0, 32, 64, 128]
    assert orc.slot_starts([7, 7], 1) == [0, 7]


@pytest.mark.parametrize("name", ["fig2_prefill_mask.txt", "fig2_decode_mask.txt"])
def test_fig2_mask_structure(golden_dir, name):
    g = read_golden(os.path.join(golden_dir, name))
    token_msg = np.asarray([int(x) for x in g["token_msg"]])
    parents = [[int(x) for x in c["parents"].split(",")] for c in g["call"]]
    new = [int(c["new"]) for c in g["call"]]
    toks = [np.asarray([int(x) for x in c["tokens"].split(",")]) for c in g["call"]]
    got = orc.batch_mask(token_msg.shape[0], token_msg, parents, new, toks)
    assert np.array_equal(got, g["mask"])


def test_visibility_matches_the_batch_mask_on_a_contiguous_layout():
    # per-call visibility (gather form) == the whole-cache mask restricted to the
    # call's gathered columns, for a physically contiguous new message
    token_msg = np.asarray([0, 0, 0, 1, 1, 2, 2, 2, 2])
    full = orc.batch_mask(9, token_msg, [[1, 0]], [2], [np.asarray([1, 2, 3])])
    cols = [3, 4, 0, 1, 2, 5, 6, 7, 8]            # list order: msg 1, msg 0, then self
    vis = orc.visibility(3, 5, 4)
    assert np.array_equal(full[:, cols], vis)


# ------------------------------------------------------------ workload sanity
def test_tiny_workload_has_the_stated_gap_and_overlap():
    w = tiny_fp32()
    lens = w.message_lengths()
    call = w.events[-1].calls[0]
    by_pos = sorted(call.sel, key=lambda e: e[1])
    ends = [s + lens[m] for m, s in by_pos]
    deltas = [by_pos[i + 1][1] - ends[i] for i in range(3)]
    assert deltas == [10, -8, 0]
    assert call.self_start == ends[-1] and call.n_q == 32 and lens[call.self_msg] == 32
    ks, vs = cache_lists(w)
    o, l = orc.attend_call(ks, vs, call.sel, call.self_msg, call.self_start, call.n_q,
                           call.q_pos, w.events[-1].q.astype(np.float64), w.rope_theta)
    assert o.shape == (32, 4, 64) and np.isfinite(o).all() and np.isfinite(l).all()


def test_batched_attend_packs_calls_in_order():
    w = small_random(21, dtype="f32", n_q_heads=4, n_kv_heads=2, head_dim=16, n_msgs=6,
                     len_hi=20, n_calls=6, max_q=5)
    ks, vs = cache_lists(w)
    ev = w.events[-1]
    q = ev.q.astype(np.float64)
    o, l = orc.attend(ks, vs, ev.calls, q, w.rope_theta)
    at = 0
    for c in ev.calls:
        ob, lb = bf.attend_call_brute(ks, vs, c.sel, c.self_msg, c.self_start, c.n_q, c.q_pos,
                                      q[at:at + c.n_q], w.rope_theta)
        assert np.allclose(o[at:at + c.n_q], np.asarray(ob).reshape(c.n_q, 4, 16), atol=1e-11)
        assert np.allclose(l[at:at + c.n_q], np.asarray(lb).reshape(c.n_q, 4), atol=1e-11)
        at += c.n_q
    assert at == o.shape[0]


# ---------------------------------------------------------------------------
# gradient oracle: pinned by numerical differentiation of the FORWARD oracle (which has its
# own pins above) and by closed forms; nothing here calls attend_call_backward to make its
# own expectation
# ---------------------------------------------------------------------------
def _grad_case(seed=5):
    rng = np.random.default_rng(seed)
    H_q, H_kv, D = 4, 2, 16
    lens = [5, 3, 7, 4]
    ks = [rng.standard_normal((L, H_kv, D)) for L in lens]
    vs = [rng.standard_normal((L, H_kv, D)) for L in lens]
    sel = [(2, 11), (0, -3), (2, 40)]                      # message 2 twice, a negative start
    self_msg, self_start, n_q = 3, 20, 3                   # rows = the last 3 of 4 own tokens (causal part)
    q = rng.standard_normal((n_q, H_q, D))
    d_out = rng.standard_normal((n_q, H_q, D))
    return ks, vs, sel, self_msg, self_start, n_q, q, d_out


def test_gradient_oracle_matches_central_differences_of_the_forward_oracle():
    ks, vs, sel, self_msg, self_start, n_q, q, d_out = _grad_case()
    theta = 10000.0

    def loss(ks_, vs_, q_):
        o, _ = orc.attend_call(ks_, vs_, sel, self_msg, self_start, n_q, None, q_, theta)
        return float((o * d_out).sum())
    d_q, d_k, d_v = orc.attend_call_backward(ks, vs, sel, self_msg, self_start, n_q, None, q, d_out, theta)
    rng = np.random.default_rng(1)
    eps = 1e-6

    def check(arr_list, which, grads, n=12):
        for _ in range(n):
            m = int(rng.integers(0, len(arr_list)))
            idx = tuple(int(rng.integers(0, s)) for s in arr_list[m].shape)
            keep = arr_list[m][idx]
            arr_list[m][idx] = keep + eps
            up = loss(ks, vs, q)
            arr_list[m][idx] = keep - eps
            dn = loss(ks, vs, q)
            arr_list[m][idx] = keep
            num = (up - dn) / (2 * eps)
            assert abs(num - grads[m][idx]) <= 1e-7 + 1e-6 * abs(num), (which, m, idx, num, grads[m][idx])
    check(ks, "K", d_k)
    check(vs, "V", d_v)
    check([q], "q", [d_q])
    assert np.abs(d_k[1]).max() == 0 and np.abs(d_v[1]).max() == 0          # message 1 is not read


def test_gradient_oracle_closed_forms():
    rng = np.random.default_rng(9)
    H_q, H_kv, D = 2, 1, 8
    # one visible key: the output IS its value row, whatever q and k are
    ks, vs = [rng.standard_normal((1, H_kv, D))], [rng.standard_normal((1, H_kv, D))]
    q, d_out = rng.standard_normal((2, H_q, D)), rng.standard_normal((2, H_q, D))
    d_q, d_k, d_v = orc.attend_call_backward(ks, vs, [(0, 7)], -1, 0, 2, np.asarray([3, 9]), q, d_out, 1e4)
    assert np.abs(d_q).max() < 1e-12 and np.abs(d_k[0]).max() < 1e-12
    assert np.allclose(d_v[0][0, 0], d_out.sum(axis=(0, 1)), atol=1e-12)
    # all positions zero and q = 0: uniform weights 1/N, so dV rows are dO/N and dK = scale * dS^T q = 0;
    # dq = scale * sum_j dS_j k_j with dS_j = (dO.v_j - mean_j dO.v_j) / N
    N = 5
    ks, vs = [rng.standard_normal((N, H_kv, D))], [rng.standard_normal((N, H_kv, D))]
    q0 = np.zeros((1, H_q, D))
    d_out = rng.standard_normal((1, H_q, D))
    d_q, d_k, d_v = orc.attend_call_backward(ks, vs, [(0, 0)], -1, 0, 1, np.asarray([0]), q0, d_out, 1e4)
    assert np.allclose(d_v[0][:, 0], np.tile(d_out[0].sum(axis=0) / N, (N, 1)), atol=1e-12)
    assert np.abs(d_k[0]).max() < 1e-12
    for h in range(H_q):
        dp = vs[0][:, 0] @ d_out[0, h]
        ds = (dp - dp.mean()) / N
        # position 0 for every key would need starts that put all N tokens at 0: they sit at 0..N-1 instead,
        # so compare through the rotation: dq (at position 0) = scale * sum_j ds_j R(j) k_j
        want = sum(ds[j] * orc.rope(ks[0][j:j + 1, 0], np.asarray([j]), 1e4)[0] for j in range(N)) / np.sqrt(D)
        assert np.allclose(d_q[0, h], want, atol=1e-12)
