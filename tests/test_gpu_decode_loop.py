"""GPU tests of pc_append_tokens / pc_append_tokens_batch: messages that grow inside their
reserve (Sec. 2.4: decode tails of parallel calls), compared with the oracle over the
concatenated messages after every step."""
import sys

import numpy as np
import pytest

import pc_inputs as gen
from pc_inputs import Call, Event, Workload
from tests.helpers import attend_events, oracle_for_event

pytestmark = pytest.mark.gpu

TOL = {"f32": dict(max_abs=1e-4, mean_abs=1e-5, lse=1e-4),
       "bf16": dict(max_abs=2e-2, mean_abs=1e-3, lse=2e-2)}


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def hip():
    import torch
    from paper_2512_23049_amd import harness
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return harness


def run_and_compare(hip, w, fused_steps=False, sharing=None, flags=0):
    import torch
    cache = hip.make_cache(w, slack_tokens=2048 if flags else 0, extra_messages=64 if flags else 0,
                           **({"flags": flags} if flags else {}))
    if sharing is not None:
        cache.set_decode_sharing(sharing)
    dw = hip.DeviceWorkload(w)
    res = dw.run(cache, fused_steps=fused_steps)
    torch.cuda.synchronize()
    tol = TOL[w.dtype]
    for k, (ei, ev) in enumerate(attend_events(w)):
        out = res[k][0].float().cpu().numpy()
        lse = res[k][1].cpu().numpy()
        for ci, rows, o, l in oracle_for_event(w, ei):
            d = np.abs(out[rows] - o)
            assert d.max() <= tol["max_abs"], (k, ci, d.max())
            assert d.mean() <= tol["mean_abs"], (k, ci, d.mean())
            assert np.abs(lse[rows] - l).max() <= tol["lse"]
        say(f"  attend {k}: {len(ev.calls)} calls ok")
    lens = w.message_lengths()
    for m, L in enumerate(lens):
        assert cache.message_info(m)[0] == L
    cache.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_small_decode_loop(hip, dtype):
    kw = dict(n_q_heads=4, n_kv_heads=2, head_dim=64) if dtype == "f32" else dict(n_q_heads=8, n_kv_heads=2)
    w = gen.decode_loop(seed=61, n_calls=6, n_steps=5, sys_len=70, n_pool=10, len_lo=5, len_hi=90, n_sel=3,
                        tail0=3, dtype=dtype, **kw)
    say(f"[decode loop] {dtype}: {w.n_messages} messages, {len(attend_events(w))} steps")
    run_and_compare(hip, w)


def test_tail_crossing_tile_and_group_boundaries(hip):
    # tails grow from 29 to 36 tokens: across the 32-slot tile edge and several 8-slot V groups
    w = gen.decode_loop(seed=62, n_calls=3, n_steps=7, sys_len=40, n_pool=4, len_lo=10, len_hi=40, n_sel=2,
                        tail0=29, n_q_heads=8, n_kv_heads=2)
    run_and_compare(hip, w)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_decode_steps_in_one_call(hip, dtype):
    """pc_decode_step (token append and attention of a parallel decode step in one call, the append running beside
    the plan builder) against the oracle at every step: plain tails, tails crossing tile and group boundaries, the
    shared walk, and tails that grow into further extents (which makes the step fall back to one after the other)."""
    from paper_2512_23049_amd import PC_FLAG_GROW_EXTENTS
    kw = dict(n_q_heads=4, n_kv_heads=2, head_dim=64) if dtype == "f32" else dict(n_q_heads=8, n_kv_heads=2)
    w = gen.decode_loop(seed=61, n_calls=6, n_steps=5, sys_len=70, n_pool=10, len_lo=5, len_hi=90, n_sel=3,
                        tail0=3, dtype=dtype, **kw)
    run_and_compare(hip, w, fused_steps=True)
    w = gen.decode_loop(seed=62, n_calls=3, n_steps=7, sys_len=40, n_pool=4, len_lo=10, len_hi=40, n_sel=2,
                        tail0=29, dtype=dtype, **kw)
    run_and_compare(hip, w, fused_steps=True)
    if dtype == "bf16":
        run_and_compare(hip, w, fused_steps=True, sharing=2)
    # reserves of one tile: the tails (29 tokens at first) outgrow them in the fourth step
    w = gen.decode_loop(seed=65, n_calls=4, n_steps=9, sys_len=40, n_pool=4, len_lo=10, len_hi=40, n_sel=2,
                        tail0=29, dtype=dtype, **kw)
    for e in w.events:
        if e.kind == "append" and e.reserve > e.k.shape[0]:
            e.reserve = 32
    run_and_compare(hip, w, fused_steps=True, flags=PC_FLAG_GROW_EXTENTS)


def test_decode_step_with_a_grown_message_listed_as_a_parent(hip):
    """A step in which one call lists another call's growing tail as a parent: the parent's length is read from the
    device table, so the append has to come first; the result must see the new token."""
    import torch
    from oracle import choreo_oracle as orc
    from paper_2512_23049_amd.binding import PC_BF16, Cache
    rng = np.random.default_rng(66)
    H_q, H_kv, D = 8, 2, 128

    def rnd(*shape):
        return gen.round_to_bf16(rng.standard_normal(shape).astype(np.float32))
    cache = Cache(H_q, H_kv, D, PC_BF16, 10000.0, 1024, 16)
    ks = [rnd(40, H_kv, D), rnd(5, H_kv, D), rnd(9, H_kv, D)]
    vs = [rnd(40, H_kv, D), rnd(5, H_kv, D), rnd(9, H_kv, D)]
    keep = []
    for k, v in zip(ks, vs):
        kd, vd = hip.to_device(k, "bf16"), hip.to_device(v, "bf16")
        keep += [kd, vd]
        cache.append_message(kd.data_ptr(), vd.data_ptr(), k.shape[0], 64)
    for step in range(3):
        k1, v1 = rnd(2, H_kv, D), rnd(2, H_kv, D)
        kd, vd = hip.to_device(k1, "bf16"), hip.to_device(v1, "bf16")
        keep += [kd, vd]
        calls = [Call([(0, 0), (2, 60)], 1, 100, 1, None),          # lists message 2, which grows in this very step
                 Call([(0, 0)], 2, 50, 1, None)]
        q = rnd(2, H_q, D)
        qd = hip.to_device(q, "bf16")
        out = torch.empty_like(qd)
        lse = torch.empty((2, H_q), dtype=torch.float32, device="cuda:0")
        cache.decode_step([1, 2], kd.data_ptr(), vd.data_ptr(), calls, qd.data_ptr(), out.data_ptr(), lse.data_ptr())
        torch.cuda.synchronize()
        ks[1] = np.concatenate([ks[1], k1[0:1]]); vs[1] = np.concatenate([vs[1], v1[0:1]])
        ks[2] = np.concatenate([ks[2], k1[1:2]]); vs[2] = np.concatenate([vs[2], v1[1:2]])
        for r, c in enumerate(calls):
            o, l = orc.attend_call(ks, vs, c.sel, c.self_msg, c.self_start, 1, None, q[r:r + 1], 10000.0)
            d = np.abs(out[r:r + 1].float().cpu().numpy() - o)
            say(f"  step {step} call {r}: max_abs={d.max():.3e}")
            assert d.max() <= 2e-2 and d.mean() <= 1e-3
            assert np.abs(lse[r:r + 1].cpu().numpy() - l).max() <= 2e-2
    cache.close()


def test_chunked_prefill_with_append_tokens(hip):
    """A message appended in three pieces (7 + 20 + 6 tokens); after each piece the new tokens
    attend as query rows aligned with the message's last tokens."""
    import torch
    rng = np.random.default_rng(63)
    H_q, H_kv, D = 8, 2, 128
    w = Workload("chunked", H_q, H_kv, D, "bf16", 10000.0)
    def rnd(*shape):
        return gen.round_to_bf16(rng.standard_normal(shape).astype(np.float32))
    w.events.append(Event("append", k=rnd(50, H_kv, D), v=rnd(50, H_kv, D)))
    pieces = [7, 20, 6]
    w.events.append(Event("append", k=rnd(pieces[0], H_kv, D), v=rnd(pieces[0], H_kv, D), reserve=sum(pieces)))
    cache = hip.make_cache(w)
    ks = [w.events[0].k, w.events[1].k]
    vs = [w.events[0].v, w.events[1].v]
    dev = lambda x: hip.to_device(x, "bf16")
    keep = []                                            # device inputs stay alive until the kernels have run
    for e in w.events:
        kd, vd = dev(e.k), dev(e.v)
        keep += [kd, vd]
        cache.append_message(kd.data_ptr(), vd.data_ptr(), e.k.shape[0], e.reserve)
    from oracle import choreo_oracle as orc
    for step, n_new in enumerate(pieces):
        if step > 0:
            k_new, v_new = rnd(n_new, H_kv, D), rnd(n_new, H_kv, D)
            kd, vd = dev(k_new), dev(v_new)
            keep += [kd, vd]
            cache.append_tokens(1, kd.data_ptr(), vd.data_ptr(), n_new)
            ks[1] = np.concatenate([ks[1], k_new]); vs[1] = np.concatenate([vs[1], v_new])
        call = Call([(0, 5)], 1, 100, n_new, None)
        q = rnd(n_new, H_q, D)
        qd = dev(q)
        out = torch.empty_like(qd)
        lse = torch.empty((n_new, H_q), dtype=torch.float32, device="cuda:0")
        cache.attend([call], qd.data_ptr(), out.data_ptr(), lse.data_ptr())
        torch.cuda.synchronize()
        o, l = orc.attend_call(ks, vs, call.sel, 1, 100, n_new, None, q, 10000.0)
        d = np.abs(out.float().cpu().numpy() - o)
        say(f"  piece {step}: message holds {ks[1].shape[0]} tokens, max_abs={d.max():.3e}")
        assert d.max() <= 2e-2 and d.mean() <= 1e-3
        assert np.abs(lse.cpu().numpy() - l).max() <= 2e-2
    cache.close()


def test_errors(hip):
    import torch
    from paper_2512_23049_amd.binding import PcError, PC_ERR_BAD_MSG_ID, PC_ERR_INVALID_ARG, PC_ERR_NO_SPACE
    w = gen.small_random(64, dtype="bf16")
    cache = hip.make_cache(w, slack_tokens=256)
    x = torch.zeros(8, w.n_kv_heads, w.head_dim, dtype=torch.bfloat16, device="cuda:0")
    a = cache.append_message(x.data_ptr(), x.data_ptr(), 3, 5)
    b = cache.append_message(x.data_ptr(), x.data_ptr(), 2, 2)
    for fn, code in [(lambda: cache.append_tokens(a, x.data_ptr(), x.data_ptr(), 3), PC_ERR_NO_SPACE),
                     (lambda: cache.append_tokens(b, x.data_ptr(), x.data_ptr(), 1), PC_ERR_NO_SPACE),
                     (lambda: cache.append_tokens(a, x.data_ptr(), x.data_ptr(), 0), PC_ERR_INVALID_ARG),
                     (lambda: cache.append_tokens(7, x.data_ptr(), x.data_ptr(), 1), PC_ERR_BAD_MSG_ID),
                     (lambda: cache.append_tokens_batch([a, a], x.data_ptr(), x.data_ptr()), PC_ERR_INVALID_ARG),
                     (lambda: cache.append_tokens_batch([a, b], x.data_ptr(), x.data_ptr()), PC_ERR_NO_SPACE)]:
        with pytest.raises(PcError) as e:
            fn()
        assert e.value.code == code
    assert cache.message_info(a)[0] == 3                 # a refused call changes nothing
    cache.append_tokens(a, x.data_ptr(), x.data_ptr(), 2)
    assert cache.message_info(a)[0] == 5
    cache.append_tokens_batch([], 0, 0)
    torch.cuda.synchronize()
    cache.close()
