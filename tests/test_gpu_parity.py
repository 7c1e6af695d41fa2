"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the
same seeded inputs.  Tolerances: fp32 max-abs 1e-4; bf16 max-abs 2e-2 and mean-abs 1e-3;
gather tables / position maps bit-exact."""
import sys

import numpy as np
import pytest

import pc_inputs as gen
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


def run_and_compare(hip, w, rows_per_call=None, calls_subset=None, events=None, tuning=None, batch_appends=False,
                    lse_rel=0.0, sharing=None, few_key_calls=False, gather=None):
    """few_key_calls: the batch is full of calls whose rows see a handful of keys, so that outputs are of order
    one.  The bf16 result itself is then rounded by about 1.4e-3 of its size on average (a quarter ulp), which
    the fixed mean bar cannot absorb: the mean bar of a call grows by 2^-9 times the mean size of its exact output."""
    import torch
    cache = hip.make_cache(w)
    if tuning:
        cache.set_tuning(*tuning)
    if sharing is not None:
        cache.set_decode_sharing(sharing)
    if gather is not None:
        cache.set_key_gather(gather)
    dw = hip.DeviceWorkload(w)
    say(f"[run] {w.name} dtype={w.dtype} Hq={w.n_q_heads} Hkv={w.n_kv_heads} D={w.head_dim} "
        f"msgs={w.n_messages} attends={len(attend_events(w))}")
    res = dw.run(cache, batch_appends=batch_appends)
    torch.cuda.synchronize()
    tol = TOL[w.dtype]
    worst = 0.0
    for k, (ei, ev) in enumerate(attend_events(w)):
        if events is not None and k not in events:
            continue
        out = res[k][0].float().cpu().numpy()
        lse = res[k][1].cpu().numpy()
        assert np.isfinite(out).all()
        for ci, rows, o, l in oracle_for_event(w, ei, rows_per_call, calls_subset):
            d = np.abs(out[rows] - o)
            say(f"  event {k} call {ci}: rows={len(rows)} max_abs={d.max() if d.size else 0:.3e} "
                f"mean_abs={d.mean() if d.size else 0:.3e}")
            assert d.size == 0 or d.max() <= tol["max_abs"]
            mean_bar = tol["mean_abs"] + (2.0 ** -9 * float(np.abs(o).mean()) if (few_key_calls and d.size) else 0.0)
            assert d.size == 0 or d.mean() <= mean_bar
            fin = np.isfinite(l)
            assert np.array_equal(np.isfinite(lse[rows]), fin)
            assert np.array_equal(np.isneginf(lse[rows]), np.isneginf(l))
            if fin.any():
                assert (np.abs(lse[rows][fin] - l[fin]) <= tol["lse"] + lse_rel * np.abs(l[fin])).all()
            worst = max(worst, d.max() if d.size else 0.0)
    cache.close()
    return worst


def tables_check(hip, w, max_calls=None):
    import torch
    from oracle import choreo_oracle as orc
    from paper_2512_23049_amd import PC_SLOT_ALIGN
    # append lengths only matter: use a host-side walk of the same events on a device cache
    cache = hip.make_cache(w)
    dw = hip.DeviceWorkload(w)
    lens, reserves = [], []
    n_checked = 0
    for s, e in zip(dw.steps, w.events):
        if s[0] == "append":
            cache.append_message(s[1].data_ptr(), s[2].data_ptr(), s[3], s[4])
            lens.append(s[3]); reserves.append(max(s[3], s[4]))
            continue
        for ci, c in enumerate(e.calls):
            if max_calls is not None and ci >= max_calls:
                break
            exp_slot, exp_pos = orc.tables_for_call(c, lens, reserves, PC_SLOT_ALIGN)
            n = cache.build_tables(c, 0, 0, 0)
            assert n == exp_slot.shape[0]
            slot = torch.full((max(n, 1),), -7, dtype=torch.int32, device="cuda:0")
            pos = torch.full((max(n, 1),), -7, dtype=torch.int32, device="cuda:0")
            n2 = cache.build_tables(c, slot.data_ptr(), pos.data_ptr(), n)
            torch.cuda.synchronize()
            assert n2 == n
            assert np.array_equal(slot.cpu().numpy()[:n], exp_slot)
            assert np.array_equal(pos.cpu().numpy()[:n], exp_pos)
            n_checked += 1
    cache.close()
    say(f"[tables] {w.name}: {n_checked} calls bit-exact")


# ------------------------------------------------------------------ config 1 (fp32)
def test_config1_tiny_fp32(hip):
    w = gen.tiny_fp32()
    tables_check(hip, w)
    run_and_compare(hip, w)


@pytest.mark.parametrize("seed", [101, 102])
def test_small_random_fp32(hip, seed):
    w = gen.small_random(seed, dtype="f32", n_q_heads=4, n_kv_heads=2, head_dim=64, len_hi=100)
    tables_check(hip, w)
    run_and_compare(hip, w)


def test_small_random_fp32_d128(hip):
    w = gen.small_random(103, dtype="f32", n_q_heads=6, n_kv_heads=2, head_dim=128, len_hi=70, max_q=20)
    run_and_compare(hip, w)


# ------------------------------------------------------------- bf16, small and ragged
@pytest.mark.parametrize("seed,hq,hkv", [(201, 8, 2), (202, 16, 2), (203, 4, 4), (204, 6, 3), (205, 32, 2)])
def test_small_random_bf16(hip, seed, hq, hkv):
    w = gen.small_random(seed, dtype="bf16", n_q_heads=hq, n_kv_heads=hkv, head_dim=128)
    tables_check(hip, w)
    run_and_compare(hip, w)


@pytest.mark.parametrize("tuning", [(1, 1), (3, 2), (1000, 1000)])
def test_small_random_bf16_split_settings(hip, tuning):
    # KV splits of 1 tile, a few tiles, and no splitting must all agree with the oracle
    w = gen.small_random(211, dtype="bf16", n_q_heads=8, n_kv_heads=2, head_dim=128, len_hi=200, max_q=90)
    run_and_compare(hip, w, tuning=tuning)
    run_and_compare(hip, w, tuning=tuning, gather=GATHER_ALWAYS)


# Key gather (Sec. 2.4 "Position Updates", applied to a copy of the call's keys): prefill calls read keys that a
# pass before the attention kernel turned to the positions the call gives them.  By default only calls with many
# rows take it; here every prefill call of the small and ragged workloads does (mode 2), and none (mode 1).
GATHER_NEVER, GATHER_ALWAYS = 1, 2


@pytest.mark.parametrize("seed,hq,hkv", [(201, 8, 2), (202, 16, 2), (203, 4, 4), (204, 6, 3), (205, 32, 2)])
def test_small_random_bf16_with_gathered_keys(hip, seed, hq, hkv):
    w = gen.small_random(seed, dtype="bf16", n_q_heads=hq, n_kv_heads=hkv, head_dim=128)
    run_and_compare(hip, w, gather=GATHER_ALWAYS)
    run_and_compare(hip, w, gather=GATHER_NEVER)


def test_scaled_configs_with_gathered_keys(hip):
    run_and_compare(hip, gen.single_prefill(n_msgs=24, len_lo=40, len_hi=300, n_sel=6, n_new=200), gather=GATHER_ALWAYS)
    run_and_compare(hip, gen.multi_agent_rounds(n_agents=3, n_rounds=3, msg_len=70), gather=GATHER_ALWAYS, batch_appends=True)
    run_and_compare(hip, gen.long_context(n_msgs=40, len_lo=30, len_hi=120, target_tokens=2500, n_decode=5, n_prefill_q=150),
                    gather=GATHER_ALWAYS)
    run_and_compare(hip, gen.prefix_cache_baseline_rounds(n_agents=3, n_rounds=3, msg_len=40, n_q_heads=8, n_kv_heads=2),
                    gather=GATHER_ALWAYS)


def test_edge_cases_bf16(hip):
    from pc_inputs import Call, Event, Workload, POS_AUTO
    rng = np.random.default_rng(9)
    w = Workload("edges", 8, 2, 128, "bf16", 10000.0)

    def app(L, reserve=0):
        k = gen.round_to_bf16(rng.standard_normal((L, 2, 128), dtype=np.float32))
        v = gen.round_to_bf16(rng.standard_normal((L, 2, 128), dtype=np.float32))
        w.events.append(Event("append", k=k, v=v, reserve=reserve))
        return w.n_messages - 1
    ids = [app(L) for L in (1, 31, 32, 33, 64, 65, 7, 8, 9)] + [app(5, reserve=100)]
    far = (1 << 24) - 70
    calls = [
        Call([], -1, 0, 3, np.array([5, 6, 7], dtype=np.int32)),              # nothing visible
        Call([], ids[0], POS_AUTO, 1, None),                                   # one own token only
        Call([(ids[2], 0)], ids[3], POS_AUTO, 33, None),                       # exact-tile parent, 33-row self
        Call([(ids[1], -far), (ids[5], far - 65)], ids[4], 0, 64, None),       # extreme positions
        Call([(ids[6], 0), (ids[6], 0), (ids[7], 0), (ids[8], 0)], ids[9], 3, 5, None),  # repeats, overlap
        Call([(ids[4], POS_AUTO)] * 5, -1, POS_AUTO, 40, None),                # parents only, AUTO rows
        Call([(ids[3], 10)], ids[3], 10, 33, None),                            # new message also a parent
    ]
    q = gen.round_to_bf16(rng.standard_normal((sum(c.n_q for c in calls), 8, 128), dtype=np.float32))
    w.events.append(Event("attend", calls=calls, q=q))
    tables_check(hip, w)
    run_and_compare(hip, w)
    run_and_compare(hip, w, gather=GATHER_ALWAYS)


def test_empty_batch_and_errors(hip):
    import torch
    from paper_2512_23049_amd import PcError, PC_ERR_BAD_MSG_ID, PC_ERR_INVALID_ARG, PC_ERR_SHAPE, PC_ERR_NO_SPACE
    from pc_inputs import Call
    w = gen.small_random(5, dtype="bf16", n_q_heads=8, n_kv_heads=2, head_dim=128, n_msgs=3, n_calls=1)
    cache = hip.make_cache(w)
    dw = hip.DeviceWorkload(w)
    for s in dw.steps:
        if s[0] == "append":
            cache.append_message(s[1].data_ptr(), s[2].data_ptr(), s[3], s[4])
    q = torch.zeros((4, 8, 128), dtype=torch.bfloat16, device="cuda:0")
    out = torch.ones_like(q)
    cache.attend([], q.data_ptr(), out.data_ptr())                  # no calls: nothing happens
    torch.cuda.synchronize()
    assert (out == 1).all()
    with pytest.raises(PcError) as ei:
        cache.attend([Call([(7, 0)], -1, 0, 1, None)], q.data_ptr(), out.data_ptr())
    assert ei.value.code == PC_ERR_BAD_MSG_ID
    L0 = cache.message_info(0)[0]
    with pytest.raises(PcError) as ei:
        cache.attend([Call([], 0, 0, L0 + 1, None)], q.data_ptr(), out.data_ptr())
    assert ei.value.code == PC_ERR_SHAPE
    with pytest.raises(PcError) as ei:
        big = torch.zeros((10 ** 6, 2, 128), dtype=torch.bfloat16, device="cuda:0")
        cache.append_message(big.data_ptr(), big.data_ptr(), 10 ** 6)
    assert ei.value.code == PC_ERR_NO_SPACE
    with pytest.raises(PcError) as ei:                               # K, V of an append must be 16-byte aligned
        small = torch.zeros((2 * 2 * 128 + 8,), dtype=torch.bfloat16, device="cuda:0")
        cache.append_message(small.data_ptr() + 2, small.data_ptr(), 2)
    assert ei.value.code == PC_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert (out == 1).all()                                          # failed calls enqueue nothing
    cache.close()


# ---------------------------------------------- scaled-down shapes of configs 2-5 (all rows)
def test_config2_scaled(hip):
    w = gen.single_prefill(n_msgs=24, len_lo=40, len_hi=300, n_sel=6, n_new=200)
    tables_check(hip, w)
    run_and_compare(hip, w)


def test_config3_scaled(hip):
    w = gen.parallel_decode(n_calls=12, sys_len=300, n_pool=20, len_lo=50, len_hi=200, n_sel=4, tail_len=64)
    tables_check(hip, w)
    run_and_compare(hip, w)


def test_config4_scaled(hip):
    w = gen.multi_agent_rounds(n_agents=3, n_rounds=3, msg_len=70)
    tables_check(hip, w)
    run_and_compare(hip, w)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_batched_appends(hip, dtype):
    # the messages of a round go through one pc_append_messages launch (ragged lengths, several tiles)
    kw = dict(n_q_heads=4, n_kv_heads=2, head_dim=64) if dtype == "f32" else {}
    w = gen.multi_agent_rounds(n_agents=3, n_rounds=3, msg_len=70, dtype=dtype, **kw)
    run_and_compare(hip, w, batch_appends=True)
    w = gen.small_random(41, dtype=dtype, **kw)
    run_and_compare(hip, w, batch_appends=True)


def test_config5_scaled(hip):
    w = gen.long_context(n_msgs=40, len_lo=30, len_hi=120, target_tokens=2500, n_decode=5, n_prefill_q=150)
    tables_check(hip, w)
    run_and_compare(hip, w)


# (full sizes, in the launch configuration of the benchmark: tests/test_gpu_full_configs.py)


# --------------------------------------------------- properties that hold at any size
def test_shift_and_permutation_on_gpu(hip):
    """Sec. 2.4 "Position Updates": only position differences matter; "Dynamic Masking": what a call sees is a set.
    The same call as listed, with every position moved by 4096, and with its parent list reversed: each of the
    three against the oracle's result for ITS OWN listing, and the oracle's three results against each other
    (they agree to fp64 rounding, so the GPU's three agree to the bf16 bars by the triangle inequality as well)."""
    import torch
    from oracle import choreo_oracle as orc
    from pc_inputs import Call
    from tests.helpers import cache_lists
    w = gen.single_prefill(n_msgs=12, len_lo=20, len_hi=90, n_sel=5, n_new=48)
    ev = w.events[-1]
    c0 = ev.calls[0]
    shifted = Call([(m, s + 4096) for m, s in c0.sel], c0.self_msg, c0.self_start + 4096, c0.n_q, None)
    perm = Call(list(reversed(c0.sel)), c0.self_msg, c0.self_start, c0.n_q, None)
    q0 = ev.q
    ev.calls = [c0, shifted, perm]
    ev.q = np.concatenate([q0, q0, q0], axis=0)
    cache = hip.make_cache(w)
    dw = hip.DeviceWorkload(w)
    (out, lse), = dw.run(cache)
    torch.cuda.synchronize()
    o = out.float().cpu().numpy().reshape(3, c0.n_q, w.n_q_heads, w.head_dim)
    l = lse.cpu().numpy().reshape(3, c0.n_q, w.n_q_heads)
    ks, vs = cache_lists(w, upto_event=len(w.events) - 1)
    refs = []
    for i, c in enumerate(ev.calls):
        ro, rl = orc.attend_call(ks, vs, c.sel, c.self_msg, c.self_start, c.n_q, c.q_pos, q0, w.rope_theta)
        refs.append(ro)
        d = np.abs(o[i] - ro)
        say(f"  listing {i}: max_abs={d.max():.3e} mean_abs={d.mean():.3e}")
        assert d.max() <= 2e-2 and d.mean() <= 1e-3
        assert np.abs(l[i] - rl).max() <= 2e-2
    assert np.abs(refs[0] - refs[1]).max() <= 1e-9 and np.abs(refs[0] - refs[2]).max() <= 1e-9
    cache.close()


def test_prefix_cache_baseline_shape_scaled(hip):
    # the comparator workload of bench.py (long causal new messages over a private prefix), small
    w = gen.prefix_cache_baseline_rounds(n_agents=3, n_rounds=3, msg_len=40, n_q_heads=8, n_kv_heads=2)
    run_and_compare(hip, w)


@pytest.mark.parametrize("n_q", [1, 48])
def test_large_logits_move_the_softmax_reference(hip, n_q):
    """Scores spanning hundreds of log2 units: the reference maximum of the prefill kernel has to
    move up (late keys dominate), start low (every early key far below zero), and the rows of one
    wave end up with different references.  n_q = 1 takes the decode kernel through the same data.
    A bf16 operand carries a relative error of 2^-9, which times a score of several hundred would
    decide which key wins; so the scores are made exact on the GPU: every message is ONE token
    placed at the queries' own position (no rotation on either side, P4: overlapping parents are
    legal) and softmax_scale * log2(e) = 2^-3 (exact when folded into bf16 queries).  One token
    per message also means a ragged tile and a new segment at every tile."""
    import torch
    from oracle import choreo_oracle as orc
    from pc_inputs import Call
    from paper_2512_23049_amd.binding import PC_BF16, Cache
    rng = np.random.default_rng(77)
    H_q, H_kv, D, N = 8, 2, 128, 150
    scale = 2.0 ** -3 / 1.4426950408889634

    def rnd(*shape):
        return gen.round_to_bf16(rng.standard_normal(shape).astype(np.float32))
    ks = [rnd(1, H_kv, D) for _ in range(N)]
    vs = [rnd(1, H_kv, D) for _ in range(N)]
    for i in (97, 98, 131):
        ks[i] *= 8.0                                      # a few dominant keys late in the gathered order
    q = rnd(n_q, H_q, D)
    q *= np.asarray([0.0625, 1.0, 4.0, 8.0, 16.0, 32.0, 2.0, 16.0], dtype=np.float32)[None, :, None]   # per head, exact
    q[::3] *= -1.0                                        # for some rows the dominant keys are the worst ones
    cache = Cache(H_q, H_kv, D, PC_BF16, 10000.0, 32 * (N + 2), N + 4, softmax_scale=scale)
    keep = []
    kd = hip.to_device(np.concatenate(ks), "bf16"); vd = hip.to_device(np.concatenate(vs), "bf16")
    ids = cache.append_messages([kd[i:i + 1].data_ptr() for i in range(N)], [vd[i:i + 1].data_ptr() for i in range(N)], [1] * N)
    qd = hip.to_device(q, "bf16")
    out = torch.empty_like(qd)
    lse = torch.empty((n_q, H_q), dtype=torch.float32, device="cuda:0")
    variants = [((0, 0), 0, 0, 7), ((7, 7), 0, 0, 7)]     # default splits, and splits of seven tiles
    if n_q == 1:
        variants += [((0, 0), 2, 0, 7), ((7, 0), 2, 0, 7)]   # ... and the one-row call on the shared decode walk
    else:
        # ... and the prefill call over a gathered copy of its keys and values: their norms rule out the loop that
        # trusts a bound on the scores, so the packed walk's tested loop has to move the references.  Everything at
        # position 0: the copy's keys are turned to the call's positions and rounded again, which only a turn by
        # nothing leaves exact.
        variants += [((0, 0), 0, 2, 0), ((3, 3), 0, 2, 0)]
    for tuning, sharing, gather, pos in variants:
        call = Call([(m, pos) for m in ids], -1, 0, n_q, np.full(n_q, pos, dtype=np.int32))
        cache.set_tuning(*tuning)
        cache.set_decode_sharing(sharing)
        cache.set_key_gather(gather)
        cache.attend([call], qd.data_ptr(), out.data_ptr(), lse.data_ptr())
        torch.cuda.synchronize()
        o, l = orc.attend_call(ks, vs, call.sel, -1, 0, n_q, call.q_pos, q, 10000.0, scale=scale)
        got = out.float().cpu().numpy()
        d = np.abs(got - o)
        e_lse = np.abs(lse.cpu().numpy() - l)
        say(f"  n_q={n_q} tuning={tuning} sharing={sharing} gather={gather}: max_abs={d.max():.3e} mean_abs={d.mean():.3e} "
            f"lse range [{l.min():.1f}, {l.max():.1f}] max lse err {e_lse.max():.3e}")
        assert np.isfinite(got).all()
        assert d.max() <= 2e-2 and d.mean() <= 1e-3
        assert (e_lse <= 2e-2 + 1e-5 * np.abs(l)).all()
    cache.close()


def test_packed_walk_with_scores_just_inside_the_norm_bound(hip):
    """The packed prefill walk skips the test for a moving softmax reference when |q| |k| (largest query row of the
    wave, largest key of the call) stays below the threshold of 2^64: then probabilities up to 2^56 are accumulated
    against the reference 0.  Keys and queries here are built so that the bound holds but is nearly reached by one
    key that is parallel to some query rows (and anti-parallel to others): entries +-1, one-token messages at position
    0 (no rotation, scores exact on the GPU), softmax_scale * log2(e) = 2^-3."""
    import torch
    from oracle import choreo_oracle as orc
    from pc_inputs import Call
    from paper_2512_23049_amd.binding import PC_BF16, Cache
    rng = np.random.default_rng(78)
    H_q, H_kv, D, N, n_q = 8, 2, 128, 150, 48
    scale = 2.0 ** -3 / 1.4426950408889634
    sign = lambda *shape: rng.choice(np.float32([-1.0, 1.0]), size=shape)
    u = sign(H_kv, D)                                     # one direction per KV head
    ks = [sign(1, H_kv, D) for _ in range(N)]
    vs = [gen.round_to_bf16(rng.standard_normal((1, H_kv, D)).astype(np.float32)) for _ in range(N)]
    ks[101] = (1.75 * u)[None]                            # |k| = 1.75 sqrt(128); every other key sqrt(128)
    q = sign(n_q, H_q, D)
    g = H_q // H_kv
    for r in range(0, n_q, 4):                            # every fourth row: +-2 u in all heads -> score +-2 * 1.75 * 128 / 8 = +-56
        for h in range(H_q):
            q[r, h] = (2.0 if r % 8 == 0 else -2.0) * u[h // g]
    cache = Cache(H_q, H_kv, D, PC_BF16, 10000.0, 32 * (N + 2), N + 4, softmax_scale=scale)
    kd = hip.to_device(np.concatenate(ks), "bf16"); vd = hip.to_device(np.concatenate(vs), "bf16")
    ids = cache.append_messages([kd[i:i + 1].data_ptr() for i in range(N)], [vd[i:i + 1].data_ptr() for i in range(N)], [1] * N)
    call = Call([(m, 0) for m in ids], -1, 0, n_q, np.zeros(n_q, dtype=np.int32))
    qd = hip.to_device(q, "bf16")
    out = torch.empty_like(qd)
    lse = torch.empty((n_q, H_q), dtype=torch.float32, device="cuda:0")
    o, l = orc.attend_call(ks, vs, call.sel, -1, 0, n_q, call.q_pos, q, 10000.0, scale=scale)
    assert l.max() > 38.0                                 # 56 log2 units: the bound is nearly reached
    for gather in (2, 1):                                 # the packed walk, and the in-place walk beside it
        cache.set_key_gather(gather)
        cache.attend([call], qd.data_ptr(), out.data_ptr(), lse.data_ptr())
        torch.cuda.synchronize()
        got = out.float().cpu().numpy()
        d = np.abs(got - o)
        e_lse = np.abs(lse.cpu().numpy() - l)
        say(f"  gather={gather}: max_abs={d.max():.3e} mean_abs={d.mean():.3e} lse range [{l.min():.1f}, {l.max():.1f}] "
            f"max lse err {e_lse.max():.3e}")
        assert np.isfinite(got).all()
        assert d.max() <= 2e-2 and d.mean() <= 1e-3
        assert (e_lse <= 2e-2 + 1e-5 * np.abs(l)).all()
    cache.close()


def test_decode_result_does_not_depend_on_parent_order(hip):
    """Sec. 2.4 "Dynamic Masking" / "Position Updates": what a call sees is a set of messages, each
    with its own start position; the order they are listed in carries no information once every
    start is given explicitly.  The decode path walks parents in cache order, so two listings of
    the same (message, start) pairs must give the same bits, and both must match the oracle."""
    import torch
    from oracle import choreo_oracle as orc
    from pc_inputs import Call
    from paper_2512_23049_amd.binding import PC_BF16, Cache
    rng = np.random.default_rng(91)
    H_q, H_kv, D = 16, 4, 128
    lens = [70, 33, 1, 128, 257, 64, 5, 96, 40, 31, 200, 17]

    def rnd(*shape):
        return gen.round_to_bf16(rng.standard_normal(shape).astype(np.float32))
    ks = [rnd(L, H_kv, D) for L in lens]
    vs = [rnd(L, H_kv, D) for L in lens]
    cache = Cache(H_q, H_kv, D, PC_BF16, 10000.0, 4096, 32)
    keep = []
    for k, v in zip(ks, vs):
        kd, vd = hip.to_device(k, "bf16"), hip.to_device(v, "bf16")
        keep += [kd, vd]
        cache.append_message(kd.data_ptr(), vd.data_ptr(), k.shape[0], 0)
    # scattered, partly overlapping, partly negative starts; message 3 is listed twice at two places
    pairs = [(0, 500), (4, -40), (3, 0), (9, 1200), (1, 77), (3, 640), (10, 900), (6, 3), (2, 1500), (7, 260), (5, 320), (8, 2000)]
    q = rnd(3, H_q, D)
    qd = hip.to_device(q, "bf16")
    q_pos = np.asarray([2100, 2100, 2100], dtype=np.int32)
    outs = []
    for order in (np.arange(len(pairs)), rng.permutation(len(pairs)), np.arange(len(pairs))[::-1]):
        sel = [pairs[i] for i in order]
        calls = [Call(sel, -1, 0, 1, q_pos[r:r + 1]) for r in range(3)]          # three one-row decode calls
        out = torch.empty_like(qd)
        lse = torch.empty((3, H_q), dtype=torch.float32, device="cuda:0")
        cache.attend(calls, qd.data_ptr(), out.data_ptr(), lse.data_ptr())
        torch.cuda.synchronize()
        outs.append((out.cpu(), lse.cpu()))
        for r in range(3):
            o, l = orc.attend_call(ks, vs, sel, -1, 0, 1, q_pos[r:r + 1], q[r:r + 1], 10000.0)
            d = np.abs(out[r:r + 1].float().cpu().numpy() - o)
            assert d.max() <= 2e-2 and d.mean() <= 1e-3
            assert np.abs(lse[r:r + 1].cpu().numpy() - l).max() <= 2e-2
    for o, l in outs[1:]:
        assert torch.equal(o.view(torch.int16), outs[0][0].view(torch.int16)), "listing order changed the result bits"
        assert torch.equal(l, outs[0][1])
    cache.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_positions_far_from_zero(hip, dtype):
    """Sec. 2.4 "Position Updates": only position differences matter, however large the positions.  The same calls
    placed around +-10^7 (angles of millions of radians at the highest frequency: the rotation tables are built in
    fp64 from integer positions) against the oracle; prefill, decode per call and decode through the shared walk."""
    import torch
    from oracle import choreo_oracle as orc
    from pc_inputs import Call
    from paper_2512_23049_amd.binding import PC_BF16, PC_F32, Cache
    rng = np.random.default_rng(55)
    H_q, H_kv, D = (8, 2, 128) if dtype == "bf16" else (4, 2, 64)
    tol = TOL[dtype]
    lens = [70, 33, 128, 40, 9]

    def rnd(*shape):
        x = rng.standard_normal(shape).astype(np.float32)
        return gen.round_to_bf16(x) if dtype == "bf16" else x
    ks = [rnd(L, H_kv, D) for L in lens]
    vs = [rnd(L, H_kv, D) for L in lens]
    cache = Cache(H_q, H_kv, D, PC_BF16 if dtype == "bf16" else PC_F32, 500000.0, 2048, 16)
    keep = []
    for k, v in zip(ks, vs):
        kd, vd = hip.to_device(k, dtype), hip.to_device(v, dtype)
        keep += [kd, vd]
        cache.append_message(kd.data_ptr(), vd.data_ptr(), k.shape[0], 0)
    far = 10_000_000
    for sign in (1, -1):
        base = sign * far
        calls = [Call([(0, base), (2, base + 70), (1, base + 150)], 3, base + 200, 40, None),              # prefill
                 Call([(2, base - 300), (0, base - 100)], 4, base, 1, None),                                # decode
                 Call([(0, base - 100), (2, base - 300), (1, base - 400)], -1, 0, 1, np.asarray([base + 5], dtype=np.int32))]
        n_rows = sum(c.n_q for c in calls)
        q = rnd(n_rows, H_q, D)
        qd = hip.to_device(q, dtype)
        for mode in ((1, 2) if dtype == "bf16" else (1,)):
            cache.set_decode_sharing(mode)
            out = torch.empty_like(qd)
            lse = torch.empty((n_rows, H_q), dtype=torch.float32, device="cuda:0")
            cache.attend(calls, qd.data_ptr(), out.data_ptr(), lse.data_ptr())
            torch.cuda.synchronize()
            at = 0
            for c in calls:
                o, l = orc.attend_call(ks, vs, c.sel, c.self_msg, c.self_start, c.n_q, c.q_pos, q[at:at + c.n_q], 500000.0)
                d = np.abs(out[at:at + c.n_q].float().cpu().numpy() - o)
                say(f"  {dtype} base {base} mode {mode}: max_abs={d.max():.3e} mean_abs={d.mean():.3e}")
                assert d.max() <= tol["max_abs"] and d.mean() <= tol["mean_abs"]
                assert np.abs(lse[at:at + c.n_q].cpu().numpy() - l).max() <= tol["lse"]
                at += c.n_q
    cache.close()


@pytest.mark.parametrize("sharing", [None, 2])
def test_calls_with_more_than_a_thousand_parents(hip, sharing):
    """Calls that list more messages than the plan builder keeps on chip (it then searches the segment
    list in device memory), most of them shorter than a tile: prefill and decode, repeats included."""
    from pc_inputs import Call, Event, Workload, POS_AUTO
    rng = np.random.default_rng(77)
    w = Workload("many_parents", 8, 2, 128, "bf16", 10000.0)
    n_msgs = 1400
    lens = rng.integers(1, 4, size=n_msgs)
    lens[::97] = 40                                        # a few that span two tiles
    for L in lens:
        k = gen.round_to_bf16(rng.standard_normal((int(L), 2, 128), dtype=np.float32))
        v = gen.round_to_bf16(rng.standard_normal((int(L), 2, 128), dtype=np.float32))
        w.events.append(Event("append", k=k, v=v))
    tails = []
    for _ in range(5):
        k = gen.round_to_bf16(rng.standard_normal((48, 2, 128), dtype=np.float32))
        v = gen.round_to_bf16(rng.standard_normal((48, 2, 128), dtype=np.float32))
        w.events.append(Event("append", k=k, v=v))
        tails.append(w.n_messages - 1)

    def parents(n, repeat=0):
        order = rng.permutation(n_msgs)[:n]
        if repeat:
            order = np.concatenate([order, order[:repeat]])
        pos, sel = 0, []
        for m in order:
            sel.append((int(m), pos))
            pos += int(lens[m]) + int(rng.integers(0, 3))
        return sel, pos
    calls = []
    sel, end = parents(1100, repeat=30)
    calls.append(Call(sel, tails[0], end + 5, 48, None))                      # prefill, 1131 segments
    for t in tails[1:]:
        sel, end = parents(1300)
        calls.append(Call(sel, t, end, 1, None))                              # decode, 1301 segments each
    q = gen.round_to_bf16(rng.standard_normal((sum(c.n_q for c in calls), 8, 128), dtype=np.float32))
    w.events.append(Event("attend", calls=calls, q=q))
    tables_check(hip, w, max_calls=2)
    run_and_compare(hip, w, sharing=sharing)
    if sharing is None:
        run_and_compare(hip, w, gather=GATHER_ALWAYS)


@pytest.mark.parametrize("sharing", [None, 2])
def test_batch_of_fifteen_hundred_one_row_calls(hip, sharing):
    """A large parallel step: 1500 one-row calls in one pc_attend (per-call walk, and groups on the shared walk)."""
    w = gen.small_random(88, dtype="bf16", n_q_heads=8, n_kv_heads=2, head_dim=128, n_msgs=40, n_calls=1500, max_q=1)
    run_and_compare(hip, w, sharing=sharing, few_key_calls=True)


def test_batch_of_many_small_prefill_calls(hip):
    """400 calls of up to 12 rows each in one pc_attend."""
    w = gen.small_random(89, dtype="bf16", n_q_heads=8, n_kv_heads=2, head_dim=128, n_msgs=40, n_calls=400, max_q=12)
    run_and_compare(hip, w, few_key_calls=True)


@pytest.mark.parametrize("n_q,sharing", [(40, 0), (1, 1), (1, 2)])
def test_first_key_far_below_every_other(hip, n_q, sharing):
    """A call whose first visible key scores thousands of log2 units below the rest, for every row: its weight
    is zero, and the softmax reference, which starts at 0, has to move down by more than fp32's exponent range
    at that first tile without disturbing what follows (prefill, per-call decode and shared decode)."""
    import torch
    from oracle import choreo_oracle as orc
    from pc_inputs import Call
    from paper_2512_23049_amd.binding import PC_BF16, Cache
    rng = np.random.default_rng(5)
    H_q, H_kv, D = 8, 2, 128
    u = np.where(np.arange(D) % 3 == 0, -1.0, 1.0).astype(np.float32)

    def rnd(*shape):
        return gen.round_to_bf16(rng.standard_normal(shape).astype(np.float32))
    k_far = gen.round_to_bf16(np.broadcast_to(-64.0 * u, (1, H_kv, D)).copy())
    ks = [k_far] + [rnd(1, H_kv, D) for _ in range(70)]   # one-token messages: each sits exactly at the queries' position
    vs = [rnd(1, H_kv, D) for _ in range(71)]
    q = gen.round_to_bf16(rnd(n_q, H_q, D) + 3.0 * u[None, None, :])
    # (scores exact on the GPU, as in the test above: no rotation, and softmax_scale * log2(e) = 2^-3 folds
    # into the bf16 queries without rounding; the bf16 bars are for scores that carry no rounding of their own)
    scale = 2.0 ** -3 / 1.4426950408889634
    cache = Cache(H_q, H_kv, D, PC_BF16, 10000.0, 4096, 80, softmax_scale=scale)
    cache.set_decode_sharing(sharing)
    keep = [(hip.to_device(k, "bf16"), hip.to_device(v, "bf16")) for k, v in zip(ks, vs)]
    ids = [cache.append_message(kd.data_ptr(), vd.data_ptr(), k.shape[0]) for (kd, vd), k in zip(keep, ks)]
    pos = 300
    # every key at the queries' own position: no rotation, so the far key stays far for every row
    call = Call([(m, pos) for m in ids], -1, 0, n_q, np.full(n_q, pos, dtype=np.int32))
    qd = hip.to_device(q, "bf16")
    out = torch.empty_like(qd)
    lse = torch.empty((n_q, H_q), dtype=torch.float32, device="cuda:0")
    for tuning in ((0, 0), (9, 9)):
        cache.set_tuning(*tuning)
        cache.attend([call], qd.data_ptr(), out.data_ptr(), lse.data_ptr())
        torch.cuda.synchronize()
        o, l = orc.attend_call(ks, vs, call.sel, -1, 0, n_q, call.q_pos, q, 10000.0, scale=scale)
        got = out.float().cpu().numpy()
        d = np.abs(got - o)
        say(f"  n_q={n_q} sharing={sharing} tuning={tuning}: max_abs={d.max():.3e} mean_abs={d.mean():.3e}")
        assert np.isfinite(got).all() and np.isfinite(lse.cpu().numpy()).all()
        assert d.max() <= 2e-2 and d.mean() <= 1e-3
        assert (np.abs(lse.cpu().numpy() - l) <= 2e-2 + 1e-3 * np.abs(l)).all()
    cache.close()
