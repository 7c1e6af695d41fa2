"""GPU tests of the shared decode walk (Sec. 2.4 "Parallel decoding": parallel one-row calls
read the same cached messages): a group of calls reads the union of their messages once.  The
result of every call must match the fp64 oracle to the bf16 bars (max-abs 2e-2, mean-abs 1e-3)
whichever walk serves it, and the two walks must agree with each other to the same bars."""
import sys

import numpy as np
import pytest

import pc_inputs as gen
from pc_inputs import Call
from tests.test_gpu_parity import run_and_compare

pytestmark = pytest.mark.gpu

ALWAYS, NEVER, AUTO = 2, 1, 0


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def hip():
    import torch
    from paper_2512_23049_amd import harness
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return harness


@pytest.mark.parametrize("hq,hkv", [(16, 2), (8, 2), (4, 2), (2, 2), (64, 8)])
def test_parallel_decode_shapes_shared(hip, hq, hkv):
    # g = 8, 4, 2, 1: one to eight blocks of 32 rows per workgroup; 40 calls = more than one block
    # for g = 8 (two groups) and a ragged block for the others
    w = gen.parallel_decode(n_calls=40, sys_len=300, n_pool=20, len_lo=50, len_hi=200, n_sel=4, tail_len=64,
                            n_q_heads=hq, n_kv_heads=hkv)
    run_and_compare(hip, w, sharing=ALWAYS)


@pytest.mark.parametrize("tuning", [(1, 0), (3, 0), (1000, 0)])
def test_shared_decode_splits(hip, tuning):
    # one tile per split, three tiles per split, everything in one split
    w = gen.parallel_decode(n_calls=12, sys_len=300, n_pool=20, len_lo=50, len_hi=200, n_sel=4, tail_len=64)
    run_and_compare(hip, w, sharing=ALWAYS, tuning=tuning)


def test_long_context_shape_shared_and_mixed(hip):
    # decode calls over mostly the same messages, each in its own order with overlapping placements, and a
    # prefill call in the same batch (which keeps its own kernel)
    w = gen.long_context(n_msgs=40, len_lo=30, len_hi=120, target_tokens=2500, n_decode=5, n_prefill_q=150)
    run_and_compare(hip, w, sharing=ALWAYS)
    run_and_compare(hip, w, sharing=AUTO)


def test_small_random_batches_shared(hip):
    # mixed batches with one-row calls scattered between longer ones: runs of one call, empty parent
    # lists, one-token messages
    # (g = 8, 16, 1, 2, 16: the walk is built for g in {1, 2, 4, 8}; other shapes keep the per-call walk)
    for seed, hq, hkv in [(201, 8, 2), (202, 16, 2), (203, 4, 4), (204, 6, 3), (205, 32, 2)]:
        w = gen.small_random(seed, n_q_heads=hq, n_kv_heads=hkv)
        run_and_compare(hip, w, sharing=ALWAYS)


def test_decode_loop_shared(hip):
    # growing tails: the tail of a call is a message only its own row sees
    w = gen.decode_loop(n_calls=6, n_steps=9, sys_len=70, n_pool=10, len_lo=20, len_hi=90, n_sel=3)
    run_and_compare(hip, w, sharing=ALWAYS)


def test_shared_walk_hand_made_cases(hip):
    """A message listed twice in one call at two places, a call that lists nothing, a call that is only
    its own tail, repositioned messages, starts that differ per call, negative and overlapping positions;
    checked against the oracle and against the per-call walk."""
    import torch
    from oracle import choreo_oracle as orc
    from paper_2512_23049_amd.binding import PC_BF16, Cache
    rng = np.random.default_rng(123)
    H_q, H_kv, D = 16, 2, 128
    lens = [70, 33, 1, 128, 257, 64, 5, 96, 40, 31]

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
    cache.reposition(4, 1000)                               # stored bases other than 0
    cache.reposition(7, -50)
    calls = [
        Call([(0, 500), (4, -40), (3, 0), (3, 640), (1, 77)], 8, 2000, 1, None),       # message 3 twice; own tail 8
        Call([(4, 1000), (0, 0)], -1, 0, 1, np.asarray([1500], dtype=np.int32)),          # message 4 at its stored base
        Call([], -1, 0, 1, np.asarray([3], dtype=np.int32)),                              # sees nothing
        Call([], 9, 10, 1, None),                                                         # only its own tail
        Call([(7, 20), (4, 30), (2, 0), (6, 1), (5, 300)], 5, 400, 1, None),              # own tail also listed as a parent
        Call([(3, 5), (3, 5)], -1, 0, 1, np.asarray([200], dtype=np.int32)),              # the same placement twice
    ]
    n = len(calls)
    q = rnd(n, H_q, D)
    qd = hip.to_device(q, "bf16")
    res = {}
    for mode in (ALWAYS, NEVER):
        cache.set_decode_sharing(mode)
        for tuning in ((0, 0), (2, 0)):
            cache.set_tuning(*tuning)
            out = torch.full_like(qd, 7.0)
            lse = torch.full((n, H_q), 7.0, dtype=torch.float32, device="cuda:0")
            cache.attend(calls, qd.data_ptr(), out.data_ptr(), lse.data_ptr())
            torch.cuda.synchronize()
            res[(mode, tuning)] = (out.float().cpu().numpy(), lse.cpu().numpy())
    bases = {4: 1000, 7: -50}
    for r, c in enumerate(calls):
        o, l = orc.attend_call(ks, vs, c.sel, c.self_msg, c.self_start, 1, c.q_pos, q[r:r + 1], 10000.0)
        for key, (out, lse) in res.items():
            d = np.abs(out[r:r + 1] - o)
            say(f"  call {r} {key}: max_abs={d.max():.3e} mean_abs={d.mean():.3e}")
            # moved messages carry one more bf16 rounding of their keys: twice the bars (error grows as sqrt(n + 1))
            moved = any(m in bases for m, _ in c.sel)
            f = 2.0 if moved else 1.0
            assert d.max() <= f * 2e-2 and d.mean() <= f * 1e-3
            if np.isfinite(l).all():
                assert np.abs(lse[r:r + 1] - l).max() <= f * 2e-2
            else:
                assert np.isneginf(lse[r]).all() and (out[r] == 0).all()
    cache.close()


# (configs[2] and configs[4] at full size through this walk: tests/test_gpu_full_configs.py)
