"""GPU test with the messages placed behind 2.9 million reserved slots: with 8 KV heads the byte offsets of
their K and V rows lie beyond 4 GiB (up to ~6 GiB), so every address computation on the way (append,
plan, prefill, per-call and shared decode, fp32 kernel, position update) has to be 64-bit."""
import sys

import numpy as np
import pytest

import pc_inputs as gen

pytestmark = pytest.mark.gpu

FAR = 2_900_000


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def hip():
    import torch
    from paper_2512_23049_amd import harness
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return harness


def far_workload(seed, dtype, hq, hkv, D, **kw):
    w = gen.small_random(seed, dtype=dtype, n_q_heads=hq, n_kv_heads=hkv, head_dim=D, **kw)
    first = next(e for e in w.events if e.kind == "append")
    first.reserve = FAR                      # message 0 keeps its tokens; everything after it starts behind its reserve
    return w


@pytest.mark.parametrize("sharing", [None, 2])
def test_bf16_rows_beyond_4_gib(hip, sharing):
    from tests.test_gpu_parity import run_and_compare, tables_check
    w = far_workload(4001, "bf16", 32, 8, 128, n_calls=8)
    say("[far] bf16, sharing", sharing)
    tables_check(hip, w, max_calls=3)
    run_and_compare(hip, w, sharing=sharing)


def test_f32_rows_beyond_4_gib(hip):
    from tests.test_gpu_parity import run_and_compare
    w = far_workload(4002, "f32", 8, 8, 64, len_hi=80, max_q=24)
    say("[far] f32")
    run_and_compare(hip, w)


def test_moved_message_beyond_4_gib(hip):
    """pc_reposition (one message and batched) on rows behind 4 GiB: attention results unchanged."""
    import torch
    from tests.helpers import attend_events, oracle_for_event
    from tests.test_gpu_parity import TOL
    w = far_workload(4003, "bf16", 16, 8, 128, n_calls=6)
    cache = hip.make_cache(w)
    dw = hip.DeviceWorkload(w)
    n_msgs = w.n_messages
    for s in dw.steps:
        if s[0] == "append":
            cache.append_message(s[1].data_ptr(), s[2].data_ptr(), s[3], s[4])
    assert cache.message_info(1)[1] >= FAR
    cache.reposition(1, 1234)
    cache.reposition_batch(list(range(2, n_msgs)), [(-1) ** m * (100 + 37 * m) for m in range(2, n_msgs)])
    res = []
    for s in dw.steps:
        if s[0] == "attend":
            _, calls, m, q, out, lse = s
            cache.attend(calls, q.data_ptr(), out.data_ptr(), lse.data_ptr(), 0, m)
            res.append((out, lse))
    torch.cuda.synchronize()
    tol = TOL["bf16"]
    for k, (ei, ev) in enumerate(attend_events(w)):
        out = res[k][0].float().cpu().numpy()
        for ci, rows, o, l in oracle_for_event(w, ei, None, None):
            d = np.abs(out[rows] - o)
            say(f"  call {ci}: max_abs={d.max() if d.size else 0:.3e} mean_abs={d.mean() if d.size else 0:.3e}")
            # moved keys carry one more bf16 rounding: twice the bars
            assert d.size == 0 or (d.max() <= 2 * tol["max_abs"] and d.mean() <= 2 * tol["mean_abs"])
    cache.close()
