"""GPU test of messages that grow into further extents (PC_FLAG_GROW_EXTENTS; Sec. 2.4: the cache maps a
message id to where its tokens live, and the tails of parallel decode calls keep growing): whatever
the physical layout, a call sees one sequence of tokens.  Every attend is checked against the fp64
oracle, which knows nothing of extents."""
import sys

import numpy as np
import pytest

import pc_inputs as gen
from pc_inputs import Call

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def hip():
    import torch
    from paper_2512_23049_amd import harness
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return harness


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_tails_growing_across_extents(hip, dtype):
    import torch
    from oracle import choreo_oracle as orc
    from paper_2512_23049_amd.binding import PC_BF16, PC_F32, PC_FLAG_GROW_EXTENTS, Cache
    rng = np.random.default_rng(31)
    H_q, H_kv, D = (8, 2, 128) if dtype == "bf16" else (4, 2, 64)
    tol = dict(max_abs=2e-2, mean_abs=1e-3, lse=2e-2) if dtype == "bf16" else dict(max_abs=1e-4, mean_abs=1e-5, lse=1e-4)

    def rnd(*shape):
        x = rng.standard_normal(shape).astype(np.float32)
        return gen.round_to_bf16(x) if dtype == "bf16" else x
    cache = Cache(H_q, H_kv, D, PC_BF16 if dtype == "bf16" else PC_F32, 10000.0, 8192, 128, flags=PC_FLAG_GROW_EXTENTS)
    ks, vs, keep = {}, {}, []

    def append(L, reserve=0):
        k, v = rnd(L, H_kv, D), rnd(L, H_kv, D)
        kd, vd = hip.to_device(k, dtype), hip.to_device(v, dtype)
        keep.extend([kd, vd])
        m = cache.append_message(kd.data_ptr(), vd.data_ptr(), L, reserve)
        ks[m], vs[m] = k, v
        return m

    def lists():
        n = max(ks) + 1
        z = np.zeros((0, H_kv, D), np.float32)
        return [ks.get(m, z) for m in range(n)], [vs.get(m, z) for m in range(n)]

    def check(calls, what, f=1.0):
        n_rows = sum(c.n_q for c in calls)
        q = rnd(n_rows, H_q, D)
        qd = hip.to_device(q, dtype)
        for mode in ((0, 1, 2) if dtype == "bf16" else (0,)):       # default rule, per-call walk, shared walk
            cache.set_decode_sharing(mode)
            out = torch.empty_like(qd)
            lse = torch.empty((n_rows, H_q), dtype=torch.float32, device="cuda:0")
            cache.attend(calls, qd.data_ptr(), out.data_ptr(), lse.data_ptr())
            torch.cuda.synchronize()
            kl, vl = lists()
            at = 0
            for c in calls:
                o, l = orc.attend_call(kl, vl, c.sel, c.self_msg, c.self_start, c.n_q, c.q_pos, q[at:at + c.n_q], 10000.0)
                d = np.abs(out[at:at + c.n_q].float().cpu().numpy() - o)
                assert d.max() <= f * tol["max_abs"] and d.mean() <= f * tol["mean_abs"], (what, mode, d.max(), d.mean())
                assert np.abs(lse[at:at + c.n_q].cpu().numpy() - l).max() <= f * tol["lse"]
                at += c.n_q
        say(f"  {dtype} {what}: ok")

    sys_m, p0, p1 = append(70), append(45), append(33)
    tails = [append(1), append(1), append(1, reserve=3)]            # reserves 1, 1, 3: further extents come soon
    n_steps = 75
    for step in range(n_steps):
        k, v = rnd(len(tails), H_kv, D), rnd(len(tails), H_kv, D)
        kd, vd = hip.to_device(k, dtype), hip.to_device(v, dtype)
        keep.extend([kd, vd])
        cache.append_tokens_batch(tails, kd.data_ptr(), vd.data_ptr())
        for j, t in enumerate(tails):
            ks[t] = np.concatenate([ks[t], k[j:j + 1]]); vs[t] = np.concatenate([vs[t], v[j:j + 1]])
        if step in (0, 1, 2, 30, 31, 32, 33, 63, 64, 65, n_steps - 1):
            calls = [Call([(sys_m, 0), (p0, 70), (p1, 100)], tails[0], 140, 1, None),
                     Call([(sys_m, 0), (p1, 70)], tails[1], 103, 1, None),
                     Call([(p0, 5), (sys_m, 60)], tails[2], 200, 1, None)]
            check(calls, f"decode step {step}")
    ext = cache.message_extents(tails[0])
    assert len(ext) >= 3 and sum(l for _, l in ext) == 1 + n_steps and cache.message_info(tails[0])[0] == 1 + n_steps
    # a tail of several extents as a PARENT of a prefill call, next to its neighbours, and a tail that is listed by
    # another call's decode row
    new = append(40)
    check([Call([(tails[0], 0), (sys_m, 80), (tails[2], 150)], new, 230, 40, None),
           Call([(tails[1], 7), (tails[0], 300)], -1, 0, 1, np.asarray([400], dtype=np.int32))], "multi-extent parents")
    # every extent moves with its message
    cache.reposition(tails[0], 300)
    cache.reposition_batch([tails[1], sys_m], [7, 60])
    check([Call([(tails[1], 7), (tails[0], 300), (sys_m, 60)], -1, 0, 1, np.asarray([400], dtype=np.int32)),
           Call([(tails[0], -10)], tails[2], 90, 1, None)], "after position updates", f=2.0)
    # out to a blob and back: same results, other slots
    nbytes = cache.message_swap_bytes(tails[0])
    blob = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    before = cache.message_extents(tails[0])
    cache.message_swap_out(tails[0], blob.data_ptr())
    filler = append(20)
    cache.message_swap_in(tails[0], blob.data_ptr())
    after = cache.message_extents(tails[0])
    assert [l for _, l in after] == [l for _, l in before] and after != before
    check([Call([(tails[0], 300), (filler, 0)], -1, 0, 1, np.asarray([400], dtype=np.int32))], "after swap", f=2.0)
    # the gather table of a multi-extent message: positions run on, slots follow the extents
    call = Call([(tails[1], 7)], -1, 0, 1, None)
    n = cache.build_tables(call, 0, 0, 0)
    slot = torch.empty(n, dtype=torch.int32, device="cuda:0"); pos = torch.empty(n, dtype=torch.int32, device="cuda:0")
    cache.build_tables(call, slot.data_ptr(), pos.data_ptr(), n)
    torch.cuda.synchronize()
    want_slot = np.concatenate([np.arange(s, s + l) for s, l in cache.message_extents(tails[1])])
    assert np.array_equal(slot.cpu().numpy(), want_slot) and np.array_equal(pos.cpu().numpy(), 7 + np.arange(n))
    cache.close()
