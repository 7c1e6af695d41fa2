"""GPU test of pc_message_free: freed slots are reused by later, shorter messages; whatever the
old message left behind in a reused tile's tail must not reach any result."""
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
def test_reused_slots_hold_only_the_new_message(hip, dtype):
    import torch
    from oracle import choreo_oracle as orc
    from paper_2512_23049_amd import PC_SLOT_ALIGN
    from paper_2512_23049_amd.binding import PC_BF16, PC_F32, Cache
    rng = np.random.default_rng(71)
    H_q, H_kv, D = (8, 2, 128) if dtype == "bf16" else (4, 2, 64)
    tol = dict(max_abs=2e-2, mean_abs=1e-3) if dtype == "bf16" else dict(max_abs=1e-4, mean_abs=1e-5)

    def rnd(*shape):
        x = rng.standard_normal(shape).astype(np.float32)              # N(0,1) like the workloads the bars are for
        return gen.round_to_bf16(x) if dtype == "bf16" else x
    cache = Cache(H_q, H_kv, D, PC_BF16 if dtype == "bf16" else PC_F32, 10000.0, 4096, 64)
    model = orc.SlotModel(PC_SLOT_ALIGN)
    ks, vs, keep = {}, {}, []

    def append(L, reserve=0):
        k, v = rnd(L, H_kv, D), rnd(L, H_kv, D)
        kd, vd = hip.to_device(k, dtype), hip.to_device(v, dtype)
        keep.extend([kd, vd])
        m = cache.append_message(kd.data_ptr(), vd.data_ptr(), L, reserve)
        assert cache.message_info(m)[1] == model.append(m, max(L, reserve))
        ks[m], vs[m] = k, v
        return m

    def check(call, what):
        q = rnd(call.n_q, H_q, D)
        qd = hip.to_device(q, dtype)
        out = torch.empty_like(qd)
        lse = torch.empty((call.n_q, H_q), dtype=torch.float32, device="cuda:0")
        cache.attend([call], qd.data_ptr(), out.data_ptr(), lse.data_ptr())
        torch.cuda.synchronize()
        n = max(ks) + 1
        kl = [ks.get(m, np.zeros((0, H_kv, D), np.float32)) for m in range(n)]
        vl = [vs.get(m, np.zeros((0, H_kv, D), np.float32)) for m in range(n)]
        o, l = orc.attend_call(kl, vl, call.sel, call.self_msg, call.self_start, call.n_q, None, q, 10000.0)
        d = np.abs(out.float().cpu().numpy() - o)
        say(f"  {what}: max_abs={d.max():.3e} mean_abs={d.mean():.3e}")
        assert np.isfinite(out.float().cpu().numpy()).all()
        assert d.max() <= tol["max_abs"] and d.mean() <= tol["mean_abs"]

    a = append(100)            # [0, 128)
    b = append(61)             # [128, 192)
    c = append(40)             # [192, 256)
    check(Call([(a, 0), (b, 300), (c, 100)], -1, 0, 5, None), "before any free")
    cache.message_free(a); model.release(a); del ks[a], vs[a]
    d = append(33)             # reuses [0, 64): its second tile holds one new token and 31 old ones
    e = append(9)              # reuses [64, 96): one ragged tile over old data
    assert cache.message_info(d)[1] == 0 and cache.message_info(e)[1] == 64
    check(Call([(d, 10), (b, 50), (e, 0)], c, 500, 40, None), "reused slots as parents, old message as the new one")
    check(Call([(c, 0)], e, 40, 9, None), "a reused span as the new message")
    cache.message_free(b); model.release(b); del ks[b], vs[b]
    f = append(5, reserve=20)  # [96,128) is too small for nothing: 20 -> 32 slots, fits [96, 128)
    assert cache.message_info(f)[1] == 96
    kd = hip.to_device(rnd(6, H_kv, D), dtype); vd = hip.to_device(rnd(6, H_kv, D), dtype)
    keep.extend([kd, vd])
    cache.append_tokens(f, kd.data_ptr(), vd.data_ptr(), 6)
    ks[f] = np.concatenate([ks[f], kd.float().cpu().numpy()]); vs[f] = np.concatenate([vs[f], vd.float().cpu().numpy()])
    check(Call([(f, 0), (d, 11)], c, 60, 3, None), "a grown message in a reused span")
    from paper_2512_23049_amd.binding import PcError, PC_ERR_BAD_MSG_ID
    with pytest.raises(PcError) as ei:
        cache.attend([Call([(a, 0)], -1, 0, 1, None)], keep[0].data_ptr(), keep[1].data_ptr())
    assert ei.value.code == PC_ERR_BAD_MSG_ID
    cache.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_infinities_left_by_a_freed_message_do_not_reach_its_successor(hip, dtype):
    """A freed message whose K and V hold Inf and NaN; its span is taken by a shorter message, by a message that then
    grows token by token, and by a swapped-in one: what the old owner left behind the new last tokens (inside their
    tiles) would turn 0 * Inf into NaN on the V side if the span were not cleared when it is taken again.  Prefill,
    per-call decode and shared decode against the oracle."""
    import torch
    from oracle import choreo_oracle as orc
    from paper_2512_23049_amd.binding import PC_BF16, PC_F32, Cache
    rng = np.random.default_rng(72)
    H_q, H_kv, D = (8, 2, 128) if dtype == "bf16" else (4, 2, 64)
    tol = dict(max_abs=2e-2, mean_abs=1e-3) if dtype == "bf16" else dict(max_abs=1e-4, mean_abs=1e-5)

    def rnd(*shape):
        x = rng.standard_normal(shape).astype(np.float32)
        return gen.round_to_bf16(x) if dtype == "bf16" else x
    cache = Cache(H_q, H_kv, D, PC_BF16 if dtype == "bf16" else PC_F32, 10000.0, 4096, 64)
    ks, vs, keep = {}, {}, []

    def append(k, v, reserve=0):
        kd, vd = hip.to_device(k, dtype), hip.to_device(v, dtype)
        keep.extend([kd, vd])
        m = cache.append_message(kd.data_ptr(), vd.data_ptr(), k.shape[0], reserve)
        ks[m], vs[m] = k, v
        return m

    def check(calls, what):
        n = max(ks) + 1
        kl = [ks.get(m, np.zeros((0, H_kv, D), np.float32)) for m in range(n)]
        vl = [vs.get(m, np.zeros((0, H_kv, D), np.float32)) for m in range(n)]
        rows = sum(c.n_q for c in calls)
        q = rnd(rows, H_q, D)
        qd = hip.to_device(q, dtype)
        for sharing in ((1, 2) if dtype == "bf16" else (1,)):
            cache.set_decode_sharing(sharing)
            out = torch.empty_like(qd)
            lse = torch.empty((rows, H_q), dtype=torch.float32, device="cuda:0")
            cache.attend(calls, qd.data_ptr(), out.data_ptr(), lse.data_ptr())
            torch.cuda.synchronize()
            got = out.float().cpu().numpy()
            assert np.isfinite(got).all(), f"{what} (sharing {sharing}): non-finite output"
            at = 0
            for c in calls:
                o, l = orc.attend_call(kl, vl, c.sel, c.self_msg, c.self_start, c.n_q, None, q[at:at + c.n_q], 10000.0)
                d = np.abs(got[at:at + c.n_q] - o)
                say(f"  {what} sharing {sharing} n_q {c.n_q}: max_abs={d.max():.3e} mean_abs={d.mean():.3e}")
                assert d.max() <= tol["max_abs"] and d.mean() <= tol["mean_abs"]
                at += c.n_q

    bad = np.full((200, H_kv, D), np.inf, dtype=np.float32)
    bad[::3] = -np.inf
    bad[1::7] = np.nan
    poison = append(bad.copy(), bad.copy())                  # slots [0, 224)
    other = append(rnd(70, H_kv, D), rnd(70, H_kv, D))        # [224, 320)
    cache.message_free(poison); del ks[poison], vs[poison]
    a = append(rnd(33, H_kv, D), rnd(33, H_kv, D))            # [0, 64): one token in its second tile, the rest the old owner's
    b = append(rnd(5, H_kv, D), rnd(5, H_kv, D), reserve=60)  # [64, 128): grows below
    assert cache.message_info(a)[1] == 0 and cache.message_info(b)[1] == 64
    calls = [Call([(a, 0), (other, 40)], b, 200, 5, None), Call([(a, 3)], b, 100, 1, None), Call([(b, 0), (a, 9)], -1, 0, 1, None)]
    check(calls, "shorter messages in the freed span")
    for step in range(30):                                    # b grows across a tile boundary, one token at a time
        k1, v1 = rnd(1, H_kv, D), rnd(1, H_kv, D)
        kd, vd = hip.to_device(k1, dtype), hip.to_device(v1, dtype)
        keep.extend([kd, vd])
        cache.append_tokens(b, kd.data_ptr(), vd.data_ptr(), 1)
        ks[b] = np.concatenate([ks[b], k1]); vs[b] = np.concatenate([vs[b], v1])
        if step in (0, 2, 26, 27, 29):
            check([Call([(a, 0)], b, 50, 1, None), Call([(b, 7), (other, 0)], -1, 0, 1, None),
                   Call([(other, 0)], b, 90, min(5 + step, 20), None)], f"grown to {5 + step + 1} tokens")
    cache.close()
