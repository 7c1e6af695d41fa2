"""GPU test of pc_message_swap_out / pc_message_swap_in (Sec. 2.2, the note on moving messages out to
CPU memory): a message that left the cache and came back, at other slots, gives bit-identical
attention results; what took its slots meanwhile does not leak into them."""
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


@pytest.mark.parametrize("dtype,where", [("bf16", "pinned"), ("bf16", "device"), ("f32", "pinned")])
def test_swapped_message_comes_back_bit_identical(hip, dtype, where):
    import torch
    from oracle import choreo_oracle as orc
    from paper_2512_23049_amd.binding import PC_BF16, PC_F32, Cache
    rng = np.random.default_rng(17)
    H_q, H_kv, D = (8, 2, 128) if dtype == "bf16" else (4, 2, 64)

    def rnd(*shape):
        x = rng.standard_normal(shape).astype(np.float32)
        return gen.round_to_bf16(x) if dtype == "bf16" else x
    cache = Cache(H_q, H_kv, D, PC_BF16 if dtype == "bf16" else PC_F32, 10000.0, 4096, 64)
    ks, vs, keep = [], [], []

    def append(L, reserve=0):
        k, v = rnd(L, H_kv, D), rnd(L, H_kv, D)
        kd, vd = hip.to_device(k, dtype), hip.to_device(v, dtype)
        keep.extend([kd, vd])
        m = cache.append_message(kd.data_ptr(), vd.data_ptr(), L, reserve)
        assert m == len(ks)
        ks.append(k); vs.append(v)
        return m

    a, b, c, d = append(100), append(61, reserve=90), append(40), append(7)
    cache.reposition(b, 300)                                   # a stored base other than 0 travels with the blob
    calls = [Call([(a, 0), (b, 300), (c, 100)], d, 500, 7, None),
             Call([(b, -20), (c, 0)], -1, 0, 1, np.asarray([90], dtype=np.int32))]
    n_rows = sum(cl.n_q for cl in calls)
    q = rnd(n_rows, H_q, D)
    qd = hip.to_device(q, dtype)

    def attend():
        out = torch.empty_like(qd)
        lse = torch.empty((n_rows, H_q), dtype=torch.float32, device="cuda:0")
        cache.attend(calls, qd.data_ptr(), out.data_ptr(), lse.data_ptr())
        torch.cuda.synchronize()
        return out.clone(), lse.clone()

    out0, lse0 = attend()
    slot_before = cache.message_info(b)[1]
    nbytes = cache.message_swap_bytes(b)
    assert nbytes == 2 * 96 * H_kv * D * (2 if dtype == "bf16" else 4)
    blob = (torch.empty(nbytes, dtype=torch.uint8, pin_memory=True) if where == "pinned"
            else torch.empty(nbytes, dtype=torch.uint8, device="cuda:0"))
    cache.message_swap_out(b, blob.data_ptr())
    # something else moves into the slots it left, with other data
    e = append(80)
    assert cache.message_info(e)[1] == slot_before
    cache.message_swap_in(b, blob.data_ptr())
    assert cache.message_info(b)[1] != slot_before and cache.message_info(b)[0] == 61 and cache.message_base(b) == 300
    out1, lse1 = attend()
    # The prefill call walks its parents in list order: the same arithmetic, bit for bit.  The one-row call
    # of a bf16 cache walks them in cache-slot order, which the move changed: the same terms summed in another
    # order (fp32 rounding in the sums; the bf16 output may differ in its last bit).
    n0 = calls[0].n_q
    assert torch.equal(out0[:n0].view(torch.uint8), out1[:n0].view(torch.uint8)), "the message changed on its way out and back"
    assert torch.equal(lse0[:n0], lse1[:n0])
    if dtype == "f32":
        assert torch.equal(out0[n0:].view(torch.uint8), out1[n0:].view(torch.uint8)) and torch.equal(lse0[n0:], lse1[n0:])
    else:
        o0, o1 = out0[n0:].float(), out1[n0:].float()
        assert ((o0 - o1).abs() <= 2.0 ** -7 * o0.abs()).all()
        assert ((lse0[n0:] - lse1[n0:]).abs() <= 1e-6 * lse0[n0:].abs() + 1e-6).all()
    # and the results are the oracle's (message b's keys carry one more rounding in bf16: twice the bars)
    off = 0
    for cl in calls:
        o, l = orc.attend_call(ks, vs, cl.sel, cl.self_msg, cl.self_start, cl.n_q, cl.q_pos, q[off:off + cl.n_q], 10000.0)
        dd = np.abs(out1[off:off + cl.n_q].float().cpu().numpy() - o)
        say(f"  {dtype} {where}: max_abs={dd.max():.3e} mean_abs={dd.mean():.3e}")
        if dtype == "bf16":
            assert dd.max() <= 4e-2 and dd.mean() <= 2e-3
        else:
            assert dd.max() <= 1e-4
        off += cl.n_q
    # the message still grows inside the reserve that came back with it
    k1, v1 = rnd(5, H_kv, D), rnd(5, H_kv, D)
    kd, vd = hip.to_device(k1, dtype), hip.to_device(v1, dtype)
    cache.append_tokens(b, kd.data_ptr(), vd.data_ptr(), 5)
    torch.cuda.synchronize()
    assert cache.message_info(b)[0] == 66
    cache.close()
