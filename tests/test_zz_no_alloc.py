"""GPU test of pc_attend_static, the entry point for callers that cannot allocate device memory: its per-call
workspace is a fixed array inside the library.  Same kernels and plan as pc_attend, so the results must be the same
bits; checked on two calls in a row, the second smaller than the first (what the first left in the array must not
leak into the second), then on a third, larger again; a batch that does not fit is rejected before anything runs."""
import sys

import numpy as np
import pytest

import pc_inputs as gen

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def both_entry_points(hip, w, tag):
    import torch
    cache = hip.make_cache(w)
    dw = hip.DeviceWorkload(w)
    n_att = 0
    for s in dw.steps:
        if s[0] == "append":
            cache.append_message(s[1].data_ptr(), s[2].data_ptr(), s[3], s[4])
            continue
        if s[0] == "extend":
            cache.append_tokens_batch(s[3], s[1].data_ptr(), s[2].data_ptr())
            continue
        _, calls, m, q, out, lse = s
        out.fill_(7.0); lse.fill_(7.0)
        out2 = torch.full_like(out, 9.0)
        lse2 = torch.full_like(lse, 9.0)
        cache.attend(calls, q.data_ptr(), out.data_ptr(), lse.data_ptr(), 0, m)
        torch.cuda.synchronize()
        cache.attend_static(calls, q.data_ptr(), out2.data_ptr(), lse2.data_ptr(), 0, m)
        torch.cuda.synchronize()
        same = torch.equal(out.view(torch.int16) if out.dtype == torch.bfloat16 else out,
                           out2.view(torch.int16) if out2.dtype == torch.bfloat16 else out2)
        say(f"  {tag}: attend {n_att}: rows={q.shape[0]} outputs identical: {same}")
        assert same
        assert torch.equal(lse, lse2)
        assert torch.isfinite(out2.float()).all()
        n_att += 1
    cache.close()
    assert n_att > 0


def test_static_entry_point_matches_pc_attend_on_calls_in_a_row():
    import torch
    from paper_2512_23049_amd import harness as hip
    assert torch.cuda.is_available(), "these tests need the MI355X"
    # 1: a mixed batch (prefill with KV splits and their merge, decode calls on both walks)
    big = gen.long_context(n_msgs=60, len_lo=30, len_hi=200, target_tokens=5000, n_decode=12, n_prefill_q=300)
    both_entry_points(hip, big, "first (large)")
    # 2: a smaller one right after it, in the same array
    small = gen.long_context(n_msgs=24, len_lo=30, len_hi=100, target_tokens=1200, n_decode=3, n_prefill_q=70,
                             n_q_heads=16, n_kv_heads=2)
    both_entry_points(hip, small, "second (smaller)")
    # 3: other shapes again: a decode batch, rounds of prefills, the fp32 path
    both_entry_points(hip, gen.parallel_decode(n_calls=12, sys_len=300, n_pool=20, len_lo=50, len_hi=200, n_sel=4,
                                               tail_len=64), "third (decode)")
    both_entry_points(hip, gen.multi_agent_rounds(n_agents=3, n_rounds=3, msg_len=70), "fourth (rounds)")
    both_entry_points(hip, gen.tiny_fp32(), "fifth (fp32)")


def test_static_entry_point_rejects_what_does_not_fit():
    import torch
    from paper_2512_23049_amd import PC_ERR_NO_SPACE, PcError, harness as hip
    w = gen.single_prefill(n_msgs=24, len_lo=200, len_hi=600, n_sel=12, n_new=512)
    cache = hip.make_cache(w)
    dw = hip.DeviceWorkload(w)
    for s in dw.steps:
        if s[0] == "append":
            cache.append_message(s[1].data_ptr(), s[2].data_ptr(), s[3], s[4])
    _, calls, m, q, out, lse = [s for s in dw.steps if s[0] == "attend"][-1]
    out.fill_(3.0)
    cache.set_tuning(0, 1)                      # one KV tile per split: gigabytes of split partials
    with pytest.raises(PcError) as ei:
        cache.attend_static(calls, q.data_ptr(), out.data_ptr(), lse.data_ptr(), 0, m)
    assert ei.value.code == PC_ERR_NO_SPACE
    say("  rejected:", ei.value)
    torch.cuda.synchronize()
    assert (out == 3.0).all()                   # nothing was enqueued
    cache.set_tuning(0, 0)
    cache.attend_static(calls, q.data_ptr(), out.data_ptr(), lse.data_ptr(), 0, m)      # the same call fits with default splits
    torch.cuda.synchronize()
    out2 = torch.empty_like(out)
    cache.attend(calls, q.data_ptr(), out2.data_ptr(), lse.data_ptr(), 0, m)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16))
    cache.close()
