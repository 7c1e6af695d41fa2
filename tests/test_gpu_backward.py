"""GPU parity of the gradient path (Sec. 2.4: position updates that gradients flow through, for
fine-tuning): pc_attend_backward + pc_grad_keys_finalize against the fp64 gradient oracle, element by
element, for q, and for the K and V of every message of the cache.
Bars: fp32 caches: fp32 arithmetic with sums of a few hundred terms in no fixed order (float atomics),
max-abs 2e-4 on gradients of order one.  bf16 caches: the arithmetic is fp32 too, but the stored keys
carry one bf16 rounding (2^-9 relative) that the oracle's exact keys do not; the gradients inherit a
relative error of that order: max-abs 2e-2 and mean-abs 1e-3 times the largest gradient, the forward bars."""
import sys

import numpy as np
import pytest

import pc_inputs as gen
from pc_inputs import Call
from tests.helpers import cache_lists

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


def run_backward_case(hip, w, reposition=None):
    import torch
    from oracle import choreo_oracle as orc
    cache = hip.make_cache(w)
    dw = hip.DeviceWorkload(w)
    rng = np.random.default_rng(99)
    ev_i = max(i for i, e in enumerate(w.events) if e.kind == "attend")
    # bring the cache to the state of the last attend event
    for s, e in zip(dw.steps, w.events[:ev_i]):
        if s[0] == "append":
            cache.append_message(s[1].data_ptr(), s[2].data_ptr(), s[3], s[4])
    if reposition:
        for m, base in reposition:
            cache.reposition(m, base)
    ev = w.events[ev_i]
    ks, vs = cache_lists(w, upto_event=ev_i)
    n_rows = sum(c.n_q for c in ev.calls)
    H_q, H_kv, D = w.n_q_heads, w.n_kv_heads, w.head_dim
    q = ev.q
    d_out = rng.standard_normal((n_rows, H_q, D)).astype(np.float32)
    if w.dtype == "bf16":
        d_out = gen.round_to_bf16(d_out)
    qd, dod = hip.to_device(q, w.dtype), hip.to_device(d_out, w.dtype)
    out = torch.empty_like(qd)
    lse = torch.empty((n_rows, H_q), dtype=torch.float32, device="cuda:0")
    cache.attend(ev.calls, qd.data_ptr(), out.data_ptr(), lse.data_ptr())
    slots = cache.cache_info()[2]
    d_q = torch.full(tuple(qd.shape), 7.0, dtype=torch.float32, device="cuda:0")
    d_k = torch.zeros((slots, H_kv, D), dtype=torch.float32, device="cuda:0")
    d_v = torch.zeros_like(d_k)
    # two backward calls into the same buffers (the batch cut in two), then one finalize
    cut = max(1, len(ev.calls) // 2)
    r0 = sum(c.n_q for c in ev.calls[:cut])
    for calls, a, b in ((ev.calls[:cut], 0, r0), (ev.calls[cut:], r0, n_rows)):
        if not calls:
            continue
        cache.attend_backward(calls, qd[a:b].data_ptr(), lse[a:b].data_ptr(), dod[a:b].data_ptr(), d_q[a:b].data_ptr(),
                              d_k.data_ptr(), d_v.data_ptr())
    cache.grad_keys_finalize(d_k.data_ptr())
    torch.cuda.synchronize()
    # oracle: sum over calls
    want_q = np.zeros((n_rows, H_q, D))
    want_k = [np.zeros(k.shape) for k in ks]
    want_v = [np.zeros(v.shape) for v in vs]
    at = 0
    for c in ev.calls:
        gq, gk, gv = orc.attend_call_backward(ks, vs, c.sel, c.self_msg, c.self_start, c.n_q, c.q_pos, q[at:at + c.n_q],
                                              d_out[at:at + c.n_q], w.rope_theta)
        want_q[at:at + c.n_q] = gq
        for m in range(len(ks)):
            want_k[m] += gk[m]
            want_v[m] += gv[m]
        at += c.n_q
    got_q = d_q.cpu().numpy()
    got_k, got_v = d_k.cpu().numpy(), d_v.cpu().numpy()
    worst = np.abs(got_q - want_q).max()
    touched = np.zeros(slots, dtype=bool)
    for m in range(len(ks)):
        L, s0, _ = cache.message_info(m)
        assert L == ks[m].shape[0]
        worst = max(worst, np.abs(got_k[s0:s0 + L] - want_k[m]).max(), np.abs(got_v[s0:s0 + L] - want_v[m]).max())
        touched[s0:s0 + L] = True
    scale_ref = max(1.0, np.abs(want_q).max(), max(np.abs(x).max() for x in want_k), max(np.abs(x).max() for x in want_v))
    say(f"  {w.name} {w.dtype}: worst abs gradient error {worst:.3e} (largest gradient {scale_ref:.2f})")
    assert worst <= (2e-4 if w.dtype == "f32" else 2e-2) * scale_ref
    if w.dtype == "bf16":
        mean = np.mean([np.abs(got_q - want_q).mean()] +
                       [np.abs(got_k[cache.message_info(m)[1]:cache.message_info(m)[1] + ks[m].shape[0]] - want_k[m]).mean()
                        for m in range(len(ks))])
        assert mean <= 1e-3 * scale_ref
    assert not got_k[~touched].any() and not got_v[~touched].any()      # slots of no message stay untouched
    cache.close()


def test_backward_config1_tiny_fp32(hip):
    run_backward_case(hip, gen.tiny_fp32())


@pytest.mark.parametrize("seed", [101, 102])
def test_backward_small_random_fp32(hip, seed):
    run_backward_case(hip, gen.small_random(seed, dtype="f32", n_q_heads=4, n_kv_heads=2, head_dim=64, len_hi=100))


def test_backward_d128_and_moved_messages(hip):
    w = gen.small_random(103, dtype="f32", n_q_heads=6, n_kv_heads=2, head_dim=128, len_hi=70, max_q=20)
    run_backward_case(hip, w, reposition=[(0, 500), (3, -40), (5, 17)])


@pytest.mark.parametrize("seed,hq,hkv", [(201, 8, 2), (203, 4, 4)])
def test_backward_small_random_bf16(hip, seed, hq, hkv):
    run_backward_case(hip, gen.small_random(seed, n_q_heads=hq, n_kv_heads=hkv))


def test_backward_bf16_scaled_prefill_shape(hip):
    run_backward_case(hip, gen.single_prefill(n_msgs=10, len_lo=20, len_hi=90, n_sel=5, n_new=48))


def test_backward_through_a_message_of_several_extents(hip):
    """The gradient of a message that lives in several spans (PC_FLAG_GROW_EXTENTS) and was moved: its rows of
    d_k, d_v are those of its extents, in token order."""
    import torch
    from oracle import choreo_oracle as orc
    from paper_2512_23049_amd.binding import PC_F32, PC_FLAG_GROW_EXTENTS, Cache
    rng = np.random.default_rng(7)
    H_q, H_kv, D = 4, 2, 64
    cache = Cache(H_q, H_kv, D, PC_F32, 10000.0, 2048, 32, flags=PC_FLAG_GROW_EXTENTS)
    keep = []

    def dev(x):
        t = hip.to_device(x, "f32"); keep.append(t); return t
    lens = [3 + 45, 20, 12]
    ks = [rng.standard_normal((L, H_kv, D)).astype(np.float32) for L in lens]
    vs = [rng.standard_normal((L, H_kv, D)).astype(np.float32) for L in lens]
    a = cache.append_message(dev(ks[0][:3]).data_ptr(), dev(vs[0][:3]).data_ptr(), 3, 0)
    b = cache.append_message(dev(ks[1]).data_ptr(), dev(vs[1]).data_ptr(), 20, 0)
    cache.append_tokens(a, dev(ks[0][3:]).data_ptr(), dev(vs[0][3:]).data_ptr(), 45)       # a second extent behind b
    new = cache.append_message(dev(ks[2]).data_ptr(), dev(vs[2]).data_ptr(), 12, 0)
    assert len(cache.message_extents(a)) == 2
    cache.reposition(a, 200)
    ids = {a: 0, b: 1, new: 2}
    assert sorted(ids) == [a, b, new]
    calls = [Call([(b, 0), (a, 30)], new, 100, 12, None), Call([(a, 200)], -1, 0, 2, np.asarray([260, 300], dtype=np.int32))]
    n_rows = 14
    q = rng.standard_normal((n_rows, H_q, D)).astype(np.float32)
    d_out = rng.standard_normal((n_rows, H_q, D)).astype(np.float32)
    qd, dod = dev(q), dev(d_out)
    out = torch.empty_like(qd); lse = torch.empty((n_rows, H_q), dtype=torch.float32, device="cuda:0")
    cache.attend(calls, qd.data_ptr(), out.data_ptr(), lse.data_ptr())
    slots = cache.cache_info()[2]
    d_q = torch.empty_like(qd)
    d_k = torch.zeros((slots, H_kv, D), dtype=torch.float32, device="cuda:0"); d_v = torch.zeros_like(d_k)
    cache.attend_backward(calls, qd.data_ptr(), lse.data_ptr(), dod.data_ptr(), d_q.data_ptr(), d_k.data_ptr(), d_v.data_ptr())
    cache.grad_keys_finalize(d_k.data_ptr())
    torch.cuda.synchronize()
    # the oracle numbers messages 0, 1, 2 in the order a, b, new
    kl, vl = [None] * 3, [None] * 3
    for m, i in ids.items():
        kl[i], vl[i] = ks[i], vs[i]
    remap = lambda sel: [(ids[m], s) for m, s in sel]
    want_k = [np.zeros(k.shape) for k in kl]; want_v = [np.zeros(v.shape) for v in vl]
    want_q = np.zeros((n_rows, H_q, D)); at = 0
    for c in calls:
        gq, gk, gv = orc.attend_call_backward(kl, vl, remap(c.sel), ids.get(c.self_msg, -1), c.self_start, c.n_q, c.q_pos,
                                              q[at:at + c.n_q], d_out[at:at + c.n_q], 10000.0)
        want_q[at:at + c.n_q] = gq
        for i in range(3):
            want_k[i] += gk[i]; want_v[i] += gv[i]
        at += c.n_q
    gk_d, gv_d = d_k.cpu().numpy(), d_v.cpu().numpy()
    worst = np.abs(d_q.cpu().numpy() - want_q).max()
    for m, i in ids.items():
        rows = np.concatenate([np.arange(s, s + l) for s, l in cache.message_extents(m)])
        worst = max(worst, np.abs(gk_d[rows] - want_k[i]).max(), np.abs(gv_d[rows] - want_v[i]).max())
    say(f"  gradient through extents: worst abs error {worst:.3e}")
    assert worst <= 2e-4
    cache.close()
