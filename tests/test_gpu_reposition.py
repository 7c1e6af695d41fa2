"""GPU tests of pc_reposition (Sec. 2.4 "Position Updates"): the stored keys of a message are
turned in place; what pc_attend computes must not change, whatever base each message has."""
import ctypes as C
import sys

import numpy as np
import pytest

import pc_inputs as gen
from tests.helpers import attend_events, oracle_for_event

pytestmark = pytest.mark.gpu

# Every move rounds the stored keys to the cache dtype once more.  In fp32 that is invisible at
# the 1e-4 bar.  In bf16 a key then carries n + 1 roundings of 2^-9 instead of one, so the score
# error (and with it the output error) grows by sqrt(n + 1): the bars below are the unmoved
# cache's (max-abs 2e-2, mean-abs 1e-3) times 2, which covers up to n = 3 moves.
TOL = {"f32": dict(max_abs=1e-4, mean_abs=1e-5, lse=1e-4),
       "bf16": dict(max_abs=4e-2, mean_abs=2e-3, lse=4e-2)}


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def hip():
    import torch
    from paper_2512_23049_amd import harness
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return harness


def compare(w, res, what):
    tol = TOL[w.dtype]
    for k, (ei, ev) in enumerate(attend_events(w)):
        out = res[k][0].float().cpu().numpy()
        lse = res[k][1].cpu().numpy()
        for ci, rows, o, l in oracle_for_event(w, ei):
            d = np.abs(out[rows] - o)
            say(f"  {what} event {k} call {ci}: max_abs={d.max() if d.size else 0:.3e} mean_abs={d.mean() if d.size else 0:.3e}")
            assert d.size == 0 or d.max() <= tol["max_abs"]
            assert d.size == 0 or d.mean() <= tol["mean_abs"]
            fin = np.isfinite(l)
            assert np.array_equal(np.isfinite(lse[rows]), fin)
            if fin.any():
                assert np.abs(lse[rows][fin] - l[fin]).max() <= tol["lse"]


def run_with_moves(hip, w, moves):
    """Appends everything, applies `moves` (msg -> new base) and runs the attend events."""
    import torch
    cache = hip.make_cache(w, max_position=1 << 20)
    dw = hip.DeviceWorkload(w)
    res = []
    moved = False
    for s in dw.steps:
        if s[0] == "append":
            cache.append_message(s[1].data_ptr(), s[2].data_ptr(), s[3], s[4])
            continue
        if not moved:
            n_msgs = cache.cache_info()[0]
            for m, base in moves(n_msgs):
                cache.reposition(m, base)
                assert cache.message_base(m) == base
            moved = True
        _, calls, mc, q, out, lse = s
        cache.attend(calls, q.data_ptr(), out.data_ptr(), lse.data_ptr(), 0, mc)
        res.append((out, lse))
    torch.cuda.synchronize()
    cache.close()
    return res


@pytest.mark.parametrize("dtype,seed", [("bf16", 31), ("bf16", 32), ("f32", 33)])
def test_random_bases_keep_attention(hip, dtype, seed):
    kw = dict(n_q_heads=4, n_kv_heads=2, head_dim=64) if dtype == "f32" else {}
    w = gen.small_random(seed, dtype=dtype, **kw)
    rng = np.random.default_rng(seed)

    def moves(n):
        return [(int(m), int(rng.integers(-3000, 3001))) for m in rng.permutation(n)[: max(1, n // 2)]]
    say(f"[reposition] {w.name} {dtype} seed {seed}")
    compare(w, run_with_moves(hip, w, moves), "random bases")


def test_moved_twice_and_back(hip):
    w = gen.small_random(34, dtype="bf16")

    def moves(n):
        out = []
        for m in range(n):
            out += [(m, 777 + m), (m, -55), (m, 0)]     # two moves, then back to the base of the append
        return out
    compare(w, run_with_moves(hip, w, moves), "moved twice and back")


def test_parents_at_their_assigned_starts(hip):
    """Every parent of the (single) call is first moved to the position the call gives it: then the
    whole call needs one turn of the queries (the fast path of the prefill kernel)."""
    w = gen.single_prefill(n_msgs=12, len_lo=40, len_hi=200, n_sel=6, n_new=96, n_q_heads=8, n_kv_heads=2)
    ev = attend_events(w)[0][1]
    call = ev.calls[0]

    def moves(n):
        return [(m, s) for m, s in call.sel] + [(call.self_msg, call.self_start)]
    compare(w, run_with_moves(hip, w, moves), "parents at their starts")


def test_batched_moves(hip):
    """All messages moved in one launch, twice (the second batch leaves some where they are)."""
    import torch
    w = gen.small_random(37, dtype="bf16")
    rng = np.random.default_rng(37)
    cache = hip.make_cache(w, max_position=1 << 20)
    dw = hip.DeviceWorkload(w)
    res = []
    for s in dw.steps:
        if s[0] == "append":
            cache.append_message(s[1].data_ptr(), s[2].data_ptr(), s[3], s[4])
            continue
        n = cache.cache_info()[0]
        b1 = [int(x) for x in rng.integers(-2000, 2001, size=n)]
        cache.reposition_batch(list(range(n)), b1)
        b2 = [b if i % 3 else b + 17 for i, b in enumerate(b1)]
        cache.reposition_batch(list(range(n)), b2)
        assert [cache.message_base(m) for m in range(n)] == b2
        _, calls, mc, q, out, lse = s
        cache.attend(calls, q.data_ptr(), out.data_ptr(), lse.data_ptr(), 0, mc)
        res.append((out, lse))
    torch.cuda.synchronize()
    from paper_2512_23049_amd.binding import PcError, PC_ERR_BAD_MSG_ID, PC_ERR_INVALID_ARG
    for ids, bases, code in [([0, 0], [1, 2], PC_ERR_INVALID_ARG), ([0, 999], [1, 2], PC_ERR_BAD_MSG_ID),
                             ([0], [(1 << 20) + 1], PC_ERR_INVALID_ARG)]:
        with pytest.raises(PcError) as e:
            cache.reposition_batch(ids, bases)
        assert e.value.code == code
    assert cache.message_base(0) == b2[0]                # a refused batch moves nothing
    cache.reposition_batch([], [])
    cache.close()
    compare(w, res, "batched moves")


def test_stored_keys_after_move(hip):
    """Reads the key store back (caller-owned arena) and compares with the oracle's rotation to
    base + t; tolerance: two roundings to bf16 (append, move) of values of magnitude |k|."""
    import torch
    from oracle import choreo_oracle as orc
    from paper_2512_23049_amd import binding
    w = gen.small_random(35, dtype="bf16")
    reserves = w.message_reserves()
    cap = sum(((r + 31) // 32) * 32 for r in reserves) + 32
    cfg = binding.pc_config(w.n_q_heads, w.n_kv_heads, w.head_dim, binding.PC_BF16, w.rope_theta, 0.0, cap,
                            len(reserves) + 8, 1 << 20, 0, None, 0)
    nbytes = binding.lib().pc_cache_storage_bytes(C.byref(cfg))
    arena = torch.zeros(nbytes // 2, dtype=torch.bfloat16, device="cuda:0")
    cache = binding.Cache(w.n_q_heads, w.n_kv_heads, w.head_dim, binding.PC_BF16, w.rope_theta, cap, len(reserves) + 8,
                          max_position=1 << 20, arena=arena.data_ptr(), arena_bytes=nbytes)
    dw = hip.DeviceWorkload(w)
    ks = []
    for s, e in zip(dw.steps, w.events):
        if s[0] == "append":
            cache.append_message(s[1].data_ptr(), s[2].data_ptr(), s[3], s[4])
            ks.append(e.k)
    bases = [0, 1234, -987, 40000]
    slots = ((cap + 31) // 32) * 32
    kstore = arena[: w.n_kv_heads * slots * w.head_dim].view(w.n_kv_heads, slots, w.head_dim)
    for m in range(min(4, len(ks))):
        cache.reposition(m, bases[m])
        torch.cuda.synchronize()
        ln, slot0, _ = cache.message_info(m)
        got = kstore[:, slot0:slot0 + ln, :].float().cpu().numpy()                   # [H_kv, L, D]
        want = orc.rope(ks[m].astype(np.float64), bases[m] + np.arange(ln), w.rope_theta)   # [L, H_kv, D]
        want = np.transpose(want, (1, 0, 2))
        err = np.abs(got - want)
        bound = 2.0 ** -7 * (np.abs(want) + np.abs(np.roll(want, w.head_dim // 2, axis=-1))) + 1e-6
        say(f"  message {m} base {bases[m]}: max err {err.max():.3e}")
        assert (err <= bound).all()
    cache.close()


def test_errors(hip):
    from paper_2512_23049_amd.binding import PcError, PC_ERR_BAD_MSG_ID, PC_ERR_INVALID_ARG
    w = gen.small_random(36, dtype="bf16")
    cache = hip.make_cache(w, max_position=1000)
    dw = hip.DeviceWorkload(w)
    s = dw.steps[0]
    m = cache.append_message(s[1].data_ptr(), s[2].data_ptr(), s[3], s[4])
    with pytest.raises(PcError) as e:
        cache.reposition(m + 5, 0)
    assert e.value.code == PC_ERR_BAD_MSG_ID
    with pytest.raises(PcError) as e:
        cache.reposition(m, 1001)
    assert e.value.code == PC_ERR_INVALID_ARG
    cache.reposition(m, 1000)
    cache.reposition(m, 1000)          # same base again: nothing to do
    assert cache.message_base(m) == 1000
    cache.close()
