"""GPU test of what the append kernels leave in the cache (Sec. 2.4: new messages are appended to the
cache; here K turned to the in-message index, V key-transposed in groups of 8 slots).  The stores are read
back through a caller-owned arena: V is a pure data movement and must match bit for bit, K is the oracle's
rotation rounded once to bf16, rows and group remainders behind a message's last token stay zero.
Covers pc_append_message, pc_append_messages, pc_append_tokens and pc_append_tokens_batch."""
import ctypes as C
import sys

import numpy as np
import pytest

import pc_inputs as gen

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("h_kv", [2, 3])
def test_stored_form_after_every_kind_of_append(h_kv):
    import torch
    from oracle import choreo_oracle as orc
    from paper_2512_23049_amd import binding
    from paper_2512_23049_amd.harness import to_device
    assert torch.cuda.is_available(), "these tests need the MI355X"
    D, theta = 128, 10000.0
    rng = np.random.default_rng(31 + h_kv)

    def rnd(L):
        return gen.round_to_bf16(rng.standard_normal((L, h_kv, D)).astype(np.float32))
    cap = 2048
    cfg = binding.pc_config(2 * h_kv, h_kv, D, binding.PC_BF16, theta, 0.0, cap, 32, 1 << 20, 0, None, 0)
    nbytes = binding.lib().pc_cache_storage_bytes(C.byref(cfg))
    arena = torch.zeros(nbytes // 2, dtype=torch.bfloat16, device="cuda:0")
    cache = binding.Cache(2 * h_kv, h_kv, D, binding.PC_BF16, theta, cap, 32, max_position=1 << 20,
                          arena=arena.data_ptr(), arena_bytes=nbytes)
    slots = cap
    k_host, v_host, keep = {}, {}, []

    def dev(x):
        t = to_device(x, "bf16", "cuda:0")
        keep.append(t)
        return t
    # one at a time
    for L, res in [(1, 0), (7, 20), (8, 0), (33, 0)]:
        k, v = rnd(L), rnd(L)
        m = cache.append_message(dev(k).data_ptr(), dev(v).data_ptr(), L, res)
        k_host[m], v_host[m] = k, v
    # several in one launch
    lens, ress = [9, 100, 4, 64], [0, 0, 40, 70]
    kk, vv = [rnd(L) for L in lens], [rnd(L) for L in lens]
    ids = cache.append_messages([dev(x).data_ptr() for x in kk], [dev(x).data_ptr() for x in vv], lens, ress)
    for m, k, v in zip(ids, kk, vv):
        k_host[m], v_host[m] = k, v
    # five more tokens for message 1 (reserve 20), then one more each for messages 1, 6 and 7
    k5, v5 = rnd(5), rnd(5)
    cache.append_tokens(1, dev(k5).data_ptr(), dev(v5).data_ptr(), 5)
    k_host[1], v_host[1] = np.concatenate([k_host[1], k5]), np.concatenate([v_host[1], v5])
    k3, v3 = rnd(3), rnd(3)
    cache.append_tokens_batch([6, 1, 7], dev(k3).data_ptr(), dev(v3).data_ptr())
    for j, m in enumerate([6, 1, 7]):
        k_host[m], v_host[m] = np.concatenate([k_host[m], k3[j:j + 1]]), np.concatenate([v_host[m], v3[j:j + 1]])
    torch.cuda.synchronize()

    n = h_kv * slots * D
    k_store = arena[:n].view(h_kv, slots, D).float().cpu().numpy()
    v_bits = arena[n:2 * n].view(torch.int16).view(h_kv, slots // 8, D, 8).cpu().numpy()
    k_bits_zero = arena[:n].view(torch.int16).view(h_kv, slots, D).cpu().numpy()
    used = np.zeros(slots, dtype=bool)
    for m in sorted(k_host):
        ln, slot0, reserved = cache.message_info(m)
        assert ln == k_host[m].shape[0]
        say(f"  message {m}: len {ln} slots [{slot0}, {slot0 + reserved})")
        used[slot0:slot0 + ln] = True
        # V: bit for bit, key-transposed
        want_v = torch.from_numpy(v_host[m]).to(torch.bfloat16).view(torch.int16).numpy()      # [L, H, D]
        for t in range(ln):
            s = slot0 + t
            assert np.array_equal(v_bits[:, s // 8, :, s % 8], want_v[t]), (m, t)
        # K: the oracle's rotation to the in-message index, rounded once
        want = np.transpose(orc.rope(k_host[m].astype(np.float64), np.arange(ln), theta), (1, 0, 2))  # [H, L, D]
        got = k_store[:, slot0:slot0 + ln, :]
        bound = 2.0 ** -8 * (np.abs(want) + np.abs(np.roll(want, D // 2, axis=-1))) + 1e-6
        assert (np.abs(got - want) <= bound).all(), m
    # nothing was written anywhere else: K rows and V columns of unused slots are still zero
    free = ~used
    assert not k_bits_zero[:, free, :].any()
    v_by_slot = np.transpose(v_bits, (0, 1, 3, 2)).reshape(h_kv, slots, D)
    assert not v_by_slot[:, free, :].any()
    cache.close()
