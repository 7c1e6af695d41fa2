#!/usr/bin/env python3
"""Benchmark of the choreographed-attention hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: append the
new message(s) to the global cache (fused append kernel), then one pc_attend over the
batch of calls (plan builder, attention kernels, split merge).  The messages the
calls select are already resident in the cache (they are the method's persistent
state), as are all inputs in HBM.

Prints ONE JSON line.  The headline is the largest configuration that fits one GPU, the
long-context mixed batch (configs[4]: one 2048-row prefill call and 32 decode calls, each
over ~64k selected tokens, 64 query heads): prefill TFLOP/s of the whole step against the
bf16 MFMA roofline, with the decode kernel of the same step against the HBM roofline beside
it.  The other configurations (configs[1] single prefill, configs[2] parallel decode,
configs[3] multi-agent rounds) and the further workloads are reported in the same line
under "extras", each with its own roofline and CPU baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0
HBM_PEAK_GBS = 8000.0


def visible_pairs(w, ev):
    """Sum over query rows of the number of visible keys, per call (algorithmic work)."""
    lens = w.message_lengths()
    out = []
    for c in ev.calls:
        n_par = sum(lens[m] for m, _ in c.sel)
        L = lens[c.self_msg] if c.self_msg >= 0 else 0
        own = sum(L - c.n_q + r + 1 for r in range(c.n_q)) if c.self_msg >= 0 else 0
        out.append((c.n_q, n_par, L, n_par * c.n_q + own))
    return out


def kernel_sources_hash():
    """sha256 over the library's sources: a committed counter summary is only quoted while it describes these kernels."""
    import hashlib
    h = hashlib.sha256()
    src = os.path.join(ROOT, "paper_2512_23049_amd", "csrc")
    for f in sorted(os.listdir(src)):
        if f.endswith((".hip", ".h")) and not f.startswith("_var_"):
            h.update(f.encode())
            h.update(open(os.path.join(src, f), "rb").read())
    return h.hexdigest()[:16]


_TRAFFIC_NOTE = None


def measured_traffic(kernel, workload):
    """HBM bytes per launch (fetch + write) from the committed rocprofv3 counter summary, or None when there is none
    for this kernel and workload or when the summary was taken with other kernel sources than the ones in the tree
    (its header names the hash of the sources it belongs to)."""
    global _TRAFFIC_NOTE
    path = os.path.join(ROOT, "profiles", "attention_kernels_hbm_traffic.txt")
    try:
        lines = open(path).read().splitlines()
    except OSError:
        _TRAFFIC_NOTE = "no counter summary under profiles/"
        return None
    tag = [ln.split(":", 1)[1].strip() for ln in lines if ln.startswith("# csrc_sha256:")]
    if not tag or tag[0] != kernel_sources_hash():
        _TRAFFIC_NOTE = ("profiles/attention_kernels_hbm_traffic.txt was taken with other kernel sources (%s, tree %s): "
                         "not quoted" % (tag[0] if tag else "untagged", kernel_sources_hash()))
        return None
    for ln in lines:
        f = ln.strip().split(",")
        if len(f) >= 6 and f[0].startswith(kernel) and f[5] == workload:
            return (float(f[3]) + float(f[4])) * 1e6
    return None


def time_steps(fn, steps, warmup, torch):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def bench_attend_workload(name, w, steps, warmup, torch, harness, reappend_self=True, tuning=None, sharing=None):
    """Loads the cache once, then times steps of (append new messages + attend)."""
    from paper_2512_23049_amd.binding import marshal_calls
    from pc_inputs import Call
    ev_idx = max(i for i, e in enumerate(w.events) if e.kind == "attend")
    ev = w.events[ev_idx]
    new_ids = sorted({c.self_msg for c in ev.calls if c.self_msg >= 0})
    lens = w.message_lengths()
    total_steps = (2 * steps + warmup + 2) if reappend_self else 0
    slack = total_steps * sum(((lens[m] + 31) // 32) * 32 for m in new_ids) + 64
    cache = harness.make_cache(w, slack_tokens=slack, extra_messages=total_steps * len(new_ids) + 16)
    if tuning:
        cache.set_tuning(*tuning)
    if sharing is not None:
        cache.set_decode_sharing(sharing)
    dw = harness.DeviceWorkload(w)
    dw.run(cache)                      # resident state: every message appended once
    torch.cuda.synchronize()
    att = [s for s in dw.steps if s[0] == "attend"][-1]
    _, calls, _, q, out, lse = att
    append_steps = [s for s in dw.steps if s[0] == "append"]
    new_kv = {m: (append_steps[m][1], append_steps[m][2], append_steps[m][3], append_steps[m][4]) for m in new_ids}

    # the call list is marshalled once; a step that appends the new messages again only patches their ids in
    # (building thousands of ctypes entries per step would otherwise be what the step waits for)
    marsh = marshal_calls(calls)
    with_self = [(i, c.self_msg) for i, c in enumerate(calls) if c.self_msg >= 0]

    k_ptrs = [new_kv[m][0].data_ptr() for m in new_ids]
    v_ptrs = [new_kv[m][1].data_ptr() for m in new_ids]
    n_lens = [new_kv[m][2] for m in new_ids]
    n_res = [new_kv[m][3] for m in new_ids]

    def step():
        if reappend_self:
            # the step's new messages go in with one pc_append_messages (one launch), as a batch of parallel calls does
            ids = cache.append_messages(k_ptrs, v_ptrs, n_lens, n_res)
            remap = dict(zip(new_ids, ids))
            for i, m in with_self:
                marsh[0][i].self_msg = remap[m]
            cache.attend(calls, q.data_ptr(), out.data_ptr(), 0, 0, marsh)
        else:
            cache.attend(calls, q.data_ptr(), out.data_ptr(), 0, 0, att[2])

    sec = time_steps(step, steps, warmup, torch)
    # same steps again with the library's per-kernel events switched on
    cache.profile_enable(True)
    cache.profile_read(reset=True)
    sec_prof = time_steps(step, steps, 2, torch)
    prof = cache.profile_read(reset=True)
    cache.profile_enable(False)
    per_kernel = {k: {"launches": n, "avg_us": (ms / n * 1e3 if n else None)} for k, (ms, n) in prof.items() if n}
    cache.close()
    return sec, sec_prof, per_kernel, visible_pairs(w, ev)


def cpu_baseline(w, sample, unit, cores_hint=None):
    """The fp64 oracle as it stands, timed on the host cores on a bounded sample."""
    from oracle import choreo_oracle as orc
    ev_idx = max(i for i, e in enumerate(w.events) if e.kind == "attend")
    ev = w.events[ev_idx]
    ks = [e.k for e in w.events[:ev_idx] if e.kind == "append"]
    vs = [e.v for e in w.events[:ev_idx] if e.kind == "append"]
    offs = np.concatenate([[0], np.cumsum([c.n_q for c in ev.calls])]).astype(int)
    lens = w.message_lengths()
    cores = len(os.sched_getaffinity(0))
    try:
        from threadpoolctl import threadpool_info
        th = [p.get("num_threads", 0) for p in threadpool_info() if p.get("user_api") == "blas"]
        if th:
            cores = min(cores, max(th))
    except Exception:
        pass
    t0 = time.perf_counter()
    pairs = 0
    tokens = 0
    for ci in sample["calls"]:
        c = ev.calls[ci]
        rows = sample["rows"](c.n_q)
        orc.attend_call(ks, vs, c.sel, c.self_msg, c.self_start, c.n_q, c.q_pos,
                        ev.q[offs[ci]:offs[ci + 1]], w.rope_theta, rows=rows)
        n_par = sum(lens[m] for m, _ in c.sel)
        L = lens[c.self_msg] if c.self_msg >= 0 else 0
        pairs += sum(n_par + (L - c.n_q + r + 1 if c.self_msg >= 0 else 0) for r in rows)
        tokens += n_par + L
    dt = time.perf_counter() - t0
    if unit == "TFLOP/s":
        val = 4.0 * w.head_dim * w.n_q_heads * pairs / dt / 1e12
    else:
        val = tokens * 2 * w.n_kv_heads * w.head_dim * 2 / dt / 1e9
    return {"value": val, "unit": unit, "cores": cores, "kind": "oracle", "sample": sample["desc"],
            "seconds": dt}


class Ctx:
    """What the sections share: the command line, the modules that need the GPU, the JSON line being built."""

    def __init__(self, args, torch, gen, harness):
        self.args, self.torch, self.gen, self.harness = args, torch, gen, harness
        self.line = {}
        self.achievable = None           # filled by section_achievable, read by section_decode


def decode_bytes(w, calls, vp):
    """(logical, unique) K/V bytes of the given one-row calls: 2 * H_kv * D * 2 bytes per selected token."""
    per_token = 2 * w.n_kv_heads * w.head_dim * 2
    lens = w.message_lengths()
    uniq = set()
    for c in calls:
        uniq.update(m for m, _ in c.sel)
        if c.self_msg >= 0:
            uniq.add(c.self_msg)
    return sum(v[1] + v[2] for v in vp) * per_token, sum(lens[m] for m in uniq) * per_token


def roofline_mfma(kernel, flops, k_us, workload):
    ach = (flops / (k_us * 1e-6) / 1e12) if k_us else None
    return {"bound": "mfma", "kernel": kernel, "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": (ach / MFMA_BF16_PEAK_TFLOPS) if ach else None, "traffic": measured_traffic(kernel, workload),
            "avg_kernel_us": k_us, "algorithmic_flops_per_launch": flops}


def roofline_hbm(kernel, b_logical, b_unique, k_us, workload):
    """HBM roofline of a decode kernel.  `achieved` / `frac` are on the bytes rocprofv3 counted for one launch (None
    while no counter summary for these kernel sources is committed); the rate on logical bytes (4096 B per
    call-selected token) is an EFFECTIVE one, because calls share messages, and is kept under its own name."""
    traffic = measured_traffic(kernel, workload)
    ach = (traffic / (k_us * 1e-6) / 1e9) if (traffic and k_us) else None
    return {"bound": "hbm", "kernel": kernel, "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": (ach / HBM_PEAK_GBS) if ach else None, "traffic": traffic, "avg_kernel_us": k_us,
            "basis": "HBM bytes counted by rocprofv3 per launch (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy)",
            "B_logical": b_logical, "B_unique": b_unique,
            "effective_gbs_on_logical_bytes": (b_logical / (k_us * 1e-6) / 1e9) if k_us else None,
            "gbs_on_unique_bytes": (b_unique / (k_us * 1e-6) / 1e9) if k_us else None}


def section_headline(cx):
    """configs[4], the largest configuration one GPU holds: fills the contract's fields of the JSON line."""
    args, torch, gen, harness = cx.args, cx.torch, cx.gen, cx.harness
    w5 = gen.long_context()
    sec, sec_prof, kern, vp = bench_attend_workload("long_context", w5, args.steps, args.warmup, torch, harness)
    ev = w5.events[-1]
    pre = [v for v in vp if v[0] > 1]
    dec = [v for v in vp if v[0] == 1]
    f_pre = 4.0 * w5.head_dim * w5.n_q_heads * sum(v[3] for v in pre)
    b_log, b_uni = decode_bytes(w5, [c for c in ev.calls if c.n_q == 1], dec)
    k_pre = kern.get("prefill", {}).get("avg_us")
    k_dec = kern.get("decode", {}).get("avg_us")
    line = {
        "metric": "choreographed attention prefill TFLOP/s + decode GB/s, % of MI355X roofline",
        "value": f_pre / sec / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[4] long-context mixed batch: 64 q heads / 8 kv heads / D 128; one 2048-row causal "
                               "prefill call over %d selected tokens + 32 one-row decode calls over ~64k selected tokens each "
                               "(all drawn from the same 512 cached messages); step = append the new messages (one "
                               "2048-token message, 32 one-token tails) + ONE pc_attend of the 33 calls; value = the "
                               "prefill call's algorithmic flops over the whole step's time" % pre[0][1],
                   "prefill_flops_per_step": f_pre, "decode_logical_bytes_per_step": b_log},
        # the dominant kernel of the step: the prefill call (it reads the packed copy the gather pass wrote)
        "roofline": roofline_mfma("pc_prefill_bf16_kernel", f_pre, k_pre, "long_context"),
        # the decode kernel of the same step (the 32 calls take the shared walk: the union of their messages is read once)
        "roofline_decode": roofline_hbm("pc_decode_shared_bf16_kernel", b_log, b_uni, k_dec, "long_context"),
        "decode_value": {"gbs_effective_on_logical_bytes_over_decode_kernel": (b_log / (k_dec * 1e-6) / 1e9) if k_dec else None},
        # kernel times come from a second pass of the same steps with the library's per-kernel events on; that pass keeps
        # every kernel on one stream (the timed pass forks the decode kernels onto a second stream), hence two step times
        "kernels_us": {k: v["avg_us"] for k, v in kern.items()},
        "ms_per_step_with_kernel_events": sec_prof * 1e3,
    }
    if _TRAFFIC_NOTE:
        line["traffic_note"] = _TRAFFIC_NOTE
    if not args.skip_cpu:
        rows = list(range(0, 2048, 8))
        line["cpu_baseline"] = cpu_baseline(
            w5, {"calls": [32, 0, 10, 21, 31], "rows": lambda n: rows if n > 1 else [0],
                 "desc": "configs[4] sample: the prefill call's every 8th query row (256 of 2048 rows, all 64 heads, all "
                         "%d keys) and 4 of the 32 decode calls; TFLOP/s on the sample's visible (row, key) pairs" % pre[0][1]},
            "TFLOP/s")
    del w5
    cx.line = line


def section_single_prefill(cx):
    """configs[1]: one 512-row prefill call over 16 selected messages."""
    args, torch, gen, harness, line = cx.args, cx.torch, cx.gen, cx.harness, cx.line
    w2 = gen.single_prefill()
    sec, sec_prof, kern, vp = bench_attend_workload("single_prefill", w2, args.steps, args.warmup, torch, harness)
    flops = 4.0 * w2.head_dim * w2.n_q_heads * sum(v[3] for v in vp)
    k_pre = kern.get("prefill", {}).get("avg_us")
    out = {
        "workload": "configs[1] single-call prefill: 32 q heads / 8 kv heads / D 128, 16 selected messages (%d keys) + causal "
                    "512-token new message; step = append new message + pc_attend" % vp[0][1],
        "value": flops / sec / 1e12, "unit": "TFLOP/s", "ms_per_step": sec * 1e3, "flops_per_step": flops,
        "roofline": roofline_mfma("pc_prefill_bf16_kernel", flops, k_pre, "single_prefill"),
        "kernels_us": {k: v["avg_us"] for k, v in kern.items()}, "ms_per_step_with_kernel_events": sec_prof * 1e3}
    if cx.achievable and out["roofline"]["achieved"]:
        out["roofline"]["frac_of_achievable"] = out["roofline"]["achieved"] / cx.achievable["mfma_bf16_random_operands_tflops"]
    if not args.skip_cpu:
        out["cpu_baseline"] = cpu_baseline(
            w2, {"calls": [0], "rows": lambda n: list(range(n)),
                 "desc": "configs[1] whole: all 512 query rows, all 32 heads, all keys"}, "TFLOP/s")
    line.setdefault("extras", {})["single_prefill"] = out
    del w2


def section_achievable(cx):
    """What this chip sustains for the two resources the kernels are priced against (probe kernels of the library)."""
    args, torch, gen, harness, line = cx.args, cx.torch, cx.gen, cx.harness, cx.line
    from paper_2512_23049_amd.probe import probe_hbm_read, probe_mfma_bf16
    sink = torch.zeros(4, dtype=torch.float32, device="cuda:0")
    g = torch.Generator(device="cpu").manual_seed(7)
    ops_rand = torch.randn(8192, generator=g).to(torch.bfloat16).to("cuda:0")
    ops_zero = torch.zeros(8192, dtype=torch.bfloat16, device="cuda:0")
    big = torch.ones(1 << 29, dtype=torch.float32, device="cuda:0")        # 2 GiB, several times the last-level cache
    st = torch.cuda.current_stream().cuda_stream
    achievable = {
        "mfma_bf16_random_operands_tflops": probe_mfma_bf16(ops_rand.data_ptr(), ops_rand.numel() * 2, sink.data_ptr(),
                                                            iters=16384, reps=5, stream=st),
        "mfma_bf16_zero_operands_tflops": probe_mfma_bf16(ops_zero.data_ptr(), ops_zero.numel() * 2, sink.data_ptr(),
                                                          iters=16384, reps=5, stream=st),
        "hbm_stream_read_gbs": probe_hbm_read(big.data_ptr(), big.numel() * 4, sink.data_ptr(), reps=10, stream=st),
        "how": "pc_probe_mfma_bf16 (bare 32x32x16 bf16 MFMA loop, 2 waves per SIMD on every CU; N(0,1) operands, "
               "then all-zero operands) and pc_probe_hbm_read (2 GiB streaming read)",
    }
    del big, ops_rand, ops_zero
    line["achievable"] = achievable
    if line["roofline"]["achieved"]:
        line["roofline"]["frac_of_achievable"] = (line["roofline"]["achieved"]
                                                  / achievable["mfma_bf16_random_operands_tflops"])
    if line["roofline_decode"]["achieved"]:
        line["roofline_decode"]["frac_of_achievable"] = line["roofline_decode"]["achieved"] / achievable["hbm_stream_read_gbs"]
    cx.achievable = achievable


def section_decode(cx):
    """configs[2]: the parallel decode step, HBM roofline on counted bytes, effective rate on logical bytes."""
    args, torch, gen, harness, line = cx.args, cx.torch, cx.gen, cx.harness, cx.line
    w3 = gen.parallel_decode()
    sec, sec_prof, kern, vp = bench_attend_workload("parallel_decode", w3, args.steps, args.warmup, torch, harness,
                                                    reappend_self=False)
    ev = w3.events[-1]
    b_logical, b_unique = decode_bytes(w3, ev.calls, vp)
    k_dec = kern.get("decode", {}).get("avg_us")
    out = {
        "workload": "configs[2] parallel decode: 64 calls x (2048-token system + 8 pool messages + 64-token tail), "
                    "one query token per call; step = pc_attend",
        "value": b_logical / sec / 1e9, "unit": "GB/s (effective: logical bytes, 4096 B per call-selected token, over the step)",
        "ms_per_step": sec * 1e3, "B_logical": b_logical, "B_unique": b_unique,
        "roofline": roofline_hbm("pc_decode_bf16_kernel", b_logical, b_unique, k_dec, "parallel_decode"),
        "kernels_us": {k: v["avg_us"] for k, v in kern.items()}, "ms_per_step_with_kernel_events": sec_prof * 1e3,
    }
    if cx.achievable and out["roofline"]["achieved"]:
        out["roofline"]["frac_of_achievable"] = out["roofline"]["achieved"] / cx.achievable["hbm_stream_read_gbs"]
    if not args.skip_cpu:
        out["cpu_baseline"] = cpu_baseline(
            w3, {"calls": list(range(64)), "rows": lambda n: [0],
                 "desc": "configs[2] whole: all 64 calls"}, "GB/s")
    line.setdefault("extras", {})["parallel_decode"] = out
    del w3


def section_long_context_decode(cx):
    """The decode calls of configs[4] as a step of their own: shared walk against per-call walk."""
    args, torch, gen, harness, line = cx.args, cx.torch, cx.gen, cx.harness, cx.line
    w5d = gen.long_context(n_prefill_q=0)
    steps5 = max(3, min(args.steps, 50))
    out_ld = {}
    for name, mode in (("shared_walk", 0), ("per_call_walk", 1)):
        sec, _, kern, vp = bench_attend_workload("long_context_decode", w5d, steps5, 20, torch, harness,
                                                 reappend_self=False, sharing=mode)
        b_dec = sum(v[1] + v[2] for v in vp) * 4096
        out_ld[name] = {"us_per_step": sec * 1e6, "gbs_logical": b_dec / sec / 1e9,
                        "kernels_us": {k: v["avg_us"] for k, v in kern.items()}}
    line.setdefault("extras", {})["long_context_decode_only"] = {
        "workload": "the 32 one-row calls of configs[4] alone (each ~64k selected tokens of the same 512 messages); "
                    "step = one pc_attend, host planning included; shared walk (default rule) against "
                    "pc_set_decode_sharing(1)",
        "B_logical": b_dec, **out_ld}
    del w5d


def section_rounds(cx):
    """configs[3]: multi-agent rounds, appends and prefills interleaved; whole sequences and a per-round breakdown."""
    args, torch, gen, harness, line = cx.args, cx.torch, cx.gen, cx.harness, cx.line
    w4 = gen.multi_agent_rounds()
    dw = harness.DeviceWorkload(w4)
    reps = max(3, min(args.steps, 20))
    caches = [harness.make_cache(w4) for _ in range(reps + 2)]
    for c in caches[:2]:
        dw.run(c, want_lse=False, batch_appends=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for c in caches[2:]:
        dw.run(c, want_lse=False, batch_appends=True)
    torch.cuda.synchronize()
    sec4 = (time.perf_counter() - t0) / reps
    for c in caches:
        c.close()
    f_round = [4.0 * w4.head_dim * w4.n_q_heads * sum(v[3] for v in visible_pairs(w4, e))
               for e in w4.events if e.kind == "attend"]
    f4 = sum(f_round)
    # one more sequence with the library's kernel events on, read round by round: kernel time per class
    # (append GB/s on 2 * 4096 B per token, prefill TFLOP/s on the kernel's own time) and wall time per round
    c = harness.make_cache(w4)
    dw.run(c, want_lse=False, batch_appends=True)
    c.close()
    c = harness.make_cache(w4)
    c.profile_enable(True)
    c.profile_read(reset=True)
    per_round, pending, tok_round = [], [], 0
    torch.cuda.synchronize()
    t_r = time.perf_counter()
    for s_ in dw.steps:
        if s_[0] == "append":
            pending.append(s_)
            tok_round += s_[3]
            continue
        c.append_messages([p_[1].data_ptr() for p_ in pending], [p_[2].data_ptr() for p_ in pending],
                          [p_[3] for p_ in pending], [p_[4] for p_ in pending])
        pending = []
        _, calls_, m_, q_, out_, lse_ = s_
        c.attend(calls_, q_.data_ptr(), out_.data_ptr(), 0, 0, m_)
        pr = c.profile_read(reset=True)                     # waits for the round's work
        now = time.perf_counter()
        k_app = pr["append"][0] * 1e-3
        k_pre = pr["prefill"][0] * 1e-3
        r = len(per_round)
        per_round.append({"wall_ms": (now - t_r) * 1e3, "append_kernel_us": k_app * 1e6,
                          "append_gbs": (2 * 4096 * tok_round / k_app / 1e9) if k_app > 0 else None,
                          "prefill_kernel_us": k_pre * 1e6,
                          "prefill_tflops_kernel": (f_round[r] / k_pre / 1e12) if k_pre > 0 else None,
                          "other_kernels_us": sum(v[0] for k_, v in pr.items() if k_ not in ("append", "prefill")) * 1e3})
        tok_round = 0
        t_r = now
    c.profile_enable(False)
    c.close()
    k_pre_total = sum(r_["prefill_kernel_us"] for r_ in per_round)         # six launches: the six rounds
    out = {
        "workload": "configs[3]: 8 agents x 6 rounds; per round one pc_append_messages of the 8 new 256-token messages "
                    "and one pc_attend of the 8 prefill calls",
        "value": f4 / sec4 / 1e12, "unit": "TFLOP/s (all six rounds' attention flops over the whole sequence, appends included)",
        "ms_per_sequence": sec4 * 1e3, "flops": f4, "reps": reps,
        # the six prefill launches of a sequence together (they differ in size: round r attends over 8 (r - 1) + 1 messages)
        "roofline": {"bound": "mfma", "kernel": "pc_prefill_bf16_kernel", "achieved": f4 / (k_pre_total * 1e-6) / 1e12,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": f4 / (k_pre_total * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": None, "sum_of_six_kernel_us": k_pre_total, "algorithmic_flops_per_sequence": f4},
        "per_round_with_kernel_events": per_round}
    if not args.skip_cpu:
        # the oracle on the whole last round (8 calls x 256 rows over all 48 messages): the largest of the six
        out["cpu_baseline"] = cpu_baseline(
            w4, {"calls": list(range(8)), "rows": lambda n: list(range(n)),
                 "desc": "configs[3] last round whole: 8 calls x 256 rows over the 40 messages of the earlier rounds + own"},
            "TFLOP/s")
    line.setdefault("extras", {})["multi_agent_rounds"] = out
    del w4


def section_baseline(cx):
    """The attention and append work a prefix-caching baseline would do for the same rounds."""
    args, torch, gen, harness, line = cx.args, cx.torch, cx.gen, cx.harness, cx.line
    def run_sequence(w, reps):
        dw_ = harness.DeviceWorkload(w)
        caches = [harness.make_cache(w) for _ in range(reps + 1)]
        dw_.run(caches[0], want_lse=False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for c_ in caches[1:]:
            dw_.run(c_, want_lse=False)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / reps
        for c_ in caches:
            c_.close()
        fl, toks = 0.0, 0
        for i, e in enumerate(w.events):
            if e.kind == "attend":
                lens = w.message_lengths(upto_event=i)
                for c in e.calls:
                    n_par = sum(lens[m] for m, _ in c.sel)
                    L = lens[c.self_msg]
                    fl += 4.0 * w.head_dim * w.n_q_heads * sum(n_par + L - c.n_q + r + 1 for r in range(c.n_q))
            elif e.kind == "append":
                toks += int(e.k.shape[0])
        return dt, fl, toks
    comp = {}
    for name, (na, nr) in {"8 agents x 6 rounds (configs[3])": (8, 6), "3 agents x 3 rounds (the paper's parallel debate)": (3, 3)}.items():
        t_c, f_c, k_c = run_sequence(gen.multi_agent_rounds(n_agents=na, n_rounds=nr), 5)
        t_b, f_b, k_b = run_sequence(gen.prefix_cache_baseline_rounds(n_agents=na, n_rounds=nr), 5)
        comp[name] = {"choreographed_ms": t_c * 1e3, "baseline_ms": t_b * 1e3, "time_ratio": t_b / t_c,
                      "choreographed_attention_gflop": f_c / 1e9, "baseline_attention_gflop": f_b / 1e9,
                      "flop_ratio": f_b / f_c, "choreographed_tokens_encoded": k_c, "baseline_tokens_encoded": k_b}
    line.setdefault("extras", {})["prefix_cache_baseline"] = {
        "workload": "attention and cache-append work only, 256-token messages: choreographed rounds (each agent "
                    "prefills its new message over the cached messages of all earlier rounds) against a prefix-caching "
                    "baseline (each agent keeps its own prompt as prefix and encodes the other agents' last-round "
                    "messages again with its new one); the model's other layers, which the baseline also runs again "
                    "for every re-encoded token, are not part of this path",
        **comp}


def section_decode_loop(cx):
    """Decode loop: tails growing one token per step (append + attend per step)."""
    args, torch, gen, harness, line = cx.args, cx.torch, cx.gen, cx.harness, cx.line
    w6 = gen.decode_loop()
    dw = harness.DeviceWorkload(w6)
    first_loop = next(i for i, s_ in enumerate(dw.steps) if s_[0] == "attend")
    n_steps = sum(1 for s_ in dw.steps if s_[0] == "attend")
    times = []
    for rep, fused in enumerate((True, True, True, False, False)):
        cache = harness.make_cache(w6)
        for s_ in dw.steps[:first_loop]:
            cache.append_message(s_[1].data_ptr(), s_[2].data_ptr(), s_[3], s_[4])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        held = None
        for s_ in dw.steps[first_loop:]:
            if s_[0] == "extend":
                if fused:
                    held = s_
                else:
                    cache.append_tokens_batch(s_[3], s_[1].data_ptr(), s_[2].data_ptr())
            elif held is not None:
                cache.decode_step(held[3], held[1].data_ptr(), held[2].data_ptr(), s_[1], s_[3].data_ptr(), s_[4].data_ptr(),
                                  0, 0, s_[2])
                held = None
            else:
                cache.attend(s_[1], s_[3].data_ptr(), s_[4].data_ptr(), 0, 0, s_[2])
        torch.cuda.synchronize()
        times.append(time.perf_counter() - t0)
        cache.close()
    sec6 = min(times[1:3])                 # one pc_decode_step per step
    sec6_two = min(times[3:])              # pc_append_tokens_batch + pc_attend per step
    b6 = 0
    for i, e in enumerate(w6.events):
        if e.kind == "attend":
            lens = w6.message_lengths(upto_event=i)
            b6 += sum(sum(lens[m] for m, _ in c.sel) + lens[c.self_msg] for c in e.calls) * 4096
    n_calls6 = len(w6.events[-1].calls)
    line.setdefault("extras", {})["decode_loop"] = {
        "workload": "configs[2]-shaped parallel decode as a loop: 64 calls (2048-token system + 8 pool messages each), "
                    "tails grow from 1 to 64 tokens; a step = one pc_decode_step (one token per call appended beside the plan "
                    "builder, then the attention); us_per_step_two_calls: the same step as pc_append_tokens_batch + pc_attend",
        "steps": n_steps, "us_per_step": sec6 / n_steps * 1e6, "us_per_step_two_calls": sec6_two / n_steps * 1e6,
        "tokens_per_s": n_calls6 * n_steps / sec6,
        "gbs_logical": b6 / sec6 / 1e9, "B_logical_total": b6}
    del w6, dw


def section_reposition(cx):
    """Position updates in place against in-kernel rotation on configs[4]'s prefill call."""
    args, torch, gen, harness, line = cx.args, cx.torch, cx.gen, cx.harness, cx.line
    from paper_2512_23049_amd.binding import marshal_calls
    w5 = gen.long_context(n_decode=0)
    cache = harness.make_cache(w5)
    cache.set_key_gather(1)            # the comparison is between the two ways of placing keys IN the cache: no gathered copy
    dw = harness.DeviceWorkload(w5)
    dw.run(cache)
    torch.cuda.synchronize()
    att = [s_ for s_ in dw.steps if s_[0] == "attend"][-1]
    _, calls, mc, q, out, lse = att
    call = calls[0]
    lens = w5.message_lengths()
    starts, s_self, _ = cache.resolve_call(call)
    reps = max(3, min(args.steps, 10))

    def attend_only():
        cache.attend(calls, q.data_ptr(), out.data_ptr(), 0, 0, mc)
    t_before = time_steps(attend_only, reps, 2, torch)
    cache.profile_enable(True)
    cache.profile_read(reset=True)
    moved = [(m, st_) for (m, _), st_ in zip(call.sel, starts)] + [(call.self_msg, s_self)]
    t0 = time.perf_counter()
    for m, st_ in moved:
        cache.reposition(m, st_)
    torch.cuda.synchronize()
    t_move = time.perf_counter() - t0
    prof = cache.profile_read(reset=True)
    t_after = time_steps(attend_only, reps, 2, torch)
    # the same moves as one launch: back to base 0, then to the starts again
    ids = [m for m, _ in moved]
    cache.reposition_batch(ids, [0] * len(ids))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    cache.reposition_batch(ids, [st_ for _, st_ in moved])
    torch.cuda.synchronize()
    t_batch = time.perf_counter() - t0
    prof_b = cache.profile_read(reset=True)
    cache.profile_enable(False)
    pairs5 = sum(v[3] for v in visible_pairs(w5, w5.events[-1]))
    f5 = 4.0 * w5.head_dim * w5.n_q_heads * pairs5
    k_bytes = sum(lens[m] for m, _ in moved) * w5.n_kv_heads * w5.head_dim * 2
    k_batch_us = (prof_b["reposition"][0] / prof_b["reposition"][1] * 1e3) if prof_b["reposition"][1] else None
    line.setdefault("extras", {})["reposition"] = {
        "workload": "configs[4] prefill call alone (2048 rows over ~64k tokens in ~410 messages of 64-256 tokens): "
                    "gather pass off; pc_attend with every parent at base 0 (queries turned per parent), then every parent moved to "
                    "the start the call gives it (one pc_reposition each, and again as one pc_reposition_batch), "
                    "then the same pc_attend (one turn in all)",
        "attend_ms_before": t_before * 1e3, "attend_ms_after": t_after * 1e3,
        "tflops_before": f5 / t_before / 1e12, "tflops_after": f5 / t_after / 1e12,
        "messages_moved": len(moved), "one_by_one_ms_host_clock": t_move * 1e3,
        "one_by_one_kernel_us_avg": (prof["reposition"][0] / prof["reposition"][1] * 1e3) if prof["reposition"][1] else None,
        "batched_ms_host_clock": t_batch * 1e3, "batched_kernel_us": k_batch_us,
        "batched_gbs": (2 * k_bytes / (k_batch_us * 1e-6) / 1e9) if k_batch_us else None,
        "bytes_read_plus_written": 2 * k_bytes,
    }
    cache.close()
    del w5


def section_backward(cx):
    """Gradient path (functional, untuned) on a small shape."""
    args, torch, gen, harness, line = cx.args, cx.torch, cx.gen, cx.harness, cx.line
    wb = gen.single_prefill(n_msgs=24, len_lo=40, len_hi=300, n_sel=6, n_new=200)
    cache = harness.make_cache(wb)
    dw = harness.DeviceWorkload(wb)
    dw.run(cache)
    torch.cuda.synchronize()
    att = [s_ for s_ in dw.steps if s_[0] == "attend"][-1]
    _, calls, mc, q, out, lse = att
    slots = cache.cache_info()[2]
    d_out = torch.randn(tuple(q.shape), device="cuda:0").to(q.dtype)
    d_q = torch.empty(tuple(q.shape), dtype=torch.float32, device="cuda:0")
    d_k = torch.zeros((slots, wb.n_kv_heads, wb.head_dim), dtype=torch.float32, device="cuda:0")
    d_v = torch.zeros_like(d_k)
    cache.attend(calls, q.data_ptr(), out.data_ptr(), lse.data_ptr(), 0, mc)

    def bwd():
        cache.attend_backward(calls, q.data_ptr(), lse.data_ptr(), d_out.data_ptr(), d_q.data_ptr(), d_k.data_ptr(),
                              d_v.data_ptr())
        cache.grad_keys_finalize(d_k.data_ptr())
    t_b = time_steps(bwd, max(3, min(args.steps, 20)), 2, torch)
    pairs_b = sum(v[3] for v in visible_pairs(wb, wb.events[-1]))
    line.setdefault("extras", {})["backward"] = {
        "workload": "scaled single prefill (200 causal rows over 6 parents of 40-300 tokens + the new message, 32/8 heads, "
                    "bf16 cache): pc_attend_backward + pc_grad_keys_finalize; a functional path (plain fp32 vector "
                    "kernels, no matrix cores), not tuned",
        "ms_per_call": t_b * 1e3,
        "gflops": 2.5 * 4.0 * wb.head_dim * wb.n_q_heads * pairs_b / t_b / 1e9,
    }
    cache.close()
    del wb


# sections after the headline, in the order they run; --only names them
SECTIONS = [("achievable", section_achievable), ("prefill", section_single_prefill), ("decode", section_decode),
            ("longdecode", section_long_context_decode), ("rounds", section_rounds), ("baseline", section_baseline),
            ("loop", section_decode_loop), ("reposition", section_reposition), ("backward", section_backward)]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--skip-extras", action="store_true")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--no-headline", action="store_true",
                    help="run only the sections --only names (profiling runs: one workload per process); the JSON line "
                         "then holds those sections alone")
    ap.add_argument("--only", default="", help="comma list of sections: achievable,prefill,decode,longdecode,rounds,baseline,loop,reposition,backward")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also launch one plain device copy of this many MiB (reference for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import pc_inputs as gen
    from paper_2512_23049_amd import harness
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    only = set(x for x in args.only.split(",") if x)
    if args.copy_probe_mib > 0:
        src = torch.ones(args.copy_probe_mib << 18, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cx = Ctx(args, torch, gen, harness)
    if args.no_headline:
        cx.line = {"note": "sections only (--no-headline)", "roofline": {"achieved": None}, "roofline_decode": {"achieved": None}}
    else:
        section_headline(cx)
    if not args.skip_extras:
        for name, section in SECTIONS:
            if not only or name in only:
                section(cx)
    line = cx.line
    line["context"] = ("paper reports whole-workflow ratios only: 2.0-6.2x faster time-to-first-token and up to 2.2x "
                       "end-to-end vs prefix caching (Llama-3.1-8B; one A100-80GB is the only GPU the paper names); "
                       "no kernel-level figure exists to compare with")
    print(json.dumps(line))


if __name__ == "__main__":
    main()
