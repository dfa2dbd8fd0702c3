#!/usr/bin/env python3
"""Benchmark of the paged GQA decode-attention hot path on one MI355X.

One "step" = one pass of the whole path over one batch already resident in
HBM: host re-plan of the sequence splits (oserve_plan_update), upload of the
per-request records, the split kernel and the log-sum-exp merge kernel.

Prints ONE JSON line on stdout: whole-job throughput as effective KV GB/s
(valid-token K+V bytes per step / step time) of the heterogeneous mix (workload
3), the roofline of the dominant (split) kernel measured with HIP events on the
launch stream, the fp64 oracle timed on the host cores on a bounded sample of
the same workload, the errors of the timed output against that oracle
(`parity`), and - under `extra` - shorter measurements of the other benchmark
workloads, the chunked-prefill kernel, the KV-block migration copies and the
mixed prefill + decode step.

Order of a measurement: W warm-up steps, a first timed block of K steps
(`value_unsettled`), an untimed settling phase (the part's clocks ramp for
seconds after idle), then the K timed steps `value` is computed from;
`untimed_steps` counts everything that ran before those.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 0..8] [--split-tokens T] [--no-extra]
                  [--prefill 0|1|2] [--migrate] [--mixed]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E peak

# HBM bytes per launch of the split kernel (read + written) from rocprofv3 FETCH_SIZE / WRITE_SIZE, each
# scaled by a plain copy of known size.  A recorded profile value, not a measurement of the run that
# prints it: it is reported only while the kernel and planner sources still hash to what they were when the
# profile was taken and the plan has the same number of work items; otherwise `traffic` is null.
RECORDED_TRAFFIC = {"config": 3, "bytes": round(3397594.7 * 2048 + 10499.5 * 1024), "work_items": 5192,
                    "sources_sha16": "ceed02d1e3708ca0", "profile": "profiles/split_kernel_cfg3_heterogeneous_mix.md"}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3, help="workload index: 0..4 are the five benchmark configs (default 3, the heterogeneous mix), "
                         "5..8 shape variants of the mix (MHA shard, 8q/1kv shard, pages of 32 and 64 tokens)")
    ap.add_argument("--split-tokens", type=int, default=0, help="0 = automatic split sizing")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--settle-seconds", type=float, default=20.0,
                    help="upper bound of the untimed settling phase before the warm-up steps (0 = none)")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="BYTES",
                    help="instead of the benchmark, run a plain device copy of BYTES bytes --steps times "
                         "(the known-size kernel that hardware byte counters are scaled by)")
    ap.add_argument("--prefill", type=int, default=-1, metavar="W",
                    help="instead of the decode benchmark, time the chunked-prefill kernel on prefill workload W "
                         "(0: 16 whole prompts of 4096 tokens; 1: 8 chunks of 2048 tokens at the end of 32768-token "
                         "contexts; 2: 64 chunks of 512 tokens on the heterogeneous mix's long requests), Llama-3-8B heads")
    ap.add_argument("--migrate", action="store_true",
                    help="instead of the decode benchmark, time the KV-block migration copies (gather into a staging "
                         "chunk, scatter into a target pool) of the long requests of the heterogeneous mix")
    ap.add_argument("--mixed", action="store_true",
                    help="instead of the decode benchmark, time one mixed step (the decode requests of the heterogeneous "
                         "mix + 8 prefill chunks of 512 tokens in one call) against the decode call followed by the prefill call")
    ap.add_argument("--no-extra", dest="extra", action="store_false",
                    help="with the default workload, skip the side measurements (other configs, prefill, migration) "
                         "that are attached under the `extra` key")
    ap.add_argument("--extra-settle-seconds", type=float, default=6.0,
                    help="cap of the settling phase of each side measurement")
    ap.add_argument("--cpu-token-heads", type=float, default=120e6,
                    help="size of the oracle's sample in (token, query head) pairs")
    return ap.parse_args()


def build_inputs(w, wl, torch):
    """Inputs on the GPU; small workloads get several independent copies so that
    successive steps do not find their K/V in the 256 MB last-level cache."""
    lens = wl.context_lens(w)
    nbytes = wl.kv_bytes(lens, w.num_kv_heads, w.head_dim)
    copies = int(min(8, max(1, -(-int(1.5e9) // max(nbytes, 1)))))
    sets = []
    for c in range(copies):
        sets.append(wl.make_inputs(w, device="cuda", seed=w.seed + 1000 * c, lens=lens,
                                   fill_unused=w.pool_pages_fixed is None or w.index == 0))
    return sets, nbytes


def cpu_baseline(inp, wl, torch, budget_token_heads, gpu_out=None):
    """Time the oracle, as it stands, on whole requests of the batch until the budget is met.  Returns the
    baseline record and, if `gpu_out` (the output tensor of the timed steps) is given, the errors of its rows
    of the sampled requests against what the oracle computed for them."""
    from oracle import paged_attention_oracle as oracle
    w = inp.workload
    lens = inp.context_lens_host
    order = wl.CounterRng(w.seed + 7).permutation(len(lens))
    chosen, acc = [], 0.0
    for b in order:
        chosen.append(int(b))
        acc += float(lens[b]) * w.num_q_heads
        if acc >= budget_token_heads:
            break
    elapsed = 0.0
    ref_rows = []
    for b in chosen:
        n = (int(lens[b]) + w.page_size - 1) // w.page_size
        ids = inp.block_table[b, :n].long()
        k = inp.k_pages[ids].cpu()
        v = inp.v_pages[ids].cpu()
        q = inp.q[b:b + 1].cpu()
        bt = np.arange(n, dtype=np.int32)[None, :]
        cl = np.array([lens[b]], dtype=np.int32)
        t0 = time.perf_counter()
        ref_rows.append(oracle.paged_decode_attn(q, k, v, bt, cl, inp.scale)[0])
        elapsed += time.perf_counter() - t0
    sample_bytes = wl.kv_bytes(lens[chosen], w.num_kv_heads, w.head_dim)
    parity = None
    if gpu_out is not None:
        ref = np.stack(ref_rows)                                          # [requests, Hq, D] float64
        got = gpu_out[torch.tensor(chosen, device=gpu_out.device)].cpu().double().numpy()
        per_row = np.linalg.norm(got - ref, axis=2) / np.linalg.norm(ref, axis=2)
        parity = {"max_abs": float(np.abs(got - ref).max()),
                  "rel_l2": float(np.linalg.norm(got - ref) / np.linalg.norm(ref)),
                  "worst_row_rel_l2": float(per_row.max()),
                  "rows": int(ref.shape[0] * ref.shape[1]), "requests": len(chosen), "of_requests": len(lens),
                  "tolerance": {"max_abs": 1e-2, "rel_l2": 2e-3},
                  "what": "output of the last timed step vs the fp64 oracle, every element of the sampled requests"}
        parity["ok"] = bool(parity["max_abs"] <= 1e-2 and parity["rel_l2"] <= 2e-3 and np.isfinite(got).all())
    return {
        "value": sample_bytes / elapsed / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"{len(chosen)} of {len(lens)} whole requests (all {w.num_q_heads} query heads, "
                  f"{int(lens[chosen].sum())} tokens, {sample_bytes / 1e9:.3f} GB of K+V) in {elapsed:.1f} s, "
                  f"single thread",
    }, parity


MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 peak


def settle(step, torch, max_s):
    """Untimed steps until the step rate has stopped improving for 4 s (at most max_s seconds).

    After idle, and for some seconds after another process has used the GPU heavily, the part runs the same
    kernels up to 6 % slower and recovers in a few discrete jumps about a second apart (its clocks ramp);
    the handful of warm-up steps of the contract end inside that ramp.  Returns (seconds, steps) spent."""
    if max_s <= 0:
        return 0.0, 0
    begin = time.perf_counter()
    best, best_at, n, block = float("inf"), begin, 0, 4
    while True:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(block):
            step(n)
            n += 1
        torch.cuda.synchronize()
        now = time.perf_counter()
        per_step = (now - t0) / block
        block = max(4, min(20000, int(0.1 / per_step)))      # blocks of about 0.1 s
        if per_step < best * 0.997:
            best, best_at = per_step, now
        if now - best_at > 4.0 or now - begin > max_s:
            return now - begin, n


def timed_block(step, n, torch):
    """n steps bracketed by synchronisations: ms per step (the larger of wall clock and GPU events)."""
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    start.record()
    for i in range(n):
        step(i)
    stop.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    gpu_ms = start.elapsed_time(stop)
    return max(wall_ms, gpu_ms) / n, gpu_ms / n


def common_fields(args, ms_per_step, untimed):
    return {"n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "untimed_steps": untimed,
            "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "data": "synthetic"}


def bench_prefill(args, torch, binding, wl, which):
    """One step = oserve_prefill_plan_update + the prefill kernel on inputs resident in HBM."""
    name = wl.PREFILL_WORKLOAD_NAMES[which]
    w, lens, qlens = wl.prefill_workload(which)
    inp = wl.make_inputs(w, device="cuda", seed=w.seed, lens=lens)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed + 1)
    q = torch.randn(int(qlens.sum()), w.num_q_heads, w.head_dim, generator=gen, device="cuda").to(torch.bfloat16)
    out = torch.empty(q.shape, dtype=torch.float32, device="cuda")
    plan = binding.PrefillPlan(lens, qlens, w.num_q_heads, w.num_kv_heads, w.head_dim, w.page_size,
                               inp.block_table.shape[1], 0)

    def step(i=0):
        plan.update(lens, qlens)
        binding.paged_prefill_attn(plan, q, inp.k_pages, inp.v_pages, inp.block_table, w.scale, out)

    for _ in range(args.warmup):
        step()
    unsettled_ms, _ = timed_block(step, args.steps, torch)
    settle_s, settle_steps = settle(step, torch, args.settle_seconds)
    plan.enable_timing(True)
    ms_per_step, _ = timed_block(step, args.steps, torch)
    kernel_ms, cnt = plan.kernel_ms()
    plan.enable_timing(False)
    # 2 products x 2 flop x head_dim per (query token, visible key) and query head; query i of a request sees L - n + i + 1 keys
    pairs = sum(int(n) * (int(L) - int(n)) + int(n) * (int(n) + 1) // 2 for L, n in zip(lens, qlens))
    flop = 4.0 * w.head_dim * w.num_q_heads * pairs
    value = flop / (ms_per_step * 1e-3) / 1e12
    achieved = flop / (kernel_ms * 1e-3) / 1e12
    res = {"metric": "chunked-prefill attention TFLOP/s (causal, paged KV)", "value": round(value, 1), "unit": "TFLOP/s",
           "value_unsettled": round(flop / (unsettled_ms * 1e-3) / 1e12, 1)}
    res.update(common_fields(args, ms_per_step, args.warmup + args.steps + settle_steps))
    res.update({
        "dtype": "bf16",
        "config": {"workload": f"prefill{which}: {name}; 32q/8kv heads, head_dim 128, page 16, "
                               f"{int(qlens.sum())} query tokens, {flop / 1e12:.3f} TFLOP per step",
                   "work_items": plan.num_work_items, "block_tokens": plan.block_tokens,
                   "settle_s": round(settle_s, 2), "settle_steps": settle_steps},
        "roofline": {"bound": "mfma", "kernel": "paged_prefill_kernel", "achieved": round(achieved, 1),
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
                     "traffic": None, "avg_kernel_ms": round(kernel_ms, 5), "launches_timed": cnt,
                     "algorithmic_flop_per_launch": flop}})
    return res


def bench_migrate(args, torch, binding, wl):
    """One step = gather of the long requests' pages (all 8 kv heads) into a staging chunk + scatter of that
    chunk into a target pool with 15 % headroom, i.e. one layer's chunk of a migration on one GPU."""
    w = wl.WORKLOADS[3]
    inp = wl.make_inputs(w, device="cuda")
    lens = inp.context_lens_host
    rows = np.nonzero(lens >= 8192)[0].astype(np.int32)
    mlens = lens[rows]
    m = binding.KvMigration(mlens, rows, w.page_size)
    n = m.num_pages
    shape = (n, w.num_kv_heads, w.page_size, w.head_dim)
    k_stage = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
    v_stage = torch.empty_like(k_stage)
    pool_pages = int(np.ceil(1.15 * n))
    perm = wl.CounterRng(w.seed + 55).permutation(pool_pages)[:n]
    need = wl.pages_needed(mlens, w.page_size)
    tt = np.full((len(rows), int(need.max())), -1, dtype=np.int32)
    off = np.concatenate([[0], np.cumsum(need)])
    for r in range(len(rows)):
        tt[r, : need[r]] = perm[off[r]: off[r + 1]]
    tt_dev = torch.from_numpy(tt).cuda()
    k_dst = torch.empty((pool_pages,) + shape[1:], dtype=torch.bfloat16, device="cuda")
    v_dst = torch.empty_like(k_dst)
    payload = 2 * n * w.num_kv_heads * w.page_size * w.head_dim * 2     # K and V bytes of the chunk

    def step(i=0):
        m.gather(inp.k_pages, inp.v_pages, inp.block_table, 0, w.num_kv_heads, k_stage, v_stage)
        m.scatter(k_stage, v_stage, tt_dev, 0, k_dst, v_dst)

    for _ in range(args.warmup):
        step()
    unsettled_ms, _ = timed_block(step, args.steps, torch)
    settle_s, settle_steps = settle(step, torch, args.settle_seconds)
    m.enable_timing(True)
    ms_per_step, _ = timed_block(step, args.steps, torch)
    kernel_ms, cnt = m.kernel_ms()
    m.enable_timing(False)
    moved = 2 * payload                                    # every byte is read once and written once
    value = 2 * moved / (ms_per_step * 1e-3) / 1e9         # two copies per step
    achieved = moved / (kernel_ms * 1e-3) / 1e9
    res = {"metric": "KV-block migration copy GB/s (bytes read + written)", "value": round(value, 1), "unit": "GB/s",
           "value_unsettled": round(2 * moved / (unsettled_ms * 1e-3) / 1e9, 1)}
    res.update(common_fields(args, ms_per_step, args.warmup + args.steps + settle_steps))
    res.update({
        "dtype": "u8",
        "config": {"workload": f"the {len(rows)} long requests of cfg3 ({int(mlens.sum())} tokens, {n} pages, "
                               f"{payload / 1e9:.3f} GB of K+V per layer chunk): gather to staging + scatter to a target pool",
                   "settle_s": round(settle_s, 2), "settle_steps": settle_steps},
        "roofline": {"bound": "hbm", "kernel": "kv_migrate_kernel", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                     "avg_kernel_ms": round(kernel_ms, 5), "launches_timed": cnt,
                     "algorithmic_bytes_per_launch": moved}})
    return res


def bench_mixed(args, torch, binding, wl):
    """One step = oserve_mixed_plan_update + oserve_paged_mixed_attn on a batch that holds decode requests and
    prefill chunks, against the same work done by the decode call followed by the prefill call."""
    w, lens, qlens = wl.mixed_workload()
    inp = wl.make_inputs(w, device="cuda", seed=w.seed, lens=lens)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed + 1)
    q = torch.randn(int(qlens.sum()), w.num_q_heads, w.head_dim, generator=gen, device="cuda").to(torch.bfloat16)
    out = torch.empty(q.shape, dtype=torch.float32, device="cuda")
    width = inp.block_table.shape[1]
    geo = (w.num_q_heads, w.num_kv_heads, w.head_dim, w.page_size, width)
    plan = binding.MixedPlan(lens, qlens, *geo, 0)
    ws = torch.empty(plan.workspace_bytes_max, dtype=torch.uint8, device="cuda")
    # the same work through the two separate calls: decode requests first in the batch, chunks after them
    nd = int((qlens == 1).sum())
    assert (qlens[:nd] == 1).all() and (qlens[nd:] > 1).all()
    dplan = binding.Plan(lens[:nd], *geo, 0, 0)
    dws = torch.empty(dplan.workspace_bytes_max, dtype=torch.uint8, device="cuda")
    pplan = binding.PrefillPlan(lens[nd:], qlens[nd:], *geo, 0)
    out2 = torch.empty_like(out)
    bt_d, bt_p = inp.block_table[:nd].contiguous(), inp.block_table[nd:].contiguous()
    cl_d = inp.context_lens[:nd].contiguous()
    q_d, q_p, o_d, o_p = q[:nd], q[nd:], out2[:nd], out2[nd:]

    def mixed(i=0):
        plan.update(lens, qlens)
        binding.paged_mixed_attn(plan, ws, q, inp.k_pages, inp.v_pages, inp.block_table, inp.context_lens, w.scale, out)

    def decode_only(i=0):
        dplan.update(lens[:nd])
        binding.paged_decode_attn(dplan, dws, q_d, inp.k_pages, inp.v_pages, bt_d, cl_d, w.scale, o_d)

    def prefill_only(i=0):
        pplan.update(lens[nd:], qlens[nd:])
        binding.paged_prefill_attn(pplan, q_p, inp.k_pages, inp.v_pages, bt_p, w.scale, o_p)

    def separate(i=0):
        decode_only()
        prefill_only()

    for _ in range(args.warmup):
        mixed()
        separate()
    torch.cuda.synchronize()
    same = bool(torch.equal(out, out2))
    unsettled_ms, _ = timed_block(mixed, args.steps, torch)
    settle_s, settle_steps = settle(mixed, torch, args.settle_seconds)
    # alternate blocks of the two ways so that both see the same state of the part
    t = {"mixed": [], "separate": [], "decode": [], "prefill": []}
    for _ in range(3):
        t["mixed"].append(timed_block(mixed, args.steps, torch)[0])
        t["separate"].append(timed_block(separate, args.steps, torch)[0])
        t["decode"].append(timed_block(decode_only, args.steps, torch)[0])
        t["prefill"].append(timed_block(prefill_only, args.steps, torch)[0])
    ms = {k: min(v) for k, v in t.items()}
    plan.enable_timing(True)
    timed_block(mixed, args.steps, torch)
    kernel_ms, cnt = plan.kernel_ms()
    plan.enable_timing(False)
    kv_bytes = wl.kv_bytes(lens[:nd], w.num_kv_heads, w.head_dim)
    pairs = sum(int(n) * (int(L) - int(n)) + int(n) * (int(n) + 1) // 2 for L, n in zip(lens[nd:], qlens[nd:]))
    flop = 4.0 * w.head_dim * w.num_q_heads * pairs
    res = {"metric": "mixed prefill+decode step: time of the decode call + the prefill call over time of the one mixed call",
           "value": round(ms["separate"] / ms["mixed"], 4), "unit": "x",
           "value_unsettled": round(ms["separate"] / unsettled_ms, 4)}
    res.update(common_fields(args, ms["mixed"], 2 * args.warmup + args.steps + settle_steps))
    res.update({
        "dtype": "bf16",
        "config": {"workload": f"mixed: the {nd} decode requests of cfg3 ({kv_bytes / 1e9:.3f} GB of K+V) + {len(lens) - nd} "
                               f"prefill chunks of 512 tokens ending contexts in [2048, 16384] ({flop / 1e12:.3f} TFLOP); "
                               f"32q/8kv heads, head_dim 128, page 16",
                   "counts": plan.counts, "ms_mixed": round(ms["mixed"], 5), "ms_decode_then_prefill": round(ms["separate"], 5),
                   "ms_decode_alone": round(ms["decode"], 5), "ms_prefill_alone": round(ms["prefill"], 5),
                   "mixed_output_equals_separate_calls_bitwise": same,
                   "settle_s": round(settle_s, 2), "settle_steps": settle_steps},
        "roofline": {"bound": "hbm", "kernel": "paged_mixed_kernel", "achieved": round(kv_bytes / (kernel_ms * 1e-3) / 1e9, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(kv_bytes / (kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "traffic": None, "avg_kernel_ms": round(kernel_ms, 5), "launches_timed": cnt,
                     "algorithmic_bytes_per_launch": kv_bytes,
                     "also": {"bound": "mfma", "achieved": round(flop / (kernel_ms * 1e-3) / 1e12, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                              "unit": "TFLOP/s", "frac": round(flop / (kernel_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                              "algorithmic_flop_per_launch": flop,
                              "note": "the decode requests' K/V bytes and the prefill chunks' flop, both over the one kernel's time"}}})
    return res


def sources_sha16():
    """Hash of the sources that decide the split kernel's memory traffic (kernel, planner)."""
    import hashlib
    h = hashlib.sha256()
    root = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2602_12151_amd", "csrc")
    for name in ("kernels.hip", "decode_body.h", "kernels.h", "plan.cpp", "plan.h"):
        with open(os.path.join(root, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def bench_decode(args, torch, binding, wl, config, with_cpu):
    """One step = host re-plan + expand + split + merge kernels of workload `config` on inputs resident in HBM."""
    w = wl.WORKLOADS[config]
    sets, nbytes = build_inputs(w, wl, torch)
    ops = [binding.DecodeAttention(s, split_tokens=args.split_tokens) for s in sets]
    plan0 = ops[0].plan

    def step(i):
        j = i % len(sets)
        ops[j].step(sets[j], replan=True)

    # The contract's W warm-up steps and a first timed block of K steps (reported as value_unsettled), then the
    # settling phase, then the K timed steps `value` is computed from.
    for i in range(args.warmup):
        step(i)
    unsettled_ms, _ = timed_block(step, args.steps, torch)
    settle_s, settle_steps = settle(step, torch, args.settle_seconds)
    for op in ops:
        op.plan.enable_timing(True)
    ms_per_step, gpu_ms_per_step = timed_block(step, args.steps, torch)
    tot, cnt = 0.0, 0
    for op in ops:
        ms, n = op.plan.split_kernel_ms()
        tot += ms * n
        cnt += n
        op.plan.enable_timing(False)
    split_ms = tot / max(cnt, 1)

    # distribution of single steps (events between the steps; not what `value` is computed from)
    n_single = min(args.steps, 50)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_single + 1)]
    evs[0].record()
    for i in range(n_single):
        step(i)
        evs[i + 1].record()
    torch.cuda.synchronize()
    singles = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(n_single))
    # one layer of a model whose layers share the step's plan: descriptors staged once, then split + merge only
    for j, op in enumerate(ops):
        op.stage(sets[j])
    layer_ms, _ = timed_block(lambda i: ops[i % len(sets)].layer(sets[i % len(sets)]), args.steps, torch)
    # the host re-plan alone
    lens_host = sets[0].context_lens_host
    n_plan = 200
    t0 = time.perf_counter()
    for _ in range(n_plan):
        plan0.update(lens_host)
    plan_us = (time.perf_counter() - t0) / n_plan * 1e6
    prop = torch.cuda.get_device_properties(0)

    value = nbytes / (ms_per_step * 1e-3) / 1e9
    achieved = nbytes / (split_ms * 1e-3) / 1e9
    traffic, traffic_note = None, "not profiled for this workload"
    if config == RECORDED_TRAFFIC["config"] and args.split_tokens == 0:
        if sources_sha16() == RECORDED_TRAFFIC["sources_sha16"] and plan0.num_work_items == RECORDED_TRAFFIC["work_items"]:
            traffic, traffic_note = RECORDED_TRAFFIC["bytes"], "recorded rocprofv3 value of " + RECORDED_TRAFFIC["profile"]
        else:
            traffic_note = "kernel or planner sources changed since " + RECORDED_TRAFFIC["profile"] + " was taken"
    result = {"metric": "decode-attn effective KV GB/s (% of HBM peak) + us/step, mixed-length batch",
              "value": round(value, 1), "unit": "GB/s",
              "value_unsettled": round(nbytes / (unsettled_ms * 1e-3) / 1e9, 1)}
    result.update(common_fields(args, ms_per_step, args.warmup + args.steps + settle_steps))
    result.update({
        "us_per_step": round(ms_per_step * 1e3, 2),
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "dtype": "bf16",
        "config": {"workload": f"cfg{w.index} {w.name}: batch {w.batch}, {w.num_q_heads}q/{w.num_kv_heads}kv heads, "
                               f"head_dim {w.head_dim}, page {w.page_size}, {int(sets[0].context_lens_host.sum())} tokens, "
                               f"{nbytes / 1e9:.3f} GB K+V per step",
                   "work_items": plan0.num_work_items, "split_tokens": plan0.split_tokens,
                   "settle_s": round(settle_s, 2), "settle_steps": settle_steps,
                   "input_copies_rotated": len(sets), "gpu_event_ms_per_step": round(gpu_ms_per_step, 5),
                   "single_step_us_median": round(singles[len(singles) // 2] * 1e3, 2),
                   "single_step_us_min": round(singles[0] * 1e3, 2),
                   "us_per_layer_plan_staged_once": round(layer_ms * 1e3, 2),
                   "pct_hbm_peak_per_layer_plan_staged_once": round(100.0 * nbytes / (layer_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 2),
                   "host_plan_update_us": round(plan_us, 2),
                   "device": f"{prop.name}, {prop.multi_processor_count} CUs, "
                             f"{prop.total_memory / 2**30:.0f} GiB"},
        "roofline": {"bound": "hbm", "kernel": "paged_decode_split_kernel", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "traffic_note": traffic_note,
                     "avg_kernel_ms": round(split_ms, 5), "launches_timed": cnt,
                     "algorithmic_bytes_per_launch": nbytes}})
    if with_cpu:
        # the output the last timed step of input set 0 left behind, against what the oracle computes below
        step(0)
        torch.cuda.synchronize()
        result["cpu_baseline"], result["parity"] = cpu_baseline(sets[0], wl, torch, args.cpu_token_heads, ops[0].out)
    return result


def brief(res):
    """The figures of a side measurement that go under the headline's `extra` key."""
    r = res["roofline"]
    out = {"value": res["value"], "unit": res["unit"], "value_unsettled": res["value_unsettled"],
           "us_per_step": round(res["ms_per_step"] * 1e3, 2), "workload": res["config"]["workload"],
           "kernel": r["kernel"], "kernel_achieved": r["achieved"], "kernel_frac_of_peak": r["frac"], "bound": r["bound"]}
    if res["unit"] == "GB/s" and r["bound"] == "hbm":
        out["pct_hbm_peak"] = round(100.0 * res["value"] / HBM_PEAK_GBS, 2)
    for k in ("single_step_us_median", "us_per_layer_plan_staged_once", "pct_hbm_peak_per_layer_plan_staged_once", "ms_mixed", "ms_decode_then_prefill", "ms_decode_alone", "ms_prefill_alone",
              "mixed_output_equals_separate_calls_bitwise"):
        if k in res["config"]:
            out[k] = res["config"][k]
    if "also" in r:
        out["also"] = {k: r["also"][k] for k in ("bound", "achieved", "unit", "frac")}
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (nothing here is sharded across GPUs); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import gc
    import torch
    from paper_2602_12151_amd import binding, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.copy_probe:
        src = torch.empty(args.copy_probe, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes": args.copy_probe, "launches": args.steps}))
        return
    if args.prefill >= 0:
        print(json.dumps(bench_prefill(args, torch, binding, wl, args.prefill)))
        return
    if args.migrate:
        print(json.dumps(bench_migrate(args, torch, binding, wl)))
        return
    if args.mixed:
        print(json.dumps(bench_mixed(args, torch, binding, wl)))
        return
    result = bench_decode(args, torch, binding, wl, args.config, not args.no_cpu_baseline)
    if args.extra and args.config == 3 and args.split_tokens == 0:
        # Side measurements, shorter (their own settling cap): the other benchmark configs, the chunked-prefill
        # kernel and the migration copies.  The headline fields above are not touched by them.
        side = argparse.Namespace(**vars(args))
        side.settle_seconds = min(args.settle_seconds, args.extra_settle_seconds)
        extra = {}
        t_extra = time.perf_counter()

        def run(name, fn):
            gc.collect()
            torch.cuda.empty_cache()
            try:
                extra[name] = brief(fn())
            except Exception as e:                 # a side measurement never costs the headline
                extra[name] = {"error": f"{type(e).__name__}: {e}"}
            print(f"bench.py: extra {name} done at {time.perf_counter() - t_extra:.1f} s", file=sys.stderr, flush=True)

        for c in (0, 1, 2, 4):
            run(f"cfg{c}", lambda c=c: bench_decode(side, torch, binding, wl, c, False))
        for which in (0, 1, 2):
            run(f"prefill{which}", lambda which=which: bench_prefill(side, torch, binding, wl, which))
        run("kv_migration", lambda: bench_migrate(side, torch, binding, wl))
        run("mixed", lambda: bench_mixed(side, torch, binding, wl))
        result["extra"] = extra
    print(json.dumps(result))


if __name__ == "__main__":
    main()
