"""GPU-vs-oracle parity of the HIP path, called through the C ABI.

Bar: max-abs error <= 1e-2 and relative L2 error <= 2e-3 against the fp64
oracle on the same seeded bits (bf16 inputs, fp32 accumulation); bit-exact
where the mathematics says the GPU result cannot change (page permutation,
run-to-run).
"""
import numpy as np
import pytest
import torch

from paper_2602_12151_amd import workloads as wl
from tests import gpu_helpers as gh

pytestmark = pytest.mark.gpu


def _case(widx, lens, seed=None, **kw):
    w = wl.WORKLOADS[widx]
    cpu = wl.make_inputs(w, device="cpu", seed=seed, lens=np.asarray(lens, dtype=np.int32), **kw)
    return cpu, gh.to_device(cpu)


def test_tiny_workload_full():
    """Workload 0 exactly: lens 17/64/200/513, 8q/2kv, D=64, 64-page permuted pool."""
    cpu = wl.make_inputs(wl.WORKLOADS[0], device="cpu")
    dev = gh.to_device(cpu)
    out, op = gh.gpu_attention(dev)
    print("tiny:", gh.assert_parity(out, gh.oracle_attention(cpu), "tiny"), "items", op.plan.num_work_items)


@pytest.mark.parametrize("split_tokens", [0, 16, 32, 64, 256])
def test_tiny_workload_all_split_sizes(split_tokens):
    cpu = wl.make_inputs(wl.WORKLOADS[0], device="cpu")
    dev = gh.to_device(cpu)
    out, _ = gh.gpu_attention(dev, split_tokens=split_tokens)
    gh.assert_parity(out, gh.oracle_attention(cpu), f"tiny split={split_tokens}")


@pytest.mark.parametrize("widx", [1, 2, 3])
def test_boundary_lengths(widx):
    """Context lengths at page and split boundaries, D=128, group 4 and 8."""
    lens = [1, 2, 15, 16, 17, 31, 32, 33, 127, 128, 129, 255, 256, 257, 1000, 1023, 1024, 1025, 48, 3]
    cpu, dev = _case(widx, lens, seed=100 + widx)
    ref = gh.oracle_attention(cpu)
    for split_tokens in (0, 16, 48, 128, 1024):
        out, _ = gh.gpu_attention(dev, split_tokens=split_tokens)
        gh.assert_parity(out, ref, f"w{widx} split={split_tokens}")


def test_llama8b_workload_full_size_full_compare():
    """Workload 1 at full size (batch 64, lens U[128, 2048]); the oracle does all of it in seconds."""
    cpu = wl.make_inputs(wl.WORKLOADS[1], device="cpu")
    dev = gh.to_device(cpu)
    out, op = gh.gpu_attention(dev)
    e = gh.assert_parity(out, gh.oracle_attention(cpu), "w1")
    print("w1:", e, "items", op.plan.num_work_items, "split pages", op.plan.split_pages)


def test_single_split_path_writes_out_directly():
    """split_tokens larger than every context: no request is split, the merge kernel is not launched."""
    lens = [5, 300, 77, 1024]
    cpu, dev = _case(1, lens, seed=7)
    out, op = gh.gpu_attention(dev, split_tokens=2048)
    assert op.plan.num_work_items == len(lens) * 8
    gh.assert_parity(out, gh.oracle_attention(cpu), "single split")


def test_mha_and_group_sizes():
    """Group sizes 1 (MHA), 2, 8, 16 at D=128 and 64."""
    for hq, hkv, d in [(4, 4, 128), (8, 4, 128), (16, 2, 128), (16, 1, 128), (4, 4, 64), (16, 1, 64)]:
        w = wl.Workload(9, "shape", batch=3, num_q_heads=hq, num_kv_heads=hkv, head_dim=d)
        cpu = wl.make_inputs(w, device="cpu", seed=hq * 100 + hkv, lens=np.array([33, 700, 129], dtype=np.int32))
        dev = gh.to_device(cpu)
        out, _ = gh.gpu_attention(dev, split_tokens=128)
        gh.assert_parity(out, gh.oracle_attention(cpu), f"hq={hq} hkv={hkv} d={d}")


@pytest.mark.parametrize("page_size", [32, 64])
@pytest.mark.parametrize("hq,hkv,d", [(32, 8, 128), (8, 2, 64), (7, 7, 128)])
def test_page_sizes_32_and_64(page_size, hq, hkv, d):
    """Pages of 2 and 4 key tiles: lengths around tile and page boundaries, splits that start inside a
    page, NaN in every dead slot of the last pages."""
    lens = np.array([1, 16, 17, 31, 33, 63, 64, 65, 127, 129, 700, 1291, 4000], dtype=np.int32)
    w = wl.Workload(9, "pages", batch=len(lens), num_q_heads=hq, num_kv_heads=hkv, head_dim=d, page_size=page_size)
    cpu = wl.make_inputs(w, device="cpu", seed=page_size + hq, lens=lens)
    bt = cpu.block_table.numpy()
    for b, L in enumerate(lens):
        if L % page_size:
            last = int(bt[b, (L - 1) // page_size])
            cpu.k_pages[last, :, L % page_size:, :] = float("nan")
            cpu.v_pages[last, :, L % page_size:, :] = float("nan")
    dev = gh.to_device(cpu)
    ref = gh.oracle_attention(cpu)
    for split_tokens in (0, page_size, 3 * page_size, 1024):
        out, _ = gh.gpu_attention(dev, split_tokens=split_tokens)
        gh.assert_parity(out, ref, f"page={page_size} hq={hq} hkv={hkv} d={d} split={split_tokens}")


@pytest.mark.parametrize("name,hq,hkv", [("OPT-30B (MHA, 56 heads) TP=2", 28, 28), ("OPT-66B (MHA, 72 heads) TP=4", 18, 18),
                                         ("Llama-30B (MHA, 52 heads) TP=4", 13, 13), ("Llama2-70B TP=2", 32, 4),
                                         ("Llama2-70B TP=8", 8, 1), ("Llama2-70B TP=1", 64, 8),
                                         ("Llama2-70B TP=3, GPU holding 3 of the 8 kv heads", 24, 3),
                                         ("Llama2-70B TP=3, GPU holding 2 of the 8 kv heads", 16, 2),
                                         ("OPT-30B (56 heads) TP=3, GPU holding 19 heads", 19, 19)])
def test_head_geometries_of_the_papers_models(name, hq, hkv):
    """Per-GPU head counts of the models of section 6.1 at tensor-parallel degrees its deployments use
    (all head_dim 128), on a small mixed-length batch."""
    lens = np.array([40, 2100, 517, 9000, 16, 1300], dtype=np.int32)
    w = wl.Workload(9, name, batch=len(lens), num_q_heads=hq, num_kv_heads=hkv, head_dim=128)
    cpu = wl.make_inputs(w, device="cpu", seed=hq * 7 + hkv, lens=lens)
    dev = gh.to_device(cpu)
    out, _ = gh.gpu_attention(dev)
    gh.assert_parity(out, gh.oracle_attention(cpu), name)


def test_unread_memory_is_poisoned_with_nan():
    """NaN in tail slots of last pages and in every page no table row names must not reach the output."""
    lens = [1, 15, 17, 100, 513, 1030]
    cpu, dev = _case(3, lens, seed=11)
    clean, _ = gh.gpu_attention(dev, split_tokens=64)
    pk, pv = dev.k_pages.clone(), dev.v_pages.clone()
    used = torch.zeros(pk.shape[0], dtype=torch.bool, device="cuda")
    used[torch.from_numpy(cpu.used_pages).cuda()] = True
    pk[~used] = float("nan")
    pv[~used] = float("nan")
    bt = cpu.block_table.numpy()
    for b, L in enumerate(lens):
        if L % 16:
            last = int(bt[b, (L - 1) // 16])
            pk[last, :, L % 16:, :] = float("nan")
            pv[last, :, L % 16:, :] = float("nan")
    poisoned = wl.Inputs(workload=dev.workload, q=dev.q, k_pages=pk, v_pages=pv, block_table=dev.block_table,
                         context_lens=dev.context_lens, context_lens_host=dev.context_lens_host,
                         scale=dev.scale, used_pages=dev.used_pages)
    out, _ = gh.gpu_attention(poisoned, split_tokens=64)
    assert torch.equal(out, clean)
    gh.assert_parity(out, gh.oracle_attention(cpu), "poisoned")


def test_page_permutation_and_reruns_are_bit_identical():
    lens = [700, 33, 2000, 16]
    w = wl.WORKLOADS[1]
    a_cpu = wl.make_inputs(w, device="cpu", seed=21, lens=np.asarray(lens, dtype=np.int32))
    a = gh.to_device(a_cpu)
    out_a, op = gh.gpu_attention(a, split_tokens=256)
    again = op.step(a).clone()
    torch.cuda.synchronize()
    assert torch.equal(out_a, again)
    # move every used page to another physical slot, consistently with the table
    npool = a.k_pages.shape[0]
    perm = torch.from_numpy(wl.CounterRng(5).permutation(npool)).cuda()      # new_id = perm[old_id]
    k2 = torch.empty_like(a.k_pages)
    v2 = torch.empty_like(a.v_pages)
    k2[perm] = a.k_pages
    v2[perm] = a.v_pages
    bt2 = a.block_table.clone()
    mask = bt2 >= 0
    bt2[mask] = perm[bt2[mask].long()].int()
    b = wl.Inputs(workload=w, q=a.q, k_pages=k2, v_pages=v2, block_table=bt2, context_lens=a.context_lens,
                  context_lens_host=a.context_lens_host, scale=a.scale, used_pages=None)
    out_b, _ = gh.gpu_attention(b, split_tokens=256)
    assert torch.equal(out_a, out_b)


def test_large_scores_do_not_overflow():
    """|score| up to ~100: the running-max subtraction must be in place."""
    lens = [300, 40]
    cpu, dev = _case(1, lens, seed=31)
    cpu.q.mul_(6.0)
    cpu.k_pages.mul_(1.5)
    dev = gh.to_device(cpu)
    ref = gh.oracle_attention(cpu)
    out, _ = gh.gpu_attention(dev, split_tokens=64)
    gh.assert_parity(out, ref, "large scores")


def test_page_ids_beyond_4gib_offsets():
    """Physical page ids >= 2^17 put byte offsets past 4 GiB (32 KiB per page): needs 64-bit addressing."""
    w = wl.WORKLOADS[1]
    lens = np.array([600, 50, 1500], dtype=np.int32)
    npool = (1 << 17) + 4096
    dev = wl.make_inputs(w, device="cuda", seed=41, lens=lens, fill_unused=False, pool_pages_override=npool)
    assert int(dev.block_table.max()) >= (1 << 17)
    out, _ = gh.gpu_attention(dev, split_tokens=128)
    pairs = [(b, h) for b in range(3) for h in (0, 13, 31)]
    ref = gh.sampled_oracle_rows(dev, pairs)
    got = torch.stack([out[b, h] for b, h in pairs])
    gh.assert_parity(got, ref, "big ids")


def test_plan_update_between_steps():
    """One plan object re-planned for a different batch (the per-step serving loop)."""
    from paper_2602_12151_amd import binding
    w = wl.WORKLOADS[1]
    a_cpu = wl.make_inputs(w, device="cpu", seed=51, lens=np.array([100, 900, 17, 2048], dtype=np.int32))
    b_cpu = wl.make_inputs(w, device="cpu", seed=52, lens=np.array([2000, 31], dtype=np.int32))
    a, b = gh.to_device(a_cpu), gh.to_device(b_cpu)
    width = max(a.block_table.shape[1], b.block_table.shape[1])

    def widen(x):
        bt = torch.full((x.block_table.shape[0], width), -1, dtype=torch.int32, device="cuda")
        bt[:, : x.block_table.shape[1]] = x.block_table
        x.block_table = bt
        return x
    a, b = widen(a), widen(b)
    plan = binding.Plan(a.context_lens_host, 32, 8, 128, 16, width, 0, 0, capacity=4)
    ws = torch.empty(plan.workspace_bytes_max, dtype=torch.uint8, device="cuda")
    for inp, cpu in ((a, a_cpu), (b, b_cpu), (a, a_cpu)):
        plan.update(inp.context_lens_host)
        assert plan.workspace_bytes <= plan.workspace_bytes_max
        out = torch.empty(inp.q.shape, dtype=torch.float32, device="cuda")
        binding.paged_decode_attn(plan, ws, inp.q, inp.k_pages, inp.v_pages, inp.block_table,
                                  inp.context_lens, inp.scale, out)
        torch.cuda.synchronize()
        gh.assert_parity(out, gh.oracle_attention(cpu), "update")
    with pytest.raises(binding.OserveError):
        plan.update(np.ones(5, dtype=np.int32))        # beyond capacity


def test_many_launches_wrap_the_staging_ring():
    cpu, dev = _case(1, [300, 1200, 64], seed=61)
    from paper_2602_12151_amd import binding
    op = binding.DecodeAttention(dev, split_tokens=128)
    first = op.step(dev).clone()
    for _ in range(3 * binding.PLAN_RING):
        out = op.step(dev)
    torch.cuda.synchronize()
    assert torch.equal(out, first)
    gh.assert_parity(out, gh.oracle_attention(cpu), "ring")


def test_layers_over_one_staged_plan():
    """The descriptors staged once serve every layer of a step: two "layers" (different q, K/V pools and page
    placement over the same lengths) through oserve_paged_decode_attn_staged equal the ordinary call bit for bit
    and the oracle within the bar; a stale stage is refused."""
    from paper_2602_12151_amd import binding
    lens = np.array([300, 5000, 64, 1, 2047, 17], dtype=np.int32)
    w = wl.WORKLOADS[1]
    cpus = [wl.make_inputs(w, device="cpu", seed=70 + layer, lens=lens) for layer in range(2)]
    devs = [gh.to_device(c) for c in cpus]
    op = binding.DecodeAttention(devs[0])
    assert op.plan.num_work_items > len(lens) * w.num_kv_heads        # some request is split
    plain = [op.step(d, replan=False).clone() for d in devs]
    torch.cuda.synchronize()
    op.stage(devs[0])
    for _ in range(3):                                                 # the stage survives many layers
        for layer, d in enumerate(devs):
            out = op.layer(d)
            torch.cuda.synchronize()
            assert torch.equal(out, plain[layer]), layer
    for layer, c in enumerate(cpus):
        gh.assert_parity(plain[layer], gh.oracle_attention(c), f"layer {layer}")
    # a different workspace, an updated plan, or the ordinary call on the same workspace: staged no longer
    other = torch.empty_like(op.workspace)
    with pytest.raises(binding.OserveError) as e:
        binding.paged_decode_attn_staged(op.plan, other, devs[0].q, devs[0].k_pages, devs[0].v_pages,
                                         devs[0].block_table, devs[0].context_lens, devs[0].scale, op.out)
    assert e.value.status == binding.ERR_PLAN_MISMATCH
    op.plan.update(devs[0].context_lens_host)
    with pytest.raises(binding.OserveError):
        op.layer(devs[0])
    op.stage(devs[0], replan=False)
    assert torch.equal(op.layer(devs[1]), plain[1])
    op.step(devs[0], replan=False)
    with pytest.raises(binding.OserveError):
        op.layer(devs[0])
    torch.cuda.synchronize()


def test_staged_layers_in_a_hip_graph():
    """The staged call enqueues kernels only (no copy, no event, no wait), so a serving loop can capture the layers
    of a step into a HIP graph: every replay, with eager work in between, gives the eager result bit for bit."""
    from paper_2602_12151_amd import binding
    lens = np.array([700, 33, 4000, 1, 129], dtype=np.int32)
    w = wl.WORKLOADS[1]
    devs = [gh.to_device(wl.make_inputs(w, device="cpu", seed=80 + layer, lens=lens)) for layer in range(2)]
    op = binding.DecodeAttention(devs[0])
    eager = [op.step(d, replan=False).clone() for d in devs]
    outs = [torch.empty_like(eager[0]) for _ in devs]
    op.stage(devs[0], replan=False)
    torch.cuda.synchronize()

    def layers():
        for _ in range(2):
            for d, o in zip(devs, outs):
                binding.paged_decode_attn_staged(op.plan, op.workspace, d.q, d.k_pages, d.v_pages, d.block_table,
                                                 d.context_lens, d.scale, o)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    import gc
    gc.collect()
    gc.disable()            # a plan object finalised during the capture would free pinned memory, which a capture forbids
    try:
        with torch.cuda.graph(graph, stream=side):
            layers()
    finally:
        gc.enable()
    for replay in range(4):
        for o in outs:
            o.fill_(float("nan"))                       # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for layer in range(2):
            assert torch.equal(outs[layer], eager[layer]), (replay, layer)
    layers()                                            # and the plan still launches eagerly afterwards
    torch.cuda.synchronize()
    assert torch.equal(outs[1], eager[1])


# ----------------------------------------------------------------------------
# full-size workloads in the launch configuration bench.py times (automatic plan): every element of
# `out` against the oracle (the oracle needs a few seconds per workload)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("widx", [2, 3, 4])
def test_full_size_workloads_whole_tensor(widx):
    w = wl.WORKLOADS[widx]
    print(f"workload {widx}: generating inputs", flush=True)
    dev = wl.make_inputs(w, device="cuda", fill_unused=w.pool_pages_fixed is None)
    out, op = gh.gpu_attention(dev)
    print(f"workload {widx}: GPU done ({op.plan.num_work_items} items, {op.plan.num_runs} runs), oracle on "
          f"{w.batch} requests", flush=True)
    ref = gh.oracle_whole_batch(dev, progress=max(1, w.batch // 4))
    err = gh.assert_parity(out, ref, f"workload {widx}, whole tensor")
    g = out.cpu().double().numpy()
    # worst single (request, head) row, relative: long contexts make max-abs slack, so rel-L2 per row binds
    per_row = np.linalg.norm(g - ref, axis=2) / np.linalg.norm(ref, axis=2)
    assert per_row.max() <= gh.REL_L2_TOL, per_row.max()
    # every run of the plan (every split size of the ladder) has been compared: all requests were
    runs = [op.plan.run(i) for i in range(op.plan.num_runs)]
    assert {r["request"] for r in runs} == set(range(w.batch))
    print(f"workload {widx}: {g.size} elements, split tiles {op.plan.split_pages}, "
          f"split sizes {sorted({r['pages_per_split'] for r in runs}, reverse=True)[:8]}, "
          f"max_abs {err[0]:.2e}, rel_l2 {err[1]:.2e}, worst row rel_l2 {per_row.max():.2e}")
    # a property that holds at any size: an output row is a convex combination of its kv head's V rows
    b = int(np.argmax(dev.context_lens_host))
    L = int(dev.context_lens_host[b])
    ids = dev.block_table[b, : (L + 15) // 16].long()
    for h in (0, w.num_q_heads - 1):
        v = dev.v_pages[ids, h // w.group].reshape(-1, w.head_dim)[:L].float()
        assert (out[b, h] <= v.max(dim=0).values + 1e-3).all() and (out[b, h] >= v.min(dim=0).values - 1e-3).all()


def test_rerun_bit_identical_at_full_size():
    w = wl.WORKLOADS[3]
    dev = wl.make_inputs(w, device="cuda")
    out, op = gh.gpu_attention(dev)
    again = op.step(dev).clone()
    torch.cuda.synchronize()
    assert torch.equal(out, again)


def test_one_request_of_a_million_tokens():
    """Batch 1, 1,048,583 tokens (65,537 pages, ragged last page): the largest context the planner's bounds are
    sized for, compared on sampled heads; every other batch shape splits less."""
    L = (1 << 20) + 7
    w = wl.Workload(11, "one very long request", batch=1, num_q_heads=32, num_kv_heads=8, head_dim=128)
    dev = wl.make_inputs(w, device="cuda", seed=11, lens=np.array([L], dtype=np.int32))
    out, op = gh.gpu_attention(dev)
    assert torch.isfinite(out).all()
    pairs = [(0, 0), (0, 13), (0, 31)]
    ref = gh.sampled_oracle_rows(dev, pairs)
    got = torch.stack([out[b, h] for b, h in pairs])
    err = gh.assert_parity(got, ref, "one request of 2^20 + 7 tokens")
    print(f"2^20+7 tokens: items {op.plan.num_work_items}, split pages {op.plan.split_pages}, "
          f"max_abs {err[0]:.2e}, rel_l2 {err[1]:.2e}")
