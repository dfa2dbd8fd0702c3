"""GPU-vs-oracle parity of the mixed prefill + decode batch (oserve_paged_mixed_attn), through the C ABI.

The oracle is the causal chunked-prefill form of paged attention, of which a decode request is the case of
one query token.  Same bar as everywhere: max-abs error <= 1e-2 and relative L2 error <= 2e-3.
"""
import numpy as np
import pytest
import torch

from oracle import paged_attention_oracle as oracle
from paper_2602_12151_amd import binding, workloads as wl
from tests import gpu_helpers as gh

pytestmark = pytest.mark.gpu


def make_case(lens, qlens, hq=32, hkv=8, page_size=16, seed=0, poison=False, head_dim=128):
    lens = np.asarray(lens, dtype=np.int32)
    qlens = np.asarray(qlens, dtype=np.int32)
    w = wl.Workload(9, "mixed", batch=len(lens), num_q_heads=hq, num_kv_heads=hkv, head_dim=head_dim, page_size=page_size)
    cpu = wl.make_inputs(w, device="cpu", seed=seed, lens=lens)
    g = torch.Generator().manual_seed(seed + 4242)
    q = torch.randn(int(qlens.sum()), hq, head_dim, generator=g).to(torch.bfloat16)
    if poison:   # NaN in every slot past a request's context, and in every page no request owns
        used = np.zeros(cpu.k_pages.shape[0], dtype=bool)
        used[cpu.used_pages] = True
        cpu.k_pages[~torch.from_numpy(used)] = float("nan")
        cpu.v_pages[~torch.from_numpy(used)] = float("nan")
        bt = cpu.block_table.numpy()
        for b, L in enumerate(lens):
            if L % page_size:
                last = int(bt[b, (L - 1) // page_size])
                cpu.k_pages[last, :, L % page_size:, :] = float("nan")
                cpu.v_pages[last, :, L % page_size:, :] = float("nan")
    return w, cpu, q, lens, qlens


def run_gpu(w, cpu, q, lens, qlens, plan=None):
    if plan is None:
        plan = binding.MixedPlan(lens, qlens, w.num_q_heads, w.num_kv_heads, w.head_dim, w.page_size,
                                 cpu.block_table.shape[1], 0)
    ws = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device="cuda")
    out = torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda")
    binding.paged_mixed_attn(plan, ws, q.cuda(), cpu.k_pages.cuda(), cpu.v_pages.cuda(), cpu.block_table.cuda(),
                             cpu.context_lens.cuda(), w.scale, out)
    torch.cuda.synchronize()
    return out, plan


def reference(w, cpu, q, lens, qlens):
    return oracle.paged_prefill_attn(q, cpu.k_pages, cpu.v_pages, cpu.block_table.numpy(), lens, qlens, w.scale)


def check_rows(out, ref, qlens, what):
    """Whole tensor, and the decode rows and the prefill rows each on their own (they take different kernels'
    paths, and the decode rows' errors are far smaller: a mistake there must not hide behind the others)."""
    err = gh.assert_parity(out, ref, what)
    row0 = np.concatenate([[0], np.cumsum(qlens)])
    dec = np.concatenate([np.arange(row0[b], row0[b + 1]) for b in range(len(qlens)) if qlens[b] == 1] or [np.array([], int)])
    pre = np.concatenate([np.arange(row0[b], row0[b + 1]) for b in range(len(qlens)) if qlens[b] > 1] or [np.array([], int)])
    g = out.cpu().double().numpy()
    parts = {}
    for name, rows in (("decode", dec), ("prefill", pre)):
        if len(rows):
            rows = rows.astype(np.int64)
            parts[name] = gh.assert_parity(g[rows], ref[rows], f"{what}, {name} rows")
    return err, parts


@pytest.mark.parametrize("hq,hkv", [(32, 8), (16, 2), (8, 8), (16, 1), (9, 3), (14, 2)])
def test_batch_with_both_kinds(hq, hkv):
    """Decode requests (short, long enough to be split, ragged last pages) next to whole prompts and chunks."""
    lens = [1, 17, 300, 5000, 1000, 64, 65, 2049, 513, 9000, 33, 700]
    qlens = [1, 17, 1, 1, 64, 1, 1, 100, 257, 1, 1, 300]
    case = make_case(lens, qlens, hq, hkv, seed=hq + hkv, poison=True)
    out, plan = run_gpu(*case)
    c = plan.counts
    assert plan.query_tokens == sum(qlens) and c["prefill_items"] > 0 and c["decode_items"] > 0
    err, parts = check_rows(out, reference(*case), case[4], f"mixed hq={hq} hkv={hkv}")
    print(f"hq={hq} hkv={hkv}: {c}, whole {err}, parts {parts}")
    assert parts["decode"][1] < 1e-4          # the decode rows keep the decode path's precision


def test_only_decode_requests_and_only_chunks():
    for lens, qlens in (([40, 2100, 517, 16, 6000], [1, 1, 1, 1, 1]), ([300, 2100, 517], [300, 77, 2])):
        case = make_case(lens, qlens, 32, 8, seed=len(lens))
        out, plan = run_gpu(*case)
        c = plan.counts
        assert (c["prefill_items"] == 0) == all(n == 1 for n in qlens)
        assert (c["decode_items"] == 0) == all(n > 1 for n in qlens)
        check_rows(out, reference(*case), case[4], f"mixed qlens={qlens}")


def test_head_dim_64():
    lens = [1, 17, 300, 5000, 1000, 64, 65, 2049, 513, 33]
    qlens = [1, 17, 1, 1, 64, 1, 1, 100, 257, 1]
    case = make_case(lens, qlens, 8, 2, seed=640, poison=True, head_dim=64)
    out, _ = run_gpu(*case)
    check_rows(out, reference(*case), case[4], "mixed head_dim 64")


@pytest.mark.parametrize("page_size", [32, 64])
def test_larger_pages(page_size):
    lens = [33, 700, 129, 4000, 4000, 90]
    qlens = [1, 128, 1, 500, 1, 90]
    case = make_case(lens, qlens, 32, 8, page_size=page_size, seed=page_size, poison=True)
    out, _ = run_gpu(*case)
    check_rows(out, reference(*case), case[4], f"mixed page={page_size}")


def test_serving_shaped_batch_whole_tensor():
    """Forty decode requests drawn like the heterogeneous mix (short ones and ones long enough to be split many
    times) plus chunks ending longer contexts: every element against the oracle."""
    rng = wl.CounterRng(4711)
    short = np.clip(np.rint(np.exp(np.log(512.0) + 0.8 * rng.normal(28))), 16, 4096).astype(np.int64)
    long_ = rng.integers(6000, 20000, 12)
    lens = np.concatenate([short, long_, [4000, 5000, 3000]]).astype(np.int32)
    qlens = np.concatenate([np.ones(40, dtype=np.int64), [128, 128, 200]]).astype(np.int32)
    case = make_case(lens, qlens, 32, 8, seed=77)
    out, plan = run_gpu(*case)
    err, parts = check_rows(out, reference(*case), case[4], "serving-shaped mixed batch")
    print(f"serving-shaped: {plan.counts}, whole {err}, parts {parts}")


def test_bench_workload_sampled():
    """The batch `bench.py --mixed` times (the 256 decode requests of the heterogeneous mix + 8 chunks of 512
    tokens), at full size and in its launch configuration: sampled decode rows and sampled prefill rows against
    the oracle, each kind to its own bar, and every row finite."""
    w, lens, qlens = wl.mixed_workload()
    inp = wl.make_inputs(w, device="cuda", seed=w.seed, lens=lens)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed + 1)
    q = torch.randn(int(qlens.sum()), w.num_q_heads, w.head_dim, generator=gen, device="cuda").to(torch.bfloat16)
    out = torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda")
    plan = binding.MixedPlan(lens, qlens, w.num_q_heads, w.num_kv_heads, w.head_dim, w.page_size,
                             inp.block_table.shape[1], 0)
    ws = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device="cuda")
    binding.paged_mixed_attn(plan, ws, q, inp.k_pages, inp.v_pages, inp.block_table, inp.context_lens, w.scale, out)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    rng = np.random.default_rng(4242)
    row0 = np.concatenate([[0], np.cumsum(qlens)])
    decode = np.nonzero(qlens == 1)[0]
    chunks = np.nonzero(qlens > 1)[0]
    picks = {"decode": [], "prefill": []}
    for b in (int(decode[0]), int(decode[-1]), int(decode[np.argmax(lens[decode])]), int(decode[np.argmin(lens[decode])])):
        picks["decode"].append((b, 0, int(rng.integers(0, w.num_q_heads))))
    for _ in range(20):
        picks["decode"].append((int(rng.choice(decode)), 0, int(rng.integers(0, w.num_q_heads))))
    for b in (int(chunks[0]), int(chunks[-1])):
        for i in (0, 31, 32, 33, 255, 510, 511):
            picks["prefill"].append((b, i, int(rng.integers(0, w.num_q_heads))))
    for _ in range(12):
        b = int(rng.choice(chunks))
        picks["prefill"].append((b, int(rng.integers(0, qlens[b])), int(rng.integers(0, w.num_q_heads))))
    for kind, rows in picks.items():
        got, ref = [], []
        for b, i, h in rows:
            row = int(row0[b]) + i
            visible = int(lens[b] - qlens[b]) + i + 1
            n = (visible + w.page_size - 1) // w.page_size
            ids = inp.block_table[b, :n].long()
            j = h // w.group
            ref.append(oracle.paged_decode_attn(q[row:row + 1, h:h + 1].cpu(), inp.k_pages[ids, j:j + 1].cpu(),
                                                inp.v_pages[ids, j:j + 1].cpu(), np.arange(n, dtype=np.int32)[None, :],
                                                np.array([visible], dtype=np.int32), inp.scale)[0, 0])
            got.append(out[row, h])
        err = gh.assert_parity(torch.stack(got), np.stack(ref), f"mixed bench workload, {kind} rows")
        print(f"mixed bench workload: {len(rows)} {kind} rows, max_abs {err[0]:.2e}, rel_l2 {err[1]:.2e}", flush=True)
        if kind == "decode":
            assert err[1] < 2e-5          # the decode items carry the weights as hi + lo halves


def test_update_and_rerun_is_bit_identical():
    case = make_case([700, 90, 3000, 50], [200, 90, 1, 1], 32, 8, seed=9)
    w, cpu, q, lens, qlens = case
    out1, plan = run_gpu(*case)
    other = make_case([100, 2000], [1, 100], 32, 8, seed=10)
    for _ in range(2 * binding.PLAN_RING + 1):     # wraps the staging ring
        plan2 = binding.MixedPlan(lens, qlens, 32, 8, 128, 16, cpu.block_table.shape[1], 0)
        out2, _ = run_gpu(*case, plan=plan2)
    assert torch.equal(out1, out2)
    # one plan object re-planned for another batch and back
    wide = max(cpu.block_table.shape[1], other[1].block_table.shape[1])
    plan3 = binding.MixedPlan(lens, qlens, 32, 8, 128, 16, cpu.block_table.shape[1], 0, capacity=8, max_query_tokens=4096)
    for _ in range(3):
        plan3.update(lens, qlens)
        out3, _ = run_gpu(*case, plan=plan3)
        assert torch.equal(out1, out3)
    assert wide >= 1


def test_plan_errors():
    with pytest.raises(binding.OserveError) as e:
        binding.MixedPlan([10], [11], 32, 8, 128, 16, 4, 0)          # n > L
    assert e.value.status == binding.ERR_CONTEXT_LEN
    with pytest.raises(binding.OserveError) as e:
        binding.MixedPlan([10], [4], 34, 2, 128, 16, 4, 0)           # group 17
    assert e.value.status == binding.ERR_SHAPE
    plan = binding.MixedPlan([100, 50], [10, 1], 32, 8, 128, 16, 8, 0, max_query_tokens=16)
    before = plan.counts
    with pytest.raises(binding.OserveError) as e:
        plan.update([100, 50], [17, 1])
    assert e.value.status == binding.ERR_PLAN_MISMATCH
    assert plan.counts == before                                    # a refused update changes nothing
