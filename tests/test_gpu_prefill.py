"""GPU-vs-oracle parity of the chunked-prefill path, called through the C ABI.

Same bar as the decode path: max-abs error <= 1e-2 and relative L2 error <= 2e-3
against the fp64 oracle on the same seeded bits.
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
    w = wl.Workload(9, "prefill", batch=len(lens), num_q_heads=hq, num_kv_heads=hkv, head_dim=head_dim, page_size=page_size)
    cpu = wl.make_inputs(w, device="cpu", seed=seed, lens=lens)
    g = torch.Generator().manual_seed(seed + 12345)
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


def run_gpu(w, cpu, q, lens, qlens):
    plan = binding.PrefillPlan(lens, qlens, w.num_q_heads, w.num_kv_heads, w.head_dim, w.page_size,
                               cpu.block_table.shape[1], 0)
    out = torch.empty(q.shape, dtype=torch.float32, device="cuda")
    binding.paged_prefill_attn(plan, q.cuda(), cpu.k_pages.cuda(), cpu.v_pages.cuda(), cpu.block_table.cuda(),
                               w.scale, out)
    torch.cuda.synchronize()
    return out, plan


def reference(w, cpu, q, lens, qlens):
    return oracle.paged_prefill_attn(q, cpu.k_pages, cpu.v_pages, cpu.block_table.numpy(), lens, qlens, w.scale)


@pytest.mark.parametrize("hq,hkv", [(32, 8), (16, 2), (8, 8), (4, 2), (16, 1), (6, 2), (10, 2), (12, 2), (7, 1), (15, 1)])
def test_mixed_chunks_all_group_sizes(hq, hkv):
    """Whole prompts, chunks at the end of longer contexts, single decode tokens, ragged last blocks."""
    lens = [1, 17, 300, 300, 1000, 64, 65, 2049, 513]
    qlens = [1, 17, 300, 37, 64, 64, 1, 100, 257]
    case = make_case(lens, qlens, hq, hkv, seed=hq + hkv, poison=True)
    out, plan = run_gpu(*case)
    assert plan.query_tokens == sum(qlens)
    print(f"hq={hq} hkv={hkv}:", gh.assert_parity(out, reference(*case), f"prefill hq={hq} hkv={hkv}"),
          "items", plan.num_work_items, "block", plan.block_tokens)


@pytest.mark.parametrize("hq,hkv,page_size", [(8, 2, 16), (32, 8, 16), (6, 6, 32), (12, 4, 64), (16, 1, 16)])
def test_head_dim_64(hq, hkv, page_size):
    lens = [1, 17, 300, 300, 1000, 64, 65, 2049, 513]
    qlens = [1, 17, 300, 37, 64, 64, 1, 100, 257]
    case = make_case(lens, qlens, hq, hkv, page_size=page_size, seed=64 + hq, poison=True, head_dim=64)
    out, plan = run_gpu(*case)
    print(f"head_dim 64, hq={hq} hkv={hkv} page={page_size}:", gh.assert_parity(out, reference(*case), "prefill head_dim 64"),
          "items", plan.num_work_items)


@pytest.mark.parametrize("page_size", [32, 64])
def test_larger_pages(page_size):
    lens = [33, 700, 129, 4000]
    qlens = [33, 128, 2, 500]
    case = make_case(lens, qlens, 32, 8, page_size=page_size, seed=page_size, poison=True)
    out, _ = run_gpu(*case)
    gh.assert_parity(out, reference(*case), f"prefill page={page_size}")


def test_one_token_per_request_matches_the_decode_path_and_oracle():
    lens = [5, 300, 77, 1024, 4097]
    case = make_case(lens, [1] * len(lens), 32, 8, seed=3)
    w, cpu, q, lens_a, qlens = case
    out, _ = run_gpu(*case)
    ref = reference(*case)
    gh.assert_parity(out, ref, "prefill n=1")


def test_whole_prompt_long():
    """One whole prompt of 3000 tokens (n = L): every block is on the diagonal at its end."""
    case = make_case([3000], [3000], 8, 2, seed=5)
    out, plan = run_gpu(*case)
    print("whole prompt:", gh.assert_parity(out, reference(*case), "whole prompt"), "items", plan.num_work_items)


def test_update_and_rerun_is_bit_identical():
    case = make_case([700, 90], [200, 90], 32, 8, seed=9)
    w, cpu, q, lens, qlens = case
    out1, plan = run_gpu(*case)
    out2 = torch.empty_like(out1)
    for _ in range(2 * binding.PLAN_RING + 1):     # wraps the staging ring
        plan.update(lens, qlens)
        binding.paged_prefill_attn(plan, q.cuda(), cpu.k_pages.cuda(), cpu.v_pages.cuda(), cpu.block_table.cuda(),
                                   w.scale, out2)
    torch.cuda.synchronize()
    assert torch.equal(out1, out2)


def test_plan_errors():
    with pytest.raises(binding.OserveError) as e:
        binding.PrefillPlan([10], [11], 32, 8, 128, 16, 4, 0)          # n > L
    assert e.value.status == binding.ERR_CONTEXT_LEN
    with pytest.raises(binding.OserveError) as e:
        binding.PrefillPlan([10], [4], 34, 2, 128, 16, 4, 0)           # group 17
    assert e.value.status == binding.ERR_SHAPE
    with pytest.raises(binding.OserveError) as e:
        binding.PrefillPlan([10], [4], 32, 8, 96, 16, 4, 0)            # head_dim 96
    assert e.value.status == binding.ERR_SHAPE
    plan = binding.PrefillPlan([100], [10], 32, 8, 128, 16, 8, 0, max_query_tokens=16)
    with pytest.raises(binding.OserveError) as e:
        plan.update([100], [17])
    assert e.value.status == binding.ERR_PLAN_MISMATCH


def _oracle_row(inp, q, row, h, b, visible, group):
    """Oracle output of query row `row`, head h, of request b, which sees the first `visible` cached tokens:
    a decode step over that prefix (only the needed pages of one kv head are copied to the host)."""
    ps = inp.workload.page_size
    n = (visible + ps - 1) // ps
    ids = inp.block_table[b, :n].long()
    j = h // group
    k = inp.k_pages[ids, j:j + 1].cpu()
    v = inp.v_pages[ids, j:j + 1].cpu()
    bt = np.arange(n, dtype=np.int32)[None, :]
    return oracle.paged_decode_attn(q[row:row + 1, h:h + 1].cpu(), k, v, bt, np.array([visible], dtype=np.int32),
                                    inp.scale)[0, 0]


@pytest.mark.parametrize("which", [0, 1, 2])
def test_bench_workloads_sampled(which):
    """The workloads `bench.py --prefill 0|1|2` times, at full size and in its launch configuration, against the
    oracle on sampled (query token, head) rows: first and last token of a chunk, both sides of block
    boundaries, random ones."""
    w, lens, qlens = wl.prefill_workload(which)
    inp = wl.make_inputs(w, device="cuda", seed=w.seed, lens=lens)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed + 1)
    q = torch.randn(int(qlens.sum()), 32, 128, generator=gen, device="cuda").to(torch.bfloat16)
    out = torch.empty(q.shape, dtype=torch.float32, device="cuda")
    plan = binding.PrefillPlan(lens, qlens, 32, 8, 128, 16, inp.block_table.shape[1], 0)
    binding.paged_prefill_attn(plan, q, inp.k_pages, inp.v_pages, inp.block_table, w.scale, out)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    rng = np.random.default_rng(77 + which)
    row0 = np.concatenate([[0], np.cumsum(qlens)])
    picks = []
    for b in (0, len(lens) - 1, int(np.argmax(lens))):
        n = int(qlens[b])
        for i in (0, 1, 63, 64, 65, n // 2, n - 2, n - 1):
            picks.append((b, i, int(rng.integers(0, 32))))
    for _ in range(24):
        b = int(rng.integers(0, len(lens)))
        picks.append((b, int(rng.integers(0, qlens[b])), int(rng.integers(0, 32))))
    got, ref = [], []
    for b, i, h in picks:
        row = int(row0[b]) + i
        got.append(out[row, h])
        ref.append(_oracle_row(inp, q, row, h, b, int(lens[b] - qlens[b]) + i + 1, w.group))
    got, ref = torch.stack(got), np.stack(ref)
    err = gh.assert_parity(got, ref, f"prefill bench workload {which}")
    per_row = np.linalg.norm(got.cpu().double().numpy() - ref, axis=1) / np.linalg.norm(ref, axis=1)
    # The bar is stated for a whole output tensor.  A single (token, head) row is a sample of 128 values of
    # the same error distribution (rms relative rounding error of bf16 weights, about 1.6e-3), so single rows
    # scatter around it; twice the bar catches a row that is wrong, not one that is unlucky.
    assert per_row.max() <= 2 * gh.REL_L2_TOL, per_row.max()
    print(f"prefill bench workload {which}: {len(picks)} rows, max_abs {err[0]:.2e}, rel_l2 {err[1]:.2e}, "
          f"worst row {per_row.max():.2e}")


def test_scores_that_keep_rising_exercise_the_lazy_reference_maximum():
    """Scores that grow with the key index: slowly (the reference maximum of the online softmax stays behind
    the true one for a few steps and the weights exceed 1), fast (it moves at every step) and with a large
    overall range; also a strongly negative trend (the first key dominates)."""
    lens, qlens = [700, 700, 300, 520], [700, 130, 300, 7]
    w, cpu, q, lens, qlens = make_case(lens, qlens, 8, 2, seed=21)
    slopes = [0.05, 1.0, -0.7, 0.013]
    bt = cpu.block_table.numpy()
    q[:] = 0
    q[:, :, 0] = 8.0
    for b, (L, slope) in enumerate(zip(lens, slopes)):
        t = torch.arange(int(L))
        pages = torch.from_numpy(bt[b, : (int(L) + 15) // 16].astype(np.int64))[t // 16]
        cpu.k_pages[pages, :, t % 16, :] = 0
        cpu.k_pages[pages, :, t % 16, 0] = (slope * t.float()).to(torch.bfloat16)[:, None]
    case = (w, cpu, q, lens, qlens)
    out, _ = run_gpu(*case)
    print("rising scores:", gh.assert_parity(out, reference(*case), "rising scores"))


def _set_keys(cpu, lens, key_of):
    """Overwrite the cached keys of every request: key t of request b, all kv heads, becomes key_of(b, t) [L, D]."""
    bt = cpu.block_table.numpy()
    for b, L in enumerate(lens):
        t = torch.arange(int(L))
        pages = torch.from_numpy(bt[b, : (int(L) + 15) // 16].astype(np.int64))[t // 16]
        cpu.k_pages[pages, :, t % 16, :] = key_of(b, int(L)).to(torch.bfloat16)[:, None, :]


def test_constant_values_are_reproduced():
    """Every value row of a request is the same vector c: whatever the weights, the output is c.  The weights are
    rounded to bf16 for the value product; the normaliser is the sum of the ROUNDED weights (it comes from the same
    matrix-core product), so the output is an exact convex combination of value rows and no rounding error of
    the weights is left in it."""
    lens, qlens = [900, 333, 2050], [300, 333, 5]
    w, cpu, q, lens, qlens = make_case(lens, qlens, 8, 2, seed=33)
    c = torch.linspace(-3.0, 5.0, 128).to(torch.bfloat16)
    cpu.v_pages[:] = c
    out, _ = run_gpu(w, cpu, q, lens, qlens)
    ref = reference(w, cpu, q, lens, qlens)
    assert np.abs(ref - c.double().numpy()).max() < 1e-12                    # the oracle agrees on what is asked
    err = np.abs(out.cpu().double().numpy() - ref).max()
    # what is left is fp32 accumulation over up to 2050 keys of values up to 5 (a few 1e-6); an error of the bf16
    # weights in the result would be of the order 5 * 2^-9 = 1e-2
    assert err <= 2e-5, err
    print(f"constant values: max_abs {err:.2e}")


def test_rounding_errors_of_one_sign_do_not_add_up():
    """All keys but the first have the same score, so all their weights are the same number, which is not a bf16
    number: every one of them is rounded the same way (the case in which rounding errors add up instead of
    averaging out), and the values are all positive.  With the normaliser taken from the rounded weights the
    common factor cancels; the error stays far inside the bar (it would be about 2^-9 relative otherwise)."""
    lens, qlens = [1500, 700], [200, 700]
    w, cpu, q, lens, qlens = make_case(lens, qlens, 8, 2, seed=34)
    g = torch.Generator().manual_seed(99)
    kstar = torch.randn(128, generator=g)

    def keys(b, L):
        k = kstar.repeat(L, 1)
        k[0] = 1.3 * kstar
        return k
    _set_keys(cpu, lens, keys)
    cpu.v_pages[:] = (cpu.v_pages.float().abs() + 0.5).to(torch.bfloat16)
    out, _ = run_gpu(w, cpu, q, lens, qlens)
    ref = reference(w, cpu, q, lens, qlens)
    max_abs, rel_l2 = gh.errors(out, ref)
    # (the largest single error sits in the first rows of the whole prompt, where the first key's different weight
    # meets one or two others: an ordinary rounding error of one weight, 2^-9 times a difference of values)
    assert rel_l2 <= 2e-4 and max_abs <= 5e-3, (max_abs, rel_l2)
    print(f"equal weights off the bf16 grid, positive values: max_abs {max_abs:.2e}, rel_l2 {rel_l2:.2e}")
