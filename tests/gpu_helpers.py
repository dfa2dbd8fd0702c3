"""Shared by the GPU parity tests: run the HIP path through the C ABI, run the oracle, compare."""
import numpy as np
import torch

from oracle import paged_attention_oracle as oracle
from paper_2602_12151_amd import workloads as wl

MAX_ABS_TOL = 1e-2     # tolerances the benchmark spec fixes for bf16 inputs / fp32 accumulation
REL_L2_TOL = 2e-3


def to_device(inp: wl.Inputs, device="cuda") -> wl.Inputs:
    """A copy of the same bits on the GPU."""
    return wl.Inputs(workload=inp.workload, q=inp.q.to(device), k_pages=inp.k_pages.to(device),
                     v_pages=inp.v_pages.to(device), block_table=inp.block_table.to(device),
                     context_lens=inp.context_lens.to(device), context_lens_host=inp.context_lens_host,
                     scale=inp.scale, used_pages=inp.used_pages)


def gpu_attention(inp_dev: wl.Inputs, split_tokens: int = 0) -> torch.Tensor:
    from paper_2602_12151_amd import binding
    op = binding.DecodeAttention(inp_dev, split_tokens=split_tokens)
    out = op.step(inp_dev)
    torch.cuda.synchronize()
    return out.clone(), op


def oracle_attention(inp_cpu: wl.Inputs) -> np.ndarray:
    return oracle.paged_decode_attn(inp_cpu.q, inp_cpu.k_pages, inp_cpu.v_pages,
                                    inp_cpu.block_table, inp_cpu.context_lens, inp_cpu.scale)


def errors(gpu_out, ref: np.ndarray):
    g = gpu_out.detach().cpu().to(torch.float64).numpy() if isinstance(gpu_out, torch.Tensor) else gpu_out
    assert g.shape == ref.shape
    assert np.all(np.isfinite(g)), "GPU output has non-finite values"
    max_abs = float(np.max(np.abs(g - ref)))
    rel_l2 = float(np.linalg.norm((g - ref).ravel()) / np.linalg.norm(ref.ravel()))
    return max_abs, rel_l2


def assert_parity(gpu_out, ref, what=""):
    max_abs, rel_l2 = errors(gpu_out, ref)
    assert max_abs <= MAX_ABS_TOL and rel_l2 <= REL_L2_TOL, f"{what}: max_abs={max_abs:.3e} rel_l2={rel_l2:.3e}"
    return max_abs, rel_l2


def sampled_oracle_rows(inp_dev: wl.Inputs, pairs):
    """Oracle rows for sampled (request, query head) pairs of a batch that lives on the GPU.

    Only the sampled request's pages of the needed kv head are copied to the
    host (input bits, never outputs), renumbered into a compact pool.
    """
    w = inp_dev.workload
    rows = []
    for b, h in pairs:
        L = int(inp_dev.context_lens_host[b])
        n = (L + w.page_size - 1) // w.page_size
        ids = inp_dev.block_table[b, :n].long()
        j = h // w.group
        k = inp_dev.k_pages[ids, j:j + 1].cpu()
        v = inp_dev.v_pages[ids, j:j + 1].cpu()
        q = inp_dev.q[b:b + 1, h:h + 1].cpu()
        bt = np.arange(n, dtype=np.int32)[None, :]
        cl = np.array([L], dtype=np.int32)
        rows.append(oracle.paged_decode_attn(q, k, v, bt, cl, inp_dev.scale)[0, 0])
    return np.stack(rows)


def oracle_whole_batch(inp_dev: wl.Inputs, progress=None) -> np.ndarray:
    """Oracle output [B, Hq, D] of a batch that lives on the GPU, request by request: only one request's pages
    (input bits, never outputs) are on the host at a time, renumbered into a compact pool."""
    w = inp_dev.workload
    B = len(inp_dev.context_lens_host)
    ref = np.empty((B, w.num_q_heads, w.head_dim), dtype=np.float64)
    for b in range(B):
        L = int(inp_dev.context_lens_host[b])
        n = (L + w.page_size - 1) // w.page_size
        ids = inp_dev.block_table[b, :n].long()
        k = inp_dev.k_pages[ids].cpu()
        v = inp_dev.v_pages[ids].cpu()
        bt = np.arange(n, dtype=np.int32)[None, :]
        ref[b] = oracle.paged_decode_attn(inp_dev.q[b:b + 1].cpu(), k, v, bt, np.array([L], dtype=np.int32),
                                          inp_dev.scale)[0]
        if progress and (b + 1) % progress == 0:
            print(f"  oracle: {b + 1}/{B} requests", flush=True)
    return ref
