"""The decode entry point that allocates nothing (oserve_paged_decode_attn_static: workspace in a fixed array
of device memory that the library holds), through the C ABI, against the ordinary entry point and the oracle:
two calls in a row on the shared array, the second with a smaller batch."""
import numpy as np
import pytest
import torch

from paper_2602_12151_amd import binding, workloads as wl
from tests import gpu_helpers as gh

pytestmark = pytest.mark.gpu


def _both(cpu, split_tokens):
    dev = gh.to_device(cpu)
    w = dev.workload
    ref_out, op = gh.gpu_attention(dev, split_tokens=split_tokens)          # caller-owned workspace
    plan = binding.Plan(dev.context_lens_host, w.num_q_heads, w.num_kv_heads, w.head_dim, w.page_size,
                        dev.block_table.shape[1], split_tokens, 0)
    assert plan.workspace_bytes <= binding.static_workspace_bytes()
    out = torch.full(dev.q.shape, float("nan"), dtype=torch.float32, device="cuda")
    binding.paged_decode_attn_static(plan, dev.q, dev.k_pages, dev.v_pages, dev.block_table, dev.context_lens,
                                     dev.scale, out)
    torch.cuda.synchronize()
    return out, ref_out, op.plan.num_work_items


def test_static_workspace_two_calls_second_smaller():
    binding.static_workspace_init(0)
    w = wl.WORKLOADS[1]
    big = wl.make_inputs(w, device="cpu", seed=71, lens=np.array([3000, 17, 1024, 555, 2047, 64, 1, 900], dtype=np.int32))
    small = wl.make_inputs(w, device="cpu", seed=72, lens=np.array([700, 33, 129], dtype=np.int32))
    for name, cpu, split in (("first, larger", big, 128), ("second, smaller", small, 64), ("third, automatic", big, 0)):
        out, ref_out, items = _both(cpu, split)
        # the same kernels on the same inputs: the workspace's address cannot change a bit of the result
        assert torch.equal(out, ref_out), name
        err = gh.assert_parity(out, gh.oracle_attention(cpu), name)
        print(f"static workspace, {name}: {items} work items, max_abs {err[0]:.2e}, rel_l2 {err[1]:.2e}")


def test_static_workspace_refuses_a_plan_that_does_not_fit():
    w = wl.WORKLOADS[1]
    lens = np.array([60000, 50000], dtype=np.int32)
    width = int(wl.pages_needed(lens).max())
    plan = binding.Plan(lens, w.num_q_heads, w.num_kv_heads, w.head_dim, 16, width, 16, 0)     # one split per page
    assert plan.workspace_bytes > binding.static_workspace_bytes()
    t = torch.zeros(256, dtype=torch.uint8, device="cuda")
    st = binding.lib.oserve_paged_decode_attn_static(plan.handle, t.data_ptr(), t.data_ptr(), t.data_ptr(), t.data_ptr(),
                                                     t.data_ptr(), 1.0, t.data_ptr(), None)
    assert st == binding.ERR_WORKSPACE
    assert "workspace" in binding.status_string(st)
