"""Thin ctypes binding over the C ABI in include/oserve.h (argument marshalling only).

Every step of the path runs in the library's kernels; torch is used for device
memory and the stream handle.  There is no fallback: if the built library is
missing, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

_LIB_PATH = os.environ.get("OSERVE_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "liboserve.so")

OK, ERR_NULL, ERR_SHAPE, ERR_CONTEXT_LEN, ERR_WORKSPACE, ERR_PLAN_MISMATCH, ERR_DEVICE, ERR_ALIGNMENT = range(8)
PLAN_RING = 8


class OserveError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} (status {status})")


def _load() -> ctypes.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is not built; run `python -m paper_2602_12151_amd.build` "
                          "(there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    i32, vp, sz = ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t
    pi32 = ctypes.POINTER(ctypes.c_int32)
    lib.oserve_plan_create.restype = ctypes.c_int
    lib.oserve_plan_create.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, i32, i32, ctypes.POINTER(vp)]
    lib.oserve_plan_update.restype = ctypes.c_int
    lib.oserve_plan_update.argtypes = [vp, vp, i32]
    lib.oserve_plan_destroy.restype = None
    lib.oserve_plan_destroy.argtypes = [vp]
    lib.oserve_plan_run.restype = ctypes.c_int
    lib.oserve_plan_run.argtypes = [vp, i32, pi32]
    for name in ("oserve_plan_batch", "oserve_plan_num_work_items", "oserve_plan_split_pages", "oserve_plan_split_tokens",
                 "oserve_plan_num_runs"):
        getattr(lib, name).restype = i32
        getattr(lib, name).argtypes = [vp]
    lib.oserve_plan_request.restype = ctypes.c_int
    lib.oserve_plan_request.argtypes = [vp, i32, pi32, pi32]
    for name in ("oserve_plan_workspace_bytes", "oserve_plan_workspace_bytes_max"):
        getattr(lib, name).restype = sz
        getattr(lib, name).argtypes = [vp]
    lib.oserve_paged_decode_attn.restype = ctypes.c_int
    lib.oserve_paged_decode_attn.argtypes = [vp, vp, sz, vp, vp, vp, vp, vp, ctypes.c_float, vp, vp]
    lib.oserve_plan_stage.restype = ctypes.c_int
    lib.oserve_plan_stage.argtypes = [vp, vp, sz, vp]
    lib.oserve_paged_decode_attn_staged.restype = ctypes.c_int
    lib.oserve_paged_decode_attn_staged.argtypes = [vp, vp, sz, vp, vp, vp, vp, vp, ctypes.c_float, vp, vp]
    lib.oserve_paged_decode_attn_static.restype = ctypes.c_int
    lib.oserve_paged_decode_attn_static.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.c_float, vp, vp]
    lib.oserve_static_workspace_bytes.restype = sz
    lib.oserve_static_workspace_bytes.argtypes = []
    lib.oserve_static_workspace_init.restype = ctypes.c_int
    lib.oserve_static_workspace_init.argtypes = [i32]
    lib.oserve_plan_enable_timing.restype = ctypes.c_int
    lib.oserve_plan_enable_timing.argtypes = [vp, i32]
    lib.oserve_plan_split_kernel_ms.restype = ctypes.c_int
    lib.oserve_plan_split_kernel_ms.argtypes = [vp, ctypes.POINTER(ctypes.c_float), pi32]
    i64 = ctypes.c_int64
    lib.oserve_prefill_plan_create.restype = ctypes.c_int
    lib.oserve_prefill_plan_create.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, i64, ctypes.POINTER(vp)]
    lib.oserve_prefill_plan_update.restype = ctypes.c_int
    lib.oserve_prefill_plan_update.argtypes = [vp, vp, vp, i32]
    lib.oserve_prefill_plan_destroy.restype = None
    lib.oserve_prefill_plan_destroy.argtypes = [vp]
    for name in ("oserve_prefill_plan_num_work_items", "oserve_prefill_plan_block_tokens"):
        getattr(lib, name).restype = i32
        getattr(lib, name).argtypes = [vp]
    lib.oserve_prefill_plan_query_tokens.restype = i64
    lib.oserve_prefill_plan_query_tokens.argtypes = [vp]
    lib.oserve_prefill_plan_item.restype = ctypes.c_int
    lib.oserve_prefill_plan_item.argtypes = [vp, i32, pi32]
    lib.oserve_paged_prefill_attn.restype = ctypes.c_int
    lib.oserve_paged_prefill_attn.argtypes = [vp, vp, vp, vp, vp, ctypes.c_float, vp, vp]
    lib.oserve_prefill_plan_enable_timing.restype = ctypes.c_int
    lib.oserve_prefill_plan_enable_timing.argtypes = [vp, i32]
    lib.oserve_prefill_plan_kernel_ms.restype = ctypes.c_int
    lib.oserve_prefill_plan_kernel_ms.argtypes = [vp, ctypes.POINTER(ctypes.c_float), pi32]
    lib.oserve_mixed_plan_create.restype = ctypes.c_int
    lib.oserve_mixed_plan_create.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, i64, ctypes.POINTER(vp)]
    lib.oserve_mixed_plan_update.restype = ctypes.c_int
    lib.oserve_mixed_plan_update.argtypes = [vp, vp, vp, i32]
    lib.oserve_mixed_plan_destroy.restype = None
    lib.oserve_mixed_plan_destroy.argtypes = [vp]
    lib.oserve_mixed_plan_query_tokens.restype = i64
    lib.oserve_mixed_plan_query_tokens.argtypes = [vp]
    lib.oserve_mixed_plan_counts.restype = ctypes.c_int
    lib.oserve_mixed_plan_counts.argtypes = [vp, pi32]
    lib.oserve_mixed_plan_prefill_item.restype = ctypes.c_int
    lib.oserve_mixed_plan_prefill_item.argtypes = [vp, i32, pi32]
    for name in ("oserve_mixed_plan_workspace_bytes", "oserve_mixed_plan_workspace_bytes_max"):
        getattr(lib, name).restype = sz
        getattr(lib, name).argtypes = [vp]
    lib.oserve_paged_mixed_attn.restype = ctypes.c_int
    lib.oserve_paged_mixed_attn.argtypes = [vp, vp, sz, vp, vp, vp, vp, vp, ctypes.c_float, vp, vp]
    lib.oserve_mixed_plan_enable_timing.restype = ctypes.c_int
    lib.oserve_mixed_plan_enable_timing.argtypes = [vp, i32]
    lib.oserve_mixed_plan_kernel_ms.restype = ctypes.c_int
    lib.oserve_mixed_plan_kernel_ms.argtypes = [vp, ctypes.POINTER(ctypes.c_float), pi32]
    lib.oserve_kv_migration_create.restype = ctypes.c_int
    lib.oserve_kv_migration_create.argtypes = [vp, vp, i32, i32, i32, ctypes.POINTER(vp)]
    lib.oserve_kv_migration_destroy.restype = None
    lib.oserve_kv_migration_destroy.argtypes = [vp]
    lib.oserve_kv_migration_num_pages.restype = i64
    lib.oserve_kv_migration_num_pages.argtypes = [vp]
    lib.oserve_kv_migration_request.restype = ctypes.c_int
    lib.oserve_kv_migration_request.argtypes = [vp, i32, pi32, pi32]
    for name in ("oserve_kv_gather", "oserve_kv_scatter"):
        getattr(lib, name).restype = ctypes.c_int
        getattr(lib, name).argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp]
    lib.oserve_kv_migration_enable_timing.restype = ctypes.c_int
    lib.oserve_kv_migration_enable_timing.argtypes = [vp, i32]
    lib.oserve_kv_migration_kernel_ms.restype = ctypes.c_int
    lib.oserve_kv_migration_kernel_ms.argtypes = [vp, ctypes.POINTER(ctypes.c_float), pi32]
    lib.oserve_switch_plan.restype = ctypes.c_int
    lib.oserve_switch_plan.argtypes = [i32, vp, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.oserve_capacity_normalise.restype = ctypes.c_int
    lib.oserve_capacity_normalise.argtypes = [vp, i32, ctypes.POINTER(i64), vp]
    lib.oserve_assign_workload.restype = ctypes.c_int
    lib.oserve_assign_workload.argtypes = [i32, i32, vp, vp, vp, vp, ctypes.POINTER(ctypes.c_double)]
    lib.oserve_status_string.restype = ctypes.c_char_p
    lib.oserve_status_string.argtypes = [ctypes.c_int]
    return lib


lib = _load()


def status_string(status: int) -> str:
    return lib.oserve_status_string(status).decode()


def _host_lens(context_lens_host) -> np.ndarray:
    a = np.ascontiguousarray(np.asarray(context_lens_host), dtype=np.int32)
    if a.ndim != 1:
        raise ValueError("context_lens_host must be 1-D")
    return a


class Plan:
    """Owns an oserve_plan_t*.  Mirrors oserve_plan_* one to one."""

    def __init__(self, context_lens_host, num_q_heads: int, num_kv_heads: int, head_dim: int,
                 page_size: int, max_pages_per_seq: int, split_tokens: int = 0,
                 device_id: int = 0, capacity: int | None = None):
        lens = _host_lens(context_lens_host)
        self._h = ctypes.c_void_p()
        # the geometry the plan was built for: the launch wrapper checks its tensors against it
        # (the C ABI carries no shapes)
        self.geometry = (num_q_heads, num_kv_heads, head_dim, page_size, max_pages_per_seq)
        st = lib.oserve_plan_create(lens.ctypes.data, len(lens), num_q_heads, num_kv_heads, head_dim,
                                    page_size, max_pages_per_seq, split_tokens, device_id,
                                    len(lens) if capacity is None else capacity, ctypes.byref(self._h))
        if st != OK:
            self._h = ctypes.c_void_p()
            raise OserveError(st, "oserve_plan_create")

    def update(self, context_lens_host) -> None:
        lens = _host_lens(context_lens_host)
        st = lib.oserve_plan_update(self._h, lens.ctypes.data, len(lens))
        if st != OK:
            raise OserveError(st, "oserve_plan_update")

    def destroy(self) -> None:
        if getattr(self, "_h", None) and self._h.value and lib is not None:
            lib.oserve_plan_destroy(self._h)
            self._h = ctypes.c_void_p()

    __del__ = destroy

    @property
    def handle(self):
        return self._h

    @property
    def batch(self) -> int:
        return lib.oserve_plan_batch(self._h)

    @property
    def num_work_items(self) -> int:
        return lib.oserve_plan_num_work_items(self._h)

    @property
    def split_pages(self) -> int:
        return lib.oserve_plan_split_pages(self._h)

    @property
    def split_tokens(self) -> int:
        return lib.oserve_plan_split_tokens(self._h)

    @property
    def workspace_bytes(self) -> int:
        return lib.oserve_plan_workspace_bytes(self._h)

    @property
    def workspace_bytes_max(self) -> int:
        return lib.oserve_plan_workspace_bytes_max(self._h)

    def request(self, b: int):
        """(num_splits of request b, 16-token tiles of its largest split)."""
        s, p = ctypes.c_int32(), ctypes.c_int32()
        st = lib.oserve_plan_request(self._h, b, ctypes.byref(s), ctypes.byref(p))
        if st != OK:
            raise OserveError(st, "oserve_plan_request")
        return s.value, p.value

    @property
    def num_runs(self) -> int:
        return lib.oserve_plan_num_runs(self._h)

    def run(self, i: int) -> dict:
        """Run i of the launch order (see oserve_plan_run)."""
        f = (ctypes.c_int32 * 8)()
        st = lib.oserve_plan_run(self._h, i, f)
        if st != OK:
            raise OserveError(st, "oserve_plan_run")
        keys = ("request", "first_item", "num_splits", "pages_per_split", "page_begin", "page_end",
                "row_base", "total_splits")
        return dict(zip(keys, list(f)))

    def enable_timing(self, enable: bool = True) -> None:
        st = lib.oserve_plan_enable_timing(self._h, int(enable))
        if st != OK:
            raise OserveError(st, "oserve_plan_enable_timing")

    def split_kernel_ms(self):
        """(mean ms of the split kernel, launches averaged) since timing was enabled."""
        ms, n = ctypes.c_float(), ctypes.c_int32()
        st = lib.oserve_plan_split_kernel_ms(self._h, ctypes.byref(ms), ctypes.byref(n))
        if st != OK:
            raise OserveError(st, "oserve_plan_split_kernel_ms")
        return ms.value, n.value


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _check_decode_tensors(plan: Plan, q, k_pages, v_pages, block_table, context_lens, out, extra=()):
    """Device, dtype, contiguity and shape checks of a decode launch against the plan's geometry."""
    tensors = (q, k_pages, v_pages, block_table, context_lens, out) + tuple(extra)
    if not all(t.is_cuda for t in tensors):
        raise ValueError("all tensors must be device tensors")
    if q.dtype != torch.bfloat16 or k_pages.dtype != torch.bfloat16 or v_pages.dtype != torch.bfloat16:
        raise TypeError("q / k_pages / v_pages must be bf16")
    if block_table.dtype != torch.int32 or context_lens.dtype != torch.int32 or out.dtype != torch.float32:
        raise TypeError("block_table / context_lens must be int32 and out fp32")
    if not all(t.is_contiguous() for t in tensors):
        raise ValueError("tensors must be contiguous")
    hq, hkv, d, page, width = plan.geometry
    b = plan.batch
    if tuple(q.shape) != (b, hq, d) or out.shape != q.shape:
        raise ValueError(f"q / out must be [{b}, {hq}, {d}] for this plan, got {tuple(q.shape)} / {tuple(out.shape)}")
    if k_pages.dim() != 4 or tuple(k_pages.shape[1:]) != (hkv, page, d) or v_pages.shape != k_pages.shape:
        raise ValueError(f"k_pages / v_pages must be [pages, {hkv}, {page}, {d}] for this plan")
    if tuple(block_table.shape) != (b, width):
        raise ValueError(f"block_table must be [{b}, {width}] for this plan, got {tuple(block_table.shape)}")
    if tuple(context_lens.shape) != (b,):
        raise ValueError(f"context_lens must be [{b}] for this plan")


def paged_decode_attn(plan: Plan, workspace: torch.Tensor, q: torch.Tensor, k_pages: torch.Tensor,
                      v_pages: torch.Tensor, block_table: torch.Tensor, context_lens: torch.Tensor,
                      scale: float, out: torch.Tensor, stream: torch.cuda.Stream | None = None) -> torch.Tensor:
    """oserve_paged_decode_attn on torch tensors (layout checks only; no arithmetic here)."""
    _check_decode_tensors(plan, q, k_pages, v_pages, block_table, context_lens, out, (workspace,))
    s = torch.cuda.current_stream(q.device) if stream is None else stream
    st = lib.oserve_paged_decode_attn(plan.handle, _ptr(workspace), workspace.numel() * workspace.element_size(),
                                      _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table),
                                      _ptr(context_lens), ctypes.c_float(scale), _ptr(out),
                                      ctypes.c_void_p(s.cuda_stream))
    if st != OK:
        raise OserveError(st, "oserve_paged_decode_attn")
    return out


def plan_stage(plan: Plan, workspace: torch.Tensor, stream: torch.cuda.Stream | None = None) -> None:
    """oserve_plan_stage: the plan's work-item descriptors written into `workspace`, once for all layers of a step."""
    if workspace.device.type != "cuda" or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous tensor on the GPU")
    s = torch.cuda.current_stream(workspace.device) if stream is None else stream
    st = lib.oserve_plan_stage(plan.handle, _ptr(workspace), workspace.numel() * workspace.element_size(),
                               ctypes.c_void_p(s.cuda_stream))
    if st != OK:
        raise OserveError(st, "oserve_plan_stage")


def paged_decode_attn_staged(plan: Plan, workspace: torch.Tensor, q: torch.Tensor, k_pages: torch.Tensor,
                             v_pages: torch.Tensor, block_table: torch.Tensor, context_lens: torch.Tensor,
                             scale: float, out: torch.Tensor, stream: torch.cuda.Stream | None = None) -> torch.Tensor:
    """oserve_paged_decode_attn_staged on torch tensors: one layer's split and merge kernels over staged descriptors."""
    _check_decode_tensors(plan, q, k_pages, v_pages, block_table, context_lens, out, (workspace,))
    s = torch.cuda.current_stream(q.device) if stream is None else stream
    st = lib.oserve_paged_decode_attn_staged(plan.handle, _ptr(workspace), workspace.numel() * workspace.element_size(),
                                             _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table),
                                             _ptr(context_lens), ctypes.c_float(scale), _ptr(out),
                                             ctypes.c_void_p(s.cuda_stream))
    if st != OK:
        raise OserveError(st, "oserve_paged_decode_attn_staged")
    return out


def static_workspace_bytes() -> int:
    return lib.oserve_static_workspace_bytes()


def static_workspace_init(device_id: int = 0) -> None:
    st = lib.oserve_static_workspace_init(device_id)
    if st != OK:
        raise OserveError(st, "oserve_static_workspace_init")


def paged_decode_attn_static(plan: Plan, q: torch.Tensor, k_pages: torch.Tensor, v_pages: torch.Tensor,
                             block_table: torch.Tensor, context_lens: torch.Tensor, scale: float,
                             out: torch.Tensor, stream: torch.cuda.Stream | None = None) -> torch.Tensor:
    """oserve_paged_decode_attn_static on torch tensors: the decode step on the library's fixed workspace."""
    _check_decode_tensors(plan, q, k_pages, v_pages, block_table, context_lens, out)
    s = torch.cuda.current_stream(q.device) if stream is None else stream
    st = lib.oserve_paged_decode_attn_static(plan.handle, _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table),
                                             _ptr(context_lens), ctypes.c_float(scale), _ptr(out),
                                             ctypes.c_void_p(s.cuda_stream))
    if st != OK:
        raise OserveError(st, "oserve_paged_decode_attn_static")
    return out


class DecodeAttention:
    """Convenience holder: one plan + a workspace sized for any update, reused every step."""

    def __init__(self, inputs, split_tokens: int = 0, capacity: int | None = None):
        w = inputs.workload
        dev = inputs.q.device
        self.plan = Plan(inputs.context_lens_host, w.num_q_heads, w.num_kv_heads, w.head_dim, w.page_size,
                         inputs.block_table.shape[1], split_tokens, dev.index or 0, capacity)
        self.workspace = torch.empty(self.plan.workspace_bytes_max, dtype=torch.uint8, device=dev)
        self.out = torch.empty(inputs.q.shape, dtype=torch.float32, device=dev)

    def step(self, inputs, replan: bool = True) -> torch.Tensor:
        if replan:
            self.plan.update(inputs.context_lens_host)
        return paged_decode_attn(self.plan, self.workspace, inputs.q, inputs.k_pages, inputs.v_pages,
                                 inputs.block_table, inputs.context_lens, inputs.scale, self.out)

    def stage(self, inputs, replan: bool = True) -> None:
        """Once per decode step: re-plan and write the descriptors that every layer's `layer` call uses."""
        if replan:
            self.plan.update(inputs.context_lens_host)
        plan_stage(self.plan, self.workspace)

    def layer(self, inputs) -> torch.Tensor:
        """One layer's attention over the staged descriptors."""
        return paged_decode_attn_staged(self.plan, self.workspace, inputs.q, inputs.k_pages, inputs.v_pages,
                                        inputs.block_table, inputs.context_lens, inputs.scale, self.out)


class PrefillPlan:
    """Owns an oserve_prefill_plan_t*.  Mirrors oserve_prefill_plan_* one to one."""

    def __init__(self, context_lens_host, q_lens_host, num_q_heads: int, num_kv_heads: int, head_dim: int,
                 page_size: int, max_pages_per_seq: int, device_id: int = 0, capacity: int | None = None,
                 max_query_tokens: int | None = None):
        lens, qlens = _host_lens(context_lens_host), _host_lens(q_lens_host)
        if lens.shape != qlens.shape:
            raise ValueError("context_lens_host and q_lens_host must have the same length")
        self._h = ctypes.c_void_p()
        self.geometry = (num_q_heads, num_kv_heads, head_dim, page_size, max_pages_per_seq)
        self.batch = len(lens)
        st = lib.oserve_prefill_plan_create(lens.ctypes.data, qlens.ctypes.data, len(lens), num_q_heads, num_kv_heads,
                                            head_dim, page_size, max_pages_per_seq, device_id,
                                            len(lens) if capacity is None else capacity,
                                            int(qlens.sum()) if max_query_tokens is None else max_query_tokens,
                                            ctypes.byref(self._h))
        if st != OK:
            raise OserveError(st, "oserve_prefill_plan_create")

    @property
    def handle(self):
        return self._h

    def update(self, context_lens_host, q_lens_host) -> None:
        lens, qlens = _host_lens(context_lens_host), _host_lens(q_lens_host)
        st = lib.oserve_prefill_plan_update(self._h, lens.ctypes.data, qlens.ctypes.data, len(lens))
        if st != OK:
            raise OserveError(st, "oserve_prefill_plan_update")
        self.batch = len(lens)

    @property
    def num_work_items(self) -> int:
        return lib.oserve_prefill_plan_num_work_items(self._h)

    @property
    def query_tokens(self) -> int:
        return lib.oserve_prefill_plan_query_tokens(self._h)

    @property
    def block_tokens(self) -> int:
        return lib.oserve_prefill_plan_block_tokens(self._h)

    def item(self, i: int) -> dict:
        f = (ctypes.c_int32 * 6)()
        st = lib.oserve_prefill_plan_item(self._h, i, f)
        if st != OK:
            raise OserveError(st, "oserve_prefill_plan_item")
        return dict(zip(("request", "kv_head", "q_begin", "q_row0", "context_len", "q_len"), list(f)))

    def enable_timing(self, enable: bool = True) -> None:
        st = lib.oserve_prefill_plan_enable_timing(self._h, int(enable))
        if st != OK:
            raise OserveError(st, "oserve_prefill_plan_enable_timing")

    def kernel_ms(self):
        ms, n = ctypes.c_float(), ctypes.c_int32()
        st = lib.oserve_prefill_plan_kernel_ms(self._h, ctypes.byref(ms), ctypes.byref(n))
        if st != OK:
            raise OserveError(st, "oserve_prefill_plan_kernel_ms")
        return ms.value, n.value

    def destroy(self) -> None:
        if getattr(self, "_h", None) and self._h.value and lib is not None:
            lib.oserve_prefill_plan_destroy(self._h)
            self._h = ctypes.c_void_p()

    __del__ = destroy


def paged_prefill_attn(plan: PrefillPlan, q: torch.Tensor, k_pages: torch.Tensor, v_pages: torch.Tensor,
                       block_table: torch.Tensor, scale: float, out: torch.Tensor,
                       stream: torch.cuda.Stream | None = None) -> torch.Tensor:
    """oserve_paged_prefill_attn on torch tensors (layout checks only; no arithmetic here)."""
    if not (q.is_cuda and k_pages.is_cuda and v_pages.is_cuda and block_table.is_cuda and out.is_cuda):
        raise ValueError("all tensors must be device tensors")
    if q.dtype != torch.bfloat16 or k_pages.dtype != torch.bfloat16 or v_pages.dtype != torch.bfloat16:
        raise TypeError("q / k_pages / v_pages must be bf16")
    if block_table.dtype != torch.int32 or out.dtype != torch.float32:
        raise TypeError("block_table must be int32 and out fp32")
    for t in (q, k_pages, v_pages, block_table, out):
        if not t.is_contiguous():
            raise ValueError("tensors must be contiguous")
    hq, hkv, d, page, width = plan.geometry
    if tuple(q.shape) != (plan.query_tokens, hq, d) or out.shape != q.shape:
        raise ValueError(f"q / out must be [{plan.query_tokens}, {hq}, {d}] for this plan")
    if k_pages.dim() != 4 or tuple(k_pages.shape[1:]) != (hkv, page, d) or v_pages.shape != k_pages.shape:
        raise ValueError(f"k_pages / v_pages must be [pages, {hkv}, {page}, {d}] for this plan")
    if tuple(block_table.shape) != (plan.batch, width):
        raise ValueError(f"block_table must be [{plan.batch}, {width}] for this plan")
    s = torch.cuda.current_stream(q.device) if stream is None else stream
    st = lib.oserve_paged_prefill_attn(plan.handle, _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table),
                                       ctypes.c_float(scale), _ptr(out), ctypes.c_void_p(s.cuda_stream))
    if st != OK:
        raise OserveError(st, "oserve_paged_prefill_attn")
    return out


class MixedPlan:
    """Owns an oserve_mixed_plan_t*.  Mirrors oserve_mixed_plan_* one to one."""

    def __init__(self, context_lens_host, q_lens_host, num_q_heads: int, num_kv_heads: int, head_dim: int,
                 page_size: int, max_pages_per_seq: int, device_id: int = 0, capacity: int | None = None,
                 max_query_tokens: int | None = None):
        lens, qlens = _host_lens(context_lens_host), _host_lens(q_lens_host)
        if lens.shape != qlens.shape:
            raise ValueError("context_lens_host and q_lens_host must have the same length")
        self._h = ctypes.c_void_p()
        self.geometry = (num_q_heads, num_kv_heads, head_dim, page_size, max_pages_per_seq)
        self.batch = len(lens)
        st = lib.oserve_mixed_plan_create(lens.ctypes.data, qlens.ctypes.data, len(lens), num_q_heads, num_kv_heads,
                                          head_dim, page_size, max_pages_per_seq, device_id,
                                          len(lens) if capacity is None else capacity,
                                          int(qlens.sum()) if max_query_tokens is None else max_query_tokens,
                                          ctypes.byref(self._h))
        if st != OK:
            self._h = ctypes.c_void_p()
            raise OserveError(st, "oserve_mixed_plan_create")

    @property
    def handle(self):
        return self._h

    def update(self, context_lens_host, q_lens_host) -> None:
        lens, qlens = _host_lens(context_lens_host), _host_lens(q_lens_host)
        st = lib.oserve_mixed_plan_update(self._h, lens.ctypes.data, qlens.ctypes.data, len(lens))
        if st != OK:
            raise OserveError(st, "oserve_mixed_plan_update")
        self.batch = len(lens)

    @property
    def query_tokens(self) -> int:
        return lib.oserve_mixed_plan_query_tokens(self._h)

    @property
    def counts(self) -> dict:
        c = (ctypes.c_int32 * 4)()
        st = lib.oserve_mixed_plan_counts(self._h, c)
        if st != OK:
            raise OserveError(st, "oserve_mixed_plan_counts")
        return dict(zip(("workgroups", "prefill_items", "decode_items", "prefill_queues"), list(c)))

    def prefill_item(self, i: int) -> dict:
        f = (ctypes.c_int32 * 7)()
        st = lib.oserve_mixed_plan_prefill_item(self._h, i, f)
        if st != OK:
            raise OserveError(st, "oserve_mixed_plan_prefill_item")
        return dict(zip(("queue", "request", "kv_head", "q_begin", "q_row0", "context_len", "q_len"), list(f)))

    @property
    def workspace_bytes(self) -> int:
        return lib.oserve_mixed_plan_workspace_bytes(self._h)

    @property
    def workspace_bytes_max(self) -> int:
        return lib.oserve_mixed_plan_workspace_bytes_max(self._h)

    def enable_timing(self, enable: bool = True) -> None:
        st = lib.oserve_mixed_plan_enable_timing(self._h, int(enable))
        if st != OK:
            raise OserveError(st, "oserve_mixed_plan_enable_timing")

    def kernel_ms(self):
        ms, n = ctypes.c_float(), ctypes.c_int32()
        st = lib.oserve_mixed_plan_kernel_ms(self._h, ctypes.byref(ms), ctypes.byref(n))
        if st != OK:
            raise OserveError(st, "oserve_mixed_plan_kernel_ms")
        return ms.value, n.value

    def destroy(self) -> None:
        if getattr(self, "_h", None) and self._h.value and lib is not None:
            lib.oserve_mixed_plan_destroy(self._h)
            self._h = ctypes.c_void_p()

    __del__ = destroy


def paged_mixed_attn(plan: MixedPlan, workspace: torch.Tensor, q: torch.Tensor, k_pages: torch.Tensor,
                     v_pages: torch.Tensor, block_table: torch.Tensor, context_lens: torch.Tensor, scale: float,
                     out: torch.Tensor, stream: torch.cuda.Stream | None = None) -> torch.Tensor:
    """oserve_paged_mixed_attn on torch tensors (layout checks only; no arithmetic here)."""
    tensors = (workspace, q, k_pages, v_pages, block_table, context_lens, out)
    if not all(t.is_cuda and t.is_contiguous() for t in tensors):
        raise ValueError("all tensors must be contiguous device tensors")
    if q.dtype != torch.bfloat16 or k_pages.dtype != torch.bfloat16 or v_pages.dtype != torch.bfloat16:
        raise TypeError("q / k_pages / v_pages must be bf16")
    if block_table.dtype != torch.int32 or context_lens.dtype != torch.int32 or out.dtype != torch.float32:
        raise TypeError("block_table / context_lens must be int32 and out fp32")
    hq, hkv, d, page, width = plan.geometry
    if tuple(q.shape) != (plan.query_tokens, hq, d) or out.shape != q.shape:
        raise ValueError(f"q / out must be [{plan.query_tokens}, {hq}, {d}] for this plan")
    if k_pages.dim() != 4 or tuple(k_pages.shape[1:]) != (hkv, page, d) or v_pages.shape != k_pages.shape:
        raise ValueError(f"k_pages / v_pages must be [pages, {hkv}, {page}, {d}] for this plan")
    if tuple(block_table.shape) != (plan.batch, width) or tuple(context_lens.shape) != (plan.batch,):
        raise ValueError(f"block_table / context_lens must be [{plan.batch}, {width}] / [{plan.batch}] for this plan")
    s = torch.cuda.current_stream(q.device) if stream is None else stream
    st = lib.oserve_paged_mixed_attn(plan.handle, _ptr(workspace), workspace.numel() * workspace.element_size(),
                                     _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table), _ptr(context_lens),
                                     ctypes.c_float(scale), _ptr(out), ctypes.c_void_p(s.cuda_stream))
    if st != OK:
        raise OserveError(st, "oserve_paged_mixed_attn")
    return out


class KvMigration:
    """Owns an oserve_kv_migration_t*.  Mirrors oserve_kv_migration_* / oserve_kv_gather / oserve_kv_scatter."""

    def __init__(self, context_lens_host, table_rows_host, page_size: int, device_id: int = 0):
        lens, rows = _host_lens(context_lens_host), _host_lens(table_rows_host)
        if lens.shape != rows.shape:
            raise ValueError("context_lens_host and table_rows_host must have the same length")
        self._h = ctypes.c_void_p()
        st = lib.oserve_kv_migration_create(lens.ctypes.data, rows.ctypes.data, len(lens), page_size, device_id,
                                            ctypes.byref(self._h))
        if st != OK:
            self._h = ctypes.c_void_p()
            raise OserveError(st, "oserve_kv_migration_create")

    @property
    def num_pages(self) -> int:
        return lib.oserve_kv_migration_num_pages(self._h)

    def request(self, r: int):
        a, b = ctypes.c_int32(), ctypes.c_int32()
        st = lib.oserve_kv_migration_request(self._h, r, ctypes.byref(a), ctypes.byref(b))
        if st != OK:
            raise OserveError(st, "oserve_kv_migration_request")
        return a.value, b.value

    def _run(self, fn, name, a_k, a_v, table, pool_heads, head_begin, num_heads, head_dim, b_k, b_v, stream):
        for t in (a_k, a_v, b_k, b_v, table):
            if not (t.is_cuda and t.is_contiguous()):
                raise ValueError("tensors must be contiguous device tensors")
        if table.dtype != torch.int32:
            raise TypeError("block table must be int32")
        s = torch.cuda.current_stream(a_k.device) if stream is None else stream
        st = fn(self._h, _ptr(a_k), _ptr(a_v), _ptr(table), table.shape[1], pool_heads, head_begin, num_heads,
                head_dim, _ptr(b_k), _ptr(b_v), ctypes.c_void_p(s.cuda_stream))
        if st != OK:
            raise OserveError(st, name)

    def gather(self, k_pool, v_pool, block_table, head_begin: int, num_heads: int, k_stage, v_stage, stream=None):
        if k_stage.shape != (self.num_pages, num_heads) + tuple(k_pool.shape[2:]) or v_stage.shape != k_stage.shape:
            raise ValueError("staging chunk must be [num_pages, num_heads, page_size, head_dim]")
        self._run(lib.oserve_kv_gather, "oserve_kv_gather", k_pool, v_pool, block_table, k_pool.shape[1],
                  head_begin, num_heads, k_pool.shape[3], k_stage, v_stage, stream)

    def scatter(self, k_stage, v_stage, target_block_table, head_begin: int, k_pool, v_pool, stream=None):
        if k_stage.shape[0] != self.num_pages or tuple(k_stage.shape[2:]) != tuple(k_pool.shape[2:]):
            raise ValueError("staging chunk does not match the plan or the pool")
        self._run(lib.oserve_kv_scatter, "oserve_kv_scatter", k_stage, v_stage, target_block_table,
                  k_pool.shape[1], head_begin, k_stage.shape[1], k_pool.shape[3], k_pool, v_pool, stream)

    def enable_timing(self, enable: bool = True) -> None:
        st = lib.oserve_kv_migration_enable_timing(self._h, int(enable))
        if st != OK:
            raise OserveError(st, "oserve_kv_migration_enable_timing")

    def kernel_ms(self):
        ms, n = ctypes.c_float(), ctypes.c_int32()
        st = lib.oserve_kv_migration_kernel_ms(self._h, ctypes.byref(ms), ctypes.byref(n))
        if st != OK:
            raise OserveError(st, "oserve_kv_migration_kernel_ms")
        return ms.value, n.value

    def destroy(self) -> None:
        if getattr(self, "_h", None) and self._h.value and lib is not None:
            lib.oserve_kv_migration_destroy(self._h)
            self._h = ctypes.c_void_p()

    __del__ = destroy


def switch_plan(device_machine, sources, targets, volumes):
    """oserve_switch_plan on Python lists: sources[m] / targets[m] list the devices holding / needing shard m,
    volumes[m][i] is the volume of (m, targets[m][i]).  Returns (chosen sources per shard, pair-load matrix)."""
    dm = np.ascontiguousarray(device_machine, dtype=np.int32)
    so = np.zeros(len(sources) + 1, dtype=np.int32)
    to = np.zeros(len(targets) + 1, dtype=np.int32)
    so[1:] = np.cumsum([len(x) for x in sources])
    to[1:] = np.cumsum([len(x) for x in targets])
    sd = np.ascontiguousarray([d for x in sources for d in x], dtype=np.int32)
    td = np.ascontiguousarray([d for x in targets for d in x], dtype=np.int32)
    vol = np.ascontiguousarray([v for x in volumes for v in x], dtype=np.int64)
    if len(vol) != len(td):
        raise ValueError("volumes must align with targets")
    chosen = np.full(max(len(td), 1), -2, dtype=np.int32)
    load = np.zeros((len(dm), len(dm)), dtype=np.int64)
    pad = np.zeros(1, dtype=np.int32)
    st = lib.oserve_switch_plan(len(dm), dm.ctypes.data, len(sources), so.ctypes.data,
                                (sd if len(sd) else pad).ctypes.data, to.ctypes.data,
                                (td if len(td) else pad).ctypes.data,
                                (vol if len(vol) else np.zeros(1, dtype=np.int64)).ctypes.data,
                                chosen.ctypes.data, load.ctypes.data)
    if st != OK:
        raise OserveError(st, "oserve_switch_plan")
    return [list(map(int, chosen[to[m]:to[m + 1]])) for m in range(len(targets))], load


def capacity_normalise(per_type_capacity):
    n = np.ascontiguousarray(per_type_capacity, dtype=np.int64)
    m = ctypes.c_int64()
    units = np.zeros(len(n), dtype=np.int64)
    st = lib.oserve_capacity_normalise(n.ctypes.data, len(n), ctypes.byref(m), units.ctypes.data)
    if st != OK:
        raise OserveError(st, "oserve_capacity_normalise")
    return m.value, [int(u) for u in units]


def assign_workload(arrivals, node_capacity, edge_capacity=None):
    """oserve_assign_workload: returns (total requests served, assignment [replicas, types])."""
    lam = np.ascontiguousarray(arrivals, dtype=np.float64)
    n = np.ascontiguousarray(node_capacity, dtype=np.int64)
    if n.ndim != 2 or n.shape[1] != len(lam):
        raise ValueError("node_capacity must be [replicas, types]")
    e = None if edge_capacity is None else np.ascontiguousarray(edge_capacity, dtype=np.float64)
    if e is not None and e.shape != n.shape:
        raise ValueError("edge_capacity must match node_capacity")
    x = np.zeros(n.shape, dtype=np.float64)
    total = ctypes.c_double()
    st = lib.oserve_assign_workload(n.shape[0], n.shape[1], lam.ctypes.data, n.ctypes.data,
                                    None if e is None else e.ctypes.data, x.ctypes.data, ctypes.byref(total))
    if st != OK:
        raise OserveError(st, "oserve_assign_workload")
    return total.value, x
