"""Pins of the fp64 CPU oracle against what the mathematics fixes.

The paper gives no worked numeric example of attention (it only cites the
scaled-dot-product definition in section 2, "Phases of LLM inference"), so the
oracle is pinned by closed forms, invariants and an independent dense
brute-force evaluation written here with numpy long doubles.  Each test is
chosen so that one plausible mistake in the oracle (dropped scale, wrong sign,
wrong head map, wrong page/slot index, transposed operand, reading masked
slots) fails it.
"""
import math

import numpy as np
import pytest
import torch

from oracle import paged_attention_oracle as oracle
from paper_2602_12151_amd import workloads as wl


# ----------------------------------------------------------------------------
# helpers (input construction only)
# ----------------------------------------------------------------------------
def bf16(x) -> torch.Tensor:
    return torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16)


def as_f64(t: torch.Tensor) -> np.ndarray:
    return t.to(torch.float64).numpy()


def paged_from_dense(k_dense, v_dense, lens, page=16, pool_extra=3, seed=0, fill=0.0):
    """Scatter dense per-request K/V ([B][L_b, Hkv, D] lists) into a permuted page pool."""
    B = len(lens)
    Hkv, D = k_dense[0].shape[1], k_dense[0].shape[2]
    n = [(L + page - 1) // page for L in lens]
    total = sum(n)
    npool = total + pool_extra
    perm = wl.CounterRng(seed).permutation(npool)
    kp = np.full((npool, Hkv, page, D), fill, dtype=np.float32)
    vp = np.full((npool, Hkv, page, D), fill, dtype=np.float32)
    bt = np.full((B, max(n)), -1, dtype=np.int32)
    off = 0
    for b in range(B):
        for p in range(n[b]):
            pid = perm[off]
            off += 1
            bt[b, p] = pid
            t0, t1 = p * page, min(lens[b], (p + 1) * page)
            kp[pid, :, : t1 - t0, :] = np.transpose(k_dense[b][t0:t1], (1, 0, 2))
            vp[pid, :, : t1 - t0, :] = np.transpose(v_dense[b][t0:t1], (1, 0, 2))
    return bf16(kp), bf16(vp), bt, np.asarray(lens, dtype=np.int32)


def dense_reference(q, k_dense, v_dense, scale_f32, group):
    """Unpaged softmax(q K^T scale) V in long double, written independently of the oracle.

    q: [B, Hq, D] float64 (exact bf16 values); k_dense/v_dense: lists of [L, Hkv, D].
    Uses the exp-normalise form without max subtraction (inputs are small), so it
    shares no structure with the oracle's two-pass loop.
    """
    B, Hq, D = q.shape
    out = np.zeros((B, Hq, D), dtype=np.float64)
    ld = np.longdouble
    for b in range(B):
        for h in range(Hq):
            j = h // group
            K = k_dense[b][:, j, :].astype(ld)      # [L, D]
            V = v_dense[b][:, j, :].astype(ld)
            s = (K @ q[b, h].astype(ld)) * ld(np.float32(scale_f32))
            e = np.exp(s)
            out[b, h] = ((e[:, None] * V).sum(axis=0) / e.sum()).astype(np.float64)
    return out


def rand_case(seed, lens, Hq, Hkv, D, amp=1.0):
    g = torch.Generator().manual_seed(seed)
    B = len(lens)
    q = (torch.randn(B, Hq, D, generator=g) * amp).to(torch.bfloat16)
    kd = [as_f64((torch.randn(L, Hkv, D, generator=g) * amp).to(torch.bfloat16)) for L in lens]
    vd = [as_f64(torch.randn(L, Hkv, D, generator=g).to(torch.bfloat16)) for L in lens]
    return q, kd, vd


# ----------------------------------------------------------------------------
# closed forms
# ----------------------------------------------------------------------------
def test_two_token_closed_form():
    """q=(1,0), keys (0,0),(1,0), values e_0,e_1: out = (1, e^s)/(1+e^s) with s = scale."""
    for scale, k1 in [(1.0, 1.0), (0.5, 1.0), (1.0, -1.0), (0.25, 2.0)]:
        q = bf16([[[1.0, 0.0]]])
        kd = [np.array([[[0.0, 0.0]], [[k1, 0.0]]])]
        vd = [np.array([[[1.0, 0.0]], [[0.0, 1.0]]])]
        kp, vp, bt, cl = paged_from_dense(kd, vd, [2], page=16)
        out = oracle.paged_decode_attn(q, kp, vp, bt, cl, scale)
        s = scale * k1
        expect = np.array([1.0, math.exp(s)]) / (1.0 + math.exp(s))
        np.testing.assert_allclose(out[0, 0], expect, rtol=0, atol=2e-16)


def test_length_one_returns_v_exactly():
    q, kd, vd = rand_case(1, [1, 1, 1], Hq=8, Hkv=2, D=64)
    kp, vp, bt, cl = paged_from_dense(kd, vd, [1, 1, 1])
    out = oracle.paged_decode_attn(q, kp, vp, bt, cl, 0.125)
    for b in range(3):
        for h in range(8):
            assert np.array_equal(out[b, h], vd[b][0, h // 4])  # bit-exact, also pins the head map


def test_identical_keys_give_mean_of_v():
    lens = [37, 5]
    q, kd, vd = rand_case(2, lens, Hq=4, Hkv=2, D=32)
    for b in range(2):
        kd[b][:] = kd[b][0:1]
    kp, vp, bt, cl = paged_from_dense(kd, vd, lens)
    out = oracle.paged_decode_attn(q, kp, vp, bt, cl, 0.3)
    for b in range(2):
        for h in range(4):
            np.testing.assert_allclose(out[b, h], vd[b][:, h // 2].mean(axis=0), rtol=0, atol=1e-14)


@pytest.mark.parametrize("which", ["q_zero", "scale_zero"])
def test_zero_scores_give_mean_of_v(which):
    lens = [50]
    q, kd, vd = rand_case(3, lens, Hq=2, Hkv=1, D=16)
    scale = 0.25
    if which == "q_zero":
        q = torch.zeros_like(q)
    else:
        scale = 0.0
    kp, vp, bt, cl = paged_from_dense(kd, vd, lens)
    out = oracle.paged_decode_attn(q, kp, vp, bt, cl, scale)
    np.testing.assert_allclose(out[0, 0], vd[0][:, 0].mean(axis=0), rtol=0, atol=1e-14)


def test_constant_v_is_returned():
    lens = [97]
    q, kd, vd = rand_case(4, lens, Hq=2, Hkv=2, D=16)
    vd[0][:] = 0.75
    kp, vp, bt, cl = paged_from_dense(kd, vd, lens)
    out = oracle.paged_decode_attn(q, kp, vp, bt, cl, 0.25)
    np.testing.assert_allclose(out, 0.75, rtol=0, atol=1e-15)


def test_dominant_key_selects_its_value_and_no_overflow():
    """One key aligned with q at |s| ~ 80+: softmax collapses onto it; max subtraction keeps it finite."""
    D, L, t_star = 16, 40, 23
    q = bf16(np.full((1, 1, D), 4.0))
    kd = [np.zeros((L, 1, D))]
    kd[0][t_star, 0, :] = 6.0          # s = 0.25 * 16 * 24 = 96
    kd[0][5, 0, :] = -6.0              # s = -96
    g = torch.Generator().manual_seed(5)
    vd = [as_f64(torch.randn(L, 1, D, generator=g).to(torch.bfloat16))]
    kp, vp, bt, cl = paged_from_dense(kd, vd, [L])
    out, lse = oracle.paged_decode_attn(q, kp, vp, bt, cl, 0.25, return_lse=True)
    assert np.all(np.isfinite(out))
    np.testing.assert_allclose(out[0, 0], vd[0][t_star, 0], rtol=0, atol=1e-30 + 38 * math.exp(-96) * 5)
    np.testing.assert_allclose(lse[0, 0], 96.0, rtol=0, atol=1e-12)


def test_duplicating_the_sequence_changes_nothing():
    L = 45
    q, kd, vd = rand_case(6, [L], Hq=4, Hkv=2, D=32)
    kd2 = [np.concatenate([kd[0], kd[0]])]
    vd2 = [np.concatenate([vd[0], vd[0]])]
    a = oracle.paged_decode_attn(q, *paged_from_dense(kd, vd, [L]), 0.2)
    b = oracle.paged_decode_attn(q, *paged_from_dense(kd2, vd2, [2 * L]), 0.2)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-14)


def test_gqa_heads_with_equal_q_agree_and_groups_differ():
    lens = [33]
    q, kd, vd = rand_case(7, lens, Hq=8, Hkv=2, D=32)
    q[:, 1:4] = q[:, 0:1]      # heads 0..3 share kv head 0
    q[:, 4] = q[:, 0]          # head 4 uses kv head 1: same q, different K/V
    kp, vp, bt, cl = paged_from_dense(kd, vd, lens)
    out = oracle.paged_decode_attn(q, kp, vp, bt, cl, 0.2)
    for h in (1, 2, 3):
        assert np.array_equal(out[0, h], out[0, 0])
    assert not np.allclose(out[0, 4], out[0, 0])


# ----------------------------------------------------------------------------
# invariants of the paged layout
# ----------------------------------------------------------------------------
def test_page_permutation_is_bit_invariant():
    lens = [17, 64, 200, 513]
    q, kd, vd = rand_case(8, lens, Hq=8, Hkv=2, D=64)
    a = oracle.paged_decode_attn(q, *paged_from_dense(kd, vd, lens, seed=1), 0.125)
    b = oracle.paged_decode_attn(q, *paged_from_dense(kd, vd, lens, seed=2, pool_extra=11), 0.125)
    assert np.array_equal(a, b)


def test_unread_slots_and_pages_do_not_matter():
    """NaN in tail slots of last pages, in unused pool pages, and -1 table padding."""
    lens = [1, 15, 16, 17, 31, 33]
    q, kd, vd = rand_case(9, lens, Hq=4, Hkv=2, D=32)
    clean = oracle.paged_decode_attn(q, *paged_from_dense(kd, vd, lens, seed=3, fill=0.0), 0.2)
    kp, vp, bt, cl = paged_from_dense(kd, vd, lens, seed=3, fill=float("nan"))
    assert torch.isnan(kp).any() and (bt == -1).any()
    poisoned = oracle.paged_decode_attn(q, kp, vp, bt, cl, 0.2)
    assert np.array_equal(clean, poisoned)


def test_strided_layout_is_honoured():
    """Same values under a [page, tok, head, dim] memory order must give the same bits."""
    lens = [40, 9]
    q, kd, vd = rand_case(10, lens, Hq=4, Hkv=2, D=32)
    kp, vp, bt, cl = paged_from_dense(kd, vd, lens)
    a = oracle.paged_decode_attn(q, kp, vp, bt, cl, 0.2)
    kp2 = kp.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)   # same logical shape, other strides
    vp2 = vp.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert kp2.stride() != kp.stride()
    b = oracle.paged_decode_attn(q, kp2, vp2, bt, cl, 0.2)
    assert np.array_equal(a, b)


# ----------------------------------------------------------------------------
# brute force against a dense, unpaged evaluation
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("seed,lens,Hq,Hkv,D", [
    (11, [1, 2, 3, 70], 4, 2, 8),
    (12, [16, 17, 48, 5], 8, 2, 64),
    (13, [33], 6, 1, 16),       # one kv head shared by six query heads
    (14, [29, 64], 3, 3, 8),    # MHA: group 1
])
def test_matches_dense_bruteforce(seed, lens, Hq, Hkv, D):
    q, kd, vd = rand_case(seed, lens, Hq, Hkv, D)
    scale = float(np.float32(1.0 / math.sqrt(D)))
    kp, vp, bt, cl = paged_from_dense(kd, vd, lens, seed=seed)
    out = oracle.paged_decode_attn(q, kp, vp, bt, cl, scale)
    ref = dense_reference(as_f64(q), kd, vd, scale, Hq // Hkv)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)


def test_tiny_workload_matches_dense_bruteforce():
    """Workload 0 exactly as the generator draws it (lens 17, 64, 200, 513; 8q/2kv; D=64)."""
    w = wl.WORKLOADS[0]
    inp = wl.make_inputs(w, device="cpu")
    assert list(inp.context_lens_host) == [17, 64, 200, 513]
    assert inp.k_pages.shape == (64, 2, 16, 64)
    out = oracle.paged_decode_attn(inp.q, inp.k_pages, inp.v_pages, inp.block_table,
                                   inp.context_lens, inp.scale)
    # dense gather written with plain indexing
    bt = inp.block_table.numpy()
    kd, vd = [], []
    for b, L in enumerate(inp.context_lens_host):
        rows_k = [as_f64(inp.k_pages[bt[b, t // 16], :, t % 16, :]) for t in range(L)]
        rows_v = [as_f64(inp.v_pages[bt[b, t // 16], :, t % 16, :]) for t in range(L)]
        kd.append(np.stack(rows_k))
        vd.append(np.stack(rows_v))
    ref = dense_reference(as_f64(inp.q), kd, vd, inp.scale, w.group)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)


def test_row_api_equals_batch_api():
    lens = [20, 45]
    q, kd, vd = rand_case(15, lens, Hq=4, Hkv=2, D=32)
    kp, vp, bt, cl = paged_from_dense(kd, vd, lens)
    full = oracle.paged_decode_attn(q, kp, vp, bt, cl, 0.2)
    for b in range(2):
        for h in range(4):
            assert np.array_equal(oracle.one_head(q, kp, vp, bt, cl, 0.2, b, h), full[b, h])


# ----------------------------------------------------------------------------
# the split / log-sum-exp merge identity the GPU path relies on
# ----------------------------------------------------------------------------
def test_merge_of_parts_by_lse_equals_unsplit():
    """Cut a sequence at page boundaries, run the oracle on each part, merge by lse."""
    L, page = 301, 16
    q, kd, vd = rand_case(16, [L], Hq=4, Hkv=2, D=32)
    kp, vp, bt, cl = paged_from_dense(kd, vd, [L])
    whole = oracle.paged_decode_attn(q, kp, vp, bt, cl, 0.3)
    cuts = [0, 3, 4, 11, 19]                       # page indices; last part ragged
    parts_bt, parts_len = [], []
    for a, b in zip(cuts[:-1], cuts[1:]):
        row = np.full((bt.shape[1],), -1, dtype=np.int32)
        row[: b - a] = bt[0, a:b]
        parts_bt.append(row)
        parts_len.append(min(L, b * page) - a * page)
    pbt = np.stack(parts_bt)
    pcl = np.asarray(parts_len, dtype=np.int32)
    assert pcl.sum() == L
    qrep = q.expand(len(pcl), -1, -1).contiguous()
    o, lse = oracle.paged_decode_attn(qrep, kp, vp, pbt, pcl, 0.3, return_lse=True)
    m = lse.max(axis=0, keepdims=True)
    wgt = np.exp(lse - m)                                   # [S, Hq]
    merged = (wgt[:, :, None] * o).sum(axis=0) / wgt.sum(axis=0)[:, None]
    np.testing.assert_allclose(merged, whole[0], rtol=0, atol=1e-14)


# ----------------------------------------------------------------------------
# error behaviour
# ----------------------------------------------------------------------------
def test_rejects_zero_length_and_bad_table():
    q, kd, vd = rand_case(17, [5], Hq=2, Hkv=1, D=8)
    kp, vp, bt, cl = paged_from_dense(kd, vd, [5])
    with pytest.raises(ValueError):
        oracle.paged_decode_attn(q, kp, vp, bt, np.array([0], dtype=np.int32), 1.0)
    bad = bt.copy()
    bad[0, 0] = kp.shape[0]
    with pytest.raises(ValueError):
        oracle.paged_decode_attn(q, kp, vp, bad, cl, 1.0)
