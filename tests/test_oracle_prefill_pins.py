"""Pins of the causal (chunked-prefill) form of the fp64 oracle.

The operation is the same scaled-dot-product attention (paper section 2), with
several query tokens per request, each seeing the cached tokens up to its own
position.  It is pinned against the decode oracle (itself pinned in
test_oracle_pins.py), against an independent dense masked softmax in numpy long
doubles, and by closed forms and invariants.
"""
import numpy as np
import pytest
import torch

from oracle import paged_attention_oracle as oracle
from tests.test_oracle_pins import as_f64, bf16, paged_from_dense


def rand_prefill_case(seed, lens, qlens, Hq, Hkv, D, page=16):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(int(sum(qlens)), Hq, D, generator=g).to(torch.bfloat16)
    kd = [as_f64(torch.randn(L, Hkv, D, generator=g).to(torch.bfloat16)) for L in lens]
    vd = [as_f64(torch.randn(L, Hkv, D, generator=g).to(torch.bfloat16)) for L in lens]
    kp, vp, bt, cl = paged_from_dense(kd, vd, lens, page=page, seed=seed)
    return q, kd, vd, kp, vp, bt, cl, np.asarray(qlens, dtype=np.int32)


def dense_causal_reference(q, kd, vd, lens, qlens, scale_f32, group):
    """softmax(mask(q K^T scale)) V with an explicit lower-triangular mask, long double, no max subtraction."""
    ld = np.longdouble
    T, Hq, D = q.shape
    out = np.zeros((T, Hq, D))
    row0 = 0
    for b, (L, n) in enumerate(zip(lens, qlens)):
        pos = np.arange(L - n, L)                                  # positions of the n queries
        mask = np.arange(L)[None, :] <= pos[:, None]               # [n, L]
        for h in range(Hq):
            j = h // group
            K = kd[b][:, j, :].astype(ld)
            V = vd[b][:, j, :].astype(ld)
            Q = q[row0:row0 + n, h, :].astype(ld)
            e = np.exp((Q @ K.T) * ld(np.float32(scale_f32))) * mask
            out[row0:row0 + n, h, :] = ((e @ V) / e.sum(axis=1, keepdims=True)).astype(np.float64)
        row0 += n
    return out


@pytest.mark.parametrize("seed,lens,qlens,Hq,Hkv,D", [
    (1, [5, 40, 17], [5, 7, 1], 4, 2, 8),
    (2, [70, 16, 33], [33, 16, 2], 8, 2, 64),
    (3, [1, 2, 64], [1, 1, 64], 2, 2, 8),
])
def test_matches_dense_masked_bruteforce(seed, lens, qlens, Hq, Hkv, D):
    q, kd, vd, kp, vp, bt, cl, ql = rand_prefill_case(seed, lens, qlens, Hq, Hkv, D)
    scale = float(np.float32(1.0 / np.sqrt(D)))
    out = oracle.paged_prefill_attn(q, kp, vp, bt, cl, ql, scale)
    ref = dense_causal_reference(as_f64(q), kd, vd, lens, qlens, scale, Hq // Hkv)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)


def test_one_query_per_request_is_the_decode_oracle_bit_for_bit():
    lens = [9, 100, 31]
    q, kd, vd, kp, vp, bt, cl, ql = rand_prefill_case(4, lens, [1, 1, 1], 8, 2, 16)
    out = oracle.paged_prefill_attn(q, kp, vp, bt, cl, ql, 0.25)
    ref = oracle.paged_decode_attn(q, kp, vp, bt, cl, 0.25)
    assert np.array_equal(out, ref)


def test_each_row_is_decode_attention_on_the_context_cut_after_it():
    """Row i of a chunk equals the (pinned) decode oracle with context length p_i + 1."""
    lens, qlens = [50, 23], [20, 23]
    q, kd, vd, kp, vp, bt, cl, ql = rand_prefill_case(5, lens, qlens, 4, 2, 16)
    out = oracle.paged_prefill_attn(q, kp, vp, bt, cl, ql, 0.3)
    row = 0
    for b, (L, n) in enumerate(zip(lens, qlens)):
        for i in range(n):
            cut = cl.copy()
            cut[b] = L - n + i + 1
            # a one-request-wide decode batch whose request b holds this query row
            qb = torch.zeros(len(lens), 4, 16, dtype=torch.bfloat16)
            qb[b] = q[row]
            ref = oracle.paged_decode_attn(qb, kp, vp, bt, cut, 0.3)
            assert np.array_equal(out[row], ref[b])
            row += 1


def test_first_token_of_a_whole_prompt_returns_v0():
    lens = [37]
    q, kd, vd, kp, vp, bt, cl, ql = rand_prefill_case(6, lens, [37], 4, 4, 8)
    out = oracle.paged_prefill_attn(q, kp, vp, bt, cl, ql, 1.0)
    for h in range(4):
        assert np.array_equal(out[0, h], vd[0][0, h, :])


def test_a_later_token_changes_no_earlier_row():
    lens, qlens = [40], [12]
    q, kd, vd, kp, vp, bt, cl, ql = rand_prefill_case(7, lens, qlens, 2, 1, 8)
    base = oracle.paged_prefill_attn(q, kp, vp, bt, cl, ql, 0.5)
    kd2 = [kd[0].copy()]; vd2 = [vd[0].copy()]
    kd2[0][39] += 3.0; vd2[0][39] -= 5.0          # the last token: visible to the last query only
    kp2, vp2, bt2, cl2 = paged_from_dense(kd2, vd2, lens, page=16, seed=7)
    out = oracle.paged_prefill_attn(q, kp2, vp2, bt2, cl2, ql, 0.5)
    assert np.array_equal(out[:11], base[:11])
    assert not np.array_equal(out[11], base[11])


def test_equal_keys_give_running_means_of_v():
    """All keys equal: query i sees a uniform softmax over tokens 0..p_i, i.e. the running mean of V."""
    L, n = 20, 20
    kd = [np.tile(np.array([[[0.5, -1.0]]]), (L, 1, 1))]
    vd = [np.arange(L, dtype=np.float64).reshape(L, 1, 1) * np.ones((1, 1, 2))]
    kp, vp, bt, cl = paged_from_dense(kd, vd, [L], page=16)
    q = bf16(np.ones((n, 1, 2)))
    out = oracle.paged_prefill_attn(q, kp, vp, bt, cl, np.array([n], dtype=np.int32), 0.7)
    for i in range(n):
        np.testing.assert_allclose(out[i, 0], [i / 2.0, i / 2.0], rtol=1e-14, atol=1e-14)


def test_rejects_bad_lengths():
    q, kd, vd, kp, vp, bt, cl, ql = rand_prefill_case(8, [10], [4], 2, 1, 8)
    with pytest.raises(ValueError):
        oracle.paged_prefill_attn(q, kp, vp, bt, cl, np.array([11], dtype=np.int32), 1.0)   # rows != sum
    q11 = torch.zeros(11, 2, 8, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        oracle.paged_prefill_attn(q11, kp, vp, bt, cl, np.array([11], dtype=np.int32), 1.0)  # n > L
