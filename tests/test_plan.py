"""Host-side split planning through the C ABI (no GPU): every page of every request is covered by
exactly one split, the launch order is longest-first, sizes and bounds are consistent."""
import numpy as np
import pytest

from paper_2602_12151_amd import binding, workloads as wl


def make_plan(lens, hq=32, hkv=8, d=128, split_tokens=0, capacity=None, page_size=16):
    lens = np.asarray(lens, dtype=np.int32)
    width = int(wl.pages_needed(lens, page_size).max())
    return binding.Plan(lens, hq, hkv, d, page_size, width, split_tokens, -1, capacity)


def check_plan(plan, lens, hkv):
    need = wl.pages_needed(np.asarray(lens))
    runs = [plan.run(i) for i in range(plan.num_runs)]
    covered = [np.zeros(n, dtype=np.int32) for n in need]
    items = 0
    prev_size = None
    rows_seen = set()
    for r in runs:
        b = r["request"]
        assert r["first_item"] == items
        items += r["num_splits"] * hkv
        assert r["num_splits"] >= 1 and r["pages_per_split"] >= 1
        assert 0 <= r["page_begin"] < r["page_end"] <= need[b]
        # all splits of a run are non-empty and only the last one may be short
        span = r["page_end"] - r["page_begin"]
        assert (r["num_splits"] - 1) * r["pages_per_split"] < span <= r["num_splits"] * r["pages_per_split"]
        covered[b][r["page_begin"]:r["page_end"]] += 1
        if prev_size is not None:
            assert r["pages_per_split"] <= prev_size          # longest first
        prev_size = r["pages_per_split"]
        assert r["pages_per_split"] <= plan.split_pages
        assert r["total_splits"] == plan.request(b)[0]
        for s in range(r["num_splits"]):
            row = r["row_base"] + s
            assert row not in rows_seen
            rows_seen.add(row)
    assert items == plan.num_work_items
    assert plan.split_tokens == 16 * plan.split_pages
    for b in range(len(lens)):
        mine = [min(r["pages_per_split"], r["page_end"] - r["page_begin"]) for r in runs if r["request"] == b]
        assert plan.request(b)[1] == max(mine)          # the request's own largest split
    for c in covered:
        assert (c == 1).all()
    total_splits = sum(plan.request(b)[0] for b in range(len(lens)))
    assert rows_seen == set(range(total_splits))
    assert plan.workspace_bytes <= plan.workspace_bytes_max


@pytest.mark.parametrize("idx", [0, 1, 2, 3, 4])
def test_automatic_plan_covers_every_page_once(idx):
    w = wl.WORKLOADS[idx]
    lens = wl.context_lens(w)
    plan = make_plan(lens, w.num_q_heads, w.num_kv_heads, w.head_dim)
    check_plan(plan, lens, w.num_kv_heads)
    assert plan.split_pages % 12 == 0


@pytest.mark.parametrize("split_tokens", [16, 48, 64, 256, 1024, 4096])
def test_explicit_split_size(split_tokens):
    lens = [1, 15, 16, 17, 255, 256, 257, 1000, 4097, 33000]
    plan = make_plan(lens, split_tokens=split_tokens)
    check_plan(plan, lens, 8)
    assert plan.split_pages == split_tokens // 16
    for b, L in enumerate(lens):
        pages = (L + 15) // 16
        s0 = -(-pages // plan.split_pages)
        pps = -(-pages // s0)
        assert plan.request(b)[0] == -(-pages // pps)      # near-equal splits


@pytest.mark.parametrize("page_size", [32, 64])
def test_larger_pages_are_planned_in_tiles_of_16_tokens(page_size):
    """With pages of 32 or 64 tokens the plan still counts 16-token tiles: same splits as for page 16."""
    lens = wl.context_lens(wl.WORKLOADS[3])
    ref = make_plan(lens)
    plan = make_plan(lens, page_size=page_size)
    check_plan(plan, lens, 8)
    assert plan.num_runs == ref.num_runs and plan.num_work_items == ref.num_work_items
    for i in range(plan.num_runs):
        assert plan.run(i) == ref.run(i)
    explicit = make_plan([1, 33, 1000, 33000], split_tokens=3 * page_size, page_size=page_size)
    check_plan(explicit, [1, 33, 1000, 33000], 8)
    assert explicit.split_pages == 3 * page_size // 16


def test_tapered_tail_of_a_long_request():
    """In automatic mode a long request ends in splits that shrink down to the granule."""
    w = wl.WORKLOADS[3]
    lens = wl.context_lens(w)
    plan = make_plan(lens, w.num_q_heads, w.num_kv_heads, w.head_dim)
    b = int(np.argmax(lens))
    mine = sorted((plan.run(i) for i in range(plan.num_runs) if plan.run(i)["request"] == b),
                  key=lambda r: r["page_begin"])
    sizes = [r["pages_per_split"] for r in mine]
    assert sizes[0] == plan.split_pages and sizes[-1] == 12
    assert all(a >= b_ for a, b_ in zip(sizes, sizes[1:]))
    assert len(set(sizes)) >= 4


def test_update_reuses_the_plan_and_errors():
    plan = make_plan([100, 5000, 20], capacity=8)
    lens2 = [7, 9000, 300, 1, 64]
    # widths: the plan was created for max_pages_per_seq = ceil(5000/16); 9000 tokens do not fit
    with pytest.raises(binding.OserveError) as e:
        plan.update(np.asarray(lens2, dtype=np.int32))
    assert e.value.status == binding.ERR_CONTEXT_LEN
    plan.update(np.asarray([7, 4000, 300, 1, 64], dtype=np.int32))
    check_plan(plan, [7, 4000, 300, 1, 64], 8)
    with pytest.raises(binding.OserveError) as e:
        plan.update(np.ones(9, dtype=np.int32))
    assert e.value.status == binding.ERR_PLAN_MISMATCH
    with pytest.raises(binding.OserveError) as e:
        plan.update(np.asarray([0, 5], dtype=np.int32))
    assert e.value.status == binding.ERR_CONTEXT_LEN


def test_create_rejects_bad_shapes():
    lens = np.asarray([100], dtype=np.int32)
    bad = [
        dict(num_q_heads=30, num_kv_heads=8),       # not a multiple
        dict(num_q_heads=64, num_kv_heads=2),       # group 32 > 16
        dict(head_dim=96),
        dict(page_size=8),
        dict(page_size=48),
        dict(page_size=128),
        dict(page_size=32, split_tokens=48),        # not a multiple of the page size
        dict(split_tokens=40),                      # not a multiple of the page size
    ]
    for kw in bad:
        args = dict(num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=16, max_pages_per_seq=16,
                    split_tokens=0, device_id=-1)
        args.update(kw)
        with pytest.raises(binding.OserveError) as e:
            binding.Plan(lens, **args)
        assert e.value.status == binding.ERR_SHAPE
    with pytest.raises(binding.OserveError) as e:
        binding.Plan(np.asarray([300], dtype=np.int32), 32, 8, 128, 16, 16, 0, -1)   # 300 tokens > 16 pages
    assert e.value.status == binding.ERR_CONTEXT_LEN


def test_plan_without_device_cannot_launch():
    import ctypes
    plan = make_plan([100, 200])
    st = binding.lib.oserve_paged_decode_attn(plan.handle, ctypes.c_void_p(256), 1 << 20, ctypes.c_void_p(256),
                                             ctypes.c_void_p(256), ctypes.c_void_p(256), ctypes.c_void_p(256),
                                             ctypes.c_void_p(256), ctypes.c_float(1.0), ctypes.c_void_p(256), None)
    assert st == binding.ERR_PLAN_MISMATCH
    st = binding.lib.oserve_paged_decode_attn(plan.handle, None, 0, None, None, None, None, None,
                                             ctypes.c_float(1.0), None, None)
    assert st == binding.ERR_NULL


def test_staged_calls_check_their_arguments_on_the_host():
    """oserve_plan_stage / oserve_paged_decode_attn_staged refuse null pointers and a plan without a device before
    anything is enqueued (the checks that need no GPU)."""
    import ctypes
    plan = make_plan([100, 200])
    p = ctypes.c_void_p(256)
    assert binding.lib.oserve_plan_stage(plan.handle, None, 1 << 20, None) == binding.ERR_NULL
    assert binding.lib.oserve_plan_stage(None, p, 1 << 20, None) == binding.ERR_NULL
    assert binding.lib.oserve_plan_stage(plan.handle, p, 1 << 20, None) == binding.ERR_PLAN_MISMATCH
    st = binding.lib.oserve_paged_decode_attn_staged(plan.handle, p, 1 << 20, p, p, p, p, p, ctypes.c_float(1.0), p, None)
    assert st == binding.ERR_PLAN_MISMATCH
    st = binding.lib.oserve_paged_decode_attn_staged(plan.handle, p, 1 << 20, None, p, p, p, p, ctypes.c_float(1.0), p, None)
    assert st == binding.ERR_NULL


def test_library_exports_every_declared_symbol():
    import re, os
    hdr = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "oserve.h")).read()
    names = set(re.findall(r"\b(oserve_[a-z_]+)\s*\(", hdr))
    assert {"oserve_plan_create", "oserve_paged_decode_attn", "oserve_plan_update"} <= names
    for n in names:
        assert hasattr(binding.lib, n), n
    assert binding.status_string(0) == "ok"


def test_prefill_plan_items_cover_every_query_block_once():
    lens = [1, 17, 300, 1000, 2049]
    qlens = [1, 17, 37, 1000, 100]
    for hq, hkv in [(32, 8), (16, 1), (8, 8), (12, 4), (14, 2)]:
        plan = binding.PrefillPlan(lens, qlens, hq, hkv, 128, 16, 129, -1)
        qb = plan.block_tokens
        padded = 1 << (hq // hkv - 1).bit_length()          # group size rounded up to a power of two
        assert qb == 128 // padded
        seen = set()
        rows = np.concatenate([[0], np.cumsum(qlens)])
        lane_of_group = {}
        for i in range(plan.num_work_items):
            it = plan.item(i)
            b = it["request"]
            assert it["context_len"] == lens[b] and it["q_len"] == qlens[b] and it["q_row0"] == rows[b]
            assert it["q_begin"] % qb == 0 and it["q_begin"] < qlens[b]
            key = (b, it["kv_head"], it["q_begin"])
            assert key not in seen
            seen.add(key)
            lane_of_group.setdefault((b, it["kv_head"]), set()).add(i % 8)
        # while all eight lists still have items, the blocks of a (request, kv head) share the index modulo 8;
        # with fewer than eight (request, kv head) pairs their blocks have to spread over the XCDs instead
        big = [g for g, lanes in lane_of_group.items() if qlens[g[0]] > qb]
        if len(lane_of_group) >= 8:
            assert any(len(lane_of_group[g]) == 1 for g in big) or not big
        assert len(seen) == sum(-(-n // qb) for n in qlens) * hkv
        assert plan.query_tokens == sum(qlens)


def test_mixed_plan_queues_hold_every_prefill_item_once():
    """A mixed batch: the requests with one query token become decode work items (the same ones a decode plan
    over them alone would hold) and get no prefill items; the others become prefill items of 32 query tokens
    (group of 4 heads) x kv heads, each in exactly one queue, the blocks of one (request, kv head) in one queue."""
    lens = wl.context_lens(wl.WORKLOADS[3])[:96].copy()
    qlens = np.ones_like(lens)
    chunks = [5, 17, 40, 77]
    for b in chunks:
        lens[b] = max(lens[b], 700)
        qlens[b] = min(lens[b], 300 + b)
    width = int(wl.pages_needed(lens).max())
    plan = binding.MixedPlan(lens, qlens, 32, 8, 128, 16, width, -1)
    c = plan.counts
    qb = 32
    assert c["prefill_items"] == sum(-(-int(qlens[b]) // qb) for b in chunks) * 8
    assert c["workgroups"] == 512 and c["prefill_queues"] == 8          # the defaults of a plan without a device
    rows = np.concatenate([[0], np.cumsum(qlens)])
    seen, queue_of_group, last_queue = set(), {}, 0
    for i in range(c["prefill_items"]):
        it = plan.prefill_item(i)
        b = it["request"]
        assert b in chunks and it["q_len"] == qlens[b] and it["context_len"] == lens[b] and it["q_row0"] == rows[b]
        assert it["q_begin"] % qb == 0 and it["q_begin"] < qlens[b]
        key = (b, it["kv_head"], it["q_begin"])
        assert key not in seen
        seen.add(key)
        assert queue_of_group.setdefault((b, it["kv_head"]), it["queue"]) == it["queue"]
        assert it["queue"] >= last_queue                                  # queue after queue
        last_queue = it["queue"]
    assert len(seen) == c["prefill_items"] and len(set(queue_of_group.values())) == 8
    assert plan.query_tokens == int(qlens.sum())
    assert plan.workspace_bytes <= plan.workspace_bytes_max
    dec = binding.Plan(lens[qlens == 1], 32, 8, 128, 16, width, 0, -1)
    assert dec.num_work_items == c["decode_items"]
