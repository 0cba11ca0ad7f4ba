"""CPU tests of the C-ABI library's host side: exports, validation, work-list coverage.

No compute call is made: plans are created host-only (device = -1).
"""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2605_24832_amd import AttnParams, OptimusError, Plan, binding, inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def make_params(**kw):
    args = dict(num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=16, block_size=32,
                num_pages=100000, max_pages_per_req=1024)
    args.update(kw)
    return AttnParams(**args)


def test_library_exports_every_declared_symbol():
    lib = binding.load_library()
    header = open(os.path.join(ROOT, "include", "optimus_attn.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)  # declarations only, no comments
    declared = set(re.findall(r"\b(optimus_[a-z_0-9]+)\s*\(", header))
    assert declared, "no declarations parsed"
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_status_strings():
    for s in range(0, -12, -1):
        assert binding.status_string(s) != "unknown status"
    assert binding.status_string(-99) == "unknown status"


@pytest.mark.parametrize("bad,code", [
    (dict(num_q_heads=30), -2), (dict(head_dim=96), -2), (dict(page_size=8), -2),
    (dict(kv_layout=0), -2), (dict(mask_mode=2), -1), (dict(out_dtype=3), -1),
    (dict(block_size=0), -1), (dict(k_stride_head=100), -1), (dict(k_stride_page=1024), -1),
    (dict(v_stride_page=1 << 31), -1),
])
def test_plan_create_rejects_bad_params(bad, code):
    with pytest.raises(OptimusError) as e:
        Plan(make_params(**bad), device=-1)
    assert e.value.status == code


def test_plan_update_error_codes():
    plan = Plan(make_params(max_pages_per_req=8, num_pages=50), device=-1)
    ok = dict(cu_q=[0, 4, 6], prefix_len=[60, 20], block_start=[32, 0])
    bt = np.full((2, 8), -1, dtype=np.int32)
    bt[0, :4] = [3, 9, 1, 7]
    bt[1, :2] = [49, 0]
    assert plan.plan_update(block_table=bt, **ok) >= 0

    def expect(code, **kw):
        args = dict(ok, block_table=bt)
        args.update(kw)
        with pytest.raises(OptimusError) as e:
            plan.plan_update(**args)
        assert e.value.status == code, (e.value.status, kw)

    expect(-3, cu_q=[1, 4, 6])
    expect(-3, cu_q=[0, 4, 3])
    expect(-4, prefix_len=[-1, 20])
    expect(-4, block_start=[61, 0])
    expect(-4, block_start=[-1, 0])
    expect(-5, block_start=[28, 0])          # d=32 plus c=4 leaves the block of 32
    expect(-5, cu_q=[0, 4, 40], prefix_len=[60, 0])  # c=36 > B
    expect(-6, prefix_len=[60, 127], block_start=[32, 127])  # 129 slots need 9 pages > 8
    bt2 = bt.copy(); bt2[0, 3] = 50
    expect(-7, block_table=bt2)
    bt3 = bt.copy(); bt3[1, 1] = -1
    expect(-7, block_table=bt3)
    # a failed update leaves the plan unplanned
    with pytest.raises(OptimusError) as e:
        plan.kv_append(None, None, None, None, None)
    assert e.value.status == -9
    # device calls on a host-only plan
    plan.plan_update(block_table=bt, **ok)
    with pytest.raises(OptimusError) as e:
        plan.kv_append(None, None, None, None, None)
    assert e.value.status == -10


def test_one_call_step_reports_planning_errors_and_needs_a_device():
    """optimus_attn_step plans first: descriptor errors come back as from plan_update, and a
    host-only plan stops at the first device call (nothing is dereferenced before that)."""
    plan = Plan(make_params(max_pages_per_req=8, num_pages=50), device=-1)
    lib = binding.load_library()

    def step(cu_q, prefix_len, block_start):
        cu, pl, bs = (np.ascontiguousarray(a, dtype=np.int32) for a in (cu_q, prefix_len, block_start))
        return lib.optimus_attn_step(plan._h, len(pl), cu.ctypes.data, pl.ctypes.data, bs.ctypes.data, None,
                                     None, None, None, None, None, None, None, None, None, 0, None)

    assert step([0, 4, 6], [60, 20], [32, 0]) == -10        # planned, then no device
    assert plan.num_work_items() > 0
    assert step([1, 4, 6], [60, 20], [32, 0]) == -3
    assert step([0, 4, 6], [60, 20], [28, 0]) == -5
    assert step([0, 4, 6], [60, 127], [32, 127]) == -6
    assert lib.optimus_attn_step(None, 0, None, None, None, None, None, None, None, None, None, None,
                                 None, None, None, 0, None) == -1


def test_block_table_too_short_boundary():
    plan = Plan(make_params(max_pages_per_req=8), device=-1)
    plan.plan_update([0, 2], [126], [126])            # 128 slots = 8 pages: fits
    with pytest.raises(OptimusError) as e:
        plan.plan_update([0, 3], [126], [126])        # 129 slots = 9 pages
    assert e.value.status == -6


def coverage_check(plan, p: AttnParams, cu_q, prefix_len):
    """Every (request, kv head, row, key) is covered exactly once; partial rows are disjoint."""
    items = plan.work_items()
    G = p.num_q_heads // p.num_kv_heads
    c = np.diff(cu_q)
    assert (items["row_count"] >= 1).all() and (items["row_count"] <= 128).all()
    assert (items["kv_begin"] % 32 == 0).all()
    assert (items["kv_begin"] < items["kv_end"]).all()
    part_rows = []
    for i in range(len(prefix_len)):
        kv_len = int(prefix_len[i] + c[i])
        rows = int(c[i]) * G
        mine = items[items["req"] == i]
        if c[i] == 0:
            assert len(mine) == 0
            continue
        assert (mine["q_token0"] == cu_q[i]).all()
        assert (mine["kv_end"] <= kv_len).all()
        for g in range(p.num_kv_heads):
            cover = np.zeros((rows, kv_len), dtype=np.int32)
            sub = mine[mine["kv_head"] == g]
            for it in sub:
                r0, rc = int(it["row_begin"]), int(it["row_count"])
                assert r0 + rc <= rows
                cover[r0:r0 + rc, int(it["kv_begin"]):int(it["kv_end"])] += 1
                if it["part_row"] >= 0:
                    part_rows.append((int(it["part_row"]), rc))
            assert (cover == 1).all(), f"request {i} head {g}: coverage not exactly once"
            # a q tile is either one unsplit item writing the output or >= 2 partial items
            for r0 in np.unique(sub["row_begin"]):
                tile = sub[sub["row_begin"] == r0]
                if len(tile) == 1:
                    assert tile[0]["part_row"] == -1
                else:
                    assert (tile["part_row"] >= 0).all()
    part_rows.sort()
    end = 0
    for start, n in part_rows:
        assert start >= end, "partial rows overlap"
        end = start + n
    assert plan.workspace_bytes == end * (p.head_dim + 2) * 4
    return items


@pytest.mark.parametrize("k", [0, 1, 2, 3])
def test_work_list_covers_each_config_exactly_once(k):
    shapes = {0: dict(num_q_heads=4, num_kv_heads=4, head_dim=64),
              1: dict(num_q_heads=32, num_kv_heads=32),
              2: dict(num_q_heads=28, num_kv_heads=4),
              3: dict(num_q_heads=32, num_kv_heads=8)}[k]
    rng = np.random.RandomState(inputs.BASE_SEED + k)
    if k == 0:
        L, c = np.array([128]), np.array([8])
    elif k == 1:
        L, c = np.array([2048]), np.array([32])
    elif k == 2:
        L, c = rng.randint(512, 4097, size=64), rng.choice([1, 2, 4, 8, 16, 32], size=64)
    else:
        L, c = rng.randint(1024, 8193, size=48), rng.choice([1, 2, 4], size=48)
    cu = np.concatenate([[0], np.cumsum(c)]).astype(np.int32)
    p = make_params(**shapes)
    plan = Plan(p, device=-1)
    plan.plan_update(cu, L, L - np.minimum(L % 32, 32 - c))
    items = coverage_check(plan, p, cu, L)
    assert len(items) == plan.num_work_items()


def test_work_list_with_forced_tuning_and_odd_shapes():
    p = make_params(num_q_heads=28, num_kv_heads=4, block_size=32)
    plan = Plan(p, device=-1)
    L = np.array([0, 31, 32, 33, 1000, 7, 64])
    c = np.array([5, 1, 0, 32, 17, 25, 32])
    cu = np.concatenate([[0], np.cumsum(c)]).astype(np.int32)
    for tuning in (dict(target_items=1 << 20, min_split_tokens=32, max_split_tokens=32),
                   dict(target_items=1, min_split_tokens=1 << 20, max_split_tokens=1 << 20),
                   dict(target_items=100, min_split_tokens=64, max_split_tokens=256), dict()):
        plan.set_tuning(**tuning)
        plan.plan_update(cu, L, L)  # d_i = 0
        coverage_check(plan, p, cu, L)
    with pytest.raises(OptimusError):
        plan.set_tuning(min_split_tokens=33)


def test_default_plan_fills_whole_rounds_of_resident_workgroups():
    """Short lists are fitted to the 512 workgroup slots of a 256-CU device (the host-only
    plan assumes 256 CUs): at most one full round when a balanced one exists, never a
    little more than a multiple of 512; an explicit target_items switches the fit off."""
    slots = 512
    # config-2-like mix: 256 (request, kv head) pairs, 352 unsplit items -> one round
    p = make_params(num_q_heads=28, num_kv_heads=4)
    rng = np.random.RandomState(11)
    for R in (24, 32, 48, 64):
        L = rng.randint(512, 4097, size=R)
        c = rng.choice([1, 2, 4, 8, 16, 32], size=R)
        cu = np.concatenate([[0], np.cumsum(c)]).astype(np.int32)
        plan = Plan(p, device=-1)
        plan.plan_update(cu, L, L)
        n = plan.num_work_items()
        assert 0.8 * slots <= n <= slots, (R, n)
        coverage_check(plan, p, cu, L)
        plan.set_tuning(target_items=1024)
        plan.plan_update(cu, L, L)
        assert plan.num_work_items() > slots
    # long-context case: 4 requests x 8 kv heads x 4 row tiles of 128 rows -> 4 splits = 512
    p = make_params(num_q_heads=32, num_kv_heads=8, page_size=64, block_size=128, max_pages_per_req=520)
    L = np.full(4, 32768)
    c = np.full(4, 128)
    cu = np.concatenate([[0], np.cumsum(c)]).astype(np.int32)
    plan = Plan(p, device=-1)
    plan.plan_update(cu, L, L)
    assert plan.num_work_items() == slots
    coverage_check(plan, p, cu, L)
    # 512 unsplit pairs of very different lengths: one round would be unbalanced, so two
    p = make_params(num_q_heads=32, num_kv_heads=8)
    rng = np.random.RandomState(12)
    L = rng.randint(1024, 8193, size=64)
    c = rng.choice([1, 2, 4], size=64)
    cu = np.concatenate([[0], np.cumsum(c)]).astype(np.int32)
    plan = Plan(p, device=-1)
    plan.plan_update(cu, L, L)
    assert slots < plan.num_work_items() <= 2 * slots
    coverage_check(plan, p, cu, L)


def interval_coverage_check(plan, p: AttnParams, cu_q, prefix_len):
    """coverage_check without the dense matrix (for long contexts): per (request, kv head) the
    row tiles partition the rows, and the key ranges of every row tile partition [0, kv_len)."""
    items = plan.work_items()
    G = p.num_q_heads // p.num_kv_heads
    c = np.diff(cu_q)
    assert (items["kv_begin"] % 32 == 0).all() and (items["kv_begin"] < items["kv_end"]).all()
    order = np.lexsort((items["kv_begin"], items["row_begin"], items["kv_head"], items["req"]))
    it = items[order]
    n_expected_groups = 0
    k = 0
    for i in range(len(prefix_len)):
        if c[i] == 0:
            continue
        rows, kv_len = int(c[i]) * G, int(prefix_len[i] + c[i])
        for g in range(p.num_kv_heads):
            r0 = 0
            while r0 < rows:
                rc = min(128, rows - r0)
                pos = 0
                first = k
                while k < len(it) and (it["req"][k], it["kv_head"][k], it["row_begin"][k]) == (i, g, r0):
                    assert it["row_count"][k] == rc and it["kv_begin"][k] == pos
                    assert it["q_token0"][k] == cu_q[i]
                    pos = int(it["kv_end"][k])
                    k += 1
                assert pos == kv_len, f"request {i} head {g} rows {r0}: keys end at {pos}, not {kv_len}"
                n_split = k - first
                assert ((it["part_row"][first:k] >= 0).all() if n_split > 1 else it["part_row"][first] == -1)
                r0 += rc
                n_expected_groups += 1
    assert k == len(it)
    parts = np.sort(items["part_row"][items["part_row"] >= 0])
    assert len(np.unique(parts)) == len(parts)
    return items


@pytest.mark.parametrize("seed", range(30))
def test_random_batches_are_covered_and_lists_stay_short(seed):
    """Seeded random geometries and batches, default tuning: exact coverage, and the fitted
    list never exceeds what the plain rule would give by more than the per-pair rounding."""
    rng = np.random.RandomState(4000 + seed)
    Hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.choice([1, 2, 4, 7, 8]))
    B = int(rng.choice([32, 64, 128]))
    P = int(rng.choice([16, 64]))
    R = int(rng.choice([1, 2, 5, 17, 64, 200, 400]))
    Lmax = int(rng.choice([300, 5000, 40000, 1000000]))
    p = make_params(num_q_heads=Hkv * G, num_kv_heads=Hkv, block_size=B, page_size=P,
                    max_pages_per_req=(Lmax + B) // P + 2, num_pages=1 << 30)
    d_in = rng.randint(0, B, size=R)
    c = np.array([rng.randint(0, B - d + 1) for d in d_in])
    L = rng.randint(0, Lmax // B + 1, size=R) * B + d_in
    cu = np.concatenate([[0], np.cumsum(c)]).astype(np.int32)
    plan = Plan(p, device=-1)
    plan.plan_update(cu, L, L - d_in)
    items = interval_coverage_check(plan, p, cu, L)
    n_pairs_tiles = int(sum(Hkv * -(-int(ci) * G // 128) for ci in c if ci > 0))
    assert len(items) >= n_pairs_tiles
    # never more than two rounds of 512 plus one item per row tile, unless unsplit is already more
    assert len(items) <= max(2 * 512 + n_pairs_tiles, n_pairs_tiles)
    if len(items) > n_pairs_tiles:   # something was split: splits respect the 256-key minimum
        split = items[items["part_row"] >= 0]
        full = split[split["kv_end"] % 32 == 0]
        assert ((full["kv_end"] - full["kv_begin"]) >= 32).all()


def test_plan_is_deterministic_and_longest_first_within_class():
    p = make_params(num_q_heads=32, num_kv_heads=4)
    rng = np.random.RandomState(5)
    L = rng.randint(1024, 8193, size=32)
    c = rng.choice([1, 2, 4, 8, 16, 32], size=32)
    cu = np.concatenate([[0], np.cumsum(c)]).astype(np.int32)
    a = Plan(p, device=-1)
    b = Plan(p, device=-1)
    a.plan_update(cu, L, L)
    b.plan_update(cu, L, L)
    ia, ib = a.work_items(), b.work_items()
    assert (ia == ib).all()
    # costliest first: the cost of an item is its tile count times the per-tile cost of the
    # widest row tile of its (request, kv head) pair
    G = p.num_q_heads // p.num_kv_heads
    widest = np.minimum(128, c[ia["req"]] * G)
    tile_cost = np.where(widest <= 16, 1.0, np.where(widest <= 32, 1.1, 1.2))
    cost = ((ia["kv_end"] - ia["kv_begin"] + 31) // 32) * tile_cost
    # costliest first inside each of the 8 XCD lanes (workgroup i runs on XCD i % 8); checked on
    # the first half of the list, before the shortest lane can have run out
    half = len(ia) // 2 // 8 * 8
    assert cost[0] == cost.max()
    for x in range(8):
        assert (np.diff(cost[x:half:8]) <= 1e-9).all()
    # row tiles of one key range are 8 apart: same XCD, same time
    wide = np.nonzero(c * G > 128)[0]
    assert len(wide)
    checked = 0
    for i in wide:
        idx = np.nonzero((ia["req"] == i) & (ia["kv_head"] == 0) & (ia["kv_begin"] == 0))[0]
        assert len(idx) == -(-int(c[i]) * G // 128)
        if idx.max() < half:
            assert (np.diff(idx) == 8).all()
            checked += 1
    assert checked


def test_empty_batch_and_zero_chunks():
    plan = Plan(make_params(), device=-1)
    assert plan.plan_update([0], [], []) == 0
    assert plan.num_work_items() == 0
    assert plan.plan_update([0, 0, 0], [10, 20], [10, 20]) == 0
    assert plan.num_work_items() == 0


def test_header_struct_sizes_match_binding():
    assert ctypes.sizeof(binding.WorkItem) == 32
    # 12 int32/float fields + 4 int64
    assert ctypes.sizeof(binding._CParams) == 12 * 4 + 4 * 8


def test_host_batch_is_marshalled_once_and_rewritten_in_place():
    """HostBatch copies the descriptors into int32 arrays whose addresses the library is given:
    rewriting them in place changes what the next call plans, replacing them is refused, and
    the one-call step on them reports planning errors like attn_step."""
    from paper_2605_24832_amd import HostBatch
    p = make_params()
    hb = HostBatch([0, 4, 6], [100, 37], [96, 32])
    assert hb.batch == 2 and hb.cu_q.dtype == np.int32 and hb.block_table is None
    with pytest.raises(AttributeError):
        hb.prefix_len = np.zeros(2, dtype=np.int32)
    with pytest.raises(ValueError):
        HostBatch([0, 4], [100, 37], [96, 32])
    plan = Plan(p, device=-1)

    class NoBuffers:   # a host-only plan stops before any device pointer is looked at
        _p = (None,) * 9
        _ws_bytes = 0
    with pytest.raises(OptimusError) as e:
        plan.attn_step_bound(hb, NoBuffers())
    assert e.value.status == -10            # planned, then: no device
    n0 = plan.num_work_items()
    assert n0 > 0
    hb.prefix_len[:] = [4000, 37]           # in place: a longer context, more items
    hb.block_start[:] = [4000, 32]
    with pytest.raises(OptimusError) as e:
        plan.attn_step_bound(hb, NoBuffers())
    # the longer context is split, and split items need a workspace: refused before any device call
    assert e.value.status == -8 and plan.num_work_items() > n0
    hb.cu_q[:] = [1, 4, 6]                  # in place: does not start at 0 any more
    with pytest.raises(OptimusError) as e:
        plan.attn_step_bound(hb, NoBuffers())
    assert e.value.status == -3
