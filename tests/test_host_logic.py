"""CPU-only tests of the C ABI: the library loads, exports what the header declares,
rejects bad arguments before touching a device, and plans every (row, key) pair once."""
import ctypes
import os
import re
import subprocess
import sys

import numpy as np
import pytest

from paper_2505_21889_amd import binding as E, workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_DEV = 0x7F0000001000  # never dereferenced by the host-only paths exercised here


def _desc(c, n, hq=4, hkv=2, d=128, page=16, table=FAKE_DEV, max_pages=None, num_pages=None):
    c = np.asarray(c, dtype=np.int32)
    n = np.asarray(n, dtype=np.int32)
    need = [-(-(int(a) + int(b)) // 16) for a, b in zip(c, n)]
    if max_pages is None:
        max_pages = max(need + [1])
    if num_pages is None:
        num_pages = sum(need) + 2
    return E.BatchDesc(c, n, table, hq, hkv, d, page, num_pages, max_pages)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "efim.h")).read() + open(os.path.join(ROOT, "include", "efim_debug.h")).read()
    declared = set(re.findall(r"^[a-z][a-z0-9_ *]*\b(efim_[a-z0-9_]+)\s*\(", header, flags=re.M))
    assert declared, "no declarations found"
    lib = ctypes.CDLL(E.LIBRARY_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(E.EXPORTED_SYMBOLS)
    assert E.efim_version() >= 100


def test_library_was_built_from_the_current_sources():
    """The loaded binary records a digest of the sources it was built from; a binary left over
    from older sources would make every other test a test of something else."""
    from paper_2505_21889_amd import binding as E, build
    assert E.efim_source_digest() == build.source_digest(), "libefim.so is stale: run __graft_entry__.build()"
    assert E.efim_status_string(0) == "ok" and "unsupported" in E.efim_status_string(-2)


def _rope_status(desc, q=FAKE_DEV, k=FAKE_DEV, v=FAKE_DEV, kc=FAKE_DEV, vc=FAKE_DEV, base=1e4, inter=0):
    return E.raw_library().efim_rope_append(ctypes.byref(desc.c), q, k, v, kc, vc, base, inter, None)


def _attn_status(desc, q=FAKE_DEV, kc=FAKE_DEV + 0x100000, vc=FAKE_DEV + 0x200000, out=FAKE_DEV + 0x300000,
                 scale=0.0, ws=None, ws_bytes=0):
    return E.raw_library().efim_extend_attention(ctypes.byref(desc.c), q, kc, vc, out, scale, ws, ws_bytes, None)


def test_argument_validation_without_a_device():
    ok = _desc([10], [5])
    assert _rope_status(_desc([10], [5], d=96)) == E.EFIM_ERR_UNSUPPORTED
    for bad_page in (4, 24, 512):
        assert _rope_status(_desc([10], [5], page=bad_page, max_pages=8, num_pages=8)) == E.EFIM_ERR_UNSUPPORTED
    assert _rope_status(_desc([10], [5], hq=5, hkv=2)) == E.EFIM_ERR_INVALID_ARG
    assert _rope_status(_desc([-1], [5])) == E.EFIM_ERR_INVALID_ARG
    assert _rope_status(_desc([10], [-5])) == E.EFIM_ERR_INVALID_ARG
    assert _rope_status(_desc([100], [5], max_pages=3)) == E.EFIM_ERR_INVALID_ARG   # block-table row too short
    assert _rope_status(_desc([100], [5], num_pages=2)) == E.EFIM_ERR_INVALID_ARG
    assert _rope_status(ok, k=None) == E.EFIM_ERR_INVALID_ARG
    assert _rope_status(ok, kc=FAKE_DEV + 2) == E.EFIM_ERR_INVALID_ARG              # misaligned
    assert _rope_status(ok, base=0.0) == E.EFIM_ERR_INVALID_ARG
    assert _rope_status(ok, inter=2) == E.EFIM_ERR_INVALID_ARG
    assert _rope_status(_desc([10], [5], table=None)) == E.EFIM_ERR_INVALID_ARG
    assert E.raw_library().efim_rope_append(None, None, None, None, None, None, 1e4, 0, None) == E.EFIM_ERR_INVALID_ARG

    assert _attn_status(_desc([10], [5], d=256)) == E.EFIM_ERR_UNSUPPORTED
    assert _attn_status(ok, q=None) == E.EFIM_ERR_INVALID_ARG
    assert _attn_status(ok, out=FAKE_DEV) == E.EFIM_ERR_INVALID_ARG                  # out aliases q
    assert _attn_status(ok, scale=-1.0) == E.EFIM_ERR_INVALID_ARG
    assert _attn_status(ok, scale=float("nan")) == E.EFIM_ERR_INVALID_ARG
    assert _attn_status(ok, ws=None, ws_bytes=1 << 20) == E.EFIM_ERR_WORKSPACE
    need = E.efim_extend_workspace_bytes(ok)
    assert need >= 256
    assert _attn_status(ok, ws=FAKE_DEV + 0x400000, ws_bytes=need - 1) == E.EFIM_ERR_WORKSPACE
    assert _attn_status(ok, ws=FAKE_DEV + 0x400010, ws_bytes=need) == E.EFIM_ERR_WORKSPACE   # not 256-aligned
    assert E.efim_extend_workspace_bytes(_desc([10], [5], d=96)) == 0


def test_empty_batches_succeed_without_launching():
    empty = E.BatchDesc(np.zeros(0, np.int32), np.zeros(0, np.int32), None, 4, 2, 128, 16, 0, 0)
    assert _rope_status(empty, None, None, None, None, None) == E.EFIM_OK
    assert _attn_status(empty, None, None, None, None) == E.EFIM_OK
    no_rows = _desc([100, 7], [0, 0])
    assert _rope_status(no_rows, None, None, None, None, None) == E.EFIM_OK
    assert _attn_status(no_rows, None, None, None, None) == E.EFIM_OK
    assert len(E.efim_extend_plan_items(no_rows)) == 0


def test_rope_table_argument_validation_without_a_device():
    lib = E.raw_library()
    d = _desc([10], [5])
    good = (ctypes.c_double * 64)(*[1.0 / (j + 1) for j in range(64)])
    call = lambda table, rd, inter=0: lib.efim_rope_append_table(
        ctypes.byref(d.c), FAKE_DEV, FAKE_DEV, FAKE_DEV, FAKE_DEV, FAKE_DEV, table, rd, inter, None)
    bad = E.EFIM_ERR_INVALID_ARG
    assert call(None, 128) == bad
    for rd in (0, 8, 24, 144, -16):
        assert call(good, rd) == bad            # multiple of 16 within [16, head_dim]
    assert call(good, 64, 2) == bad
    nan = (ctypes.c_double * 64)(*([1.0] * 10 + [float("nan")] + [1.0] * 53))
    inf = (ctypes.c_double * 64)(*([float("inf")] + [1.0] * 63))
    assert call(nan, 128) == bad and call(inf, 16) == bad
    assert call(nan, 16) != bad                 # entries behind rotary_dim / 2 are not read
    empty = _desc([10], [0])
    assert lib.efim_rope_append_table(ctypes.byref(empty.c), None, None, None, None, None, good, 64, 0, None) == E.EFIM_OK


def test_tuning_knobs_validate():
    lib = E.raw_library()
    assert lib.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, 100) == E.EFIM_ERR_INVALID_ARG   # not a multiple of 64
    assert lib.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, -2) == E.EFIM_ERR_INVALID_ARG
    assert lib.efim_set_tuning(99, 0) == E.EFIM_ERR_INVALID_ARG
    assert lib.efim_set_tuning(E.EFIM_TUNE_XCD_GROUPING, 2) == E.EFIM_ERR_INVALID_ARG
    assert lib.efim_set_tuning(E.EFIM_TUNE_FUSED_MERGE, 2) == E.EFIM_ERR_INVALID_ARG
    assert lib.efim_set_tuning(E.EFIM_TUNE_FUSED_MERGE, -2) == E.EFIM_ERR_INVALID_ARG
    assert lib.efim_set_tuning(E.EFIM_TUNE_FUSED_MERGE, -1) == E.EFIM_OK
    assert lib.efim_set_kernel_events(FAKE_DEV, None) == E.EFIM_ERR_INVALID_ARG
    assert lib.efim_set_kernel_events(None, None) == E.EFIM_OK


def _check_plan(c, n, hq, hkv, items):
    """Every visible (row, key) pair of every (request, kv head) is covered exactly once."""
    g = hq // hkv
    items = items[items["row_count"] > 0]
    slots = items["partial_slot"][items["partial_slot"] >= 0]
    assert len(set(slots.tolist())) == len(slots)
    by_tile = {}
    for it in items:
        by_tile.setdefault((int(it["req"]), int(it["kv_head"]), int(it["row_begin"]), int(it["row_count"])), []).append(it)
    rows_seen = {}
    for (r, h, rb, rc), parts in by_tile.items():
        assert 0 <= h < hkv and rb >= 0 and rb + rc <= g * int(n[r])
        rows_seen.setdefault((r, h), []).append((rb, rc))
        last_tok = (rb + rc - 1) // g
        need_end = int(c[r]) + last_tok + 1
        parts = sorted(parts, key=lambda p: int(p["key_begin"]))
        at = 0
        for p in parts:
            assert int(p["key_begin"]) == at and int(p["key_begin"]) % 64 == 0
            assert int(p["key_end"]) > at
            at = int(p["key_end"])
        assert at == need_end
        if len(parts) == 1:
            assert int(parts[0]["partial_slot"]) == -1
        else:
            assert all(int(p["partial_slot"]) >= 0 for p in parts)
            assert len({int(p["merge_id"]) for p in parts}) == 1
    for r in range(len(n)):
        for h in range(hkv):
            total = g * int(n[r])
            tiles = sorted(rows_seen.get((r, h), []))
            at = 0
            for rb, rc in tiles:
                assert rb == at
                at += rc
            assert at == total


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4", "c5"])
def test_plan_covers_named_workloads(name):
    b = W.make_batch(name, with_history=False, with_tensors=False)
    d = E.BatchDesc(b.cached_len, b.new_len, FAKE_DEV, b.num_q_heads, b.num_kv_heads, b.head_dim,
                    b.page_size, b.num_pages, b.max_pages_per_req)
    items = E.efim_extend_plan_items(d)
    _check_plan(b.cached_len, b.new_len, b.num_q_heads, b.num_kv_heads, items)
    assert E.efim_extend_workspace_bytes(d) >= 256


def test_long_items_of_the_mixed_step_start_early():
    """The work list of the mixed serving step, XCD by XCD (items whose indices agree modulo 8):
    the longest items -- cache hits with long contexts and few new rows, light groups of one or
    two very long items -- are among the first to start, not the last."""
    b = W.make_batch("c5", with_history=False, with_tensors=False)
    d = E.BatchDesc(b.cached_len, b.new_len, FAKE_DEV, b.num_q_heads, b.num_kv_heads, b.head_dim,
                    b.page_size, b.num_pages, b.max_pages_per_req)
    items = E.efim_extend_plan_items(d)
    keys = (items["key_end"] - items["key_begin"]).astype(np.int64)
    for x in range(8):
        mine = keys[x::8]
        longest = int(mine.max())
        where = np.flatnonzero(mine >= 0.9 * longest)
        assert where.max() < 0.15 * len(mine), (x, where.max(), len(mine))
        # and the list ends with short items
        assert mine[-len(mine) // 20:].max() <= 0.5 * longest


@pytest.mark.parametrize("split", [-1, 0, 64, 512])
@pytest.mark.parametrize("xcd", [0, 1])
def test_plan_covers_random_ragged_batches(split, xcd):
    rng = np.random.default_rng(100 + split + xcd)
    E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, split)
    E.efim_set_tuning(E.EFIM_TUNE_XCD_GROUPING, xcd)
    try:
        for trial in range(12):
            bsz = int(rng.integers(1, 20))
            c = rng.integers(0, 3000, bsz) * (rng.random(bsz) < 0.7)
            n = rng.integers(0, 600, bsz) * (rng.random(bsz) < 0.9)
            hkv = int(rng.choice([1, 2, 4, 8]))
            hq = hkv * int(rng.choice([1, 2, 4, 7]))
            d = _desc(c, n, hq=hq, hkv=hkv)
            items = E.efim_extend_plan_items(d)
            _check_plan(c, n, hq, hkv, items)
    finally:
        E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, -1)
        E.efim_set_tuning(E.EFIM_TUNE_XCD_GROUPING, 1)


def test_xcd_grouping_places_tiles_sharing_kv_on_one_residue_class():
    # 4 requests x 8 kv heads, 32 query tiles each: tiles of one (request, kv head) read the
    # same K/V and must get workgroup ids congruent modulo 8 (workgroups go round-robin to XCDs)
    c, n = [4096] * 4, [1024] * 4
    d = _desc(c, n, hq=32, hkv=8)
    items = E.efim_extend_plan_items(d)
    _check_plan(c, n, 32, 8, items)
    groups = {}
    for p, it in enumerate(items):
        if it["row_count"] > 0:
            groups.setdefault((int(it["req"]), int(it["kv_head"])), set()).add(p % 8)
    assert len(groups) == 32 and all(len(v) == 1 for v in groups.values())
    per_xcd = [sum(1 for v in groups.values() if v == {x}) for x in range(8)]
    assert max(per_xcd) - min(per_xcd) <= 1


def test_row_tile_choice():
    """128-row tiles by default; 256-row tiles for compute-heavy steps and for steps bound by
    HBM that have at least two such tiles per compute unit."""
    E.efim_set_tuning(E.EFIM_TUNE_NUM_SLOTS, 512)
    try:
        def rows_per_item(c, n, hq, hkv):
            items = E.efim_extend_plan_items(_desc(c, n, hq=hq, hkv=hkv, d=128))
            _check_plan(np.asarray(c), np.asarray(n), hq, hkv, items)
            return 256 if items["row_count"].max() > 128 else 128
        assert rows_per_item([16384] * 4, [512] * 4, 32, 8) == 256           # compute heavy
        assert rows_per_item([4000] * 32, [16] * 32, 28, 4) == 128            # 128 pairs: HBM bound, few tiles
        many = E.efim_extend_plan_items(_desc([3000] * 16, [1] * 16, hq=32, hkv=32, d=128))
        assert len(many[many["row_count"] > 0]) == 512 and (many["partial_slot"] < 0).all()   # 512 pairs: one item each, no split
    finally:
        E.efim_set_tuning(E.EFIM_TUNE_NUM_SLOTS, 0)


def test_split_policy_packs_the_pieces_into_the_slots():
    """Automatic split of a step with fewer (request, kv head) pairs than workgroup slots: the
    pieces fit the slots in one round (one piece too many would cost an extra round with most
    slots idle), none is much longer than a slot's fair share, and coverage stays exact."""
    E.efim_set_tuning(E.EFIM_TUNE_NUM_SLOTS, 512)
    try:
        spec = W.make_batch("c3", with_history=False, with_tensors=False)
        for inc in (1, 16):
            n = np.full_like(spec.new_len, inc)
            d = _desc(spec.cached_len.tolist(), n.tolist(), hq=28, hkv=4, d=128)
            items = E.efim_extend_plan_items(d)
            _check_plan(spec.cached_len, n, 28, 4, items)
            live = items[items["row_count"] > 0]
            tiles = (live["key_end"] - live["key_begin"] + 63) // 64
            assert 400 <= len(live) <= 512
            assert tiles.max() <= 1.25 * tiles.sum() / 512 + 2
    finally:
        E.efim_set_tuning(E.EFIM_TUNE_NUM_SLOTS, 0)


def test_plan_is_deterministic_and_cached_plan_matches_fresh_one():
    d = _desc([700, 0, 3000], [40, 300, 2])
    a = E.efim_extend_plan_items(d)
    other = E.efim_extend_plan_items(_desc([5], [5]))   # evicts the cached plan
    assert len(other) >= 1
    b = E.efim_extend_plan_items(d)
    assert np.array_equal(a, b)


def test_bench_refuses_more_than_one_gpu():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr


def test_static_call_refuses_batches_beyond_its_fixed_array():
    """efim_extend_attention_static checks the sizes on the host, before any device call."""
    b = W.make_batch("c3", with_history=False, with_tensors=False)
    desc = E.BatchDesc(b.cached_len, b.new_len, FAKE_DEV, b.num_q_heads, b.num_kv_heads, b.head_dim, b.page_size,
                       b.num_pages, b.max_pages_per_req)
    assert E.efim_extend_workspace_bytes(desc) > E.efim_extend_static_limit_bytes() == 30 << 20
    with pytest.raises(E.EfimError) as err:
        E.efim_extend_attention_static(desc, 1 << 20, 2 << 20, 3 << 20, 4 << 20, 0.0)
    assert err.value.status == E.EFIM_ERR_WORKSPACE


def test_plan_objects_on_the_host():
    """efim_plan_create / efim_plan_workspace_bytes are pure host functions: a plan is made from the
    lengths alone; a decode plan wants a short step (1..16 new tokens per request, at most 32
    query rows per kv head)."""
    d = _desc([700, 0, 5000], [40, 300, 3])
    plan = E.Plan(d)
    items = E.efim_extend_plan_items(d)
    split = int((items["partial_slot"] >= 0).sum())
    need = E.efim_plan_workspace_bytes(plan)
    # work list (48 bytes per item) + partial results; the batch call's workspace holds the latter only
    assert need >= 48 * len(items) + (E.efim_extend_workspace_bytes(d) if split else 0)
    assert need % 256 == 0
    plan.close()
    plan.close()   # idempotent
    with pytest.raises(E.EfimError):
        E.Plan(d, decode=True)
    dec = E.Plan(_desc([700, 0, 5000], [1, 1, 1]), decode=True)
    assert E.efim_plan_workspace_bytes(dec) >= 256
    with pytest.raises(E.EfimError):   # invalid batch: head_dim
        E.Plan(_desc([4], [1], d=96))
    # an upload into a workspace that is too small is refused before any device call
    with pytest.raises(E.EfimError) as err:
        E.efim_plan_upload(dec, FAKE_DEV, 64)
    assert err.value.status == E.EFIM_ERR_WORKSPACE
    # an empty batch plans to nothing and uploads nothing
    empty = E.Plan(_desc([5, 6], [0, 0]))
    E.efim_plan_upload(empty, FAKE_DEV + 0 if FAKE_DEV % 256 == 0 else (FAKE_DEV // 256 + 1) * 256, E.efim_plan_workspace_bytes(empty))
