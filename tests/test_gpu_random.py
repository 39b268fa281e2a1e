"""Seeded random batches through the whole path (efim_rope_append then efim_extend_attention)
against the oracle: ragged lengths with zeros, cached lengths on and around page and tile
boundaries, every supported head layout and page size, random planner knobs.  Caches start poisoned, so a
read of any slot that is not part of a request shows up as NaN."""
import numpy as np
import pytest
import torch

from oracle import efim_oracle as O
from paper_2505_21889_amd import workloads as W

import gpu_util as U

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def E():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2505_21889_amd import binding
    return binding


HEADS = [(1, 1), (4, 4), (4, 2), (8, 2), (6, 1), (14, 2), (12, 4)]
EDGES = [0, 1, 15, 16, 17, 31, 63, 64, 65, 127, 128, 129, 255, 256, 1000]


def draw_case(rng):
    batch = int(rng.integers(1, 7))
    cached = [int(rng.choice(EDGES)) if rng.random() < 0.6 else int(rng.integers(0, 1500)) for _ in range(batch)]
    new = [int(rng.choice([0, 1, 2, 15, 16, 17, 33, 64, 65, 130])) if rng.random() < 0.7 else int(rng.integers(1, 300))
           for _ in range(batch)]
    if sum(new) == 0:
        new[0] = 3
    heads = HEADS[int(rng.integers(len(HEADS)))]
    d = int(rng.choice([64, 128]))
    knobs = {"split": int(rng.choice([-1, -1, 0, 64, 128, 256])), "row_tile": int(rng.choice([0, 0, 128, 256])),
             "xcd": int(rng.integers(0, 2)), "merge": int(rng.choice([-1, 0, 1])), "interleaved": int(rng.integers(0, 2))}
    return cached, new, heads, d, knobs


@pytest.mark.parametrize("seed", range(24))
def test_random_batch(E, seed):
    rng = np.random.default_rng(9000 + seed)
    cached, new, heads, d, knobs = draw_case(rng)
    b = W.make_batch("c1", seed=500 + seed, lengths=(np.array(cached, dtype=np.int32), np.array(new, dtype=np.int32)),
                     heads=heads, head_dim=d, sigma=float(rng.choice([0.5, 1.0, 2.0])),
                     page_size=int(rng.choice([8, 16, 16, 32, 64, 128, 256])))
    kc, vc = U.oracle_cache(b)
    kc_ref, vc_ref = kc.copy(), vc.copy()
    inter = bool(knobs["interleaved"])
    q_ref, _ = O.rope_append(b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new, b.k_new, b.v_new,
                             kc_ref, vc_ref, b.rope_base, inter)
    ref = O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q_ref, kc_ref, vc_ref)
    E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, knobs["split"])
    E.efim_set_tuning(E.EFIM_TUNE_ROW_TILE, knobs["row_tile"])
    E.efim_set_tuning(E.EFIM_TUNE_XCD_GROUPING, knobs["xcd"])
    E.efim_set_tuning(E.EFIM_TUNE_FUSED_MERGE, knobs["merge"])
    try:
        q_gpu, kc_gpu, vc_gpu = U.gpu_rope_append(E, b, kc, vc, interleaved=int(inter))
        assert np.array_equal(q_gpu, q_ref) and np.array_equal(kc_gpu, kc_ref) and np.array_equal(vc_gpu, vc_ref), \
            (cached, new, heads, d, knobs)
        got = U.gpu_extend_attention(E, b, q_ref, kc_ref, vc_ref)
        # activations of standard deviation 2 make the softmax pick single value rows of
        # magnitude up to ~8, whose bf16 rounding alone exceeds 1e-2: the absolute bound is
        # taken element by element and in units of the value scale (relative L2 unchanged)
        U.assert_close(got, ref, "%s %s %s d%d %s" % (cached, new, heads, d, knobs), large_outputs=True,
                       value_scale=b.sigma)
    finally:
        E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, -1)
        E.efim_set_tuning(E.EFIM_TUNE_ROW_TILE, 0)
        E.efim_set_tuning(E.EFIM_TUNE_XCD_GROUPING, 1)
        E.efim_set_tuning(E.EFIM_TUNE_FUSED_MERGE, -1)


@pytest.mark.parametrize("seed", range(12))
def test_random_decode_step(E, seed):
    """The single-launch decode step on random batches: caches bit-exact, output within the bar
    and identical to what the two calls produce."""
    rng = np.random.default_rng(7000 + seed)
    batch = int(rng.integers(1, 9))
    cached = np.array([int(rng.choice(EDGES)) if rng.random() < 0.5 else int(rng.integers(0, 3000))
                       for _ in range(batch)], dtype=np.int32)
    heads = HEADS[int(rng.integers(len(HEADS)))]
    d = int(rng.choice([64, 128]))
    inter = int(rng.integers(0, 2))
    b = W.make_batch("c1", seed=800 + seed, lengths=(cached, np.ones_like(cached)), heads=heads, head_dim=d,
                     page_size=int(rng.choice([8, 16, 16, 32, 128])))
    kc, vc = U.oracle_cache(b)
    kc_ref, vc_ref = kc.copy(), vc.copy()
    q_ref, _ = O.rope_append(b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new, b.k_new, b.v_new,
                             kc_ref, vc_ref, b.rope_base, bool(inter))
    ref = O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q_ref, kc_ref, vc_ref)
    E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, int(rng.choice([-1, 64, 192, 0])))
    E.efim_set_tuning(E.EFIM_TUNE_ROW_TILE, int(rng.choice([0, 0, 256])))
    try:
        table = torch.from_numpy(b.block_table).cuda()
        desc = U.make_desc(E, b, table)
        q = U.dev_bits(b.q_new)
        kcd, vcd = U.dev_bits(kc), U.dev_bits(vc)
        out = torch.full(q.shape, 0x7FC1, dtype=torch.int16, device="cuda")
        nbytes = E.efim_decode_workspace_bytes(desc)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        E.efim_decode_step(desc, q, U.dev_bits(b.k_new), U.dev_bits(b.v_new), kcd, vcd, out, b.rope_base, inter, 0.0,
                           ws, nbytes)
        torch.cuda.synchronize()
        assert np.array_equal(U.host_bits(kcd), kc_ref) and np.array_equal(U.host_bits(vcd), vc_ref)
        U.assert_close(U.host_bits(out), ref, "%s %s d%d" % (cached.tolist(), heads, d))
        assert np.array_equal(U.host_bits(out), U.gpu_extend_attention(E, b, q_ref, kc_ref, vc_ref))
    finally:
        E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, -1)
        E.efim_set_tuning(E.EFIM_TUNE_ROW_TILE, 0)


@pytest.mark.parametrize("seed", range(12))
def test_random_short_step(E, seed):
    """The single-launch step with several new tokens per request (as many as the head grouping
    allows: at most 16, and at most 32 query rows per kv head) on random batches: caches
    bit-exact, output within the bar and identical to what the two calls produce."""
    rng = np.random.default_rng(7500 + seed)
    batch = int(rng.integers(1, 9))
    cached = np.array([int(rng.choice(EDGES)) if rng.random() < 0.5 else int(rng.integers(0, 3000))
                       for _ in range(batch)], dtype=np.int32)
    heads = HEADS[int(rng.integers(len(HEADS)))]
    d = int(rng.choice([64, 128]))
    inter = int(rng.integers(0, 2))
    most = min(16, 32 // (heads[0] // heads[1]))
    new = rng.integers(1, most + 1, batch).astype(np.int32)
    b = W.make_batch("c1", seed=850 + seed, lengths=(cached, new), heads=heads, head_dim=d,
                     page_size=int(rng.choice([8, 16, 16, 32, 128])))
    kc, vc = U.oracle_cache(b)
    kc_ref, vc_ref = kc.copy(), vc.copy()
    q_ref, _ = O.rope_append(b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new, b.k_new, b.v_new,
                             kc_ref, vc_ref, b.rope_base, bool(inter))
    ref = O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q_ref, kc_ref, vc_ref)
    E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, int(rng.choice([-1, 64, 192, 0])))
    E.efim_set_tuning(E.EFIM_TUNE_ROW_TILE, int(rng.choice([0, 0, 256])))
    try:
        table = torch.from_numpy(b.block_table).cuda()
        desc = U.make_desc(E, b, table)
        q = U.dev_bits(b.q_new)
        kcd, vcd = U.dev_bits(kc), U.dev_bits(vc)
        out = torch.full(q.shape, 0x7FC1, dtype=torch.int16, device="cuda")
        nbytes = E.efim_decode_workspace_bytes(desc)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        E.efim_decode_step(desc, q, U.dev_bits(b.k_new), U.dev_bits(b.v_new), kcd, vcd, out, b.rope_base, inter, 0.0,
                           ws, nbytes)
        torch.cuda.synchronize()
        assert np.array_equal(U.host_bits(kcd), kc_ref) and np.array_equal(U.host_bits(vcd), vc_ref)
        U.assert_close(U.host_bits(out), ref, "%s %s %s d%d" % (cached.tolist(), new.tolist(), heads, d), large_outputs=True)
        assert np.array_equal(U.host_bits(out), U.gpu_extend_attention(E, b, q_ref, kc_ref, vc_ref))
    finally:
        E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, -1)
        E.efim_set_tuning(E.EFIM_TUNE_ROW_TILE, 0)
