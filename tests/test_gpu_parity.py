"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Integer/byte work (append, gather) must be bit-exact; attention outputs from
bf16 inputs with fp32 accumulation must reach max abs error <= 1e-2 and relative L2 <= 5e-3."""
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


def _ragged(seed, cached, new, **kw):
    return W.make_batch("c1", seed=seed, lengths=(np.array(cached, dtype=np.int32), np.array(new, dtype=np.int32)), **kw)


# ------------------------------------------------------------ rope_append ----

@pytest.mark.parametrize("name", ["c1", "c2", "c3"])
def test_rope_append_bit_exact(E, name):
    b = W.make_batch(name)
    kc, vc = U.oracle_cache(b, fill=0xABCD)
    q_gpu, kc_gpu, vc_gpu = U.gpu_rope_append(E, b, kc, vc)
    q_ref, _ = O.rope_append(b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new, b.k_new,
                             b.v_new, kc, vc, b.rope_base)
    assert np.array_equal(vc_gpu, vc)          # values: bit copy, and no other byte touched
    assert np.array_equal(kc_gpu, kc)          # rotated keys: fp64 rotation, one rounding
    assert np.array_equal(q_gpu, q_ref)


@pytest.mark.parametrize("interleaved", [0, 1])
@pytest.mark.parametrize("d", [64, 128])
def test_rope_append_ragged_edges(E, interleaved, d):
    # mid-page start, page-aligned start, empty request, single token, full miss, >3 pages
    b = _ragged(77 + d, [5, 16, 9, 0, 0, 31], [27, 16, 0, 1, 70, 3], heads=(6, 2), head_dim=d)
    kc, vc = U.oracle_cache(b, fill=0x1234)
    q_gpu, kc_gpu, vc_gpu = U.gpu_rope_append(E, b, kc, vc, interleaved=interleaved)
    q_ref, _ = O.rope_append(b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new, b.k_new,
                             b.v_new, kc, vc, b.rope_base, interleaved=bool(interleaved))
    assert np.array_equal(vc_gpu, vc) and np.array_equal(kc_gpu, kc) and np.array_equal(q_gpu, q_ref)


def test_rope_append_without_queries_and_large_positions(E):
    b = _ragged(78, [100000, 65535], [5, 40], heads=(2, 2), head_dim=128, rope_base=1.0e6)
    b.k_hist = b.v_hist = None
    kc, vc = U.oracle_cache(b, fill=0)
    _, kc_gpu, vc_gpu = U.gpu_rope_append(E, b, kc, vc, with_q=False)
    O.rope_append(b.cached_len, b.new_len, b.block_table, b.page_size, None, b.k_new, b.v_new, kc, vc, b.rope_base)
    assert np.array_equal(kc_gpu, kc) and np.array_equal(vc_gpu, vc)


# ------------------------------------------------------- extend attention ----

def _oracle_inputs(b):
    kc, vc = U.oracle_cache(b)
    q_roped, _ = O.rope_append(b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new, b.k_new,
                               b.v_new, kc, vc, b.rope_base)
    return q_roped, kc, vc


def test_extend_attention_c1_exhaustive(E):
    b = W.make_batch("c1")
    q_roped, kc, vc = _oracle_inputs(b)
    ref = O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q_roped, kc, vc)
    got = U.gpu_extend_attention(E, b, q_roped, kc, vc)
    U.assert_close(got, ref, "c1")


@pytest.mark.parametrize("heads,d", [((4, 4), 64), ((6, 2), 128), ((8, 1), 128), ((7, 1), 64)])
def test_extend_attention_ragged_small(E, heads, d):
    # several 64-key tiles with ragged tails, rows spanning several waves, empty request,
    # decode-like single token, full misses, a request shorter than one page
    b = _ragged(90 + d + heads[0], [200, 0, 63, 129, 0, 5, 1000], [37, 150, 1, 64, 3, 0, 9], heads=heads, head_dim=d)
    q_roped, kc, vc = _oracle_inputs(b)
    ref = O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q_roped, kc, vc)
    got = U.gpu_extend_attention(E, b, q_roped, kc, vc)
    U.assert_close(got, ref, "ragged")


@pytest.mark.parametrize("row_tile", [128, 256])
@pytest.mark.parametrize("heads,d", [((4, 4), 64), ((8, 2), 128)])
def test_extend_attention_both_row_tiles(E, row_tile, heads, d):
    # the 128-row (4 waves, 2 LDS stages) and 256-row (8 waves, 3 stages) configurations on
    # the same ragged batch: long enough for the 3-stage ring to wrap several times
    b = _ragged(93 + d, [700, 0, 129, 5], [100, 333, 64, 1], heads=heads, head_dim=d)
    q_roped, kc, vc = _oracle_inputs(b)
    ref = O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q_roped, kc, vc)
    E.efim_set_tuning(E.EFIM_TUNE_ROW_TILE, row_tile)
    try:
        got = U.gpu_extend_attention(E, b, q_roped, kc, vc)
    finally:
        E.efim_set_tuning(E.EFIM_TUNE_ROW_TILE, 0)
    U.assert_close(got, ref, "row tile %d" % row_tile)


@pytest.mark.parametrize("split", [0, 64, 256])
def test_extend_attention_split_kv_agrees(E, split):
    b = _ragged(95, [700, 0, 300], [40, 300, 2], heads=(4, 2), head_dim=128)
    q_roped, kc, vc = _oracle_inputs(b)
    ref = O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q_roped, kc, vc)
    E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, split)
    try:
        got = U.gpu_extend_attention(E, b, q_roped, kc, vc)
        # the parts of a split range combined inside the kernel instead of by a second launch:
        # same arithmetic, so the same bits
        E.efim_set_tuning(E.EFIM_TUNE_FUSED_MERGE, 1)
        one_launch = U.gpu_extend_attention(E, b, q_roped, kc, vc)
    finally:
        E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, -1)
        E.efim_set_tuning(E.EFIM_TUNE_FUSED_MERGE, -1)
    U.assert_close(got, ref, "split %d" % split)
    assert np.array_equal(got, one_launch)


@pytest.mark.parametrize("power", [20, -20, 60])
def test_split_ranges_scale_exactly_with_the_values(E, power):
    """Values 2^k times larger give outputs exactly 2^k times larger, also where key ranges are
    split: the partial results travel as 16-bit rows with a scale of their own, which must
    neither overflow nor lose small rows.  (No oracle needed: every product and sum scales by a
    power of two without rounding differently.)"""
    b = _ragged(96, [900, 130, 2500], [33, 5, 70], heads=(8, 2), head_dim=128)
    q_roped, kc, vc = _oracle_inputs(b)
    vc_scaled = O.f64_to_bf16(O.bf16_to_f64(vc) * 2.0 ** power)
    assert np.array_equal(O.bf16_to_f64(vc_scaled), O.bf16_to_f64(vc) * 2.0 ** power, equal_nan=True)   # (exact; unused slots hold NaN)
    for merge in (0, 1):
        E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, 128)
        E.efim_set_tuning(E.EFIM_TUNE_FUSED_MERGE, merge)
        try:
            base = U.gpu_extend_attention(E, b, q_roped, kc, vc)
            scaled = U.gpu_extend_attention(E, b, q_roped, kc, vc_scaled)
        finally:
            E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, -1)
            E.efim_set_tuning(E.EFIM_TUNE_FUSED_MERGE, -1)
        assert np.array_equal(O.bf16_to_f64(scaled), O.bf16_to_f64(base) * 2.0 ** power), "merge path %d" % merge


def test_many_splits_and_overlapping_calls(E):
    """More than eight parts per query tile (the merge takes them in groups of eight), and
    several calls in flight on different streams: each uses its own block of arrival counters."""
    b = _ragged(97, [5000, 1300], [3, 70], heads=(8, 2), head_dim=128)
    q_roped, kc, vc = _oracle_inputs(b)
    ref = O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q_roped, kc, vc)
    E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, 256)
    E.efim_set_tuning(E.EFIM_TUNE_FUSED_MERGE, 1)
    try:
        got = U.gpu_extend_attention(E, b, q_roped, kc, vc)
        U.assert_close(got, ref, "20 parts")
        table = torch.from_numpy(b.block_table).cuda()
        desc = U.make_desc(E, b, table)
        q, kcd, vcd = U.dev_bits(q_roped), U.dev_bits(kc), U.dev_bits(vc)
        nbytes = E.efim_extend_workspace_bytes(desc)
        streams = [torch.cuda.Stream() for _ in range(3)]
        outs = [torch.full(q.shape, 0x7FC1, dtype=torch.int16, device="cuda") for _ in range(12)]
        wss = [torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda") for _ in range(12)]
        torch.cuda.synchronize()
        for i in range(12):
            E.efim_extend_attention(desc, q, kcd, vcd, outs[i], 0.0, wss[i], nbytes, streams[i % 3])
        torch.cuda.synchronize()
        for o in outs:
            assert np.array_equal(U.host_bits(o), got)
    finally:
        E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, -1)
        E.efim_set_tuning(E.EFIM_TUNE_FUSED_MERGE, -1)


def test_single_key_is_bit_exact_value_row(E):
    b = _ragged(96, [0, 0], [1, 1], heads=(6, 2), head_dim=128)
    q_roped, kc, vc = _oracle_inputs(b)
    got = U.gpu_extend_attention(E, b, q_roped, kc, vc)
    for r in range(2):
        for a in range(6):
            assert np.array_equal(got[r, a], b.v_new[r, a // 3])


def test_zero_query_gives_running_mean(E):
    b = _ragged(97, [130, 0], [70, 66], heads=(2, 1), head_dim=128)
    q_roped, kc, vc = _oracle_inputs(b)
    q0 = np.zeros_like(q_roped)
    ref = O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q0, kc, vc)
    got = U.gpu_extend_attention(E, b, q0, kc, vc)
    U.assert_close(got, ref, "q=0")


def test_page_permutation_invariance_bit_exact(E):
    b = W.make_batch("c1", seed=98)
    q_roped, kc, vc = _oracle_inputs(b)
    got = U.gpu_extend_attention(E, b, q_roped, kc, vc)
    perm = np.random.default_rng(2).permutation(b.num_pages)
    kc2, vc2 = np.empty_like(kc), np.empty_like(vc)
    kc2[perm], vc2[perm] = kc, vc
    got2 = U.gpu_extend_attention(E, b, q_roped, kc2, vc2, table=perm[b.block_table].astype(np.int32))
    assert np.array_equal(got, got2)


@pytest.mark.parametrize("heads,d,cached,new,j,knobs", [
    ((8, 2), 128, [300, 0], [90, 200], 50, {}),                       # several waves per tile
    ((8, 2), 128, [300, 0], [90, 200], 50, {"ROW_TILE": 256}),
    ((8, 2), 128, [1500, 0], [90, 200], 17, {"SPLIT_KV": 256}),       # cut key ranges + merge pass
    ((4, 4), 64, [700, 40], [6, 3], 3, {}),                           # at most 32 rows: key-parallel kernel
    ((4, 4), 64, [700, 40], [6, 3], 3, {"SPLIT_KV": 128, "FUSED_MERGE": 1}),
])
def test_causality_later_tokens_do_not_touch_earlier_rows(E, heads, d, cached, new, j, knobs):
    """Changing new token j of a request (its query, and its key and value in the cache) leaves
    every output row of earlier tokens, and every row of the other requests, bit for bit as it
    was: a row's arithmetic depends only on that row's query and its visible keys."""
    b = _ragged(160 + d + j, cached, new, heads=heads, head_dim=d)
    q_roped, kc, vc = _oracle_inputs(b)
    rng = np.random.default_rng(3)
    q2, kc2, vc2 = q_roped.copy(), kc.copy(), vc.copy()
    pos = int(b.cached_len[0]) + j
    page, slot = int(b.block_table[0, pos // b.page_size]), pos % b.page_size
    kc2[page, :, slot, :] = W.gaussian_bf16(rng, (b.num_kv_heads, d), 3.0)   # finite, much larger scores
    vc2[page, :, slot, :] = W.gaussian_bf16(rng, (b.num_kv_heads, d), 3.0)
    q2[j] = W.gaussian_bf16(rng, (b.num_q_heads, d), 3.0)
    for key, val in knobs.items():
        E.efim_set_tuning(getattr(E, "EFIM_TUNE_" + key), val)
    try:
        got = U.gpu_extend_attention(E, b, q_roped, kc, vc)
        got2 = U.gpu_extend_attention(E, b, q2, kc2, vc2)
    finally:
        E.efim_set_tuning(E.EFIM_TUNE_ROW_TILE, 0)
        E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, -1)
        E.efim_set_tuning(E.EFIM_TUNE_FUSED_MERGE, -1)
    n0 = int(b.new_len[0])
    assert np.array_equal(got[:j], got2[:j]), "rows of earlier tokens changed"
    assert np.array_equal(got[n0:], got2[n0:]), "rows of another request changed"
    assert not np.array_equal(got[j:n0], got2[j:n0]), "the change must reach the later rows"
    ref2 = O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q2, kc2, vc2)
    U.assert_close(got2, ref2, "perturbed", large_outputs=True, value_scale=3.0)


def _one_request_of(b, r, q_roped, kc, vc):
    """Request r of batch b as a batch of its own over the same caches (same pages)."""
    starts = np.concatenate([[0], np.cumsum(b.new_len)])
    sub = W.ExtendBatch(b.name, b.num_q_heads, b.num_kv_heads, b.head_dim, b.page_size, b.rope_base, b.sigma,
                        b.cached_len[r:r + 1].copy(), b.new_len[r:r + 1].copy(),
                        np.ascontiguousarray(b.block_table[r:r + 1]), b.num_pages, None, None, None)
    return sub, q_roped[int(starts[r]):int(starts[r + 1])]


def test_batch_independence(E):
    """A request computed alone equals the same request inside a batch: bit for bit when both
    launches run the same configuration (row tile fixed, key ranges not cut, every request with
    more than 32 rows per kv head so that the same kernel variant is chosen), and within the
    parity bar of the oracle under the default planner, which cuts key ranges according to the
    whole batch."""
    b = _ragged(171, [900, 0, 130, 2500], [40, 150, 64, 17], heads=(8, 2), head_dim=128)
    q_roped, kc, vc = _oracle_inputs(b)
    ref = O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q_roped, kc, vc)
    starts = np.concatenate([[0], np.cumsum(b.new_len)])
    for fixed in (True, False):
        if fixed:
            E.efim_set_tuning(E.EFIM_TUNE_ROW_TILE, 128)
            E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, 0)
        try:
            whole = U.gpu_extend_attention(E, b, q_roped, kc, vc)
            for r in range(b.batch):
                sub, q_r = _one_request_of(b, r, q_roped, kc, vc)
                alone = U.gpu_extend_attention(E, sub, q_r, kc, vc)
                sl = slice(int(starts[r]), int(starts[r + 1]))
                if fixed:
                    assert np.array_equal(alone, whole[sl]), "request %d differs alone and in the batch" % r
                else:
                    U.assert_close(alone, ref[sl], "request %d alone" % r)
            if not fixed:
                U.assert_close(whole, ref, "batch")
        finally:
            E.efim_set_tuning(E.EFIM_TUNE_ROW_TILE, 0)
            E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, -1)


def test_sm_scale_argument(E):
    b = _ragged(99, [90], [20], heads=(2, 2), head_dim=64)
    q_roped, kc, vc = _oracle_inputs(b)
    ref = O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q_roped, kc, vc, sm_scale=0.31)
    got = U.gpu_extend_attention(E, b, q_roped, kc, vc, sm_scale=0.31)
    U.assert_close(got, ref, "scale", large_outputs=True)


def test_repeated_runs_are_deterministic(E):
    b = _ragged(100, [500, 0], [33, 200], heads=(4, 1), head_dim=128)
    q_roped, kc, vc = _oracle_inputs(b)
    first = U.gpu_extend_attention(E, b, q_roped, kc, vc)
    for _ in range(3):
        assert np.array_equal(U.gpu_extend_attention(E, b, q_roped, kc, vc), first)


def test_end_to_end_gpu_append_then_attention_equals_full_recompute(E):
    """Both calls on the GPU, cache built by the library itself in two shots (history, then
    the new tokens), against the oracle's cache-free recomputation of the whole prompt."""
    rng = np.random.default_rng(5)
    b = _ragged(101, [150, 0, 64], [45, 80, 17], heads=(4, 2), head_dim=128)
    # shot 1: the history as a miss (C = 0, N = C_r); shot 2: the new tokens
    hist = W.ExtendBatch(b.name, b.num_q_heads, b.num_kv_heads, b.head_dim, b.page_size, b.rope_base, b.sigma,
                         np.zeros_like(b.cached_len), b.cached_len.copy(), b.block_table, b.num_pages,
                         W.gaussian_bf16(rng, (int(b.cached_len.sum()), b.num_q_heads, b.head_dim), 1.0),
                         b.k_hist, b.v_hist)
    kc, vc = W.poisoned_cache(b), W.poisoned_cache(b)
    _, kc, vc = U.gpu_rope_append(E, hist, kc, vc)
    q_gpu, kc, vc = U.gpu_rope_append(E, b, kc, vc)
    got = U.gpu_extend_attention(E, b, q_gpu, kc, vc)
    hs = ns = 0
    for r in range(b.batch):
        c, n = int(b.cached_len[r]), int(b.new_len[r])
        k_all = np.concatenate([b.k_hist[hs:hs + c], b.k_new[ns:ns + n]])
        v_all = np.concatenate([b.v_hist[hs:hs + c], b.v_new[ns:ns + n]])
        q_all = np.concatenate([hist.q_new[hs:hs + c], b.q_new[ns:ns + n]])
        ref = O.full_recompute(q_all, k_all, v_all, b.rope_base)[-n:]
        U.assert_close(got[ns:ns + n], ref, "request %d" % r)
        hs += c
        ns += n


@pytest.mark.parametrize("d,rotary_dim,interleaved", [(128, 128, 0), (128, 64, 0), (128, 32, 1), (64, 64, 1),
                                                     (64, 16, 0), (128, 96, 0)])
def test_rope_append_table_bit_exact(E, d, rotary_dim, interleaved):
    """Caller-given frequency table (the Llama 3.1 long-context scaling of the plain table) and
    rotation of the leading rotary_dim elements only: roped q, K cache and V cache bit for bit."""
    b = _ragged(140 + rotary_dim, [0, 33, 4000, 250], [70, 5, 1, 129], heads=(8, 2), head_dim=d)
    table = O.scaled_inv_freq(rotary_dim, 5.0e5, 8.0, 1.0, 4.0, 8192)
    kc, vc = U.oracle_cache(b)
    kc_ref, vc_ref = kc.copy(), vc.copy()
    q_ref, _ = O.rope_append_table(b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new, b.k_new, b.v_new,
                                   kc_ref, vc_ref, table, rotary_dim, bool(interleaved))
    tab = torch.from_numpy(b.block_table).cuda()
    desc = U.make_desc(E, b, tab)
    q, kcd, vcd = U.dev_bits(b.q_new), U.dev_bits(kc), U.dev_bits(vc)
    E.efim_rope_append_table(desc, q, U.dev_bits(b.k_new), U.dev_bits(b.v_new), kcd, vcd, table, rotary_dim, interleaved)
    torch.cuda.synchronize()
    assert np.array_equal(U.host_bits(q), q_ref)
    assert np.array_equal(U.host_bits(kcd), kc_ref)
    assert np.array_equal(U.host_bits(vcd), vc_ref)
    if rotary_dim < d:   # the tail of every head row is the input, untouched
        assert np.array_equal(U.host_bits(q)[..., rotary_dim:], b.q_new[..., rotary_dim:])


@pytest.mark.parametrize("page_size", [8, 32, 64, 128, 256])
def test_other_page_sizes(E, page_size):
    """Pages of 8 to 256 tokens (a power of two): append bit-exact, attention within the bar, with
    and without cut key ranges, and the decode step on top of the resulting cache."""
    b = _ragged(300 + page_size, [0, 5, 700, 129, 2000], [200, 1, 33, 64, 7], heads=(8, 2), head_dim=128,
                page_size=page_size)
    assert b.page_size == page_size
    kc, vc = U.oracle_cache(b, fill=0xABCD)
    kc_ref, vc_ref = kc.copy(), vc.copy()
    q_ref, _ = O.rope_append(b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new, b.k_new, b.v_new,
                             kc_ref, vc_ref, b.rope_base)
    q_gpu, kc_gpu, vc_gpu = U.gpu_rope_append(E, b, kc, vc)
    assert np.array_equal(q_gpu, q_ref) and np.array_equal(kc_gpu, kc_ref) and np.array_equal(vc_gpu, vc_ref)
    kc_p, vc_p = U.oracle_cache(b)          # poisoned outside the requests
    q_ref, _ = O.rope_append(b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new, b.k_new, b.v_new,
                             kc_p, vc_p, b.rope_base)
    ref = O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q_ref, kc_p, vc_p)
    for split in (-1, 128):
        E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, split)
        try:
            got = U.gpu_extend_attention(E, b, q_ref, kc_p, vc_p)
        finally:
            E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, -1)
        # (requests with a handful of keys give outputs of magnitude 2-4, whose bf16 rounding
        # alone is up to 7.8e-3: the absolute bound is taken relative to the largest output)
        U.assert_close(got, ref, "page %d split %d" % (page_size, split), large_outputs=True)
