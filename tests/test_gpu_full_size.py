"""GPU parity at the full sizes of the benchmark workloads, in the launch configuration the
benchmark times (default planner settings).  The whole output of every benchmark workload is
compared; only the 131072-token context is checked on sampled (head, row) outputs that the
oracle computes one by one."""
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


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5"])
def test_full_output_matches_oracle(E, name):
    """Every element of the output of every benchmark workload, the headline mixed step
    included, against the oracle at the flat bar (max abs 1e-2, relative L2 5e-3)."""
    b = W.make_batch(name)
    max_abs, rel = U.full_check(E, b, name)
    print("%s: max_abs %.3e rel_l2 %.3e" % (name, max_abs, rel))


def test_c5_rope_append_bit_exact_on_sampled_requests(E):
    """The library appends the whole mixed step; the oracle re-does a sample of its requests
    (hits and misses) and every byte it writes, and the roped queries, must be identical."""
    b = W.make_batch("c5", with_history=False)
    kc = np.full(b.cache_shape(), 0x5A5A, dtype=np.uint16)
    vc = np.full(b.cache_shape(), 0x5A5A, dtype=np.uint16)
    q_gpu, kc_gpu, vc_gpu = U.gpu_rope_append(E, b, kc, vc)
    hits = [r for r in range(b.batch) if b.cached_len[r] > 0][:3]
    misses = [r for r in range(b.batch) if b.cached_len[r] == 0][:3]
    starts = np.concatenate([[0], np.cumsum(b.new_len)])
    touched = np.zeros((b.num_pages, b.page_size), dtype=bool)
    for r in range(b.batch):
        for p_ in range(int(b.cached_len[r]), int(b.cached_len[r] + b.new_len[r])):
            touched[int(b.block_table[r, p_ // b.page_size]), p_ % b.page_size] = True
    # no byte outside the appended slots changed
    assert np.all(kc_gpu.transpose(0, 2, 1, 3)[~touched] == 0x5A5A)
    assert np.all(vc_gpu.transpose(0, 2, 1, 3)[~touched] == 0x5A5A)
    for r in hits + misses:
        sl = slice(int(starts[r]), int(starts[r + 1]))
        kc_ref = np.full(b.cache_shape(), 0x5A5A, dtype=np.uint16)
        vc_ref = np.full(b.cache_shape(), 0x5A5A, dtype=np.uint16)
        q_ref, _ = O.rope_append(b.cached_len[r:r + 1], b.new_len[r:r + 1], b.block_table[r:r + 1], b.page_size,
                                 b.q_new[sl], b.k_new[sl], b.v_new[sl], kc_ref, vc_ref, b.rope_base)
        assert np.array_equal(q_gpu[sl], q_ref)
        pages = b.block_table[r, : -(-int(b.cached_len[r] + b.new_len[r]) // b.page_size)]
        assert np.array_equal(kc_gpu[pages], kc_ref[pages])
        assert np.array_equal(vc_gpu[pages], vc_ref[pages])


@pytest.mark.parametrize("heads,d,new", [((4, 1), 128, [3, 40]), ((2, 2), 64, [1, 1])])
def test_one_very_long_context(E, heads, d, new):
    """131072 cached tokens behind one request (2048 key tiles cut into many ranges, a block table
    of 8192 pages) next to a short one; sampled rows (first, middle and last always) of a query
    head per kv head against the oracle."""
    c = np.array([131072, 300], dtype=np.int32)
    b = W.make_batch("c1", seed=131, lengths=(c, np.array(new, dtype=np.int32)), heads=heads, head_dim=d)
    assert b.block_table.shape[1] >= 8192
    items = E.efim_extend_plan_items(U.make_desc(E, b, torch.from_numpy(b.block_table).cuda()))
    assert len(items) > 64, "the long request is expected to be cut into many key ranges"
    worst, rel = U.sampled_check(E, b, heads_per_req=heads[1], rows_per_head=max(new), seed=9)
    print("long context: max_abs %.3e rel_l2 %.3e" % (worst, rel))
