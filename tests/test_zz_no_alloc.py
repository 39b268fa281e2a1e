"""efim_extend_attention_static (the entry point that allocates nothing: work list and partial
results in a fixed array of the library) against efim_extend_attention on the same inputs:
two calls in a row, the second with a smaller batch, outputs bit for bit; sizes beyond the
fixed array are refused."""
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


def _batch(seed, cached, new, heads, d):
    return W.make_batch("c1", seed=seed, lengths=(np.array(cached, dtype=np.int32), np.array(new, dtype=np.int32)),
                        heads=heads, head_dim=d)


def _both_ways(E, b):
    """(out of efim_extend_attention, out of efim_extend_attention_static, oracle reference)."""
    q_roped, kc, vc = U.oracle_inputs(b)
    ref = O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q_roped, kc, vc)
    want = U.gpu_extend_attention(E, b, q_roped, kc, vc)
    table = torch.from_numpy(b.block_table).cuda()
    desc = U.make_desc(E, b, table)
    q, kcd, vcd = U.dev_bits(q_roped), U.dev_bits(kc), U.dev_bits(vc)
    out = torch.full(q.shape, 0x7FC1, dtype=torch.int16, device="cuda")
    torch.cuda.synchronize()
    E.efim_extend_attention_static(desc, q, kcd, vcd, out, 0.0)
    torch.cuda.synchronize()
    return want, U.host_bits(out), ref, desc


def test_two_calls_in_a_row_second_smaller(E):
    # first: long cached contexts behind few rows -> key ranges are cut, partial results and a
    # merge pass use the fixed array; then a smaller batch (fewer, shorter requests) that also
    # cuts its key ranges and must not see anything the first call left behind
    big = _batch(401, [6000, 3000, 4500, 0, 800], [3, 1, 40, 150, 9], (8, 2), 128)
    small = _batch(402, [2500, 70], [2, 5], (8, 2), 128)
    for b in (big, small):
        want, got, ref, desc = _both_ways(E, b)
        items = E.efim_extend_plan_items(desc)
        assert (items["partial_slot"] >= 0).any(), "the case is meant to use partial results"
        assert np.array_equal(got, want)
        U.assert_close(got, ref, "static")
    # and the first one again: the array is reused from the start
    want, got, ref, _ = _both_ways(E, big)
    assert np.array_equal(got, want)


def test_without_split_and_other_head_dim(E):
    b = _batch(403, [100, 0], [40, 90], (4, 4), 64)
    want, got, ref, _ = _both_ways(E, b)
    assert np.array_equal(got, want)
    U.assert_close(got, ref, "static d64")


def test_sizes_beyond_the_fixed_array_are_refused(E):
    # the GQA workload (32 requests, 56..448 rows per kv head, key ranges cut for balance) keeps
    # about 67 MB of partial results: more than the 30 MiB of the array
    b = W.make_batch("c3", with_history=False, with_tensors=False)
    table = torch.from_numpy(b.block_table).cuda()
    desc = U.make_desc(E, b, table)
    assert E.efim_extend_workspace_bytes(desc) > E.efim_extend_static_limit_bytes()
    with pytest.raises(E.EfimError) as err:
        E.efim_extend_attention_static(desc, 1 << 20, 2 << 20, 3 << 20, 4 << 20, 0.0)
    assert err.value.status == E.EFIM_ERR_WORKSPACE
