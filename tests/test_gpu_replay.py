"""GPU parity on the shapes of the service replay (EFIM Sec. 4.2): the (cached, new) lengths of a
steady-state round under each scheme come from the ORACLE's session pool; the library's
attention output for those batches is checked on sampled rows that the oracle computes."""
import numpy as np
import pytest
import torch

from oracle import session_oracle as SO
from paper_2505_21889_amd import workloads as W

import gpu_util as U

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def E():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2505_21889_amd import binding
    return binding


def oracle_round_lengths(scheme, round_index):
    docs = W.replay_documents()
    pool = SO.SessionPool(*W.REPLAY_MARKERS, granularity=16, always_psm=(scheme == "fim"))
    for k in range(round_index + 1):
        res = [pool.transform(u, p.tolist(), s.tolist()) for u, (p, s) in enumerate(docs[k])]
    c = np.array([r["cached_len"] for r in res], dtype=np.int32)
    n = np.array([r["new_len"] for r in res], dtype=np.int32)
    return c, n


@pytest.mark.parametrize("spec,scheme,round_index", [("replay", "efim", 2), ("replay", "fim", 2),
                                                     ("replay_mha", "efim", 1)])
def test_replay_round_matches_oracle_on_sampled_rows(E, spec, scheme, round_index):
    c, n = oracle_round_lengths(scheme, round_index)
    b = W.make_batch(spec, lengths=(c, n))
    worst, rel = U.sampled_check(E, b, heads_per_req=2, rows_per_head=12, seed=11 + round_index)
    print("%s %s round %d: max_abs %.3e rel_l2 %.3e" % (spec, scheme, round_index, worst, rel))


def test_replay_first_round_is_a_full_prefill(E):
    docs = W.replay_documents()
    n = np.array([len(p) + len(s) + 3 for p, s in docs[0]], dtype=np.int32)
    b = W.make_batch("replay", lengths=(np.zeros_like(n), n))
    worst, rel = U.sampled_check(E, b, heads_per_req=1, rows_per_head=8, seed=5)
    print("replay round 0: max_abs %.3e rel_l2 %.3e" % (worst, rel))
