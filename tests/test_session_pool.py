"""The library's session pool (host code behind the C ABI) against the oracle, value by value,
on seeded random edit sequences and on the error paths.  Integer work: everything is exact."""
import ctypes
import random

import numpy as np
import pytest

from oracle import session_oracle as SO
from paper_2505_21889_amd import binding as E

P, S, M = 32001, 32002, 32003
KEYS = ("order", "common_len", "inc_len", "suffix_len", "prompt_len", "cached_len", "new_len")


def _edit(rng, pre, suf):
    kind = rng.randrange(8)
    if kind <= 3:      # typing at the insertion point: the prefix tail grows
        pre = pre + [rng.randrange(32000) for _ in range(rng.randrange(1, 40))]
    elif kind == 4:    # growth at the head of the suffix
        suf = [rng.randrange(32000) for _ in range(rng.randrange(1, 20))] + suf
    elif kind == 5 and pre:   # an edit inside the prefix
        cut = rng.randrange(len(pre))
        pre = pre[:cut] + [rng.randrange(32000)] + pre[cut + rng.randrange(0, 3):]
    elif kind == 6 and suf:   # suffix shortened
        suf = suf[rng.randrange(len(suf)):]
    # kind 7: the same request again
    return pre, suf


@pytest.mark.parametrize("granularity", [1, 16])
@pytest.mark.parametrize("always_psm", [False, True])
def test_matches_oracle_on_random_sessions(granularity, always_psm):
    rng = random.Random(100 * granularity + always_psm)
    ref = SO.SessionPool(P, S, M, granularity=granularity, always_psm=always_psm)
    got = E.SessionPool(P, S, M, reuse_granularity=granularity, always_psm=always_psm)
    docs = {}
    orders = set()
    for step in range(1500):
        user = rng.randrange(12)
        if user not in docs:
            docs[user] = ([rng.randrange(32000) for _ in range(rng.randrange(0, 300))],
                          [rng.randrange(32000) for _ in range(rng.randrange(0, 300))])
        else:
            docs[user] = _edit(rng, *docs[user])
        pre, suf = docs[user]
        r = ref.transform(user, pre, suf)
        g = got.efim_session_transform(user, pre, suf)
        assert {k: r[k] for k in KEYS} == g, (step, user)
        assert got.efim_session_prompt(user).tolist() == r["prompt"], (step, user)
        orders.add(g["order"])
        if rng.randrange(200) == 0:  # the user leaves: both sides forget the session
            assert got.efim_session_drop(user) is True
            del ref.sessions[user], docs[user]
        assert got.efim_session_count() == len(ref.sessions)
    assert orders == ({E.EFIM_ORDER_PSM} if always_psm else {E.EFIM_ORDER_PSM, E.EFIM_ORDER_EFIM})
    got.close()


def test_error_returns_and_edge_cases():
    lib = E.raw_library()
    assert not lib.efim_session_pool_create(1, 1, 2, 1, 0)      # markers must differ
    assert not lib.efim_session_pool_create(1, 2, 3, 0, 0)      # granularity >= 1
    pool = E.SessionPool(P, S, M)
    info = E.EfimPromptInfo()
    arr = (ctypes.c_int32 * 4)(1, 2, S, 4)
    ok = (ctypes.c_int32 * 4)(1, 2, 3, 4)
    bad = E.EFIM_ERR_INVALID_ARG
    assert lib.efim_session_transform(None, 0, ok, 4, ok, 4, ctypes.byref(info)) == bad
    assert lib.efim_session_transform(pool.handle, 0, ok, 4, ok, 4, None) == bad
    assert lib.efim_session_transform(pool.handle, 0, ok, -1, ok, 4, ctypes.byref(info)) == bad
    assert lib.efim_session_transform(pool.handle, 0, None, 4, ok, 4, ctypes.byref(info)) == bad
    assert lib.efim_session_transform(pool.handle, 0, arr, 4, ok, 4, ctypes.byref(info)) == bad   # marker in prefix
    assert lib.efim_session_transform(pool.handle, 0, ok, 4, arr, 4, ctypes.byref(info)) == bad   # marker in suffix
    assert pool.efim_session_count() == 0                       # failed calls create nothing
    assert lib.efim_session_prompt(pool.handle, 0, None, 0) == 0
    assert lib.efim_session_prompt(pool.handle, 0, None, 3) == bad
    assert lib.efim_session_prompt(None, 0, None, 0) == bad
    assert lib.efim_session_drop(None, 0) == bad and lib.efim_session_count(None) == bad
    # empty prefix and suffix: the prompt is just the three markers
    r = pool.efim_session_transform(7, [], [])
    assert (r["prompt_len"], r["cached_len"], r["new_len"], r["order"]) == (3, 0, 3, E.EFIM_ORDER_PSM)
    assert pool.efim_session_prompt(7).tolist() == [P, S, M]
    buf = (ctypes.c_int32 * 2)()
    assert lib.efim_session_prompt(pool.handle, 7, buf, 2) == 3 and list(buf) == [P, S]  # truncated copy
    r = pool.efim_session_transform(7, [5], [])
    assert (r["order"], r["common_len"], r["inc_len"], r["cached_len"], r["new_len"]) == (E.EFIM_ORDER_EFIM, 0, 1, 3, 1)
    assert pool.efim_session_drop(7) is True and pool.efim_session_drop(7) is False
    lib.efim_session_pool_destroy(None)                         # NULL is accepted
    pool.close()


def test_large_user_ids_and_long_documents():
    ref = SO.SessionPool(P, S, M, granularity=16)
    got = E.SessionPool(P, S, M, reuse_granularity=16)
    rng = np.random.default_rng(3)
    user = 2**64 - 1
    pre = rng.integers(0, 32000, 50_000).tolist()
    suf = rng.integers(0, 32000, 30_000).tolist()
    for extra in (0, 1, 17, 400):
        pre = pre + rng.integers(0, 32000, extra).tolist()
        r = ref.transform(user, pre, suf)
        assert {k: r[k] for k in KEYS} == got.efim_session_transform(user, pre, suf)
    got.close()


def test_replay_lengths_follow_the_three_reuse_levels():
    """The benchmark's service replay: the library pool gives the oracle pool's lengths, and in
    rounds >= 1 they are the closed forms of the three reuse levels of EFIM Sec. 4.2 (none /
    prefix / prefix + suffix), with 16-token pages."""
    import bench as B
    from paper_2505_21889_amd import workloads as W
    docs = W.replay_documents()
    assert len(docs) == W.REPLAY_ROUNDS and all(len(r) == W.REPLAY_USERS for r in docs)
    mean_len = np.mean([[len(p) + len(s) + 3 for p, s in r] for r in docs])
    assert abs(mean_len - 2355) < 40          # the paper's average input length
    got = {sch: B.replay_lengths(E, W, sch, docs) for sch in ("baseline", "fim", "efim")}
    for sch, psm in (("fim", True), ("efim", False)):
        ref = SO.SessionPool(*W.REPLAY_MARKERS, granularity=16, always_psm=psm)
        for k, round_docs in enumerate(docs):
            for u, (p, s) in enumerate(round_docs):
                r = ref.transform(u, p.tolist(), s.tolist())
                assert (got[sch][k][0][u], got[sch][k][1][u]) == (r["cached_len"], r["new_len"])
    for k, round_docs in enumerate(docs):
        for u, (p, s) in enumerate(round_docs):
            total = len(p) + len(s) + 3
            assert (got["baseline"][k][0][u], got["baseline"][k][1][u]) == (0, total)
            if k == 0:
                assert got["fim"][k][0][u] == got["efim"][k][0][u] == 0
                continue
            old_p = len(docs[k - 1][u][0])
            assert got["fim"][k][0][u] == (1 + old_p) // 16 * 16                      # <P> + old prefix
            assert got["efim"][k][0][u] == (old_p + len(s) + 3) // 16 * 16            # everything before the new inc
            assert got["fim"][k][0][u] + got["fim"][k][1][u] == total
            assert got["efim"][k][0][u] + got["efim"][k][1][u] == total
