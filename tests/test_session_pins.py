"""Pins of the session-pool oracle (EFIM Sec. 3.1): closed forms worked out by hand from the
reuse figure of Sec. 2.2, the prompt -> (prefix, suffix) round trip, and a planted mistake."""
import random

from oracle import session_oracle as SO

P, S, M = -1, -2, -3
PREFIX0 = [1, 2, 3, 4, 5]
SUFFIX0 = [11, 12, 13, 14]


def pool(**kw):
    return SO.SessionPool(P, S, M, **kw)


def pick(res, *keys):
    return tuple(res[k] for k in keys)


def test_first_request_is_psm_and_computes_everything():
    r = pool().transform("u", PREFIX0, SUFFIX0)
    assert r["prompt"] == [P, 1, 2, 3, 4, 5, S, 11, 12, 13, 14, M]
    assert pick(r, "order", "common_len", "inc_len", "prompt_len", "cached_len", "new_len") == (SO.PSM, 5, 0, 12, 0, 12)


def test_prefix_tail_growth_reuses_everything_before_inc():
    # Sec. 2.2 reuse figure, growth at the prefix tail: EFIM keeps prefix AND suffix, PSM only the prefix
    e, f = pool(), pool(always_psm=True)
    for p_ in (e, f):
        p_.transform("u", PREFIX0, SUFFIX0)
    re_ = e.transform("u", PREFIX0 + [6, 7, 8], SUFFIX0)
    rf = f.transform("u", PREFIX0 + [6, 7, 8], SUFFIX0)
    assert re_["prompt"] == [P, 1, 2, 3, 4, 5, S, 11, 12, 13, 14, M, 6, 7, 8]
    assert pick(re_, "order", "common_len", "inc_len", "prompt_len", "cached_len", "new_len") == (SO.EFIM, 5, 3, 15, 12, 3)
    assert rf["prompt"] == [P, 1, 2, 3, 4, 5, 6, 7, 8, S, 11, 12, 13, 14, M]
    assert pick(rf, "order", "common_len", "inc_len", "prompt_len", "cached_len", "new_len") == (SO.PSM, 8, 0, 15, 6, 9)


def test_typing_on_keeps_the_whole_previous_prompt():
    e = pool()
    e.transform("u", PREFIX0, SUFFIX0)
    e.transform("u", PREFIX0 + [6, 7, 8], SUFFIX0)
    r = e.transform("u", PREFIX0 + [6, 7, 8, 9, 10], SUFFIX0)
    assert pick(r, "order", "common_len", "inc_len", "prompt_len", "cached_len", "new_len") == (SO.EFIM, 5, 5, 17, 15, 2)


def test_suffix_head_growth_falls_back_to_psm_and_keeps_the_prefix():
    for kw in ({}, {"always_psm": True}):
        e = pool(**kw)
        e.transform("u", PREFIX0, SUFFIX0)
        r = e.transform("u", PREFIX0, [10] + SUFFIX0)
        assert r["prompt"] == [P, 1, 2, 3, 4, 5, S, 10, 11, 12, 13, 14, M]
        # <P> + prefix + <S> survive: 7 tokens
        assert pick(r, "order", "prompt_len", "cached_len", "new_len") == (SO.PSM, 13, 7, 6)
        # the session now holds the new suffix: typing on is EFIM again relative to it
        r2 = e.transform("u", PREFIX0 + [6, 7], [10] + SUFFIX0)
        if kw:
            assert pick(r2, "order", "cached_len", "new_len") == (SO.PSM, 6, 9)
        else:
            assert pick(r2, "order", "common_len", "inc_len", "prompt_len", "cached_len", "new_len") == (SO.EFIM, 5, 2, 15, 13, 2)


def test_suffix_change_after_efim_rounds_resets_to_the_full_prefix():
    e = pool()
    e.transform("u", PREFIX0, SUFFIX0)
    e.transform("u", PREFIX0 + [6, 7, 8], SUFFIX0)                # <P>1-5<S>11-14<M>6 7 8
    r = e.transform("u", PREFIX0 + [6, 7, 8], [10] + SUFFIX0)     # <P>1-8<S>10 11-14<M>
    assert r["prompt"] == [P, 1, 2, 3, 4, 5, 6, 7, 8, S, 10, 11, 12, 13, 14, M]
    assert pick(r, "order", "common_len", "cached_len", "new_len") == (SO.PSM, 8, 6, 10)


def test_edited_prefix_is_not_an_extension():
    e = pool()
    e.transform("u", PREFIX0, SUFFIX0)
    r = e.transform("u", [1, 2, 9, 4, 5, 6], SUFFIX0)
    assert pick(r, "order", "common_len", "inc_len", "cached_len") == (SO.PSM, 6, 0, 3)
    r = e.transform("u", [1, 2, 9], SUFFIX0)  # shortened prefix
    assert pick(r, "order", "common_len", "cached_len") == (SO.PSM, 3, 4)


def test_identical_request_computes_one_token():
    e = pool()
    e.transform("u", PREFIX0, SUFFIX0)
    r = e.transform("u", PREFIX0, SUFFIX0)
    assert pick(r, "order", "prompt_len", "cached_len", "new_len") == (SO.PSM, 12, 11, 1)
    e.transform("u", PREFIX0 + [6], SUFFIX0)
    r = e.transform("u", PREFIX0 + [6], SUFFIX0)
    assert pick(r, "order", "inc_len", "prompt_len", "cached_len", "new_len") == (SO.EFIM, 1, 13, 12, 1)


def test_page_granular_reuse_rounds_down():
    e = pool(granularity=4)
    e.transform("u", PREFIX0 + [6], SUFFIX0)                       # 13 tokens
    r = e.transform("u", PREFIX0 + [6, 7, 8], SUFFIX0)
    assert pick(r, "cached_len", "new_len") == (12, 3)
    e16 = pool(granularity=16)
    e16.transform("u", list(range(100, 140)), SUFFIX0)             # 47 tokens
    r = e16.transform("u", list(range(100, 150)), SUFFIX0)
    assert pick(r, "order", "cached_len", "new_len") == (SO.EFIM, 32, 25)


def test_users_do_not_share_sessions():
    e = pool()
    e.transform("a", PREFIX0, SUFFIX0)
    r = e.transform("b", PREFIX0 + [6], SUFFIX0)
    assert pick(r, "order", "cached_len") == (SO.PSM, 0)
    r = e.transform("a", PREFIX0 + [6], SUFFIX0)
    assert pick(r, "order", "cached_len") == (SO.EFIM, 12)


def _split_prompt(prompt):
    ip, is_, im = prompt.index(P), prompt.index(S), prompt.index(M)
    assert ip == 0 and prompt.count(P) == prompt.count(S) == prompt.count(M) == 1
    return prompt[1:is_] + prompt[im + 1:], prompt[is_ + 1:im]


def test_prompt_round_trip_on_random_edit_sequences():
    rng = random.Random(7)
    for mode in (False, True):
        e = pool(always_psm=mode, granularity=rng.choice([1, 4, 16]))
        state = {}
        last_prompt = {}
        for step in range(600):
            u = rng.randrange(5)
            pre, suf = state.get(u, ([], []))
            kind = rng.randrange(6)
            if kind <= 2:
                pre = pre + [rng.randrange(1000) for _ in range(rng.randrange(1, 9))]
            elif kind == 3:
                suf = [rng.randrange(1000) for _ in range(rng.randrange(1, 5))] + suf
            elif kind == 4 and pre:
                pre = pre[:rng.randrange(len(pre))] + [rng.randrange(1000)]
            state[u] = (pre, suf)
            r = e.transform(u, pre, suf)
            assert _split_prompt(r["prompt"]) == (pre, suf)
            assert r["prompt_len"] == len(pre) + len(suf) + 3 == r["cached_len"] + r["new_len"]
            assert r["common_len"] + r["inc_len"] == len(pre) and (r["order"] == SO.EFIM) == (r["inc_len"] > 0)
            # reuse is a true token-prefix match with what was sent before, page aligned, never everything
            prev = last_prompt.get(u, [])
            assert r["prompt"][:r["cached_len"]] == prev[:r["cached_len"]]
            assert r["cached_len"] % e.granularity == 0 and 1 <= r["new_len"]
            if r["cached_len"] + e.granularity < r["prompt_len"] and r["cached_len"] + e.granularity <= len(prev):
                lo = r["cached_len"]
                assert r["prompt"][lo:lo + e.granularity] != prev[lo:lo + e.granularity]
            last_prompt[u] = r["prompt"]


def test_planted_mistake_is_caught():
    # a pool that stores the whole new prefix after an EFIM request loses the suffix on the next round
    class Wrong(SO.SessionPool):
        def transform(self, user, prefix, suffix):
            r = super().transform(user, prefix, suffix)
            self.sessions[user]["prefix"] = list(prefix)
            return r
    e = Wrong(P, S, M)
    e.transform("u", PREFIX0, SUFFIX0)
    e.transform("u", PREFIX0 + [6, 7, 8], SUFFIX0)
    r = e.transform("u", PREFIX0 + [6, 7, 8, 9, 10], SUFFIX0)
    assert pick(r, "cached_len", "new_len") != (15, 2)
