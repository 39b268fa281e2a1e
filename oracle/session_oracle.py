"""TEST INFRASTRUCTURE ONLY -- never imported by the product path.

Plain-Python reference of the per-user session pool that rewrites an infilling request from
FIM order to EFIM order (EFIM Sec. 3.1, steps 1-5 of the prompt transformation figure), plus
the bookkeeping a prefix-matching KV cache does with the result.

Token sequences are Python lists of ints.  A prompt is laid out as

    PSM :  <P> prefix <S> suffix <M>
    EFIM:  <P> common <S> suffix <M> inc        (prefix == common + inc)

so the EFIM prompt of an unchanged (common, suffix) pair only ever grows at its tail.

Readings taken where the paper leaves a choice (each is listed in the design notes):
  * the session keeps the prefix and suffix of the previous request *as it was laid out in
    the prompt*: after an EFIM request that is the common part, not the whole prefix, so the
    next EFIM prompt extends the cached one whenever the user keeps typing;
  * step 5 names only growth at the head of the suffix; every other change that step 4 does
    not cover (edited or shortened prefix, changed suffix) is handled the same way: PSM
    order, session replaced by the new (prefix, suffix);
  * a request identical to the stored session (no new prefix content) keeps PSM order;
  * the cache reuses the longest common token prefix of this prompt and the user's previous
    one, rounded down to `granularity` tokens (a paged cache reuses whole pages) and never
    the whole prompt: at least one token is computed so that there is something to sample
    from.

Parity: every value here is an integer or a token list; the checks in
tests/test_session_pins.py tie it to closed forms worked out by hand from the paper's
reuse figure (Sec. 2.2) and to the round trip prompt -> (prefix, suffix).
"""
from __future__ import annotations

PSM = 0
EFIM = 1


def common_prefix_len(a, b):
    """Number of leading positions at which the two sequences agree."""
    n = 0
    while n < len(a) and n < len(b) and a[n] == b[n]:
        n += 1
    return n


class SessionPool:
    def __init__(self, tok_p, tok_s, tok_m, granularity=1, always_psm=False):
        self.tok_p, self.tok_s, self.tok_m = tok_p, tok_s, tok_m
        self.granularity = granularity
        self.always_psm = always_psm  # the experiment's "FIM" scheme: PSM order, cache reuse on
        self.sessions = {}            # user -> {"prefix": [...], "suffix": [...], "prompt": [...]}

    def transform(self, user, prefix, suffix):
        prefix, suffix = list(prefix), list(suffix)
        session = self.sessions.get(user)                       # step 1
        order, common, inc = PSM, prefix, []
        if session is None:                                     # step 2: new session, PSM
            session = {"prefix": prefix, "suffix": suffix, "prompt": []}
            self.sessions[user] = session
        else:                                                   # step 3: compare with the session
            old_prefix, old_suffix = session["prefix"], session["suffix"]
            grew = (len(prefix) > len(old_prefix) and prefix[:len(old_prefix)] == old_prefix)
            if suffix == old_suffix and grew and not self.always_psm:
                order = EFIM                                    # step 4: common + suffix + inc
                common, inc = old_prefix, prefix[len(old_prefix):]
            elif suffix == old_suffix and prefix == old_prefix:
                pass                                            # nothing new: same prompt again
            else:                                               # step 5 (and all other edits): PSM
                session["prefix"], session["suffix"] = prefix, suffix
        prompt = [self.tok_p] + common + [self.tok_s] + suffix + [self.tok_m] + inc
        match = common_prefix_len(session["prompt"], prompt)
        cached = min(match, len(prompt) - 1)
        cached -= cached % self.granularity
        session["prompt"] = prompt
        return {
            "order": order, "common_len": len(common), "inc_len": len(inc), "suffix_len": len(suffix),
            "prompt": prompt, "prompt_len": len(prompt), "cached_len": cached, "new_len": len(prompt) - cached,
        }
