"""Plan objects: the attention call and the decode step as pure kernel launches over a work list
that lives in the caller's workspace.  Results bit for bit those of the batch-description calls
(themselves held to the oracle), from several threads' worth of plans at once, and under HIP graph
capture: a captured decode step replayed with eager work in between, every replay against the
oracle."""
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


def _batch(seed, cached, new, heads=(8, 2), d=128, **kw):
    return W.make_batch("c1", seed=seed, lengths=(np.array(cached, dtype=np.int32), np.array(new, dtype=np.int32)),
                        heads=heads, head_dim=d, **kw)


def _planned_attention(E, b, q_roped, kc, vc, stream=None):
    table = torch.from_numpy(b.block_table).cuda()
    desc = U.make_desc(E, b, table)
    plan = E.Plan(desc)
    nbytes = E.efim_plan_workspace_bytes(plan)
    ws = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device="cuda")   # contents must not matter
    q, kcd, vcd = U.dev_bits(q_roped), U.dev_bits(kc), U.dev_bits(vc)
    out = torch.full(q.shape, 0x7FC1, dtype=torch.int16, device="cuda")
    E.efim_plan_upload(plan, ws, nbytes, stream)
    for _ in range(2):   # the second launch finds the arrival counters back at zero
        out.fill_(0x7FC1)
        E.efim_extend_attention_planned(plan, table, q, kcd, vcd, out, 0.0, ws, stream)
    torch.cuda.synchronize()
    plan.close()
    return U.host_bits(out)


@pytest.mark.parametrize("cached,new,heads,d,knobs", [
    ([700, 0, 300, 5000], [40, 300, 2, 3], (4, 2), 128, {}),                      # cut key ranges, second-launch merge
    ([5000, 1300, 64], [1, 1, 1], (8, 2), 128, {}),                               # few rows: merge inside the kernel
    ([5000, 1300, 64], [3, 2, 1], (8, 2), 128, {"SPLIT_KV": 256, "FUSED_MERGE": 1}),
    ([100, 0], [40, 90], (4, 4), 64, {}),
])
def test_planned_attention_equals_the_batch_call(E, cached, new, heads, d, knobs):
    b = _batch(501, cached, new, heads, d)
    q_roped, kc, vc = U.oracle_inputs(b)
    ref = O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q_roped, kc, vc)
    for key, val in knobs.items():
        E.efim_set_tuning(getattr(E, "EFIM_TUNE_" + key), val)
    try:
        want = U.gpu_extend_attention(E, b, q_roped, kc, vc)
        got = _planned_attention(E, b, q_roped, kc, vc)
    finally:
        E.efim_set_tuning(E.EFIM_TUNE_SPLIT_KV, -1)
        E.efim_set_tuning(E.EFIM_TUNE_FUSED_MERGE, -1)
    assert np.array_equal(got, want)
    U.assert_close(got, ref, "planned")


class DecodeCase:
    def __init__(self, E, seed, cached, heads=(8, 2), d=128, new=None):
        c = np.array(cached, dtype=np.int32)
        n = np.ones_like(c) if new is None else np.array(new, dtype=np.int32)
        self.b = b = _batch(seed, c, n, heads, d)
        self.kc0, self.vc0 = U.oracle_cache(b)
        kc, vc = self.kc0.copy(), self.vc0.copy()
        q_roped, _ = O.rope_append(b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new, b.k_new, b.v_new,
                                   kc, vc, b.rope_base)
        self.kc_ref, self.vc_ref = kc, vc
        self.ref = O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q_roped, kc, vc)
        self.table = torch.from_numpy(b.block_table).cuda()
        self.desc = U.make_desc(E, b, self.table)
        self.q, self.k_new, self.v_new = U.dev_bits(b.q_new), U.dev_bits(b.k_new), U.dev_bits(b.v_new)
        self.kcd, self.vcd = U.dev_bits(self.kc0), U.dev_bits(self.vc0)
        self.out = torch.full(self.q.shape, 0x7FC1, dtype=torch.int16, device="cuda")
        self.plan = E.Plan(self.desc, decode=True)
        self.nbytes = E.efim_plan_workspace_bytes(self.plan)
        self.ws = torch.full((self.nbytes,), 0x5A, dtype=torch.uint8, device="cuda")

    def launch(self, E, stream=None):
        E.efim_decode_step_planned(self.plan, self.table, self.q, self.k_new, self.v_new, self.kcd, self.vcd,
                                   self.out, self.b.rope_base, 0, 0.0, self.ws, stream)

    def check(self, what):
        assert np.array_equal(U.host_bits(self.kcd), self.kc_ref), what + ": k_cache"
        assert np.array_equal(U.host_bits(self.vcd), self.vc_ref), what + ": v_cache"
        U.assert_close(U.host_bits(self.out), self.ref, what)


@pytest.mark.parametrize("cached,heads,d", [([0, 1, 15, 16, 17, 63, 64, 300, 1000, 2047], (8, 2), 128),
                                            ([777, 31, 4096], (28, 4), 128), ([0, 100, 1025, 48], (8, 4), 64)])
def test_planned_decode_step_equals_the_batch_call(E, cached, heads, d):
    case = DecodeCase(E, 520 + d, cached, heads, d)
    b = case.b
    # the batch-description call on its own copies of the caches
    kcd, vcd = U.dev_bits(case.kc0), U.dev_bits(case.vc0)
    want = torch.full(case.q.shape, 0x7FC1, dtype=torch.int16, device="cuda")
    nbytes = E.efim_decode_workspace_bytes(case.desc)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    E.efim_decode_step(case.desc, case.q, case.k_new, case.v_new, kcd, vcd, want, b.rope_base, 0, 0.0, ws, nbytes)
    E.efim_plan_upload(case.plan, case.ws, case.nbytes)
    case.launch(E)
    torch.cuda.synchronize()
    case.check("planned decode step")
    assert np.array_equal(U.host_bits(case.out), U.host_bits(want))
    assert np.array_equal(U.host_bits(case.q), b.q_new), "q must stay as given"


def test_planned_short_step_equals_the_batch_call(E):
    """Several new tokens per request through the plan-object call."""
    case = DecodeCase(E, 540, [60, 63, 64, 56, 120, 0, 127, 4095], (8, 2), 128, new=[8, 1, 3, 4, 8, 2, 5, 7])
    b = case.b
    kcd, vcd = U.dev_bits(case.kc0), U.dev_bits(case.vc0)
    want = torch.full(case.q.shape, 0x7FC1, dtype=torch.int16, device="cuda")
    nbytes = E.efim_decode_workspace_bytes(case.desc)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    E.efim_decode_step(case.desc, case.q, case.k_new, case.v_new, kcd, vcd, want, b.rope_base, 0, 0.0, ws, nbytes)
    E.efim_plan_upload(case.plan, case.ws, case.nbytes)
    case.launch(E)
    torch.cuda.synchronize()
    case.check("planned short step")
    assert np.array_equal(U.host_bits(case.out), U.host_bits(want))


def test_captured_decode_step_replays(E):
    """A decode step captured into a HIP graph (kernels only: no copy, no memset, no event) and
    replayed three times, with eager work of the library and synchronisations in between; after
    every replay the caches and the output are compared with the oracle.  (Replaying the same step
    writes the same token into the same slot again.)"""
    case = DecodeCase(E, 531, [4100, 17, 900, 2047, 64, 5, 3000, 1200], (8, 2), 128)
    other = DecodeCase(E, 532, [333, 2500], (4, 4), 128)
    stream = torch.cuda.Stream()
    E.efim_plan_upload(case.plan, case.ws, case.nbytes, stream)
    E.efim_plan_upload(other.plan, other.ws, other.nbytes)
    stream.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        case.launch(E, torch.cuda.current_stream())
    for replay in range(3):
        # forget the previous result: cache slots of the new tokens and the output
        case.kcd.copy_(U.dev_bits(case.kc0))
        case.vcd.copy_(U.dev_bits(case.vc0))
        case.out.fill_(0x7FC1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        case.check("replay %d" % replay)
        # eager work of the library between the replays: another planned step and a batch call
        other.launch(E)
        torch.cuda.synchronize()
        other.check("eager step after replay %d" % replay)
        other.kcd.copy_(U.dev_bits(other.kc0))
        other.vcd.copy_(U.dev_bits(other.vc0))
    # the plan was cut into several key ranges, so the arrival counters were used and put back
    items = E.efim_extend_plan_items(case.desc)
    assert (items["partial_slot"] >= 0).any()


def test_plans_share_nothing(E):
    """Two plans with their own workspaces launched alternately on two streams: neither sees the
    other (no process-wide state behind the planned calls)."""
    a = DecodeCase(E, 541, [3000, 100, 64, 1500], (8, 2), 128)
    c = DecodeCase(E, 542, [2200, 9], (4, 1), 64)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    E.efim_plan_upload(a.plan, a.ws, a.nbytes, s1)
    E.efim_plan_upload(c.plan, c.ws, c.nbytes, s2)
    for _ in range(4):
        a.launch(E, s1)
        c.launch(E, s2)
    torch.cuda.synchronize()
    a.check("plan a")
    c.check("plan c")


def test_planned_calls_reject_bad_arguments(E):
    b = _batch(551, [40, 3], [1, 1], (4, 4), 64)
    table = torch.from_numpy(b.block_table).cuda()
    desc = U.make_desc(E, b, table)
    attn, dec = E.Plan(desc), E.Plan(desc, decode=True)
    ws = torch.empty(max(E.efim_plan_workspace_bytes(attn), E.efim_plan_workspace_bytes(dec)), dtype=torch.uint8, device="cuda")
    with pytest.raises(E.EfimError) as err:
        E.efim_plan_upload(attn, ws, 16)
    assert err.value.status == E.EFIM_ERR_WORKSPACE
    with pytest.raises(E.EfimError):   # a decode call on an attention plan
        E.efim_decode_step_planned(attn, table, 1 << 20, 2 << 20, 3 << 20, 4 << 20, 5 << 20, 6 << 20, 1e4, 0, 0.0, ws)
    with pytest.raises(E.EfimError):   # and the reverse
        E.efim_extend_attention_planned(dec, table, 1 << 20, 2 << 20, 3 << 20, 4 << 20, 0.0, ws)
    with pytest.raises(E.EfimError):   # misaligned query pointer
        E.efim_extend_attention_planned(attn, table, (1 << 20) + 2, 2 << 20, 3 << 20, 4 << 20, 0.0, ws)
    b2 = _batch(552, [40, 3], [1, 17], (4, 4), 64)
    with pytest.raises(E.EfimError):   # not a decode batch
        E.Plan(U.make_desc(E, b2, table), decode=True)
