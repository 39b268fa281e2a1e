"""Where the kernels read their work list from must not show in the results.  The first launch of a
batch reads the list from pinned host memory; later launches of the unchanged batch read a copy in
device memory (two buffers used in turn).  Every output here is compared bit for bit with the one
computed with the copies switched off, itself held to the oracle."""
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


class Case:
    """One batch resident on the device, with its oracle result."""

    def __init__(self, E, seed, cached, new, heads=(8, 2), head_dim=128):
        c, n = np.array(cached, dtype=np.int32), np.array(new, dtype=np.int32)
        self.b = b = W.make_batch("c1", seed=seed, lengths=(c, n), heads=heads, head_dim=head_dim)
        q_roped, kc, vc = U.oracle_inputs(b)
        self.ref = O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q_roped, kc, vc)
        self.table = torch.from_numpy(b.block_table).cuda()
        self.desc = U.make_desc(E, b, self.table)
        self.q, self.kc, self.vc = U.dev_bits(q_roped), U.dev_bits(kc), U.dev_bits(vc)

    def run(self, E, stream=None):
        out = torch.full(self.q.shape, 0x7FC1, dtype=torch.int16, device="cuda")
        nbytes = E.efim_extend_workspace_bytes(self.desc)
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        E.efim_extend_attention(self.desc, self.q, self.kc, self.vc, out, 0.0, ws, nbytes, stream)
        torch.cuda.synchronize()
        return U.host_bits(out)

    def launch(self, E, stream):
        """Enqueues one call on `stream` without waiting; returns the output tensor."""
        out = torch.full(self.q.shape, 0x7FC1, dtype=torch.int16, device="cuda")
        nbytes = E.efim_extend_workspace_bytes(self.desc)
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        E.efim_extend_attention(self.desc, self.q, self.kc, self.vc, out, 0.0, ws, nbytes, stream)
        return out, ws

    def baseline(self, E):
        E.efim_set_tuning(E.EFIM_TUNE_DEVICE_PLAN, 0)
        try:
            got = self.run(E)
        finally:
            E.efim_set_tuning(E.EFIM_TUNE_DEVICE_PLAN, 1)
        U.assert_close(got, self.ref, "work list read from host memory")
        return got


@pytest.fixture(scope="module")
def cases(E):
    # split key ranges with a merge, many small items, and one request with several row tiles
    return [Case(E, 301, [0, 17, 640, 3000, 5, 2047], [1, 1, 1, 1, 1, 1]),
            Case(E, 302, [100, 0, 1000], [300, 64, 7], heads=(4, 4)),
            Case(E, 303, [12, 4000], [16, 3], heads=(8, 4), head_dim=64)]


def test_repeated_launches_of_one_batch(E, cases):
    for c in cases:
        want = c.baseline(E)
        for i in range(5):      # the first reads the pinned slot, the rest the device copy
            assert np.array_equal(c.run(E), want), "launch %d differs" % i


def test_batches_taking_turns(E, cases):
    want = [c.baseline(E) for c in cases]
    order = [0, 1, 0, 1, 2, 2, 0, 0, 0, 1, 1, 2, 0, 2, 2, 2, 1]     # every change of batch is a new plan
    for step, i in enumerate(order):
        assert np.array_equal(cases[i].run(E), want[i]), "step %d (batch %d) differs" % (step, i)


def test_launches_without_waiting_in_between(E, cases):
    """Launches queued back to back: the copy of a new work list is enqueued behind kernels that
    may still be reading the buffer's previous contents."""
    want = [c.baseline(E) for c in cases]
    outs = []
    for rep in range(3):
        for i, c in enumerate(cases):
            for _ in range(3):
                out = torch.full(c.q.shape, 0x7FC1, dtype=torch.int16, device="cuda")
                nbytes = E.efim_extend_workspace_bytes(c.desc)
                ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
                E.efim_extend_attention(c.desc, c.q, c.kc, c.vc, out, 0.0, ws, nbytes)
                outs.append((i, out, ws))
    torch.cuda.synchronize()
    for n, (i, out, _) in enumerate(outs):
        assert np.array_equal(U.host_bits(out), want[i]), "queued launch %d (batch %d) differs" % (n, i)


def test_many_queued_launches_on_two_streams(E, cases):
    """160 launches queued without waiting, more than the library keeps launch tokens for: the
    batch changes every 7 calls and the stream every 5, so completion events are shared by runs
    of calls of different lengths and tokens, pinned buffers and device copies all come round
    several times."""
    want = [c.baseline(E) for c in cases]
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    side.wait_stream(main)
    outs = []
    for n in range(160):
        i = (n // 7) % len(cases)
        st = side if (n // 5) % 2 else main
        c = cases[i]
        with torch.cuda.stream(st):
            out = torch.full(c.q.shape, 0x7FC1, dtype=torch.int16, device="cuda")
            nbytes = E.efim_extend_workspace_bytes(c.desc)
            ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
            E.efim_extend_attention(c.desc, c.q, c.kc, c.vc, out, 0.0, ws, nbytes, st)
        outs.append((i, out, ws))
    torch.cuda.synchronize()
    for n, (i, out, _) in enumerate(outs):
        assert np.array_equal(U.host_bits(out), want[i]), "queued launch %d (batch %d) differs" % (n, i)


def test_a_second_stream_reads_the_copy(E, cases):
    c = cases[0]
    want = c.baseline(E)
    side = torch.cuda.Stream()
    assert np.array_equal(c.run(E), want)               # enqueues the copy on the current stream
    with torch.cuda.stream(side):
        for _ in range(2):
            assert np.array_equal(c.run(E, side), want)
    assert np.array_equal(c.run(E), want)
    # a new work list arrives on the side stream while the other buffer was last read on the main one
    d = cases[1]
    want_d = d.baseline(E)
    with torch.cuda.stream(side):
        assert np.array_equal(d.run(E, side), want_d)
        assert np.array_equal(d.run(E, side), want_d)
    assert np.array_equal(d.run(E), want_d)
    assert np.array_equal(c.run(E), want)


def test_an_older_reader_on_a_third_stream(E, cases):
    """Stream A reads a work list's device copy behind a long queue of other work; stream B then
    reads the same copy and goes on to two new work lists, the second of which refills the buffer
    A's launch is still to read.  The refill must wait for A's launch (readers are chained), so
    every output is what it is with the copies switched off."""
    c, d, e = cases
    want = [x.baseline(E) for x in cases]
    a_stream, b_stream = torch.cuda.Stream(), torch.cuda.Stream()
    assert np.array_equal(c.run(E), want[0])            # first launch: enqueues the copy
    torch.cuda.synchronize()
    big = torch.empty(8192, 8192, dtype=torch.float32, device="cuda").normal_()
    held = []
    with torch.cuda.stream(a_stream):
        for _ in range(6):
            big = big @ big * 1e-4                        # keeps stream A busy for a while
        held.append(c.launch(E, a_stream))                # reader on A, far back in A's queue
    with torch.cuda.stream(b_stream):
        held.append(c.launch(E, b_stream))                # reader on B
        out_d = [d.launch(E, b_stream) for _ in range(2)] # new list: the other buffer
        out_e = [e.launch(E, b_stream) for _ in range(2)] # new list: refills the buffer A still reads
    torch.cuda.synchronize()
    for out, _ in held:
        assert np.array_equal(U.host_bits(out), want[0])
    for out, _ in out_d:
        assert np.array_equal(U.host_bits(out), want[1])
    for out, _ in out_e:
        assert np.array_equal(U.host_bits(out), want[2])
    E.efim_stream_release(a_stream)
    E.efim_stream_release(b_stream)


def test_decode_steps_repeat(E):
    """The fused decode step launched again with the unchanged batch (it rewrites the same cache
    slots with the same values) gives the same bits from either copy of the work list."""
    c = np.array([0, 9, 500, 2500, 64], dtype=np.int32)
    b = W.make_batch("c1", seed=310, lengths=(c, np.ones_like(c)), heads=(8, 2), head_dim=128)
    kc, vc = U.oracle_cache(b)
    table = torch.from_numpy(b.block_table).cuda()
    desc = U.make_desc(E, b, table)
    q, k_new, v_new = U.dev_bits(b.q_new), U.dev_bits(b.k_new), U.dev_bits(b.v_new)
    kcd, vcd = U.dev_bits(kc), U.dev_bits(vc)
    nbytes = E.efim_decode_workspace_bytes(desc)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")

    def step():
        out = torch.full(q.shape, 0x7FC1, dtype=torch.int16, device="cuda")
        E.efim_decode_step(desc, q, k_new, v_new, kcd, vcd, out, b.rope_base, 0, 0.0, ws, ws.numel())
        torch.cuda.synchronize()
        return U.host_bits(out)

    E.efim_set_tuning(E.EFIM_TUNE_DEVICE_PLAN, 0)
    try:
        want = step()
    finally:
        E.efim_set_tuning(E.EFIM_TUNE_DEVICE_PLAN, 1)
    kc_ref, vc_ref = kc.copy(), vc.copy()
    q_roped, _ = O.rope_append(b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new, b.k_new, b.v_new,
                               kc_ref, vc_ref, b.rope_base)
    U.assert_close(want, O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q_roped,
                                            kc_ref, vc_ref), "decode step")
    for i in range(4):
        assert np.array_equal(step(), want), "step %d differs" % i
    assert np.array_equal(U.host_bits(kcd), kc_ref) and np.array_equal(U.host_bits(vcd), vc_ref)


def test_a_work_list_too_large_for_the_copy(E):
    """More work items than a copy buffer holds: every launch reads the pinned slot."""
    n = 3000
    b = W.make_batch("c1", seed=320, lengths=(np.full(n, 5, dtype=np.int32), np.ones(n, dtype=np.int32)),
                     heads=(16, 16), head_dim=64)
    table = torch.from_numpy(b.block_table).cuda()
    items = E.efim_extend_plan_items(U.make_desc(E, b, table))
    assert len(items) * 48 > (2 << 20), "the case no longer exceeds the buffer"
    for seed in (1, 2, 3):
        U.sampled_check(E, b, heads_per_req=1, rows_per_head=1, seed=seed)


def test_knob_values(E):
    with pytest.raises(E.EfimError):
        E.efim_set_tuning(E.EFIM_TUNE_DEVICE_PLAN, 2)
    E.efim_set_tuning(E.EFIM_TUNE_DEVICE_PLAN, 1)
