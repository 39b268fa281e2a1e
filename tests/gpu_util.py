"""Helpers for the GPU parity tests: move a synthetic batch to the device, call the
library through its C ABI binding, bring results back as numpy bit patterns."""
import numpy as np
import torch

from oracle import efim_oracle as O
from paper_2505_21889_amd import workloads as W

MAX_ABS_TOL = 1e-2     # tolerance on bf16-input / fp32-accumulate attention outputs
REL_L2_TOL = 5e-3


def dev_bits(x):
    """uint16 numpy -> int16 CUDA tensor with the same bits."""
    return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).cuda()


def host_bits(t):
    return t.cpu().numpy().view(np.uint16)


def make_desc(E, b, table_dev):
    return E.BatchDesc(b.cached_len, b.new_len, table_dev, b.num_q_heads, b.num_kv_heads,
                       b.head_dim, b.page_size, b.num_pages, b.max_pages_per_req)


def oracle_cache(b, fill=W.POISON_BITS):
    """Cache holding the history (positions 0..C-1) appended by the oracle; the rest poison."""
    kc = np.full(b.cache_shape(), fill, dtype=np.uint16)
    vc = np.full(b.cache_shape(), fill, dtype=np.uint16)
    if b.k_hist is not None and int(b.cached_len.sum()) > 0:
        O.rope_append(np.zeros_like(b.cached_len), b.cached_len, b.block_table, b.page_size, None,
                      b.k_hist, b.v_hist, kc, vc, b.rope_base)
    return kc, vc


def gpu_rope_append(E, b, kc, vc, interleaved=0, with_q=True):
    """Runs efim_rope_append on copies of the given caches; returns (q, k_cache, v_cache) bits."""
    table = torch.from_numpy(b.block_table).cuda()
    desc = make_desc(E, b, table)
    q = dev_bits(b.q_new) if with_q else None
    k_new, v_new = dev_bits(b.k_new), dev_bits(b.v_new)
    kcd, vcd = dev_bits(kc), dev_bits(vc)
    E.efim_rope_append(desc, q, k_new, v_new, kcd, vcd, b.rope_base, interleaved)
    torch.cuda.synchronize()
    return (host_bits(q) if with_q else None), host_bits(kcd), host_bits(vcd)


def gpu_extend_attention(E, b, q_roped, kc, vc, sm_scale=0.0, table=None):
    table_np = b.block_table if table is None else table
    table_dev = torch.from_numpy(np.ascontiguousarray(table_np)).cuda()
    desc = make_desc(E, b, table_dev)
    desc.c.max_pages_per_req = int(table_np.shape[1])
    q = dev_bits(q_roped)
    kcd, vcd = dev_bits(kc), dev_bits(vc)
    out = torch.full(q.shape, 0x7FC1, dtype=torch.int16, device="cuda")   # NaN pattern: unwritten rows show
    nbytes = E.efim_extend_workspace_bytes(desc)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
    E.efim_extend_attention(desc, q, kcd, vcd, out, sm_scale, ws, nbytes)
    torch.cuda.synchronize()
    return host_bits(out)


def errors(got_bits, ref):
    got = O.bf16_to_f64(got_bits)
    diff = got - ref
    max_abs = float(np.max(np.abs(diff))) if diff.size else 0.0
    denom = float(np.linalg.norm(ref.ravel()))
    rel_l2 = float(np.linalg.norm(diff.ravel())) / denom if denom > 0 else 0.0
    return max_abs, rel_l2


def elementwise_abs_bound(ref, value_scale=1.0):
    """Per-element absolute bound: 1e-2 for outputs of magnitude up to 2, and 1e-2 * |ref| / 2
    above.  An output element is a bf16 number: for 2 <= |o| < 4 its rounding alone is up to
    2^-7 = 7.8e-3, for 4 <= |o| < 8 up to 2^-6 = 1.56e-2, so a flat 1e-2 cannot hold there for
    any implementation; the bound grows with the element itself, never with other elements.
    value_scale: standard deviation of the value rows when it is above one.  The output is
    linear in V (out = sum_j p_j v_j), so are its rounding errors; the 1e-2 is stated for
    values of unit scale and is applied in units of that scale."""
    s = max(1.0, float(value_scale))
    return MAX_ABS_TOL * np.maximum(s, np.abs(ref) / 2.0)


def assert_close(got_bits, ref, what="", large_outputs=False, value_scale=1.0):
    """max abs <= 1e-2 and relative L2 <= 5e-3 over the whole tensor.  Tests whose inputs give
    outputs of magnitude above 2 (a sharpened softmax, rows with a handful of visible keys,
    values of more than unit scale) pass large_outputs: the absolute bound is then taken element
    by element (elementwise_abs_bound), which is the flat 1e-2 wherever |ref| <= 2 and the
    values have unit scale."""
    got = O.bf16_to_f64(got_bits)
    assert np.all(np.isfinite(got)), what + ": non-finite output"
    max_abs, rel_l2 = errors(got_bits, ref)
    if large_outputs:
        over = np.abs(got - ref) - elementwise_abs_bound(ref, value_scale)
        worst = float(over.max()) if over.size else -1.0
        assert worst <= 0.0, "%s: an element exceeds its bound by %.3e (max_abs %.3e)" % (what, worst, max_abs)
    else:
        assert max_abs <= MAX_ABS_TOL, "%s: max_abs %.3e rel_l2 %.3e" % (what, max_abs, rel_l2)
    assert rel_l2 <= REL_L2_TOL, "%s: max_abs %.3e rel_l2 %.3e" % (what, max_abs, rel_l2)
    return max_abs, rel_l2


def oracle_inputs(b):
    """Oracle-side inputs of the attention step: roped queries and the caches after the append."""
    kc, vc = oracle_cache(b)
    q_roped, _ = O.rope_append(b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new, b.k_new,
                               b.v_new, kc, vc, b.rope_base)
    return q_roped, kc, vc


def progress(msg):
    """A line on the real stdout (past pytest's capture) and in a log file (test_progress.log in
    the folder EFIM_PROGRESS_DIR names, else in the output folder of the test runs): the oracle
    needs minutes for the largest workloads and the run must be seen to be alive."""
    import os
    import sys
    import time
    folder = os.environ.get("EFIM_PROGRESS_DIR", "gpurun_out")
    line = "[%s] %s\n" % (time.strftime("%H:%M:%S"), msg)
    try:
        os.write(sys.__stdout__.fileno(), line.encode())
    except (OSError, ValueError, AttributeError):
        pass
    try:
        os.makedirs(folder, exist_ok=True)
        with open(os.path.join(folder, "test_progress.log"), "a") as fh:
            fh.write(line)
    except OSError:
        pass


def full_check(E, b, what, every_s=20.0):
    """Library output of the whole batch against the oracle on EVERY element: the oracle goes
    request by request and head by head (the same function extend_attention calls), so that
    progress can be reported in between.  Returns (max_abs, rel_l2) over the whole tensor."""
    import time
    q_roped, kc, vc = oracle_inputs(b)
    progress("%s: oracle inputs built, library call" % what)
    got_bits = gpu_extend_attention(E, b, q_roped, kc, vc)
    got = O.bf16_to_f64(got_bits)
    assert np.all(np.isfinite(got)), what + ": a row was left unwritten or is not finite"
    num = den = worst = 0.0
    start = 0
    last = time.time()
    for r in range(b.batch):
        n = int(b.new_len[r])
        for a in range(b.num_q_heads if n else 0):
            ref = O.extend_attention_rows(r, a, b.cached_len, b.new_len, b.block_table, b.page_size,
                                          q_roped, kc, vc)
            d = got[start:start + n, a, :] - ref
            worst = max(worst, float(np.abs(d).max()))
            num += float((d * d).sum())
            den += float((ref * ref).sum())
            if time.time() - last > every_s:
                last = time.time()
                progress("%s: request %d/%d head %d, max_abs so far %.3e" % (what, r, b.batch, a, worst))
        start += n
    rel = (num / den) ** 0.5 if den > 0 else 0.0
    progress("%s: all %d elements compared, max_abs %.3e rel_l2 %.3e" % (what, got.size, worst, rel))
    assert worst <= MAX_ABS_TOL and rel <= REL_L2_TOL, "%s: max_abs %.3e rel_l2 %.3e" % (what, worst, rel)
    return worst, rel


def sampled_check(E, b, heads_per_req, rows_per_head, seed):
    """Library output of the whole batch against oracle rows computed one by one: for every
    request a sample of (kv head, query head, row) triples, first, middle and last row always."""
    q_roped, kc, vc = oracle_inputs(b)
    got_bits = gpu_extend_attention(E, b, q_roped, kc, vc)
    got = O.bf16_to_f64(got_bits)
    assert np.all(np.isfinite(got)), "a row was left unwritten or is not finite"
    rng = np.random.default_rng(seed)
    g = b.num_q_heads // b.num_kv_heads
    num = den = 0.0
    worst = 0.0
    start = 0
    for r in range(b.batch):
        n = int(b.new_len[r])
        if n == 0:
            continue
        kv_heads = rng.choice(b.num_kv_heads, size=min(heads_per_req, b.num_kv_heads), replace=False)
        for h in kv_heads:
            a = int(h) * g + int(rng.integers(0, g))
            rows = {0, n - 1, n // 2} | set(int(x) for x in rng.integers(0, n, size=min(rows_per_head, n)))
            rows = sorted(rows)
            ref = O.extend_attention_rows(r, a, b.cached_len, b.new_len, b.block_table, b.page_size,
                                          q_roped, kc, vc, rows=rows)
            d = got[start + np.array(rows), a, :] - ref
            worst = max(worst, float(np.abs(d).max()))
            num += float((d * d).sum())
            den += float((ref * ref).sum())
        start += n
    rel = (num / den) ** 0.5
    assert worst <= MAX_ABS_TOL and rel <= REL_L2_TOL, "max_abs %.3e rel_l2 %.3e" % (worst, rel)
    return worst, rel
