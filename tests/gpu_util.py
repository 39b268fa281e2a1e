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


def assert_close(got_bits, ref, what="", scale_abs_with_output=False):
    """max abs <= 1e-2 and relative L2 <= 5e-3.  The absolute bound is stated for outputs of
    order one (N(0,1) values averaged by a softmax at the default scale).  A test that sharpens
    the softmax on purpose gets outputs of magnitude up to ~4, whose bf16 rounding alone is up
    to 2^-7 = 7.8e-3; such a test sets scale_abs_with_output and the bound scales with max|ref|."""
    assert np.all(np.isfinite(O.bf16_to_f64(got_bits))), what + ": non-finite output"
    max_abs, rel_l2 = errors(got_bits, ref)
    abs_tol = MAX_ABS_TOL * (max(1.0, float(np.abs(ref).max())) if scale_abs_with_output else 1.0)
    assert max_abs <= abs_tol and rel_l2 <= REL_L2_TOL, "%s: max_abs %.3e rel_l2 %.3e" % (what, max_abs, rel_l2)
    return max_abs, rel_l2
