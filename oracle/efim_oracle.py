"""Plain fp64 CPU definition of what the EFIM serving hot path computes.

TEST INFRASTRUCTURE ONLY -- slow, untiled, unfused, written to be checked
against the paper by eye.  It shares no code with the HIP library and must
never be imported by the product package.

What is modelled (EFIM paper, Sec. 1 and Sec. 3.1 step 4): the prompt is
reordered to ``<P>prefix<S>suffix<M>inc``; the keys/values of everything in
front of ``inc`` are already in the serving engine's KV cache (cross-request
reuse needs an identical token prefix, Sec. 1), so a request consists of
``C`` cached tokens and ``N`` new tokens (``inc``, or the whole prompt when
nothing is cached -- the "Baseline" scheme of Sec. 4.2).  The paper changes
nothing in the model (Sec. 3, "no architectural changes"), so each layer
performs ordinary causal softmax attention with rotary position embedding;
the cache is the paged one of the engine the paper serves with (Sec. 4.2,
"Environment").  The functions below are those textbook definitions written
out with the cache addressed through a block table.

The paper gives no equations for this path; the readings taken where it is
silent are listed next to each function.

Parity status: every function here is pinned by tests that do not call it to
produce their expected values (closed forms, brute force in pure Python,
torch's fp64 scaled_dot_product_attention, torch's bf16 cast, invariants).
The absolute values of the attention output on the benchmark workloads are
printed nowhere in the paper: for those, "parity unpinned" by the paper; they
are pinned only through the properties above.

Conventions
-----------
* bf16 tensors travel as ``numpy.uint16`` bit patterns.
* ``cached_len[r] = C_r``, ``new_len[r] = N_r``, ``L_r = C_r + N_r``.
* New-token tensors are ragged and packed: rows of request ``r`` start at
  ``sum(new_len[:r])``; shapes ``[T, H, D]``.
* Caches: ``k_cache``/``v_cache`` are ``uint16[num_pages, Hkv, P, D]``;
  logical position ``p`` of request ``r`` lives in page
  ``block_table[r, p // P]`` at slot ``p % P``.
"""
from __future__ import annotations

import numpy as np

# --------------------------------------------------------------------------
# bf16 <-> fp64
# --------------------------------------------------------------------------


def bf16_to_f64(bits):
    """Value of bf16 bit patterns: a bf16 is the upper half of an IEEE binary32."""
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f64_to_bf16(x):
    """Round fp64 to the nearest bf16 (ties to even), return the bit patterns.

    bf16 carries 8 significant bits, so in the binade [2^(e-1), 2^e) its values
    are spaced 2^(e-8) apart; below the smallest normal 2^-126 the spacing stays
    2^-133.  Dividing by the spacing is exact (power of two), ``rint`` rounds
    half to even, and the product is exactly a binary32 value.
    Reading: the paper does not state a rounding mode; round-to-nearest-even is
    what bf16 hardware conversion and the common tensor libraries use.
    """
    x = np.asarray(x, dtype=np.float64)
    with np.errstate(over="ignore", invalid="ignore"):
        _, e = np.frexp(x)
        e = np.maximum(e, -125)
        spacing = np.ldexp(1.0, e - 8)
        y = np.rint(x / spacing) * spacing
        f = y.astype(np.float32)
    return (f.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


# --------------------------------------------------------------------------
# Rotary position embedding at offset positions
# --------------------------------------------------------------------------


def rope_inv_freq(head_dim, base):
    """inv_freq[j] = base^(-2j/D), j < D/2, each an fp64 ``pow`` of the C library.

    Reading: no frequency scaling and the whole head is rotated.
    """
    half = head_dim // 2
    return np.array([float(base) ** (-2.0 * j / head_dim) for j in range(half)], dtype=np.float64)


def rope_cos_sin(positions, head_dim, base):
    """cos/sin of theta[p, j] = p * inv_freq[j].

    theta is the fp64 product; cos and sin are evaluated in extended precision
    and rounded to fp64 so that the table does not depend on which vector math
    routine numpy was built with.
    """
    positions = np.asarray(positions, dtype=np.int64)
    theta = positions[:, None].astype(np.float64) * rope_inv_freq(head_dim, base)[None, :]
    wide = theta.astype(np.longdouble)
    return np.cos(wide).astype(np.float64), np.sin(wide).astype(np.float64)


def rope_rotate(x, cos, sin, interleaved=False):
    """Rotate rows ``x[n, H, D]`` (fp64) by the per-row angle tables ``[n, D/2]``.

    rotate-half pairing (default): pair j is (x[j], x[j + D/2]);
    interleaved pairing: pair j is (x[2j], x[2j + 1]).
    Reading: the paper's two models (Sec. 4) are rotary models; rotate-half is
    the pairing their public checkpoints are served with.
    """
    x = np.asarray(x, dtype=np.float64)
    half = x.shape[-1] // 2
    c = cos[:, None, :]
    s = sin[:, None, :]
    y = np.empty_like(x)
    if interleaved:
        a, b = x[..., 0::2], x[..., 1::2]
        y[..., 0::2] = a * c - b * s
        y[..., 1::2] = b * c + a * s
    else:
        a, b = x[..., :half], x[..., half:]
        y[..., :half] = a * c - b * s
        y[..., half:] = b * c + a * s
    return y


def new_token_positions(cached_len, new_len):
    """Position of the i-th new token of request r is C_r + i: its index in the
    reordered prompt (Sec. 1: ``inc`` comes after ``<P>prefix<S>suffix<M>``), which is
    what keeps the cached keys valid."""
    out = []
    for c, n in zip(cached_len, new_len):
        out.append(np.arange(int(c), int(c) + int(n), dtype=np.int64))
    return np.concatenate(out) if out else np.zeros(0, dtype=np.int64)


def rope_append(cached_len, new_len, block_table, page_size, q_new, k_new, v_new,
                k_cache, v_cache, rope_base, interleaved=False):
    """RoPE the new tokens at their offset positions and append K/V to the paged cache.

    q_new  uint16[T, Hq, D]  raw queries     -> returns roped queries (bf16 bits)
    k_new  uint16[T, Hkv, D] raw keys        -> roped, written into k_cache
    v_new  uint16[T, Hkv, D] values          -> copied unchanged into v_cache
    The caches are modified in place; only slots [C_r, C_r + N_r) are written.
    Returns (q_roped, k_roped) as bf16 bit patterns.
    """
    head_dim = k_new.shape[-1]
    pos = new_token_positions(cached_len, new_len)
    cos, sin = rope_cos_sin(pos, head_dim, rope_base)
    k_roped = f64_to_bf16(rope_rotate(bf16_to_f64(k_new), cos, sin, interleaved))
    q_roped = None
    if q_new is not None:
        q_roped = f64_to_bf16(rope_rotate(bf16_to_f64(q_new), cos, sin, interleaved))
    row = 0
    for r, (c, n) in enumerate(zip(cached_len, new_len)):
        for i in range(int(n)):
            p = int(c) + i
            page = int(block_table[r, p // page_size])
            slot = p % page_size
            k_cache[page, :, slot, :] = k_roped[row]
            v_cache[page, :, slot, :] = v_new[row]
            row += 1
    return q_roped, k_roped


# --------------------------------------------------------------------------
# Rotary variants: caller-given frequency table, rotation of the leading part only
# --------------------------------------------------------------------------


def scaled_inv_freq(head_dim, base, factor, low_freq_factor, high_freq_factor, original_context):
    """Frequency table with the long-context scaling published with the Llama 3.1 models
    (one of the paper's two models, Sec. 4): with wavelength w_j = 2*pi / f_j of the plain
    table f_j = base^(-2j/D),
        w_j < original_context / high_freq_factor   ->  f_j unchanged,
        w_j > original_context / low_freq_factor    ->  f_j / factor,
        in between: blend (1 - t) * f_j / factor + t * f_j with
                    t = (original_context / w_j - low_freq_factor) / (high_freq_factor - low_freq_factor).
    """
    plain = rope_inv_freq(head_dim, base)
    out = np.empty_like(plain)
    for j, f in enumerate(plain):
        wavelen = 2.0 * np.pi / f
        if wavelen < original_context / high_freq_factor:
            out[j] = f
        elif wavelen > original_context / low_freq_factor:
            out[j] = f / factor
        else:
            t = (original_context / wavelen - low_freq_factor) / (high_freq_factor - low_freq_factor)
            out[j] = (1.0 - t) * f / factor + t * f
    return out


def rope_cos_sin_table(positions, inv_freq):
    """cos/sin of theta[p, j] = p * inv_freq[j] for a given table (same evaluation as rope_cos_sin)."""
    positions = np.asarray(positions, dtype=np.int64)
    theta = positions[:, None].astype(np.float64) * np.asarray(inv_freq, dtype=np.float64)[None, :]
    wide = theta.astype(np.longdouble)
    return np.cos(wide).astype(np.float64), np.sin(wide).astype(np.float64)


def rope_rotate_leading(x, cos, sin, rotary_dim, interleaved=False):
    """Rotate the first ``rotary_dim`` elements of every head row of ``x[n, H, D]`` (pairs taken
    inside that part: (j, j + rotary_dim/2), or (2j, 2j+1) when interleaved; tables
    ``[n, rotary_dim/2]``); the remaining D - rotary_dim elements pass through."""
    x = np.asarray(x, dtype=np.float64)
    y = x.copy()
    y[..., :rotary_dim] = rope_rotate(x[..., :rotary_dim], cos, sin, interleaved)
    return y


def rope_append_table(cached_len, new_len, block_table, page_size, q_new, k_new, v_new,
                      k_cache, v_cache, inv_freq, rotary_dim, interleaved=False):
    """rope_append with a caller-given frequency table (rotary_dim/2 entries) and a rotation of
    the leading rotary_dim elements only; everything else as rope_append."""
    pos = new_token_positions(cached_len, new_len)
    cos, sin = rope_cos_sin_table(pos, inv_freq)
    k_roped = f64_to_bf16(rope_rotate_leading(bf16_to_f64(k_new), cos, sin, rotary_dim, interleaved))
    q_roped = None
    if q_new is not None:
        q_roped = f64_to_bf16(rope_rotate_leading(bf16_to_f64(q_new), cos, sin, rotary_dim, interleaved))
    row = 0
    for r, (c, n) in enumerate(zip(cached_len, new_len)):
        for i in range(int(n)):
            p = int(c) + i
            page = int(block_table[r, p // page_size])
            k_cache[page, :, p % page_size, :] = k_roped[row]
            v_cache[page, :, p % page_size, :] = v_new[row]
            row += 1
    return q_roped, k_roped


# --------------------------------------------------------------------------
# Paged gather and extend attention
# --------------------------------------------------------------------------


def gather_kv(cache, block_table_row, length, page_size, kv_head):
    """Logical rows 0..length-1 of one request and kv head, as stored (bf16 bits) [length, D]."""
    pos = np.arange(length)
    pages = np.asarray(block_table_row)[pos // page_size]
    return cache[pages, kv_head, pos % page_size]


def extend_attention_rows(r, q_head, cached_len, new_len, block_table, page_size,
                          q_roped, k_cache, v_cache, sm_scale=None, rows=None,
                          k_values=bf16_to_f64, v_values=bf16_to_f64):
    """Attention output (fp64, [len(rows), D]) of request r, query head q_head.

    New row i sees keys 0 .. C_r + i (causal, itself included):
        s_j = sm_scale * <q_i, k_j>,  p = softmax(s),  o = sum_j p_j v_j.
    Query head a reads kv head a // (Hq / Hkv).
    Readings: scale 1/sqrt(D) unless given; no soft-cap, window or bias.
    k_values / v_values turn stored cache entries into their fp64 values (bf16 bit patterns
    unless the cache holds another number format).
    """
    c, n = int(cached_len[r]), int(new_len[r])
    num_q_heads, head_dim = q_roped.shape[1], q_roped.shape[2]
    num_kv_heads = k_cache.shape[1]
    kv_head = q_head // (num_q_heads // num_kv_heads)
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(head_dim)
    if rows is None:
        rows = range(n)
    rows = np.asarray(list(rows), dtype=np.int64)
    start = int(np.sum(np.asarray(new_len[:r], dtype=np.int64)))
    length = c + n
    k = k_values(gather_kv(k_cache, block_table[r], length, page_size, kv_head))
    v = v_values(gather_kv(v_cache, block_table[r], length, page_size, kv_head))
    q = bf16_to_f64(q_roped[start + rows, q_head, :])
    s = sm_scale * (q @ k.T)
    visible = np.arange(length)[None, :] <= (c + rows)[:, None]
    s = np.where(visible, s, -np.inf)
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=1, keepdims=True)
    return p @ v


def extend_attention(cached_len, new_len, block_table, page_size, q_roped,
                     k_cache, v_cache, sm_scale=None):
    """Whole-batch extend attention, fp64 [T, Hq, D]."""
    total, num_q_heads, head_dim = q_roped.shape
    out = np.zeros((total, num_q_heads, head_dim), dtype=np.float64)
    start = 0
    for r in range(len(new_len)):
        n = int(new_len[r])
        if n == 0:
            continue
        for a in range(num_q_heads):
            out[start:start + n, a, :] = extend_attention_rows(
                r, a, cached_len, new_len, block_table, page_size,
                q_roped, k_cache, v_cache, sm_scale)
        start += n
    return out


# --------------------------------------------------------------------------
# The equivalence the paper rests on: reuse == recomputation
# --------------------------------------------------------------------------


def full_recompute(q_raw, k_raw, v_raw, rope_base, sm_scale=None, interleaved=False):
    """Attention of one whole reordered prompt with no cache and no paging.

    q_raw uint16[L, Hq, D], k_raw/v_raw uint16[L, Hkv, D]: raw rows of every
    position 0..L-1.  RoPE at positions 0..L-1, round to bf16, plain causal
    softmax attention on all L rows.  Returns fp64 [L, Hq, D].
    Reusing the cache of the first C positions must give the last L - C rows of
    this (Sec. 1: the reused part is exactly what is not recomputed).
    """
    length, num_q_heads, head_dim = q_raw.shape
    num_kv_heads = k_raw.shape[1]
    group = num_q_heads // num_kv_heads
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(head_dim)
    cos, sin = rope_cos_sin(np.arange(length), head_dim, rope_base)
    q = bf16_to_f64(f64_to_bf16(rope_rotate(bf16_to_f64(q_raw), cos, sin, interleaved)))
    k = bf16_to_f64(f64_to_bf16(rope_rotate(bf16_to_f64(k_raw), cos, sin, interleaved)))
    v = bf16_to_f64(v_raw)
    out = np.zeros((length, num_q_heads, head_dim), dtype=np.float64)
    causal = np.tril(np.ones((length, length), dtype=bool))
    for a in range(num_q_heads):
        h = a // group
        s = sm_scale * (q[:, a, :] @ k[:, h, :].T)
        s = np.where(causal, s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=1, keepdims=True)
        out[:, a, :] = p @ v[:, h, :]
    return out
