"""TEST INFRASTRUCTURE ONLY -- never imported by the product path.

The serving hot path of the EFIM paper (Sec. 1, Sec. 3.1 step 4: cached prefix+suffix, new
``inc`` tokens) with the KV cache held in 8-bit floating point.  The paper serves unmodified
models on a stock engine (Sec. 4.2) and says nothing about the cache's number format; this
variant is the common engine option of storing K/V as OCP FP8 E4M3 codes with one scale per
tensor.  Everything that is not about the number format is delegated to ``efim_oracle``.

Readings (the paper is silent on all of them; each is listed in the design notes):
  * format: OCP 8-bit floating point E4M3 -- 1 sign, 4 exponent (bias 7), 3 mantissa bits, no
    infinities, S.1111.111 is NaN, largest finite value 448, subnormals m * 2^-9;
  * quantisation: code = nearest E4M3 value to x / scale, ties to the even code, magnitudes
    beyond 448 saturate to +-448; x is the bf16 value that the bf16 cache would hold (the key
    after its rotary embedding was rounded to bf16, the value as given);
  * the quotient x / scale is formed in IEEE binary32, correctly rounded: the interface gives the
    scales as binary32 numbers and x (a bf16 value) is one too, and engines that keep an FP8
    cache for the models the paper serves (Sec. 4) quantise in the activations' working
    precision, not in a wider one; the code is decided on that binary32 quotient;
  * attention uses the exact products code_value * scale in place of the bf16 cache values;
    queries stay bf16.

Parity: the decode table and the encoder are pinned in tests/test_fp8_pins.py against the
format's published special values, a brute-force nearest-value search, and torch's CPU cast
to float8_e4m3fn inside its non-overflowing range.
"""
from __future__ import annotations

import numpy as np

from oracle import efim_oracle as O

E4M3_MAX = 448.0


def e4m3_decode(codes):
    """Value (fp64) of E4M3 codes: (-1)^s * 2^(e-7) * (1 + m/8), or (-1)^s * 2^-6 * m/8 for e == 0."""
    codes = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    s = codes >> 7
    e = (codes >> 3) & 0xF
    m = codes & 0x7
    mag = np.where(e == 0, np.ldexp(m / 8.0, -6), np.ldexp(1.0 + m / 8.0, e - 7))
    mag = np.where((e == 15) & (m == 7), np.nan, mag)
    return np.where(s == 1, -mag, mag)


def e4m3_encode(x):
    """Nearest finite E4M3 code of each fp64 value: ties go to the even code, magnitudes of 448
    and above give +-448, NaN gives the NaN code 0x7F.  The sign bit of zero results is kept."""
    x = np.asarray(x, dtype=np.float64)
    grid = e4m3_decode(np.arange(127, dtype=np.uint8))  # the non-negative finite values, ascending
    mag = np.minimum(np.abs(np.where(np.isnan(x), 0.0, x)), E4M3_MAX)
    up = np.minimum(np.searchsorted(grid, mag, side="left"), 126)  # first code with value >= mag
    dn = np.maximum(up - 1, 0)
    d_up = grid[up] - mag
    d_dn = mag - grid[dn]
    pick_dn = (d_dn < d_up) | ((d_dn == d_up) & (dn % 2 == 0))
    code = np.where(pick_dn, dn, up).astype(np.uint8)
    code = code | (np.signbit(x).astype(np.uint8) << 7)
    return np.where(np.isnan(x), np.uint8(0x7F), code).astype(np.uint8)


def quantize_bf16(bits, scale):
    """E4M3 codes of bf16 values (bit patterns) for a per-tensor scale: the quotient is the
    binary32 division, the rounding to E4M3 is done on that quotient exactly."""
    x = O.bf16_to_f64(bits).astype(np.float32)
    with np.errstate(over="ignore"):
        quotient = x / np.float32(scale)
    return e4m3_encode(quotient.astype(np.float64))


def dequantize(codes, scale):
    """fp64 values code_value * scale (scale taken as the binary32 value the kernel receives)."""
    return e4m3_decode(codes) * float(np.float32(scale))


def rope_append_fp8(cached_len, new_len, block_table, page_size, q_new, k_new, v_new,
                    k_cache, v_cache, rope_base, k_scale, v_scale, interleaved=False):
    """As efim_oracle.rope_append, with ``k_cache`` / ``v_cache`` uint8[num_pages, Hkv, P, D]
    receiving the E4M3 codes of the rotated keys (after their rounding to bf16) and of the
    values.  Returns (q_roped bf16 bits, k codes [T, Hkv, D])."""
    head_dim = k_new.shape[-1]
    pos = O.new_token_positions(cached_len, new_len)
    cos, sin = O.rope_cos_sin(pos, head_dim, rope_base)
    k_roped = O.f64_to_bf16(O.rope_rotate(O.bf16_to_f64(k_new), cos, sin, interleaved))
    q_roped = None
    if q_new is not None:
        q_roped = O.f64_to_bf16(O.rope_rotate(O.bf16_to_f64(q_new), cos, sin, interleaved))
    k_codes = quantize_bf16(k_roped, k_scale)
    v_codes = quantize_bf16(v_new, v_scale)
    row = 0
    for r, (c, n) in enumerate(zip(cached_len, new_len)):
        for i in range(int(n)):
            p = int(c) + i
            page = int(block_table[r, p // page_size])
            k_cache[page, :, p % page_size, :] = k_codes[row]
            v_cache[page, :, p % page_size, :] = v_codes[row]
            row += 1
    return q_roped, k_codes


def rope_append_fp8_table(cached_len, new_len, block_table, page_size, q_new, k_new, v_new,
                          k_cache, v_cache, inv_freq, rotary_dim, k_scale, v_scale, interleaved=False):
    """rope_append_fp8 with a caller-given frequency table (rotary_dim/2 entries) and a rotation
    of the leading rotary_dim elements only, as efim_oracle.rope_append_table rotates."""
    pos = O.new_token_positions(cached_len, new_len)
    cos, sin = O.rope_cos_sin_table(pos, inv_freq)
    k_roped = O.f64_to_bf16(O.rope_rotate_leading(O.bf16_to_f64(k_new), cos, sin, rotary_dim, interleaved))
    q_roped = None
    if q_new is not None:
        q_roped = O.f64_to_bf16(O.rope_rotate_leading(O.bf16_to_f64(q_new), cos, sin, rotary_dim, interleaved))
    k_codes = quantize_bf16(k_roped, k_scale)
    v_codes = quantize_bf16(v_new, v_scale)
    row = 0
    for r, (c, n) in enumerate(zip(cached_len, new_len)):
        for i in range(int(n)):
            p = int(c) + i
            page = int(block_table[r, p // page_size])
            k_cache[page, :, p % page_size, :] = k_codes[row]
            v_cache[page, :, p % page_size, :] = v_codes[row]
            row += 1
    return q_roped, k_codes


def extend_attention_rows_fp8(r, q_head, cached_len, new_len, block_table, page_size, q_roped,
                              k_cache, v_cache, k_scale, v_scale, sm_scale=None, rows=None):
    """efim_oracle.extend_attention_rows over E4M3 caches (fp64 [len(rows), D])."""
    return O.extend_attention_rows(
        r, q_head, cached_len, new_len, block_table, page_size, q_roped, k_cache, v_cache, sm_scale, rows,
        k_values=lambda codes: dequantize(codes, k_scale), v_values=lambda codes: dequantize(codes, v_scale))


def extend_attention_fp8(cached_len, new_len, block_table, page_size, q_roped, k_cache, v_cache,
                         k_scale, v_scale, sm_scale=None):
    """Whole-batch extend attention over E4M3 caches, fp64 [T, Hq, D]."""
    total, num_q_heads, head_dim = q_roped.shape
    out = np.zeros((total, num_q_heads, head_dim), dtype=np.float64)
    start = 0
    for r in range(len(new_len)):
        n = int(new_len[r])
        if n == 0:
            continue
        for a in range(num_q_heads):
            out[start:start + n, a, :] = extend_attention_rows_fp8(
                r, a, cached_len, new_len, block_table, page_size, q_roped, k_cache, v_cache,
                k_scale, v_scale, sm_scale)
        start += n
    return out
