"""Pins for the 8-bit-cache part of the CPU oracle.  Expected values come from the OCP FP8 (E4M3)
format definition, a brute-force nearest-value search written out here, torch's CPU cast to
float8_e4m3fn, hand-worked cases and reductions to the (separately pinned) bf16 oracle -- never
from the functions under test and never from the GPU path."""
import math

import numpy as np
import pytest
import torch

from oracle import efim_oracle as O
from oracle import fp8_oracle as F
from paper_2505_21889_amd import workloads as W


# -------------------------------------------------------------- decode ----

def test_e4m3_decode_published_special_values():
    want = {
        0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x0F: 1.875 * 2.0 ** -6,
        0x30: 0.5, 0x38: 1.0, 0x39: 1.125, 0x3C: 1.5, 0x40: 2.0, 0x77: 240.0, 0x78: 256.0,
        0x7E: 448.0, 0xB8: -1.0, 0xFE: -448.0, 0x81: -(2.0 ** -9),
    }
    got = F.e4m3_decode(np.array(list(want), dtype=np.uint8))
    assert got.tolist() == list(want.values())
    z = F.e4m3_decode(np.array([0x80], dtype=np.uint8))[0]
    assert z == 0.0 and math.copysign(1.0, z) == -1.0
    assert np.isnan(F.e4m3_decode(np.array([0x7F, 0xFF], dtype=np.uint8))).all()


def test_e4m3_decode_matches_torch_on_every_code():
    codes = np.arange(256, dtype=np.uint8)
    want = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = F.e4m3_decode(codes)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok]) and np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))


def test_e4m3_values_are_strictly_increasing_with_the_code():
    v = F.e4m3_decode(np.arange(127, dtype=np.uint8))
    assert np.all(np.diff(v) > 0)
    # neighbouring values differ by one unit of the last of 3 mantissa bits of the lower one
    e = np.maximum(np.arange(126) >> 3, 1)
    assert np.array_equal(np.diff(v), np.ldexp(1.0, e - 7 - 3))


# -------------------------------------------------------------- encode ----

def test_e4m3_encode_inverts_decode_on_every_finite_code():
    codes = np.array([c for c in range(256) if c & 0x7F != 0x7F], dtype=np.uint8)
    assert np.array_equal(F.e4m3_encode(F.e4m3_decode(codes)), codes)


def _nearest_code_brute_force(x, table):
    """Pure-Python search over the finite non-negative values: nearest, even code on a tie."""
    a = min(abs(x), 448.0)
    best = 0
    for c in range(1, 127):
        d, db = abs(table[c] - a), abs(table[best] - a)
        if d < db or (d == db and c % 2 == 0):
            best = c
    return best | (0x80 if math.copysign(1.0, x) < 0 else 0)


def test_e4m3_encode_is_the_nearest_value_brute_force():
    # table typed from the definition, independent of the decoder under test
    table = [(m / 8.0) * 2.0 ** -6 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7)
             for e in range(16) for m in range(8)][:127]
    rng = np.random.default_rng(11)
    x = np.concatenate([
        rng.standard_normal(3000) * 2.0,
        rng.standard_normal(1500) * 200.0,           # reaches the saturating range
        rng.standard_normal(1500) * 2.0 ** -7,       # subnormal range
        np.array([0.0, -0.0, 448.0, -448.0, 463.9, 464.0, 480.0, 2.0 ** -10, -(2.0 ** -10), 3 * 2.0 ** -10]),
    ])
    mids = [(table[c] + table[c + 1]) / 2 for c in range(126)]
    x = np.concatenate([x, np.array(mids), -np.array(mids),
                        np.nextafter(np.array(mids), 0.0), np.nextafter(np.array(mids), 1e9)])
    want = np.array([_nearest_code_brute_force(float(v), table) for v in x], dtype=np.uint8)
    assert np.array_equal(F.e4m3_encode(x), want)


def test_e4m3_encode_ties_go_to_the_even_code():
    # 1.0625 lies between 1.0 (0x38) and 1.125 (0x39); 1.1875 between 0x39 and 1.25 (0x3A);
    # 2^-10 between 0 and the smallest subnormal 2^-9 (0x01); 3 * 2^-10 between 0x01 and 0x02;
    # 7.5 * 2^-9 between the largest subnormal (0x07) and the smallest normal 2^-6 (0x08)
    x = np.array([1.0625, 1.1875, 2.0 ** -10, 3 * 2.0 ** -10, -1.0625, 7.5 * 2.0 ** -9])
    assert F.e4m3_encode(x).tolist() == [0x38, 0x3A, 0x00, 0x02, 0xB8, 0x08]


def test_e4m3_encode_saturates_and_keeps_nan():
    x = np.array([448.0, 449.0, 464.0, 465.0, 1e9, np.inf, -1e9, -np.inf, np.nan])
    assert F.e4m3_encode(x).tolist() == [0x7E, 0x7E, 0x7E, 0x7E, 0x7E, 0x7E, 0xFE, 0xFE, 0x7F]


def test_e4m3_encode_matches_torch_cast_where_torch_does_not_overflow():
    rng = np.random.default_rng(12)
    x = np.concatenate([
        rng.standard_normal(200000).astype(np.float32) * np.float32(3.0),
        rng.standard_normal(100000).astype(np.float32) * np.float32(2.0 ** -6),
        rng.uniform(-464, 464, 100000).astype(np.float32),
    ])
    x = x[np.abs(x) <= 464.0]          # torch turns larger magnitudes into NaN instead of saturating
    want = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(F.e4m3_encode(x.astype(np.float64)), want)


def test_quantize_divides_in_binary32():
    # x = 2^-7 (bf16 0x3C00), scale = 0x1.af286cp-8: the exact quotient is 1.18749999115...,
    # nearer to 1.125 (0x39); its binary32 rounding is exactly 1.1875, a tie that goes to the
    # even code 0x3A.  x = 0x3C01, scale = 0x1.e5a5a4p-8: exact quotient 1.06250005498... would
    # go up to 0x39; the binary32 quotient is the tie 1.0625, which goes to the even code 0x38.
    s1 = float.fromhex("0x1.af286cp-8")
    s2 = float.fromhex("0x1.e5a5a4p-8")
    assert 2.0 ** -7 / s1 < 1.1875 and float(np.float32(2.0 ** -7) / np.float32(s1)) == 1.1875
    assert F.quantize_bf16(np.array([0x3C00], dtype=np.uint16), s1).tolist() == [0x3A]
    assert F.quantize_bf16(np.array([0x3C01], dtype=np.uint16), s2).tolist() == [0x38]
    # plain cases: scale 1 keeps the value, scale 0.5 doubles it, beyond the range saturates
    bits = np.array([0x3F80, 0xBFC0, 0x43E0, 0x4400, 0x0000, 0x8000], dtype=np.uint16)  # 1, -1.5, 448, 512, 0, -0
    assert F.quantize_bf16(bits, 1.0).tolist() == [0x38, 0xBC, 0x7E, 0x7E, 0x00, 0x80]
    assert F.quantize_bf16(bits, 0.5).tolist() == [0x40, 0xC4, 0x7E, 0x7E, 0x00, 0x80]


def test_dequantize_is_code_value_times_scale():
    codes = np.array([0x38, 0xBC, 0x7E, 0x01], dtype=np.uint8)
    assert F.dequantize(codes, 0.25).tolist() == [0.25, -0.375, 112.0, 2.0 ** -11]


# ------------------------------------------------- append and attention ----

def _small_batch(seed=3):
    return W.make_batch("c1", seed=seed, lengths=(np.array([37, 0, 16], dtype=np.int32), np.array([5, 9, 1], dtype=np.int32)),
                        heads=(4, 2), head_dim=64)


def test_rope_append_fp8_writes_the_codes_of_the_bf16_cache_and_nothing_else():
    b = _small_batch()
    kc16 = np.zeros(b.cache_shape(), dtype=np.uint16)
    vc16 = np.zeros(b.cache_shape(), dtype=np.uint16)
    q16, _ = O.rope_append(b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new.copy(), b.k_new, b.v_new,
                           kc16, vc16, b.rope_base)
    kc8 = np.full(b.cache_shape(), 0x55, dtype=np.uint8)
    vc8 = np.full(b.cache_shape(), 0x55, dtype=np.uint8)
    q8, k_codes = F.rope_append_fp8(b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new.copy(), b.k_new, b.v_new,
                                    kc8, vc8, b.rope_base, 0.5, 0.25)
    assert np.array_equal(q8, q16)
    written = np.zeros(b.cache_shape()[:1] + b.cache_shape()[2:3], dtype=bool)  # [page, slot]
    for r in range(b.batch):
        for p in range(int(b.cached_len[r]), int(b.cached_len[r] + b.new_len[r])):
            written[b.block_table[r, p // b.page_size], p % b.page_size] = True
    w = np.broadcast_to(written[:, None, :, None], kc8.shape)
    assert np.all(kc8[~w] == 0x55) and np.all(vc8[~w] == 0x55)
    # every written entry is within half a code step of value / scale (or saturated)
    for cache8, cache16, scale in ((kc8, kc16, 0.5), (vc8, vc16, 0.25)):
        x = O.bf16_to_f64(cache16[w]) / scale
        got = F.e4m3_decode(cache8[w])
        step = np.ldexp(1.0, np.maximum(np.floor(np.log2(np.maximum(np.abs(got), 2.0 ** -6))), -6).astype(int) - 3)
        assert np.all(np.abs(got - np.clip(x, -448, 448)) <= step / 2 + 1e-12)
    assert k_codes.shape == b.k_new.shape


def test_rope_append_fp8_table_reduces_to_the_plain_call_and_to_the_bf16_table_call():
    b = _small_batch()
    d = b.head_dim
    # the plain table over the whole head: byte for byte the plain 8-bit append
    kc_a = np.full(b.cache_shape(), 0x55, dtype=np.uint8)
    vc_a = kc_a.copy()
    kc_b, vc_b = kc_a.copy(), vc_a.copy()
    q_a, _ = F.rope_append_fp8(b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new.copy(), b.k_new,
                               b.v_new, kc_a, vc_a, b.rope_base, 0.5, 0.25)
    q_b, _ = F.rope_append_fp8_table(b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new.copy(), b.k_new,
                                     b.v_new, kc_b, vc_b, O.rope_inv_freq(d, b.rope_base), d, 0.5, 0.25)
    assert np.array_equal(q_a, q_b) and np.array_equal(kc_a, kc_b) and np.array_equal(vc_a, vc_b)
    # a partial rotation with another table: the codes of what the bf16 table call stores
    rotary_dim = d // 2
    table = O.scaled_inv_freq(rotary_dim, 5.0e5, 8.0, 1.0, 4.0, 8192)
    kc16 = np.zeros(b.cache_shape(), dtype=np.uint16)
    vc16 = np.zeros(b.cache_shape(), dtype=np.uint16)
    q16, k16 = O.rope_append_table(b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new.copy(), b.k_new,
                                   b.v_new, kc16, vc16, table, rotary_dim, True)
    kc8 = np.zeros(b.cache_shape(), dtype=np.uint8)
    vc8 = np.zeros(b.cache_shape(), dtype=np.uint8)
    q8, k_codes = F.rope_append_fp8_table(b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new.copy(),
                                          b.k_new, b.v_new, kc8, vc8, table, rotary_dim, 0.5, 0.25, True)
    assert np.array_equal(q8, q16)
    assert np.array_equal(k_codes, F.quantize_bf16(k16, 0.5))
    assert np.array_equal(k_codes[..., rotary_dim:], F.quantize_bf16(b.k_new[..., rotary_dim:], 0.5)), \
        "features past rotary_dim are stored unrotated"
    assert not np.array_equal(k_codes[..., :rotary_dim], F.quantize_bf16(b.k_new[..., :rotary_dim], 0.5))
    written = kc16 != 0
    assert np.array_equal(kc8[written], F.quantize_bf16(kc16[written], 0.5))


def test_fp8_attention_equals_bf16_attention_when_the_codes_are_bf16_values():
    # E4M3 values times a power-of-two scale are bf16 numbers: the 8-bit cache and a bf16 cache
    # holding the same numbers must give the same attention output.
    b = _small_batch(seed=4)
    rng = np.random.default_rng(5)
    shape = b.cache_shape()
    kc8 = rng.integers(0, 256, shape, dtype=np.uint8)
    vc8 = rng.integers(0, 256, shape, dtype=np.uint8)
    kc8[(kc8 & 0x7F) == 0x7F] = 0x38
    vc8[(vc8 & 0x7F) == 0x7F] = 0x38
    kc8 = (kc8 & 0xBF).astype(np.uint8)   # clear the top exponent bit: keep the scores moderate
    k_scale, v_scale = 0.25, 2.0
    kc16 = O.f64_to_bf16(F.e4m3_decode(kc8) * k_scale)
    vc16 = O.f64_to_bf16(F.e4m3_decode(vc8) * v_scale)
    assert np.array_equal(O.bf16_to_f64(kc16), F.e4m3_decode(kc8) * k_scale)
    q = b.q_new
    want = O.extend_attention(b.cached_len, b.new_len, b.block_table, b.page_size, q, kc16, vc16)
    got = F.extend_attention_fp8(b.cached_len, b.new_len, b.block_table, b.page_size, q, kc8, vc8, k_scale, v_scale)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)


def test_fp8_attention_scales_act_as_they_should():
    b = _small_batch(seed=6)
    rng = np.random.default_rng(7)
    shape = b.cache_shape()
    kc8 = (rng.integers(0, 256, shape, dtype=np.uint8) & 0xB7).astype(np.uint8)
    vc8 = (rng.integers(0, 256, shape, dtype=np.uint8) & 0xB7).astype(np.uint8)
    args = (b.cached_len, b.new_len, b.block_table, b.page_size, b.q_new, kc8, vc8)
    base = F.extend_attention_fp8(*args, 0.5, 0.5, sm_scale=0.125)
    # the value scale multiplies the output; the key scale acts like the softmax scale
    assert np.allclose(F.extend_attention_fp8(*args, 0.5, 1.5, sm_scale=0.125), 3.0 * base, rtol=1e-12, atol=1e-14)
    assert np.allclose(F.extend_attention_fp8(*args, 1.0, 0.5, sm_scale=0.0625), base, rtol=1e-12, atol=1e-14)
    # a single visible key returns its value row exactly
    one = W.make_batch("c1", seed=8, lengths=(np.array([0], dtype=np.int32), np.array([1], dtype=np.int32)),
                       heads=(2, 1), head_dim=64)
    kc = np.zeros(one.cache_shape(), dtype=np.uint8)
    vc = np.zeros(one.cache_shape(), dtype=np.uint8)
    page = one.block_table[0, 0]
    vc[page, 0, 0, :] = np.arange(64, dtype=np.uint8) + 0x20
    out = F.extend_attention_fp8(one.cached_len, one.new_len, one.block_table, one.page_size, one.q_new, kc, vc, 1.0, 0.75)
    assert np.array_equal(out[0, 0], F.e4m3_decode(vc[page, 0, 0, :]) * 0.75)
