"""Pins of the oracle's FP8 page functions (an extension beyond the paper; no GPU).

The format is OCP FP8 E4M3: 1 sign bit, 4 exponent bits of bias 7, 3 mantissa bits, no infinities, S.1111.111 is
NaN, largest finite magnitude 448.  Pinned by the format's landmark values, by round trips and ordering of all
codes, by hand-computed ties and saturation cases, by a library float8 conversion (torch's CPU float8_e4m3fn),
and -- for attention on FP8 pages -- by the already pinned 16-bit oracle run on a pool that holds the decoded
values.
"""
import math

import numpy as np
import torch

import oracle
import synthetic_inputs as si
from helpers import SENTINEL, bits_to_f32

NAN_CODE = 0x7F


def test_e4m3_landmarks():
    v = oracle.e4m3_value
    assert v(0x00) == 0.0 and v(0x80) == 0.0 and math.copysign(1.0, v(0x80)) == -1.0
    assert v(0x38) == 1.0 and v(0xB8) == -1.0
    assert v(0x3C) == 1.5 and v(0x40) == 2.0 and v(0x30) == 0.5
    assert v(0x01) == 2.0 ** -9 and v(0x07) == 7 * 2.0 ** -9      # subnormals: multiples of 2^-9
    assert v(0x08) == 2.0 ** -6                                    # smallest normal
    assert v(0x7E) == 448.0 and v(0xFE) == -448.0                  # largest finite
    assert v(0x78) == 256.0 and v(0x77) == 240.0
    assert math.isnan(v(0x7F)) and math.isnan(v(0xFF))


def test_codes_round_trip_and_are_ordered():
    vals = [oracle.e4m3_value(c) for c in range(0x7F)]
    assert all(b > a for a, b in zip(vals, vals[1:]))
    for c in range(0x7F):
        assert oracle.e4m3_code(vals[c]) == c
        assert oracle.e4m3_code(-vals[c]) == (c | 0x80)
    # every value is a multiple of 2^-9 with at most 4 significant bits
    for x in vals[1:]:
        m, _ = math.frexp(x)
        assert (m * 16) == int(m * 16)


def test_rounding_ties_and_saturation():
    code = oracle.e4m3_code
    assert code(1.0625) == 0x38          # halfway 1.0 (0x38) .. 1.125 (0x39): the even code
    assert code(1.1875) == 0x3A          # halfway 1.125 (0x39) .. 1.25 (0x3A)
    assert code(np.nextafter(np.float32(1.0625), np.float32(2))) == 0x39
    assert code(np.nextafter(np.float32(1.0625), np.float32(0))) == 0x38
    assert code(2.0 ** -10) == 0x00      # halfway 0 .. smallest subnormal
    assert code(3 * 2.0 ** -10) == 0x02  # halfway 0x01 .. 0x02
    assert code(np.nextafter(np.float32(2.0 ** -10), np.float32(1))) == 0x01
    assert code(15 * 2.0 ** -10) == 0x08  # halfway largest subnormal (0x07) .. smallest normal (0x08)
    assert code(431.9) == 0x7D and code(432.0) == 0x7E and code(447.9) == 0x7E
    for big in (448.0, 463.9, 464.0, 480.0, 1e9, float("inf")):
        assert code(big) == 0x7E and code(-big) == 0xFE
    assert code(float("nan")) & 0x7F == NAN_CODE
    assert code(-0.0) == 0x80


def _torch_codes(y):
    """Library conversion binary32 -> float8_e4m3fn (round to nearest even), as uint8; valid below 448."""
    return torch.from_numpy(np.ascontiguousarray(y, np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def test_codes_against_a_library_float8_conversion():
    rng = np.random.default_rng(5)
    mag = np.exp2(rng.uniform(-13.0, math.log2(447.0), 6000)).astype(np.float32)
    y = (mag * rng.choice([-1.0, 1.0], mag.shape)).astype(np.float32)
    # plus every midpoint between neighbouring codes, and its two binary32 neighbours
    vals = np.array([oracle.e4m3_value(c) for c in range(0x7F)], np.float64)
    mid = ((vals[:-1] + vals[1:]) / 2).astype(np.float32)
    y = np.concatenate([y, mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(1000))])
    want = _torch_codes(y)
    got = np.array([oracle.e4m3_code(t) for t in y], np.uint8)
    assert (got == want).all(), np.argwhere(got != want)[:5]


def _batch(seed=2):
    return si.make_batch("f8", L=[0, 37, 100, 16], n=[5, 1, 20, 1], Hq=8, Hkv=2, D=64, seed=seed, slack_pages=3)


def _fp8_pool(b, k_scale, v_scale, fill=NAN_CODE):
    pool = np.full(oracle.pool_elems(b.num_pages, b.Hkv, b.D, b.P), fill, dtype=np.uint8)
    for part in (b.cached_part(), b.new_part()):
        k, v, slots = part
        oracle.kv_append_fp8(k, v, pool, slots, b.Hkv, b.D, b.P, b.num_pages, k_scale, v_scale)
    return pool


def test_fp8_append_stores_the_library_codes_in_the_16_bit_layout():
    """Same element positions as the 16-bit append; each element is the library's code of x * (1 / scale)."""
    b = _batch()
    k_scale, v_scale = 0.0173, 0.0421   # not powers of two: the binary32 product rounds
    pool8 = _fp8_pool(b, k_scale, v_scale)
    # reference positions and source values through the (separately pinned) 16-bit append
    pool16 = np.full(pool8.size, SENTINEL, np.uint16)
    poolk = np.full(pool8.size, SENTINEL, np.uint16)
    for k, v, slots in (b.cached_part(), b.new_part()):
        oracle.kv_append(k, v, pool16, slots, b.Hkv, b.D, b.P, b.num_pages)
        oracle.kv_append(k, np.full_like(v, SENTINEL), poolk, slots, b.Hkv, b.D, b.P, b.num_pages)
    written = pool16 != SENTINEL
    assert ((pool8 != NAN_CODE) == written).all()       # N(0,1) values never encode to NaN
    is_k = written & (poolk != SENTINEL)                # the K elements among the written ones
    x = bits_to_f32(pool16)
    inv = np.where(is_k, np.float32(1.0) / np.float32(k_scale), np.float32(1.0) / np.float32(v_scale)).astype(np.float32)
    y = (x * inv).astype(np.float32)
    assert np.abs(y[written]).max() < 448.0
    assert (pool8[written] == _torch_codes(y[written])).all()


def test_fp8_append_saturates():
    b = si.make_batch("sat", L=[0], n=[4], Hq=2, Hkv=1, D=64, seed=1)
    k, v, slots = b.new_part()
    pool = np.full(oracle.pool_elems(b.num_pages, 1, 64, b.P), NAN_CODE, np.uint8)
    oracle.kv_append_fp8(k, v, pool, slots, 1, 64, b.P, b.num_pages, 2.0 ** -12, 1.0)   # K / scale up to ~2e4
    codes = pool[pool != NAN_CODE]
    assert ((codes & 0x7F) <= 0x7E).all() and ((codes & 0x7F) == 0x7E).sum() > 50


def test_fp8_attention_is_16_bit_attention_on_the_decoded_pool():
    """With power-of-two scales value(code) * scale is a bf16 number: the 16-bit oracle on that pool must agree."""
    b = _batch(3)
    k_scale, v_scale = 2.0 ** -5, 2.0 ** -4
    pool8 = _fp8_pool(b, k_scale, v_scale, fill=0)
    half = b.Hkv * b.P * b.D
    is_v = (np.arange(pool8.size) % (2 * half)) >= half            # layout sentence: K half then V half of a page
    table = np.array([oracle.e4m3_value(c) if (c & 0x7F) != NAN_CODE else 0.0 for c in range(256)], np.float64)
    dec = table[pool8] * np.where(is_v, v_scale, k_scale)
    pool16 = si.f32_to_bf16_bits(dec.astype(np.float32))
    assert (bits_to_f32(pool16).astype(np.float64) == dec).all()   # exact in bf16
    got = oracle.mixed_attention_fp8(b.q, pool8, k_scale, v_scale, b.page_tables, b.L, b.n, b.Hq, b.Hkv, b.D, b.P,
                                     b.num_pages, b.scale)
    ref = oracle.mixed_attention(b.q, pool16, b.page_tables, b.L, b.n, b.Hq, b.Hkv, b.D, b.P, b.num_pages, b.scale)
    assert np.abs(got - ref).max() < 1e-6
    # and the result is close to attention on the unquantised values (3 mantissa bits: a few percent)
    exact = oracle.mixed_attention(b.q, _pool16_exact(b), b.page_tables, b.L, b.n, b.Hq, b.Hkv, b.D, b.P, b.num_pages,
                                   b.scale)
    assert np.abs(got - exact).max() < 0.15 and np.abs(got - exact).mean() < 0.02


def _pool16_exact(b):
    pool = np.zeros(oracle.pool_elems(b.num_pages, b.Hkv, b.D, b.P), np.uint16)
    for k, v, slots in (b.cached_part(), b.new_part()):
        oracle.kv_append(k, v, pool, slots, b.Hkv, b.D, b.P, b.num_pages)
    return pool


def test_fp8_scales_act_as_score_scale_and_output_factor():
    """K = value * k_scale only rescales the scores, V = value * v_scale only rescales the output."""
    b = _batch(4)
    k_scale, v_scale = 0.0173, 0.0421
    pool8 = _fp8_pool(b, k_scale, v_scale)
    got = oracle.mixed_attention_fp8(b.q, pool8, k_scale, v_scale, b.page_tables, b.L, b.n, b.Hq, b.Hkv, b.D, b.P,
                                     b.num_pages, b.scale)
    unit = oracle.mixed_attention_fp8(b.q, pool8, 1.0, 1.0, b.page_tables, b.L, b.n, b.Hq, b.Hkv, b.D, b.P,
                                      b.num_pages, b.scale * k_scale)
    assert np.abs(got - unit * v_scale).max() < 1e-5 * np.abs(got).max() + 1e-7
    # never-written slots hold the NaN code and must not leak
    assert np.isfinite(got).all()


def test_fp8_land_is_one_append_per_layer():
    b = si.make_batch("land", L=[0], n=[40], Hq=4, Hkv=2, D=64, seed=9, slack_pages=2)
    layers = 3
    rng = np.random.default_rng(1)
    k = si.normal_bf16(rng, (layers, 40, 2, 64))
    v = si.normal_bf16(rng, (layers, 40, 2, 64))
    _, _, slots = b.new_part()
    per = oracle.pool_elems(b.num_pages, 2, 64, b.P)
    stride = per + 4096
    pools = np.full(stride * (layers - 1) + per, NAN_CODE, np.uint8)
    oracle.kv_land_fp8(k, v, pools, stride, layers, slots, 2, 64, b.P, b.num_pages, 0.03, 0.05)
    for l in range(layers):
        one = np.full(per, NAN_CODE, np.uint8)
        oracle.kv_append_fp8(k[l], v[l], one, slots, 2, 64, b.P, b.num_pages, 0.03, 0.05)
        assert (pools[l * stride:l * stride + per] == one).all()
    for l in range(layers - 1):
        assert (pools[l * stride + per:(l + 1) * stride] == NAN_CODE).all()   # the padding between pools
