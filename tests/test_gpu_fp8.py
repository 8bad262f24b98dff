"""FP8 E4M3 KV pages (an extension beyond the paper's 16-bit KV) on the GPU against the oracle, through the C ABI.

Bar: the appended codes bit for bit (the quantisation is an integer decision, taken in binary32 on both sides);
attention within max-abs 2e-2 / relative-L2 1e-2 of the double-precision oracle reading the SAME codes.
"""
import numpy as np
import pytest

import oracle
import synthetic_inputs as si
from helpers import bits_to_f32, check_close, random_mixed_batch

pytestmark = pytest.mark.gpu

NAN_CODE = 0x7F


def _oracle_fp8(b, k_scale, v_scale):
    pool = np.full(oracle.pool_elems(b.num_pages, b.Hkv, b.D, b.P), NAN_CODE, dtype=np.uint8)
    for k, v, slots in (b.cached_part(), b.new_part()):
        oracle.kv_append_fp8(k, v, pool, slots, b.Hkv, b.D, b.P, b.num_pages, k_scale, v_scale)
    return pool


def _compare(b, k_scale=0.0173, v_scale=0.0421, row_mask=None, **kw):
    from gpu_helpers import gpu_step_fp8
    print("fp8 case", b.name, "L", b.L.tolist()[:8], "n", b.n.tolist()[:8], k_scale, v_scale, kw, flush=True)
    ref_pool = _oracle_fp8(b, k_scale, v_scale)
    pool, out, stats = gpu_step_fp8(b, k_scale, v_scale, **kw)
    assert np.array_equal(pool, ref_pool), "FP8 codes differ at %s" % np.argwhere(pool != ref_pool)[:4].tolist()
    ref = oracle.mixed_attention_fp8(b.q, ref_pool, k_scale, v_scale, b.page_tables, b.L, b.n, b.Hq, b.Hkv, b.D, b.P,
                                     b.num_pages, b.scale, row_mask=row_mask)
    got = bits_to_f32(out)
    if row_mask is not None:
        got, ref = got[row_mask.astype(bool)], ref[row_mask.astype(bool)]
    worst = check_close(got, ref)
    print("  max-abs %.3e  items %d (narrow %d, mfma %d, groups %d)" %
          (worst, stats["n_items"], stats["n_narrow"], stats["n_mfma"], stats["n_groups"]), flush=True)
    return out, stats


@pytest.mark.parametrize("seed", [0, 1])
def test_cfg1_tiny_mixed_fp8(seed):
    _compare(si.cfg1_tiny(seed))


def test_cfg1_peaky_queries_fp8():
    _compare(si.cfg1_tiny(0, q_std=4.0))


@pytest.mark.parametrize("Hq,Hkv,D", [(32, 8, 128), (8, 4, 64), (8, 1, 128), (40, 8, 128), (6, 2, 64), (7, 1, 64)])
def test_shapes_and_ragged_lengths_fp8(Hq, Hkv, D):
    """Decode rows, multi-row narrow tiles, append-prefill and full prefill, lengths around page, tile and octet
    boundaries, group sizes 1..8, both head sizes."""
    L = [0, 0, 1, 15, 16, 17, 63, 64, 65, 300, 1000, 129, 191, 0]
    n = [1, 130, 1, 1, 3, 40, 2, 1, 70, 5, 1, 260, 66, 64]
    _compare(si.make_batch("ragged8", L=L, n=n, Hq=Hq, Hkv=Hkv, D=D, seed=41, slack_pages=7))


@pytest.mark.parametrize("seed", range(8))
def test_random_mixed_batches_fp8(seed):
    """The random batches of the 16-bit parity tests (shapes, row mix, lengths and split sizes drawn from the seed) on
    FP8 pages."""
    b, opts = random_mixed_batch(seed)
    _compare(b, options=opts)


def test_scales_that_saturate_and_underflow_fp8():
    """A K scale so small that many elements saturate at 448, a V scale so large that most become subnormal codes."""
    b = si.make_batch("sat8", L=[100, 0, 500], n=[1, 40, 70], Hq=8, Hkv=2, D=128, seed=42, slack_pages=2)
    _compare(b, k_scale=2.0 ** -9, v_scale=9.0)


def test_split_chunks_and_merge_fp8():
    b = si.make_batch("splits8", L=[700, 0, 1500, 333, 4000], n=[1, 200, 90, 2, 1], Hq=32, Hkv=8, D=128, seed=43,
                      slack_pages=3)
    _compare(b, options={"narrow_chunk": 64, "mfma_chunk": 64})
    _compare(b, options={"narrow_chunk": 256, "mfma_chunk": 128, "grid": 3})
    out, _ = _compare(b, options={"narrow_chunk": 512, "mfma_chunk": 512})
    again, _ = _compare(b, options={"narrow_chunk": 512, "mfma_chunk": 512, "pref_mode": 3, "grid": 40})
    assert np.array_equal(out, again), "scheduling changed the result"


def test_wave_tiles_fp8():
    L = [1, 15, 16, 17, 255, 256, 382, 383, 384, 300, 3, 64, 2000, 5000, 333, 90, 0, 400]
    n = [1, 1, 1, 1, 1, 1, 1, 1, 1, 2, 1, 1, 1, 1, 1, 1, 1, 70]
    b = si.make_batch("wave8", L=L, n=n, Hq=32, Hkv=8, D=128, seed=44, slack_pages=3)
    _compare(b, options={"wave_tiles": 1})
    _compare(b, options={"wave_tiles": 1, "narrow_chunk": 512, "mfma_chunk": 512, "grid": 3})


def test_long_rows_of_tiles_fp8():
    """Row-block tiles of many key tiles (the staging ring wraps many times), whole ranges and split ones, and a long
    decode row; sampled rows against the oracle."""
    b = si.make_batch("long8", L=[9000, 0, 20000], n=[300, 700, 1], Hq=32, Hkv=8, D=128, seed=45, slack_pages=2)
    mask = np.zeros(b.T, np.uint8)
    mask[[0, 1, 63, 64, 255, 256, 299, 300, 301, 363, 364, 700, 999, 1000]] = 1
    _compare(b, row_mask=mask)
    _compare(b, row_mask=mask, options={"mfma_chunk": 2048})


def test_static_entry_point_fp8():
    b = si.make_batch("static8", L=[700, 0, 1500, 333], n=[1, 200, 90, 2], Hq=32, Hkv=8, D=128, seed=46, slack_pages=3)
    out, _ = _compare(b)
    out2, _ = _compare(b, static=True)
    assert np.array_equal(out, out2)


def test_kv_land_fp8_bit_exact():
    import torch
    import paper_2603_13358_amd as ppd
    from gpu_helpers import to_dev_u16
    b = si.make_batch("land8", L=[0], n=[333], Hq=8, Hkv=4, D=128, seed=47, slack_pages=3)
    layers = 3
    rng = np.random.default_rng(3)
    k = si.normal_bf16(rng, (layers, 333, 4, 128))
    v = si.normal_bf16(rng, (layers, 333, 4, 128))
    _, _, slots = b.new_part()
    per = oracle.pool_elems(b.num_pages, 4, 128, b.P)
    stride = per + 4096
    ref = np.full(stride * (layers - 1) + per, NAN_CODE, np.uint8)
    oracle.kv_land_fp8(k, v, ref, stride, layers, slots, 4, 128, b.P, b.num_pages, 0.02, 0.05)
    dev = torch.device("cuda:0")
    ctx = ppd.Context(8, 4, 128, b.num_pages)
    ctx.set_kv_format(ppd.PPD_KV_FP8_E4M3, 0.02, 0.05)
    pools = torch.full((ref.size,), NAN_CODE, dtype=torch.uint8, device=dev)
    ctx.kv_land(to_dev_u16(k, torch, dev), to_dev_u16(v, torch, dev), pools, stride, layers,
                torch.from_numpy(slots.astype(np.int64)).to(dev))
    torch.cuda.synchronize()
    assert ctx.device_error_flags() == 0
    assert np.array_equal(pools.cpu().numpy(), ref)
    ctx.close()


def test_fp8_needs_the_one_launch_kernel_and_valid_scales():
    import paper_2603_13358_amd as ppd
    ctx = ppd.Context(8, 2, 64, 16)
    for bad in (0.0, -1.0, float("inf"), float("nan"), 1e-39):
        with pytest.raises(ppd.PPDError):
            ctx.set_kv_format(ppd.PPD_KV_FP8_E4M3, bad, 1.0)
    ctx.close()
    b = si.cfg1_tiny(0)
    from gpu_helpers import gpu_step_fp8
    with pytest.raises(ppd.PPDError):
        gpu_step_fp8(b, 0.02, 0.02, options={"launch_mode": 1})


@pytest.mark.parametrize("k_scale,v_scale", [(1.0, 0.0173), (2.0 ** -9, 9.0), (448.0, 1.0 / 448.0), (3.0e-5, 2.0 ** -120)])
def test_append_codes_of_every_bf16_value(k_scale, v_scale):
    """All 65 536 bf16 bit patterns (zeros, subnormals, ties, the saturation range, infinities, NaNs) through the
    quantising append, for K and for V, against the oracle's codes: bit for bit."""
    import torch
    import paper_2603_13358_amd as ppd
    from gpu_helpers import to_dev_u16
    Hkv, D, P = 2, 64, 16
    T = 65536 // (Hkv * D)
    allbits = np.arange(65536, dtype=np.uint16)
    k = allbits.reshape(T, Hkv, D)
    v = allbits[::-1].copy().reshape(T, Hkv, D)
    num_pages = T // P + 3
    rng = np.random.default_rng(5)
    pages = rng.permutation(num_pages)[:T // P]
    t = np.arange(T)
    slots = pages[t // P].astype(np.int64) * P + t % P
    ref = np.full(oracle.pool_elems(num_pages, Hkv, D, P), NAN_CODE, np.uint8)
    oracle.kv_append_fp8(k, v, ref, slots, Hkv, D, P, num_pages, k_scale, v_scale)
    dev = torch.device("cuda:0")
    ctx = ppd.Context(2 * Hkv, Hkv, D, num_pages)
    ctx.set_kv_format(ppd.PPD_KV_FP8_E4M3, k_scale, v_scale)
    pool = torch.full((ref.size,), NAN_CODE, dtype=torch.uint8, device=dev)
    ctx.kv_append(to_dev_u16(k, torch, dev), to_dev_u16(v, torch, dev), pool, torch.from_numpy(slots).to(dev))
    torch.cuda.synchronize()
    assert ctx.device_error_flags() == 0
    got = pool.cpu().numpy()
    bad = np.argwhere(got != ref)
    assert bad.size == 0, "%d codes differ, first at %s: got %s want %s" % (len(bad), bad[:3].ravel(), got[bad[:3].ravel()], ref[bad[:3].ravel()])
    ctx.close()


def test_single_key_is_exact_fp8():
    """L = 0, n = 1: softmax over one key is 1, so out = value(code) * v_scale rounded once to bf16 -- exactly."""
    from gpu_helpers import gpu_step_fp8
    b = si.make_batch("one8", L=[0, 0, 0], n=[1, 1, 1], Hq=8, Hkv=2, D=128, seed=49, slack_pages=2)
    v_scale = 0.0421
    pool, out, _ = gpu_step_fp8(b, 0.0173, v_scale)
    ref_pool = _oracle_fp8(b, 0.0173, v_scale)
    assert np.array_equal(pool, ref_pool)
    table = np.array([oracle.e4m3_value(c) for c in range(256)], np.float64)
    G = b.Hq // b.Hkv
    for i in range(b.B):
        page = int(b.page_tables[i, 0])
        for hq in range(b.Hq):
            g = hq // G
            S = 2 * b.Hkv * b.P * b.D
            base = page * S + b.Hkv * b.P * b.D + g * b.P * b.D      # V block of the head; token 0: octet 0, slot 0
            codes = ref_pool[base + np.arange(b.D) * 8]
            want = si.f32_to_bf16_bits((table[codes].astype(np.float32) * np.float32(v_scale)).astype(np.float32))
            assert np.array_equal(out[i, hq], want), (i, hq)
