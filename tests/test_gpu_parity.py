"""Parity of the HIP path against the CPU oracle, element by element, through the C ABI (needs an MI355X).

Bar: KV append bit-exact; attention max-abs <= 2e-2 and per-(row, head) relative L2 <= 1e-2 against the
double-precision oracle (bf16 inputs, fp32 accumulation, bf16 probabilities and output on the GPU side).
"""
import numpy as np
import pytest

import synthetic_inputs as si
from helpers import bits_to_f32, check_close, oracle_out, oracle_pool, random_mixed_batch

pytestmark = pytest.mark.gpu


def _step(b, **kw):
    from gpu_helpers import gpu_step
    return gpu_step(b, **kw)


def _compare(b, **kw):
    print("case", b.name, "L", b.L.tolist()[:8], "n", b.n.tolist()[:8], kw, flush=True)
    ref_pool = oracle_pool(b)
    pool, out, stats = _step(b, **kw)
    assert np.array_equal(pool, ref_pool), "KV append is not bit-exact"
    ref = oracle_out(b, ref_pool)
    worst = check_close(bits_to_f32(out), ref)
    print("  max-abs %.3e  items %d (narrow %d, mfma %d, groups %d)" %
          (worst, stats["n_items"], stats["n_narrow"], stats["n_mfma"], stats["n_groups"]), flush=True)
    return out, stats


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_cfg1_tiny_mixed(seed):
    _compare(si.cfg1_tiny(seed))


def test_cfg1_peaky_queries():
    """q scaled x4: outputs are O(1) so the absolute bound bites."""
    _compare(si.cfg1_tiny(0, q_std=4.0))


@pytest.mark.parametrize("Hq,Hkv,D", [(32, 8, 128), (8, 8, 128), (8, 4, 64), (8, 1, 128), (16, 2, 64),
                                      (40, 8, 128), (32, 4, 128), (6, 2, 64), (12, 2, 128), (7, 1, 64)])
def test_shapes_and_ragged_lengths(Hq, Hkv, D):
    """Group sizes G = Hq/Hkv from 1 to 8, powers of two or not (40/8 and 32/4 are the head shapes of the other
    two models the paper serves, section 5.1)."""
    L = [0, 0, 1, 15, 16, 17, 63, 64, 65, 300, 1000, 129]
    n = [1, 130, 1, 1, 3, 40, 2, 1, 70, 5, 1, 260]
    _compare(si.make_batch("ragged", L=L, n=n, Hq=Hq, Hkv=Hkv, D=D, seed=21, slack_pages=7))


def test_split_chunks_and_merge():
    """Small forced split sizes: many partials per row block, several tiles per split, ragged tails."""
    b = si.make_batch("splits", L=[700, 0, 1500, 333], n=[1, 200, 90, 2], Hq=32, Hkv=8, D=128, seed=22, slack_pages=3)
    _compare(b, options={"narrow_chunk": 64, "mfma_chunk": 64})
    _compare(b, options={"narrow_chunk": 256, "mfma_chunk": 128, "grid": 3})


def test_split_chunks_and_merge_group_of_five():
    """G = 5: row blocks of 51 rows (255 of 256 columns), narrow tiles up to 3 rows, split and merged."""
    b = si.make_batch("splits5", L=[700, 0, 1500, 333, 64], n=[1, 200, 90, 2, 3], Hq=40, Hkv=8, D=128, seed=24,
                      slack_pages=3)
    _compare(b, options={"narrow_chunk": 256, "mfma_chunk": 512})


@pytest.mark.parametrize("options", [{"pref_mode": 0}, {"pref_mode": 1}, {"pref_mode": 3}, {"narrow_cus": 0},
                                     {"narrow_cus": 5}, {"narrow_cus": 32}, {"grid": 1}, {"grid": 40, "narrow_cus": 16}])
def test_scheduling_options_do_not_change_the_result(options):
    """Which workgroup takes which tile (kind preference, split of the compute units, grid size) is scheduling
    only: same tiles, same partials, bitwise the same output."""
    b = si.make_batch("sched", L=[900, 0, 2500, 333, 64, 4000, 17], n=[1, 150, 70, 2, 3, 1, 1], Hq=32, Hkv=8, D=128,
                      seed=25, slack_pages=3)
    base, _ = _compare(b, options={"narrow_chunk": 512, "mfma_chunk": 512})
    out, _ = _compare(b, options=dict(options, narrow_chunk=512, mfma_chunk=512))
    assert np.array_equal(out, base)


@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("shape", [(32, 8, 128), (8, 2, 64), (40, 8, 128), (16, 2, 128)])
def test_resident_pair_of_kernels_matches_oracle(mode, shape):
    """launch_mode 1 / 2: narrow tiles on the stream kernel (4 waves, its own stream), row-block tiles on the
    row-block kernel (half-tile loop), both resident on every compute unit at once; split key ranges so that partials
    and the merge are in play; decode rows, small multi-row narrow tiles, append-prefill and full prefill together."""
    Hq, Hkv, D = shape
    b = si.make_batch("pair", L=[900, 0, 2500, 333, 64, 4000, 17, 1203, 0, 5000], n=[1, 150, 70, 2, 3, 1, 1, 65, 1, 1],
                      Hq=Hq, Hkv=Hkv, D=D, seed=26 + mode, slack_pages=3)
    for opts in ({}, {"narrow_chunk": 512, "mfma_chunk": 512}):
        out, stats = _compare(b, options=dict(opts, launch_mode=mode))
        assert stats["n_narrow"] > 0 and stats["n_mfma"] > 0
        again, _ = _compare(b, options=dict(opts, launch_mode=mode))
        assert np.array_equal(out, again), "not deterministic"


@pytest.mark.parametrize("shape", [(32, 8, 128), (64, 8, 128), (8, 2, 64), (40, 8, 128), (6, 6, 64)])
def test_wave_tiles_match_oracle(shape):
    """Option wave_tiles = 1: narrow tiles of at most 384 keys run one per wave, eight to a claim (no combine through
    LDS, output straight from the accumulators): decode rows of lengths around page and claim boundaries, multi-row
    narrow tiles, a count that is no multiple of eight, longer tiles and an append-prefill beside them, and split
    ranges whose short pieces write partials."""
    Hq, Hkv, D = shape
    L = [1, 15, 16, 17, 255, 256, 382, 383, 384, 300, 3, 64, 2000, 5000, 333, 90, 0, 400]
    n = [1, 1, 1, 1, 1, 1, 1, 1, 1, 2, 1, 1, 1, 1, 1, 1, 1, 70]
    b = si.make_batch("wave", L=L, n=n, Hq=Hq, Hkv=Hkv, D=D, seed=33, slack_pages=3)
    out, stats = _compare(b, options={"wave_tiles": 1})
    base, _ = _compare(b, options={"wave_tiles": 0})
    check_close(bits_to_f32(out), bits_to_f32(base), max_abs=2e-2, rel=1e-2)
    again, _ = _compare(b, options={"wave_tiles": 1})
    assert np.array_equal(out, again), "not deterministic"
    _compare(b, options={"wave_tiles": 1, "narrow_chunk": 512, "mfma_chunk": 512, "grid": 3})


def test_wave_tiles_chosen_automatically_for_large_decode_batches():
    """2048 short decode tiles (256 sequences x 8 KV heads): the planner picks the wave queue by itself."""
    rng = np.random.default_rng(8)
    b = si.make_batch("wave_auto", L=rng.integers(1, 380, size=256), n=np.ones(256, np.int64), Hq=16, Hkv=8, D=128,
                      seed=34, slack_pages=5)
    out, stats = _compare(b)
    assert stats["grid"] == 256 and stats["n_narrow"] == 2048


def test_decode_only_kernel_is_the_mixed_kernel_bit_for_bit():
    """A step without row-block tiles runs ppd_narrow_kernel (first tiles by workgroup index): against the oracle, and
    bit for bit against the one-launch kernel (option narrow_kernel = 0), with fewer slots than workgroups, with more
    (claims through the cursor), with one-wave tiles, with split ranges, and twice in a row on one context."""
    rng = np.random.default_rng(9)
    few = si.make_batch("dec_few", L=[900, 17, 4000, 0, 2047], n=[1, 1, 1, 3, 1], Hq=32, Hkv=8, D=128, seed=35, slack_pages=3)
    many = si.make_batch("dec_many", L=rng.integers(1, 700, size=300), n=np.ones(300, np.int64), Hq=16, Hkv=8, D=128,
                         seed=36, slack_pages=5)
    small_heads = si.make_batch("dec_d64", L=rng.integers(0, 3000, size=40), n=np.ones(40, np.int64), Hq=8, Hkv=2, D=64,
                                seed=37, slack_pages=2)
    for b, extra in ((few, {}), (few, {"narrow_chunk": 256}), (few, {"grid": 3}), (many, {}), (many, {"wave_tiles": 0}),
                     (many, {"grid": 7, "wave_tiles": 1}), (small_heads, {})):
        out, stats = _compare(b, options=dict(extra))
        assert stats["n_mfma"] == 0
        base, _ = _compare(b, options=dict(extra, narrow_kernel=0))
        assert np.array_equal(out, base), "the two kernels disagree"
    # the cursor is left re-armed: one context runs a claiming launch three times, then the one-launch kernel (which
    # claims from the same cursor) on the same batch
    import torch
    import paper_2603_13358_amd as ppd
    from gpu_helpers import to_dev_u16, from_dev_u16
    dev = torch.device("cuda:0")
    ctx = ppd.Context(many.Hq, many.Hkv, many.D, many.num_pages)
    ctx.set_option("grid", 16)
    pool = torch.zeros(ctx.pool_elems(), dtype=torch.int16, device=dev)
    for k, v, slots in (many.cached_part(), many.new_part()):
        if len(slots):
            ctx.kv_append(to_dev_u16(k, torch, dev), to_dev_u16(v, torch, dev), pool, torch.from_numpy(slots.astype(np.int64)).to(dev))
    q = to_dev_u16(many.q, torch, dev)
    pt = torch.from_numpy(many.page_tables).to(dev)
    outs = []
    for call in range(4):
        if call == 3:
            ctx.set_option("narrow_kernel", 0)
        out = torch.zeros((many.T, many.Hq, many.D), dtype=torch.int16, device=dev)
        ctx.mixed_attention(q, pool, pt, many.L, many.n, many.scale, out)
        torch.cuda.synchronize()
        outs.append(from_dev_u16(out))
    assert ctx.device_error_flags() == 0
    assert all(np.array_equal(outs[0], o) for o in outs[1:])
    check_close(bits_to_f32(outs[0]).reshape(many.T, many.Hq, many.D), oracle_out(many, oracle_pool(many, fill=0)))
    ctx.close()


def test_resident_pair_only_one_kind_present():
    """launch_mode 2 with batches of one kind: each specialised kernel alone, no fork to the side stream."""
    dec = si.make_batch("pair_dec", L=[900, 17, 4000, 0, 2047, 2048, 2049], n=[1, 1, 1, 1, 1, 2, 1], Hq=32, Hkv=8,
                        D=128, seed=29, slack_pages=3)
    ap = si.make_batch("pair_ap", L=[900, 0, 2500], n=[150, 70, 257], Hq=32, Hkv=8, D=128, seed=30, slack_pages=3)
    for b in (dec, ap):
        _compare(b, options={"launch_mode": 2})
        _compare(b, options={"launch_mode": 2, "narrow_chunk": 256, "mfma_chunk": 256})


@pytest.mark.parametrize("seed", range(8))
def test_random_mixed_batches(seed):
    """Random batches: sequence count, head shape, the mix of decode / append-prefill / full-prefill rows, lengths
    around page, tile and row-block boundaries, and split sizes all drawn from the seed."""
    b, opts = random_mixed_batch(seed)
    _compare(b, options=opts)


def test_decode_batch_scaled():
    _compare(si.cfg2_decode(0, B=12, Lmin=100, Lmax=3000))


def test_append_prefill_batch_scaled():
    _compare(si.cfg3_append_prefill(0, B=4, Lmin=200, Lmax=1500, n_median=60, n_lo=16, n_hi=200))


def test_mixed_batch_scaled_and_full_prefill_variant():
    kw = dict(n_decode=10, n_ap=2, dec_L=(100, 2000), ap_L=(300, 1500), ap_n=(40, 150))
    _compare(si.cfg4_mixed(0, **kw))
    _compare(si.cfg4_mixed(0, full_prefill=True, **kw))


def test_n1_append_prefill_equals_decode():
    """The same decode rows through the narrow path and through the MFMA row-block path."""
    b = si.cfg2_decode(3, B=6, Lmin=50, Lmax=900)
    out_a, st_a = _compare(b)
    out_b, st_b = _compare(b, options={"force_kind": 1})
    assert st_a["n_mfma"] == 0 and st_b["n_narrow"] == 0
    check_close(bits_to_f32(out_b), bits_to_f32(out_a).astype(np.float64), max_abs=2e-2, rel=1e-2)


def test_append_prefill_equals_tail_of_recompute_on_gpu():
    b = si.make_batch("ap", L=[500, 77], n=[100, 30], Hq=32, Hkv=8, D=128, seed=23)
    _, out_ap, _ = _step(b)
    tot = (b.L + b.n).astype(np.int32)
    rng = np.random.default_rng(5)
    qf = si.normal_bf16(rng, (int(tot.sum()), b.Hq, b.D))
    at = 0
    for i in range(b.B):
        qf[at + int(b.L[i]):at + int(tot[i])] = b.q[int(b.row_off[i]):int(b.row_off[i + 1])]
        at += int(tot[i])
    full = si.MixedBatch(name="full", Hq=b.Hq, Hkv=b.Hkv, D=b.D, P=b.P, num_pages=b.num_pages, scale=b.scale,
                         L=np.zeros(b.B, np.int32), n=tot, page_tables=b.page_tables, q=qf, k=b.k, v=b.v)
    _, out_full, _ = _step(full)
    at = 0
    for i in range(b.B):
        tail = bits_to_f32(out_full[at + int(b.L[i]):at + int(tot[i])])
        mine = bits_to_f32(out_ap[int(b.row_off[i]):int(b.row_off[i + 1])])
        check_close(mine, tail.astype(np.float64))
        at += int(tot[i])


def test_page_relabelling_and_determinism():
    b = si.cfg1_tiny(1)
    _, out1, _ = _step(b)
    _, out2, _ = _step(b)
    assert np.array_equal(out1, out2), "not run-to-run deterministic"
    rng = np.random.default_rng(99)
    relabel = rng.permutation(b.num_pages).astype(np.int32)
    pt = np.where(b.page_tables >= 0, relabel[np.maximum(b.page_tables, 0)], -1).astype(np.int32)
    b2 = si.MixedBatch(name="perm", Hq=b.Hq, Hkv=b.Hkv, D=b.D, P=b.P, num_pages=b.num_pages, scale=b.scale,
                       L=b.L, n=b.n, page_tables=pt, q=b.q, k=b.k, v=b.v)
    _, out3, _ = _step(b2)
    assert np.array_equal(out1, out3), "page order changed the result"


def test_single_key_is_exact_and_scale_zero():
    b = si.make_batch("one", L=[0, 0], n=[1, 1], Hq=8, Hkv=2, D=64, seed=24)
    _, out, _ = _step(b)
    for i in range(2):
        _, v = b.seq_kv(i)
        for h in range(8):
            assert np.array_equal(out[i, h], v[0, h // 4])
    bz = si.make_batch("z", L=[40, 0], n=[1, 20], Hq=8, Hkv=2, D=64, seed=25)
    bz.scale = 0.0
    _compare(bz)


def test_append_in_one_call_and_skipped_slots():
    import torch
    import paper_2603_13358_amd as ppd
    from gpu_helpers import from_dev_u16, to_dev_u16
    b = si.cfg1_tiny(2)
    pool_a, _, _ = _step(b)
    pool_b, _, _ = _step(b, append_in_one_call=True)
    assert np.array_equal(pool_a, pool_b)
    # negative slots are skipped; slots beyond the pool are skipped and flagged
    dev = torch.device("cuda:0")
    ctx = ppd.Context(b.Hq, b.Hkv, b.D, b.num_pages)
    pool = torch.zeros((ctx.pool_elems(),), dtype=torch.int16, device=dev)
    k, v, slots = b.new_part()
    slots = slots.copy()
    slots[3] = -1
    slots[10] = b.num_pages * b.P + 5
    ctx.kv_append(to_dev_u16(k, torch, dev), to_dev_u16(v, torch, dev), pool, torch.from_numpy(slots).to(dev))
    assert ctx.device_error_flags() == 1
    assert ctx.device_error_flags() == 0
    import oracle
    ref = np.zeros(ctx.pool_elems(), np.uint16)
    slots[10] = -1
    oracle.kv_append(k, v, ref, slots, b.Hkv, b.D, b.P, b.num_pages)
    assert np.array_equal(from_dev_u16(pool), ref)
    ctx.close()


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_append_slot_patterns_bit_exact(seed):
    """Runs of consecutive slots that start anywhere, whole aligned groups of 8, skipped tokens inside a run,
    groups written back to front, isolated tokens, a batch that is not a multiple of 8 tokens long."""
    import torch
    import oracle
    import paper_2603_13358_amd as ppd
    from gpu_helpers import from_dev_u16, to_dev_u16
    rng = np.random.default_rng(100 + seed)
    Hkv, D, P, num_pages = (2, 64, 16, 96) if seed % 2 else (8, 128, 16, 96)
    free = list(rng.permutation(num_pages * P // 8))           # aligned groups of 8 slots, each used at most once
    slots = []
    while len(slots) < 300 + 3 * seed:
        kind = rng.integers(0, 5)
        g = int(free.pop()) * 8
        if kind == 0:                                          # a whole aligned group
            slots += list(range(g, g + 8))
        elif kind == 1:                                        # a run that starts inside a group and goes on in another
            g2 = int(free.pop()) * 8
            a = int(rng.integers(1, 8))
            slots += list(range(g + a, g + 8)) + list(range(g2, g2 + int(rng.integers(1, 9))))
        elif kind == 2:                                        # a group with one token skipped
            run = list(range(g, g + 8))
            run[int(rng.integers(0, 8))] = -1
            slots += run
        elif kind == 3:                                        # an isolated token
            slots += [g + int(rng.integers(0, 8))]
        else:                                                  # a group written back to front
            slots += list(range(g + 7, g - 1, -1))
    slots = np.asarray(slots, np.int64)
    T = len(slots)
    print("case append patterns seed", seed, "T", T, "Hkv", Hkv, "D", D, flush=True)
    k = si.normal_bf16(rng, (T, Hkv, D))
    v = si.normal_bf16(rng, (T, Hkv, D))
    dev = torch.device("cuda:0")
    ctx = ppd.Context(Hkv, Hkv, D, num_pages)
    pool = torch.full((ctx.pool_elems(),), 0x1234, dtype=torch.int16, device=dev)
    ctx.kv_append(to_dev_u16(k, torch, dev), to_dev_u16(v, torch, dev), pool, torch.from_numpy(slots).to(dev))
    assert ctx.device_error_flags() == 0
    ref = np.full(ctx.pool_elems(), 0x1234, np.uint16)
    oracle.kv_append(k, v, ref, slots, Hkv, D, P, num_pages)
    assert np.array_equal(from_dev_u16(pool), ref)
    ctx.close()


def test_bad_page_id_is_flagged_not_dereferenced():
    import torch
    import paper_2603_13358_amd as ppd
    from gpu_helpers import to_dev_u16
    b = si.make_batch("bad", L=[40], n=[1], Hq=8, Hkv=2, D=64, seed=26)
    dev = torch.device("cuda:0")
    ctx = ppd.Context(b.Hq, b.Hkv, b.D, b.num_pages)
    pool = torch.zeros((ctx.pool_elems(),), dtype=torch.int16, device=dev)
    pt = b.page_tables.copy()
    pt[0, 1] = b.num_pages + 1000
    out = torch.zeros((b.T, b.Hq, b.D), dtype=torch.int16, device=dev)
    ctx.mixed_attention(to_dev_u16(b.q, torch, dev), pool, torch.from_numpy(pt).to(dev), b.L, b.n, b.scale, out)
    assert ctx.device_error_flags() == 2
    ctx.close()


def test_host_argument_errors_enqueue_nothing():
    import torch
    import paper_2603_13358_amd as ppd
    from gpu_helpers import to_dev_u16
    b = si.cfg1_tiny(0)
    dev = torch.device("cuda:0")
    ctx = ppd.Context(b.Hq, b.Hkv, b.D, b.num_pages)
    pool = torch.zeros((ctx.pool_elems(),), dtype=torch.int16, device=dev)
    out = torch.full((b.T, b.Hq, b.D), 7, dtype=torch.int16, device=dev)
    q = to_dev_u16(b.q, torch, dev)
    pt = torch.from_numpy(b.page_tables).to(dev)
    cases = [
        (dict(n=[64, 0, 12, 1]), -3), (dict(L=[0, -1, 100, 256]), -3), (dict(scale=-1.0), -3),
        (dict(scale=float("nan")), -3), (dict(max_pages=3), -4),
    ]
    for kw, code in cases:
        args = dict(L=b.L, n=b.n, scale=b.scale, max_pages=None)
        args.update(kw)
        with pytest.raises(ppd.PPDError) as e:
            ppd.ppd_mixed_attention(ctx.handle, q, pool, pt, args["L"], args["n"], args["scale"], out,
                                    max_pages=args["max_pages"])
        assert e.value.status == code, (kw, e.value)
    with pytest.raises(ppd.PPDError) as e:
        ppd.ppd_mixed_attention(ctx.handle, None, pool, pt, b.L, b.n, b.scale, out)
    assert e.value.status == -1
    # tensors that do not start on a 16-byte boundary are rejected (views shifted by one element)
    q_odd = torch.empty(q.numel() + 1, dtype=torch.int16, device=dev)[1:]
    pool_odd = torch.empty(pool.numel() + 1, dtype=torch.int16, device=dev)[1:]
    for args in [(q_odd, pool, out), (q, pool_odd, out), (q, pool, q_odd)]:
        with pytest.raises(ppd.PPDError) as e:
            ppd.ppd_mixed_attention(ctx.handle, args[0], args[1], pt, b.L, b.n, b.scale, args[2])
        assert e.value.status == -3
    kk, vv, slots = b.new_part()
    with pytest.raises(ppd.PPDError) as e:
        ppd.ppd_kv_append(ctx.handle, to_dev_u16(kk, torch, dev), to_dev_u16(vv, torch, dev), pool_odd,
                          torch.from_numpy(slots.astype(np.int64)).to(dev))
    assert e.value.status == -3
    torch.cuda.synchronize()
    assert bool((out == 7).all()), "a rejected call touched the output"
    assert bool((pool == 0).all()), "a rejected call touched the pool"
    # empty batch and empty append are no-ops
    ppd.ppd_mixed_attention(ctx.handle, q, pool, pt, np.zeros(0, np.int32), np.zeros(0, np.int32), b.scale, out)
    ppd.ppd_kv_append(ctx.handle, None, None, pool, None, T=0)
    ctx.close()
    for shape, code in [((8, 2, 96, 16, 4), -2), ((8, 2, 64, 32, 4), -2), ((8, 3, 64, 16, 4), -2),
                        ((32, 2, 64, 16, 4), -2), ((8, 2, 64, 16, 0), -2)]:
        with pytest.raises(ppd.PPDError) as e:
            ppd.ppd_create(*shape)
        assert e.value.status == code


def test_many_short_sequences():
    """2000 sequences in one launch (many more tiles than workgroups), decode rows and two-row blocks."""
    rng = np.random.default_rng(41)
    B = 2000
    L = rng.integers(0, 120, size=B)
    n = np.where(rng.random(B) < 0.9, 1, 2)
    _compare(si.make_batch("many", L=L, n=n, Hq=16, Hkv=4, D=64, seed=41, slack_pages=3))


def test_side_stream_and_two_contexts():
    """Both calls are asynchronous on the stream they are given; two contexts of different shapes used in turn on
    two streams do not disturb each other."""
    import torch
    import paper_2603_13358_amd as ppd
    from gpu_helpers import from_dev_u16, to_dev_u16
    dev = torch.device("cuda:0")
    batches = [si.make_batch("s0", L=[300, 0, 77], n=[1, 90, 3], Hq=32, Hkv=8, D=128, seed=51, slack_pages=2),
               si.make_batch("s1", L=[40, 900], n=[20, 1], Hq=8, Hkv=2, D=64, seed=52, slack_pages=2)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    state = []
    for b, st in zip(batches, streams):
        ctx = ppd.Context(b.Hq, b.Hkv, b.D, b.num_pages)
        with torch.cuda.stream(st):
            pool = torch.full((ctx.pool_elems(),), 0x7FC1, dtype=torch.int16, device=dev)
            out = torch.zeros((b.T, b.Hq, b.D), dtype=torch.int16, device=dev)
            dev_in = [(to_dev_u16(k, torch, dev), to_dev_u16(v, torch, dev), torch.from_numpy(s_.astype(np.int64)).to(dev))
                      for k, v, s_ in (b.cached_part(), b.new_part()) if len(s_)]
            q = to_dev_u16(b.q, torch, dev)
            pt = torch.from_numpy(b.page_tables).to(dev)
        st.synchronize()
        state.append((ctx, pool, out, dev_in, q, pt))
    for rep in range(3):                                   # interleave the two contexts, nothing waits in between
        for (ctx, pool, out, dev_in, q, pt), b, st in zip(state, batches, streams):
            for k, v, s_ in dev_in:
                ctx.kv_append(k, v, pool, s_, stream=st.cuda_stream)
            ctx.mixed_attention(q, pool, pt, b.L, b.n, b.scale, out, stream=st.cuda_stream)
    for (ctx, pool, out, dev_in, q, pt), b, st in zip(state, batches, streams):
        st.synchronize()
        assert ctx.device_error_flags(stream=st.cuda_stream) == 0
        ref_pool = oracle_pool(b)
        assert np.array_equal(from_dev_u16(pool), ref_pool)
        check_close(bits_to_f32(from_dev_u16(out).reshape(b.T, b.Hq, b.D)), oracle_out(b, ref_pool))
        ctx.close()


def test_step_replays_from_a_hip_graph():
    """A step whose plan is already on the device is two or three kernel launches and nothing else: captured into a
    HIP graph it replays bit-identically, also with eager work and synchronisations between the replays."""
    import torch
    from gpu_helpers import from_dev_u16, to_dev_u16
    b = si.make_batch("graph", L=[900, 0, 2500, 333, 64, 4000], n=[1, 150, 70, 2, 3, 1], Hq=32, Hkv=8, D=128, seed=61,
                      slack_pages=3)
    pool_ref, out_ref, stats, ctx = _step(b, return_ctx=True, options={"narrow_chunk": 512, "mfma_chunk": 512})
    assert stats["n_groups"] > 0                      # the merge kernel is part of the step
    dev = torch.device("cuda:0")
    pool = to_dev_u16(oracle_pool(b, parts=("cached",)), torch, dev)
    k, v, slots = b.new_part()
    kd, vd = to_dev_u16(k, torch, dev), to_dev_u16(v, torch, dev)
    sd = torch.from_numpy(slots.astype(np.int64)).to(dev)
    q = to_dev_u16(b.q, torch, dev)
    pt = torch.from_numpy(b.page_tables).to(dev)
    out = torch.zeros((b.T, b.Hq, b.D), dtype=torch.int16, device=dev)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # same L, n, options as the step above: the plan is reused
        ctx.kv_append(kd, vd, pool, sd, stream=side.cuda_stream)
        ctx.mixed_attention(q, pool, pt, b.L, b.n, b.scale, out, stream=side.cuda_stream)
    side.synchronize()
    assert np.array_equal(from_dev_u16(out).reshape(out_ref.shape), out_ref)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        s = torch.cuda.current_stream().cuda_stream
        ctx.kv_append(kd, vd, pool, sd, stream=s)
        ctx.mixed_attention(q, pool, pt, b.L, b.n, b.scale, out, stream=s)
    for rep in range(4):
        out.fill_(7)
        scratch = torch.randn(1 << 20, device=dev).sum().item()      # eager work and a synchronisation in between
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(from_dev_u16(out).reshape(out_ref.shape), out_ref), "replay %d differs" % rep
    assert np.array_equal(from_dev_u16(pool), pool_ref)
    assert ctx.device_error_flags() == 0
    del graph
    ctx.close()


def test_decode_only_step_replays_from_a_hip_graph():
    """The same for a step without row-block tiles (the decode-only kernel), with more slots than workgroups so that
    every replay claims from the cursor the replay before it has re-armed."""
    import torch
    from gpu_helpers import from_dev_u16, to_dev_u16
    rng = np.random.default_rng(63)
    b = si.make_batch("graph_dec", L=rng.integers(1, 900, size=60), n=np.ones(60, np.int64), Hq=32, Hkv=8, D=128, seed=63,
                      slack_pages=3)
    pool_ref, out_ref, stats, ctx = _step(b, return_ctx=True, options={"grid": 16})
    assert stats["n_mfma"] == 0 and stats["n_narrow"] > 16
    dev = torch.device("cuda:0")
    pool = to_dev_u16(pool_ref, torch, dev)
    q = to_dev_u16(b.q, torch, dev)
    pt = torch.from_numpy(b.page_tables).to(dev)
    out = torch.zeros((b.T, b.Hq, b.D), dtype=torch.int16, device=dev)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ctx.mixed_attention(q, pool, pt, b.L, b.n, b.scale, out, stream=torch.cuda.current_stream().cuda_stream)
    for rep in range(4):
        out.fill_(7)
        scratch = torch.randn(1 << 20, device=dev).sum().item()      # eager work and a synchronisation in between
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(from_dev_u16(out).reshape(out_ref.shape), out_ref), "replay %d differs" % rep
    assert ctx.device_error_flags() == 0
    del graph
    ctx.close()


def test_plan_change_under_capture_is_refused():
    """A call whose plan is not on the device yet would have to synchronise and allocate: under stream capture it is
    refused on the host, with nothing enqueued, and the capture stays valid."""
    import torch
    import paper_2603_13358_amd as ppd
    from gpu_helpers import from_dev_u16, to_dev_u16
    b = si.make_batch("cap", L=[300, 0, 70], n=[1, 40, 3], Hq=16, Hkv=2, D=128, seed=62, slack_pages=2)
    pool_ref, out_ref, stats, ctx = _step(b, return_ctx=True)
    dev = torch.device("cuda:0")
    pool = to_dev_u16(pool_ref, torch, dev)
    q = to_dev_u16(b.q, torch, dev)
    pt = torch.from_numpy(b.page_tables).to(dev)
    out = torch.zeros((b.T, b.Hq, b.D), dtype=torch.int16, device=dev)
    other_L = b.L.copy()
    other_L[0] -= 1
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        s = torch.cuda.current_stream().cuda_stream
        with pytest.raises(ppd.PPDError) as e:
            ctx.mixed_attention(q, pool, pt, other_L, b.n, b.scale, out, stream=s)
        assert e.value.status == -3 and "capture" in str(e.value)
        ctx.mixed_attention(q, pool, pt, b.L, b.n, b.scale, out, stream=s)      # same lengths: launches only
    graph.replay()
    torch.cuda.synchronize()
    assert np.array_equal(from_dev_u16(out).reshape(out_ref.shape), out_ref)
    assert ctx.device_error_flags() == 0
    del graph
    ctx.close()


def test_kernel_timing_series():
    """Option "timing": one pair of events per launch; the series is read (and restarted) in one call."""
    import torch
    import paper_2603_13358_amd as ppd
    b = si.cfg1_tiny(0)
    pool, out, stats, ctx = _step(b, return_ctx=True)
    with pytest.raises(ppd.PPDError):
        ctx.last_kernel_ms()                       # nothing was timed yet
    assert ctx.timed_kernels_ms() == (0.0, 0)
    dev = torch.device("cuda:0")
    from gpu_helpers import to_dev_u16
    q = to_dev_u16(b.q, torch, dev)
    pl = to_dev_u16(pool, torch, dev)
    pt = torch.from_numpy(b.page_tables).to(dev)
    o = torch.empty((b.T, b.Hq, b.D), dtype=torch.int16, device=dev)
    ctx.set_option("timing", 1)
    for _ in range(3):
        ctx.mixed_attention(q, pl, pt, b.L, b.n, b.scale, o)
    last = ctx.last_kernel_ms()
    total, launches = ctx.timed_kernels_ms()
    assert launches == 3 and 0.0 < last < total < 50.0
    assert ctx.timed_kernels_ms() == (0.0, 0)
    ctx.set_option("timing", 0)
    ctx.mixed_attention(q, pl, pt, b.L, b.n, b.scale, o)
    assert ctx.timed_kernels_ms() == (0.0, 0)
    torch.cuda.synchronize()
    assert np.array_equal(o.cpu().numpy().view(np.uint16), out)
    ctx.close()


def test_chunked_append_prefill_equals_one_shot():
    """An append-prefill fed in chunks over several steps (token-budgeted steps, as chunked-prefill schedulers
    do; the paper's related work, section 2.2) gives the rows of the one-shot append-prefill: each chunk is an
    append-prefill whose cached length is everything before it."""
    import torch
    import paper_2603_13358_amd as ppd
    from gpu_helpers import from_dev_u16, to_dev_u16
    b = si.make_batch("chunks", L=[700, 90], n=[300, 300], Hq=32, Hkv=8, D=128, seed=41, slack_pages=2)
    ref = oracle_out(b)
    dev = torch.device("cuda:0")
    ctx = ppd.Context(b.Hq, b.Hkv, b.D, b.num_pages)
    pool = torch.zeros((ctx.pool_elems(),), dtype=torch.int16, device=dev)
    k, v, slots = b.cached_part()
    ctx.kv_append(to_dev_u16(k, torch, dev), to_dev_u16(v, torch, dev), pool, torch.from_numpy(slots).to(dev))
    pt = torch.from_numpy(b.page_tables).to(dev)
    done = np.zeros(2, np.int32)
    for chunk in (64, 100, 136):
        ks, vs, ss, qs = [], [], [], []
        for i in range(2):
            kk, vv = b.seq_kv(i)
            a = int(b.L[i] + done[i])
            ks.append(kk[a:a + chunk]); vs.append(vv[a:a + chunk]); ss.append(b.slots(i, a, a + chunk))
            r0 = int(b.row_off[i] + done[i])
            qs.append(b.q[r0:r0 + chunk])
        ctx.kv_append(to_dev_u16(np.concatenate(ks), torch, dev), to_dev_u16(np.concatenate(vs), torch, dev), pool,
                      torch.from_numpy(np.concatenate(ss)).to(dev))
        out = torch.zeros((2 * chunk, b.Hq, b.D), dtype=torch.int16, device=dev)
        ctx.mixed_attention(to_dev_u16(np.concatenate(qs), torch, dev), pool, pt, b.L + done, [chunk, chunk], b.scale, out)
        got = bits_to_f32(from_dev_u16(out).reshape(2 * chunk, b.Hq, b.D))
        for i in range(2):
            r0 = int(b.row_off[i] + done[i])
            check_close(got[i * chunk:(i + 1) * chunk], ref[r0:r0 + chunk])
        done += chunk
    assert ctx.device_error_flags() == 0
    ctx.close()


def test_kv_land_all_layers_bit_exact():
    import torch
    import oracle
    import paper_2603_13358_amd as ppd
    from gpu_helpers import from_dev_u16, to_dev_u16
    from helpers import SENTINEL
    b = si.make_batch("land", L=[333, 40, 1000], n=[1, 1, 1], Hq=32, Hkv=8, D=128, seed=51, slack_pages=4)
    layers, pe = 4, oracle.pool_elems(b.num_pages, b.Hkv, b.D, b.P)
    stride = pe + 4096
    rng = np.random.default_rng(6)
    _, _, slots = b.cached_part()
    slots = slots.copy()
    slots[7] = -1                                   # a skipped token
    T = len(slots)
    k = si.normal_bf16(rng, (layers, T, b.Hkv, b.D))
    v = si.normal_bf16(rng, (layers, T, b.Hkv, b.D))
    total = stride * (layers - 1) + pe
    ref = np.full(total, SENTINEL, np.uint16)
    oracle.kv_land(k, v, ref, stride, layers, slots, b.Hkv, b.D, b.P, b.num_pages)
    dev = torch.device("cuda:0")
    ctx = ppd.Context(b.Hq, b.Hkv, b.D, b.num_pages)
    fill = int(np.array([SENTINEL], np.uint16).view(np.int16)[0])
    pools = torch.full((total,), fill, dtype=torch.int16, device=dev)
    ctx.kv_land(to_dev_u16(k, torch, dev), to_dev_u16(v, torch, dev), pools, stride, layers,
                torch.from_numpy(slots).to(dev))
    torch.cuda.synchronize()
    assert ctx.device_error_flags() == 0
    assert np.array_equal(from_dev_u16(pools), ref)
    with pytest.raises(ppd.PPDError) as e:
        ctx.kv_land(pools, pools, pools, pe - 1, 2, torch.from_numpy(slots).to(dev))
    assert e.value.status == -3
    assert abs(ppd.ppd_transfer_delay_s(5115, 131072, 25e9, 0.0045) -
               oracle.transfer_delay(5115, 131072, 25e9, 0.0045)) < 1e-15
    ctx.close()


def test_measured_route_table_reproduces_the_papers_regime():
    """Offline phase of the routing algorithm (section 5) fed with this repository's own measurements, on four cells of
    the grid: where the paper finds local append-prefill to win -- large accumulated context, prefill-heavy turn,
    KV transfer over a 25 GB/s link (94-96 % lower TTFT for a few percent of decode slowdown, sections 4 and 6) -- the
    measured table says x = 1 with a TTFT gain above one half; an operator who weights only decode smoothness gets
    x = 0 in every cell that costs decode time at all; cells never measured stay on the prefill-node path."""
    import torch
    import bench
    import paper_2603_13358_amd as ppd
    cells = [(2, 8, 5), (2, 6, 9), (1, 8, 3), (0, 0, 0)]          # (context class, workload type, QPS level)
    res = bench.run_route_table(torch, 0, 5, 25.0, only=cells)
    table = np.asarray(res["x_table"])
    idx = lambda c, r, q: (c * 9 + r) * 10 + q
    for c, r, q in cells[:3]:
        assert table[idx(c, r, q)] == 1 and res["delta_ttft"][idx(c, r, q)] > 0.5
    assert table.sum() <= len(cells)
    dt, dp = np.asarray(res["delta_ttft"]), np.asarray(res["delta_tpot"])
    only_tpot = ppd.ppd_route_table_build(dt, dp, 0.0, 1.0)
    assert all(only_tpot[idx(*cell)] == 0 for cell in cells if dp[idx(*cell)] > 0)
    # the online phase on top of it: a turn-3 request of the first cell's shape runs locally, its turn 1 does not
    centers = res["ratio_centers"]
    assert ppd.ppd_route_decide(table, centers, 3, 1024, 32, 9000, 8.0) == 1
    assert ppd.ppd_route_decide(table, centers, 1, 1024, 32, 9000, 8.0) == 0


def test_debugging_aids_from_the_environment():
    """PPD_LOG=1 prints one line per call; PPD_DEBUG_SLOTS=1 finds a duplicate slot within an append (flag bit 2) and
    stays silent on a clean one.  Both are read by ppd_create, so the check runs in a process of its own."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = r"""
import sys
sys.path.insert(0, %r); sys.path.insert(0, %r)
import numpy as np, torch
import paper_2603_13358_amd as ppd
import synthetic_inputs as si
from gpu_helpers import gpu_step, to_dev_u16
b = si.cfg1_tiny(0)
pool, out, stats, ctx = gpu_step(b, return_ctx=True)          # clean appends + one attention call
assert ctx.device_error_flags() == 0
dev = torch.device("cuda:0")
k, v, slots = b.new_part()
slots = slots.copy(); slots[5] = slots[9]                      # two tokens into one slot
pool_d = torch.zeros(ctx.pool_elems(), dtype=torch.int16, device=dev)
ctx.kv_append(to_dev_u16(k, torch, dev), to_dev_u16(v, torch, dev), pool_d, torch.from_numpy(slots).to(dev))
flags = ctx.device_error_flags()
assert flags == 4, flags
ctx.kv_append(to_dev_u16(k, torch, dev), to_dev_u16(v, torch, dev), pool_d, torch.from_numpy(b.new_part()[2]).to(dev))
assert ctx.device_error_flags() == 0                           # the bitmap was cleared again
print("aids ok")
""" % (root, os.path.join(root, "tests"))
    env = dict(os.environ, PPD_LOG="1", PPD_DEBUG_SLOTS="1")
    res = subprocess.run([sys.executable, "-c", code], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, env=env,
                         timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "aids ok" in res.stdout
    assert "ppd: kv_append T=" in res.stderr and "ppd: mixed_attention B=4 tiles=" in res.stderr
