"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

The paper prints no numeric attention output, so the oracle is pinned by: a dense brute force that never
sees pages; the paper's premise that append-prefill over cached KV equals the tail of a full recompute
(section 4.1, and section 1's lossless-reuse statement); n=1 append-prefill == decode; page relabelling;
chunking; closed forms of softmax; GQA replication; a library softmax-attention routine; a sentinel
check of the append; and the KV-footprint arithmetic the paper prints (appendix "Bandwidth Simulation").
"""
import numpy as np
import pytest

import oracle
import synthetic_inputs as si
from helpers import SENTINEL, bits_to_f32, dense_out, oracle_out, oracle_pool


def test_bruteforce_cfg1_all_seeds():
    for seed in (0, 1, 2):
        b = si.cfg1_tiny(seed)
        got = oracle_out(b)
        ref = dense_out(b)
        assert np.abs(got - ref).max() < 1e-6


@pytest.mark.parametrize("Hq,Hkv,D", [(4, 4, 64), (8, 1, 128), (6, 3, 64), (32, 8, 128)])
def test_bruteforce_shapes(Hq, Hkv, D):
    b = si.make_batch("t", L=[0, 1, 15, 16, 17, 200], n=[1, 1, 33, 16, 2, 7], Hq=Hq, Hkv=Hkv, D=D, seed=7,
                      slack_pages=5)
    assert np.abs(oracle_out(b) - dense_out(b)).max() < 1e-6


def test_append_prefill_equals_tail_of_recompute():
    """AP(L, n) == last n rows of a full prefill (L'=0, n'=L+n) of the same tokens."""
    b = si.make_batch("ap", L=[100, 37], n=[12, 20], Hq=8, Hkv=2, D=64, seed=3)
    rng = np.random.default_rng(11)
    out_ap = oracle_out(b)
    # the recompute run needs query rows for the cached positions too; any values do, their rows are dropped
    tot = (b.L + b.n).astype(np.int32)
    qf = si.normal_bf16(rng, (int(tot.sum()), b.Hq, b.D))
    at = 0
    for i in range(b.B):
        r0, r1 = int(b.row_off[i]), int(b.row_off[i + 1])
        qf[at + int(b.L[i]):at + int(tot[i])] = b.q[r0:r1]
        at += int(tot[i])
    full = si.MixedBatch(name="full", Hq=b.Hq, Hkv=b.Hkv, D=b.D, P=b.P, num_pages=b.num_pages, scale=b.scale,
                         L=np.zeros(b.B, np.int32), n=tot, page_tables=b.page_tables, q=qf, k=b.k, v=b.v)
    out_full = oracle_out(full)
    at = 0
    for i in range(b.B):
        r0, r1 = int(b.row_off[i]), int(b.row_off[i + 1])
        tail = out_full[at + int(b.L[i]):at + int(tot[i])]
        assert np.abs(tail - out_ap[r0:r1]).max() < 1e-6
        at += int(tot[i])


def test_n1_append_prefill_is_decode_and_chunking():
    """Row j of AP(L, n) == the single row of a decode step at cached length L+j (same keys, same query);
    hence AP(L, n) == AP(L, n1) followed by AP(L+n1, n2)."""
    b = si.make_batch("c", L=[50], n=[9], Hq=4, Hkv=2, D=64, seed=5)
    pool = oracle_pool(b)
    whole = oracle_out(b, pool)
    for j in range(9):
        one = si.MixedBatch(name="d", Hq=4, Hkv=2, D=64, P=b.P, num_pages=b.num_pages, scale=b.scale,
                            L=[50 + j], n=[1], page_tables=b.page_tables, q=b.q[j:j + 1])
        got = oracle.mixed_attention(one.q, pool, one.page_tables, one.L, one.n, 4, 2, 64, b.P, b.num_pages, b.scale)
        assert np.abs(got[0] - whole[j]).max() < 1e-6
    for n1 in (1, 4, 8):
        a = oracle.mixed_attention(b.q[:n1], pool, b.page_tables, [50], [n1], 4, 2, 64, b.P, b.num_pages, b.scale)
        c = oracle.mixed_attention(b.q[n1:], pool, b.page_tables, [50 + n1], [9 - n1], 4, 2, 64, b.P, b.num_pages,
                                   b.scale)
        assert np.abs(np.concatenate([a, c]) - whole).max() < 1e-6


def test_page_relabelling_is_bitwise_invariant():
    b = si.cfg1_tiny(1)
    ref = oracle_out(b)
    rng = np.random.default_rng(99)
    relabel = rng.permutation(b.num_pages).astype(np.int32)
    pt = np.where(b.page_tables >= 0, relabel[np.maximum(b.page_tables, 0)], -1).astype(np.int32)
    b2 = si.MixedBatch(name="perm", Hq=b.Hq, Hkv=b.Hkv, D=b.D, P=b.P, num_pages=b.num_pages, scale=b.scale,
                       L=b.L, n=b.n, page_tables=pt, q=b.q, k=b.k, v=b.v)
    got = oracle_out(b2)
    assert np.array_equal(got, ref)


def test_closed_forms():
    b = si.make_batch("cf", L=[0, 0, 40, 77], n=[1, 5, 1, 3], Hq=4, Hkv=2, D=64, seed=8)
    # L=0, n=1: one visible key, out == V_0 exactly (bf16 values are exact in fp32)
    out = oracle_out(b)
    k0, v0 = b.seq_kv(0)
    for h in range(4):
        assert np.array_equal(out[0, h], bits_to_f32(v0[0, h // 2]))
    # q == 0 (and, separately, scale == 0): out == mean of the visible V rows
    for variant in ("q0", "scale0"):
        bz = si.make_batch("cf", L=[0, 0, 40, 77], n=[1, 5, 1, 3], Hq=4, Hkv=2, D=64, seed=8)
        if variant == "q0":
            bz.q[:] = 0
        else:
            bz.scale = 0.0
        oz = oracle_out(bz)
        for i in range(bz.B):
            _, v = bz.seq_kv(i)
            vf = bits_to_f32(v).astype(np.float64)
            for j in range(int(bz.n[i])):
                vis = int(bz.L[i]) + j + 1
                for h in range(4):
                    assert np.abs(oz[int(bz.row_off[i]) + j, h] - vf[:vis, h // 2].mean(0)).max() < 1e-6
    # all V rows equal -> out == that row, whatever the scores
    bv = si.make_batch("cf", L=[33], n=[4], Hq=4, Hkv=2, D=64, seed=9)
    bv.v[:] = bv.v[0]
    ov = oracle_out(bv)
    for h in range(4):
        assert np.abs(ov[:, h] - bits_to_f32(bv.v[0, h // 2])).max() < 1e-6
    # one key dominating by a wide margin -> out ~= its V row; it must be VISIBLE to count:
    # put it at position L+1 (the second new token): row 0 must not see it, rows 1.. must
    bd = si.make_batch("cf", L=[20], n=[3], Hq=2, Hkv=2, D=64, seed=10)
    bd.k[:] = 0
    bd.k[21, :, 0] = si.f32_to_bf16_bits(np.float32(64.0))
    bd.q[:, :, 0] = si.f32_to_bf16_bits(np.float32(8.0))   # score = 8*64/8 = 64 above the rest
    od = oracle_out(bd)
    vf = bits_to_f32(bd.v).astype(np.float64)
    for h in range(2):
        assert np.abs(od[0, h] - vf[:21, h].mean(0)).max() < 1e-6
        assert np.abs(od[1, h] - vf[21, h]).max() < 1e-6
        assert np.abs(od[2, h] - vf[21, h]).max() < 1e-6


def test_gqa_equals_replicated_mha():
    b = si.make_batch("g", L=[60, 5], n=[1, 10], Hq=8, Hkv=2, D=64, seed=12)
    ref = oracle_out(b)
    G = b.Hq // b.Hkv
    rep = si.MixedBatch(name="mha", Hq=8, Hkv=8, D=64, P=b.P, num_pages=b.num_pages, scale=b.scale, L=b.L, n=b.n,
                        page_tables=b.page_tables, q=b.q, k=np.repeat(b.k, G, axis=1), v=np.repeat(b.v, G, axis=1))
    assert np.abs(oracle_out(rep) - ref).max() < 1e-6


def test_library_sdpa_contiguous_single_sequence():
    torch = pytest.importorskip("torch")
    L, n, Hq, Hkv, D = 70, 9, 4, 2, 64
    b = si.make_batch("sdpa", L=[L], n=[n], Hq=Hq, Hkv=Hkv, D=D, seed=13,
                      page_tables=np.arange(5, dtype=np.int32)[None, :], num_pages=5)
    got = oracle_out(b)
    q = torch.from_numpy(bits_to_f32(b.q)).double().permute(1, 0, 2)              # [Hq, n, D]
    k = torch.from_numpy(bits_to_f32(b.k)).double().permute(1, 0, 2).repeat_interleave(2, 0)
    v = torch.from_numpy(bits_to_f32(b.v)).double().permute(1, 0, 2).repeat_interleave(2, 0)
    mask = torch.arange(L + n)[None, :] <= (L + torch.arange(n))[:, None]
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=mask, scale=float(np.float32(b.scale)))
    assert np.abs(ref.permute(1, 0, 2).numpy() - got).max() < 1e-6


def test_append_touches_exactly_its_slots():
    b = si.cfg1_tiny(2)
    pool = oracle_pool(b, parts=("cached",))
    before = pool.copy()
    k, v, slots = b.new_part()
    # a skipped token (negative slot) must leave the pool alone
    slots = slots.copy()
    skipped = 5
    slots[skipped] = -1
    oracle.kv_append(k, v, pool, slots, b.Hkv, b.D, b.P, b.num_pages)
    changed = np.flatnonzero(pool != before)
    assert changed.size <= (len(slots) - 1) * 2 * b.Hkv * b.D
    # every written element holds the right value: read back token by token through an independent gather
    S = 2 * b.Hkv * b.P * b.D
    for t, s in enumerate(slots):
        if s < 0:
            continue
        page, off = divmod(int(s), b.P)
        blk = pool[page * S:(page + 1) * S]
        kk = blk[:S // 2].reshape(b.Hkv, b.D // 8, b.P, 8)[:, :, off, :].reshape(b.Hkv, b.D)
        vv = blk[S // 2:].reshape(b.Hkv, b.P // 8, b.D, 8)[:, off // 8, :, off % 8]
        assert np.array_equal(kk, k[t]) and np.array_equal(vv, v[t])
    # untouched elements: still sentinel or the cached part
    total_written = np.count_nonzero(oracle_pool(b, parts=("cached", "new")) != SENTINEL)
    assert total_written <= int((b.L + b.n).sum()) * 2 * b.Hkv * b.D
    with pytest.raises(ValueError):
        oracle.kv_append(k[:1], v[:1], pool, np.asarray([b.num_pages * b.P]), b.Hkv, b.D, b.P, b.num_pages)


def test_stale_pool_contents_never_leak():
    """Unwritten slots hold a NaN pattern; a finite oracle output shows that only visible keys were read."""
    b = si.cfg1_tiny(0)
    assert np.isfinite(oracle_out(b)).all()


def test_kv_footprint_arithmetic():
    """The paper's figures: 128 KiB per token over 32 layers -> 4 KiB per token per layer for 8 KV heads of
    128 in bf16; 5,115 tokens -> ~670 MB."""
    b = si.cfg2_decode(0, B=2, Lmin=16, Lmax=32, with_data=False)
    assert b.kv_bytes_per_token() == 4096
    assert b.kv_bytes_per_token() * 32 == 128 * 1024
    assert 5115 * 32 * b.kv_bytes_per_token() == 670_433_280
    assert b.kv_read_bytes() == int((b.L + b.n).sum()) * 4096
    # cost of append-prefill is O(n(L+n)): exactly 4*Hq*D flops per visible (row, key) pair
    one = si.make_batch("f", L=[100], n=[10], Hq=2, Hkv=1, D=64, seed=0, with_data=False)
    assert one.attention_flops() == 4 * 2 * 64 * (10 * 100 + 55)


def _golden_transfer():
    import os
    vals = {}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "kv_transfer_numbers.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        parts = line.split()
        vals[parts[0]] = float(parts[1])
    return vals


def test_transfer_delay_model_against_the_papers_numbers():
    """The injected-delay equation of the appendix "Bandwidth Simulation" and the figures printed next to it."""
    g = _golden_transfer()
    B = g["p90_context_tokens"] * g["s_kv_bytes_per_token"]
    assert B == g["footprint_bytes"]
    t_nv = g["time_nvlink_ms"] * 1e-3
    # with t_fast = 0 the delay is the plain transfer time B / beta: the paper's ~27 ms at 25 GB/s
    assert abs(oracle.transfer_delay(g["p90_context_tokens"], g["s_kv_bytes_per_token"], g["ib_hdr_bytes_per_s"], 0.0) * 1e3
               - g["time_ib_hdr_ms"]) < 0.5
    # ~67 ms over 100GbE corresponds to 10 GB/s
    assert abs(oracle.transfer_delay(g["p90_context_tokens"], g["s_kv_bytes_per_token"], 10e9, 0.0) * 1e3
               - g["time_100gbe_ms"]) < 0.5
    # the injected delay subtracts the NVLink time already spent and never goes negative
    d = oracle.transfer_delay(g["p90_context_tokens"], g["s_kv_bytes_per_token"], g["ib_hdr_bytes_per_s"], t_nv)
    assert abs(d - (B / 25e9 - t_nv)) < 1e-12 and 0.022 < d < 0.023
    assert oracle.transfer_delay(g["p90_context_tokens"], g["s_kv_bytes_per_token"], 1e12, t_nv) == 0.0
    # delay is linear in tokens above the break-even point
    d2 = oracle.transfer_delay(2 * g["p90_context_tokens"], g["s_kv_bytes_per_token"], g["ib_hdr_bytes_per_s"], t_nv)
    assert abs((d2 + t_nv) - 2 * (d + t_nv)) < 1e-12


def test_kv_land_is_one_append_per_layer():
    b = si.cfg1_tiny(1)
    layers, pe = 3, oracle.pool_elems(b.num_pages, b.Hkv, b.D, b.P)
    stride = pe + 640                       # padding between the layers' pools must stay untouched
    rng = np.random.default_rng(5)
    k0, v0, slots = b.cached_part()
    T = len(slots)
    k = si.normal_bf16(rng, (layers, T, b.Hkv, b.D))
    v = si.normal_bf16(rng, (layers, T, b.Hkv, b.D))
    pools = np.full(stride * (layers - 1) + pe, SENTINEL, np.uint16)
    oracle.kv_land(k, v, pools, stride, layers, slots, b.Hkv, b.D, b.P, b.num_pages)
    for l in range(layers):
        ref = np.full(pe, SENTINEL, np.uint16)
        oracle.kv_append(k[l], v[l], ref, slots, b.Hkv, b.D, b.P, b.num_pages)
        assert np.array_equal(pools[l * stride:l * stride + pe], ref)
        if l + 1 < layers:
            assert (pools[l * stride + pe:(l + 1) * stride] == SENTINEL).all()
