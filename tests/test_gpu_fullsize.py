"""Full-size workloads in the launch configuration bench.py times, checked on sampled outputs the oracle can
compute one by one: KV append bit-exact on the sampled sequences' pages, attention within the parity bar on
sampled rows (all heads), plus properties that hold at any size (finite output, determinism)."""
import numpy as np
import pytest

import oracle
import synthetic_inputs as si
from helpers import check_close

pytestmark = pytest.mark.gpu


def _edge_rows(n_i, rows_per_block, cap=None):
    """First and last row and the rows either side of every row-block edge (at most `cap` edges, evenly spread)."""
    edges = list(range(rows_per_block, n_i, rows_per_block))
    if cap is not None and len(edges) > cap:
        edges = [edges[i] for i in np.linspace(0, len(edges) - 1, cap).astype(int)]
    pick = {0, n_i - 1}
    for e in edges:
        pick.update((e - 1, e))
    return sorted(pick)


def _run_and_check(name, seq_ids_fn, rows_per_seq=4, edge_rows=False, edge_cap=None, fp8=False):
    import torch
    import bench
    b = bench.make_shapes(name, 0) if isinstance(name, str) else name
    print("workload", b.name, "B", b.B, "T", b.T, flush=True)
    r = bench.Runner(b, torch, 0, fp8=fp8)   # fp8: FP8 E4M3 pages, the scale of the benchmark for K and for V
    sc = si.FP8_BENCH_SCALE
    w = r.w
    seqs = seq_ids_fn(b)
    # pages of the sampled sequences before the append
    sub0, pool_before, rows = si.compact_subbatch(b, seqs, w["pool"], w["q"], torch)
    r.step()
    torch.cuda.synchronize()
    assert r.ctx.device_error_flags() == 0
    out1 = w["out"].clone()
    sub, pool_after, rows = si.compact_subbatch(b, seqs, w["pool"], w["q"], torch)
    # --- append: oracle-append the sampled sequences' new tokens into the 'before' pages
    idx = torch.from_numpy(rows).to(w["k_new"].device)
    k_new = w["k_new"].view(torch.int16)[idx].cpu().numpy().view(np.uint16)
    v_new = w["v_new"].view(torch.int16)[idx].cpu().numpy().view(np.uint16)
    slots = np.concatenate([sub.slots(i, int(sub.L[i]), int(sub.L[i] + sub.n[i])) for i in range(sub.B)])
    ref_pool = pool_before.copy()
    if fp8:
        oracle.kv_append_fp8(k_new, v_new, ref_pool, slots, sub.Hkv, sub.D, sub.P, sub.num_pages, sc, sc)
    else:
        oracle.kv_append(k_new, v_new, ref_pool, slots, sub.Hkv, sub.D, sub.P, sub.num_pages)
    assert np.array_equal(ref_pool, pool_after), "KV append is not bit-exact at full size"
    # --- attention on sampled rows
    mask = np.zeros(sub.T, np.uint8)
    for i in range(sub.B):
        n_i = int(sub.n[i])
        pick = sorted(set([0, n_i - 1] + list(np.linspace(0, n_i - 1, rows_per_seq).astype(int))))
        if edge_rows:
            pick = sorted(set(pick) | set(_edge_rows(n_i, 256 // (sub.Hq // sub.Hkv), edge_cap)))
        mask[int(sub.row_off[i]) + np.asarray(pick)] = 1
    if fp8:
        ref = oracle.mixed_attention_fp8(sub.q, pool_after, sc, sc, sub.page_tables, sub.L, sub.n, sub.Hq, sub.Hkv, sub.D,
                                         sub.P, sub.num_pages, sub.scale, row_mask=mask)
    else:
        ref = oracle.mixed_attention(sub.q, pool_after, sub.page_tables, sub.L, sub.n, sub.Hq, sub.Hkv, sub.D, sub.P,
                                     sub.num_pages, sub.scale, row_mask=mask)
    got = out1.float().cpu().numpy()[rows]
    sel = mask.astype(bool)
    worst = check_close(got[sel], ref[sel])
    print("  sampled %d rows of %d sequences: max-abs %.3e" % (int(sel.sum()), len(seqs), worst), flush=True)
    # --- any-size properties
    assert bool(torch.isfinite(out1.float()).all())
    r.step()
    torch.cuda.synchronize()
    assert torch.equal(w["out"], out1), "not run-to-run deterministic"
    r.close()


def _shortest_longest(b, k=1):
    order = np.argsort(b.L.astype(np.int64) + b.n)
    return [int(order[0]), int(order[len(order) // 2]), int(order[-1])][:max(1, k)] if k < 3 else \
        [int(order[0]), int(order[len(order) // 2]), int(order[-1])]


def test_cfg2_decode_full_size():
    """Every one of the 64 decode sequences, all heads."""
    _run_and_check("cfg2_decode", lambda b: list(range(b.B)))


def test_cfg3_append_prefill_full_size():
    """Every one of the 16 append-prefills: first, last, block-edge rows and a few in between."""
    _run_and_check("cfg3_ap", lambda b: list(range(b.B)), rows_per_seq=5, edge_rows=True)


def test_cfg4_mixed_full_size():
    """Every sequence of the batch: all 128 decode rows; of every append-prefill the first and last row, the rows
    either side of each 64-row block edge and a few in between; KV append bit-exact on every page of the batch."""
    _run_and_check("cfg4_mixed_ap", lambda b: list(range(b.B)), rows_per_seq=4, edge_rows=True)


def test_cfg2_decode_full_size_fp8_pages():
    """The decode batch on FP8 E4M3 pages (extension beyond the paper): every sequence, codes of the append bit for bit."""
    _run_and_check("cfg2_decode", lambda b: list(range(b.B)), fp8=True)


def test_cfg4_mixed_full_size_fp8_pages():
    """The mixed batch on FP8 pages: every 4th decode sequence and every append-prefill with its block-edge rows."""
    def pick(b):
        return [i for i in range(b.B) if b.n[i] > 1] + [i for i in range(b.B) if b.n[i] == 1][::4]
    _run_and_check("cfg4_mixed_ap", pick, rows_per_seq=4, edge_rows=True, edge_cap=8, fp8=True)


def test_cfg4_full_prefill_variant_full_size():
    def pick(b):
        full = sorted([i for i in range(b.B) if b.n[i] > 1], key=lambda i: int(b.n[i]))
        dec = sorted([i for i in range(b.B) if b.n[i] == 1], key=lambda i: int(b.L[i]))
        return dec[::8] + [full[0], full[-1]]            # every 8th decode, the shortest and longest full prefill
    _run_and_check("cfg4_mixed_full", pick, rows_per_seq=5, edge_rows=True, edge_cap=12)


def test_mixed_batch_with_group_of_five_heads():
    """40 query heads over 8 KV heads (G = 5, the head shape of the second model the paper serves, section 5.1):
    64 decodes at 1K-8K context and 3 append-prefills in one step."""
    rng = np.random.default_rng(77)
    L = np.concatenate([rng.integers(1024, 8193, size=64), rng.integers(4096, 16385, size=3)])
    n = np.concatenate([np.ones(64, np.int64), rng.integers(200, 700, size=3)])
    b = si.make_batch("mixed_g5", L=L, n=n, Hq=40, Hkv=8, D=128, seed=7, slack_pages=64, with_data=False)
    _run_and_check(b, lambda b: [0, 63, 64, 66], rows_per_seq=4)


def test_long_context_single_sequences():
    """Largest shapes of the context sweep the paper reports (64K-token contexts, appendix on context-length
    sensitivity) and beyond: one 131072-token decode, one append-prefill of 300 tokens over 100000 cached
    tokens, one 70000-token decode whose last page is partial."""
    import torch
    import paper_2603_13358_amd as ppd
    b = si.make_batch("long", L=[131071, 100000, 70003], n=[1, 300, 1], Hq=32, Hkv=8, D=128, seed=31,
                      slack_pages=9, with_data=False)
    dev = torch.device("cuda:0")
    w = si.device_workload(b, torch, dev, seed=4)
    ctx = ppd.Context(b.Hq, b.Hkv, b.D, b.num_pages)
    ctx.kv_append(w["k_new"], w["v_new"], w["pool"], w["slots"])
    ctx.mixed_attention(w["q"], w["pool"], w["page_tables"], b.L, b.n, b.scale, w["out"])
    torch.cuda.synchronize()
    assert ctx.device_error_flags() == 0
    st = ctx.plan_stats()
    print("  tiles", st.n_items, "narrow", st.n_narrow, "mfma", st.n_mfma, "groups", st.n_groups, flush=True)
    sub, pool, rows = si.compact_subbatch(b, [0, 1, 2], w["pool"], w["q"], torch)
    mask = np.zeros(sub.T, np.uint8)
    mask[[0, 1, 150, 300, 301]] = 1            # the decode rows, first / middle / last append-prefill rows
    ref = oracle.mixed_attention(sub.q, pool, sub.page_tables, sub.L, sub.n, sub.Hq, sub.Hkv, sub.D, sub.P,
                                 sub.num_pages, sub.scale, row_mask=mask)
    got = w["out"].float().cpu().numpy()[rows]
    sel = mask.astype(bool)
    worst = check_close(got[sel], ref[sel])
    print("  max-abs %.3e" % worst, flush=True)
    assert bool(torch.isfinite(w["out"].float()).all())
    ctx.close()
