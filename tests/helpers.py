"""Shared test plumbing (no arithmetic of the method)."""
import numpy as np

import oracle
from oracle.bruteforce import dense_attention

SENTINEL = 0x7FC1  # a bf16 NaN pattern: stale pool contents must never leak into a result


def oracle_pool(b, fill=SENTINEL, parts=("cached", "new")):
    """Page pool built through the oracle's own append."""
    pool = np.full(oracle.pool_elems(b.num_pages, b.Hkv, b.D, b.P), fill, dtype=np.uint16)
    for part in parts:
        k, v, slots = b.cached_part() if part == "cached" else b.new_part()
        oracle.kv_append(k, v, pool, slots, b.Hkv, b.D, b.P, b.num_pages)
    return pool


def oracle_out(b, pool=None, row_mask=None):
    if pool is None:
        pool = oracle_pool(b)
    return oracle.mixed_attention(b.q, pool, b.page_tables, b.L, b.n, b.Hq, b.Hkv, b.D, b.P, b.num_pages,
                                  b.scale, row_mask=row_mask)


def dense_out(b):
    """Brute force per sequence from the un-paged token arrays."""
    outs = []
    for i in range(b.B):
        k, v = b.seq_kv(i)
        r0, r1 = int(b.row_off[i]), int(b.row_off[i + 1])
        outs.append(dense_attention(b.q[r0:r1], k, v, int(b.L[i]), int(b.n[i]), b.scale))
    return np.concatenate(outs) if outs else np.zeros((0, b.Hq, b.D))


def bits_to_f32(a):
    return (np.asarray(a, np.uint16).astype(np.uint32) << 16).view(np.float32)


def check_close(got, ref, max_abs=2e-2, rel=1e-2):
    """The parity bar: max-abs <= 2e-2 AND per-(row, head) relative L2 <= 1e-2 (+1e-6 absolute slack)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape
    assert np.isfinite(got).all(), "non-finite output"
    d = got - ref
    worst = float(np.abs(d).max()) if d.size else 0.0
    assert worst <= max_abs, "max-abs %.3e > %.1e" % (worst, max_abs)
    num = np.sqrt((d * d).sum(-1))
    den = np.sqrt((ref * ref).sum(-1))
    bad = num > rel * den + 1e-6
    assert not bad.any(), "rel-L2 %.3e > %.1e at %s" % (float((num / np.maximum(den, 1e-30)).max()), rel,
                                                        np.argwhere(bad)[:4].tolist())
    return worst
