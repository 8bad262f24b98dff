"""Shared test plumbing (no arithmetic of the method)."""
import numpy as np

import oracle
import synthetic_inputs as si
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


def random_mixed_batch(seed):
    """A random batch and planner options, all drawn from the seed: sequence count, head shape, the mix of decode /
    append-prefill / full-prefill rows, lengths around page, tile and row-block boundaries, split sizes."""
    rng = np.random.default_rng(7000 + seed)
    Hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.integers(1, 9))
    D = int(rng.choice([64, 128]))
    B = int(rng.integers(1, 25))
    L, n = [], []
    budget = 4e6 / (G * Hkv / 8.0)                 # visible (row, key) pairs: keeps the oracle to a few seconds
    for _ in range(B):
        kind = rng.integers(0, 4)
        if kind == 0:                              # decode
            Li, ni = int(rng.integers(0, 5000)), 1
        elif kind == 1:                            # a few new tokens (still a narrow tile for small G)
            Li, ni = int(rng.integers(0, 3000)), int(rng.integers(2, 8))
        elif kind == 2:                            # append-prefill, lengths near multiples of 64
            Li = int(rng.integers(1, 40)) * 64 + int(rng.integers(-2, 3))
            ni = int(rng.integers(1, 6)) * 64 // max(1, G // 2) + int(rng.integers(-2, 3))
        else:                                      # full prefill
            Li, ni = 0, int(rng.integers(1, 400))
        ni = max(1, ni)
        cost = ni * (Li + (ni + 1) / 2)
        if cost > budget:
            continue
        budget -= cost
        L.append(max(0, Li))
        n.append(ni)
    if not L:
        L, n = [5], [1]
    opts = {}
    if rng.integers(0, 2):
        opts = {"narrow_chunk": int(rng.choice([64, 256, 1024])), "mfma_chunk": int(rng.choice([64, 192, 512, 2048]))}
    return si.make_batch("random%d" % seed, L=L, n=n, Hq=G * Hkv, Hkv=Hkv, D=D, seed=7100 + seed,
                         slack_pages=int(rng.integers(0, 9))), opts
