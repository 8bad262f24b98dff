"""Multi-turn trace on the GPU against the oracle, step by step on one persistent page pool: turn-1 KV
landing (append only), decode steps, turn-2+ append-prefill over everything cached so far."""
import numpy as np
import pytest

import oracle
import synthetic_inputs as si
from helpers import SENTINEL, bits_to_f32, check_close

pytestmark = pytest.mark.gpu


def _trace_against_oracle(n_conv, turns, prompt_mean, response_mean, sigma, start_spread, len_clip, seed,
                          sample_ap_rows=False):
    """Runs a whole trace on one persistent pool, the oracle beside it step by step (its own pool, its own appends);
    every decode row is compared, append-prefill rows all or -- sample_ap_rows -- first, last, block edges and a few."""
    import torch
    import paper_2603_13358_amd as ppd
    from gpu_helpers import from_dev_u16, to_dev_u16

    Hq, Hkv, D, P = 16, 2, 128, 16
    steps, max_tokens = si.cfg5_trace(seed=seed, n_conv=n_conv, turns=turns, prompt_mean=prompt_mean,
                                      response_mean=response_mean, sigma=sigma, start_spread=start_spread,
                                      len_clip=len_clip)
    rng = np.random.default_rng(77)
    need = (max_tokens + P - 1) // P
    num_pages = int(need.sum()) + 5
    perm = rng.permutation(num_pages).astype(np.int32)
    pt = np.full((n_conv, int(need.max())), -1, np.int32)
    at = 0
    for c in range(n_conv):
        pt[c, :need[c]] = perm[at:at + need[c]]
        at += int(need[c])
    dev = torch.device("cuda:0")
    ctx = ppd.Context(Hq, Hkv, D, num_pages)
    fill = int(np.array([SENTINEL], np.uint16).view(np.int16)[0])
    pool_d = torch.full((ctx.pool_elems(),), fill, dtype=torch.int16, device=dev)
    pool_h = np.full(ctx.pool_elems(), SENTINEL, np.uint16)
    scale = 1.0 / np.sqrt(D)
    n_att, longest = 0, 0
    for st in steps:
        T = int(st.n.sum())
        k = si.normal_bf16(rng, (T, Hkv, D))
        v = si.normal_bf16(rng, (T, Hkv, D))
        slots = np.concatenate([pt[c, (np.arange(L, L + n)) // P].astype(np.int64) * P + np.arange(L, L + n) % P
                                for c, L, n in zip(st.conv, st.L, st.n)])
        oracle.kv_append(k, v, pool_h, slots, Hkv, D, P, num_pages)
        ctx.kv_append(to_dev_u16(k, torch, dev), to_dev_u16(v, torch, dev), pool_d, torch.from_numpy(slots).to(dev))
        if not st.attend:
            continue
        q = si.normal_bf16(rng, (T, Hq, D))
        sub_pt = np.ascontiguousarray(pt[st.conv])
        out = torch.zeros((T, Hq, D), dtype=torch.int16, device=dev)
        ctx.mixed_attention(to_dev_u16(q, torch, dev), pool_d, torch.from_numpy(sub_pt).to(dev), st.L, st.n, scale, out)
        mask = None
        if sample_ap_rows:
            mask = np.zeros(T, np.uint8)
            o = 0
            for n_i in st.n:
                mask[o + np.asarray(_sample_rows(int(n_i), 256 // (Hq // Hkv), rng))] = 1
                o += int(n_i)
        ref = oracle.mixed_attention(q, pool_h, sub_pt, st.L, st.n, Hq, Hkv, D, P, num_pages, scale, row_mask=mask)
        got = bits_to_f32(from_dev_u16(out).reshape(T, Hq, D))
        sel = np.ones(T, bool) if mask is None else mask.astype(bool)
        check_close(got[sel], ref[sel])
        n_att += 1
        longest = max(longest, int((st.L + st.n).max()))
    assert ctx.device_error_flags() == 0
    assert np.array_equal(from_dev_u16(pool_d), pool_h), "pools diverged over the trace"
    ctx.close()
    return n_att, longest


def test_short_trace_matches_oracle_every_step():
    n_att, _ = _trace_against_oracle(n_conv=6, turns=3, prompt_mean=40.0, response_mean=6.0, sigma=0.8, start_spread=4,
                                     len_clip=(1, 200), seed=3)
    assert n_att > 10


def test_sixteen_turn_trace_matches_oracle():
    """Turn scaling (the paper's scaling-validation appendix runs conversations of 2 to 16 turns): 16 turns of long
    prompts and short answers, so that the accumulated context passes 16K tokens while the turn's append-prefill
    still sees all of it from the pages; every decode row and sampled append-prefill rows of every step."""
    n_att, longest = _trace_against_oracle(n_conv=4, turns=16, prompt_mean=1100.0, response_mean=5.0, sigma=0.5,
                                           start_spread=3, len_clip=(1, 2500), seed=5, sample_ap_rows=True)
    print("attention steps", n_att, "longest context", longest, flush=True)
    assert longest > 16384 and n_att > 60


def _sample_rows(n_i, rows_per_block, rng, extra=3):
    """Rows of an append-prefill worth checking: first, last, either side of every row-block edge, a few at random."""
    if n_i == 1:
        return [0]
    pick = {0, n_i - 1}
    for e in range(rows_per_block, n_i, rows_per_block):
        pick.update((e - 1, e))
    pick.update(int(x) for x in rng.integers(0, n_i, size=extra))
    return sorted(pick)


def test_cfg5_trace_at_full_shape_sampled_steps_match_oracle():
    """The multi-turn trace at its stated shape: 64 q / 8 kv heads, D = 128, 256 conversations x 5 turns, pages drawn
    without replacement over a pool of (up to) 200 GB, so that element offsets reach ~1e11.  Every engine step runs on
    the GPU; 16 tracked conversations are mirrored on the host, their KV appended by the ORACLE into a compact pool of
    its own from the same new-token K/V (the oracle never reads what the library wrote).  On 32 seeded steps --
    decode-only steps, steps in which a tracked conversation runs its append-prefill, and each kind's first step
    after a tracked conversation's turn-1 landing -- the tracked conversations' pages on the device are compared
    bit for bit with the mirror, and their attention rows with the oracle's."""
    import torch
    import paper_2603_13358_amd as ppd

    Hq, Hkv, D, P = 64, 8, 128, 16
    seed = 0
    steps, max_tokens = si.cfg5_trace(seed)
    page_elems = 2 * Hkv * P * D
    page_bytes = page_elems * 2
    free_b, _ = torch.cuda.mem_get_info()
    num_pages = int(min(200e9, free_b * 0.9) // page_bytes)
    rng = np.random.default_rng(9100 + seed)
    need = (max_tokens + P - 1) // P
    n_conv = len(need)
    pages = rng.choice(num_pages, size=int(need.sum()), replace=False).astype(np.int32)
    pt = np.full((n_conv, int(need.max())), -1, np.int32)
    at = 0
    for c in range(n_conv):
        pt[c, :need[c]] = pages[at:at + need[c]]
        at += int(need[c])
    tracked = sorted(int(c) for c in rng.choice(n_conv, size=16, replace=False))
    # one tracked conversation gets the top pages of the pool, so the largest offsets are certainly compared
    top = tracked[0]
    used = set(pages.tolist())
    hi = [p for p in range(num_pages - 1, num_pages - 1 - 4 * int(need[top]), -1) if p not in used][:int(need[top])]
    pt[top, :need[top]] = np.asarray(hi, np.int32)
    assert int(pt[top, :need[top]].max()) * page_elems > 2 ** 32 or num_pages * page_elems <= 2 ** 32
    print("pool pages", num_pages, "= %.1f GB; largest tracked element offset %.3e" %
          (num_pages * page_bytes / 1e9, float(pt[tracked].max()) * page_elems), flush=True)
    # compact mirror: tracked conversation c owns pages base[c] .. base[c] + need[c] - 1
    base, acc = {}, 0
    for c in tracked:
        base[c] = acc
        acc += int(need[c])
    mirror_pages = acc
    mirror = np.full(oracle.pool_elems(mirror_pages, Hkv, D, P), SENTINEL, np.uint16)

    dev = torch.device("cuda:0")
    ctx = ppd.Context(Hq, Hkv, D, num_pages)
    pool = torch.empty((num_pages * page_elems,), dtype=torch.int16, device=dev)          # contents: whatever
    fill = int(np.array([SENTINEL], np.uint16).view(np.int16)[0])
    all_used = np.unique(pt[pt >= 0]).astype(np.int64)
    pool.view(num_pages, page_elems)[torch.from_numpy(all_used).to(dev)] = fill
    pt_d = torch.from_numpy(pt).to(dev)
    scale = 1.0 / np.sqrt(D)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)

    # which steps are compared
    tracked_set = set(tracked)
    landed, first_after = set(), []
    cand_ap, cand_dec = [], []
    for idx, st in enumerate(steps):
        here = [int(c) for c in st.conv if int(c) in tracked_set]
        if not st.attend:
            landed.update(here)
            continue
        if not here:
            continue
        if any(c in landed for c in here):
            first_after.append(idx)
            landed.difference_update(here)
        if any(int(n) > 1 for c, n in zip(st.conv, st.n) if int(c) in tracked_set):
            cand_ap.append(idx)
        elif int(st.n.max()) == 1:
            cand_dec.append(idx)
    pick = rng.choice(cand_ap, size=min(12, len(cand_ap)), replace=False).tolist()
    pick += rng.choice(first_after, size=min(10, len(first_after)), replace=False).tolist()
    rest = [i for i in cand_dec if i not in pick]
    pick += rng.choice(rest, size=32 - len(set(pick)), replace=False).tolist()
    pick = set(int(i) for i in pick)
    assert len(pick) >= 30
    rows_per_block = 256 // (Hq // Hkv)

    worst, checked_rows, n_ap_checked = 0.0, 0, 0
    for idx, st in enumerate(steps):
        T = int(st.n.sum())
        k = torch.empty((T, Hkv, D), dtype=torch.bfloat16, device=dev).normal_(generator=gen)
        v = torch.empty((T, Hkv, D), dtype=torch.bfloat16, device=dev).normal_(generator=gen)
        slots = np.concatenate([pt[c, (np.arange(L, L + n)) // P].astype(np.int64) * P + np.arange(L, L + n) % P
                                for c, L, n in zip(st.conv, st.L, st.n)])
        ctx.kv_append(k, v, pool, torch.from_numpy(slots).to(dev))
        # mirror the tracked conversations' new tokens through the oracle's append
        row_off = np.concatenate([[0], np.cumsum(st.n)])
        here = [(j, int(c)) for j, c in enumerate(st.conv) if int(c) in tracked_set]
        if here:
            rows = np.concatenate([np.arange(row_off[j], row_off[j + 1]) for j, _ in here])
            ridx = torch.from_numpy(rows).to(dev)
            kh = k.view(torch.int16)[ridx].cpu().numpy().view(np.uint16)
            vh = v.view(torch.int16)[ridx].cpu().numpy().view(np.uint16)
            mslots = np.concatenate([(base[c] + np.arange(int(st.L[j]), int(st.L[j] + st.n[j])) // P) * P +
                                     np.arange(int(st.L[j]), int(st.L[j] + st.n[j])) % P for j, c in here])
            oracle.kv_append(kh, vh, mirror, mslots.astype(np.int64), Hkv, D, P, mirror_pages)
        if not st.attend:
            continue
        q = torch.empty((T, Hq, D), dtype=torch.bfloat16, device=dev).normal_(generator=gen)
        out = torch.empty((T, Hq, D), dtype=torch.bfloat16, device=dev)
        sub_pt = pt_d[torch.from_numpy(st.conv.astype(np.int64)).to(dev)].contiguous()
        ctx.mixed_attention(q, pool, sub_pt, st.L, st.n, scale, out)
        if idx not in pick:
            continue
        print("step", idx, "sequences", len(st.n), "append-prefills", int((st.n > 1).sum()), "tracked", len(here),
              flush=True)
        # (1) append parity at the pool's real addresses: the tracked conversations' pages, whole pages, bit for bit
        for j, c in here:
            used_pages = int((st.L[j] + st.n[j] + P - 1) // P)
            ids = torch.from_numpy(pt[c, :used_pages].astype(np.int64)).to(dev)
            got = pool.view(num_pages, page_elems).index_select(0, ids).cpu().numpy().view(np.uint16).reshape(-1)
            want = mirror[base[c] * page_elems:(base[c] + used_pages) * page_elems]
            assert np.array_equal(got, want), "pool pages of conversation %d differ from the oracle's at step %d" % (c, idx)
        # (2) attention of the tracked conversations against the oracle on its own mirror
        sub_L = np.asarray([st.L[j] for j, _ in here], np.int32)
        sub_n = np.asarray([st.n[j] for j, _ in here], np.int32)
        opt = np.full((len(here), pt.shape[1]), -1, np.int32)
        for r, (j, c) in enumerate(here):
            opt[r, :need[c]] = base[c] + np.arange(need[c])
        qh = q.view(torch.int16)[ridx].cpu().numpy().view(np.uint16)
        mask = np.zeros(int(sub_n.sum()), np.uint8)
        o = 0
        for r in range(len(here)):
            mask[o + np.asarray(_sample_rows(int(sub_n[r]), rows_per_block, rng))] = 1
            n_ap_checked += int(sub_n[r] > 1)
            o += int(sub_n[r])
        ref = oracle.mixed_attention(qh, mirror, opt, sub_L, sub_n, Hq, Hkv, D, P, mirror_pages, scale, row_mask=mask)
        got = out.float()[ridx].cpu().numpy()
        sel = mask.astype(bool)
        worst = max(worst, check_close(got[sel], ref[sel]))
        checked_rows += int(sel.sum())
        assert bool(torch.isfinite(out.float()).all())
    torch.cuda.synchronize()
    assert ctx.device_error_flags() == 0
    print("compared %d steps, %d rows (%d append-prefills), max-abs %.3e" % (len(pick), checked_rows, n_ap_checked, worst),
          flush=True)
    assert n_ap_checked >= 8 and checked_rows >= 200
    ctx.close()
