"""Host-side tests that need no GPU: the C ABI exports what include/ppd.h declares, and the planner's
work list covers every visible (row, key) pair exactly once with non-overlapping partials."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2603_13358_amd as ppd
import synthetic_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ppd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ppd_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 10
    lib = ctypes.CDLL(ppd.lib_path())
    for name in names:
        assert hasattr(lib, name), "libppd.so does not export " + name
    # and the binding wraps every one of them under the same name
    for name in names:
        assert hasattr(ppd, name), "binding lacks " + name


def test_create_fails_loudly_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(ppd.PPDError) as e:
        ppd.ppd_create(32, 8, 128, 16, 64)
    assert e.value.status == -6 and "no CPU path" in str(e.value)


def replay(items, L, n, Hkv, G, D):
    """Checks the tile list against the definition: row j of sequence i sees keys 0 .. L_i + j."""
    B = len(L)
    cover = {}
    for it in items:
        assert 0 <= it.seq < B and 0 <= it.kvh < Hkv
        assert it.L == L[it.seq] and it.kv_total == L[it.seq] + n[it.seq]
        assert 0 <= it.row0 and it.nrows >= 1 and it.row0 + it.nrows <= n[it.seq]
        assert it.grow0 == int(np.sum(n[:it.seq])) + it.row0
        assert it.kv_begin % 64 == 0 and it.kv_begin < it.kv_end <= it.L + it.row0 + it.nrows
        if it.kind == 0:
            assert it.nrows * G <= 16 and it.row0 == 0 and it.nrows == n[it.seq]
        else:
            assert it.nrows * G <= 256
        cover.setdefault((it.seq, it.kvh, it.row0, it.nrows), []).append(it)
    # every row of every (sequence, kv head) is in exactly one row block
    for i in range(B):
        for h in range(Hkv):
            rows = sorted((k[2], k[3]) for k in cover if k[0] == i and k[1] == h)
            at = 0
            for r0, nr in rows:
                assert r0 == at
                at += nr
            assert at == n[i]
    # the key ranges of a block tile [0, L + row0 + nrows) without gaps or overlap
    part_ranges = []
    for (i, h, r0, nr), its in cover.items():
        its = sorted(its, key=lambda t: t.kv_begin)
        at = 0
        for t in its:
            assert t.kv_begin == at
            at = t.kv_end
        assert at == L[i] + r0 + nr
        if len(its) == 1:
            assert its[0].part_off == -1 and its[0].group == -1
        else:
            g = {t.group for t in its}
            assert len(g) == 1 and -1 not in g
            stride = nr * G * (D + 2)
            offs = [t.part_off for t in its]
            assert offs == [offs[0] + stride * k for k in range(len(its))]
            part_ranges.append((offs[0], offs[0] + stride * len(its)))
    part_ranges.sort()
    for a, b in zip(part_ranges, part_ranges[1:]):
        assert a[1] <= b[0], "partials overlap"
    return part_ranges[-1][1] if part_ranges else 0


@pytest.mark.parametrize("opts", [{}, {"narrow_chunk": 64, "mfma_chunk": 64}, {"narrow_chunk": 1024, "mfma_chunk": 256},
                                  {"force_kind": 1}, {"grid": 7}])
def test_plan_covers_every_pair_once(opts):
    rng = np.random.default_rng(3)
    for Hq, Hkv, D in [(32, 8, 128), (8, 2, 64), (8, 8, 128), (8, 1, 64), (40, 8, 128), (6, 2, 64), (7, 1, 128)]:
        L = rng.integers(0, 3000, size=24)
        n = np.where(rng.random(24) < 0.5, 1, rng.integers(1, 400, size=24))
        L[0], n[0] = 0, 1
        L[1], n[1] = 0, 300
        items, st = ppd.ppd_plan_build(Hq, Hkv, D, 16, 1 << 20, L, n, **opts)
        assert st.n_items == len(items) == st.n_narrow + st.n_mfma
        used = replay(items, L, n, Hkv, Hq // Hkv, D)
        assert used == st.partial_floats
        # queues: eight MFMA queues, then the narrow queue (longest first); tiles that read the same K/V
        # (same sequence, KV head and key range) sit in one queue, next to each other
        queues = [t.queue for t in items]
        assert queues == sorted(queues)
        assert all((t.kind == 0) == (t.queue in (8, 9)) for t in items)
        lens = [t.kv_end - t.kv_begin for t in items if t.kind == 0]
        assert lens == sorted(lens, reverse=True)
        seen, last = set(), None
        for t in items:
            if t.kind == 0:
                continue
            key = (t.seq, t.kvh, t.kv_begin)
            if key != last:
                assert key not in seen, "a sharing group is split"
                seen.add(key)
                last = key
        b = si.make_batch("x", L=L, n=n, Hq=Hq, Hkv=Hkv, D=D, seed=0, with_data=False)
        assert st.kv_bytes == b.kv_read_bytes()
        assert abs(st.flops - b.attention_flops()) <= 1e-9 * st.flops
        assert st.kv_bytes_tiles >= st.kv_bytes - 1
        assert 1 <= st.grid <= max(1, st.n_items)


def test_short_narrow_tiles_form_the_wave_queue_when_there_are_many():
    """Narrow tiles of at most 384 keys go to queue 9 (one tile per wave, eight to a claim) once the launch has six
    of them per workgroup; they stay the tail of the longest-first narrow list, and the rest of the plan is as before."""
    rng = np.random.default_rng(5)
    L = np.concatenate([rng.integers(1, 380, size=40), rng.integers(1500, 6000, size=6), [300, 5000]])
    n = np.concatenate([np.ones(46, np.int64), [70, 200]])
    for num_cus, expect_wave in ((4, True), (256, False)):
        items, st = ppd.ppd_plan_build(16, 2, 128, 16, 1 << 20, L, n, num_cus=num_cus)
        replay(items, L, n, 2, 8, 128)
        wave = [t for t in items if t.queue == 9]
        assert bool(wave) == expect_wave
        assert all(t.kind == 0 and t.kv_end - t.kv_begin <= 384 for t in wave)
        assert all(t.kv_end - t.kv_begin > 384 for t in items if t.queue == 8) or not wave
        queues = [t.queue for t in items]
        assert queues == sorted(queues)
        lens = [t.kv_end - t.kv_begin for t in items if t.kind == 0]
        assert lens == sorted(lens, reverse=True)
        if wave:
            assert len(wave) >= 80 and st.grid <= 4


def test_plan_of_random_batches_covers_every_pair_once():
    """Random head shapes, batch sizes and length mixes (decode, few-row, append-prefill, full prefill; contexts up
    to 70K) through the automatic split choices: coverage, partial layout and the 32768-key limit of an MFMA tile."""
    rng = np.random.default_rng(17)
    for trial in range(60):
        Hkv = int(rng.choice([1, 2, 4, 8, 16]))
        G = int(rng.integers(1, 9))
        D = int(rng.choice([64, 128]))
        B = int(rng.choice([1, 2, 5, 30, 120]))
        kind = rng.integers(0, 4, B)
        L = np.where(kind == 3, 0, rng.integers(0, int(rng.choice([100, 5000, 70000])), B)).astype(np.int64)
        n = np.where(kind == 0, 1, np.where(kind == 1, rng.integers(2, 9, B),
                                            rng.integers(1, int(rng.choice([70, 700, 3000])), B))).astype(np.int64)
        items, st = ppd.ppd_plan_build(G * Hkv, Hkv, D, 16, 1 << 24, L, n)
        assert replay(items, L, n, Hkv, G, D) == st.partial_floats
        assert all(t.kv_end - t.kv_begin <= 32768 for t in items if t.kind == 1)
        assert all(t.kv_begin % 64 == 0 for t in items)


def test_mfma_split_size_and_queue_order():
    """The split size of the row-block tiles comes from a scheduling estimate: enough equal row blocks stay whole
    (no partials); a single short append-prefill over a long context is cut until the tiles occupy the
    workgroups; inside every MFMA queue the groups run longest tile first."""
    # 8 sequences x 8 row blocks x 8 KV heads = 512 equal tiles on 256 workgroups: nothing to gain from splitting
    items, st = ppd.ppd_plan_build(32, 8, 128, 16, 1 << 20, [8192] * 8, [512] * 8)
    assert st.n_groups == 0 and st.n_items == 512 and st.mfma_chunk == 32768
    # one row block per KV head over 32000 cached tokens: 8 whole tiles would leave 248 workgroups idle
    items, st = ppd.ppd_plan_build(32, 8, 128, 16, 1 << 20, [32000], [64])
    assert st.n_groups == 8 and 128 <= st.n_items <= 512
    assert all(t.kv_end - t.kv_begin <= st.mfma_chunk + 64 for t in items)
    # a fixed option overrides the estimate
    items, st = ppd.ppd_plan_build(32, 8, 128, 16, 1 << 20, [32000], [64], mfma_chunk=4096)
    assert st.mfma_chunk == 4096 and st.n_items == 8 * 8
    # queue order: by the longest tile of a group, descending
    rng = np.random.default_rng(11)
    L = rng.integers(2048, 16384, size=16)
    n = rng.integers(16, 1024, size=16)
    items, st = ppd.ppd_plan_build(32, 8, 128, 16, 1 << 20, L, n)
    for q in range(8):
        longest, last = [], None
        for t in items:
            if t.queue != q:
                continue
            key = (t.seq, t.kvh, t.kv_begin)
            if key != last:
                longest.append(0)
                last = key
            longest[-1] = max(longest[-1], t.kv_end - t.kv_begin)
        assert longest == sorted(longest, reverse=True)


def test_narrow_split_size_of_small_decode_batches():
    """Few sequences, long context: the key ranges are cut until the tiles occupy the workgroups without leaving a
    nearly empty last round; many sequences keep their ranges whole."""
    for B, L in [(1, 65536), (4, 16384), (2, 16384), (8, 65536)]:
        items, st = ppd.ppd_plan_build(32, 8, 128, 16, 1 << 22, [L] * B, [1] * B)
        assert st.n_narrow == st.n_items
        per_round = st.n_items % 256 or 256
        assert st.n_items >= 128 and per_round >= 128, (B, L, st.n_items)
        assert 512 <= st.narrow_chunk <= 8192
    items, st = ppd.ppd_plan_build(32, 8, 128, 16, 1 << 22, [4000] * 256, [1] * 256)
    assert st.n_groups == 0 and st.n_items == 256 * 8
    # a fixed option overrides the estimate
    items, st = ppd.ppd_plan_build(32, 8, 128, 16, 1 << 22, [16384] * 4, [1] * 4, narrow_chunk=1024)
    assert st.narrow_chunk == 1024 and st.n_items == 4 * 8 * 17


def test_plan_refuses_a_batch_that_needs_millions_of_tiles():
    # 2^29 new tokens in one sequence: 8.4M row blocks x 8 KV heads, far beyond one launch's work list
    with pytest.raises(ppd.PPDError) as e:
        ppd.ppd_plan_build(32, 8, 128, 16, 1 << 24, [0], [1 << 29])
    assert e.value.status == -3
    # many long decode sequences: tiles counted as they are made
    with pytest.raises(ppd.PPDError) as e:
        ppd.ppd_plan_build(32, 8, 128, 16, 1 << 24, [(1 << 30) - 2] * 64, [1] * 64, narrow_chunk=64)
    assert e.value.status == -3


def test_plan_classification_follows_L_and_n():
    # n*G <= 16 columns is the narrow (decode-like) path; more rows go to the MFMA row blocks
    items, st = ppd.ppd_plan_build(32, 8, 128, 16, 1024, [100, 100, 100, 0], [1, 4, 5, 64])
    kinds = {}
    for t in items:
        kinds.setdefault(t.seq, set()).add(t.kind)
    assert kinds == {0: {0}, 1: {0}, 2: {1}, 3: {1}}
    # cost of append-prefill vs full prefill of the same total length: roughly (L+n)/n times cheaper when n << L
    _, ap = ppd.ppd_plan_build(32, 8, 128, 16, 1 << 20, [8192], [128])
    _, full = ppd.ppd_plan_build(32, 8, 128, 16, 1 << 20, [0], [8192 + 128])
    ratio = full.flops / ap.flops
    assert 0.45 * (8320 / 128) < ratio < 0.55 * (8320 / 128)   # ~ (L+n)/(2n): the causal half of the square


def test_plan_rejects_bad_arguments():
    for L, n, code in [([5], [0], -3), ([-1], [1], -3), ([2 ** 30], [5], -3)]:
        with pytest.raises(ppd.PPDError) as e:
            ppd.ppd_plan_build(32, 8, 128, 16, 64, L, n)
        assert e.value.status == code
    for shape in [(32, 8, 100, 16, 64), (32, 8, 128, 8, 64), (32, 5, 128, 16, 64), (64, 2, 128, 16, 64), (9, 1, 128, 16, 64),
                  (32, 8, 128, 16, 0)]:
        with pytest.raises(ppd.PPDError) as e:
            ppd.ppd_plan_build(*shape, [5], [1])
        assert e.value.status == -2
    with pytest.raises(ppd.PPDError) as e:
        ppd.ppd_plan_build(32, 8, 128, 16, 64, [5], [1], narrow_chunk=100)
    assert e.value.status == -3
    items, st = ppd.ppd_plan_build(32, 8, 128, 16, 64, [], [])
    assert items == [] and st.n_items == 0


def test_trace_schedule_is_consistent():
    steps, max_tokens = si.cfg5_trace(seed=0, n_conv=12, turns=3, start_spread=20)
    cached = np.zeros(12, np.int64)
    seen_attend = False
    for s in steps:
        assert np.array_equal(s.L, cached[s.conv]) and (s.n >= 1).all()
        if not s.attend:
            assert (s.L == 0).all()          # landing of transferred KV happens on turn 1 only
        else:
            seen_attend = True
        cached[s.conv] += s.n
    assert seen_attend and np.array_equal(cached, max_tokens)


def test_bench_refuses_more_than_one_gpu_and_reads_its_traffic_file():
    """bench.py measures one GPU (its --gpus N > 1 exits with a message, before anything touches a GPU), and its
    roofline.traffic comes from the committed counter summary."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE,
                         stderr=subprocess.PIPE, text=True)
    assert res.returncode != 0 and "one GPU" in (res.stderr + res.stdout)
    import bench
    for w in ("cfg4_mixed_ap", "cfg2_decode", "cfg3_ap", "cfg4_decode_only"):
        t = bench.measured_traffic(w)
        b = bench.make_shapes(w, 0)
        assert t is not None and 0.9 * b.kv_read_bytes() < t < 3.0 * b.kv_read_bytes()
    assert bench.measured_traffic("no_such_workload") is None
