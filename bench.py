#!/usr/bin/env python3
"""Benchmark of the decode-node mixed step on one MI355X.

A step = one pass of the whole hot path over one synthetic batch: ppd_kv_append of the new tokens'
K/V, then ppd_mixed_attention (plan on the host, one launch of the mixed kernel, LSE merge).  Inputs are
resident in HBM before the timed region.  Default workload: the decode-node mixed batch (128 decode
sequences co-batched with 4 append-prefills on a Llama-3-8B-shaped layer); the same run also times the
decode-only and full-prefill variants (decode-step slowdown), the decode-only batch (HBM fraction) and
the append-prefill-only batch (MFMA fraction), and the CPU oracle on a bounded sample.

Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

import numpy as np

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published
POOL_COPIES = 3              # page-pool copies a benchmark rotates over, one per step (when they fit)
SETTLE_STEPS = 20            # untimed steps before any timed region (warm-up steps count towards them)


def measured_traffic(workload):
    """HBM bytes per launch of the mixed kernel from the counter runs summarised in profiles/hbm_traffic.json
    (FETCH_SIZE + WRITE_SIZE, each scaled by the factor a plain copy of known size gives); None if absent."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            return json.load(f)["workloads"][workload]["hbm_bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def per_sequence_roofline_us(b):
    """Sum over the sequences of max(KV bytes / HBM peak, attention flops / MFMA peak): the time at peak if every
    sequence ran alone against the bound that governs it (decode rows: bytes; append-prefill rows above ~80 new
    tokens at G = 4: flops)."""
    import numpy as np
    L = b.L.astype(np.float64)
    n = b.n.astype(np.float64)
    t_hbm = (L + n) * b.kv_bytes_per_token() / (HBM_PEAK_GBS * 1e9)
    t_mfma = 4.0 * b.Hq * b.D * (n * L + n * (n + 1) / 2) / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    return float(np.sum(np.maximum(t_hbm, t_mfma)) * 1e6)


def make_shapes(name, seed):
    import synthetic_inputs as si
    if name == "cfg4_mixed_ap":
        return si.cfg4_mixed(seed, with_data=False)
    if name == "cfg4_mixed_full":
        return si.cfg4_mixed(seed, full_prefill=True, with_data=False)
    if name == "cfg4_decode_only":
        return si.cfg4_mixed(seed, with_ap=False, with_data=False)
    if name == "cfg2_decode":
        return si.cfg2_decode(seed, with_data=False)
    if name == "cfg3_ap":
        return si.cfg3_append_prefill(seed, with_data=False)
    raise SystemExit("unknown workload " + name)


class Runner:
    def __init__(self, b, torch, seed=0, options=None, fp8=False):
        import paper_2603_13358_amd as ppd
        import synthetic_inputs as si
        self.torch, self.b, self.fp8 = torch, b, fp8
        self.dev = torch.device("cuda:0")
        self.ctx = ppd.Context(b.Hq, b.Hkv, b.D, b.num_pages)
        if fp8:  # FP8 E4M3 pages (an extension beyond the paper's 16-bit KV): half the bytes per cached token
            self.ctx.set_kv_format(ppd.PPD_KV_FP8_E4M3, si.FP8_BENCH_SCALE, si.FP8_BENCH_SCALE)
        for k, v in (options or {}).items():
            self.ctx.set_option(k, v)
        self.w = si.device_workload(b, torch, self.dev, seed, fp8=fp8)
        # Consecutive steps read different copies of the page pool, as the layers of a model do: nothing of a
        # step's K/V is left in the 256 MB Infinity Cache (or an L2) by the step before.  Identical contents, so
        # every step computes the same result.
        copies = POOL_COPIES if self.w["pool"].numel() * self.w["pool"].element_size() * POOL_COPIES <= 64e9 else 1
        self.pools = [self.w["pool"]] + [self.w["pool"].clone() for _ in range(copies - 1)]
        self.at = 0
        self.stream = torch.cuda.current_stream().cuda_stream

    def step(self):
        w, b = self.w, self.b
        pool = self.pools[self.at % len(self.pools)]
        self.at += 1
        self.ctx.kv_append(w["k_new"], w["v_new"], pool, w["slots"], stream=self.stream)
        self.ctx.mixed_attention(w["q"], pool, w["page_tables"], b.L, b.n, b.scale, w["out"], stream=self.stream)

    def time_steps(self, steps, warmup):
        torch = self.torch
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    def step_distribution_us(self, steps):
        """p10 / p50 / p90 of single steps (append + attention), each bracketed by events on the stream the work
        runs on (torch's current stream), back to back, read after the region."""
        torch = self.torch
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        torch.cuda.synchronize()
        ev[0].record()
        for i in range(steps):
            self.step()
            ev[i + 1].record()
        torch.cuda.synchronize()
        us = sorted(ev[i].elapsed_time(ev[i + 1]) * 1e3 for i in range(steps))
        pick = lambda f: us[min(steps - 1, int(f * steps))]
        return {"p10": pick(0.10), "p50": pick(0.50), "p90": pick(0.90), "steps": steps}

    def kernel_ms(self, steps, warmup=0):
        """Mean duration of the mixed kernel alone over a timed region of its own: the same back-to-back steps as
        time_steps, with a pair of HIP events recorded by the library around every launch of the kernel, on the
        stream it is launched on; the events are read after the region has ended."""
        for _ in range(warmup):
            self.step()
        self.torch.cuda.synchronize()
        self.ctx.set_option("timing", 1)
        for _ in range(steps):
            self.step()
        self.torch.cuda.synchronize()
        total, launches = self.ctx.timed_kernels_ms()
        self.ctx.set_option("timing", 0)
        assert launches == steps
        return total / launches

    def warm_replan_us(self, reps=4):
        """Host cost of planning and staging a step whose lengths differ from the previous call's, once the
        context's buffers have grown (every real decode step moves each L by one): alternates between the batch
        and the batch with every cached length one shorter (same pages, one key fewer), reads the library's own
        timer of the non-reused calls; the launches they enqueue are drained, results of the shorter batch unused."""
        w, b = self.w, self.b
        shorter = np.maximum(b.L - 1, 0).astype(np.int32)
        pool = self.pools[0]
        us = []
        for _ in range(reps):
            for L in (shorter, b.L):
                self.ctx.mixed_attention(w["q"], pool, w["page_tables"], L, b.n, b.scale, w["out"], stream=self.stream)
                us.append(self.ctx.plan_stats().plan_host_us)
        self.torch.cuda.synchronize()
        return float(np.median(us))

    def close(self):
        self.ctx.close()
        self.w = None
        self.pools = None
        self.torch.cuda.empty_cache()


def cpu_baseline(runner, budget_s=15.0):
    """Times the oracle, as it stands, on a bounded sample of the workload and scales to one step.

    The sample is whole decode sequences (shortest first) plus the first rows of one append-prefill, sized
    from a short calibration run so that the measured part takes about budget_s seconds."""
    import oracle
    import synthetic_inputs as si
    b, torch = runner.b, runner.torch
    runner.step()
    torch.cuda.synchronize()
    cores = len(os.sched_getaffinity(0))
    order = np.argsort(b.L.astype(np.int64) + b.n)
    dec_all = [int(i) for i in order if b.n[i] == 1]
    ap_all = [int(i) for i in order if b.n[i] > 1]

    def run_sample(n_dec, n_ap_rows):
        dec = dec_all[:n_dec]
        ap = ap_all[:1] if n_ap_rows > 0 else []
        seqs = dec + ap
        sub, pool, rows = si.compact_subbatch(b, seqs, runner.w["pool"], runner.w["q"], torch)
        mask = np.zeros(sub.T, np.uint8)
        mask[:len(dec)] = 1
        ap_rows = int(min(n_ap_rows, b.n[ap[0]])) if ap else 0
        mask[len(dec):len(dec) + ap_rows] = 1
        pairs = float(sum(int(b.L[i]) + 1 for i in dec))
        if ap:
            pairs += sum(int(b.L[ap[0]]) + j + 1 for j in range(ap_rows))
        t0 = time.perf_counter()
        if runner.fp8:
            ref = oracle.mixed_attention_fp8(sub.q, pool, si.FP8_BENCH_SCALE, si.FP8_BENCH_SCALE, sub.page_tables, sub.L,
                                             sub.n, sub.Hq, sub.Hkv, sub.D, sub.P, sub.num_pages, sub.scale,
                                             row_mask=mask, threads=cores)
        else:
            ref = oracle.mixed_attention(sub.q, pool, sub.page_tables, sub.L, sub.n, sub.Hq, sub.Hkv, sub.D, sub.P,
                                         sub.num_pages, sub.scale, row_mask=mask, threads=cores)
        dt = time.perf_counter() - t0
        got = runner.w["out"].float().cpu().numpy()[rows]
        sel = mask.astype(bool)
        err = float(np.abs(got[sel] - ref[sel]).max()) if sel.any() else 0.0
        return dt, pairs, len(dec), ap_rows, err

    dt, pairs, _, _, _ = run_sample(min(2, len(dec_all)), 4 if ap_all else 0)
    rate = pairs / max(dt, 1e-6)                       # (row, key) pairs per second, all heads
    want = rate * budget_s
    n_dec, acc = 0, 0.0
    while n_dec < len(dec_all) and acc < want / (2 if ap_all else 1):
        acc += int(b.L[dec_all[n_dec]]) + 1
        n_dec += 1
    n_ap_rows = 0
    if ap_all:
        per_row = int(b.L[ap_all[0]]) + 1
        n_ap_rows = int(max(4, min(b.n[ap_all[0]], (want - acc) / per_row)))
    dt, pairs, nd, nr, err = run_sample(n_dec, n_ap_rows)
    pairs_total = float(np.sum(b.n.astype(np.float64) * b.L + b.n.astype(np.float64) * (b.n + 1) / 2))
    return {"value": dt * 1e6 * pairs_total / pairs, "unit": "us/step (extrapolated by visible (row,key) pairs)",
            "cores": cores, "kind": "oracle",
            "sample": "%d whole decode sequences + first %d rows of one append-prefill, all heads: %.3g of %.3g "
                      "(row,key) pairs, %.2f s measured" % (nd, nr, pairs, pairs_total, dt),
            "max_abs_err_vs_gpu": err}


def run_trace(torch, seed, max_steps, pool_gb, turns=5, options=None):
    """Multi-turn trace on a 70B-class GQA layer (64 q / 8 kv heads): every engine step = one KV append plus one
    mixed attention over all active conversations, pages drawn at random from a large shared pool."""
    import paper_2603_13358_amd as ppd
    import synthetic_inputs as si
    Hq, Hkv, D, P = 64, 8, 128, 16
    steps, max_tokens = si.cfg5_trace(seed, turns=turns)
    page_bytes = 2 * Hkv * P * D * 2
    free_b, _ = torch.cuda.mem_get_info()
    num_pages = int(min(pool_gb * 1e9, free_b * 0.9) // page_bytes)
    rng = np.random.default_rng(9000 + seed)
    need = (max_tokens + P - 1) // P
    pages = rng.choice(num_pages, size=int(need.sum()), replace=False).astype(np.int32)
    pt = np.full((len(need), int(need.max())), -1, np.int32)
    at = 0
    for c in range(len(need)):
        pt[c, :need[c]] = pages[at:at + need[c]]
        at += int(need[c])
    dev = torch.device("cuda:0")
    ctx = ppd.Context(Hq, Hkv, D, num_pages)
    for k_, v_ in (options or {}).items():
        ctx.set_option(k_, v_)
    pool = torch.empty((num_pages * page_bytes // 2,), dtype=torch.bfloat16, device=dev)   # contents: whatever
    # only the pages in use need defined values
    pool.view(num_pages, -1)[torch.from_numpy(pages.astype(np.int64)).to(dev)] = 0
    pt_d = torch.from_numpy(pt).to(dev)
    stream = torch.cuda.current_stream().cuda_stream
    scale = 1.0 / np.sqrt(D)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    rec, plan_us, first_us = [], [], []
    turn_of = np.ones(len(need), np.int64)          # turn each conversation is in (turn 1 = its landing)
    by_turn = {}                                    # turn -> [accumulated context, new tokens, step us] per append-prefill
    if max_steps:
        steps = steps[:max_steps]
    t_all0 = time.perf_counter()
    for st in steps:
        T = int(st.n.sum())
        k = torch.empty((T, Hkv, D), dtype=torch.bfloat16, device=dev).normal_(generator=gen)
        v = torch.empty((T, Hkv, D), dtype=torch.bfloat16, device=dev).normal_(generator=gen)
        slots = np.concatenate([pt[c, (np.arange(L, L + n)) // P].astype(np.int64) * P + np.arange(L, L + n) % P
                                for c, L, n in zip(st.conv, st.L, st.n)])
        slots_d = torch.from_numpy(slots).to(dev)
        q = torch.empty((T, Hq, D), dtype=torch.bfloat16, device=dev).normal_(generator=gen)
        out = torch.empty((T, Hq, D), dtype=torch.bfloat16, device=dev)
        sub_pt = pt_d[torch.from_numpy(st.conv.astype(np.int64)).to(dev)].contiguous()
        # "layer 0" plans and uploads (the lengths changed since the previous step); "layer 1" repeats the
        # same append + attention with the plan already on the device, as every further layer of a model would
        e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        torch.cuda.synchronize()
        e0.record()
        ctx.kv_append(k, v, pool, slots_d, stream=stream)
        if st.attend:
            ctx.mixed_attention(q, pool, sub_pt, st.L, st.n, scale, out, stream=stream)
        e1.record()
        ctx.kv_append(k, v, pool, slots_d, stream=stream)
        if st.attend:
            ctx.mixed_attention(q, pool, sub_pt, st.L, st.n, scale, out, stream=stream)
        e2.record()
        e2.synchronize()
        us0 = e0.elapsed_time(e1) * 1e3
        us = e1.elapsed_time(e2) * 1e3
        plan_us.append(ctx.plan_stats().plan_host_us if st.attend else 0)
        first_us.append(us0)
        kv_bytes = int((st.L + st.n).sum()) * 2 * Hkv * D * 2 if st.attend else 0
        flops = float(4.0 * Hq * D * np.sum(st.n * st.L + st.n * (st.n + 1) / 2.0)) if st.attend else 0.0
        rec.append((us, st.attend, int((st.n > 1).sum()), int(len(st.n)), kv_bytes, flops))
        if st.attend:
            for c, Lc, nc in zip(st.conv, st.L, st.n):
                if nc > 1:
                    turn_of[c] += 1
                    by_turn.setdefault(int(turn_of[c]), []).append((int(Lc), int(nc), us))
    wall = time.perf_counter() - t_all0
    ctx.close()
    us = np.array([r[0] for r in rec])
    dec = np.array([r[1] and r[2] == 0 for r in rec])
    apm = np.array([r[1] and r[2] > 0 for r in rec])
    land = np.array([not r[1] for r in rec])
    kvb = np.array([r[4] for r in rec], np.float64)
    fl = np.array([r[5] for r in rec], np.float64)

    def dist(x):
        return {"n": int(x.size), "p10": float(np.percentile(x, 10)), "p50": float(np.percentile(x, 50)),
                "p90": float(np.percentile(x, 90)), "mean": float(x.mean())} if x.size else {"n": 0}
    kv_tok_bytes_model = 2 * Hkv * D * 2 * 80       # 80 layers of this 70B-class shape
    turn_rows = {}
    for t in sorted(by_turn):
        a = np.array(by_turn[t], np.float64)
        ctx_mean = float(a[:, 0].mean())
        turn_rows[str(t)] = {"append_prefills": int(a.shape[0]), "mean_accumulated_context": ctx_mean,
                             "mean_new_tokens": float(a[:, 1].mean()), "mean_step_us_one_layer": float(a[:, 2].mean()),
                             "kv_transfer_ms_of_that_context_at_25GBs": ctx_mean * kv_tok_bytes_model / 25e9 * 1e3}
    return {"turns": turns, "append_prefill_steps_by_turn": turn_rows, "steps": len(rec), "pool_pages": num_pages, "pool_GB": num_pages * page_bytes / 1e9,
            "total_gpu_ms": float(us.sum() / 1e3), "wall_s_incl_input_generation": wall,
            "decode_only_steps_us": dist(us[dec]), "steps_with_append_prefill_us": dist(us[apm]),
            "first_layer_decode_only_steps_us": dist(np.array(first_us)[dec]),
            "first_layer_steps_with_append_prefill_us": dist(np.array(first_us)[apm]),
            "plan_host_us": dist(np.array(plan_us, np.float64)[dec | apm]),
            "kv_landing_steps_us": dist(us[land]),
            "decode_only_aggregate_HBM_GBs": float(kvb[dec].sum() / (us[dec].sum() * 1e-6) / 1e9) if dec.any() else None,
            "ap_steps_aggregate_TFLOPs": float(fl[apm].sum() / (us[apm].sum() * 1e-6) / 1e12) if apm.any() else None,
            "note": "per-step times = HIP events around kv_append + mixed_attention of one layer with the step's plan "
                    "already on the device (every layer but the first of an engine step); first_layer_* include "
                    "planning and upload; 70B-class layer 64q/8kv heads, D=128"}


def run_landing(torch, seed, steps, fp8=False):
    """KV landing of one transferred request: 5115 tokens (the context length the paper quotes for its ~670 MB
    example) x 32 layers of an 8-KV-head, D=128 model scattered into 32 per-layer page pools in one launch.
    fp8: the pools hold FP8 E4M3 pages (extension beyond the paper): the landing quantises on the way."""
    import synthetic_inputs as si
    import oracle
    import paper_2603_13358_amd as ppd
    layers, T, Hkv, D, P = 32, 5115, 8, 128, 16
    num_pages = (T + P - 1) // P + 64
    rng = np.random.default_rng(seed)
    pages = rng.permutation(num_pages)[:(T + P - 1) // P]
    t = np.arange(T)
    slots = pages[t // P].astype(np.int64) * P + t % P
    dev = torch.device("cuda:0")
    pe = num_pages * 2 * Hkv * P * D
    ctx = ppd.Context(32, Hkv, D, num_pages)
    if fp8:
        ctx.set_kv_format(ppd.PPD_KV_FP8_E4M3, si.FP8_BENCH_SCALE, si.FP8_BENCH_SCALE)
    k = torch.empty((layers, T, Hkv, D), dtype=torch.bfloat16, device=dev).normal_()
    v = torch.empty((layers, T, Hkv, D), dtype=torch.bfloat16, device=dev).normal_()
    pools = torch.zeros((layers * pe,), dtype=torch.uint8 if fp8 else torch.bfloat16, device=dev)
    slots_d = torch.from_numpy(slots).to(dev)
    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(3):
        ctx.kv_land(k, v, pools, pe, layers, slots_d, stream=stream)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        ctx.kv_land(k, v, pools, pe, layers, slots_d, stream=stream)
    e1.record()
    e1.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / steps
    moved = 2 * layers * T * Hkv * D * 2          # K and V payload
    # ceiling of a read-once write-once pattern on this machine: a plain contiguous device copy of the same payload
    dst = torch.empty_like(k)
    for _ in range(3):
        dst.copy_(k)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(steps):
        dst.copy_(k)
        dst.copy_(v)
    c1.record()
    c1.synchronize()
    copy_us = c0.elapsed_time(c1) * 1e3 / steps
    del dst
    # oracle on the host: 4 layers, scaled
    kh = k[:4].view(torch.int16).cpu().numpy().view(np.uint16)
    vh = v[:4].view(torch.int16).cpu().numpy().view(np.uint16)
    ref = np.zeros(4 * pe, np.uint8 if fp8 else np.uint16)
    t0 = time.perf_counter()
    if fp8:
        oracle.kv_land_fp8(kh, vh, ref, pe, 4, slots, Hkv, D, P, num_pages, si.FP8_BENCH_SCALE, si.FP8_BENCH_SCALE)
    else:
        oracle.kv_land(kh, vh, ref, pe, 4, slots, Hkv, D, P, num_pages)
    cpu_s = (time.perf_counter() - t0) * layers / 4
    got = pools[:4 * pe].cpu().numpy() if fp8 else pools[:4 * pe].view(torch.int16).cpu().numpy().view(np.uint16)
    ctx.close()
    rw = moved + moved // 2 if fp8 else 2 * moved   # bytes read + bytes written
    return {"tokens": T, "layers": layers, "payload_bytes": moved, "kv_pages": "fp8_e4m3" if fp8 else "bf16", "us": us,
            "achieved_GBs_read_plus_write": rw / (us * 1e-6) / 1e9,
            "hbm_frac": rw / (us * 1e-6) / 1e9 / HBM_PEAK_GBS,
            "plain_copy_of_same_payload_us": copy_us,
            "plain_copy_GBs_read_plus_write": 2 * moved / (copy_us * 1e-6) / 1e9,
            "frac_of_plain_copy": copy_us / us, "bit_exact_vs_oracle_4_layers": bool(np.array_equal(got, ref)),
            "cpu_oracle_us_extrapolated_from_4_layers": cpu_s * 1e6,
            "paper_context": "moving the same ~670 MB between nodes takes ~4.5 ms over NVLink, ~27 ms over IB HDR, "
                             "~67 ms over 100GbE (appendix, bandwidth simulation); landing it in the pools is the "
                             "decode node's share"}


# Representative request of every cell of the routing grid (paper appendix "Decision-Engine Discretization"): one
# accumulated context per context class and (new input, expected output) token counts of the nine workload types,
# decode-heavy to prefill-heavy (the two settings the paper names, 32/512 and 1024/32, are the extremes).
ROUTE_CTX = (256, 2048, 8192)
ROUTE_TYPES = ((32, 512), (64, 512), (64, 256), (128, 256), (256, 256), (512, 256), (512, 64), (1024, 64), (1024, 32))
ROUTE_QPS = (0.5, 1, 2, 4, 6, 8, 10, 12, 16, 20)
ROUTE_RATIO_CENTERS = tuple(a / b for a, b in ROUTE_TYPES)


def run_route_table(torch, seed, steps, beta_gbs, layers=32, w_ttft=1.0, w_tpot=1.0, tpot_s=0.010, only=None):
    """Offline phase of the paper's routing algorithm with this repository's own measurements in place of the
    paper's whole-system ones: per cell, the turn's time to first token and the decode slowdown when the
    append-prefill runs on the decode node (x = 1) against the prefill-node path (x = 0), at attention level.

      x = 1: TTFT = layers * (mixed step: the decode batch + the append-prefill over the cached context)
             extra decode-node time per request = layers * (mixed step - decode-only step)
      x = 0: TTFT = layers * (append-prefill step alone, on a prefill node that holds the context)
                    + transfer of the whole context's KV at `beta_gbs` (injected-delay equation of the appendix
                      "Bandwidth Simulation" on top of the fast-interconnect time) + landing it in the page pools
             extra decode-node time per request = the landing
      delta_ttft = (TTFT0 - TTFT1) / TTFT0;  delta_tpot = qps * (extra1 - extra0): the share of the decode
      node's time the choice costs, i.e. the relative lengthening of its decode steps.
    The decode batch next to a request is the concurrency its QPS level implies at a whole-model time per output
    token of `tpot_s` (qps * n_out * tpot_s, snapped to a power of two in 1..256).  Weight-bound GEMMs are outside
    this repository, so both deltas are attention-only.  `only`: measure just these (context class, workload type,
    QPS level) cells and leave the others at delta = 0 (x = 0)."""
    import paper_2603_13358_amd as ppd
    import synthetic_inputs as si
    kv_bytes_token = 2 * 8 * 128 * 2 * layers                    # 128 KiB per token over 32 layers of 8 KV heads
    fast_bw = 670433280 / 4.5e-3                                 # the fast interconnect of the appendix' example

    def concurrency(qps, n_out):
        b = max(1.0, min(256.0, qps * n_out * tpot_s))
        return int(2 ** round(np.log2(b)))

    memo = {}

    def step_us(L, n):
        key = (tuple(L), tuple(n))
        if key not in memo:
            b = si.make_batch("route", L=list(L), n=list(n), Hq=32, Hkv=8, D=128, seed=seed, slack_pages=16, with_data=False)
            r = Runner(b, torch, seed)
            memo[key] = r.time_steps(steps, 3) * 1e3
            r.close()
        return memo[key]

    land_memo = {}

    def land_us(T):
        if T not in land_memo:
            Hkv, D, P = 8, 128, 16
            num_pages = (T + P - 1) // P + 8
            pe = num_pages * 2 * Hkv * P * D
            dev = torch.device("cuda:0")
            ctx = ppd.Context(32, Hkv, D, num_pages)
            k = torch.empty((layers, T, Hkv, D), dtype=torch.bfloat16, device=dev).normal_()
            v = torch.empty((layers, T, Hkv, D), dtype=torch.bfloat16, device=dev).normal_()
            pools = torch.zeros((layers * pe,), dtype=torch.bfloat16, device=dev)
            t = np.arange(T)
            slots = torch.from_numpy((np.random.default_rng(seed).permutation(num_pages)[t // P].astype(np.int64) * P + t % P)).to(dev)
            stream = torch.cuda.current_stream().cuda_stream
            for _ in range(3):
                ctx.kv_land(k, v, pools, pe, layers, slots, stream=stream)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(steps):
                ctx.kv_land(k, v, pools, pe, layers, slots, stream=stream)
            e1.record()
            e1.synchronize()
            land_memo[T] = e0.elapsed_time(e1) * 1e3 / steps
            ctx.close()
        return land_memo[T]

    d_ttft, d_tpot, cells = np.zeros(270), np.zeros(270), []
    for c, n_ctx in enumerate(ROUTE_CTX):
        for r_, (n_in, n_out) in enumerate(ROUTE_TYPES):
            for q, qps in enumerate(ROUTE_QPS):
                if only is not None and (c, r_, q) not in only:
                    continue
                bsz = concurrency(qps, n_out)
                t_dec = step_us([n_ctx] * bsz, [1] * bsz)
                t_mix = step_us([n_ctx] * bsz + [n_ctx], [1] * bsz + [n_in])
                t_ap = step_us([n_ctx], [n_in])
                T = n_ctx + n_in
                t_land = land_us(T)
                t_fast = T * kv_bytes_token / fast_bw
                t_xfer = t_fast + ppd.ppd_transfer_delay_s(T, kv_bytes_token, beta_gbs * 1e9, t_fast)
                ttft1 = layers * t_mix * 1e-6
                ttft0 = layers * t_ap * 1e-6 + t_xfer + t_land * 1e-6
                extra1 = layers * (t_mix - t_dec) * 1e-6
                extra0 = t_land * 1e-6
                cell = (c * 9 + r_) * 10 + q
                d_ttft[cell] = (ttft0 - ttft1) / ttft0
                d_tpot[cell] = qps * (extra1 - extra0)
                cells.append({"cell": cell, "n_ctx": n_ctx, "n_in": n_in, "n_out": n_out, "qps": qps, "decode_batch": bsz,
                              "decode_step_us": t_dec, "mixed_step_us": t_mix, "ap_alone_step_us": t_ap,
                              "landing_us": t_land, "transfer_ms": t_xfer * 1e3, "ttft_local_ms": ttft1 * 1e3,
                              "ttft_pd_ms": ttft0 * 1e3, "delta_ttft": d_ttft[cell], "delta_tpot": d_tpot[cell]})
    table = ppd.ppd_route_table_build(d_ttft, d_tpot, w_ttft, w_tpot)
    by_ctx = {str(ROUTE_CTX[c]): int(table[c * 90:(c + 1) * 90].sum()) for c in range(3)}
    return {"beta_GBs": beta_gbs, "layers": layers, "weights": [w_ttft, w_tpot], "assumed_tpot_s": tpot_s,
            "ratio_centers": list(ROUTE_RATIO_CENTERS), "x_table": table.tolist(), "cells_local_of_90_by_context": by_ctx,
            "delta_ttft": d_ttft.tolist(), "delta_tpot": d_tpot.tolist(), "cells": cells,
            "measurements": len(memo) + len(land_memo)}


def run_sweeps(torch, seed, steps, options):
    """Attention-level analogues of the paper's interference experiments (section 4.1 and its appendix): a decode
    batch co-located with append-prefill or with a full prefill of equal context, over batch size, over context
    length, with 4 concurrent prefills, and with the append-prefill fed in token-budgeted chunks."""
    import synthetic_inputs as si

    def time_batch(L, n, Hq=32, Hkv=8, want_batch=False):
        b = si.make_batch("sweep", L=L, n=n, Hq=Hq, Hkv=Hkv, D=128, seed=seed, slack_pages=16, with_data=False)
        r = Runner(b, torch, seed, options)
        ms = r.time_steps(steps, 2)
        r.close()
        return (ms * 1e3, b) if want_batch else ms * 1e3

    def trio(dec_L, ap_L, ap_n, n_prefill=1):
        dec_L = list(dec_L)
        base = time_batch(dec_L, [1] * len(dec_L))
        with_ap = time_batch(dec_L + [ap_L] * n_prefill, [1] * len(dec_L) + [ap_n] * n_prefill)
        with_full = time_batch(dec_L + [0] * n_prefill, [1] * len(dec_L) + [ap_L + ap_n] * n_prefill)
        return {"decode_only_us": base, "with_append_prefill_us": with_ap, "with_full_prefill_us": with_full,
                "slowdown_append": with_ap / base - 1.0, "slowdown_full": with_full / base - 1.0}

    rng = np.random.default_rng(seed)
    out = {"setup": "32q/8kv heads, D=128; decode sequences at the stated context; one co-located prefill adds "
                    "1024 new tokens either over the cached context (append) or recomputing it (full, L=0)"}
    out["batch_size_sweep_ctx4096"] = {str(bs): trio([4096] * bs, 4096, 1024) for bs in (16, 64, 128, 200, 256)}
    out["four_prefills_batch200_ctx4096"] = trio([4096] * 200, 4096, 1024, n_prefill=4)
    out["context_sweep_batch128"] = {str(c): trio([c] * 128, c, 1024) for c in (2048, 8192, 16384, 32768, 65536)}
    # chunked append-prefill: 2048 new tokens over 16384 cached, fed in chunks next to 128 decodes at 8192
    dec = [8192] * 128
    base = time_batch(dec, [1] * 128)
    chunked = {}
    for chunk in (128, 256, 512, 1024, 2048):
        per_step = []
        for c0 in range(0, 2048, chunk):
            per_step.append(time_batch(dec + [16384 + c0], [1] * 128 + [chunk]))
        chunked[str(chunk)] = {"steps": len(per_step), "mean_step_us": float(np.mean(per_step)),
                               "decode_step_slowdown": float(np.mean(per_step)) / base - 1.0,
                               "total_us_until_prefill_done": float(np.sum(per_step))}
    out["chunked_append_prefill"] = {"decode_only_us": base, "by_chunk_tokens": chunked}
    # head shapes of the three models the paper serves (section 5.1), one attention layer each: 128 decodes at
    # 8192 context (HBM-bound), 8 append-prefills of 512 tokens over 8192 (MFMA-bound), and both together
    shapes = {"llama3_8b_32q_8kv": (32, 8), "qwen2.5_14b_40q_8kv": (40, 8), "qwen3_30b_a3b_32q_4kv": (32, 4)}
    by_shape = {}
    for name, (Hq, Hkv) in shapes.items():
        dec_us, bd = time_batch([8192] * 128, [1] * 128, Hq, Hkv, True)
        ap_us, ba = time_batch([8192] * 8, [512] * 8, Hq, Hkv, True)
        mix_us = time_batch([8192] * 136, [1] * 128 + [512] * 8, Hq, Hkv)
        by_shape[name] = {"decode_step_us": dec_us, "decode_hbm_gbs": bd.kv_read_bytes() / dec_us / 1e3,
                          "append_prefill_step_us": ap_us, "append_prefill_tflops": ba.attention_flops() / ap_us / 1e6,
                          "mixed_step_us": mix_us, "decode_step_slowdown": mix_us / dec_us - 1.0}
    out["model_head_shapes_ctx8192"] = by_shape
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg4_mixed_ap",
                    choices=["cfg4_mixed_ap", "cfg4_mixed_full", "cfg4_decode_only", "cfg2_decode", "cfg3_ap"])
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-extras", action="store_true", help="time the chosen workload only")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--kv-fp8", action="store_true",
                    help="run the chosen workload on FP8 E4M3 KV pages (extension beyond the paper; half the KV bytes)")
    ap.add_argument("--opt", action="append", default=[], help="library option key=value (tuning sweeps)")
    ap.add_argument("--trace", action="store_true", help="run the multi-turn conversation trace (cfg5) and exit")
    ap.add_argument("--trace-steps", type=int, default=0, help="limit the trace to its first N engine steps")
    ap.add_argument("--trace-pool-gb", type=float, default=200.0)
    ap.add_argument("--turns", type=int, default=5, help="turns per conversation of the trace (the paper scales 2..16)")
    ap.add_argument("--landing", action="store_true", help="time the multi-layer KV landing of one request and exit")
    ap.add_argument("--route-table", action="store_true",
                    help="measure the routing grid (local append-prefill vs transfer + landing) and build the decision table")
    ap.add_argument("--route-beta-gbs", type=float, default=25.0, help="interconnect bandwidth of the x = 0 path, GB/s")
    ap.add_argument("--route-weights", default="1,1", help="w_ttft,w_tpot")
    ap.add_argument("--sweeps", action="store_true",
                    help="interference sweeps (batch size, context, 4 prefills, chunked append-prefill) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py measures one GPU: the step has no multi-GPU part in this build (--gpus 1 only)")
    import torch
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs an MI355X: the library has no CPU path")
    options = {kv.split("=")[0]: int(kv.split("=")[1]) for kv in args.opt}
    if args.trace:
        print(json.dumps({"workload": "cfg5_multi_turn_trace", "trace": run_trace(torch, args.seed, args.trace_steps,
                                                                                 args.trace_pool_gb, args.turns, options)}))
        return
    if args.landing:
        print(json.dumps({"workload": "kv_landing_5115_tokens_32_layers", "landing": run_landing(torch, args.seed, args.steps, fp8=args.kv_fp8)}))
        return
    if args.route_table:
        w = [float(x) for x in args.route_weights.split(",")]
        print(json.dumps({"workload": "route_table", "route_table": run_route_table(
            torch, args.seed, max(5, args.steps // 5), args.route_beta_gbs, w_ttft=w[0], w_tpot=w[1])}))
        return
    if args.sweeps:
        print(json.dumps({"workload": "interference_sweeps", "sweeps": run_sweeps(torch, args.seed, max(10, args.steps // 2),
                                                                                  options)}))
        return
    def run(name, steps, warmup, want_cpu=False, fp8=False):
        b = make_shapes(name, args.seed)
        r = Runner(b, torch, args.seed, options, fp8=fp8)
        r.step()                                   # first call: plans and uploads
        first_plan_us = r.ctx.plan_stats().plan_host_us
        # After an idle gap the chip's power controller needs ~12 back-to-back launches of the MFMA-bound kernel to
        # settle (they run up to 35 % slower meanwhile): when fewer warm-up steps were asked for, run the rest
        # here, untimed, so that the timed region measures the settled state whatever --warmup says.
        for _ in range(max(0, SETTLE_STEPS - warmup)):
            r.step()
        ms = r.time_steps(steps, warmup)
        kms = r.kernel_ms(steps)
        dist = r.step_distribution_us(steps) if want_cpu or name == args.workload else None
        warm_plan_us = r.warm_replan_us() if want_cpu or name == args.workload else None
        st = r.ctx.plan_stats().as_dict()
        st["plan_host_us_first_call"] = first_plan_us
        st["plan_host_us"] = warm_plan_us
        res = {"workload": name, "ms_per_step": ms, "mixed_kernel_ms": kms, "plan": st, "step_us": dist,
               "kv_bytes": b.kv_read_bytes() // (2 if fp8 else 1), "flops": b.attention_flops(), "rows": b.T,
               "sequences": b.B,
               "seq_roofline_us": per_sequence_roofline_us(b)}
        if want_cpu:
            res["cpu"] = cpu_baseline(r)
        r.close()
        return res

    main_res = run(args.workload, args.steps, args.warmup, want_cpu=not args.no_cpu, fp8=args.kv_fp8)
    b_bytes, b_flops = main_res["kv_bytes"], main_res["flops"]
    t_hbm = b_bytes / (HBM_PEAK_GBS * 1e9)
    t_mfma = b_flops / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    kernel_s = main_res["mixed_kernel_ms"] * 1e-3
    if t_hbm >= t_mfma:
        roofline = {"bound": "hbm", "achieved": b_bytes / kernel_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    else:
        roofline = {"bound": "mfma", "achieved": b_flops / kernel_s / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s"}
    roofline["frac"] = roofline["achieved"] / roofline["peak"]
    # A mixed step has a memory-bound and a matrix-bound part that run on different compute units of the same
    # launch: time at peak of each, and the kernel against the two in series (1.0 = each part at its own peak,
    # no overlap between them; `frac` above is against the larger one alone, i.e. perfect overlap).
    roofline["time_at_peak_us"] = {"hbm": t_hbm * 1e6, "mfma": t_mfma * 1e6}
    roofline["frac_of_both_in_series"] = (t_hbm + t_mfma) / kernel_s
    # ... and against the sum over the sequences of the bound that governs each (see per_sequence_roofline_us)
    roofline["per_sequence_bound_us"] = main_res["seq_roofline_us"]
    roofline["frac_of_per_sequence_bounds"] = main_res["seq_roofline_us"] * 1e-6 / kernel_s
    roofline["traffic"] = None if args.kv_fp8 else measured_traffic(args.workload)
    fp8_s = "true" if args.kv_fp8 else "false"
    if main_res["plan"]["n_mfma"] == 0 and options.get("narrow_kernel", 1) and not options.get("launch_mode", 0):
        roofline["kernel"] = "ppd_narrow_kernel<128, %s, 8>" % fp8_s  # a step without row-block tiles: <head_dim, FP8 pages, waves>
    else:
        roofline["kernel"] = "ppd_mixed_kernel<128, %s>" % fp8_s  # <head_dim, FP8 pages>
    roofline["kernel_ms"] = main_res["mixed_kernel_ms"]

    extras = {}
    if not args.no_extras:
        few, fw = max(5, args.steps // 2), max(3, args.warmup // 2)
        for name in ["cfg4_decode_only", "cfg4_mixed_full", "cfg2_decode", "cfg3_ap", "cfg4_mixed_ap"]:
            if name == args.workload:
                continue
            steps = 5 if name == "cfg4_mixed_full" else few
            r = run(name, steps, 2 if name == "cfg4_mixed_full" else fw)
            ks = r["mixed_kernel_ms"] * 1e-3
            extras[name] = {"us_per_step": r["ms_per_step"] * 1e3, "mixed_kernel_us": r["mixed_kernel_ms"] * 1e3,
                            "hbm_GBs": r["kv_bytes"] / ks / 1e9, "hbm_frac": r["kv_bytes"] / ks / 1e9 / HBM_PEAK_GBS,
                            "mfma_TFLOPs": r["flops"] / ks / 1e12,
                            "mfma_frac": r["flops"] / ks / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                            "frac_of_per_sequence_bounds": r["seq_roofline_us"] * 1e-6 / ks,
                            "tiles": r["plan"]["n_items"]}
        extras[args.workload] = {"us_per_step": main_res["ms_per_step"] * 1e3,
                                 "mixed_kernel_us": main_res["mixed_kernel_ms"] * 1e3}
        # the same batches on FP8 E4M3 pages (extension beyond the paper: half the KV bytes; bf16 q, out, matrix math)
        fp8_pages = {}
        for name in ["cfg2_decode", "cfg4_decode_only", "cfg3_ap", "cfg4_mixed_ap"]:
            r = run(name, few, fw, fp8=True)
            ks = r["mixed_kernel_ms"] * 1e-3
            fp8_pages[name] = {"us_per_step": r["ms_per_step"] * 1e3, "mixed_kernel_us": r["mixed_kernel_ms"] * 1e3,
                               "kv_bytes_per_step": r["kv_bytes"], "hbm_GBs": r["kv_bytes"] / ks / 1e9,
                               "hbm_frac": r["kv_bytes"] / ks / 1e9 / HBM_PEAK_GBS,
                               "mfma_frac": r["flops"] / ks / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                               "speedup_vs_bf16_pages": (extras[name]["us_per_step"] / (r["ms_per_step"] * 1e3)
                                                         if name in extras else None)}
        extras["fp8_kv_pages"] = fp8_pages
        if "cfg4_decode_only" in extras and "cfg4_mixed_ap" in extras and "cfg4_mixed_full" in extras:
            base = extras["cfg4_decode_only"]["us_per_step"]
            extras["decode_step_slowdown"] = {
                "with_append_prefill": extras["cfg4_mixed_ap"]["us_per_step"] / base - 1.0,
                "with_full_prefill_of_equal_context": extras["cfg4_mixed_full"]["us_per_step"] / base - 1.0,
                "paper_context": "whole-model vLLM on 1xH100, Llama-3.1-8B, batch 200, one 1024-token prefill: "
                                 "+2% append vs +48% full (section 4.1)"}

    line = {
        "metric": "mixed AP+decode paged-attn step us; decode HBM TB/s & AP MFMA util vs peak",
        "value": main_res["ms_per_step"] * 1e3, "unit": "us/step", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": main_res["ms_per_step"], "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "sequences": main_res["sequences"], "new_token_rows": main_res["rows"],
                   "heads": "32q/8kv", "head_dim": 128, "page_size": 16, "seed": args.seed,
                   "kv_pages": "fp8_e4m3" if args.kv_fp8 else "bf16",
                   "kv_bytes_per_step": b_bytes, "attention_flops_per_step": b_flops,
                   "tiles": main_res["plan"]["n_items"], "grid": main_res["plan"]["grid"],
                   "plan_host_us": main_res["plan"]["plan_host_us"],
                   "plan_host_us_first_call": main_res["plan"]["plan_host_us_first_call"],
                   "step_us_incl_plan_amortised_over_32_layers":
                       main_res["ms_per_step"] * 1e3 + (main_res["plan"]["plan_host_us"] or 0.0) / 32.0,
                   "step_us_distribution": main_res["step_us"],
                   "note": "steady state: the device plan is reused while L, n are unchanged, as across the "
                           "layers of one engine step; plan_host_us is the warm once-per-engine-step host cost of "
                           "planning and staging a batch whose lengths changed (buffers already grown), "
                           "plan_host_us_first_call the cold first call including the workspace allocations"},
        "roofline": roofline,
        "cpu_baseline": main_res.get("cpu"),
        "extras": extras,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
