"""Seeded synthetic inputs for the mixed append-prefill + decode paged-attention step.

This module serves both the CPU oracle and the HIP path and holds none of the method's arithmetic: it
draws lengths, page tables and N(0,1) bf16 values, and states where each token lives (slot = page*P +
offset, the interface's own definition).  It never lays K/V out in the page pool -- each side does that
through its own KV append.

Shapes follow the workloads the build is measured on: a tiny mixed batch, a decode-only batch and an
append-prefill-only batch on a Llama-3-8B-shaped layer (32 q heads / 8 kv heads, head_dim 128, page 16),
a decode-node mixed batch with its full-prefill comparison run, and a multi-turn conversation trace on a
70B-class GQA layer (64 / 8).  Public conversation datasets are not available here; the log-normal
trace stands in for their shape.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

PAGE = 16


def f32_to_bf16_bits(x):
    """Round-to-nearest-even fp32 -> bf16 bit patterns (uint16).  Inputs are finite."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def normal_bf16(rng, shape, std=1.0):
    return f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32) * np.float32(std))


@dataclass
class MixedBatch:
    name: str
    Hq: int
    Hkv: int
    D: int
    P: int
    num_pages: int
    scale: float
    L: np.ndarray                      # [B] int32, cached tokens per sequence
    n: np.ndarray                      # [B] int32, new tokens per sequence
    page_tables: np.ndarray            # [B, max_pages] int32, -1 = unused
    q: Optional[np.ndarray] = None     # [T, Hq, D] uint16 (bf16 bits), rows grouped by sequence
    k: Optional[np.ndarray] = None     # [sum(L+n), Hkv, D] uint16, token-major, sequences concatenated
    v: Optional[np.ndarray] = None
    tok_off: np.ndarray = field(default=None)   # [B+1] int64 offsets of each sequence in k / v
    row_off: np.ndarray = field(default=None)   # [B+1] int64 offsets of each sequence in q / out

    def __post_init__(self):
        self.L = np.asarray(self.L, dtype=np.int32)
        self.n = np.asarray(self.n, dtype=np.int32)
        tot = self.L.astype(np.int64) + self.n.astype(np.int64)
        self.tok_off = np.concatenate([[0], np.cumsum(tot)]).astype(np.int64)
        self.row_off = np.concatenate([[0], np.cumsum(self.n.astype(np.int64))]).astype(np.int64)

    @property
    def B(self):
        return int(self.L.shape[0])

    @property
    def T(self):
        return int(self.row_off[-1])

    @property
    def max_pages(self):
        return int(self.page_tables.shape[1])

    def seq_kv(self, i):
        a, b = int(self.tok_off[i]), int(self.tok_off[i + 1])
        return self.k[a:b], self.v[a:b]

    def slots(self, i, t0, t1):
        """Pool slots of tokens t0..t1-1 of sequence i."""
        t = np.arange(t0, t1, dtype=np.int64)
        return self.page_tables[i, t // self.P].astype(np.int64) * self.P + t % self.P

    def _part(self, which):
        ks, vs, ss = [], [], []
        for i in range(self.B):
            Li, ni = int(self.L[i]), int(self.n[i])
            t0, t1 = (0, Li) if which == "cached" else (Li, Li + ni)
            ss.append(self.slots(i, t0, t1))
            if self.k is not None:
                a = int(self.tok_off[i])
                ks.append(self.k[a + t0:a + t1])
                vs.append(self.v[a + t0:a + t1])
        slots = np.concatenate(ss) if ss else np.zeros((0,), np.int64)
        if self.k is None:
            return None, None, slots
        shape = (0, self.Hkv, self.D)
        k = np.concatenate(ks) if ks else np.zeros(shape, np.uint16)
        v = np.concatenate(vs) if vs else np.zeros(shape, np.uint16)
        return k, v, slots

    def cached_part(self):
        """(k, v, slots) of every sequence's cached prefix (tokens 0..L-1)."""
        return self._part("cached")

    def new_part(self):
        """(k, v, slots) of the new tokens, in q-row order (tokens L..L+n-1 of each sequence)."""
        return self._part("new")

    def kv_bytes_per_token(self):
        return 2 * self.Hkv * self.D * 2

    def attention_flops(self):
        """4*Hq*D flops per visible (row, key) pair: new row j of a sequence sees L+j+1 keys."""
        L = self.L.astype(np.float64)
        n = self.n.astype(np.float64)
        return float(4.0 * self.Hq * self.D * np.sum(n * L + n * (n + 1) / 2))

    def kv_read_bytes(self):
        """Bytes of resident K/V that one step has to read at least once."""
        return int(np.sum(self.L.astype(np.int64) + self.n) * self.kv_bytes_per_token())


def _assign_pages(rng, L, n, P, num_pages=None, slack_pages=0):
    """One seeded permutation of the pool, handed out as consecutive disjoint slices."""
    need = (np.asarray(L, np.int64) + np.asarray(n, np.int64) + P - 1) // P
    total = int(need.sum())
    if num_pages is None:
        num_pages = total + slack_pages
    assert total <= num_pages, "pool too small"
    perm = rng.permutation(num_pages).astype(np.int32)
    max_pages = int(need.max()) if len(need) else 1
    pt = np.full((len(need), max(max_pages, 1)), -1, dtype=np.int32)
    at = 0
    for i, c in enumerate(need):
        pt[i, :c] = perm[at:at + c]
        at += int(c)
    return pt, int(num_pages)


def make_batch(name, L, n, Hq, Hkv, D, seed, P=PAGE, num_pages=None, slack_pages=0, with_data=True,
               q_std=1.0, page_tables=None):
    rng = np.random.default_rng(seed)
    L = np.asarray(L, np.int32)
    n = np.asarray(n, np.int32)
    if page_tables is None:
        page_tables, num_pages = _assign_pages(rng, L, n, P, num_pages, slack_pages)
    b = MixedBatch(name=name, Hq=Hq, Hkv=Hkv, D=D, P=P, num_pages=int(num_pages), scale=1.0 / np.sqrt(D),
                   L=L, n=n, page_tables=page_tables)
    if with_data:
        b.q = normal_bf16(rng, (b.T, Hq, D), q_std)
        tot = int(b.tok_off[-1])
        b.k = normal_bf16(rng, (tot, Hkv, D))
        b.v = normal_bf16(rng, (tot, Hkv, D))
    return b


# ---------------------------------------------------------------------------------------------------
# The five workload configurations.
# ---------------------------------------------------------------------------------------------------

def cfg1_tiny(seed=0, with_data=True, q_std=1.0):
    """4 sequences, 8 q / 2 kv heads, D=64: one full prefill, two decodes, one append-prefill."""
    return make_batch("cfg1_tiny_mixed", L=[0, 37, 100, 256], n=[64, 1, 12, 1], Hq=8, Hkv=2, D=64, seed=seed,
                      num_pages=64, with_data=with_data, q_std=q_std)


def cfg2_decode(seed=0, B=64, Lmin=1024, Lmax=8192, with_data=True, slack_pages=64):
    rng = np.random.default_rng(1000 + seed)
    L = rng.integers(Lmin, Lmax + 1, size=B)
    return make_batch("cfg2_decode_only", L=L, n=np.ones(B, np.int32), Hq=32, Hkv=8, D=128, seed=seed,
                      slack_pages=slack_pages, with_data=with_data)


def lognormal_int(rng, median, sigma, lo, hi, size):
    x = np.exp(np.log(median) + sigma * rng.standard_normal(size))
    return np.clip(np.rint(x), lo, hi).astype(np.int32)


def cfg3_append_prefill(seed=0, B=16, Lmin=2048, Lmax=16384, n_median=200, n_lo=16, n_hi=1024,
                        with_data=True, slack_pages=64):
    """New-token counts log-normal (median 200, sigma 1 in log space, clipped to [16, 1024])."""
    rng = np.random.default_rng(2000 + seed)
    L = rng.integers(Lmin, Lmax + 1, size=B)
    n = lognormal_int(rng, n_median, 1.0, n_lo, n_hi, B)
    return make_batch("cfg3_append_prefill_only", L=L, n=n, Hq=32, Hkv=8, D=128, seed=seed,
                      slack_pages=slack_pages, with_data=with_data)


def cfg4_mixed(seed=0, n_decode=128, n_ap=4, dec_L=(1024, 32768), ap_L=(4096, 32768), ap_n=(256, 2048),
               full_prefill=False, with_ap=True, with_data=True, slack_pages=64):
    """Decode-node mixed batch.  full_prefill=True replaces each append-prefill (L, n) by a full prefill
    (0, L+n) of equal context; with_ap=False keeps the decode sequences only (the slowdown baseline)."""
    rng = np.random.default_rng(3000 + seed)
    Ld = rng.integers(dec_L[0], dec_L[1] + 1, size=n_decode)
    La = rng.integers(ap_L[0], ap_L[1] + 1, size=n_ap)
    na = rng.integers(ap_n[0], ap_n[1] + 1, size=n_ap)
    if full_prefill:
        na = La + na
        La = np.zeros_like(La)
    if with_ap:
        L = np.concatenate([Ld, La])
        n = np.concatenate([np.ones(n_decode, np.int64), na])
    else:
        L, n = Ld, np.ones(n_decode, np.int64)
    tag = "decode_only" if not with_ap else ("full_prefill" if full_prefill else "append_prefill")
    return make_batch("cfg4_mixed_" + tag, L=L, n=n, Hq=32, Hkv=8, D=128, seed=seed, slack_pages=slack_pages,
                      with_data=with_data)


@dataclass
class TraceStep:
    """One engine step of the conversation trace: append `n` tokens per active conversation, then attend."""
    conv: np.ndarray   # [b] conversation ids active in this step
    L: np.ndarray      # [b] cached tokens before the step
    n: np.ndarray      # [b] new tokens (1 = decode, >1 = append-prefill of a new prompt)
    attend: bool       # False for the turn-1 landing of transferred KV (append only)


def cfg5_trace(seed=0, n_conv=256, turns=5, prompt_mean=200.0, response_mean=300.0, sigma=1.0,
               start_spread=300, len_clip=(1, 4096)):
    """Continuous-batching schedule of a multi-turn trace (lengths only; data is drawn per step).

    Conversation c starts at a step drawn from U[0, start_spread).  Turn 1: its prompt's KV lands on the
    node (append only, models KV handed over after a remote prefill), then r_1 decode steps.  Turn t >= 2:
    one step with an append-prefill of the new prompt over everything cached so far, then r_t decode
    steps.  Log-normal lengths with the stated means (mu = ln(mean) - sigma^2/2).
    Returns (steps, max_tokens_per_conversation).
    """
    rng = np.random.default_rng(5000 + seed)
    mu_p = np.log(prompt_mean) - sigma * sigma / 2
    mu_r = np.log(response_mean) - sigma * sigma / 2
    prompts = np.clip(np.rint(np.exp(mu_p + sigma * rng.standard_normal((n_conv, turns)))), *len_clip).astype(np.int64)
    resps = np.clip(np.rint(np.exp(mu_r + sigma * rng.standard_normal((n_conv, turns)))), *len_clip).astype(np.int64)
    start = rng.integers(0, start_spread, size=n_conv)
    # per-conversation event list: (n_new, attend)
    events: List[List] = []
    for c in range(n_conv):
        ev = []
        for t in range(turns):
            ev.append((int(prompts[c, t]), t > 0))
            ev.extend([(1, True)] * int(resps[c, t]))
        events.append(ev)
    cached = np.zeros(n_conv, np.int64)
    cursor = np.zeros(n_conv, np.int64)
    steps: List[TraceStep] = []
    step = 0
    remaining = n_conv
    while remaining > 0:
        ids_att, ids_land = [], []
        for c in range(n_conv):
            if start[c] <= step and cursor[c] < len(events[c]):
                (ids_att if events[c][cursor[c]][1] else ids_land).append(c)
        for ids, att in ((ids_land, False), (ids_att, True)):
            if ids:
                ids = np.asarray(ids)
                nn = np.asarray([events[c][cursor[c]][0] for c in ids], np.int64)
                steps.append(TraceStep(conv=ids, L=cached[ids].copy(), n=nn, attend=att))
                cached[ids] += nn
                cursor[ids] += 1
        remaining = int(np.sum(cursor < np.asarray([len(e) for e in events])))
        step += 1
    max_tokens = (prompts.sum(1) + resps.sum(1)).astype(np.int64)
    return steps, max_tokens


# ---------------------------------------------------------------------------------------------------
# Full-size workloads: the data is drawn on the GPU (torch is used for device memory only).  The pool is
# filled with iid N(0,1) bf16 in place -- iid values are iid in any layout, so no layout arithmetic is
# needed here -- and the new tokens' K/V go in through the library's own append.
# ---------------------------------------------------------------------------------------------------

def new_token_slots(b):
    return b.new_part()[2]


FP8_BENCH_SCALE = 2.0 ** -5  # K and V scale of the FP8 workloads: N(0,1) values / scale stay far below 448


def device_workload(b, torch, device, seed=0, fp8=False):
    """Device tensors of a shapes-only batch b (made with with_data=False).  fp8: the resident pool holds one-byte
    FP8 E4M3 codes instead of bf16 values -- the codes of N(0,1) / FP8_BENCH_SCALE numbers through the tensor
    library's own cast (resident data only: any valid code would do; the new tokens still arrive as bf16)."""
    gen = torch.Generator(device=device)
    gen.manual_seed(10_000 + seed)
    page_elems = 2 * b.Hkv * b.P * b.D
    step = 1 << 28
    if fp8:
        pool = torch.empty((b.num_pages * page_elems,), dtype=torch.uint8, device=device)
        for a in range(0, pool.numel(), step):
            e = min(a + step, pool.numel())
            x = torch.empty((e - a,), dtype=torch.float32, device=device).normal_(generator=gen)
            pool[a:e] = (x / FP8_BENCH_SCALE).clamp_(-448.0, 448.0).to(torch.float8_e4m3fn).view(torch.uint8)
            del x
    else:
        pool = torch.empty((b.num_pages * page_elems,), dtype=torch.bfloat16, device=device)
        for a in range(0, pool.numel(), step):
            pool[a:a + step].normal_(generator=gen)
    q = torch.empty((b.T, b.Hq, b.D), dtype=torch.bfloat16, device=device).normal_(generator=gen)
    k_new = torch.empty((b.T, b.Hkv, b.D), dtype=torch.bfloat16, device=device).normal_(generator=gen)
    v_new = torch.empty((b.T, b.Hkv, b.D), dtype=torch.bfloat16, device=device).normal_(generator=gen)
    return dict(pool=pool, q=q, k_new=k_new, v_new=v_new,
                slots=torch.from_numpy(new_token_slots(b)).to(device),
                page_tables=torch.from_numpy(b.page_tables).to(device),
                out=torch.zeros((b.T, b.Hq, b.D), dtype=torch.bfloat16, device=device))


def compact_subbatch(b, seq_ids, pool_dev, q_dev, torch):
    """Host copy of the pages of the sequences seq_ids only, with page ids renumbered 0..k-1, as a
    MixedBatch carrying q but no dense K/V (the pool bytes are the data).  Returns (sub_batch, pool_u16)."""
    seq_ids = [int(s) for s in seq_ids]
    page_elems = 2 * b.Hkv * b.P * b.D
    pts, pages = [], []
    at = 0
    need = (b.L.astype(np.int64) + b.n + b.P - 1) // b.P
    for s in seq_ids:
        c = int(need[s])
        pages.append(b.page_tables[s, :c].astype(np.int64))
        pts.append(np.arange(at, at + c, dtype=np.int32))
        at += c
    maxp = max(len(p) for p in pts)
    pt = np.full((len(seq_ids), maxp), -1, np.int32)
    for i, p in enumerate(pts):
        pt[i, :len(p)] = p
    idx = torch.from_numpy(np.concatenate(pages)).to(pool_dev.device)
    if pool_dev.dtype == torch.uint8:   # FP8 pages: one-byte codes
        sub_pool8 = pool_dev.view(b.num_pages, page_elems).index_select(0, idx).cpu().numpy().reshape(-1)
    else:
        sub_pool8 = None
        sub_pool = pool_dev.view(torch.int16).view(b.num_pages, page_elems).index_select(0, idx).cpu().numpy()
    rows = np.concatenate([np.arange(b.row_off[s], b.row_off[s + 1]) for s in seq_ids])
    q = q_dev.view(torch.int16)[torch.from_numpy(rows).to(q_dev.device)].cpu().numpy().view(np.uint16)
    sub = MixedBatch(name=b.name + "_sub", Hq=b.Hq, Hkv=b.Hkv, D=b.D, P=b.P, num_pages=at, scale=b.scale,
                     L=b.L[seq_ids], n=b.n[seq_ids], page_tables=pt, q=q)
    if sub_pool8 is not None:
        return sub, sub_pool8, rows
    return sub, sub_pool.view(np.uint16).reshape(-1), rows
