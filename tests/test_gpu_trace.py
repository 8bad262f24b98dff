"""Multi-turn trace on the GPU against the oracle, step by step on one persistent page pool: turn-1 KV
landing (append only), decode steps, turn-2+ append-prefill over everything cached so far."""
import numpy as np
import pytest

import oracle
import synthetic_inputs as si
from helpers import SENTINEL, bits_to_f32, check_close

pytestmark = pytest.mark.gpu


def test_short_trace_matches_oracle_every_step():
    import torch
    import paper_2603_13358_amd as ppd
    from gpu_helpers import from_dev_u16, to_dev_u16

    Hq, Hkv, D, P = 16, 2, 128, 16
    steps, max_tokens = si.cfg5_trace(seed=3, n_conv=6, turns=3, prompt_mean=40.0, response_mean=6.0, sigma=0.8,
                                      start_spread=4, len_clip=(1, 200))
    rng = np.random.default_rng(77)
    need = (max_tokens + P - 1) // P
    num_pages = int(need.sum()) + 5
    perm = rng.permutation(num_pages).astype(np.int32)
    pt = np.full((6, int(need.max())), -1, np.int32)
    at = 0
    for c in range(6):
        pt[c, :need[c]] = perm[at:at + need[c]]
        at += int(need[c])
    dev = torch.device("cuda:0")
    ctx = ppd.Context(Hq, Hkv, D, num_pages)
    fill = int(np.array([SENTINEL], np.uint16).view(np.int16)[0])
    pool_d = torch.full((ctx.pool_elems(),), fill, dtype=torch.int16, device=dev)
    pool_h = np.full(ctx.pool_elems(), SENTINEL, np.uint16)
    scale = 1.0 / np.sqrt(D)
    n_att = 0
    for si_, st in enumerate(steps):
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
        ref = oracle.mixed_attention(q, pool_h, sub_pt, st.L, st.n, Hq, Hkv, D, P, num_pages, scale)
        check_close(bits_to_f32(from_dev_u16(out).reshape(T, Hq, D)), ref)
        n_att += 1
    assert ctx.device_error_flags() == 0
    assert np.array_equal(from_dev_u16(pool_d), pool_h), "pools diverged over the trace"
    assert n_att > 10
    ctx.close()
