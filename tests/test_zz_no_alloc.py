"""The entry point that allocates nothing (ppd_mixed_attention_static) against ppd_mixed_attention: same kernels, the
work list, merge tables, split partials and queue counters in the library's static device array instead of the
context's workspace.  Two calls in a row, the second with a smaller batch; device memory in use must not move."""
import numpy as np
import pytest

import synthetic_inputs as si
from helpers import bits_to_f32, check_close, oracle_out, oracle_pool

pytestmark = pytest.mark.gpu


def _inputs(b, torch, dev):
    from gpu_helpers import to_dev_u16
    pool = to_dev_u16(oracle_pool(b), torch, dev)          # both entry points read the same, oracle-built pool
    q = to_dev_u16(b.q, torch, dev)
    pt = torch.from_numpy(b.page_tables).to(dev)
    return pool, q, pt


def test_static_entry_point_matches_the_allocating_one_twice():
    import torch
    import paper_2603_13358_amd as ppd
    from gpu_helpers import from_dev_u16
    dev = torch.device("cuda:0")
    big = si.make_batch("noalloc_big", L=[900, 0, 2500, 333, 64, 4000, 1500, 7000], n=[1, 150, 70, 2, 3, 1, 300, 1],
                        Hq=32, Hkv=8, D=128, seed=71, slack_pages=3)
    small = si.make_batch("noalloc_small", L=[700, 100, 0], n=[1, 40, 33], Hq=32, Hkv=8, D=128, seed=72,
                          slack_pages=2)
    ctx_ref = ppd.Context(32, 8, 128, max(big.num_pages, small.num_pages))
    ctx = ppd.Context(32, 8, 128, max(big.num_pages, small.num_pages))
    for c in (ctx_ref, ctx):                              # split key ranges: partials and the merge are in play
        c.set_option("narrow_chunk", 512)
        c.set_option("mfma_chunk", 512)
    prepared = []
    for b in (big, small):
        pool, q, pt = _inputs(b, torch, dev)
        out_ref = torch.full((b.T, b.Hq, b.D), 7, dtype=torch.int16, device=dev)
        out = torch.full((b.T, b.Hq, b.D), 9, dtype=torch.int16, device=dev)
        prepared.append((b, pool, q, pt, out_ref, out))
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    for name, (b, pool, q, pt, out_ref, out) in zip(("big", "small"), prepared):
        print("static call on batch", name, "B", b.B, "T", b.T, flush=True)
        ctx.mixed_attention_static(q, pool, pt, b.L, b.n, b.scale, out)
        torch.cuda.synchronize()
        assert ctx.plan_stats().n_groups > 0
    free_after, _ = torch.cuda.mem_get_info()
    assert free_after == free_before, "device memory moved across the calls that must not allocate"
    for name, (b, pool, q, pt, out_ref, out) in zip(("big", "small"), prepared):
        ctx_ref.mixed_attention(q, pool, pt, b.L, b.n, b.scale, out_ref)
        torch.cuda.synchronize()
    # the static calls ran before the reference calls; run them once more, in the same order, and compare each
    for name, (b, pool, q, pt, out_ref, out) in zip(("big", "small"), prepared):
        first = out.clone()
        out.fill_(5)
        ctx.mixed_attention_static(q, pool, pt, b.L, b.n, b.scale, out)
        torch.cuda.synchronize()
        assert torch.equal(out, first), "static entry point is not deterministic on batch " + name
        assert torch.equal(out, out_ref), "static and allocating entry points differ on batch " + name
        got = bits_to_f32(from_dev_u16(out).reshape(b.T, b.Hq, b.D))
        check_close(got, oracle_out(b))
    assert ctx.device_error_flags() == 0 and ctx_ref.device_error_flags() == 0
    ctx.close()
    ctx_ref.close()


def test_static_entry_point_refuses_what_does_not_fit():
    import torch
    import paper_2603_13358_amd as ppd
    dev = torch.device("cuda:0")
    # 64 append-prefills of 1024 rows, key ranges cut into 512-token pieces: far more split partials than the array holds
    b = si.make_batch("noalloc_too_big", L=[8192] * 64, n=[1024] * 64, Hq=32, Hkv=8, D=128, seed=73, slack_pages=2,
                      with_data=False)
    ctx = ppd.Context(b.Hq, b.Hkv, b.D, b.num_pages)
    ctx.set_option("mfma_chunk", 512)
    dummy = torch.zeros(64, dtype=torch.int16, device=dev)          # never dereferenced: the call must fail on the host
    pt = torch.from_numpy(b.page_tables).to(dev)
    with pytest.raises(ppd.PPDError) as e:
        ctx.mixed_attention_static(dummy, dummy, pt, b.L, b.n, b.scale, dummy)
    assert e.value.status == -5 and "static scratch" in str(e.value)
    torch.cuda.synchronize()
    assert ctx.device_error_flags() == 0
    ctx.close()
