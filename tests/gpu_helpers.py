"""GPU-side test plumbing: torch is used for device memory and streams only."""
import numpy as np

from helpers import SENTINEL


def to_dev_u16(a, torch, dev):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(dev)


def from_dev_u16(t):
    return t.cpu().numpy().view(np.uint16)


def gpu_step(b, options=None, fill=SENTINEL, append_in_one_call=False, return_ctx=False):
    """Runs the whole step for batch b through the C ABI: append the cached prefix (stands for earlier
    steps), append the new tokens, mixed attention.  Returns (pool bits, out bits, plan stats dict)."""
    import torch
    import paper_2603_13358_amd as ppd

    dev = torch.device("cuda:0")
    ctx = ppd.Context(b.Hq, b.Hkv, b.D, b.num_pages)
    for k_, v_ in (options or {}).items():
        ctx.set_option(k_, v_)
    fill_signed = int(np.array([fill], np.uint16).view(np.int16)[0])
    pool = torch.full((ctx.pool_elems(),), fill_signed, dtype=torch.int16, device=dev)
    parts = [b.cached_part(), b.new_part()]
    if append_in_one_call:
        parts = [tuple(np.concatenate([p[i] for p in parts]) for i in range(3))]
    for k, v, slots in parts:
        if len(slots) == 0:
            continue
        ctx.kv_append(to_dev_u16(k, torch, dev), to_dev_u16(v, torch, dev), pool,
                      torch.from_numpy(slots.astype(np.int64)).to(dev))
    q = to_dev_u16(b.q, torch, dev)
    out = torch.full((b.T, b.Hq, b.D), fill_signed, dtype=torch.int16, device=dev)
    pt = torch.from_numpy(b.page_tables).to(dev)
    ctx.mixed_attention(q, pool, pt, b.L, b.n, b.scale, out)
    torch.cuda.synchronize()
    flags = ctx.device_error_flags()
    assert flags == 0, "device error flags %d" % flags
    stats = ctx.plan_stats().as_dict()
    res = (from_dev_u16(pool), from_dev_u16(out).reshape(b.T, b.Hq, b.D), stats)
    if return_ctx:
        return res + (ctx,)
    ctx.close()
    return res


NAN_CODE = 0x7F  # the FP8 E4M3 NaN code: what never-written bytes of an FP8 pool hold in the tests


def gpu_step_fp8(b, k_scale, v_scale, options=None, static=False):
    """The same step on FP8 pages (one-byte codes, one scale per tensor).  Returns (pool codes, out bits, stats)."""
    import torch
    import paper_2603_13358_amd as ppd

    dev = torch.device("cuda:0")
    ctx = ppd.Context(b.Hq, b.Hkv, b.D, b.num_pages)
    ctx.set_kv_format(ppd.PPD_KV_FP8_E4M3, k_scale, v_scale)
    for k_, v_ in (options or {}).items():
        ctx.set_option(k_, v_)
    pool = torch.full((ctx.pool_elems(),), NAN_CODE, dtype=torch.uint8, device=dev)
    for k, v, slots in (b.cached_part(), b.new_part()):
        if len(slots) == 0:
            continue
        ctx.kv_append(to_dev_u16(k, torch, dev), to_dev_u16(v, torch, dev), pool,
                      torch.from_numpy(slots.astype(np.int64)).to(dev))
    q = to_dev_u16(b.q, torch, dev)
    fill_signed = int(np.array([SENTINEL], np.uint16).view(np.int16)[0])
    out = torch.full((b.T, b.Hq, b.D), fill_signed, dtype=torch.int16, device=dev)
    pt = torch.from_numpy(b.page_tables).to(dev)
    (ctx.mixed_attention_static if static else ctx.mixed_attention)(q, pool, pt, b.L, b.n, b.scale, out)
    torch.cuda.synchronize()
    flags = ctx.device_error_flags()
    assert flags == 0, "device error flags %d" % flags
    stats = ctx.plan_stats().as_dict()
    res = (pool.cpu().numpy(), from_dev_u16(out).reshape(b.T, b.Hq, b.D), stats)
    ctx.close()
    return res
