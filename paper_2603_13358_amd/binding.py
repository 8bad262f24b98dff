"""ctypes binding of libppd.so: argument marshalling only."""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libppd.so")
_lib = None

STATUS_NAMES = {0: "PPD_OK", -1: "PPD_ERR_NULL", -2: "PPD_ERR_SHAPE", -3: "PPD_ERR_RANGE",
                -4: "PPD_ERR_PAGETABLE", -5: "PPD_ERR_WORKSPACE", -6: "PPD_ERR_HIP"}


class PPDError(RuntimeError):
    def __init__(self, status, message=""):
        self.status = int(status)
        super().__init__("%s: %s" % (STATUS_NAMES.get(self.status, str(status)), message))


class Shape(ctypes.Structure):
    _fields_ = [("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("page_size", ctypes.c_int32), ("num_pages", ctypes.c_int64)]


class WorkItem(ctypes.Structure):
    _fields_ = [(name, ctypes.c_int32) for name in
                ("kind", "seq", "kvh", "row0", "nrows", "grow0", "L", "kv_total", "kv_begin", "kv_end", "group",
                 "queue")] + [("part_off", ctypes.c_int64)]


class PlanStats(ctypes.Structure):
    _fields_ = [("n_items", ctypes.c_int64), ("n_narrow", ctypes.c_int64), ("n_mfma", ctypes.c_int64),
                ("n_groups", ctypes.c_int64), ("partial_floats", ctypes.c_int64), ("kv_bytes", ctypes.c_int64),
                ("kv_bytes_tiles", ctypes.c_int64), ("flops", ctypes.c_double), ("narrow_chunk", ctypes.c_int32),
                ("mfma_chunk", ctypes.c_int32), ("grid", ctypes.c_int32), ("plan_host_us", ctypes.c_int32)]

    def as_dict(self):
        return {f: getattr(self, f) for f, _ in self._fields_ if f != "reserved"}


EXPORTS = ["ppd_create", "ppd_destroy", "ppd_last_error", "ppd_set_option", "ppd_kv_append", "ppd_kv_land",
           "ppd_transfer_delay_s", "ppd_mixed_attention", "ppd_mixed_attention_static",
           "ppd_get_plan_stats", "ppd_plan_build", "ppd_device_error_flags", "ppd_last_kernel_ms", "ppd_timed_kernels_ms",
           "ppd_route_score", "ppd_route_table_build", "ppd_route_cell", "ppd_route_decide", "ppd_route_decide_batch", "ppd_version"]


def lib_path():
    return _LIB_PATH


def load_library():
    """Loads libppd.so; raises if it has not been built (no fallback of any kind)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libppd.so is not built: run `python -m paper_2603_13358_amd.build` "
                          "(or __graft_entry__.build()); there is no CPU path")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.ppd_create.argtypes = [ctypes.POINTER(Shape), i32, ctypes.POINTER(vp)]
    lib.ppd_destroy.argtypes = [vp]
    lib.ppd_last_error.argtypes = [vp]
    lib.ppd_last_error.restype = ctypes.c_char_p
    lib.ppd_set_option.argtypes = [vp, ctypes.c_char_p, i64]
    lib.ppd_set_kv_format.argtypes = [vp, i32, ctypes.c_float, ctypes.c_float]
    lib.ppd_kv_append.argtypes = [vp, vp, vp, vp, vp, i64, vp]
    lib.ppd_kv_land.argtypes = [vp, vp, vp, vp, i64, i32, vp, i64, vp]
    lib.ppd_transfer_delay_s.argtypes = [i64, i64, ctypes.c_double, ctypes.c_double]
    lib.ppd_transfer_delay_s.restype = ctypes.c_double
    lib.ppd_mixed_attention.argtypes = [vp, vp, vp, vp, i32, vp, vp, i32, ctypes.c_float, vp, vp]
    lib.ppd_mixed_attention_static.argtypes = lib.ppd_mixed_attention.argtypes
    lib.ppd_get_plan_stats.argtypes = [vp, ctypes.POINTER(PlanStats)]
    lib.ppd_plan_build.argtypes = [ctypes.POINTER(Shape), vp, vp, i32, i32, i32, i32, i32, i32,
                                   ctypes.POINTER(WorkItem), i64, ctypes.POINTER(PlanStats)]
    lib.ppd_device_error_flags.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_uint32)]
    lib.ppd_last_kernel_ms.argtypes = [vp, ctypes.POINTER(ctypes.c_float)]
    lib.ppd_timed_kernels_ms.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)]
    dbl = ctypes.c_double
    lib.ppd_route_score.argtypes = [dbl, dbl, dbl, dbl]
    lib.ppd_route_score.restype = dbl
    lib.ppd_route_table_build.argtypes = [vp, vp, dbl, dbl, vp]
    lib.ppd_route_cell.argtypes = [vp, i64, i64, i64, dbl]
    lib.ppd_route_decide.argtypes = [vp, vp, i32, i64, i64, i64, dbl]
    lib.ppd_route_decide_batch.argtypes = [vp, vp, i64, vp, vp, vp, vp, vp, vp]
    lib.ppd_version.argtypes = []
    lib.ppd_version.restype = ctypes.c_char_p
    for name in EXPORTS:
        if name not in ("ppd_last_error", "ppd_version", "ppd_transfer_delay_s", "ppd_route_score"):
            getattr(lib, name).restype = i32
    _lib = lib
    return lib


def _dev_ptr(x):
    """Device address of a torch tensor (or an int that already is one)."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _host_i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _check(status, ctx=None):
    if status != 0:
        raise PPDError(status, ppd_last_error(ctx))


def ppd_version():
    return load_library().ppd_version().decode()


def ppd_last_error(ctx=None):
    return load_library().ppd_last_error(ctx).decode()


def ppd_create(num_q_heads, num_kv_heads, head_dim, page_size, num_pages, device=0):
    shape = Shape(num_q_heads, num_kv_heads, head_dim, page_size, num_pages)
    handle = ctypes.c_void_p()
    _check(load_library().ppd_create(ctypes.byref(shape), device, ctypes.byref(handle)))
    return handle


def ppd_destroy(ctx):
    _check(load_library().ppd_destroy(ctx))


def ppd_set_option(ctx, key, value):
    _check(load_library().ppd_set_option(ctx, key.encode(), int(value)), ctx)


PPD_KV_BF16, PPD_KV_FP8_E4M3 = 0, 1


def ppd_set_kv_format(ctx, fmt, k_scale=1.0, v_scale=1.0):
    _check(load_library().ppd_set_kv_format(ctx, int(fmt), float(k_scale), float(v_scale)), ctx)


def ppd_kv_append(ctx, k, v, kv_pages, slot_mapping, T=None, stream=None):
    if T is None:
        T = int(slot_mapping.shape[0])
    _check(load_library().ppd_kv_append(ctx, _dev_ptr(k), _dev_ptr(v), _dev_ptr(kv_pages), _dev_ptr(slot_mapping),
                                        int(T), stream), ctx)


def ppd_kv_land(ctx, k, v, kv_pages, layer_stride_elems, num_layers, slot_mapping, T=None, stream=None):
    if T is None:
        T = int(slot_mapping.shape[0])
    _check(load_library().ppd_kv_land(ctx, _dev_ptr(k), _dev_ptr(v), _dev_ptr(kv_pages), int(layer_stride_elems),
                                      int(num_layers), _dev_ptr(slot_mapping), int(T), stream), ctx)


def ppd_transfer_delay_s(n_tokens, kv_bytes_per_token, beta_target_bytes_per_s, t_fast_s):
    return float(load_library().ppd_transfer_delay_s(int(n_tokens), int(kv_bytes_per_token),
                                                     float(beta_target_bytes_per_s), float(t_fast_s)))


def ppd_mixed_attention(ctx, q, kv_pages, page_tables, L, n, scale, out, max_pages=None, stream=None, static=False):
    L = _host_i32(L)
    n = _host_i32(n)
    if max_pages is None:
        max_pages = int(page_tables.shape[1])
    lib = load_library()
    fn = lib.ppd_mixed_attention_static if static else lib.ppd_mixed_attention
    _check(fn(ctx, _dev_ptr(q), _dev_ptr(kv_pages), _dev_ptr(page_tables), int(max_pages), L.ctypes.data,
              n.ctypes.data, int(L.shape[0]), float(scale), _dev_ptr(out), stream), ctx)


def ppd_mixed_attention_static(ctx, q, kv_pages, page_tables, L, n, scale, out, max_pages=None, stream=None):
    ppd_mixed_attention(ctx, q, kv_pages, page_tables, L, n, scale, out, max_pages=max_pages, stream=stream,
                        static=True)


def ppd_get_plan_stats(ctx):
    st = PlanStats()
    _check(load_library().ppd_get_plan_stats(ctx, ctypes.byref(st)), ctx)
    return st


def ppd_device_error_flags(ctx, stream=None):
    flags = ctypes.c_uint32(0)
    _check(load_library().ppd_device_error_flags(ctx, stream, ctypes.byref(flags)), ctx)
    return int(flags.value)


def ppd_last_kernel_ms(ctx):
    ms = ctypes.c_float(0)
    _check(load_library().ppd_last_kernel_ms(ctx, ctypes.byref(ms)), ctx)
    return float(ms.value)


def ppd_timed_kernels_ms(ctx):
    """(sum of the mixed kernel's durations in ms, number of launches) since timing was switched on / last asked."""
    total = ctypes.c_double(0)
    count = ctypes.c_int32(0)
    _check(load_library().ppd_timed_kernels_ms(ctx, ctypes.byref(total), ctypes.byref(count)), ctx)
    return float(total.value), int(count.value)


ROUTE_CELLS = 3 * 9 * 10


def ppd_route_score(w_ttft, w_tpot, delta_ttft, delta_tpot):
    return float(load_library().ppd_route_score(w_ttft, w_tpot, delta_ttft, delta_tpot))


def ppd_route_table_build(delta_ttft, delta_tpot, w_ttft, w_tpot):
    """Returns the uint8 [270] decision table for per-cell measured deltas (float64 [270] each)."""
    a = np.ascontiguousarray(delta_ttft, dtype=np.float64).reshape(-1)
    b = np.ascontiguousarray(delta_tpot, dtype=np.float64).reshape(-1)
    assert a.size == ROUTE_CELLS and b.size == ROUTE_CELLS
    table = np.zeros(ROUTE_CELLS, np.uint8)
    status = load_library().ppd_route_table_build(a.ctypes.data, b.ctypes.data, float(w_ttft), float(w_tpot),
                                                  table.ctypes.data)
    if status != 0:
        raise PPDError(status, "ppd_route_table_build")
    return table


def ppd_route_cell(ratio_centers, n_in, n_out, n_ctx, qps):
    c = np.ascontiguousarray(ratio_centers, dtype=np.float64)
    assert c.size == 9
    return int(load_library().ppd_route_cell(c.ctypes.data, int(n_in), int(n_out), int(n_ctx), float(qps)))


def ppd_route_decide(x_table, ratio_centers, turn, n_in, n_out, n_ctx, qps):
    t = np.ascontiguousarray(x_table, dtype=np.uint8)
    c = np.ascontiguousarray(ratio_centers, dtype=np.float64)
    assert t.size == ROUTE_CELLS and c.size == 9
    return int(load_library().ppd_route_decide(t.ctypes.data, c.ctypes.data, int(turn), int(n_in), int(n_out),
                                               int(n_ctx), float(qps)))


def ppd_route_decide_batch(x_table, ratio_centers, turn, n_in, n_out, n_ctx, qps):
    """Online decisions for arrays of requests in one call; returns int8 [count]."""
    t = np.ascontiguousarray(x_table, dtype=np.uint8)
    c = np.ascontiguousarray(ratio_centers, dtype=np.float64)
    assert t.size == ROUTE_CELLS and c.size == 9
    turn = np.ascontiguousarray(turn, dtype=np.int32)
    a, b, d = (np.ascontiguousarray(x, dtype=np.int64) for x in (n_in, n_out, n_ctx))
    qps = np.ascontiguousarray(qps, dtype=np.float64)
    count = turn.size
    assert a.size == count and b.size == count and d.size == count and qps.size == count
    out = np.empty(count, np.int8)
    status = load_library().ppd_route_decide_batch(t.ctypes.data, c.ctypes.data, count, turn.ctypes.data, a.ctypes.data,
                                                   b.ctypes.data, d.ctypes.data, qps.ctypes.data, out.ctypes.data)
    if status != 0:
        raise PPDError(status, "ppd_route_decide_batch")
    return out


def ppd_plan_build(num_q_heads, num_kv_heads, head_dim, page_size, num_pages, L, n, narrow_chunk=0, mfma_chunk=0,
                   grid=0, force_kind=-1, num_cus=256):
    """Host-only planner.  Returns (list of WorkItem, PlanStats)."""
    lib = load_library()
    shape = Shape(num_q_heads, num_kv_heads, head_dim, page_size, num_pages)
    L = _host_i32(L)
    n = _host_i32(n)
    st = PlanStats()
    args = (ctypes.byref(shape), L.ctypes.data, n.ctypes.data, int(L.shape[0]), narrow_chunk, mfma_chunk, grid,
            force_kind, num_cus)
    status = lib.ppd_plan_build(*args, None, 0, ctypes.byref(st))
    if status != 0:
        raise PPDError(status, "ppd_plan_build")
    items = (WorkItem * max(1, st.n_items))()
    status = lib.ppd_plan_build(*args, items, st.n_items, ctypes.byref(st))
    if status != 0:
        raise PPDError(status, "ppd_plan_build")
    return [items[i] for i in range(st.n_items)], st


class Context:
    """Owns one ppd_ctx handle (created on the current torch device's index)."""

    def __init__(self, num_q_heads, num_kv_heads, head_dim, num_pages, page_size=16, device=0):
        self.shape = (num_q_heads, num_kv_heads, head_dim, page_size, num_pages)
        self.handle = ppd_create(num_q_heads, num_kv_heads, head_dim, page_size, num_pages, device)

    def pool_elems(self):
        Hq, Hkv, D, P, N = self.shape
        return N * 2 * Hkv * P * D

    def set_option(self, key, value):
        ppd_set_option(self.handle, key, value)

    def set_kv_format(self, fmt, k_scale=1.0, v_scale=1.0):
        ppd_set_kv_format(self.handle, fmt, k_scale, v_scale)

    def kv_append(self, k, v, kv_pages, slot_mapping, stream=None):
        ppd_kv_append(self.handle, k, v, kv_pages, slot_mapping, stream=stream)

    def kv_land(self, k, v, kv_pages, layer_stride_elems, num_layers, slot_mapping, stream=None):
        ppd_kv_land(self.handle, k, v, kv_pages, layer_stride_elems, num_layers, slot_mapping, stream=stream)

    def mixed_attention(self, q, kv_pages, page_tables, L, n, scale, out, stream=None):
        ppd_mixed_attention(self.handle, q, kv_pages, page_tables, L, n, scale, out, stream=stream)

    def mixed_attention_static(self, q, kv_pages, page_tables, L, n, scale, out, stream=None):
        ppd_mixed_attention_static(self.handle, q, kv_pages, page_tables, L, n, scale, out, stream=stream)

    def plan_stats(self):
        return ppd_get_plan_stats(self.handle)

    def last_kernel_ms(self):
        return ppd_last_kernel_ms(self.handle)

    def timed_kernels_ms(self):
        return ppd_timed_kernels_ms(self.handle)

    def device_error_flags(self, stream=None):
        return ppd_device_error_flags(self.handle, stream)

    def close(self):
        if self.handle is not None:
            ppd_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
