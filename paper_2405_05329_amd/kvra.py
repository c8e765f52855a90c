"""ctypes binding of libkvra: the same entry points as include/kvra.h, argument marshalling only.

Tensor arguments may be torch tensors (their data_ptr() is passed; they must live on the GPU and
be contiguous) or plain integer device addresses.  Every step of the path runs inside the library's
HIP kernels; there is no Python or CPU fallback: if the shared library is missing, importing this
module raises.
"""
from __future__ import annotations

import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libkvra.so")

KVRA_OK = 0
KVRA_EINVAL = -1
KVRA_EUNSUPPORTED = -2
KVRA_ERANGE = -3
KVRA_ELAUNCH = -4
KVRA_ENODEVICE = -5
KVRA_ESCRATCH = -6

COST_FN = ctypes.CFUNCTYPE(ctypes.c_double, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p)


class KvraError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {kvra_strerror(code)} ({code})")


class KvraAttnPlan(ctypes.Structure):
    """Mirror of `kvra_attn_plan` in include/kvra.h."""
    _fields_ = [("row_tiles", ctypes.c_int), ("rows_per_tile", ctypes.c_int), ("key_tile", ctypes.c_int),
                ("groups", ctypes.c_int), ("slots", ctypes.c_int), ("units", ctypes.c_int),
                ("rounds", ctypes.c_int), ("head_steps", ctypes.c_int), ("cut_units", ctypes.c_int),
                ("segments", ctypes.c_int),
                ("steps_per_slot", ctypes.c_int), ("partial_pieces", ctypes.c_int),
                ("gangs", ctypes.c_int), ("gang_heads", ctypes.c_int),
                ("scratch_bytes", ctypes.c_int64)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2405_05329_amd.build` "
            "(there is no fallback path)")
    # torch owns the device memory and streams handed to the library, so both must talk to ONE HIP
    # runtime: torch ships its own libamdhip64 (same soname as ROCm's) and must be loaded first,
    # otherwise the process ends up with two runtimes that do not know each other's allocations.
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    i64, i32, f32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_float, ctypes.c_void_p
    lib.kvra_strerror.restype = ctypes.c_char_p
    lib.kvra_strerror.argtypes = [i32]
    lib.kvra_version.restype = i32
    lib.kvra_version.argtypes = []
    lib.kvra_append_kv.restype = i32
    lib.kvra_append_kv.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, i32, i32, f32, vp]
    lib.kvra_chunk_attn.restype = i32
    lib.kvra_chunk_attn.argtypes = [vp, vp, vp, i64, i64, i32, i32, i32, f32, vp, vp]
    lib.kvra_chunk_attn_noalloc.restype = i32
    lib.kvra_chunk_attn_noalloc.argtypes = [vp, vp, vp, i64, i64, i32, i32, i32, f32, vp, vp]
    lib.kvra_chunk_attn_noalloc_scratch_bytes.restype = i64
    lib.kvra_chunk_attn_noalloc_scratch_bytes.argtypes = []
    lib.kvra_chunk_attn_plan.restype = i32
    lib.kvra_chunk_attn_plan.argtypes = [i64, i64, i32, i32, i32, i32, ctypes.POINTER(KvraAttnPlan)]
    lib.kvra_chunk_attn_pieces.restype = i32
    lib.kvra_chunk_attn_pieces.argtypes = [i64, i64, i32, i32, i32, i32, ctypes.POINTER(ctypes.c_int32), i64,
                                           ctypes.POINTER(i64)]
    lib.kvra_balance.restype = i32
    lib.kvra_balance.argtypes = [i64, i32, i64, ctypes.c_void_p, vp, ctypes.POINTER(i64), ctypes.POINTER(ctypes.c_double)]
    lib.kvra_equal_split.restype = i32
    lib.kvra_equal_split.argtypes = [i64, i32, i64, ctypes.POINTER(i64)]
    lib.kvra_chain_ttft.restype = i32
    lib.kvra_chain_ttft.argtypes = [ctypes.POINTER(i64), i32, i32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                    vp, ctypes.POINTER(ctypes.c_double)]
    lib.kvra_makespan.restype = i32
    lib.kvra_makespan.argtypes = [ctypes.POINTER(i64), i32, ctypes.c_void_p, vp, ctypes.POINTER(ctypes.c_double)]
    pi64, pf64 = ctypes.POINTER(i64), ctypes.POINTER(ctypes.c_double)
    lib.kvra_search_two_way.restype = i32
    lib.kvra_search_two_way.argtypes = [i64, i64, ctypes.c_void_p, vp, pi64, pf64, pi64]
    lib.kvra_search_grid.restype = i32
    lib.kvra_search_grid.argtypes = [i64, i32, i64, pi64, ctypes.c_void_p, vp, pi64, pf64, pi64]
    lib.kvra_search_grid_objective.restype = i32
    lib.kvra_search_grid_objective.argtypes = [i64, i32, i64, pi64, ctypes.c_void_p, vp, pi64, pf64, pi64]
    lib.kvra_interpolate.restype = i32
    lib.kvra_interpolate.argtypes = [i64, i32, i64, i64, pi64, i64, pi64, pi64]
    lib.kvra_table_predict.restype = i32
    lib.kvra_table_predict.argtypes = [i64, i32, i64, i32, pi64, pi64, pi64]
    lib.kvra_rms_norm.restype = i32
    lib.kvra_rms_norm.argtypes = [vp, vp, vp, i64, i32, f32, vp]
    lib.kvra_linear.restype = i32
    lib.kvra_linear.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, vp]
    lib.kvra_qkv_proj.restype = i32
    lib.kvra_qkv_proj.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32, i32, i64, vp]
    lib.kvra_layer_workspace_bytes.restype = i64
    lib.kvra_layer_workspace_bytes.argtypes = [ctypes.POINTER(KvraLayer), i64]
    lib.kvra_layer_chunk.restype = i32
    lib.kvra_layer_chunk.argtypes = [ctypes.POINTER(KvraLayer), vp, vp, vp, vp, i64, i64, i64, vp, i64, vp]
    return lib


class KvraLayer(ctypes.Structure):
    """Mirror of the C struct kvra_layer."""
    _fields_ = [("hidden", ctypes.c_int), ("ffn", ctypes.c_int), ("n_q_heads", ctypes.c_int),
                ("n_kv_heads", ctypes.c_int), ("head_dim", ctypes.c_int),
                ("rms_eps", ctypes.c_float), ("rope_base", ctypes.c_float), ("scale", ctypes.c_float),
                ("norm1", ctypes.c_void_p), ("wqkv", ctypes.c_void_p), ("wo", ctypes.c_void_p),
                ("norm2", ctypes.c_void_p), ("w_gate", ctypes.c_void_p), ("w_up", ctypes.c_void_p),
                ("w_down", ctypes.c_void_p)]


_lib = _load()


def _ptr(x):
    """Device address of a torch tensor (or pass an int / None through)."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if not x.is_contiguous():
        raise ValueError("tensor must be contiguous")
    if not x.is_cuda:
        raise ValueError("tensor must live in GPU memory")
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream     # torch.cuda.Stream


def _cost(cost):
    if cost is None:
        return None, None
    cb = COST_FN(lambda prefix, c, _user: float(cost(prefix, c)))
    return cb, ctypes.cast(cb, ctypes.c_void_p)


def kvra_strerror(code: int) -> str:
    return _lib.kvra_strerror(int(code)).decode()


def kvra_version() -> int:
    return int(_lib.kvra_version())


def kvra_append_kv(k_in, v_in, q_inout, k_cache, v_cache, prefix_len, chunk_len, capacity,
                   n_q_heads, n_kv_heads, head_dim, rope_base, stream=None, check=True) -> int:
    rc = _lib.kvra_append_kv(_ptr(k_in), _ptr(v_in), _ptr(q_inout), _ptr(k_cache), _ptr(v_cache),
                             int(prefix_len), int(chunk_len), int(capacity),
                             int(n_q_heads), int(n_kv_heads), int(head_dim), float(rope_base),
                             _stream(stream))
    if check and rc != KVRA_OK:
        raise KvraError(rc, "kvra_append_kv")
    return rc


def kvra_chunk_attn(q, k_cache, v_cache, prefix_len, chunk_len, n_q_heads, n_kv_heads, head_dim,
                    scale, out, stream=None, check=True) -> int:
    rc = _lib.kvra_chunk_attn(_ptr(q), _ptr(k_cache), _ptr(v_cache), int(prefix_len), int(chunk_len),
                              int(n_q_heads), int(n_kv_heads), int(head_dim), float(scale),
                              _ptr(out), _stream(stream))
    if check and rc != KVRA_OK:
        raise KvraError(rc, "kvra_chunk_attn")
    return rc


def kvra_chunk_attn_noalloc(q, k_cache, v_cache, prefix_len, chunk_len, n_q_heads, n_kv_heads, head_dim,
                            scale, out, stream=None, check=True) -> int:
    rc = _lib.kvra_chunk_attn_noalloc(_ptr(q), _ptr(k_cache), _ptr(v_cache), int(prefix_len), int(chunk_len),
                                      int(n_q_heads), int(n_kv_heads), int(head_dim), float(scale),
                                      _ptr(out), _stream(stream))
    if check and rc != KVRA_OK:
        raise KvraError(rc, "kvra_chunk_attn_noalloc")
    return rc


def kvra_chunk_attn_noalloc_scratch_bytes() -> int:
    return int(_lib.kvra_chunk_attn_noalloc_scratch_bytes())


def kvra_chunk_attn_plan(prefix_len, chunk_len, n_q_heads, n_kv_heads, head_dim, n_cus) -> dict:
    plan = KvraAttnPlan()
    rc = _lib.kvra_chunk_attn_plan(prefix_len, chunk_len, n_q_heads, n_kv_heads, head_dim, n_cus,
                                   ctypes.byref(plan))
    if rc != 0:
        raise KvraError(rc, "kvra_chunk_attn_plan")
    return {name: getattr(plan, name) for name, _ in KvraAttnPlan._fields_}


PIECE_FIELDS = ("workgroup", "kv_head", "row_tile", "jt0", "jt1", "unit_steps", "slot", "merge_pieces",
                "in_merge_list", "counter")


def kvra_chunk_attn_pieces(prefix_len, chunk_len, n_q_heads, n_kv_heads, head_dim, n_cus) -> list:
    """The pieces of the launch plan as a list of dicts with the keys PIECE_FIELDS."""
    count = ctypes.c_int64()
    rc = _lib.kvra_chunk_attn_pieces(prefix_len, chunk_len, n_q_heads, n_kv_heads, head_dim, n_cus, None, 0,
                                     ctypes.byref(count))
    if rc != 0:
        raise KvraError(rc, "kvra_chunk_attn_pieces")
    n = count.value
    buf = (ctypes.c_int32 * (10 * max(n, 1)))()
    rc = _lib.kvra_chunk_attn_pieces(prefix_len, chunk_len, n_q_heads, n_kv_heads, head_dim, n_cus, buf, n,
                                     ctypes.byref(count))
    if rc != 0:
        raise KvraError(rc, "kvra_chunk_attn_pieces")
    return [dict(zip(PIECE_FIELDS, buf[10 * i:10 * i + 10])) for i in range(n)]


def kvra_balance(context_len, n_chunks, granularity, cost=None):
    """Returns (boundaries list, makespan).  cost(prefix_len, chunk_len) -> float, or None for the
    analytic causal-work model."""
    n = int(n_chunks)
    out = (ctypes.c_int64 * (max(n, 0) + 1))()
    mk = ctypes.c_double()
    cb, cbp = _cost(cost)
    rc = _lib.kvra_balance(int(context_len), n, int(granularity), cbp, None, out, ctypes.byref(mk))
    if rc != KVRA_OK:
        raise KvraError(rc, "kvra_balance")
    return list(out), mk.value


def kvra_equal_split(context_len, n_chunks, granularity):
    n = int(n_chunks)
    out = (ctypes.c_int64 * (max(n, 0) + 1))()
    rc = _lib.kvra_equal_split(int(context_len), n, int(granularity), out)
    if rc != KVRA_OK:
        raise KvraError(rc, "kvra_equal_split")
    return list(out)


def kvra_makespan(boundaries, cost=None) -> float:
    b = [int(x) for x in boundaries]
    arr = (ctypes.c_int64 * len(b))(*b)
    mk = ctypes.c_double()
    cb, cbp = _cost(cost)
    rc = _lib.kvra_makespan(arr, len(b) - 1, cbp, None, ctypes.byref(mk))
    if rc != KVRA_OK:
        raise KvraError(rc, "kvra_makespan")
    return mk.value


def kvra_chain_ttft(boundaries, n_layers, before_attn, attn, handoff=None) -> float:
    b = [int(x) for x in boundaries]
    arr = (ctypes.c_int64 * len(b))(*b)
    out = ctypes.c_double()
    cb_a, p_a = _cost(before_attn)
    cb_t, p_t = _cost(attn)
    cb_x, p_x = _cost(handoff)
    rc = _lib.kvra_chain_ttft(arr, len(b) - 1, n_layers, p_a, p_t, p_x, None, ctypes.byref(out))
    if rc != KVRA_OK:
        raise KvraError(rc, "kvra_chain_ttft")
    return out.value


def _i64_array(values):
    v = [int(x) for x in values]
    return (ctypes.c_int64 * len(v))(*v)


def kvra_search_two_way(context_len, granularity, cost=None):
    """Returns (boundaries list of 3, makespan, cost evaluations)."""
    out = (ctypes.c_int64 * 3)()
    mk, ev = ctypes.c_double(), ctypes.c_int64()
    cb, cbp = _cost(cost)
    rc = _lib.kvra_search_two_way(int(context_len), int(granularity), cbp, None, out, ctypes.byref(mk),
                                  ctypes.byref(ev))
    if rc != KVRA_OK:
        raise KvraError(rc, "kvra_search_two_way")
    return list(out), mk.value, ev.value


def kvra_search_grid(context_len, n_chunks, granularity, cost=None, start=None):
    """Returns (boundaries list, makespan, cost evaluations).  start: a partition on the grid, or None
    for the even split."""
    n = int(n_chunks)
    out = (ctypes.c_int64 * (max(n, 0) + 1))()
    mk, ev = ctypes.c_double(), ctypes.c_int64()
    cb, cbp = _cost(cost)
    st = None
    if start is not None:
        if len(start) != n + 1:
            raise KvraError(KVRA_EINVAL, "kvra_search_grid")
        st = _i64_array(start)
    rc = _lib.kvra_search_grid(int(context_len), n, int(granularity), st, cbp, None, out, ctypes.byref(mk),
                               ctypes.byref(ev))
    if rc != KVRA_OK:
        raise KvraError(rc, "kvra_search_grid")
    return list(out), mk.value, ev.value


PARTITION_FN = ctypes.CFUNCTYPE(ctypes.c_double, ctypes.POINTER(ctypes.c_int64), ctypes.c_int, ctypes.c_void_p)


def kvra_search_grid_objective(context_len, n_chunks, granularity, objective, start=None):
    """objective(list of n_chunks + 1 boundaries) -> float.  Returns (boundaries, value, evaluations)."""
    cb = PARTITION_FN(lambda bptr, n, _user: float(objective([bptr[k] for k in range(n + 1)])))
    out = (ctypes.c_int64 * (n_chunks + 1))()
    val = ctypes.c_double()
    ev = ctypes.c_int64()
    st = _i64_array(start) if start is not None else None
    rc = _lib.kvra_search_grid_objective(context_len, n_chunks, granularity, st, ctypes.cast(cb, ctypes.c_void_p), None,
                                         out, ctypes.byref(val), ctypes.byref(ev))
    if rc != KVRA_OK:
        raise KvraError(rc, "kvra_search_grid_objective")
    return list(out), val.value, ev.value


def kvra_interpolate(context_len, granularity, len_lo, bounds_lo, len_hi, bounds_hi):
    n = len(bounds_lo) - 1
    if n < 1 or len(bounds_hi) != n + 1:
        raise KvraError(KVRA_EINVAL, "kvra_interpolate")
    out = (ctypes.c_int64 * (n + 1))()
    rc = _lib.kvra_interpolate(int(context_len), n, int(granularity), int(len_lo), _i64_array(bounds_lo),
                               int(len_hi), _i64_array(bounds_hi), out)
    if rc != KVRA_OK:
        raise KvraError(rc, "kvra_interpolate")
    return list(out)


def kvra_table_predict(context_len, granularity, table):
    """table: {context length: boundaries}; all entries with the same number of chunks."""
    lens = list(table)
    if not lens:
        raise KvraError(KVRA_EINVAL, "kvra_table_predict")
    n = len(table[lens[0]]) - 1
    flat = []
    for length in lens:
        if len(table[length]) != n + 1:
            raise KvraError(KVRA_EINVAL, "kvra_table_predict")
        flat.extend(table[length])
    out = (ctypes.c_int64 * (n + 1))()
    rc = _lib.kvra_table_predict(int(context_len), n, int(granularity), len(lens), _i64_array(lens),
                                 _i64_array(flat), out)
    if rc != KVRA_OK:
        raise KvraError(rc, "kvra_table_predict")
    return list(out)


def kvra_rms_norm(x, gain, y, rows, hidden, eps, stream=None):
    rc = _lib.kvra_rms_norm(_ptr(x), _ptr(gain), _ptr(y), int(rows), int(hidden), float(eps), _stream(stream))
    if rc != KVRA_OK:
        raise KvraError(rc, "kvra_rms_norm")


def kvra_linear(x, w, w2, residual, out, m, n, k, stream=None):
    rc = _lib.kvra_linear(_ptr(x), _ptr(w), _ptr(w2), _ptr(residual), _ptr(out), int(m), int(n), int(k),
                          _stream(stream))
    if rc != KVRA_OK:
        raise KvraError(rc, "kvra_linear")


def kvra_qkv_proj(x, wqkv, q_out, k_out, v_out, m, n_q_heads, n_kv_heads, head_dim, k, stream=None):
    rc = _lib.kvra_qkv_proj(_ptr(x), _ptr(wqkv), _ptr(q_out), _ptr(k_out), _ptr(v_out), int(m), int(n_q_heads),
                            int(n_kv_heads), int(head_dim), int(k), _stream(stream))
    if rc != KVRA_OK:
        raise KvraError(rc, "kvra_qkv_proj")


def make_layer(hidden, ffn, n_q_heads, n_kv_heads, head_dim, rms_eps, rope_base, scale,
               norm1, wqkv, wo, norm2, w_gate, w_up, w_down) -> KvraLayer:
    """Fills a kvra_layer from device tensors (or raw pointers); the caller keeps the tensors alive."""
    return KvraLayer(int(hidden), int(ffn), int(n_q_heads), int(n_kv_heads), int(head_dim),
                     float(rms_eps), float(rope_base), float(scale),
                     _ptr(norm1), _ptr(wqkv), _ptr(wo), _ptr(norm2), _ptr(w_gate), _ptr(w_up), _ptr(w_down))


def kvra_layer_workspace_bytes(layer: KvraLayer, chunk_len) -> int:
    n = _lib.kvra_layer_workspace_bytes(ctypes.byref(layer), int(chunk_len))
    if n < 0:
        raise KvraError(KVRA_EINVAL, "kvra_layer_workspace_bytes")
    return n


def kvra_layer_chunk(layer: KvraLayer, x, y, k_cache, v_cache, prefix_len, chunk_len, capacity,
                     workspace, workspace_bytes, stream=None):
    rc = _lib.kvra_layer_chunk(ctypes.byref(layer), _ptr(x), _ptr(y), _ptr(k_cache), _ptr(v_cache),
                               int(prefix_len), int(chunk_len), int(capacity), _ptr(workspace),
                               int(workspace_bytes), _stream(stream))
    if rc != KVRA_OK:
        raise KvraError(rc, "kvra_layer_chunk")
