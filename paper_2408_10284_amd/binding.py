"""ctypes binding of libadapmoe.so: same names as the C entry points, argument
marshalling only.  Tensors are torch tensors (device memory and streams come
from PyTorch-ROCm); every step of the path runs inside the library's kernels.
There is no fallback: if the library is missing or no GPU is usable, calls fail.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libadapmoe.so")

OK, EINVAL, ENOMEM, ENOTREG, ENORES, EHIP, ESTATE = 0, -1, -2, -3, -4, -5, -6
F32, BF16, INT4G64, INT2G64 = 0, 1, 2, 3
EVENT_KINDS = ("HIT", "HIT_PF", "MISS", "BYPASS", "PF_TOUCH", "PF_LOAD", "PF_LAND")
OPT_BATCH_MIN, OPT_BATCH_TWO_TERMS, OPT_FUSED, OPT_DYN_PCT, OPT_GATEUP_BLOCKS, OPT_DOWN_BLOCKS, OPT_BATCH_DIRECT, OPT_POISON_SLOTS = range(8)


class Config(C.Structure):
    _fields_ = [("H", C.c_int32), ("F", C.c_int32), ("N", C.c_int32), ("L", C.c_int32),
                ("dtype", C.c_int32), ("max_B", C.c_int32), ("device", C.c_int32),
                ("trace_capacity", C.c_int32)]


class Event(C.Structure):
    _fields_ = [("token", C.c_int32), ("layer", C.c_int32), ("kind", C.c_int32),
                ("expert", C.c_int32), ("victim", C.c_int32), ("slot", C.c_int32)]


class Counters(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in
                ("tokens_gated", "single_expert", "hits", "hits_after_prefetch", "misses", "bypasses",
                 "prefetch_touches", "prefetch_loads", "h2d_bytes", "ffn_launches", "tiled_ffn", "prefetch_landed")]


class AdapMoEError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"adapmoe error {code}: {text}")
        self.code = code


_lib = None

_P = C.c_void_p
_SIGS = {
    "adapmoe_strerror": (C.c_char_p, [C.c_int]),
    "adapmoe_last_error": (C.c_char_p, [_P]),
    "adapmoe_create": (C.c_int, [C.POINTER(Config), C.POINTER(_P)]),
    "adapmoe_destroy": (C.c_int, [_P]),
    "adapmoe_set_router": (C.c_int, [_P, C.c_int, _P]),
    "adapmoe_set_tau": (C.c_int, [_P, C.POINTER(C.c_float)]),
    "adapmoe_expert_bytes": (C.c_int, [C.POINTER(Config), C.POINTER(C.c_size_t)]),
    "adapmoe_pack_expert": (C.c_int, [C.POINTER(Config), _P, _P, _P, _P]),
    "adapmoe_pack_expert_int4": (C.c_int, [C.POINTER(Config)] + [_P] * 10),
    "adapmoe_pack_expert_int2": (C.c_int, [C.POINTER(Config)] + [_P] * 10),
    "adapmoe_register_expert": (C.c_int, [_P, C.c_int, C.c_int, _P, C.c_size_t]),
    "adapmoe_bind_expert_dev": (C.c_int, [_P, C.c_int, C.c_int, _P]),
    "cache_plan": (C.c_int, [C.c_int, C.c_int, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double),
                             C.POINTER(C.c_int32), C.POINTER(C.c_double)]),
    "cache_cost": (C.c_double, [C.c_int, C.c_int, C.c_double, C.c_double]),
    "cache_alloc": (C.c_int, [_P, C.POINTER(C.c_int32)]),
    "cache_lookup": (C.c_int, [_P, C.c_int, C.POINTER(C.c_int32), C.c_int, C.POINTER(C.c_int32), C.c_int]),
    "moe_gate": (C.c_int, [_P, C.c_int, _P, C.c_int, _P, _P, _P, _P, _P, _P]),
    "moe_expert_ffn": (C.c_int, [_P, C.c_int, _P, C.c_int, _P, _P, _P, _P, _P]),
    "moe_demand": (C.c_int, [_P, C.c_int, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int, C.POINTER(C.c_int32)]),
    "moe_prefetch": (C.c_int, [_P, C.c_int, C.POINTER(C.c_int32), C.c_int]),
    "moe_expert_ffn_static": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, C.c_int32, _P, _P, C.c_int, _P, _P, _P, _P, _P, _P]),
    "adapmoe_set_option": (C.c_int, [_P, C.c_int, C.c_int]),
    "adapmoe_get_option": (C.c_int, [_P, C.c_int, C.POINTER(C.c_int)]),
    "moe_layer_step": (C.c_int, [_P, C.c_int, _P, C.c_int, _P, _P]),
    "moe_residual_rmsnorm": (C.c_int, [_P, _P, _P, C.c_float, _P, C.c_int, _P]),
    "moe_stack_token": (C.c_int, [_P, C.c_int, _P, _P, _P, C.c_int, C.c_float, _P]),
    "adapmoe_set_first_layer_predictor": (C.c_int, [_P, _P]),
    "adapmoe_set_tiles": (C.c_int, [_P, C.c_int]),
    "adapmoe_set_staging": (C.c_int, [_P, C.c_int, C.c_int]),
    "adapmoe_set_lookahead": (C.c_int, [_P, C.c_int]),
    "adapmoe_last_lookahead": (C.c_int, [_P, C.c_int, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int]),
    "adapmoe_set_token": (C.c_int, [_P, C.c_int]),
    "adapmoe_trace_read": (C.c_int, [_P, C.POINTER(Event), C.c_size_t, C.POINTER(C.c_size_t)]),
    "adapmoe_counters": (C.c_int, [_P, C.POINTER(Counters)]),
    "adapmoe_last_decision": (C.c_int, [_P, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                        C.POINTER(C.c_int32), C.c_int]),
    "adapmoe_set_decision_log": (C.c_int, [_P, _P, C.c_int]),
    "adapmoe_check": (C.c_int, [_P, _P]),
    "adapmoe_profile": (C.c_int, [_P, C.c_int]),
    "adapmoe_profile_read": (C.c_int, [_P, C.c_int, C.POINTER(C.c_uint64), C.POINTER(C.c_double)]),
    "adapmoe_stream_probe": (C.c_int, [_P, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_double), _P]),
}


def exported_names():
    return sorted(_SIGS)


def load():
    """Loads the shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2408_10284_amd.build`")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _ptr(t):
    """Address of a torch tensor / numpy array / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return t.ctypes.data


def _stream(s):
    if s is None:
        return None
    return s.cuda_stream if hasattr(s, "cuda_stream") else int(s)


def _chk(ctx, rc):
    if rc != 0:
        lib = load()
        text = lib.adapmoe_strerror(rc).decode()
        if ctx:
            detail = lib.adapmoe_last_error(ctx).decode()
            if detail:
                text += f" ({detail})"
        raise AdapMoEError(rc, text)


# The C boundary takes raw addresses and cannot see how large a buffer is; a tensor that is too
# small would make a kernel read or write out of bounds.  The wrappers therefore check, for every
# tensor or array they are given (plain integer addresses are passed through unchecked), that it is
# contiguous, lives where the call expects it (device or host) and holds at least the bytes the
# header states for that argument.
_CFG = {}   # context address -> Config of adapmoe_create


def _cfg_of(ctx):
    cfg = _CFG.get(ctx.value if hasattr(ctx, "value") else ctx)
    if cfg is None:
        raise ValueError("unknown context (not created through this module, or already destroyed)")
    return cfg


def _esz(cfg):
    return 4 if cfg.dtype == F32 else 2


def _need(name, t, nbytes, where=None):
    if t is None or isinstance(t, int):
        return
    if hasattr(t, "element_size"):
        have, contiguous, on_dev = t.numel() * t.element_size(), t.is_contiguous(), t.is_cuda
    else:
        have, contiguous, on_dev = t.nbytes, t.flags["C_CONTIGUOUS"], False
    if not contiguous:
        raise ValueError(f"{name}: must be contiguous")
    if have < nbytes:
        raise ValueError(f"{name}: {have} bytes given, {nbytes} needed")
    if where == "dev" and not on_dev:
        raise ValueError(f"{name}: must be a device tensor")
    if where == "host" and on_dev:
        raise ValueError(f"{name}: must be in host memory")


def _need_step(cfg, B, x=None, y=None, h=None, ids=None, w=None, k=None):
    if not 1 <= B <= cfg.max_B:
        return   # the library rejects the call before touching any buffer
    _need("x", x, B * cfg.H * _esz(cfg), "dev")
    _need("y", y, B * cfg.H * 4, "dev")
    _need("h", h, B * cfg.H * 4, "dev")
    _need("ids", ids, 2 * B * 4, "dev")
    _need("w", w, 2 * B * 4, "dev")
    _need("k", k, B * 4, "dev")


# ---- same names as the C entry points ---------------------------------------

def adapmoe_create(H, F, N, L, dtype, max_B=1, device=0, trace_capacity=0):
    cfg = Config(H, F, N, L, dtype, max_B, device, trace_capacity)
    ctx = _P()
    _chk(None, load().adapmoe_create(C.byref(cfg), C.byref(ctx)))
    _CFG[ctx.value] = cfg
    return ctx, cfg


def adapmoe_destroy(ctx):
    _chk(None, load().adapmoe_destroy(ctx))
    _CFG.pop(ctx.value if hasattr(ctx, "value") else ctx, None)


def adapmoe_set_router(ctx, layer, Wg_dev):
    cfg = _cfg_of(ctx)
    _need("Wg", Wg_dev, cfg.N * cfg.H * _esz(cfg), "dev")
    _chk(ctx, load().adapmoe_set_router(ctx, layer, _ptr(Wg_dev)))


def adapmoe_set_tau(ctx, tau):
    if len(tau) != _cfg_of(ctx).L:
        raise ValueError("tau: one threshold per layer")
    arr = (C.c_float * len(tau))(*[float(t) for t in tau])
    _chk(ctx, load().adapmoe_set_tau(ctx, arr))


def adapmoe_expert_bytes(cfg):
    n = C.c_size_t()
    _chk(None, load().adapmoe_expert_bytes(C.byref(cfg), C.byref(n)))
    return n.value


def adapmoe_pack_expert(cfg, W1, W3, W2, out):
    for name, m in (("W1", W1), ("W3", W3), ("W2", W2)):
        _need(name, m, cfg.H * cfg.F * _esz(cfg), "host")
    _need("out", out, 3 * cfg.H * cfg.F * _esz(cfg), "host")
    _chk(None, load().adapmoe_pack_expert(C.byref(cfg), _ptr(W1), _ptr(W3), _ptr(W2), _ptr(out)))


def _need_quant(cfg, q1, s1, z1, q3, s3, z3, q2, s2, z2, out):
    n = cfg.H * cfg.F
    for name, m in (("q1", q1), ("q3", q3), ("q2", q2)):
        _need(name, m, n, "host")                 # one code per byte
    for name, m in (("s1", s1), ("z1", z1), ("s3", s3), ("z3", z3), ("s2", s2), ("z2", z2)):
        _need(name, m, n // 64 * 2, "host")       # fp16 per group of 64
    _need("out", out, adapmoe_expert_bytes(cfg), "host")


def adapmoe_pack_expert_int4(cfg, q1, s1, z1, q3, s3, z3, q2, s2, z2, out):
    _need_quant(cfg, q1, s1, z1, q3, s3, z3, q2, s2, z2, out)
    _chk(None, load().adapmoe_pack_expert_int4(C.byref(cfg), *[_ptr(a) for a in (q1, s1, z1, q3, s3, z3, q2, s2, z2, out)]))


def adapmoe_pack_expert_int2(cfg, q1, s1, z1, q3, s3, z3, q2, s2, z2, out):
    _need_quant(cfg, q1, s1, z1, q3, s3, z3, q2, s2, z2, out)
    _chk(None, load().adapmoe_pack_expert_int2(C.byref(cfg), *[_ptr(a) for a in (q1, s1, z1, q3, s3, z3, q2, s2, z2, out)]))


def adapmoe_register_expert(ctx, layer, expert, image_host, nbytes):
    _need("image_host", image_host, nbytes, "host")
    _chk(ctx, load().adapmoe_register_expert(ctx, layer, expert, _ptr(image_host), nbytes))


def adapmoe_bind_expert_dev(ctx, layer, expert, image_dev):
    _need("image_dev", image_dev, adapmoe_expert_bytes(_cfg_of(ctx)), "dev")
    _chk(ctx, load().adapmoe_bind_expert_dev(ctx, layer, expert, _ptr(image_dev)))


def cache_plan(L, N, Ctot, a, beta):
    da = (C.c_double * L)(*[float(v) for v in a])
    db = (C.c_double * L)(*[float(v) for v in beta])
    t = (C.c_int32 * L)()
    cost = C.c_double()
    _chk(None, load().cache_plan(L, N, Ctot, da, db, t, C.byref(cost)))
    return list(t), cost.value


def cache_cost(N, t, a, beta):
    return load().cache_cost(N, t, a, beta)


def cache_alloc(ctx, slots_per_layer):
    if len(slots_per_layer) != _cfg_of(ctx).L:
        raise ValueError("slots_per_layer: one count per layer")
    arr = (C.c_int32 * len(slots_per_layer))(*[int(v) for v in slots_per_layer])
    _chk(ctx, load().cache_alloc(ctx, arr))


def cache_lookup(ctx, layer, ids, touch=False):
    n = len(ids)
    arr = (C.c_int32 * n)(*[int(v) for v in ids])
    out = (C.c_int32 * n)()
    _chk(ctx, load().cache_lookup(ctx, layer, arr, n, out, 1 if touch else 0))
    return list(out)


def moe_gate(ctx, layer, x, B, ids, w, k, pred_ids=None, pred_k=None, stream=None):
    _need_step(_cfg_of(ctx), B, x=x, ids=ids, w=w, k=k)
    _need("pred_ids", pred_ids, 2 * B * 4, "dev")
    _need("pred_k", pred_k, B * 4, "dev")
    _chk(ctx, load().moe_gate(ctx, layer, _ptr(x), B, _ptr(ids), _ptr(w), _ptr(k), _ptr(pred_ids), _ptr(pred_k), _stream(stream)))


def moe_expert_ffn(ctx, layer, x, B, ids, w, k, y, stream=None):
    _need_step(_cfg_of(ctx), B, x=x, y=y, ids=ids, w=w, k=k)
    _chk(ctx, load().moe_expert_ffn(ctx, layer, _ptr(x), B, _ptr(ids), _ptr(w), _ptr(k), _ptr(y), _stream(stream)))


def moe_demand(ctx, layer, ids, k):
    """ids: 2 per token (flat or nested), k: one per token; returns the number of on-demand loads started."""
    k = [int(v) for v in k]
    flat = [int(v) for row in ids for v in (row if hasattr(row, "__len__") else [row])]
    if len(flat) != 2 * len(k):
        raise ValueError("ids: two per token")
    a = (C.c_int32 * len(flat))(*flat)
    kk = (C.c_int32 * len(k))(*k)
    loads = C.c_int32()
    _chk(ctx, load().moe_demand(ctx, layer, a, kk, len(k), C.byref(loads)))
    return loads.value


def moe_expert_ffn_static(H, F, N, dtype, table, x, B, ids, w, k, y, err=None, stream=None):
    esz = 4 if dtype == F32 else 2
    _need("table", table, N * 8, "dev")
    if 1 <= B <= 4:
        _need("x", x, B * H * esz, "dev")
        _need("y", y, B * H * 4, "dev")
        _need("ids", ids, 2 * B * 4, "dev")
        _need("w", w, 2 * B * 4, "dev")
        _need("k", k, B * 4, "dev")
    _need("err", err, 4, "dev")
    _chk(None, load().moe_expert_ffn_static(H, F, N, dtype, _ptr(table), _ptr(x), B, _ptr(ids), _ptr(w), _ptr(k), _ptr(y),
                                           _ptr(err), _stream(stream)))


def moe_prefetch(ctx, layer, ids):
    arr = (C.c_int32 * len(ids))(*[int(v) for v in ids])
    _chk(ctx, load().moe_prefetch(ctx, layer, arr, len(ids)))


def moe_layer_step(ctx, layer, x, B, y, stream=None):
    _need_step(_cfg_of(ctx), B, x=x, y=y)
    _chk(ctx, load().moe_layer_step(ctx, layer, _ptr(x), B, _ptr(y), _stream(stream)))


def moe_residual_rmsnorm(ctx, h, y, gamma, x, B, stream=None):
    _need_step(_cfg_of(ctx), B, x=x, y=y, h=h)
    _chk(ctx, load().moe_residual_rmsnorm(ctx, _ptr(h), _ptr(y), float(gamma), _ptr(x), B, _stream(stream)))


def moe_stack_token(ctx, token, h, x, y, B, gamma, stream=None):
    _need_step(_cfg_of(ctx), B, x=x, y=y, h=h)
    _chk(ctx, load().moe_stack_token(ctx, token, _ptr(h), _ptr(x), _ptr(y), B, float(gamma), _stream(stream)))


def adapmoe_set_first_layer_predictor(ctx, Gpre):
    cfg = _cfg_of(ctx)
    _need("Gpre", Gpre, cfg.N * cfg.H * _esz(cfg), "dev")
    _chk(ctx, load().adapmoe_set_first_layer_predictor(ctx, _ptr(Gpre) if Gpre is not None else None))


def adapmoe_set_option(ctx, option, value):
    _chk(ctx, load().adapmoe_set_option(ctx, int(option), int(value)))


def adapmoe_get_option(ctx, option):
    v = C.c_int()
    _chk(ctx, load().adapmoe_get_option(ctx, int(option), C.byref(v)))
    return v.value


def adapmoe_set_staging(ctx, buffers, host_threads=0):
    _chk(ctx, load().adapmoe_set_staging(ctx, int(buffers), int(host_threads)))


def adapmoe_set_tiles(ctx, tiles):
    _chk(ctx, load().adapmoe_set_tiles(ctx, tiles))


def adapmoe_set_lookahead(ctx, depth):
    _chk(ctx, load().adapmoe_set_lookahead(ctx, depth))


def adapmoe_last_lookahead(ctx, depth, B):
    pids = (C.c_int32 * (2 * B))()
    pk = (C.c_int32 * B)()
    _chk(ctx, load().adapmoe_last_lookahead(ctx, depth, pids, pk, B))
    return list(pids), list(pk)


def adapmoe_set_token(ctx, token):
    _chk(ctx, load().adapmoe_set_token(ctx, token))


def adapmoe_trace_read(ctx, cap=1 << 16):
    buf = (Event * cap)()
    n = C.c_size_t()
    _chk(ctx, load().adapmoe_trace_read(ctx, buf, cap, C.byref(n)))
    return [(e.token, e.layer, EVENT_KINDS[e.kind], e.expert, e.victim, e.slot) for e in buf[: n.value]]


def adapmoe_counters(ctx):
    c = Counters()
    _chk(ctx, load().adapmoe_counters(ctx, C.byref(c)))
    return {n: getattr(c, n) for n, _ in Counters._fields_}


def adapmoe_last_decision(ctx, B):
    ids = (C.c_int32 * (2 * B))()
    k = (C.c_int32 * B)()
    pids = (C.c_int32 * (2 * B))()
    pk = (C.c_int32 * B)()
    _chk(ctx, load().adapmoe_last_decision(ctx, ids, k, pids, pk, B))
    return list(ids), list(k), list(pids), list(pk)


def adapmoe_set_decision_log(ctx, log_dev, capacity):
    if log_dev is not None:
        _need("log_dev", log_dev, capacity * 6 * _cfg_of(ctx).max_B * 4, "dev")
    _chk(ctx, load().adapmoe_set_decision_log(ctx, _ptr(log_dev), int(capacity)))


def adapmoe_check(ctx, stream=None):
    _chk(ctx, load().adapmoe_check(ctx, _stream(stream)))


def adapmoe_profile(ctx, on):
    _chk(ctx, load().adapmoe_profile(ctx, 1 if on else 0))


def adapmoe_stream_probe(buf, nrows, row_bytes, rows_per_unit, chunk_bytes, workgroups, reps, stream=None):
    """Average duration in microseconds of one load-only pass over `buf` ([nrows, row_bytes] bytes on the device)."""
    if buf.numel() * buf.element_size() < nrows * row_bytes:
        raise ValueError("stream_probe: buffer smaller than nrows * row_bytes")
    us = C.c_double()
    _chk(None, load().adapmoe_stream_probe(_ptr(buf), int(nrows), int(row_bytes), int(rows_per_unit), int(chunk_bytes), int(workgroups),
                                           int(reps), C.byref(us), _stream(stream)))
    return us.value


def adapmoe_profile_read(ctx, kernel_class):
    n = C.c_uint64()
    ms = C.c_double()
    _chk(ctx, load().adapmoe_profile_read(ctx, kernel_class, C.byref(n), C.byref(ms)))
    return n.value, ms.value
