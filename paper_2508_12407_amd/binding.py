"""ctypes binding of include/zz.h.  Argument marshalling only: every step of the
path runs inside libzz.so.  There is no fallback: a missing library is an error."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
# (ZZ_LIBRARY=libzz_debug.so selects the bounds-checking debug build of the same sources, for the test that runs it)
LIB_PATH = os.path.join(_PKG, os.environ.get("ZZ_LIBRARY", "libzz.so"))

ZZ_ZIGZAG, ZZ_MIXED = 0, 1
ZZ_TILE_SLOTS = 32
ZZ_MAX_SPLITS = 128
ZZ_MAX_RAGGED_BATCH = 256
ERR = dict(OK=0, EINVAL=-1, ERANGE=-2, ENOSPC=-3, EALIGN=-4, ESTATE=-5, EUNSUPPORTED=-6, EHIP=-7)
TUNE_DECODE_WG_PER_CU, TUNE_DECODE_SPLITS, TUNE_NUM_CU, TUNE_PREFILL_PAIRING, TUNE_DECODE_XCD_SKEW = 1, 2, 3, 4, 5


class ZzConfig(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("batch", C.c_int32), ("max_ctx", C.c_int32),
                ("sink", C.c_int32), ("window", C.c_int32), ("max_chunk", C.c_int32),
                ("layout", C.c_int32), ("softmax_scale", C.c_float),
                ("layer_is_streaming", C.POINTER(C.c_uint8)),
                ("kvhead_is_streaming", C.POINTER(C.c_uint8))]


class ZzError(RuntimeError):
    def __init__(self, code, where):
        self.code = int(code)
        detail = ""
        if int(code) == ERR["EHIP"] or (int(code) == ERR["ENOSPC"] and where == "zz_attn_decode_static"):
            detail = lib.zz_last_error_detail().decode()
        super().__init__(f"{where}: {strerror(code)} ({code}) {detail}")


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no fallback path)")
    # torch ships its own libamdhip64 and the device memory handed to this library
    # comes from it: load torch's runtime first so that libzz.so binds to the same
    # one (a second HIP runtime in the process would not see torch's device state).
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    P, I, I64, V = C.POINTER, C.c_int, C.c_int64, C.c_void_p
    sig = {
        "zz_arena_bytes": (C.c_size_t, [P(ZzConfig)]),
        "zz_workspace_bytes": (C.c_size_t, [P(ZzConfig)]),
        "zz_create": (I, [P(ZzConfig), V, C.c_size_t, V, C.c_size_t, P(V)]),
        "zz_destroy": (I, [V]),
        "zz_reset": (I, [V]),
        "zz_kv_append": (I, [V, I, V, V, I, V]),
        "zz_attn_prefill": (I, [V, I, V, V, V, I, V, V]),
        "zz_attn_decode": (I, [V, I, V, V, V]),
        "zz_attn_decode_static": (I, [V, I, V, V, V]),
        "zz_decode_step": (I, [V, I, V, V, V, V, V]),
        "zz_kv_append_seq": (I, [V, I, I, V, V, I, V]),
        "zz_attn_prefill_seq": (I, [V, I, I, V, V, V, I, V, V]),
        "zz_seq_len": (I64, [V, I, I]),
        "zz_set_seq_len": (I, [V, I, I, I64]),
        "zz_layer_len": (I64, [V, I]),
        "zz_set_layer_len": (I, [V, I, I64]),
        "zz_layer_launches": (I, [V, I]),
        "zz_set_rope_tables": (I, [V, V, V, I64]),
        "zz_slot_of": (I64, [P(ZzConfig), I, I, I64]),
        "zz_kv_elem_offset": (I64, [V, I, I, I, I, I64, I]),
        "zz_tune": (I, [V, I, I]),
        "zz_decode_plan": (I, [V, I, I, P(I), P(I)]),
        "zz_prefill_tile_counts": (I, [V, I, I, P(I64), P(I64)]),
        "zz_transport_select": (I, [P(C.c_float), I, I, C.c_float, C.c_float, P(C.c_uint8), P(C.c_double)]),
        "zz_probe_read": (I, [V, V, C.c_size_t, I, V]),
        "zz_debug_word_offset": (C.c_size_t, [P(ZzConfig)]),
        "zz_is_debug_build": (I, []),
        "zz_strerror": (C.c_char_p, [I]),
        "zz_last_error_detail": (C.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    return L


lib = _load()


def strerror(code):
    return lib.zz_strerror(int(code)).decode()


def make_config(n_layers, n_q_heads, n_kv_heads, head_dim, batch, max_ctx, sink, window, max_chunk=0,
                layout=ZZ_ZIGZAG, softmax_scale=0.0, layer_is_streaming=None, kvhead_is_streaming=None):
    """Returns (ZzConfig, keepalive) - keepalive owns the host mask arrays."""
    keep = []
    cfg = ZzConfig(n_layers, n_q_heads, n_kv_heads, head_dim, batch, max_ctx, sink, window, max_chunk, layout,
                   softmax_scale, None, None)
    if layer_is_streaming is not None:
        a = np.ascontiguousarray(np.asarray(layer_is_streaming, dtype=np.uint8))
        keep.append(a)
        cfg.layer_is_streaming = a.ctypes.data_as(C.POINTER(C.c_uint8))
    if kvhead_is_streaming is not None:
        a = np.ascontiguousarray(np.asarray(kvhead_is_streaming, dtype=np.uint8))
        keep.append(a)
        cfg.kvhead_is_streaming = a.ctypes.data_as(C.POINTER(C.c_uint8))
    return cfg, keep


def arena_bytes(cfg):
    return int(lib.zz_arena_bytes(C.byref(cfg)))


def workspace_bytes(cfg):
    return int(lib.zz_workspace_bytes(C.byref(cfg)))


def slot_of(cfg, layer, kv_head, pos):
    return int(lib.zz_slot_of(C.byref(cfg), layer, kv_head, pos))


def transport_select(alpha, sparsity, omega):
    """Section 2.2, Eq. 5 on the host: alpha [L,H] float32 -> (uint8[L] layer mask, loss)."""
    a = np.ascontiguousarray(np.asarray(alpha, dtype=np.float32))
    L, H = a.shape
    mask = np.zeros(L, dtype=np.uint8)
    loss = C.c_double()
    rc = lib.zz_transport_select(a.ctypes.data_as(C.POINTER(C.c_float)), L, H, sparsity, omega,
                                 mask.ctypes.data_as(C.POINTER(C.c_uint8)), C.byref(loss))
    if rc != 0:
        raise ZzError(rc, "zz_transport_select")
    return mask, loss.value


def _ptr(t):
    """Device (or host, for CPU-side error-path tests) address of a torch tensor / int."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


class Context:
    """Owns a zz_ctx.  `arena` and `workspace` are caller-allocated tensors (or raw
    addresses); the context keeps references so they outlive it."""

    def __init__(self, cfg, arena, workspace, arena_nbytes=None, workspace_nbytes=None, keep=None):
        self.cfg, self._keep, self.arena, self.workspace = cfg, keep, arena, workspace
        an = arena_nbytes if arena_nbytes is not None else arena.numel() * arena.element_size()
        wn = workspace_nbytes if workspace_nbytes is not None else workspace.numel() * workspace.element_size()
        h = C.c_void_p()
        rc = lib.zz_create(C.byref(cfg), _ptr(arena), an, _ptr(workspace), wn, C.byref(h))
        if rc != 0:
            raise ZzError(rc, "zz_create")
        self._h = h

    def close(self):
        if getattr(self, "_h", None) and lib is not None:   # (module globals may be gone at interpreter exit)
            lib.zz_destroy(self._h)
            self._h = None

    __del__ = close

    @staticmethod
    def _chk(rc, where):
        if rc != 0:
            raise ZzError(rc, where)

    def reset(self):
        self._chk(lib.zz_reset(self._h), "zz_reset")

    def kv_append(self, layer, k_new, v_new, n_new, stream=None):
        self._chk(lib.zz_kv_append(self._h, layer, _ptr(k_new), _ptr(v_new), n_new, stream), "zz_kv_append")

    def attn_prefill(self, layer, q, k_new, v_new, n_new, out, stream=None):
        self._chk(lib.zz_attn_prefill(self._h, layer, _ptr(q), _ptr(k_new), _ptr(v_new), n_new, _ptr(out), stream),
                  "zz_attn_prefill")

    def kv_append_seq(self, layer, b, k_new, v_new, n_new, stream=None):
        self._chk(lib.zz_kv_append_seq(self._h, layer, b, _ptr(k_new), _ptr(v_new), n_new, stream), "zz_kv_append_seq")

    def attn_prefill_seq(self, layer, b, q, k_new, v_new, n_new, out, stream=None):
        self._chk(lib.zz_attn_prefill_seq(self._h, layer, b, _ptr(q), _ptr(k_new), _ptr(v_new), n_new, _ptr(out),
                                          stream), "zz_attn_prefill_seq")

    def seq_len(self, layer, b):
        return int(lib.zz_seq_len(self._h, layer, b))

    def set_seq_len(self, layer, b, n):
        self._chk(lib.zz_set_seq_len(self._h, layer, b, n), "zz_set_seq_len")

    def attn_decode(self, layer, q, out, stream=None):
        self._chk(lib.zz_attn_decode(self._h, layer, _ptr(q), _ptr(out), stream), "zz_attn_decode")

    def attn_decode_static(self, layer, q, out, stream=None):
        self._chk(lib.zz_attn_decode_static(self._h, layer, _ptr(q), _ptr(out), stream), "zz_attn_decode_static")

    def decode_step(self, layer, q, k_new, v_new, out, stream=None):
        self._chk(lib.zz_decode_step(self._h, layer, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), stream),
                  "zz_decode_step")

    def layer_len(self, layer):
        return int(lib.zz_layer_len(self._h, layer))

    def set_layer_len(self, layer, n):
        self._chk(lib.zz_set_layer_len(self._h, layer, n), "zz_set_layer_len")

    def set_rope_tables(self, cos, sin, rows):
        self._rope = (cos, sin)      # the tables stay alive with the context
        self._chk(lib.zz_set_rope_tables(self._h, _ptr(cos), _ptr(sin), rows), "zz_set_rope_tables")

    def layer_launches(self, layer):
        return int(lib.zz_layer_launches(self._h, layer))

    def kv_elem_offset(self, layer, which, b, kv_head, slot, d):
        return int(lib.zz_kv_elem_offset(self._h, layer, which, b, kv_head, slot, d))

    def prefill_tile_counts(self, layer, n_new):
        a, b = C.c_int64(), C.c_int64()
        self._chk(lib.zz_prefill_tile_counts(self._h, layer, n_new, C.byref(a), C.byref(b)), "zz_prefill_tile_counts")
        return a.value, b.value

    def probe_read(self, buf, nbytes, nontemporal, stream=None):
        self._chk(lib.zz_probe_read(self._h, _ptr(buf), nbytes, int(nontemporal), stream), "zz_probe_read")

    def tune(self, key, value):
        self._chk(lib.zz_tune(self._h, key, value), "zz_tune")

    def decode_plan(self, layer, group):
        a, b = C.c_int(), C.c_int()
        self._chk(lib.zz_decode_plan(self._h, layer, group, C.byref(a), C.byref(b)), "zz_decode_plan")
        return a.value, b.value
