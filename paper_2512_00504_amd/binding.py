"""ctypes binding of libgkv.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI declared in
include/gkv.h; the functions here have the same names and pass device
pointers of torch tensors and the current torch stream straight through.
There is no fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_double, c_float, c_int32, c_int64, c_size_t, c_void_p

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("GKV_LIB_PATH") or os.path.join(_HERE, "libgkv.so")

GKV_F32, GKV_BF16 = 0, 1
GKV_COMBINE = {"max": 0, "avg": 1, "sum": 2}
ST_LEN, ST_LEN_STEP, ST_N_HIST, ST_N_TILED = 0, 1, 2, 3     # fields of a d_state record
KERNEL_IDS = {"attend": 0, "score": 1, "global": 2, "topk": 3, "compact": 4, "redundancy": 5}

EXPORTS = [
    "gkv_create", "gkv_destroy", "gkv_status_string", "gkv_workspace_bytes", "gkv_workspace_init",
    "gkv_cache_bytes", "gkv_k_offset", "gkv_set_param", "gkv_attend_decode", "gkv_score_window",
    "gkv_global_update", "gkv_select_topk", "gkv_compact", "gkv_evict", "gkv_profile_enable",
    "gkv_profile_read", "gkv_profile_reset", "gkv_probe_attend_read", "gkv_redundancy_combine", "gkv_evicted_positions", "gkv_pool_scores",
    "gkv_evict_static", "gkv_set_step_base", "gkv_advance_step_base",
]


class GkvConfig(ctypes.Structure):
    _fields_ = [
        ("n_layers", c_int32), ("batch", c_int32), ("n_q_heads", c_int32), ("n_kv_heads", c_int32),
        ("head_dim", c_int32), ("budget", c_int32), ("window", c_int32), ("interval", c_int32),
        ("capacity", c_int32), ("dtype", c_int32), ("combine", c_int32), ("alpha", c_float),
        ("softmax_scale", c_float),
    ]


class GkvError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: gkv status {status}")


_lib = None


def load_library():
    """Load libgkv.so (built in-tree by __graft_entry__.build()).  Raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32 = c_void_p, c_int32
    lib.gkv_create.argtypes = [POINTER(GkvConfig), POINTER(vp)]
    lib.gkv_destroy.argtypes = [vp]; lib.gkv_destroy.restype = None
    lib.gkv_status_string.argtypes = [i32]; lib.gkv_status_string.restype = c_char_p
    lib.gkv_workspace_bytes.argtypes = [vp, POINTER(c_size_t)]
    lib.gkv_workspace_init.argtypes = [vp, vp, vp]
    lib.gkv_cache_bytes.argtypes = [POINTER(GkvConfig), i32, i32, POINTER(c_size_t), POINTER(c_size_t)]
    lib.gkv_k_offset.argtypes = [POINTER(GkvConfig), i32, i32, i32]; lib.gkv_k_offset.restype = c_int64
    lib.gkv_set_param.argtypes = [vp, c_char_p, i32]
    lib.gkv_attend_decode.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, i32, vp, vp, vp]
    lib.gkv_score_window.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, vp]
    lib.gkv_global_update.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp]
    lib.gkv_select_topk.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp]
    lib.gkv_compact.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp]
    lib.gkv_evict.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp]
    lib.gkv_set_step_base.argtypes = [vp, vp]
    lib.gkv_advance_step_base.argtypes = [vp, i32, vp]
    lib.gkv_evict_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp]
    lib.gkv_redundancy_combine.argtypes = [vp, vp, vp, i32, i32, vp, c_float, c_float, c_float, i32, vp, vp, vp, vp]
    lib.gkv_pool_scores.argtypes = [vp, vp, vp, i32, i32, vp, vp]
    lib.gkv_evicted_positions.argtypes = [vp, vp, vp, vp, i32, vp, vp]
    lib.gkv_profile_enable.argtypes = [vp, i32]
    lib.gkv_profile_read.argtypes = [vp, i32, POINTER(c_double), POINTER(c_int64)]
    lib.gkv_profile_reset.argtypes = [vp]
    lib.gkv_probe_attend_read.argtypes = [vp, vp, i32, i32, i32, vp, vp]
    for name in EXPORTS:
        fn = getattr(lib, name)
        if name not in ("gkv_destroy", "gkv_status_string", "gkv_k_offset"):
            fn.restype = c_int32
    _lib = lib
    return lib


def make_config(n_layers, batch, n_q_heads, n_kv_heads, head_dim, budget, window, interval,
                capacity, dtype, combine="max", alpha=0.8, softmax_scale=0.0) -> GkvConfig:
    dt = {"f32": GKV_F32, "bf16": GKV_BF16}[dtype] if isinstance(dtype, str) else int(dtype)
    cb = GKV_COMBINE[combine] if isinstance(combine, str) else int(combine)
    return GkvConfig(n_layers, batch, n_q_heads, n_kv_heads, head_dim, budget, window, interval,
                     capacity, dt, cb, alpha, softmax_scale)


def _ptr(t):
    """Device pointer of a torch tensor (or None)."""
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("gkv: tensors must be contiguous")
    return c_void_p(t.data_ptr())


def _stream():
    import torch
    return c_void_p(torch.cuda.current_stream().cuda_stream)


class Context:
    """Owns a gkv_ctx.  Methods mirror the C entry points one to one."""

    def __init__(self, cfg: GkvConfig):
        self.lib = load_library()
        self.cfg = cfg
        h = c_void_p()
        st = self.lib.gkv_create(byref(cfg), byref(h))
        if st != 0:
            raise GkvError(st, "gkv_create")
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.gkv_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st, what):
        if st != 0:
            raise GkvError(st, what)

    def set_param(self, name: str, value: int):
        self._check(self.lib.gkv_set_param(self.h, name.encode(), value), "gkv_set_param")

    def workspace_bytes(self) -> int:
        n = c_size_t()
        self._check(self.lib.gkv_workspace_bytes(self.h, byref(n)), "gkv_workspace_bytes")
        return n.value

    def set_step_base(self, d_step_base):
        """d_step_base: int32 device tensor of one element (or None for absolute steps)."""
        self._check(self.lib.gkv_set_step_base(self.h, _ptr(d_step_base)), "gkv_set_step_base")

    def advance_step_base(self, delta: int):
        self._check(self.lib.gkv_advance_step_base(self.h, delta, _stream()), "gkv_advance_step_base")

    def workspace_init(self, workspace):
        self._check(self.lib.gkv_workspace_init(self.h, _ptr(workspace), _stream()), "gkv_workspace_init")

    def attend_decode(self, q, k_new, v_new, K, V, pos, step, qwin, d_state, len_max_host, out, workspace):
        self._check(self.lib.gkv_attend_decode(self.h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(K), _ptr(V),
                                               _ptr(pos), step, _ptr(qwin), _ptr(d_state), len_max_host,
                                               _ptr(out), _ptr(workspace), _stream()), "gkv_attend_decode")

    def score_window(self, qwin, K, d_state, step, len_max_host, S, workspace):
        self._check(self.lib.gkv_score_window(self.h, _ptr(qwin), _ptr(K), _ptr(d_state), step, len_max_host,
                                              _ptr(S), _ptr(workspace), _stream()), "gkv_score_window")

    def global_update(self, S, F_hist, d_state, step, len_max_host, F_out):
        self._check(self.lib.gkv_global_update(self.h, _ptr(S), _ptr(F_hist), _ptr(d_state), step,
                                               len_max_host, _ptr(F_out), _stream()), "gkv_global_update")

    def select_topk(self, F, d_state, step, len_max_host, keep_idx, workspace):
        self._check(self.lib.gkv_select_topk(self.h, _ptr(F), _ptr(d_state), step, len_max_host, _ptr(keep_idx),
                                             _ptr(workspace), _stream()), "gkv_select_topk")

    def compact(self, keep_idx, F, K, V, F_hist, pos, d_state, step, workspace):
        self._check(self.lib.gkv_compact(self.h, _ptr(keep_idx), _ptr(F), _ptr(K), _ptr(V), _ptr(F_hist),
                                         _ptr(pos), _ptr(d_state), step, _ptr(workspace), _stream()),
                    "gkv_compact")

    def evict(self, qwin, K, V, F_hist, pos, d_state, step, len_max_host, S, F, keep_idx, workspace):
        self._check(self.lib.gkv_evict(self.h, _ptr(qwin), _ptr(K), _ptr(V), _ptr(F_hist), _ptr(pos),
                                       _ptr(d_state), step, len_max_host, _ptr(S), _ptr(F),
                                       _ptr(keep_idx), _ptr(workspace), _stream()), "gkv_evict")

    def evict_static(self, qwin, K, V, F_hist, pos, d_state, step, len_max_host, workspace):
        self._check(self.lib.gkv_evict_static(self.h, _ptr(qwin), _ptr(K), _ptr(V), _ptr(F_hist), _ptr(pos),
                                              _ptr(d_state), step, len_max_host, _ptr(workspace), _stream()),
                    "gkv_evict_static")

    def redundancy_combine(self, K, d_state, step, len_max_host, F, lam, tau, eps, n_recent, R_norm, F_sel, workspace):
        self._check(self.lib.gkv_redundancy_combine(self.h, _ptr(K), _ptr(d_state), step, len_max_host, _ptr(F),
                                                    lam, tau, eps, n_recent, _ptr(R_norm), _ptr(F_sel),
                                                    _ptr(workspace), _stream()), "gkv_redundancy_combine")

    def pool_scores(self, F, d_state, step, kernel, F_out):
        self._check(self.lib.gkv_pool_scores(self.h, _ptr(F), _ptr(d_state), step, kernel, _ptr(F_out), _stream()),
                    "gkv_pool_scores")

    def evicted_positions(self, keep_idx, pos, d_state, step, evicted):
        self._check(self.lib.gkv_evicted_positions(self.h, _ptr(keep_idx), _ptr(pos), _ptr(d_state), step,
                                                   _ptr(evicted), _stream()), "gkv_evicted_positions")

    def profile_enable(self, on: bool):
        self._check(self.lib.gkv_profile_enable(self.h, int(on)), "gkv_profile_enable")

    def profile_reset(self):
        self._check(self.lib.gkv_profile_reset(self.h), "gkv_profile_reset")

    def profile_read(self, kernel: str):
        ms, n = c_double(), c_int64()
        self._check(self.lib.gkv_profile_read(self.h, KERNEL_IDS[kernel], byref(ms), byref(n)), "gkv_profile_read")
        return ms.value, n.value


def probe_attend_read(K, V, rows, sink):
    """Enqueue one pass of the decode kernel's read pattern over rows [0, rows) of every unit of the
    bf16, d = 128 caches K, V [..., capacity, 128] (measurement aid)."""
    lib = load_library()
    cap = K.shape[-2]
    units = K.numel() // (cap * K.shape[-1])
    st = lib.gkv_probe_attend_read(_ptr(K), _ptr(V), units, cap, rows, _ptr(sink), _stream())
    if st != 0:
        raise GkvError(st, "gkv_probe_attend_read")


def cache_bytes(cfg: GkvConfig, rows: int, score_elem_bytes: int = 4):
    lib = load_library()
    kv, sc = c_size_t(), c_size_t()
    st = lib.gkv_cache_bytes(byref(cfg), rows, score_elem_bytes, byref(kv), byref(sc))
    if st != 0:
        raise GkvError(st, "gkv_cache_bytes")
    return kv.value, sc.value


def k_offset(cfg: GkvConfig, row: int, channel: int, n_tiled: int) -> int:
    return load_library().gkv_k_offset(byref(cfg), row, channel, n_tiled)
