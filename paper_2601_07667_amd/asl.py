"""ctypes binding of libasl.so: argument marshalling only.

Every function takes torch CUDA tensors (device memory) and forwards their pointers to the
C ABI declared in include/asl.h; all computation happens in the HIP kernels.  There is no CPU
fallback: if the shared library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("ASL_LIBRARY_PATH") or os.path.join(_PKG, "libasl.so")

ASL_OK, ASL_EINVAL, ASL_ENOMEM, ASL_EHIP, ASL_EUNSUPPORTED = 0, -1, -2, -3, -4
ASL_BF16, ASL_F32 = 0, 1
ASL_FLAG_GENERIC_SCORE = 1
ASL_FLAG_DEFER_JOIN = 2
_STATUS = {0: "ASL_OK", -1: "ASL_EINVAL", -2: "ASL_ENOMEM", -3: "ASL_EHIP", -4: "ASL_EUNSUPPORTED"}

EXPORTS = ["asl_create", "asl_destroy", "asl_last_error", "asl_workspace_bytes", "asl_score_layer",
           "asl_window_lse", "asl_gather_kv_layers", "asl_rank_static", "asl_static_last_error", "asl_pool", "asl_rank", "asl_rankvar", "asl_rank_stat", "asl_select_topk", "asl_gather_kv",
           "asl_gather_rows", "asl_layer_step", "asl_join", "asl_device_fault", "asl_profile_enable", "asl_profile_collect"]


class AslParams(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("seq_len", C.c_int32), ("window", C.c_int32), ("pool_kernel", C.c_int32),
                ("budget", C.c_int32), ("dtype", C.c_int32),
                ("k_stride_head", C.c_int64), ("k_stride_tok", C.c_int64),
                ("v_stride_head", C.c_int64), ("v_stride_tok", C.c_int64),
                ("scale", C.c_float), ("flags", C.c_int32)]


class AslState(C.Structure):
    _fields_ = [("init_var", C.c_double), ("init_set", C.c_int32), ("n_valid_rows", C.c_int32),
                ("last_layer", C.c_int32), ("reserved", C.c_int32)]


class AslStat(C.Structure):
    _fields_ = [("var_top", C.c_double), ("rel_var", C.c_double), ("numerator", C.c_uint64),
                ("union_size", C.c_int32), ("n_rows", C.c_int32), ("evaluated", C.c_int32),
                ("selected", C.c_int32)]


class AslError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status


_lib = None


def load() -> C.CDLL:
    """Load libasl.so (built in-tree by paper_2601_07667_amd.build).  Fails loudly if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} not found: build it with `python -m paper_2601_07667_amd.build`")
    # The tensors handed to the library are PyTorch allocations, so the process must run ONE HIP runtime:
    # the one PyTorch ships.  Loading it first makes libasl.so bind to it instead of pulling in a second copy.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.asl_create.argtypes = [C.POINTER(vp), C.c_int, i32, i32, i32]
    lib.asl_create.restype = C.c_int
    lib.asl_destroy.argtypes = [vp]
    lib.asl_destroy.restype = C.c_int
    lib.asl_last_error.argtypes = [vp]
    lib.asl_last_error.restype = C.c_char_p
    lib.asl_workspace_bytes.argtypes = [i32, i32, i32]
    lib.asl_workspace_bytes.restype = C.c_size_t
    lib.asl_score_layer.argtypes = [vp, C.POINTER(AslParams), vp, vp, vp, vp, vp, vp]
    lib.asl_score_layer.restype = C.c_int
    lib.asl_window_lse.argtypes = [vp, C.POINTER(AslParams), vp, vp, vp, vp]
    lib.asl_window_lse.restype = C.c_int
    lib.asl_gather_kv_layers.argtypes = [vp, C.POINTER(AslParams), vp, vp, vp, i32, i32, i32, vp, vp, vp]
    lib.asl_gather_kv_layers.restype = C.c_int
    lib.asl_pool.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp]
    lib.asl_pool.restype = C.c_int
    lib.asl_rank.argtypes = [vp, vp, i32, vp, vp]
    lib.asl_rank.restype = C.c_int
    lib.asl_rank_static.argtypes = [vp, i32, vp, vp]
    lib.asl_rank_static.restype = C.c_int
    lib.asl_static_last_error.argtypes = []
    lib.asl_static_last_error.restype = C.c_char_p
    lib.asl_rankvar.argtypes = [vp, vp, i32, i32, i32, i32, i32, C.c_double, vp, vp, vp]
    lib.asl_rankvar.restype = C.c_int
    lib.asl_rank_stat.argtypes = [vp, C.POINTER(AslParams), vp, i32, i32, i32, C.c_double, vp, vp, vp, vp]
    lib.asl_rank_stat.restype = C.c_int
    lib.asl_select_topk.argtypes = [vp, C.POINTER(AslParams), vp, i32, vp, vp]
    lib.asl_select_topk.restype = C.c_int
    lib.asl_gather_kv.argtypes = [vp, C.POINTER(AslParams), vp, vp, vp, i32, i32, vp, vp, vp]
    lib.asl_gather_kv.restype = C.c_int
    lib.asl_gather_rows.argtypes = [vp, vp, i64, i32, vp, i32, vp, vp]
    lib.asl_gather_rows.restype = C.c_int
    lib.asl_layer_step.argtypes = [vp, C.POINTER(AslParams), vp, vp, vp, vp, i32, i32, i32, C.c_double,
                                   vp, vp, vp, vp, vp, vp, vp, vp]
    lib.asl_layer_step.restype = C.c_int
    lib.asl_device_fault.argtypes = [vp, C.POINTER(i32)]
    lib.asl_device_fault.restype = C.c_int
    lib.asl_join.argtypes = [vp, vp]
    lib.asl_join.restype = C.c_int
    lib.asl_profile_enable.argtypes = [vp, C.c_uint32, i32]
    lib.asl_profile_enable.restype = C.c_int
    lib.asl_profile_collect.argtypes = [vp, i32, C.POINTER(C.c_double), C.POINTER(i32)]
    lib.asl_profile_collect.restype = C.c_int
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def make_params(Hq: int, Hk: int, d: int, N: int, W: int, S: int, budget: int, dtype: int = ASL_BF16,
                k_strides=None, v_strides=None, scale: float = 0.0, flags: int = 0) -> AslParams:
    ks = k_strides or (N * d, d)
    vs = v_strides or (N * d, d)
    return AslParams(Hq, Hk, d, N, W, S, budget, dtype, ks[0], ks[1], vs[0], vs[1], scale, flags)


class Asl:
    """One libasl context (device workspace) and thin wrappers around its entry points."""

    def __init__(self, max_seq_len: int, max_kv_heads: int, max_q_rows: int, device: int = 0):
        self.lib = load()
        h = C.c_void_p()
        st = self.lib.asl_create(C.byref(h), device, max_seq_len, max_kv_heads, max_q_rows)
        if st != ASL_OK:
            raise AslError(st, "asl_create failed")
        self.h = h
        self.device = device

    def close(self) -> None:
        if getattr(self, "h", None):
            self.lib.asl_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int) -> None:
        if st != ASL_OK:
            raise AslError(st, self.lib.asl_last_error(self.h).decode())

    # -- entry points (same names as the C ABI) ------------------------------------------------
    def asl_score_layer(self, params: AslParams, q_obs, k, p_head, s_all, lse=None) -> None:
        self._check(self.lib.asl_score_layer(self.h, C.byref(params), _ptr(q_obs), _ptr(k), _ptr(lse),
                                             _ptr(p_head), _ptr(s_all), _stream()))

    def asl_window_lse(self, params: AslParams, q_obs, k, lse_out) -> None:
        self._check(self.lib.asl_window_lse(self.h, C.byref(params), _ptr(q_obs), _ptr(k), _ptr(lse_out),
                                            _stream()))

    def asl_gather_kv_layers(self, params: AslParams, k_ptrs, v_ptrs, idx, idx_rows: int, n_idx: int,
                             n_layers: int, k_out_ptrs, v_out_ptrs) -> None:
        """k_ptrs .. v_out_ptrs: int64 device tensors holding one device pointer per layer."""
        self._check(self.lib.asl_gather_kv_layers(self.h, C.byref(params), _ptr(k_ptrs), _ptr(v_ptrs), _ptr(idx),
                                                  idx_rows, n_idx, n_layers, _ptr(k_out_ptrs), _ptr(v_out_ptrs),
                                                  _stream()))

    def asl_pool(self, u, rows: int, T: int, S: int, p_out, s_out=None) -> None:
        self._check(self.lib.asl_pool(self.h, _ptr(u), rows, T, S, _ptr(p_out), _ptr(s_out), _stream()))

    def asl_rank(self, s, T: int, rank_out) -> None:
        self._check(self.lib.asl_rank(self.h, _ptr(s), T, _ptr(rank_out), _stream()))

    def asl_rankvar(self, rank_ring, l_obs: int, T: int, layer_idx: int, l_min: int, k: int, tau: float,
                    state, out) -> None:
        self._check(self.lib.asl_rankvar(self.h, _ptr(rank_ring), l_obs, T, layer_idx, l_min, k, tau,
                                         _ptr(state), _ptr(out), _stream()))

    def asl_rank_stat(self, params: AslParams, s_all, layer_idx: int, l_min: int, l_obs: int, tau: float,
                      rank_ring, state, out) -> None:
        self._check(self.lib.asl_rank_stat(self.h, C.byref(params), _ptr(s_all), layer_idx, l_min, l_obs,
                                           tau, _ptr(rank_ring), _ptr(state), _ptr(out), _stream()))

    def asl_select_topk(self, params: AslParams, scores, rows: int, idx_out) -> None:
        self._check(self.lib.asl_select_topk(self.h, C.byref(params), _ptr(scores), rows, _ptr(idx_out),
                                             _stream()))

    def asl_gather_rows(self, src, src_row_stride_bytes: int, row_bytes: int, idx, n_idx: int, dst) -> None:
        self._check(self.lib.asl_gather_rows(self.h, _ptr(src), src_row_stride_bytes, row_bytes, _ptr(idx), n_idx,
                                             _ptr(dst), _stream()))

    def asl_layer_step(self, params: AslParams, q_obs, k, v, layer_idx: int, l_min: int, l_obs: int, tau: float,
                       scores, rank_ring, state, out, idx_out, k_out=None, v_out=None, lse=None) -> None:
        self._check(self.lib.asl_layer_step(self.h, C.byref(params), _ptr(q_obs), _ptr(k), _ptr(v), _ptr(lse),
                                            layer_idx, l_min, l_obs, tau, _ptr(scores), _ptr(rank_ring),
                                            _ptr(state), _ptr(out), _ptr(idx_out), _ptr(k_out), _ptr(v_out),
                                            _stream()))

    def asl_device_fault(self) -> int:
        """Waits for the device, returns and clears the fault word (0 = every in-launch wait was met)."""
        v = C.c_int32()
        self._check(self.lib.asl_device_fault(self.h, C.byref(v)))
        return v.value

    def asl_join(self) -> None:
        self._check(self.lib.asl_join(self.h, _stream()))

    def asl_profile_enable(self, kernel_mask: int, max_records: int) -> None:
        self._check(self.lib.asl_profile_enable(self.h, kernel_mask, max_records))

    def asl_profile_collect(self, kernel_id: int):
        """(total milliseconds, launches) of the recorded launches of one kernel id; -1 clears."""
        ms, n = C.c_double(), C.c_int32()
        self._check(self.lib.asl_profile_collect(self.h, kernel_id, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def asl_gather_kv(self, params: AslParams, k, v, idx, idx_rows: int, n_idx: int, k_out, v_out) -> None:
        self._check(self.lib.asl_gather_kv(self.h, C.byref(params), _ptr(k), _ptr(v), _ptr(idx), idx_rows,
                                           n_idx, _ptr(k_out), _ptr(v_out), _stream()))


ASL_RANK_STATIC_MAX_T = 262144


def asl_rank_static(s, T: int, rank_out) -> None:
    """The context-free, allocation-free variant of asl_rank (scratch in a static device array)."""
    lib = load()
    st = lib.asl_rank_static(_ptr(s), T, _ptr(rank_out), _stream())
    if st != ASL_OK:
        raise AslError(st, lib.asl_static_last_error().decode())


KERNEL_NAMES = ["score_rowstats", "score_combine", "score_colsum", "pool", "sort_hist", "sort_scatter",
                "rankvar_final", "rankvar", "select_hist", "select_write", "gather", "score_generic", "tail_fused"]


# -- helpers for the device-resident structs (plumbing only) ---------------------------------------
def new_state(device="cuda:0"):
    """A zeroed asl_state in device memory (24 bytes)."""
    import torch
    return torch.zeros(C.sizeof(AslState), dtype=torch.uint8, device=device)


def new_stat(device="cuda:0"):
    import torch
    return torch.zeros(C.sizeof(AslStat), dtype=torch.uint8, device=device)


def read_struct(t, cls):
    """Copy a device-resident struct to the host (synchronises)."""
    return cls.from_buffer_copy(bytes(t.cpu().numpy().tobytes()))


def write_state(t, init_var: float = 0.0, init_set: int = 0, n_valid_rows: int = 0, last_layer: int = 0):
    import numpy as np
    import torch
    s = AslState(init_var, init_set, n_valid_rows, last_layer, 0)
    t.copy_(torch.from_numpy(np.frombuffer(bytes(s), dtype=np.uint8).copy()))
