"""ctypes binding of libtkphi with the same entry-point names as include/tkphi.h.

Argument marshalling only: every step of the path runs in the library's HIP kernels.
torch is used for device memory and streams (tensor.data_ptr(), current stream).
The shared library is loaded on first use; if it has not been built the call raises
(there is no CPU fallback).
"""
from __future__ import annotations

import ctypes as C
import os
import threading

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libtkphi.so")

TKPHI_OK = 0
TKPHI_EINVAL, TKPHI_ESHAPE, TKPHI_EALIGN, TKPHI_EWORKSPACE, TKPHI_EHIP, TKPHI_EUNSUPPORTED = -1, -2, -3, -4, -5, -6
TKPHI_F32, TKPHI_BF16 = 0, 1
TKPHI_MODE_SUB, TKPHI_MODE_NOSUB, TKPHI_MODE_TOPK_ONLY = 0, 1, 2
TKPHI_FLAG_DIAG = 0x100
TKPHI_PHI_EXP_AFFINE, TKPHI_PHI_MLP = 0, 1
TKPHI_DIAG_STRIDE = 8
TKPHI_DEV_BAD_LENGTH, TKPHI_DEV_CLAMPED = 1, 2

EXPORTS = (
    "tkphi_workspace_bytes", "tkphi_build_summaries", "tkphi_decode", "tkphi_decode_static", "tkphi_decode_stage_times",
    "tkphi_check_problems",
    "tkphi_read_device_status", "tkphi_budget_paper", "tkphi_budget_mid", "tkphi_status_string",
    "tkphi_last_error",
)


def aux_stride(d_head: int) -> int:
    return 4 + 2 * d_head


class tkphi_tuning(C.Structure):
    _fields_ = [
        ("force_generic", C.c_int32), ("scan_chunk", C.c_int32), ("interleave", C.c_int32),
        ("build_chunk", C.c_int32), ("mlp_block", C.c_int32), ("mlp_mode", C.c_int32),
        ("select_mode", C.c_int32), ("select_test", C.c_int32),
        ("reserved", C.c_int32 * 4),
    ]


MLP_MODES = {"": 0, "chain": 0, "blocks": 1, "unfused": 2}


class tkphi_config(C.Structure):
    _fields_ = [
        ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("d_head", C.c_int32), ("d_phi", C.c_int32),
        ("n_sink", C.c_int32), ("n_tail", C.c_int32), ("kv_dtype", C.c_int32),
        ("score_scale", C.c_float), ("phi_in_scale", C.c_float), ("phi_norm_coef", C.c_float),
        ("cache_features", C.c_int32), ("phi_kind", C.c_int32), ("d_emb", C.c_int32), ("max_gen", C.c_int32),
        ("tuning", tkphi_tuning),
    ]


class tkphi_mlp(C.Structure):
    _fields_ = [
        ("Ws", C.c_void_p), ("bs", C.c_void_p), ("W1", C.c_void_p), ("b1", C.c_void_p),
        ("W2", C.c_void_p), ("b2", C.c_void_p), ("Wo", C.c_void_p), ("bo", C.c_void_p),
        ("alpha", C.c_float), ("reserved", C.c_int32),
    ]


class tkphi_problem(C.Structure):
    _fields_ = [
        ("K", C.c_void_p), ("V", C.c_void_p), ("stride_head", C.c_int64), ("stride_tok", C.c_int64),
        ("Wq", C.c_void_p), ("bq", C.c_void_p), ("Wk", C.c_void_p), ("bk", C.c_void_p),
        ("S", C.c_void_p), ("u", C.c_void_p), ("q", C.c_void_p), ("out", C.c_void_p),
        ("topk_idx", C.c_void_p), ("aux", C.c_void_p), ("scores", C.c_void_p), ("diag", C.c_void_p), ("phi_cache", C.c_void_p),
        ("mlp_q", C.c_void_p), ("mlp_k", C.c_void_p),
        ("L", C.c_int32), ("topk", C.c_int32), ("n_gen", C.c_int32), ("reserved", C.c_int32),
    ]


_lib = None
_lock = threading.Lock()


def lib() -> C.CDLL:
    """Loads libtkphi.so (once).  Raises if it is missing: build it with
    `python -m paper_2604_05438_amd.build`."""
    global _lib
    with _lock:
        if _lib is not None:
            return _lib
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not built; run `python -m paper_2604_05438_amd.build`")
        L = C.CDLL(LIB_PATH)
        cfgp, probp = C.POINTER(tkphi_config), C.c_void_p
        L.tkphi_workspace_bytes.restype = C.c_size_t
        L.tkphi_workspace_bytes.argtypes = [cfgp, C.c_int32, C.c_int32, C.c_int32]
        L.tkphi_build_summaries.restype = C.c_int
        L.tkphi_build_summaries.argtypes = [cfgp, probp, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
        L.tkphi_decode.restype = C.c_int
        L.tkphi_decode.argtypes = [cfgp, probp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                   C.c_size_t, C.c_void_p]
        L.tkphi_decode_static.restype = C.c_int
        L.tkphi_decode_static.argtypes = [cfgp, probp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
        L.tkphi_decode_stage_times.restype = C.c_int
        L.tkphi_decode_stage_times.argtypes = [cfgp, probp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                               C.c_size_t, C.c_void_p, C.POINTER(C.c_float)]
        L.tkphi_check_problems.restype = C.c_int
        L.tkphi_check_problems.argtypes = [cfgp, C.POINTER(tkphi_problem), C.c_int32, C.c_int32, C.c_int32, C.c_int32]
        L.tkphi_read_device_status.restype = C.c_int
        L.tkphi_read_device_status.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_uint32)]
        L.tkphi_budget_paper.restype = C.c_int32
        L.tkphi_budget_paper.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int32]
        L.tkphi_budget_mid.restype = C.c_int32
        L.tkphi_budget_mid.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int32]
        L.tkphi_status_string.restype = C.c_char_p
        L.tkphi_status_string.argtypes = [C.c_int32]
        L.tkphi_last_error.restype = C.c_char_p
        L.tkphi_last_error.argtypes = []
        _lib = L
        return L


class TkphiError(RuntimeError):
    def __init__(self, status: int, detail: str):
        self.status = status
        super().__init__(f"tkphi status {status} ({tkphi_status_string(status)}): {detail}")


def _check(status: int) -> None:
    if status != TKPHI_OK:
        raise TkphiError(status, tkphi_last_error())


# ---- entry points (same names as the C ABI) ---------------------------------------------
def tkphi_status_string(status: int) -> str:
    return lib().tkphi_status_string(status).decode()


def tkphi_last_error() -> str:
    return lib().tkphi_last_error().decode()


def tkphi_budget_paper(L: int, r_bp: int, n_sink: int, n_tail: int) -> int:
    return lib().tkphi_budget_paper(L, r_bp, n_sink, n_tail)


def tkphi_budget_mid(L: int, r_bp: int, n_sink: int, n_tail: int) -> int:
    return lib().tkphi_budget_mid(L, r_bp, n_sink, n_tail)


def tkphi_workspace_bytes(cfg: tkphi_config, n_problems: int, max_L: int, max_K: int) -> int:
    return lib().tkphi_workspace_bytes(C.byref(cfg), n_problems, max_L, max_K)


def tkphi_check_problems(cfg: tkphi_config, problems_host, n_problems: int, max_L: int, max_K: int,
                         for_decode: bool) -> None:
    _check(lib().tkphi_check_problems(C.byref(cfg), problems_host, n_problems, max_L, max_K, int(for_decode)))


def tkphi_build_summaries(cfg: tkphi_config, problems_dev_ptr: int, n_problems: int, max_L: int,
                          workspace_ptr: int, workspace_bytes: int, stream: int) -> None:
    _check(lib().tkphi_build_summaries(C.byref(cfg), problems_dev_ptr, n_problems, max_L, workspace_ptr,
                                       workspace_bytes, stream))


def tkphi_decode(cfg: tkphi_config, problems_dev_ptr: int, n_problems: int, max_L: int, max_K: int,
                 mode: int, workspace_ptr: int, workspace_bytes: int, stream: int) -> None:
    _check(lib().tkphi_decode(C.byref(cfg), problems_dev_ptr, n_problems, max_L, max_K, mode, workspace_ptr,
                              workspace_bytes, stream))


def tkphi_decode_static(cfg: tkphi_config, problems_dev_ptr: int, n_problems: int, max_L: int, max_K: int,
                        mode: int, stream: int) -> None:
    _check(lib().tkphi_decode_static(C.byref(cfg), problems_dev_ptr, n_problems, max_L, max_K, mode, stream))


STATIC_SCRATCH_BYTES = 32 << 20


STAGES = ("score_mid", "select_plan", "select_emit", "select_resolve", "gather", "merge", "phi_q", "prep", "select")
SELECT_SPILL, SELECT_FILTERED = 1, 2          # tkphi_tuning::select_mode


def tkphi_decode_stage_times(cfg: tkphi_config, problems_dev_ptr: int, n_problems: int, max_L: int, max_K: int,
                             mode: int, workspace_ptr: int, workspace_bytes: int, stream: int) -> list:
    out = (C.c_float * len(STAGES))()
    _check(lib().tkphi_decode_stage_times(C.byref(cfg), problems_dev_ptr, n_problems, max_L, max_K, mode,
                                          workspace_ptr, workspace_bytes, stream, out))
    return list(out)


def tkphi_read_device_status(workspace_ptr: int, stream: int) -> int:
    out = C.c_uint32(0)
    _check(lib().tkphi_read_device_status(workspace_ptr, stream, C.byref(out)))
    return out.value


# ---- marshalling helpers (device memory via torch) -----------------------------------------
def make_config(n_q_heads, n_kv_heads, d_head, d_phi, n_sink, n_tail, dtype, score_scale, phi_in_scale,
                phi_norm_coef, cache_features=0, phi_kind=0, d_emb=0, max_gen=0, tuning=None) -> tkphi_config:
    """tuning: optional dict of tkphi_tuning fields (launch-geometry overrides; omitted fields stay 0 = default)."""
    kv = {"bf16": TKPHI_BF16, "f32": TKPHI_F32}[dtype] if isinstance(dtype, str) else int(dtype)
    cfg = tkphi_config(n_q_heads, n_kv_heads, d_head, d_phi, n_sink, n_tail, kv, score_scale, phi_in_scale,
                       phi_norm_coef, int(cache_features), int(phi_kind), int(d_emb), int(max_gen))
    for name, value in (tuning or {}).items():
        setattr(cfg.tuning, name, int(value))
    return cfg


def _ptr(t) -> int:
    return 0 if t is None else int(t.data_ptr())


def make_problem(K, V, Wq, bq, Wk, bk, S, u, q=None, out=None, topk_idx=None, aux=None, scores=None,
                 L=None, topk=0, diag=None, phi_cache=None, mlp_q=None, mlp_k=None, n_gen=0) -> tkphi_problem:
    """Fills a tkphi_problem from torch device tensors (K, V: [Hkv][L + n_gen][d], last dim contiguous)."""
    assert K.stride(-1) == 1 and V.stride(-1) == 1 and K.stride() == V.stride()
    return tkphi_problem(
        _ptr(K), _ptr(V), K.stride(0), K.stride(1), _ptr(Wq), _ptr(bq), _ptr(Wk), _ptr(bk), _ptr(S), _ptr(u),
        _ptr(q), _ptr(out), _ptr(topk_idx), _ptr(aux), _ptr(scores), _ptr(diag), _ptr(phi_cache), _ptr(mlp_q), _ptr(mlp_k),
        int(K.shape[1] - n_gen if L is None else L), int(topk), int(n_gen), 0)


def upload_mlp(maps: dict, device="cuda"):
    """One side ("q" or "k") of inputs.make_mlp_phi, already on the device as torch tensors ->
    (device uint8 tensor holding the tkphi_mlp array [H], list of tensors to keep alive)."""
    import torch
    H = maps["alpha"].shape[0]
    arr = (tkphi_mlp * H)()
    for h in range(H):
        arr[h] = tkphi_mlp(_ptr(maps["Ws"][h]), _ptr(maps["bs"][h]), _ptr(maps["W1"][h]), _ptr(maps["b1"][h]),
                           _ptr(maps["W2"][h]), _ptr(maps["b2"][h]), _ptr(maps["Wo"][h]), _ptr(maps["bo"][h]),
                           float(maps["alpha"][h]), 0)
    raw = bytes(memoryview(arr).cast("B"))
    return torch.frombuffer(bytearray(raw), dtype=torch.uint8).to(device)


def upload_problems(problems, device="cuda"):
    """Host list of tkphi_problem -> (host ctypes array, device uint8 tensor holding the table)."""
    import torch
    arr = (tkphi_problem * len(problems))(*problems)
    raw = bytes(memoryview(arr).cast("B"))
    host = torch.frombuffer(bytearray(raw), dtype=torch.uint8)
    return arr, host.to(device)


def alloc_workspace(nbytes: int, device="cuda"):
    import torch
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def current_stream_ptr() -> int:
    import torch
    return int(torch.cuda.current_stream().cuda_stream)
