"""Thin Python binding of libhola.so: same names as the C ABI (include/hola.h), argument
marshalling only.  Every step of the verify path runs in the library's HIP kernels; this
module owns no arithmetic and has no fallback: if the library is missing it raises.

Tensors are PyTorch CUDA(ROCm) tensors used purely as device memory (``data_ptr()``);
bf16 logits may be ``torch.bfloat16`` or raw ``torch.uint16``/``torch.int16`` bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhola.so")

HOLA_OK, HOLA_ERR_INVALID_ARG, HOLA_ERR_UNSUPPORTED, HOLA_ERR_WORKSPACE, HOLA_ERR_HIP = range(5)
HOLA_DTYPE_F32, HOLA_DTYPE_BF16 = 0, 1
HOLA_N_STAGES = 11
STAGE_NAMES = ("row_stats", "accept", "tile_sums", "select", "glue", "fused", "tail", "filter", "filter_scan",
               "filter_decide", "read_probe")

EXPORTS = (
    "hola_verify_f32", "hola_verify_bf16", "hola_verify_ex", "hola_verify_literal_ex", "hola_workspace_bytes",
    "hola_workspace_bytes_ex", "hola_verify_ex_static",
    "hola_hsd_verify", "hola_hsd_verify_ex", "hola_hsd_workspace_bytes", "hola_verify_tree",
    "hola_tree_workspace_bytes", "hola_row_stats", "hola_tile_stats",
    "hola_tile_stats_workspace_bytes", "hola_merge_tile_stats", "hola_set_tuning",
    "hola_profile_enable", "hola_profile_collect", "hola_profile_collect_launches", "hola_copy_bytes", "hola_read_probe", "hola_shutdown", "hola_status_string",
    "hola_last_hip_error", "hola_version",
)


class HolaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().hola_status_string(status).decode()
        if status == HOLA_ERR_HIP:
            msg += " (" + lib().hola_last_hip_error().decode() + ")"
        super().__init__(f"{where}: {msg}")


class Tuning(C.Structure):
    _fields_ = [("stats_split", C.c_int32), ("stats_unroll", C.c_int32), ("path", C.c_int32),
                ("fused_waves", C.c_int32), ("filter_path", C.c_int32), ("tail_split", C.c_int32)]


class VerifyArgs(C.Structure):
    _fields_ = [
        ("target_logits", C.c_void_p), ("draft_logits", C.c_void_p), ("dtype", C.c_int32),
        ("target_ld", C.c_int64), ("draft_ld", C.c_int64),
        ("draft_tokens", C.c_void_p), ("draft_len", C.c_void_p), ("row_temperature", C.c_void_p),
        ("draft_stats_in", C.c_void_p), ("target_stats_out", C.c_void_p), ("target_stats_in", C.c_void_p),
        ("top_k", C.c_int32), ("top_p", C.c_float), ("out_keep_count", C.c_void_p),
        ("seed", C.c_uint64), ("level", C.c_uint32), ("seq_base", C.c_int64),
        ("B", C.c_int32), ("gamma", C.c_int32), ("V", C.c_int32),
        ("temperature", C.c_float), ("entropy_threshold", C.c_float),
        ("out_accept_len", C.c_void_p), ("out_next_token", C.c_void_p), ("out_entropy", C.c_void_p),
        ("entropy_ld", C.c_int64),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t), ("stream", C.c_void_p),
        ("tuning", C.POINTER(Tuning)),
    ]


class ModelLogits(C.Structure):
    _fields_ = [("logits", C.c_void_p), ("ld", C.c_int64)]


class HsdArgs(C.Structure):
    _fields_ = [
        ("models", C.POINTER(ModelLogits)), ("n_models", C.c_int32), ("dtype", C.c_int32),
        ("draft_tokens", C.c_void_p), ("seed", C.c_uint64), ("seq_base", C.c_int64),
        ("B", C.c_int32), ("gamma", C.c_int32), ("V", C.c_int32),
        ("row_temperature", C.c_void_p), ("temperature", C.c_float), ("tau", C.POINTER(C.c_float)),
        ("survivors_only", C.c_int32),
        ("out_tokens", C.c_void_p), ("out_accept_len", C.c_void_p), ("out_next_token", C.c_void_p),
        ("out_entropy", C.c_void_p),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t), ("stream", C.c_void_p),
        ("top_k", C.c_int32), ("top_p", C.c_float),
        ("tuning", C.POINTER(Tuning)),
    ]


class TreeArgs(C.Structure):
    _fields_ = [
        ("target_logits", C.c_void_p), ("draft_logits", C.c_void_p), ("dtype", C.c_int32),
        ("target_ld", C.c_int64), ("draft_ld", C.c_int64),
        ("node_token", C.c_void_p), ("node_parent", C.c_void_p), ("n_nodes", C.c_void_p),
        ("seed", C.c_uint64), ("level", C.c_uint32), ("seq_base", C.c_int64),
        ("B", C.c_int32), ("N", C.c_int32), ("V", C.c_int32),
        ("temperature", C.c_float), ("entropy_threshold", C.c_float),
        ("out_accept_len", C.c_void_p), ("out_path", C.c_void_p), ("out_next_token", C.c_void_p),
        ("out_entropy", C.c_void_p),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t), ("stream", C.c_void_p),
        ("tuning", C.POINTER(Tuning)),
    ]


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    """Load libhola.so (built in-tree by ``build.py``).  No fallback: a missing library is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2506_18952_amd.build` "
                              "(or __graft_entry__.build()) first -- there is no CPU fallback")
        L = C.CDLL(LIB_PATH)
        short = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_int32, C.c_int32, C.c_int32,
                 C.c_float, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.hola_verify_f32.argtypes = short
        L.hola_verify_bf16.argtypes = short
        L.hola_verify_ex.argtypes = [C.POINTER(VerifyArgs)]
        L.hola_verify_ex_static.argtypes = [C.POINTER(VerifyArgs)]
        L.hola_verify_ex_static.restype = C.c_int32
        L.hola_verify_literal_ex.argtypes = [C.POINTER(VerifyArgs), C.c_void_p, C.c_void_p]
        L.hola_verify_literal_ex.restype = C.c_int32
        L.hola_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
        L.hola_workspace_bytes.restype = C.c_size_t
        L.hola_workspace_bytes_ex.argtypes = [C.POINTER(VerifyArgs)]
        L.hola_workspace_bytes_ex.restype = C.c_size_t
        L.hola_hsd_verify.argtypes = [C.POINTER(ModelLogits), C.c_int32, C.c_int32, C.c_void_p, C.c_uint64,
                                      C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_float,
                                      C.POINTER(C.c_float), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_size_t, C.c_void_p]
        L.hola_hsd_verify_ex.argtypes = [C.POINTER(HsdArgs)]
        L.hola_hsd_verify_ex.restype = C.c_int32
        L.hola_hsd_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32]
        L.hola_hsd_workspace_bytes.restype = C.c_size_t
        L.hola_verify_tree.argtypes = [C.POINTER(TreeArgs)]
        L.hola_verify_tree.restype = C.c_int32
        L.hola_tree_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
        L.hola_tree_workspace_bytes.restype = C.c_size_t
        L.hola_row_stats.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_int32, C.c_int32, C.c_float,
                                     C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.hola_tile_stats.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_float,
                                      C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.hola_tile_stats.restype = C.c_int32
        L.hola_tile_stats_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
        L.hola_tile_stats_workspace_bytes.restype = C.c_size_t
        L.hola_merge_tile_stats.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.hola_merge_tile_stats.restype = C.c_int32
        L.hola_set_tuning.argtypes = [C.POINTER(Tuning)]
        L.hola_profile_enable.argtypes = [C.c_int32]
        L.hola_profile_collect.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        L.hola_copy_bytes.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.hola_copy_bytes.restype = C.c_int32
        L.hola_read_probe.argtypes = [C.c_void_p, C.c_size_t, C.c_size_t, C.c_int32, C.c_int32, C.c_void_p]
        L.hola_read_probe.restype = C.c_int32
        L.hola_profile_collect_launches.argtypes = [C.POINTER(C.c_int32), C.POINTER(C.c_float), C.c_int64, C.POINTER(C.c_int64)]
        L.hola_profile_collect_launches.restype = C.c_int32
        L.hola_shutdown.argtypes = []
        L.hola_shutdown.restype = None
        for name in ("hola_status_string", "hola_last_hip_error", "hola_version"):
            getattr(L, name).restype = C.c_char_p
        L.hola_status_string.argtypes = [C.c_int32]
        for name in ("hola_verify_f32", "hola_verify_bf16", "hola_verify_ex", "hola_hsd_verify", "hola_row_stats",
                     "hola_set_tuning", "hola_profile_enable", "hola_profile_collect"):
            getattr(L, name).restype = C.c_int32
        _lib = L
    return _lib


# --------------------------------------------------------------------------- marshalling helpers
def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream_handle(stream) -> Optional[int]:
    """HIP stream handle of a torch stream (None => torch's current stream)."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream) or None


def _logit_dtype(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return HOLA_DTYPE_F32
    if t.dtype in (torch.bfloat16, torch.uint16, torch.int16):
        return HOLA_DTYPE_BF16
    raise TypeError(f"logits must be float32 or bfloat16 (or its 16-bit patterns), got {t.dtype}")


def _check(status: int, where: str) -> None:
    if status != HOLA_OK:
        raise HolaError(status, where)


def _need(t, name, device=None):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")


# --------------------------------------------------------------------------- C ABI, same names
def hola_workspace_bytes(B: int, gamma: int, V: int) -> int:
    return int(lib().hola_workspace_bytes(B, gamma, V))


def hola_workspace_bytes_ex(B: int, gamma: int, V: int, top_k: int = 0, top_p: float = 0.0) -> int:
    """Workspace of one call of this shape with these filters (hola_workspace_bytes_ex reads nothing else)."""
    a = VerifyArgs()
    a.B, a.gamma, a.V, a.top_k, a.top_p = int(B), int(gamma), int(V), int(top_k), float(top_p)
    return int(lib().hola_workspace_bytes_ex(C.byref(a)))


def _tuning_ptr(tuning):
    """hola_tuning of one call: None, a Tuning, or a dict of its fields."""
    if tuning is None:
        return None
    if isinstance(tuning, dict):
        tuning = Tuning(**{k: int(v) for k, v in tuning.items()})
    return C.pointer(tuning)


def hola_hsd_workspace_bytes(n_models: int, B: int, gamma: int, V: int) -> int:
    return int(lib().hola_hsd_workspace_bytes(n_models, B, gamma, V))


def _verify_short(fn_name, target_logits, draft_logits, draft_tokens, seed, B, gamma, V, temperature,
                  entropy_threshold, out_accept_len, out_next_token, out_entropy, stream=None):
    for t, n in ((target_logits, "target_logits"), (draft_logits, "draft_logits"), (draft_tokens, "draft_tokens"),
                 (out_accept_len, "out_accept_len"), (out_next_token, "out_next_token"), (out_entropy, "out_entropy")):
        _need(t, n)
    st = getattr(lib(), fn_name)(_ptr(target_logits), _ptr(draft_logits), _ptr(draft_tokens), int(seed), B, gamma, V,
                                 float(temperature), float(entropy_threshold), _ptr(out_accept_len),
                                 _ptr(out_next_token), _ptr(out_entropy), _stream_handle(stream))
    _check(st, fn_name)


def hola_verify_f32(target_logits, draft_logits, draft_tokens, seed, B, gamma, V, temperature, entropy_threshold,
                    out_accept_len, out_next_token, out_entropy, stream=None) -> None:
    _verify_short("hola_verify_f32", target_logits, draft_logits, draft_tokens, seed, B, gamma, V, temperature,
                  entropy_threshold, out_accept_len, out_next_token, out_entropy, stream)


def hola_verify_bf16(target_logits, draft_logits, draft_tokens, seed, B, gamma, V, temperature, entropy_threshold,
                     out_accept_len, out_next_token, out_entropy, stream=None) -> None:
    _verify_short("hola_verify_bf16", target_logits, draft_logits, draft_tokens, seed, B, gamma, V, temperature,
                  entropy_threshold, out_accept_len, out_next_token, out_entropy, stream)


def hola_verify_ex(*, target_logits, draft_logits, draft_tokens, seed, B, gamma, V, temperature, entropy_threshold,
                   out_accept_len, out_next_token, out_entropy=None, workspace, draft_len=None,
                   row_temperature=None, draft_stats_in=None, target_stats_out=None, target_stats_in=None, level=0,
                   seq_base=0, target_ld=0, draft_ld=0, entropy_ld=0, top_k=0, top_p=0.0, out_keep_count=None,
                   stream=None, tuning=None, _entry="hola_verify_ex") -> None:
    a = VerifyArgs()
    a.tuning = _tuning_ptr(tuning)
    a.target_logits, a.draft_logits = _ptr(target_logits), _ptr(draft_logits)
    a.dtype = _logit_dtype(target_logits)
    a.target_ld, a.draft_ld = int(target_ld), int(draft_ld)
    a.draft_tokens, a.draft_len = _ptr(draft_tokens), _ptr(draft_len)
    a.row_temperature = _ptr(row_temperature)
    a.draft_stats_in, a.target_stats_out = _ptr(draft_stats_in), _ptr(target_stats_out)
    a.target_stats_in = _ptr(target_stats_in)
    a.top_k, a.top_p, a.out_keep_count = int(top_k), float(top_p), _ptr(out_keep_count)
    a.seed, a.level, a.seq_base = int(seed), int(level), int(seq_base)
    a.B, a.gamma, a.V = int(B), int(gamma), int(V)
    a.temperature, a.entropy_threshold = float(temperature), float(entropy_threshold)
    a.out_accept_len, a.out_next_token, a.out_entropy = _ptr(out_accept_len), _ptr(out_next_token), _ptr(out_entropy)
    a.entropy_ld = int(entropy_ld)
    a.workspace = _ptr(workspace)
    a.workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    a.stream = _stream_handle(stream)
    _check(getattr(lib(), _entry)(C.byref(a)), _entry)


HOLA_STATIC_SCRATCH_BYTES = 16 << 20


def hola_verify_ex_static(**kw) -> None:
    """hola_verify_ex on the library's static scratch array: same keyword arguments, no workspace."""
    kw.setdefault("workspace", None)
    hola_verify_ex(_entry="hola_verify_ex_static", **kw)


def hola_verify_literal_ex(*, target_logits, draft_logits, draft_tokens, seed, B, gamma, V, temperature,
                           entropy_threshold, out_tokens, out_verifier_calls=None, out_entropy=None, workspace,
                           draft_len=None, row_temperature=None, level=0, seq_base=0, target_ld=0, draft_ld=0,
                           entropy_ld=0, stream=None, tuning=None) -> None:
    a = VerifyArgs()
    a.tuning = _tuning_ptr(tuning)
    a.target_logits, a.draft_logits = _ptr(target_logits), _ptr(draft_logits)
    a.dtype = _logit_dtype(target_logits)
    a.target_ld, a.draft_ld = int(target_ld), int(draft_ld)
    a.draft_tokens, a.draft_len = _ptr(draft_tokens), _ptr(draft_len)
    a.row_temperature = _ptr(row_temperature)
    a.seed, a.level, a.seq_base = int(seed), int(level), int(seq_base)
    a.B, a.gamma, a.V = int(B), int(gamma), int(V)
    a.temperature, a.entropy_threshold = float(temperature), float(entropy_threshold)
    a.out_entropy, a.entropy_ld = _ptr(out_entropy), int(entropy_ld)
    a.workspace = _ptr(workspace)
    a.workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    a.stream = _stream_handle(stream)
    _check(lib().hola_verify_literal_ex(C.byref(a), _ptr(out_tokens), _ptr(out_verifier_calls)), "hola_verify_literal_ex")


def hola_hsd_verify(models: Sequence, draft_tokens, seed, B, gamma, V, temperature, tau: Sequence[float],
                    out_tokens, out_accept_len, out_next_token, out_entropy, workspace,
                    row_temperature=None, seq_base=0, lds: Optional[Sequence[int]] = None, stream=None) -> None:
    n = len(models)
    arr = (ModelLogits * n)()
    for k, m in enumerate(models):
        arr[k].logits = _ptr(m)
        arr[k].ld = int(lds[k]) if lds else 0
    taus = (C.c_float * (n - 1))(*[float(x) for x in tau])
    st = lib().hola_hsd_verify(arr, n, _logit_dtype(models[0]), _ptr(draft_tokens), int(seed), int(seq_base),
                               int(B), int(gamma), int(V), _ptr(row_temperature), float(temperature), taus,
                               _ptr(out_tokens), _ptr(out_accept_len), _ptr(out_next_token), _ptr(out_entropy),
                               _ptr(workspace), workspace.numel() * workspace.element_size(), _stream_handle(stream))
    _check(st, "hola_hsd_verify")


def hola_hsd_verify_ex(models: Sequence, draft_tokens, seed, B, gamma, V, temperature, tau: Sequence[float],
                       out_tokens, out_accept_len, out_next_token, out_entropy, workspace, survivors_only=False,
                       row_temperature=None, seq_base=0, lds: Optional[Sequence[int]] = None, stream=None,
                       top_k=0, top_p=0.0, tuning=None) -> None:
    n = len(models)
    arr = (ModelLogits * n)()
    for k, m in enumerate(models):
        arr[k].logits = _ptr(m)
        arr[k].ld = int(lds[k]) if lds else 0
    taus = (C.c_float * (n - 1))(*[float(x) for x in tau])
    a = HsdArgs()
    a.models, a.n_models, a.dtype = arr, n, _logit_dtype(models[0])
    a.draft_tokens, a.seed, a.seq_base = _ptr(draft_tokens), int(seed), int(seq_base)
    a.B, a.gamma, a.V = int(B), int(gamma), int(V)
    a.row_temperature, a.temperature, a.tau = _ptr(row_temperature), float(temperature), taus
    a.survivors_only = 1 if survivors_only else 0
    a.out_tokens, a.out_accept_len, a.out_next_token = _ptr(out_tokens), _ptr(out_accept_len), _ptr(out_next_token)
    a.out_entropy = _ptr(out_entropy)
    a.workspace, a.workspace_bytes = _ptr(workspace), workspace.numel() * workspace.element_size()
    a.stream = _stream_handle(stream)
    a.top_k, a.top_p = int(top_k), float(top_p)
    a.tuning = _tuning_ptr(tuning)
    _check(lib().hola_hsd_verify_ex(C.byref(a)), "hola_hsd_verify_ex")


def hola_tree_workspace_bytes(B: int, N: int, V: int) -> int:
    return int(lib().hola_tree_workspace_bytes(B, N, V))


def hola_verify_tree(target_logits, draft_logits, node_token, node_parent, seed, B, N, V, temperature,
                     entropy_threshold, out_accept_len, out_next_token, workspace, out_path=None, out_entropy=None,
                     n_nodes=None, level=0, seq_base=0, target_ld=0, draft_ld=0, stream=None, tuning=None) -> None:
    a = TreeArgs()
    a.tuning = _tuning_ptr(tuning)
    a.target_logits, a.draft_logits, a.dtype = _ptr(target_logits), _ptr(draft_logits), _logit_dtype(target_logits)
    a.target_ld, a.draft_ld = int(target_ld), int(draft_ld)
    a.node_token, a.node_parent, a.n_nodes = _ptr(node_token), _ptr(node_parent), _ptr(n_nodes)
    a.seed, a.level, a.seq_base = int(seed), int(level), int(seq_base)
    a.B, a.N, a.V = int(B), int(N), int(V)
    a.temperature, a.entropy_threshold = float(temperature), float(entropy_threshold)
    a.out_accept_len, a.out_path, a.out_next_token = _ptr(out_accept_len), _ptr(out_path), _ptr(out_next_token)
    a.out_entropy = _ptr(out_entropy)
    a.workspace, a.workspace_bytes = _ptr(workspace), workspace.numel() * workspace.element_size()
    a.stream = _stream_handle(stream)
    _check(lib().hola_verify_tree(C.byref(a)), "hola_verify_tree")


def hola_row_stats(logits, R, V, temperature, stats_out, workspace, ld=0, stream=None) -> None:
    st = lib().hola_row_stats(_ptr(logits), _logit_dtype(logits), int(ld), int(R), int(V), float(temperature),
                              _ptr(stats_out), _ptr(workspace), workspace.numel() * workspace.element_size(),
                              _stream_handle(stream))
    _check(st, "hola_row_stats")


def hola_tile_stats_workspace_bytes(R: int, V: int, tile_cols: int) -> int:
    return int(lib().hola_tile_stats_workspace_bytes(int(R), int(V), int(tile_cols)))


def hola_tile_stats(logits, R, V, tile_cols, temperature, tile_stats_out, workspace, ld=0, stream=None) -> None:
    st = lib().hola_tile_stats(_ptr(logits), _logit_dtype(logits), int(ld), int(R), int(V), int(tile_cols),
                               float(temperature), _ptr(tile_stats_out), _ptr(workspace),
                               workspace.numel() * workspace.element_size(), _stream_handle(stream))
    _check(st, "hola_tile_stats")


def hola_merge_tile_stats(tile_stats, R, ntiles, stats_out, stream=None) -> None:
    st = lib().hola_merge_tile_stats(_ptr(tile_stats), int(R), int(ntiles), _ptr(stats_out), _stream_handle(stream))
    _check(st, "hola_merge_tile_stats")


PATH_AUTO, PATH_SPLIT, PATH_FUSED, PATH_SPLIT4 = 0, 1, 2, 3


def hola_set_tuning(stats_split: int = 0, stats_unroll: int = 0, path: int = 0, fused_waves: int = 0,
                    filter_path: int = 0, tail_split: int = 0) -> None:
    t = Tuning(int(stats_split), int(stats_unroll), int(path), int(fused_waves), int(filter_path), int(tail_split))
    _check(lib().hola_set_tuning(C.byref(t)), "hola_set_tuning")


def hola_profile_enable(on: bool) -> None:
    _check(lib().hola_profile_enable(1 if on else 0), "hola_profile_enable")


def hola_profile_collect() -> tuple[list[float], list[int]]:
    ms = (C.c_double * HOLA_N_STAGES)()
    n = (C.c_int64 * HOLA_N_STAGES)()
    _check(lib().hola_profile_collect(ms, n), "hola_profile_collect")
    return list(ms), list(n)


def hola_profile_collect_launches(capacity: int = 1 << 16) -> list[tuple[int, float]]:
    """(stage, milliseconds) of every kernel recorded since the last collect, in launch order."""
    st = (C.c_int32 * capacity)()
    ms = (C.c_float * capacity)()
    n = C.c_int64(0)
    _check(lib().hola_profile_collect_launches(st, ms, capacity, C.byref(n)), "hola_profile_collect_launches")
    k = min(int(n.value), capacity)
    return [(int(st[i]), float(ms[i])) for i in range(k)]


def hola_read_probe(src, nbytes: int, block_bytes: int, nontemporal: bool = True, arithmetic: bool = False, stream=None) -> None:
    _check(lib().hola_read_probe(_ptr(src), int(nbytes), int(block_bytes), 1 if nontemporal else 0, 1 if arithmetic else 0,
                                 _stream_handle(stream)), "hola_read_probe")


def hola_copy_bytes(dst, src, nbytes: int, stream=None) -> None:
    _check(lib().hola_copy_bytes(_ptr(dst), _ptr(src), int(nbytes), _stream_handle(stream)), "hola_copy_bytes")


def hola_shutdown() -> None:
    lib().hola_shutdown()


def hola_version() -> str:
    return lib().hola_version().decode()


def alloc_workspace(nbytes: int, device="cuda:0"):
    """Device buffer for a workspace (torch memory; 256-byte alignment comes with the allocator)."""
    import torch
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
