"""ctypes front end of the float64 CPU oracle (``hola_oracle.c``).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only ``tests/``, the smoke check and the
benchmark's CPU-baseline leg may import this module.  It shares nothing with the
HIP path.  The arithmetic lives in the C file; this module only marshals numpy
arrays (argument passing, no method steps).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hola_oracle.c")
_LIB = os.path.join(_HERE, "libhola_oracle.so")

F32, BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math, OpenMP over sequences)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Args(C.Structure):
    _fields_ = [
        ("target_logits", C.c_void_p), ("draft_logits", C.c_void_p), ("dtype", C.c_int32),
        ("target_ld", C.c_int64), ("draft_ld", C.c_int64),
        ("draft_tokens", C.c_void_p), ("draft_len", C.c_void_p), ("row_temperature", C.c_void_p),
        ("force_accept_len", C.c_void_p),
        ("seed", C.c_uint64), ("level", C.c_uint32), ("seq_base", C.c_int64),
        ("B", C.c_int32), ("gamma", C.c_int32), ("V", C.c_int32),
        ("temperature", C.c_float), ("entropy_threshold", C.c_float),
        ("out_accept_len", C.c_void_p), ("out_next_token", C.c_void_p), ("out_entropy", C.c_void_p),
        ("out_entropy64", C.c_void_p), ("out_lse_draft", C.c_void_p), ("out_lse_target", C.c_void_p),
        ("out_H_target", C.c_void_p),
        ("out_gate", C.c_void_p), ("out_ratio_ok", C.c_void_p),
        ("out_gate_margin", C.c_void_p), ("out_ratio_margin", C.c_void_p),
        ("out_sample_margin", C.c_void_p), ("out_Z", C.c_void_p),
        ("num_threads", C.c_int32),
    ]


class _TreeArgs(C.Structure):
    _fields_ = [
        ("target_logits", C.c_void_p), ("draft_logits", C.c_void_p), ("dtype", C.c_int32),
        ("target_ld", C.c_int64), ("draft_ld", C.c_int64),
        ("node_token", C.c_void_p), ("node_parent", C.c_void_p), ("n_nodes", C.c_void_p),
        ("seed", C.c_uint64), ("level", C.c_uint32), ("seq_base", C.c_int64),
        ("B", C.c_int32), ("N", C.c_int32), ("V", C.c_int32),
        ("temperature", C.c_float), ("entropy_threshold", C.c_float),
        ("out_accept_len", C.c_void_p), ("out_path", C.c_void_p), ("out_next_token", C.c_void_p),
        ("out_entropy", C.c_void_p), ("out_entropy64", C.c_void_p),
        ("out_gate_margin", C.c_void_p), ("out_ratio_margin", C.c_void_p), ("out_sample_margin", C.c_void_p),
        ("num_threads", C.c_int32),
        ("force_node", C.c_void_p), ("force_outcome", C.c_void_p), ("probe_token", C.c_void_p),
        ("out_probe_lo", C.c_void_p), ("out_probe_hi", C.c_void_p),
    ]


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.oracle_philox4x32_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_philox4x32_10.restype = None
        L.oracle_u24.argtypes = [C.c_uint32]
        L.oracle_u24.restype = C.c_double
        L.oracle_row_stats.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_int32, C.c_double,
                                       C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_row_stats.restype = None
        L.oracle_merge_tile_stats.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        L.oracle_merge_tile_stats.restype = None
        L.oracle_ratio_accept.argtypes = [C.c_double, C.c_double, C.c_double]
        L.oracle_ratio_accept.restype = C.c_int32
        L.oracle_inverse_cdf.argtypes = [C.c_void_p, C.c_int32, C.c_double, C.c_void_p, C.c_void_p]
        L.oracle_inverse_cdf.restype = C.c_int32
        L.oracle_ratio_accept_lattice_count.argtypes = [C.c_double, C.c_double, C.c_int32]
        L.oracle_ratio_accept_lattice_count.restype = C.c_int64
        L.oracle_inverse_cdf_lattice_hist.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        L.oracle_inverse_cdf_lattice_hist.restype = None
        L.oracle_residual_weights.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int64,
                                              C.c_int32, C.c_double, C.c_double, C.c_double, C.c_int32,
                                              C.c_void_p]
        L.oracle_residual_weights.restype = None
        L.oracle_verify.argtypes = [C.POINTER(_Args)]
        L.oracle_verify.restype = C.c_int32
        L.oracle_filter_row.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_int32, C.c_double, C.c_int32,
                                        C.c_double, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_filter_row.restype = C.c_int32
        L.oracle_verify_filtered.argtypes = [C.POINTER(_Args), C.c_int32, C.c_double, C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_verify_filtered.restype = C.c_int32
        L.oracle_sample_interval.argtypes = [C.POINTER(_Args), C.c_int32, C.c_int32, C.c_int32,
                                             C.c_void_p, C.c_void_p]
        L.oracle_sample_interval.restype = C.c_int32
        L.oracle_sample_interval_filtered.argtypes = [C.POINTER(_Args), C.c_int32, C.c_double, C.c_void_p, C.c_int32,
                                                      C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.oracle_sample_interval_filtered.restype = C.c_int32
        L.oracle_row_interval.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_int32, C.c_double, C.c_int32,
                                          C.c_void_p, C.c_void_p]
        L.oracle_row_interval.restype = C.c_int32
        L.oracle_hsd_verify.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                        C.c_uint64, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                                        C.c_void_p, C.c_float, C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_double, C.c_int32]
        L.oracle_hsd_verify.restype = C.c_int32
        L.oracle_verify_literal.argtypes = [C.POINTER(_Args), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_verify_literal.restype = C.c_int32
        L.oracle_verify_tree.argtypes = [C.POINTER(_TreeArgs)]
        L.oracle_verify_tree.restype = C.c_int32
        L.oracle_max_threads.argtypes = []
        L.oracle_max_threads.restype = C.c_int32
        _lib = L
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def _logits(a: np.ndarray) -> tuple[np.ndarray, int]:
    """Accept float32 logits or bf16 logits given as uint16 bit patterns."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float32:
        return a, F32
    if a.dtype == np.uint16:
        return a, BF16
    raise TypeError(f"logits must be float32 or uint16 (bf16 bits), got {a.dtype}")


def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> tuple[int, int, int, int]:
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return tuple(int(x) for x in out)


def u24(r: int) -> float:
    return float(lib().oracle_u24(C.c_uint32(r)))


def hsd_uniforms(seed: int, seq: int, pos: int, level: int = 0) -> tuple[float, float]:
    """(accept uniform, sampling uniform) of one (sequence, position, level)."""
    r = philox4x32_10([pos & 0xFFFFFFFF, seq & 0xFFFFFFFF, (seq >> 32) & 0xFFFFFFFF, level],
                      [seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF])
    return u24(r[0]), u24(r[1])


def row_stats(row: np.ndarray, T: float = 1.0) -> tuple[float, float, int]:
    """(lse, entropy in nats, argmax) of softmax(row / T); T == 0 means T = 1 (greedy rows)."""
    row, dt = _logits(row)
    lse, H, am = C.c_double(), C.c_double(), C.c_int32()
    lib().oracle_row_stats(_ptr(row), dt, 0, row.shape[-1], float(T),
                           C.addressof(lse), C.addressof(H), C.addressof(am))
    return lse.value, H.value, am.value


def tile_stats(rows: np.ndarray, tile_cols: int, T: float = 1.0) -> np.ndarray:
    """(lse_t, H_t) of every column tile [t*tile_cols, min(V, (t+1)*tile_cols)) of every row: [R, ntiles, 2].
    Each tile is a row of its own to oracle_row_stats."""
    rows, dt = _logits(rows)
    rows = rows.reshape(-1, rows.shape[-1])
    R, V = rows.shape
    nt = (V + tile_cols - 1) // tile_cols
    out = np.empty((R, nt, 2), dtype=np.float64)
    lse, H = C.c_double(), C.c_double()
    for r in range(R):
        for t in range(nt):
            c0 = t * tile_cols
            lib().oracle_row_stats(_ptr(rows), dt, r * V + c0, min(tile_cols, V - c0), float(T),
                                   C.addressof(lse), C.addressof(H), None)
            out[r, t] = (lse.value, H.value)
    return out


def merge_tile_stats(ts: np.ndarray) -> np.ndarray:
    """[R, ntiles, 2] tile statistics -> [R, 2] row statistics (entropy chain rule)."""
    ts = np.ascontiguousarray(ts, dtype=np.float64)
    R, nt, _ = ts.shape
    out = np.empty((R, 2), dtype=np.float64)
    lse, H = C.c_double(), C.c_double()
    for r in range(R):
        lib().oracle_merge_tile_stats(ts[r].ctypes.data, nt, C.addressof(lse), C.addressof(H))
        out[r] = (lse.value, H.value)
    return out


def ratio_accept(u: float, p_x: float, q_x: float) -> bool:
    return bool(lib().oracle_ratio_accept(u, p_x, q_x))


def inverse_cdf(w: np.ndarray, u: float) -> tuple[int, float, float]:
    """(token, Z, margin) of the inverse-CDF draw from unnormalised weights w."""
    w = np.ascontiguousarray(w, dtype=np.float64)
    Z, m = C.c_double(), C.c_double()
    tok = lib().oracle_inverse_cdf(_ptr(w), w.shape[0], float(u), C.addressof(Z), C.addressof(m))
    return int(tok), Z.value, m.value


def ratio_accept_lattice_count(p_x: float, q_x: float, stride: int = 1) -> int:
    """Number of lattice uniforms k*stride*2^-24 that pass the acceptance test."""
    return int(lib().oracle_ratio_accept_lattice_count(float(p_x), float(q_x), int(stride)))


def inverse_cdf_lattice_hist(w: np.ndarray, stride: int = 1) -> np.ndarray:
    """How many lattice uniforms select each token."""
    w = np.ascontiguousarray(w, dtype=np.float64)
    hist = np.zeros(w.shape[0], dtype=np.int64)
    lib().oracle_inverse_cdf_lattice_hist(_ptr(w), w.shape[0], int(stride), _ptr(hist))
    return hist


def residual_weights(target_row: np.ndarray, draft_row: Optional[np.ndarray], T: float,
                     bonus: bool = False) -> np.ndarray:
    """max(0, p - q) over one position (or p itself when bonus)."""
    target_row, dt = _logits(target_row)
    V = target_row.shape[-1]
    lseP, _, _ = row_stats(target_row, T)
    if bonus:
        draft_row, lseD = target_row, 0.0
    else:
        draft_row, dt2 = _logits(draft_row)
        assert dt2 == dt
        lseD, _, _ = row_stats(draft_row, T)
    w = np.zeros(V, dtype=np.float64)
    lib().oracle_residual_weights(_ptr(target_row), _ptr(draft_row), dt, 0, 0, V, float(T),
                                  lseP, lseD, int(bonus), _ptr(w))
    return w


@dataclass
class VerifyResult:
    accept_len: np.ndarray
    next_token: np.ndarray
    entropy: np.ndarray          # float32 [B, gamma]
    entropy64: np.ndarray        # float64 [B, gamma]
    lse_draft: np.ndarray
    lse_target: np.ndarray
    H_target: np.ndarray
    gate: np.ndarray
    ratio_ok: np.ndarray
    gate_margin: np.ndarray
    ratio_margin: np.ndarray
    sample_margin: np.ndarray
    Z: np.ndarray
    filter_margin: Optional[np.ndarray] = None   # [B, 2 gamma + 1], filtered step only
    keep_count: Optional[np.ndarray] = None


class VerifyCall:
    """Holds the marshalled arguments of one ``oracle_verify`` call (keeps arrays alive)."""

    def __init__(self, target_logits, draft_logits, draft_tokens, seed, temperature, entropy_threshold,
                 draft_len=None, row_temperature=None, level=0, seq_base=0, force_accept_len=None,
                 num_threads=0):
        self.P, dt = _logits(target_logits)
        self.D, dt2 = _logits(draft_logits)
        assert dt == dt2, "target and draft logits must share a dtype"
        B, g1, V = self.P.shape
        g = g1 - 1
        assert self.D.shape == (B, g, V), (self.D.shape, (B, g, V))
        self.tok = np.ascontiguousarray(draft_tokens, dtype=np.int32)
        assert self.tok.shape == (B, g)
        self.len = None if draft_len is None else np.ascontiguousarray(draft_len, dtype=np.int32)
        self.rowT = None if row_temperature is None else np.ascontiguousarray(row_temperature, dtype=np.float32)
        self.force = None if force_accept_len is None else np.ascontiguousarray(force_accept_len, dtype=np.int32)
        self.B, self.g, self.V = B, g, V
        a = _Args()
        a.target_logits, a.draft_logits, a.dtype = _ptr(self.P), _ptr(self.D), dt
        a.target_ld = a.draft_ld = 0
        a.draft_tokens, a.draft_len = _ptr(self.tok), _ptr(self.len)
        a.row_temperature, a.force_accept_len = _ptr(self.rowT), _ptr(self.force)
        a.seed, a.level, a.seq_base = int(seed), int(level), int(seq_base)
        a.B, a.gamma, a.V = B, g, V
        a.temperature, a.entropy_threshold = float(temperature), float(entropy_threshold)
        a.num_threads = int(num_threads)
        self.args = a

    def run(self, top_k: Optional[int] = None, top_p: Optional[float] = None,
            force_keep_count: Optional[np.ndarray] = None) -> VerifyResult:
        """top_k / top_p given: the step on filtered distributions (oracle_verify_filtered)."""
        B, g = self.B, self.g
        r = VerifyResult(
            accept_len=np.zeros(B, np.int32), next_token=np.zeros(B, np.int32),
            entropy=np.zeros((B, g), np.float32), entropy64=np.zeros((B, g), np.float64),
            lse_draft=np.zeros((B, g), np.float64), lse_target=np.zeros((B, g + 1), np.float64),
            H_target=np.zeros((B, g + 1), np.float64),
            gate=np.zeros((B, g), np.uint8), ratio_ok=np.zeros((B, g), np.uint8),
            gate_margin=np.zeros((B, g), np.float64), ratio_margin=np.zeros((B, g), np.float64),
            sample_margin=np.zeros(B, np.float64), Z=np.zeros(B, np.float64))
        a = self.args
        a.out_accept_len, a.out_next_token = _ptr(r.accept_len), _ptr(r.next_token)
        a.out_entropy, a.out_entropy64 = _ptr(r.entropy), _ptr(r.entropy64)
        a.out_lse_draft, a.out_lse_target, a.out_H_target = _ptr(r.lse_draft), _ptr(r.lse_target), _ptr(r.H_target)
        a.out_gate, a.out_ratio_ok = _ptr(r.gate), _ptr(r.ratio_ok)
        a.out_gate_margin, a.out_ratio_margin = _ptr(r.gate_margin), _ptr(r.ratio_margin)
        a.out_sample_margin, a.out_Z = _ptr(r.sample_margin), _ptr(r.Z)
        if top_k is None and top_p is None:
            rc = lib().oracle_verify(C.byref(a))
        else:
            R = 2 * g + 1
            r.filter_margin = np.zeros((B, R), np.float64)
            r.keep_count = np.zeros((B, R), np.int32)
            fk = None if force_keep_count is None else np.ascontiguousarray(force_keep_count, np.int32).reshape(B, R)
            rc = lib().oracle_verify_filtered(C.byref(a), int(top_k or 0), float(1.0 if top_p is None else top_p),
                                              _ptr(r.filter_margin), _ptr(r.keep_count), _ptr(fk))
        if rc != 0:
            raise ValueError("the oracle rejected its arguments")
        return r

    def sample_interval(self, b: int, acc_len: int, tok: int, top_k: Optional[int] = None,
                        top_p: Optional[float] = None, force_keep_count: Optional[np.ndarray] = None
                        ) -> Optional[tuple[float, float]]:
        """CDF interval of `tok` in the distribution the stop row `acc_len` of sequence b is sampled from
        (top_k / top_p given: on the filtered distributions, keep counts as forced)."""
        lo, hi = C.c_double(), C.c_double()
        if top_k is None and top_p is None:
            rc = lib().oracle_sample_interval(C.byref(self.args), int(b), int(acc_len), int(tok),
                                              C.addressof(lo), C.addressof(hi))
        else:
            fk = None if force_keep_count is None else np.ascontiguousarray(force_keep_count, np.int32)
            rc = lib().oracle_sample_interval_filtered(C.byref(self.args), int(top_k or 0),
                                                       float(1.0 if top_p is None else top_p), _ptr(fk), int(b),
                                                       int(acc_len), int(tok), C.addressof(lo), C.addressof(hi))
        return None if rc != 0 else (lo.value, hi.value)


def verify(target_logits, draft_logits, draft_tokens, seed, temperature, entropy_threshold, **kw) -> VerifyResult:
    return VerifyCall(target_logits, draft_logits, draft_tokens, seed, temperature, entropy_threshold, **kw).run()


def verify_filtered(target_logits, draft_logits, draft_tokens, seed, temperature, entropy_threshold, top_k=0,
                    top_p=1.0, force_keep_count=None, **kw) -> VerifyResult:
    call = VerifyCall(target_logits, draft_logits, draft_tokens, seed, temperature, entropy_threshold, **kw)
    return call.run(top_k=top_k, top_p=top_p, force_keep_count=force_keep_count)


def filter_row(row: np.ndarray, T: float = 1.0, top_k: int = 0, top_p: float = 1.0):
    """(keep mask [V] bool, lse and entropy of the kept, renormalised tokens, nucleus cut margin)."""
    row, dt = _logits(row)
    V = row.shape[-1]
    keep = np.zeros(V, np.uint8)
    lse, H, mg = C.c_double(), C.c_double(), C.c_double()
    n = lib().oracle_filter_row(_ptr(row), dt, 0, V, float(T), int(top_k), float(top_p), -1, _ptr(keep),
                                C.addressof(lse), C.addressof(H), C.addressof(mg))
    assert n == int(keep.sum())
    return keep.astype(bool), lse.value, H.value, mg.value


@dataclass
class HsdResult:
    tokens: np.ndarray           # [B, gamma + n_models - 1]
    accept_len: np.ndarray       # [B]
    next_token: np.ndarray       # [B]
    entropy: np.ndarray          # [n_models-1, B, gamma + n_models - 2]
    level_accept: np.ndarray     # [n_models-1, B]
    level_next: np.ndarray       # [n_models-1, B]


def hsd_verify(models: Sequence[np.ndarray], draft_tokens, seed, temperature, tau: Sequence[float],
               row_temperature=None, seq_base=0, survivors_only=False, num_threads=0,
               top_k=0, top_p=1.0) -> HsdResult:
    """Hierarchical verify: models[0] is the smallest drafter [B,gamma,V], models[k] has gamma+k rows.
    top_k / top_p: every level runs the filtered step on its pair of models."""
    arrs, dts = zip(*[_logits(m) for m in models])
    assert len(set(dts)) == 1
    n = len(arrs)
    B, g, V = arrs[0].shape
    for k, m in enumerate(arrs):
        assert m.shape == (B, g + k, V), (k, m.shape)
    tok = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    rowT = None if row_temperature is None else np.ascontiguousarray(row_temperature, dtype=np.float32)
    tau_a = np.ascontiguousarray(tau, dtype=np.float32)
    assert tau_a.shape == (n - 1,)
    ptrs = (C.c_void_p * n)(*[m.ctypes.data for m in arrs])
    L, gmax = n - 1, g + n - 2
    r = HsdResult(tokens=np.zeros((B, g + n - 1), np.int32), accept_len=np.zeros(B, np.int32),
                  next_token=np.zeros(B, np.int32), entropy=np.zeros((L, B, gmax), np.float32),
                  level_accept=np.zeros((L, B), np.int32), level_next=np.zeros((L, B), np.int32))
    rc = lib().oracle_hsd_verify(C.addressof(ptrs), None, n, dts[0], _ptr(tok), int(seed), int(seq_base),
                                 B, g, V, _ptr(rowT), float(temperature), _ptr(tau_a),
                                 _ptr(r.tokens), _ptr(r.accept_len), _ptr(r.next_token), _ptr(r.entropy),
                                 _ptr(r.level_accept), _ptr(r.level_next), int(bool(survivors_only)),
                                 int(top_k or 0), float(1.0 if top_p is None else top_p), int(num_threads))
    if rc != 0:
        raise ValueError("oracle_hsd_verify rejected its arguments")
    return r


@dataclass
class LiteralResult:
    tokens: np.ndarray           # [B, gamma]
    calls: np.ndarray            # [B] verifier invocations
    entropy: np.ndarray          # float32 [B, gamma]
    entropy64: np.ndarray
    gate: np.ndarray
    gate_margin: np.ndarray
    sample_margin: np.ndarray    # [B, gamma], NaN where no sample was drawn


def row_interval(row: np.ndarray, T: float, tok: int) -> Optional[tuple[float, float]]:
    """CDF interval [C_{tok-1}, C_tok] / Z of `tok` under softmax(row / T), ascending index order."""
    row, dt = _logits(row)
    lo, hi = C.c_double(), C.c_double()
    rc = lib().oracle_row_interval(_ptr(row), dt, 0, row.shape[-1], float(T), int(tok), C.addressof(lo), C.addressof(hi))
    return None if rc != 0 else (lo.value, hi.value)


def verify_literal(target_logits, draft_logits, draft_tokens, seed, temperature, entropy_threshold, force_gate=None,
                   **kw) -> LiteralResult:
    """Equation (1) without stopping: gate keeps the draft token, otherwise a draw from the target row.
    force_gate [B, gamma] int8 (test aid): 0 / 1 overrides that position's gate, -1 leaves it."""
    call = VerifyCall(target_logits, draft_logits, draft_tokens, seed, temperature, entropy_threshold, **kw)
    B, g = call.B, call.g
    r = LiteralResult(tokens=np.zeros((B, g), np.int32), calls=np.zeros(B, np.int32),
                      entropy=np.zeros((B, g), np.float32), entropy64=np.zeros((B, g), np.float64),
                      gate=np.zeros((B, g), np.uint8), gate_margin=np.zeros((B, g), np.float64),
                      sample_margin=np.zeros((B, g), np.float64))
    a = call.args
    a.out_entropy, a.out_entropy64 = _ptr(r.entropy), _ptr(r.entropy64)
    a.out_gate, a.out_gate_margin = _ptr(r.gate), _ptr(r.gate_margin)
    fg = None if force_gate is None else np.ascontiguousarray(force_gate, np.int8).reshape(B, g)
    rc = lib().oracle_verify_literal(C.byref(a), _ptr(r.tokens), _ptr(r.calls), _ptr(r.sample_margin), _ptr(fg))
    if rc != 0:
        raise ValueError("oracle_verify_literal rejected its arguments")
    return r


@dataclass
class TreeResult:
    accept_len: np.ndarray       # [B] kept nodes
    path: np.ndarray             # [B, N] kept nodes from the prefix on, -1 beyond
    next_token: np.ndarray       # [B]
    entropy: np.ndarray          # float32 [B, N], -1 for contexts without children
    entropy64: np.ndarray
    gate_margin: np.ndarray      # [B, N] per context, NaN where not visited
    ratio_margin: np.ndarray     # [B, N] per node, NaN where not tested
    sample_margin: np.ndarray    # [B]
    probe_lo: Optional[np.ndarray] = None   # [B] CDF interval of probe_token in the final draw (NaN: not asked)
    probe_hi: Optional[np.ndarray] = None


def verify_tree(target_logits, draft_logits, node_token, node_parent, seed, temperature, entropy_threshold,
                n_nodes=None, level=0, seq_base=0, num_threads=0, force_node=None, force_outcome=None,
                probe_token=None) -> TreeResult:
    """Verify step over token trees: target [B,N+1,V] and draft [B,N,V] rows by context (0: the prefix,
    n+1: after node n), node_parent -1 or an earlier node; children are tried in node order."""
    P, dt = _logits(target_logits)
    D, dt2 = _logits(draft_logits)
    assert dt == dt2
    B, N1, V = P.shape
    N = N1 - 1
    assert D.shape == (B, N, V), (D.shape, (B, N, V))
    tok = np.ascontiguousarray(node_token, dtype=np.int32)
    par = np.ascontiguousarray(node_parent, dtype=np.int32)
    assert tok.shape == (B, N) and par.shape == (B, N)
    nn = None if n_nodes is None else np.ascontiguousarray(n_nodes, dtype=np.int32)
    r = TreeResult(accept_len=np.zeros(B, np.int32), path=np.zeros((B, N), np.int32), next_token=np.zeros(B, np.int32),
                   entropy=np.zeros((B, N), np.float32), entropy64=np.zeros((B, N), np.float64),
                   gate_margin=np.zeros((B, N), np.float64), ratio_margin=np.zeros((B, N), np.float64),
                   sample_margin=np.zeros(B, np.float64))
    a = _TreeArgs()
    a.target_logits, a.draft_logits, a.dtype = _ptr(P), _ptr(D), dt
    a.target_ld = a.draft_ld = 0
    a.node_token, a.node_parent, a.n_nodes = _ptr(tok), _ptr(par), _ptr(nn)
    a.seed, a.level, a.seq_base = int(seed), int(level), int(seq_base)
    a.B, a.N, a.V = B, N, V
    a.temperature, a.entropy_threshold = float(temperature), float(entropy_threshold)
    a.out_accept_len, a.out_path, a.out_next_token = _ptr(r.accept_len), _ptr(r.path), _ptr(r.next_token)
    a.out_entropy, a.out_entropy64 = _ptr(r.entropy), _ptr(r.entropy64)
    a.out_gate_margin, a.out_ratio_margin = _ptr(r.gate_margin), _ptr(r.ratio_margin)
    a.out_sample_margin = _ptr(r.sample_margin)
    a.num_threads = int(num_threads)
    # test aids: one node's decision overridden, the interval of a given token in the final draw
    fn = None if force_node is None else np.ascontiguousarray(force_node, dtype=np.int32)
    fo = None if force_outcome is None else np.ascontiguousarray(force_outcome, dtype=np.int32)
    pt = None if probe_token is None else np.ascontiguousarray(probe_token, dtype=np.int32)
    assert (fn is None) == (fo is None)
    a.force_node, a.force_outcome, a.probe_token = _ptr(fn), _ptr(fo), _ptr(pt)
    if pt is not None:
        r.probe_lo, r.probe_hi = np.zeros(B, np.float64), np.zeros(B, np.float64)
        a.out_probe_lo, a.out_probe_hi = _ptr(r.probe_lo), _ptr(r.probe_hi)
    if lib().oracle_verify_tree(C.byref(a)) != 0:
        raise ValueError("oracle_verify_tree rejected its arguments")
    return r


def max_threads() -> int:
    return int(lib().oracle_max_threads())
