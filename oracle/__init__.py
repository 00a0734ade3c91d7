"""CPU oracle for the CQIL hot path -- TEST INFRASTRUCTURE, not product code.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package.
It wraps ``cqil_oracle.c`` (plain C, double arithmetic) through ctypes and adds nothing to
its arithmetic: every function here only marshals numpy arrays.

Weights are numpy arrays in their storage type: ``float32`` or ``uint16`` (bf16 bit
patterns).  Activations, caches and outputs are ``float64``.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cqil_oracle.c")
# CQIL_ORACLE_SANITIZE=1 builds and loads an AddressSanitizer + UndefinedBehaviorSanitizer build of the oracle (host code
# only).  The sanitizer runtime has to be in the process before python starts:
#   LD_PRELOAD=$(gcc -print-file-name=libasan.so) ASAN_OPTIONS=detect_leaks=0 CQIL_ORACLE_SANITIZE=1 \
#       python -m pytest tests -m "not gpu"
SANITIZE = os.environ.get("CQIL_ORACLE_SANITIZE", "") not in ("", "0")
_LIB = os.path.join(_HERE, "libcqil_oracle_san.so" if SANITIZE else "libcqil_oracle.so")

F32, BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP for independent rows/heads only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g",
               "-O1"] if SANITIZE else ["-O2"]
        subprocess.check_call(
            ["gcc", *san, "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


class _Dims(C.Structure):
    _fields_ = [
        ("d_model", C.c_int), ("n_heads", C.c_int), ("head_dim", C.c_int), ("d_ffn", C.c_int),
        ("max_seq", C.c_int), ("rope_base", C.c_double), ("rms_eps", C.c_double), ("wdtype", C.c_int),
    ]


class _Layer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "g_attn", "g_ffn")]


@dataclass
class Dims:
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    max_seq: int
    rope_base: float = 10000.0
    rms_eps: float = 1e-6
    wdtype: int = F32

    def c(self) -> _Dims:
        return _Dims(self.d_model, self.n_heads, self.head_dim, self.d_ffn, self.max_seq,
                     self.rope_base, self.rms_eps, self.wdtype)


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_silu.restype = C.c_double
        _lib.orc_silu.argtypes = [C.c_double]
    return _lib


def _wdtype(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"weights must be float32 or uint16 (bf16 bits), got {a.dtype}")


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


_LAYER_KEYS = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "g_attn", "g_ffn")


def _layers(layers: Sequence[dict], wdtype: int):
    arr = (_Layer * len(layers))()
    keep = []
    for i, L in enumerate(layers):
        for k in _LAYER_KEYS:
            a = np.ascontiguousarray(L[k])
            assert _wdtype(a) == wdtype, "all weights of a call share one storage type"
            keep.append(a)
            setattr(arr[i], k, a.ctypes.data)
    return arr, keep


def num_threads() -> int:
    return int(lib().orc_num_threads())


def set_threads(n: int) -> None:
    lib().orc_set_threads(int(n))


def linear(W: np.ndarray, x) -> np.ndarray:
    W = np.ascontiguousarray(W)
    x = _f64(x)
    y = np.empty(W.shape[0], dtype=np.float64)
    lib().orc_linear(_p(W), _wdtype(W), W.shape[0], W.shape[1], _p(x), _p(y))
    return y


def merge_lora(W: np.ndarray, A: np.ndarray, Bm: np.ndarray, scale: float = 1.0) -> np.ndarray:
    """W + scale * Bm @ A in float64 (unrounded): W [out,in], A [r,in], Bm [out,r], one storage type."""
    W, A, Bm = np.ascontiguousarray(W), np.ascontiguousarray(A), np.ascontiguousarray(Bm)
    assert _wdtype(W) == _wdtype(A) == _wdtype(Bm)
    n_out, n_in = W.shape
    r = A.shape[0]
    assert A.shape == (r, n_in) and Bm.shape == (n_out, r)
    out = np.empty((n_out, n_in), dtype=np.float64)
    lib().orc_merge_lora(_p(W), _p(A), _p(Bm), _wdtype(W), n_out, n_in, r, C.c_double(scale), _p(out))
    return out


def input_similarity(X) -> np.ndarray:
    """Sec.3.1: X [L, M, n] layer inputs for the same M tokens -> [L, L] mean per-token cosine similarity."""
    X = _f64(X)
    L, M, n = X.shape
    sim = np.empty((L, L), dtype=np.float64)
    lib().orc_input_similarity(_p(X), L, M, n, _p(sim))
    return sim


def rmsnorm(x, g: np.ndarray, eps: float) -> np.ndarray:
    x = _f64(x)
    g = np.ascontiguousarray(g)
    out = np.empty_like(x)
    lib().orc_rmsnorm(_p(x), _p(g), _wdtype(g), x.shape[0], C.c_double(eps), _p(out))
    return out


def rope(v, pos: int, base: float = 10000.0) -> np.ndarray:
    v = _f64(v).copy()
    lib().orc_rope(_p(v), v.shape[0], C.c_long(pos), C.c_double(base))
    return v


def silu(z: float) -> float:
    return float(lib().orc_silu(float(z)))


def new_cache(n_layers: int, b_max: int, dims: Dims) -> np.ndarray:
    return np.zeros((n_layers, b_max, dims.n_heads, dims.max_seq, dims.head_dim), dtype=np.float64)


def attn_module(dims: Dims, layer: dict, lg: int, kcache, vcache, kv_len, x) -> np.ndarray:
    """ATTN_l(x); x [B,T,d_model]; caches [P,b_max,n,max_seq,d_k] float64, written in place."""
    x = _f64(x)
    B, T, _ = x.shape
    arr, keep = _layers([layer], dims.wdtype)
    kv = np.ascontiguousarray(kv_len, dtype=np.int32)
    out = np.empty_like(x)
    rc = lib().orc_attn_module(C.byref(dims.c()), arr, lg, _p(kcache), _p(vcache), kcache.shape[1],
                               _p(kv), _p(x), B, T, _p(out))
    if rc:
        raise RuntimeError(f"orc_attn_module rc={rc}")
    return out


def ffn_module(dims: Dims, layer: dict, h) -> np.ndarray:
    h = _f64(h)
    arr, keep = _layers([layer], dims.wdtype)
    out = np.empty_like(h)
    M = int(np.prod(h.shape[:-1]))
    rc = lib().orc_ffn_module(C.byref(dims.c()), arr, _p(h), M, _p(out))
    if rc:
        raise RuntimeError(f"orc_ffn_module rc={rc}")
    return out


def seq_layer(dims: Dims, layer: dict, kcache, vcache, kv_len, x) -> np.ndarray:
    """Eq.1.  Caches [1,b_max,n,max_seq,d_k]."""
    x = _f64(x)
    B, T, _ = x.shape
    arr, keep = _layers([layer], dims.wdtype)
    kv = np.ascontiguousarray(kv_len, dtype=np.int32)
    out = np.empty_like(x)
    rc = lib().orc_seq_layer(C.byref(dims.c()), arr, _p(kcache), _p(vcache), kcache.shape[1], _p(kv),
                             _p(x), _p(out), B, T)
    if rc:
        raise RuntimeError(f"orc_seq_layer rc={rc}")
    return out


def group_forward(dims: Dims, layers: Sequence[dict], d: int, kcache, vcache, kv_len, x, debug: bool = False):
    """Eq.3 / Eq.4 (d >= 0) or the attention-FFN parallel form of App. A, Eq.5 (d = -1).  Returns x_out, or
    (x_out, attn[P,B,T,dm], h[P,B,T,dm]) with debug=True."""
    x = _f64(x)
    B, T, dm = x.shape
    P = len(layers)
    assert kcache.shape[0] >= P and kcache.dtype == np.float64 and kcache.flags.c_contiguous
    arr, keep = _layers(layers, dims.wdtype)
    kv = np.ascontiguousarray(kv_len, dtype=np.int32)
    out = np.empty_like(x)
    da = np.empty((P, B, T, dm)) if debug else None
    dh = np.empty((P, B, T, dm)) if debug else None
    rc = lib().orc_group_forward(C.byref(dims.c()), P, d, arr, _p(kcache), _p(vcache), kcache.shape[1],
                                 _p(kv), _p(x), _p(out), B, T, _p(da), _p(dh))
    if rc:
        raise RuntimeError(f"orc_group_forward rc={rc}")
    return (out, da, dh) if debug else out


def group_forward_rows(dims: Dims, layers: Sequence[dict], d: int, kcache, vcache, kv_len, x, rows):
    """group_forward with the outputs restricted to the rows flagged in ``rows`` [B, T] (bool): keys and values
    of every row are cached, the flagged rows of (x_out, attn, h) equal those of the full call, the rest are 0."""
    x = _f64(x)
    B, T, dm = x.shape
    P = len(layers)
    assert kcache.shape[0] >= P and kcache.dtype == np.float64 and kcache.flags.c_contiguous
    arr, keep = _layers(layers, dims.wdtype)
    kv = np.ascontiguousarray(kv_len, dtype=np.int32)
    flags = np.ascontiguousarray(np.asarray(rows).reshape(B, T), dtype=np.uint8)
    out = np.empty_like(x)
    da = np.empty((P, B, T, dm))
    dh = np.empty((P, B, T, dm))
    rc = lib().orc_group_forward_rows(C.byref(dims.c()), P, d, arr, _p(kcache), _p(vcache), kcache.shape[1],
                                      _p(kv), _p(x), _p(out), B, T, _p(flags), _p(da), _p(dh))
    if rc:
        raise RuntimeError(f"orc_group_forward_rows rc={rc}")
    return out, da, dh


def bypass_transfers(p: int, d: int) -> int:
    return int(lib().orc_bypass_transfers(p, d))


def partition(L: int, p: int, s: int, e: int) -> list:
    sizes = (C.c_int * max(L, 1))()
    n = lib().orc_partition(L, p, s, e, sizes)
    if n < 0:
        raise ValueError("bad (L, p, s, e)")
    return [int(sizes[i]) for i in range(n)]


def model_forward(dims: Dims, layers: Sequence[dict], group_sizes: Sequence[int], d: int,
                  embedding: np.ndarray, g_final: np.ndarray, lm_head: np.ndarray,
                  kcache, vcache, kv_len, tokens, want_logits: bool = True, sub_group: int = -1, sub_k: int = 0):
    """Alg.1 around the LLaMA embedding / final norm / lm head.  With sub_group >= 0: Sec.3.2's input substitution
    (group sub_group reads the input of group sub_group - sub_k).
    Returns dict(hidden [B,T,dm], logits [B,V] of the last position, next [B])."""
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    B, T = tokens.shape
    L = len(layers)
    V = lm_head.shape[0]
    arr, keep = _layers(layers, dims.wdtype)
    gs = (C.c_int * len(group_sizes))(*[int(g) for g in group_sizes])
    kv = np.ascontiguousarray(kv_len, dtype=np.int32)
    embedding = np.ascontiguousarray(embedding)
    g_final = np.ascontiguousarray(g_final)
    lm_head = np.ascontiguousarray(lm_head)
    hidden = np.empty((B, T, dims.d_model))
    logits = np.empty((B, V)) if want_logits else None
    nxt = np.empty(B, dtype=np.int32)
    if sub_group >= 0:
        rc = lib().orc_model_forward_substituted(C.byref(dims.c()), L, arr, len(group_sizes), gs, d, int(sub_group),
                                                 int(sub_k), _p(embedding), _p(g_final), _p(lm_head), V, _p(kcache),
                                                 _p(vcache), kcache.shape[1], _p(kv), _p(tokens), B, T, _p(hidden),
                                                 _p(logits), _p(nxt))
    else:
        rc = lib().orc_model_forward(C.byref(dims.c()), L, arr, len(group_sizes), gs, d, _p(embedding),
                                     _p(g_final), _p(lm_head), V, _p(kcache), _p(vcache), kcache.shape[1],
                                     _p(kv), _p(tokens), B, T, _p(hidden), _p(logits), _p(nxt))
    if rc:
        raise RuntimeError(f"orc_model_forward rc={rc}")
    return {"hidden": hidden, "logits": logits, "next": nxt}
