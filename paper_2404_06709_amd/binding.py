"""Thin ctypes binding of libcqil.so: argument marshalling only.

Function names follow the C ABI in ``include/cqil.h``.  torch tensors supply device memory
(``data_ptr()``) and the current HIP stream; every step of the path runs inside the library.
There is no fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# CQIL_HOST_SANITIZE=1 loads the build whose host code runs under AddressSanitizer + UBSan (see build.py)
LIB_PATH = os.path.join(_HERE, "libcqil_san.so" if os.environ.get("CQIL_HOST_SANITIZE", "") not in ("", "0")
                        else "libcqil.so")

CQIL_F32, CQIL_BF16 = 0, 1
CQIL_ATTN_FFN_PARALLEL = -1   # bypass_d value selecting App. A, Eq.5
CQIL_OK, CQIL_EINVAL, CQIL_ESIZE, CQIL_ERANGE, CQIL_EHIP = 0, -1, -2, -3, -4


class cqil_dims(C.Structure):
    _fields_ = [("d_model", C.c_int), ("n_heads", C.c_int), ("head_dim", C.c_int), ("d_ffn", C.c_int),
                ("max_seq", C.c_int), ("rope_base", C.c_float), ("rms_eps", C.c_float), ("dtype", C.c_int)]


class cqil_layer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "g_attn", "g_ffn")]


class cqil_kv(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("kv_len", C.c_void_p), ("b_max", C.c_int),
                ("max_kv_len", C.c_int)]


class cqil_packed_layout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in
                ("wqkv", "wo", "wgu", "wdown", "g_attn", "g_ffn", "rope", "total")]


class cqil_model(C.Structure):
    _fields_ = [("dims", cqil_dims), ("vocab", C.c_int), ("n_groups", C.c_int),
                ("group_sizes", C.POINTER(C.c_int)), ("packed", C.POINTER(C.c_void_p)),
                ("k_cache", C.POINTER(C.c_void_p)), ("v_cache", C.POINTER(C.c_void_p)),
                ("kv_len", C.c_void_p), ("b_max", C.c_int), ("max_kv_len", C.c_int),
                ("embedding", C.c_void_p), ("g_final", C.c_void_p), ("lm_head", C.c_void_p)]


class CqilError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


_lib = None


def lib() -> C.CDLL:
    """Loads libcqil.so; raises if it has not been built (there is no other implementation)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2404_06709_amd.build` first")
        L = C.CDLL(LIB_PATH)
        L.cqil_version.restype = C.c_char_p
        L.cqil_strerror.restype = C.c_char_p
        L.cqil_strerror.argtypes = [C.c_int]
        L.cqil_packed_layout_of.argtypes = [C.POINTER(cqil_dims), C.c_int, C.POINTER(cqil_packed_layout)]
        L.cqil_packed_bytes.restype = C.c_size_t
        L.cqil_packed_bytes.argtypes = [C.POINTER(cqil_dims), C.c_int]
        L.cqil_workspace_bytes.restype = C.c_size_t
        L.cqil_workspace_bytes.argtypes = [C.POINTER(cqil_dims), C.c_int, C.c_int, C.c_int]
        L.cqil_workspace_attn_out_offset.restype = C.c_size_t
        L.cqil_workspace_attn_out_offset.argtypes = [C.POINTER(cqil_dims), C.c_int, C.c_int, C.c_int]
        L.cqil_partition.argtypes = [C.c_int] * 4 + [C.POINTER(C.c_int), C.POINTER(C.c_int)]
        L.cqil_pack_group.argtypes = [C.POINTER(cqil_dims), C.c_int, C.POINTER(cqil_layer), C.c_void_p, C.c_size_t,
                                      C.c_void_p]
        L.cqil_group_forward.argtypes = [C.POINTER(cqil_dims), C.c_int, C.c_int, C.c_void_p, C.POINTER(cqil_kv),
                                         C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_size_t,
                                         C.c_void_p]
        L.cqil_stream_read_probe.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_void_p]
        L.cqil_static_scratch_bytes.restype = C.c_size_t
        L.cqil_static_scratch_bytes.argtypes = []
        L.cqil_group_forward_static.argtypes = [C.POINTER(cqil_dims), C.c_int, C.c_int, C.c_void_p, C.POINTER(cqil_kv),
                                                C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
        L.cqil_decode_step_profile.argtypes = [C.POINTER(cqil_dims), C.c_int, C.c_int, C.c_void_p, C.POINTER(cqil_kv),
                                               C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p,
                                               C.POINTER(C.c_float)]
        L.cqil_set_tuning.argtypes = [C.c_char_p, C.c_int]
        L.cqil_input_similarity_workspace_bytes.restype = C.c_size_t
        L.cqil_input_similarity_workspace_bytes.argtypes = [C.c_int, C.c_int]
        L.cqil_input_similarity.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                            C.c_size_t, C.c_void_p]
        L.cqil_merge_lora.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_float,
                                      C.c_void_p]
        L.cqil_model_workspace_bytes.restype = C.c_size_t
        L.cqil_model_workspace_bytes.argtypes = [C.POINTER(cqil_model), C.c_int, C.c_int]
        L.cqil_model_forward.argtypes = [C.POINTER(cqil_model), C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int,
                                         C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.cqil_model_substituted_workspace_bytes.restype = C.c_size_t
        L.cqil_model_substituted_workspace_bytes.argtypes = [C.POINTER(cqil_model), C.c_int, C.c_int]
        L.cqil_model_forward_substituted.argtypes = [C.POINTER(cqil_model), C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int,
                                                     C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                     C.c_size_t, C.c_void_p]
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().cqil_strerror(int(status)).decode()


def version() -> str:
    return lib().cqil_version().decode()


def dtype_code(dt: torch.dtype) -> int:
    if dt == torch.float32:
        return CQIL_F32
    if dt == torch.bfloat16:
        return CQIL_BF16
    raise TypeError(f"unsupported dtype {dt}")


def make_dims(d_model: int, n_heads: int, head_dim: int, d_ffn: int, max_seq: int, dtype: torch.dtype,
              rope_base: float = 10000.0, rms_eps: float = 1e-6) -> cqil_dims:
    return cqil_dims(d_model, n_heads, head_dim, d_ffn, max_seq, rope_base, rms_eps, dtype_code(dtype))


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def cqil_packed_layout_of(dims: cqil_dims, P: int) -> cqil_packed_layout:
    out = cqil_packed_layout()
    rc = lib().cqil_packed_layout_of(C.byref(dims), P, C.byref(out))
    if rc:
        raise CqilError(rc, "cqil_packed_layout_of")
    return out


def cqil_packed_bytes(dims: cqil_dims, P: int) -> int:
    return int(lib().cqil_packed_bytes(C.byref(dims), P))


def cqil_workspace_bytes(dims: cqil_dims, P: int, B: int, T: int) -> int:
    return int(lib().cqil_workspace_bytes(C.byref(dims), P, B, T))


def cqil_workspace_attn_out_offset(dims: cqil_dims, P: int, B: int, T: int) -> int:
    return int(lib().cqil_workspace_attn_out_offset(C.byref(dims), P, B, T))


def cqil_partition(L: int, p: int, s: int, e: int) -> List[int]:
    sizes = (C.c_int * max(L, 1))()
    n = C.c_int(0)
    rc = lib().cqil_partition(L, p, s, e, sizes, C.byref(n))
    if rc:
        raise CqilError(rc, "cqil_partition")
    return [int(sizes[i]) for i in range(n.value)]


def layer_struct(layer: Dict[str, torch.Tensor]) -> cqil_layer:
    return cqil_layer(*[layer[k].data_ptr() for k in
                        ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "g_attn", "g_ffn")])


def cqil_pack_group(dims: cqil_dims, layers: Sequence[Dict[str, torch.Tensor]], packed: torch.Tensor) -> None:
    """layers: P dicts of contiguous device tensors; packed: uint8 device tensor of cqil_packed_bytes()."""
    P = len(layers)
    arr = (cqil_layer * P)(*[layer_struct(L) for L in layers])
    rc = lib().cqil_pack_group(C.byref(dims), P, arr, _ptr(packed), packed.numel() * packed.element_size(), _stream())
    if rc:
        raise CqilError(rc, "cqil_pack_group")


def make_kv(k: torch.Tensor, v: torch.Tensor, kv_len: torch.Tensor, max_kv_len: int) -> cqil_kv:
    """k, v: [P, b_max, n_heads, max_seq, head_dim]; kv_len: int32 [b_max] on the device."""
    assert kv_len.dtype == torch.int32
    return cqil_kv(k.data_ptr(), v.data_ptr(), kv_len.data_ptr(), k.shape[1], int(max_kv_len))


def cqil_group_forward(dims: cqil_dims, P: int, bypass_d: int, packed: torch.Tensor, kv: cqil_kv,
                       x_in: torch.Tensor, x_out: torch.Tensor, B: int, T: int, advance_kv_len: bool,
                       workspace: torch.Tensor) -> None:
    rc = lib().cqil_group_forward(C.byref(dims), P, bypass_d, _ptr(packed), C.byref(kv), _ptr(x_in), _ptr(x_out), B, T,
                                  1 if advance_kv_len else 0, _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream())
    if rc:
        raise CqilError(rc, "cqil_group_forward")


def cqil_stream_read_probe(buf: torch.Tensor, sink: torch.Tensor) -> None:
    """Reads every byte of buf once (measurement aid); sink: device tensor of at least 16384 bytes."""
    rc = lib().cqil_stream_read_probe(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink),
                                      sink.numel() * sink.element_size(), _stream())
    if rc:
        raise CqilError(rc, "cqil_stream_read_probe")


def cqil_static_scratch_bytes() -> int:
    return int(lib().cqil_static_scratch_bytes())


def cqil_group_forward_static(dims: cqil_dims, P: int, bypass_d: int, packed: torch.Tensor, kv: cqil_kv,
                              x_in: torch.Tensor, x_out: torch.Tensor, B: int, T: int, advance_kv_len: bool) -> None:
    """cqil_group_forward with the library's static scratch array as the workspace (allocates nothing)."""
    rc = lib().cqil_group_forward_static(C.byref(dims), P, bypass_d, _ptr(packed), C.byref(kv), _ptr(x_in), _ptr(x_out),
                                         B, T, 1 if advance_kv_len else 0, _stream())
    if rc:
        raise CqilError(rc, "cqil_group_forward_static")


def cqil_set_tuning(key: str, value: int) -> None:
    rc = lib().cqil_set_tuning(key.encode(), int(value))
    if rc:
        raise CqilError(rc, f"cqil_set_tuning({key}, {value})")


TUNING_DEFAULTS = {"ksplit_qkv": 0, "ksplit_o": 0, "ksplit_gu": 0, "ksplit_d": 0, "down_slice_max": 3072,
                   "gemm_tile": 0, "eq5_fused": 1, "attn_prefill": 0}


def reset_tuning() -> None:
    """Puts every launch-shape knob back to the library's default."""
    for k, v in TUNING_DEFAULTS.items():
        cqil_set_tuning(k, v)


def cqil_input_similarity(X: torch.Tensor) -> torch.Tensor:
    """X [L, M, n] (bf16 or fp32, contiguous, on the GPU) -> fp32 [L, L] mean per-token cosine similarity (Sec.3.1)."""
    assert X.dim() == 3 and X.is_contiguous()
    L_, M, n = X.shape
    sim = torch.empty(L_, L_, dtype=torch.float32, device=X.device)
    nbytes = int(lib().cqil_input_similarity_workspace_bytes(L_, M))
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=X.device)
    rc = lib().cqil_input_similarity(_ptr(X), CQIL_BF16 if X.dtype == torch.bfloat16 else CQIL_F32, L_, M, n, _ptr(sim),
                                     _ptr(ws), nbytes, _stream())
    if rc:
        raise CqilError(rc, "cqil_input_similarity")
    return sim


def cqil_merge_lora(W: torch.Tensor, A: torch.Tensor, Bm: torch.Tensor, scale: float = 1.0) -> None:
    """W += scale * Bm @ A in place (W [out,in], A [r,in], Bm [out,r], one dtype, contiguous, on the GPU)."""
    assert W.dtype == A.dtype == Bm.dtype and W.is_contiguous() and A.is_contiguous() and Bm.is_contiguous()
    n_out, n_in = W.shape
    r = A.shape[0]
    assert A.shape == (r, n_in) and Bm.shape == (n_out, r)
    rc = lib().cqil_merge_lora(_ptr(W), _ptr(A), _ptr(Bm), CQIL_BF16 if W.dtype == torch.bfloat16 else CQIL_F32, n_out,
                               n_in, r, float(scale), _stream())
    if rc:
        raise CqilError(rc, "cqil_merge_lora")


DECODE_KERNELS = ("qkv_rope", "attn_decode", "oproj", "gateup", "down", "merge")


def cqil_decode_step_profile(dims: cqil_dims, P: int, bypass_d: int, packed: torch.Tensor, kv: cqil_kv,
                             x_in: torch.Tensor, x_out: torch.Tensor, workspace: torch.Tensor,
                             B: int = 1) -> List[float]:
    """Per-kernel milliseconds of one single-token decode step (B must be 1), in DECODE_KERNELS order."""
    ms = (C.c_float * 6)()
    rc = lib().cqil_decode_step_profile(C.byref(dims), P, bypass_d, _ptr(packed), C.byref(kv), _ptr(x_in), _ptr(x_out),
                                        B, _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(), ms)
    if rc:
        raise CqilError(rc, "cqil_decode_step_profile")
    return [float(v) for v in ms]


class Model:
    """Owns the host-side arrays a cqil_model points to (and keeps the tensors alive)."""

    def __init__(self, dims: cqil_dims, group_sizes: Sequence[int], packed: Sequence[torch.Tensor],
                 k_cache: Sequence[torch.Tensor], v_cache: Sequence[torch.Tensor], kv_len: torch.Tensor,
                 embedding: torch.Tensor, g_final: torch.Tensor, lm_head: torch.Tensor, max_kv_len: int = 0):
        n = len(group_sizes)
        assert len(packed) == n and len(k_cache) == n and len(v_cache) == n
        self._keep = (list(packed), list(k_cache), list(v_cache), kv_len, embedding, g_final, lm_head)
        self._gs = (C.c_int * n)(*[int(g) for g in group_sizes])
        self._pk = (C.c_void_p * n)(*[t.data_ptr() for t in packed])
        self._kc = (C.c_void_p * n)(*[t.data_ptr() for t in k_cache])
        self._vc = (C.c_void_p * n)(*[t.data_ptr() for t in v_cache])
        self.c = cqil_model(dims, lm_head.shape[0], n, self._gs, self._pk, self._kc, self._vc, kv_len.data_ptr(),
                            k_cache[0].shape[1], int(max_kv_len), embedding.data_ptr(), g_final.data_ptr(),
                            lm_head.data_ptr())


def cqil_model_workspace_bytes(model: Model, B: int, T: int) -> int:
    return int(lib().cqil_model_workspace_bytes(C.byref(model.c), B, T))


def cqil_model_forward(model: Model, tokens: torch.Tensor, B: int, T: int, bypass_d: int, advance_kv_len: bool,
                       hidden_out: Optional[torch.Tensor], logits_out: Optional[torch.Tensor],
                       next_token_out: Optional[torch.Tensor], workspace: torch.Tensor) -> None:
    assert tokens.dtype == torch.int32
    rc = lib().cqil_model_forward(C.byref(model.c), _ptr(tokens), B, T, bypass_d, 1 if advance_kv_len else 0,
                                  _ptr(hidden_out), _ptr(logits_out), _ptr(next_token_out), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream())
    if rc:
        raise CqilError(rc, "cqil_model_forward")


def cqil_model_substituted_workspace_bytes(model: Model, B: int, T: int) -> int:
    return int(lib().cqil_model_substituted_workspace_bytes(C.byref(model.c), B, T))


def cqil_model_forward_substituted(model: Model, tokens: torch.Tensor, B: int, T: int, bypass_d: int,
                                   advance_kv_len: bool, group: int, k: int, hidden_out: Optional[torch.Tensor],
                                   logits_out: Optional[torch.Tensor], next_token_out: Optional[torch.Tensor],
                                   workspace: torch.Tensor) -> None:
    """Sec.3.2: group `group` reads the input of group `group - k`; everything else as cqil_model_forward."""
    assert tokens.dtype == torch.int32
    rc = lib().cqil_model_forward_substituted(C.byref(model.c), _ptr(tokens), B, T, bypass_d, 1 if advance_kv_len else 0,
                                              group, k, _ptr(hidden_out), _ptr(logits_out), _ptr(next_token_out),
                                              _ptr(workspace), workspace.numel() * workspace.element_size(), _stream())
    if rc:
        raise CqilError(rc, "cqil_model_forward_substituted")
