"""Thin ctypes binding of libkvcapsule.so (C ABI in include/kvcapsule.h).

Argument marshalling only: every step of the hot path runs in the HIP kernels of
the library.  PyTorch is used for device memory and the current stream.  There is
no CPU fallback: if the library is missing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvcapsule.so")

KVC_OK = 0
KVC_ERR_NULL = -1
KVC_ERR_SHAPE = -2
KVC_ERR_DTYPE = -3
KVC_ERR_ALIGN = -4
KVC_ERR_WORKSPACE = -5
KVC_ERR_UNSUPPORTED = -6
KVC_ERR_HIP = -7
KVC_F32 = 0
KVC_BF16 = 1
KVC_ACT_IDENTITY = 0
KVC_ACT_RELU = 1
KVC_ACT_GELU = 2

EXPORTS = [
    "kvc_compressed_len", "kvc_workspace_bytes", "kvc_memory_footprint", "kvc_compress",
    "kvc_reconstruct_attend_decode", "kvc_reconstruct_attend_decode_generic",
    "kvc_compress_generic", "kvc_probe_read", "kvc_status_string", "kvc_version",
    "kvc_static_scratch_bytes", "kvc_reconstruct_attend_decode_static",
    "kvc_attend_full_workspace_bytes", "kvc_attend_full_decode", "kvc_dev_full_decode_chunk_steps",
    "kvc_dev_decode_knobs", "kvc_dev_decode_fallbacks", "kvc_dev_compress_knobs",
    "kvc_capsule_value_offset", "kvc_unpack_values",
    "kvc_reconstruct_attend_decode_ragged", "kvc_mlp_hidden", "kvc_static_attend_decode",
    "kvc_pack_theta", "kvc_pack_u", "kvc_dev_stream_decode", "kvc_dev_stream_calls",
]


class KvcShape(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("n_img_tokens", ctypes.c_int32), ("n_images", ctypes.c_int32),
                ("m", ctypes.c_int32), ("dtype", ctypes.c_int32)]


class KvcParams(ctypes.Structure):
    _fields_ = [("key_idx", ctypes.c_void_p), ("theta", ctypes.c_void_p),
                ("U", ctypes.c_void_p), ("mu", ctypes.c_void_p), ("theta_packed", ctypes.c_void_p), ("U_packed", ctypes.c_void_p)]


class KvcError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (what, status_string(status), status))


_lib = None


def lib() -> ctypes.CDLL:
    """Load the HIP library; fail loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "libkvcapsule.so is not built: run `python -c 'import __graft_entry__ as g; "
                "g.build()'` (or python paper_2605_16439_amd/build.py) first")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        L.kvc_compressed_len.restype = i32
        L.kvc_compressed_len.argtypes = [i32, ctypes.c_double]
        L.kvc_workspace_bytes.restype = ctypes.c_size_t
        L.kvc_workspace_bytes.argtypes = [ctypes.POINTER(KvcShape), i32]
        L.kvc_memory_footprint.restype = i32
        L.kvc_memory_footprint.argtypes = [ctypes.POINTER(KvcShape), i64, i64,
                                           ctypes.POINTER(i64), ctypes.POINTER(i64)]
        comp = [ctypes.POINTER(KvcShape), ctypes.POINTER(KvcParams), vp, vp, i64, i64, i64, i32, i32,
                vp, vp, vp, ctypes.c_size_t, vp]
        dec = [ctypes.POINTER(KvcShape), ctypes.POINTER(KvcParams), vp, vp, vp, vp, vp, i32, i32,
               vp, vp, ctypes.c_float, vp, vp, vp, ctypes.c_size_t, vp]
        for name in ("kvc_compress", "kvc_compress_generic"):
            getattr(L, name).restype = i32
            getattr(L, name).argtypes = comp
        for name in ("kvc_reconstruct_attend_decode", "kvc_reconstruct_attend_decode_generic"):
            getattr(L, name).restype = i32
            getattr(L, name).argtypes = dec
        L.kvc_static_scratch_bytes.restype = ctypes.c_size_t
        L.kvc_static_scratch_bytes.argtypes = []
        L.kvc_reconstruct_attend_decode_static.restype = i32
        L.kvc_reconstruct_attend_decode_static.argtypes = dec[:-3] + [vp]
        L.kvc_attend_full_workspace_bytes.restype = ctypes.c_size_t
        L.kvc_attend_full_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32]
        L.kvc_attend_full_decode.restype = i32
        L.kvc_attend_full_decode.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, i64, i64, i64, i32, i32,
                                             vp, vp, ctypes.c_float, vp, vp, vp, ctypes.c_size_t, vp]
        L.kvc_dev_full_decode_chunk_steps.restype = None
        L.kvc_dev_full_decode_chunk_steps.argtypes = [i32]
        L.kvc_dev_decode_knobs.restype = None
        L.kvc_dev_decode_knobs.argtypes = [i32, i32, i32]
        L.kvc_dev_decode_fallbacks.restype = i64
        L.kvc_dev_decode_fallbacks.argtypes = []
        L.kvc_dev_compress_knobs.restype = None
        L.kvc_dev_compress_knobs.argtypes = [i32, i32]
        L.kvc_reconstruct_attend_decode_ragged.restype = i32
        L.kvc_reconstruct_attend_decode_ragged.argtypes = [ctypes.POINTER(KvcShape), ctypes.POINTER(KvcParams), vp, vp, vp,
                                                           vp, vp, vp, vp, i32, vp, vp, ctypes.c_float, vp, vp, vp,
                                                           ctypes.c_size_t, vp]
        L.kvc_mlp_hidden.restype = i32
        L.kvc_mlp_hidden.argtypes = [ctypes.POINTER(KvcShape), vp, i32, vp, vp, vp]
        L.kvc_static_attend_decode.restype = i32
        L.kvc_static_attend_decode.argtypes = [ctypes.POINTER(KvcShape), vp, vp, vp, vp, vp, i32, i32, vp, vp,
                                               ctypes.c_float, vp, vp, vp, ctypes.c_size_t, vp]
        L.kvc_pack_theta.restype = i32
        L.kvc_pack_theta.argtypes = [ctypes.POINTER(KvcShape), vp, vp, vp]
        L.kvc_pack_u.restype = i32
        L.kvc_pack_u.argtypes = [ctypes.POINTER(KvcShape), vp, vp, vp]
        L.kvc_dev_stream_decode.restype = None
        L.kvc_dev_stream_decode.argtypes = [i32]
        L.kvc_dev_stream_calls.restype = i64
        L.kvc_dev_stream_calls.argtypes = []
        L.kvc_capsule_value_offset.restype = i64
        L.kvc_capsule_value_offset.argtypes = [i32, i32, i32, i32]
        L.kvc_unpack_values.restype = i32
        L.kvc_unpack_values.argtypes = [vp, vp, i64, i32, i32, i32, vp]
        L.kvc_probe_read.restype = i32
        L.kvc_probe_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
        L.kvc_status_string.restype = ctypes.c_char_p
        L.kvc_status_string.argtypes = [i32]
        L.kvc_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


def kvc_probe_read(buf: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    """Streaming read of all of `buf` (measurement aid); `sink` is any device tensor of >= 4 bytes."""
    st = lib().kvc_probe_read(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink), _stream(stream))
    if st != KVC_OK:
        raise KvcError(st, "kvc_probe_read")


def status_string(status: int) -> str:
    return lib().kvc_status_string(int(status)).decode()


def version() -> str:
    return lib().kvc_version().decode()


def kvc_compressed_len(n: int, compression_ratio: float) -> int:
    return int(lib().kvc_compressed_len(int(n), float(compression_ratio)))


def _dtype_code(dt: torch.dtype) -> int:
    if dt == torch.float32:
        return KVC_F32
    if dt == torch.bfloat16:
        return KVC_BF16
    raise TypeError("unsupported dtype %s (float32 or bfloat16)" % dt)


def make_shape(batch, n_q_heads, n_kv_heads, head_dim, n_img_tokens, n_images, m, dtype) -> KvcShape:
    code = dtype if isinstance(dtype, int) else _dtype_code(dtype)
    return KvcShape(batch, n_q_heads, n_kv_heads, head_dim, n_img_tokens, n_images, m, code)


def kvc_workspace_bytes(shape: KvcShape, max_text_len: int) -> int:
    return int(lib().kvc_workspace_bytes(ctypes.byref(shape), int(max_text_len)))


def kvc_memory_footprint(shape: KvcShape, c_prompt: int, t: int):
    a, b = ctypes.c_int64(), ctypes.c_int64()
    st = lib().kvc_memory_footprint(ctypes.byref(shape), int(c_prompt), int(t), ctypes.byref(a),
                                    ctypes.byref(b))
    if st != KVC_OK:
        raise KvcError(st, "kvc_memory_footprint")
    return int(a.value), int(b.value)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def make_params(key_idx, theta, U, mu, theta_packed=None, U_packed=None) -> KvcParams:
    return KvcParams(_ptr(key_idx), _ptr(theta), _ptr(U), _ptr(mu), _ptr(theta_packed), _ptr(U_packed))


def kvc_pack_u(shape: KvcShape, U: torch.Tensor, stream=None) -> torch.Tensor:
    """U [H_kv, m, n] -> the packed form of the same size (a new tensor), for KvcParams.U_packed."""
    packed = torch.empty_like(U)
    st = lib().kvc_pack_u(ctypes.byref(shape), _ptr(U), _ptr(packed), _stream(stream))
    if st != KVC_OK:
        raise KvcError(st, "kvc_pack_u")
    return packed


def kvc_pack_theta(shape: KvcShape, theta: torch.Tensor, stream=None) -> torch.Tensor:
    """theta [H_kv, m, n] -> the packed form of the same size (a new tensor), for KvcParams.theta_packed."""
    packed = torch.empty_like(theta)
    st = lib().kvc_pack_theta(ctypes.byref(shape), _ptr(theta), _ptr(packed), _stream(stream))
    if st != KVC_OK:
        raise KvcError(st, "kvc_pack_theta")
    return packed


def new_workspace(shape: KvcShape, max_text_len: int, device="cuda") -> torch.Tensor:
    nbytes = kvc_workspace_bytes(shape, max_text_len)
    if nbytes == 0:
        raise KvcError(KVC_ERR_SHAPE, "kvc_workspace_bytes")
    return torch.empty(nbytes + 256, dtype=torch.uint8, device=device)


def _ws(workspace: torch.Tensor):
    base = workspace.data_ptr()
    off = (-base) % 256
    return ctypes.c_void_p(base + off), workspace.numel() - off


def kvc_compress(shape: KvcShape, params: KvcParams, K: torch.Tensor, V: torch.Tensor,
                 vis_start: int, Kc: torch.Tensor, Vc: torch.Tensor, workspace: torch.Tensor,
                 stream=None, generic: bool = False, check: bool = True) -> int:
    """K, V: [B, H_kv, S, d] (d contiguous); Kc, Vc: [B, H_kv, I, m, d] outputs."""
    assert K.stride() == V.stride() and K.stride(3) == 1
    wp, wb = _ws(workspace)
    fn = lib().kvc_compress_generic if generic else lib().kvc_compress
    st = fn(ctypes.byref(shape), ctypes.byref(params), _ptr(K), _ptr(V), K.stride(0), K.stride(1),
            K.stride(2), int(vis_start), K.shape[2], _ptr(Kc), _ptr(Vc), wp, wb, _stream(stream))
    if check and st != KVC_OK:
        raise KvcError(st, "kvc_compress")
    return st


def kvc_reconstruct_attend_decode(shape: KvcShape, params: KvcParams, q, Kc, Vc, K_text, V_text,
                                  text_len: int, text_cap: int, k_new, v_new, softmax_scale: float,
                                  out, lse_out, workspace, stream=None, generic: bool = False,
                                  check: bool = True) -> int:
    """q, out: [B, H_q, d]; Kc, Vc: capsule; K_text, V_text: [B, H_kv, text_cap, d]."""
    wp, wb = _ws(workspace)
    fn = lib().kvc_reconstruct_attend_decode_generic if generic else \
        lib().kvc_reconstruct_attend_decode
    st = fn(ctypes.byref(shape), ctypes.byref(params), _ptr(q), _ptr(Kc), _ptr(Vc), _ptr(K_text),
            _ptr(V_text), int(text_len), int(text_cap), _ptr(k_new), _ptr(v_new),
            ctypes.c_float(softmax_scale), _ptr(out), _ptr(lse_out), wp, wb, _stream(stream))
    if check and st != KVC_OK:
        raise KvcError(st, "kvc_reconstruct_attend_decode")
    return st


def kvc_attend_full_workspace_bytes(batch, n_q_heads, n_kv_heads, head_dim, dtype, max_kv_len) -> int:
    code = dtype if isinstance(dtype, int) else _dtype_code(dtype)
    return int(lib().kvc_attend_full_workspace_bytes(batch, n_q_heads, n_kv_heads, head_dim, code,
                                                     int(max_kv_len)))


def kvc_attend_full_decode(q, K, V, kv_len: int, k_new, v_new, softmax_scale: float, out, lse_out,
                           workspace, stream=None, check: bool = True) -> int:
    """Full-cache decode attention.  q, out: [B, H_q, d]; K, V: [B, H_kv, kv_cap, d] (d contiguous)."""
    assert K.stride() == V.stride() and K.stride(3) == 1
    B, Hq, d = q.shape
    wp, wb = _ws(workspace)
    st = lib().kvc_attend_full_decode(B, Hq, K.shape[1], d, _dtype_code(q.dtype), _ptr(q), _ptr(K), _ptr(V),
                                      K.stride(0), K.stride(1), K.stride(2), int(kv_len), K.shape[2],
                                      _ptr(k_new), _ptr(v_new), ctypes.c_float(softmax_scale), _ptr(out),
                                      _ptr(lse_out), wp, wb, _stream(stream))
    if check and st != KVC_OK:
        raise KvcError(st, "kvc_attend_full_decode")
    return st


def kvc_reconstruct_attend_decode_static(shape: KvcShape, params: KvcParams, q, Kc, Vc, K_text, V_text,
                                         text_len: int, text_cap: int, k_new, v_new, softmax_scale: float,
                                         out, lse_out, stream=None, check: bool = True) -> int:
    """kvc_reconstruct_attend_decode with the library's own scratch array instead of a workspace."""
    st = lib().kvc_reconstruct_attend_decode_static(
        ctypes.byref(shape), ctypes.byref(params), _ptr(q), _ptr(Kc), _ptr(Vc), _ptr(K_text), _ptr(V_text),
        int(text_len), int(text_cap), _ptr(k_new), _ptr(v_new), ctypes.c_float(softmax_scale), _ptr(out),
        _ptr(lse_out), _stream(stream))
    if check and st != KVC_OK:
        raise KvcError(st, "kvc_reconstruct_attend_decode_static")
    return st


def kvc_unpack_values(Vc: torch.Tensor, m: int, d: int, stream=None) -> torch.Tensor:
    """Compressed values as kvc_compress stores them ([..., m*d] records) -> dense [..., m, d] (new tensor)."""
    dense = torch.empty(Vc.shape[:-2] + (m, d), dtype=Vc.dtype, device=Vc.device)
    records = Vc.numel() // (m * d)
    if records == 0:
        return dense
    st = lib().kvc_unpack_values(_ptr(Vc), _ptr(dense), records, int(m), int(d), _dtype_code(Vc.dtype),
                                 _stream(stream))
    if st != KVC_OK:
        raise KvcError(st, "kvc_unpack_values")
    return dense


def kvc_reconstruct_attend_decode_ragged(shape: KvcShape, params: KvcParams, q, Kc, Vc, K_text, V_text,
                                         n_images: torch.Tensor, text_len: torch.Tensor, text_cap: int, k_new,
                                         v_new, softmax_scale: float, out, lse_out, workspace, stream=None,
                                         check: bool = True) -> int:
    """n_images, text_len: int32 device tensors [B]."""
    assert n_images.dtype == torch.int32 and text_len.dtype == torch.int32
    wp, wb = _ws(workspace)
    st = lib().kvc_reconstruct_attend_decode_ragged(
        ctypes.byref(shape), ctypes.byref(params), _ptr(q), _ptr(Kc), _ptr(Vc), _ptr(K_text), _ptr(V_text),
        _ptr(n_images), _ptr(text_len), int(text_cap), _ptr(k_new), _ptr(v_new), ctypes.c_float(softmax_scale),
        _ptr(out), _ptr(lse_out), wp, wb, _stream(stream))
    if check and st != KVC_OK:
        raise KvcError(st, "kvc_reconstruct_attend_decode_ragged")
    return st


def kvc_mlp_hidden(shape: KvcShape, W1: torch.Tensor, activation: int, Kc: torch.Tensor, H: torch.Tensor,
                   stream=None, check: bool = True) -> int:
    st = lib().kvc_mlp_hidden(ctypes.byref(shape), _ptr(W1), int(activation), _ptr(Kc), _ptr(H), _stream(stream))
    if check and st != KVC_OK:
        raise KvcError(st, "kvc_mlp_hidden")
    return st


def kvc_static_attend_decode(shape: KvcShape, q, Kc, Vc, K_text, V_text, text_len: int, text_cap: int, k_new, v_new,
                             softmax_scale: float, out, lse_out, workspace, stream=None, check: bool = True) -> int:
    wp, wb = _ws(workspace)
    st = lib().kvc_static_attend_decode(ctypes.byref(shape), _ptr(q), _ptr(Kc), _ptr(Vc), _ptr(K_text), _ptr(V_text),
                                        int(text_len), int(text_cap), _ptr(k_new), _ptr(v_new),
                                        ctypes.c_float(softmax_scale), _ptr(out), _ptr(lse_out), wp, wb, _stream(stream))
    if check and st != KVC_OK:
        raise KvcError(st, "kvc_static_attend_decode")
    return st
