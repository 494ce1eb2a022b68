"""ctypes binding of libmlra.so: argument marshalling only.

Function names and argument order follow include/mlra.h.  Tensors are torch CUDA (ROCm) tensors
used purely as device memory; work is enqueued on torch's current stream.  Every step of the
path runs inside the library's HIP kernels; there is no fallback: if the library has not been
built, or an entry point reports an error, a RuntimeError is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmlra.so")
_lib: Optional[ctypes.CDLL] = None

MLRA_BF16, MLRA_F32 = 0, 1

EXPORTS = ("mlra_strerror", "mlra_append_kv", "mlra_absorb_q", "mlra_absorb_q_folded", "mlra2_absorb_q_folded",
           "mlra_decode_workspace_bytes",
           "mlra_decode_attn", "mlra_decode_attn_static", "mla_decode_attn", "mlra2_absorb_q", "mlra2_decode_workspace_bytes",
           "mlra2_decode_attn", "mlra_decode_attn_gated", "mlra_decode_multi_workspace_bytes", "mlra_decode_attn_multi",
           "mlra_pre_attention_workspace_bytes", "mlra_pre_attention",
           "gqa_decode_workspace_bytes", "gqa_decode_attn", "mlra_kernel_timing_begin",
           "mlra_kernel_timing_end", "mlra_decode_plan_info", "mlra_probe_stream_read", "mlra_probe_shader_clock")


class _CacheStruct(ctypes.Structure):
    _fields_ = [("latent", ctypes.c_void_p), ("rope", ctypes.c_void_p),
                ("page_table", ctypes.c_void_p), ("seq_lens", ctypes.c_void_p),
                ("num_pages", ctypes.c_int32), ("page_size", ctypes.c_int32),
                ("max_pages_per_seq", ctypes.c_int32), ("n_blocks", ctypes.c_int32),
                ("d_cb", ctypes.c_int32), ("d_r", ctypes.c_int32), ("dtype", ctypes.c_int32)]


class _PreWeightsStruct(ctypes.Structure):
    _fields_ = [("w_dq", ctypes.c_void_p), ("w_dkv", ctypes.c_void_p), ("w_kr", ctypes.c_void_p),
                ("w_uq", ctypes.c_void_p), ("w_qr", ctypes.c_void_p), ("gain_q", ctypes.c_void_p),
                ("gain_kv", ctypes.c_void_p), ("d", ctypes.c_int32), ("d_cq", ctypes.c_int32),
                ("h", ctypes.c_int32), ("d_h", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("alpha_q", ctypes.c_float), ("alpha_kv", ctypes.c_float), ("eps", ctypes.c_float),
                ("rope_base", ctypes.c_float)]


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Loads libmlra.so (built by `python -m paper_2603_02188_amd.build`); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2603_02188_amd.build` "
                           "(there is no CPU or PyTorch fallback for the MLRA decode path)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
    cp = ctypes.POINTER(_CacheStruct)
    lib.mlra_strerror.restype = ctypes.c_char_p
    lib.mlra_strerror.argtypes = [ctypes.c_int]
    lib.mlra_append_kv.restype = ctypes.c_int
    lib.mlra_append_kv.argtypes = [cp, i32, vp, vp, i32, vp, vp]
    lib.mlra_absorb_q.restype = ctypes.c_int
    lib.mlra_absorb_q.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, i32, vp]
    for fn in (lib.mlra_absorb_q_folded, lib.mlra2_absorb_q_folded):
        fn.restype = ctypes.c_int
        fn.argtypes = [i32, i32, i32, i32, i32, i32, vp, vp, vp, f32, vp, vp, i32, vp]
    lib.mlra_decode_workspace_bytes.restype = sz
    lib.mlra_decode_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
    lib.mlra_decode_attn.restype = ctypes.c_int
    lib.mlra_decode_attn.argtypes = [cp, i32, i32, i32, vp, vp, vp, f32, f32, vp, i32, vp, vp, sz, vp]
    lib.mlra_decode_attn_static.restype = ctypes.c_int
    lib.mlra_decode_attn_static.argtypes = [cp, i32, i32, i32, vp, vp, vp, f32, f32, vp, i32, vp, vp]
    lib.mlra2_absorb_q.restype = ctypes.c_int
    lib.mlra2_absorb_q.argtypes = lib.mlra_absorb_q.argtypes
    lib.mlra2_decode_workspace_bytes.restype = sz
    lib.mlra2_decode_workspace_bytes.argtypes = lib.mlra_decode_workspace_bytes.argtypes
    lib.mlra2_decode_attn.restype = ctypes.c_int
    lib.mlra2_decode_attn.argtypes = lib.mlra_decode_attn.argtypes
    lib.mlra_decode_attn_gated.restype = ctypes.c_int
    lib.mlra_decode_attn_gated.argtypes = [cp, i32, i32, i32, vp, vp, vp, vp, f32, f32, vp, i32, vp, vp, sz, vp]
    lib.mlra_decode_multi_workspace_bytes.restype = sz
    lib.mlra_decode_multi_workspace_bytes.argtypes = [i32] * 7
    lib.mlra_decode_attn_multi.restype = ctypes.c_int
    lib.mlra_decode_attn_multi.argtypes = [cp, i32, i32, i32, i32, vp, vp, vp, f32, f32, vp, i32, vp, vp, sz, vp]
    lib.mlra_pre_attention_workspace_bytes.restype = sz
    lib.mlra_pre_attention_workspace_bytes.argtypes = [i32] * 9
    lib.mlra_pre_attention.restype = ctypes.c_int
    lib.mlra_pre_attention.argtypes = [cp, ctypes.POINTER(_PreWeightsStruct), i32, vp, vp, vp, vp, vp, sz, vp]
    lib.mla_decode_attn.restype = ctypes.c_int
    lib.mla_decode_attn.argtypes = [cp, i32, i32, i32, vp, vp, vp, f32, vp, i32, vp, vp, sz, vp]
    lib.mlra_decode_plan_info.restype = ctypes.c_int
    lib.mlra_decode_plan_info.argtypes = [i32] * 10 + [ctypes.POINTER(ctypes.c_int32)]
    lib.gqa_decode_workspace_bytes.restype = sz
    lib.gqa_decode_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.gqa_decode_attn.restype = ctypes.c_int
    lib.gqa_decode_attn.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, vp, f32, vp, i32, vp,
                                    sz, vp]
    lib.mlra_probe_stream_read.restype = ctypes.c_int
    lib.mlra_probe_stream_read.argtypes = [vp, sz, vp, i32, vp]
    lib.mlra_probe_shader_clock.restype = ctypes.c_int
    lib.mlra_probe_shader_clock.argtypes = [vp, i32, vp]
    lib.mlra_kernel_timing_begin.restype = ctypes.c_int
    lib.mlra_kernel_timing_begin.argtypes = [i32]
    lib.mlra_kernel_timing_end.restype = ctypes.c_int
    lib.mlra_kernel_timing_end.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                           ctypes.POINTER(ctypes.c_int32)]
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load_library().mlra_strerror(int(status)).decode()


def _check(status: int, what: str) -> None:
    if status != 0:
        raise RuntimeError(f"{what} failed: {strerror(status)} (status {status})")


def _dt(t: torch.dtype) -> int:
    if t == torch.bfloat16:
        return MLRA_BF16
    if t == torch.float32:
        return MLRA_F32
    raise TypeError(f"libmlra supports bfloat16 and float32, not {t}")


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("libmlra takes contiguous device tensors")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


@dataclass
class Cache:
    """Paged latent KV cache (struct mlra_cache): device tensors plus their dimensions."""

    latent: torch.Tensor      # [num_pages][n_blocks][page_size][d_cb]
    rope: torch.Tensor        # [num_pages][page_size][d_r]
    page_table: torch.Tensor  # [batch][max_pages_per_seq] int32
    seq_lens: torch.Tensor    # [batch] int32

    def struct(self) -> _CacheStruct:
        P, NB, ps, dcb = self.latent.shape
        assert self.rope.shape[0] == P and self.rope.shape[1] == ps
        assert self.page_table.dtype == torch.int32 and self.seq_lens.dtype == torch.int32
        assert self.rope.dtype == self.latent.dtype
        return _CacheStruct(self.latent.data_ptr(), self.rope.data_ptr(), self.page_table.data_ptr(),
                            self.seq_lens.data_ptr(), P, ps, self.page_table.shape[1], NB, dcb,
                            self.rope.shape[2], _dt(self.latent.dtype))

    @property
    def max_seq_len(self) -> int:
        return int(self.page_table.shape[1] * self.latent.shape[2])


def mlra_append_kv(cache: Cache, c_kv_new: torch.Tensor, k_rope_new: torch.Tensor, positions: torch.Tensor,
                   stream=None) -> None:
    lib = load_library()
    cs = cache.struct()
    batch = int(positions.shape[0])
    assert c_kv_new.dtype == k_rope_new.dtype and positions.dtype == torch.int32
    _check(lib.mlra_append_kv(ctypes.byref(cs), batch, _ptr(c_kv_new), _ptr(k_rope_new), _dt(c_kv_new.dtype),
                              _ptr(positions), _stream(stream)), "mlra_append_kv")


def mlra_absorb_q(q_nope: torch.Tensor, w_uk: torch.Tensor, q_abs: Optional[torch.Tensor] = None,
                  stream=None) -> torch.Tensor:
    lib = load_library()
    batch, h, d_h = q_nope.shape
    n_blocks, d_cb, hd = w_uk.shape
    assert hd == h * d_h and w_uk.dtype == q_nope.dtype
    if q_abs is None:
        q_abs = torch.empty((batch, n_blocks, h, d_cb), dtype=q_nope.dtype, device=q_nope.device)
    _check(lib.mlra_absorb_q(batch, h, d_h, n_blocks, d_cb, _ptr(q_nope), _ptr(w_uk), _ptr(q_abs),
                             _dt(q_nope.dtype), _stream(stream)), "mlra_absorb_q")
    return q_abs


SCALE_FOLDED = 0.0   # softmax_scale for the decode calls when the queries come from *_absorb_q_folded


def _absorb_folded(entry: str, groups: int, q_nope, w_uk, q_rope, softmax_scale, q_abs, q_rope_out, stream):
    lib = load_library()
    batch, h, d_h = q_nope.shape
    n_blocks, d_cb, hd = w_uk.shape
    d_r = q_rope.shape[-1]
    assert h % groups == 0 and hd == (h // groups) * d_h and w_uk.dtype == q_nope.dtype == q_rope.dtype
    assert q_rope.numel() == batch * h * d_r
    if q_abs is None:
        q_abs = torch.empty((batch, n_blocks, h // groups, d_cb), dtype=q_nope.dtype, device=q_nope.device)
    if q_rope_out is None:
        q_rope_out = torch.empty_like(q_rope)
    _check(getattr(lib, entry)(batch, h, d_h, n_blocks, d_cb, d_r, _ptr(q_nope), _ptr(w_uk), _ptr(q_rope),
                               float(softmax_scale), _ptr(q_abs), _ptr(q_rope_out), _dt(q_nope.dtype),
                               _stream(stream)), entry)
    return q_abs, q_rope_out


def mlra_absorb_q_folded(q_nope: torch.Tensor, w_uk: torch.Tensor, q_rope: torch.Tensor, softmax_scale: float,
                         q_abs: Optional[torch.Tensor] = None, q_rope_out: Optional[torch.Tensor] = None,
                         stream=None):
    """(q_abs, q_rope_out), both multiplied by softmax_scale * log2(e): pass them to the decode calls with
    softmax_scale = SCALE_FOLDED."""
    return _absorb_folded("mlra_absorb_q_folded", 1, q_nope, w_uk, q_rope, softmax_scale, q_abs, q_rope_out, stream)


def mlra2_absorb_q_folded(q_nope: torch.Tensor, w_uk: torch.Tensor, q_rope: torch.Tensor, softmax_scale: float,
                          q_abs: Optional[torch.Tensor] = None, q_rope_out: Optional[torch.Tensor] = None,
                          stream=None):
    return _absorb_folded("mlra2_absorb_q_folded", 2, q_nope, w_uk, q_rope, softmax_scale, q_abs, q_rope_out, stream)


def mlra_decode_workspace_bytes(batch: int, h: int, n_blocks: int, d_cb: int, max_seq_len: int) -> int:
    return int(load_library().mlra_decode_workspace_bytes(batch, h, n_blocks, d_cb, max_seq_len))


def _decode(entry: str, cache: Cache, q_abs, q_rope, w_uv, softmax_scale, out_scale, out, out_dtype, lse,
            workspace, stream):
    lib = load_library()
    cs = cache.struct()
    batch, n_blocks, h, d_cb = q_abs.shape
    d_h = w_uv.shape[2] // h
    assert w_uv.shape == (n_blocks, d_cb, h * d_h) and q_rope.shape[:2] == (batch, h)
    if out is None:
        out = torch.empty((batch, h, d_h), dtype=out_dtype or q_abs.dtype, device=q_abs.device)
    if workspace is None:
        need = mlra_decode_workspace_bytes(batch, h, n_blocks, d_cb, cache.max_seq_len)
        workspace = torch.empty(need, dtype=torch.uint8, device=q_abs.device)
    args = [ctypes.byref(cs), batch, h, d_h, _ptr(q_abs), _ptr(q_rope), _ptr(w_uv), float(softmax_scale)]
    if entry == "mlra_decode_attn":
        args.append(float(out_scale))
    args += [_ptr(out), _dt(out.dtype), _ptr(lse), _ptr(workspace), workspace.numel() * workspace.element_size(),
             _stream(stream)]
    _check(getattr(lib, entry)(*args), entry)
    return out


def mlra_decode_attn(cache: Cache, q_abs: torch.Tensor, q_rope: torch.Tensor, w_uv: torch.Tensor,
                     softmax_scale: float, out_scale: float = 1.0, out: Optional[torch.Tensor] = None,
                     out_dtype: Optional[torch.dtype] = None, lse: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    return _decode("mlra_decode_attn", cache, q_abs, q_rope, w_uv, softmax_scale, out_scale, out, out_dtype, lse,
                   workspace, stream)


def mlra_decode_attn_static(cache: Cache, q_abs: torch.Tensor, q_rope: torch.Tensor, w_uv: torch.Tensor,
                            softmax_scale: float, out_scale: float, out: torch.Tensor,
                            lse: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """mlra_decode_attn on the library's built-in scratch memory: the caller passes every buffer (out
    included) and nothing is allocated, here or in the library."""
    lib = load_library()
    cs = cache.struct()
    batch, n_blocks, h, d_cb = q_abs.shape
    d_h = w_uv.shape[2] // h
    assert w_uv.shape == (n_blocks, d_cb, h * d_h) and q_rope.shape[:2] == (batch, h) and out.shape == (batch, h, d_h)
    _check(lib.mlra_decode_attn_static(ctypes.byref(cs), batch, h, d_h, _ptr(q_abs), _ptr(q_rope), _ptr(w_uv),
                                       float(softmax_scale), float(out_scale), _ptr(out), _dt(out.dtype), _ptr(lse),
                                       _stream(stream)), "mlra_decode_attn_static")
    return out


def mla_decode_attn(cache: Cache, q_abs: torch.Tensor, q_rope: torch.Tensor, w_uv: torch.Tensor,
                    softmax_scale: float, out: Optional[torch.Tensor] = None,
                    out_dtype: Optional[torch.dtype] = None, lse: Optional[torch.Tensor] = None,
                    workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    return _decode("mla_decode_attn", cache, q_abs, q_rope, w_uv, softmax_scale, 1.0, out, out_dtype, lse,
                   workspace, stream)


def mlra_decode_attn_gated(cache: Cache, q_abs: torch.Tensor, q_rope: torch.Tensor, w_uv: torch.Tensor,
                           gate: torch.Tensor, softmax_scale: float, out_scale: float = 1.0,
                           out: Optional[torch.Tensor] = None, out_dtype: Optional[torch.dtype] = None,
                           lse: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                           stream=None) -> torch.Tensor:
    """mlra_decode_attn with the output multiplied elementwise by gate [batch][h][d_h] (Appendix E)."""
    lib = load_library()
    cs = cache.struct()
    batch, n_blocks, h, d_cb = q_abs.shape
    d_h = w_uv.shape[2] // h
    assert gate.shape == (batch, h, d_h) and gate.dtype == q_abs.dtype
    if out is None:
        out = torch.empty((batch, h, d_h), dtype=out_dtype or q_abs.dtype, device=q_abs.device)
    if workspace is None:
        need = mlra_decode_workspace_bytes(batch, h, n_blocks, d_cb, cache.max_seq_len)
        workspace = torch.empty(need, dtype=torch.uint8, device=q_abs.device)
    _check(lib.mlra_decode_attn_gated(ctypes.byref(cs), batch, h, d_h, _ptr(q_abs), _ptr(q_rope), _ptr(w_uv),
                                      _ptr(gate), float(softmax_scale), float(out_scale), _ptr(out), _dt(out.dtype),
                                      _ptr(lse), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                      _stream(stream)), "mlra_decode_attn_gated")
    return out


def mlra_decode_multi_workspace_bytes(batch: int, q_len: int, h: int, n_blocks: int, d_cb: int, page_size: int,
                                      max_pages_per_seq: int) -> int:
    return int(load_library().mlra_decode_multi_workspace_bytes(batch, q_len, h, n_blocks, d_cb, page_size,
                                                                max_pages_per_seq))


def mlra_decode_attn_multi(cache: Cache, q_abs: torch.Tensor, q_rope: torch.Tensor, w_uv: torch.Tensor,
                           softmax_scale: float, out_scale: float = 1.0, out: Optional[torch.Tensor] = None,
                           out_dtype: Optional[torch.dtype] = None, lse: Optional[torch.Tensor] = None,
                           workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """q_abs [batch][q_len][n_blocks][h][d_cb], q_rope [batch][q_len][h][d_r] -> out [batch][q_len][h][d_h]."""
    lib = load_library()
    cs = cache.struct()
    batch, q_len, n_blocks, h, d_cb = q_abs.shape
    d_h = w_uv.shape[2] // h
    assert w_uv.shape == (n_blocks, d_cb, h * d_h) and q_rope.shape[:3] == (batch, q_len, h)
    if out is None:
        out = torch.empty((batch, q_len, h, d_h), dtype=out_dtype or q_abs.dtype, device=q_abs.device)
    if workspace is None:
        need = mlra_decode_multi_workspace_bytes(batch, q_len, h, n_blocks, d_cb, cs.page_size, cs.max_pages_per_seq)
        workspace = torch.empty(need, dtype=torch.uint8, device=q_abs.device)
    _check(lib.mlra_decode_attn_multi(ctypes.byref(cs), batch, q_len, h, d_h, _ptr(q_abs), _ptr(q_rope), _ptr(w_uv),
                                      float(softmax_scale), float(out_scale), _ptr(out), _dt(out.dtype), _ptr(lse),
                                      _ptr(workspace), workspace.numel() * workspace.element_size(),
                                      _stream(stream)), "mlra_decode_attn_multi")
    return out


def mlra2_absorb_q(q_nope: torch.Tensor, w_uk: torch.Tensor, q_abs: Optional[torch.Tensor] = None,
                   stream=None) -> torch.Tensor:
    """MLRA-2: w_uk [n_blocks][d_cb][(h/2)*d_h] -> q_abs [batch][n_blocks][h/2][d_cb]."""
    lib = load_library()
    batch, h, d_h = q_nope.shape
    n_blocks, d_cb, hd = w_uk.shape
    assert h % 2 == 0 and hd == (h // 2) * d_h and w_uk.dtype == q_nope.dtype
    if q_abs is None:
        q_abs = torch.empty((batch, n_blocks, h // 2, d_cb), dtype=q_nope.dtype, device=q_nope.device)
    _check(lib.mlra2_absorb_q(batch, h, d_h, n_blocks, d_cb, _ptr(q_nope), _ptr(w_uk), _ptr(q_abs),
                              _dt(q_nope.dtype), _stream(stream)), "mlra2_absorb_q")
    return q_abs


def mlra2_decode_workspace_bytes(batch: int, h: int, n_blocks: int, d_cb: int, max_seq_len: int) -> int:
    return int(load_library().mlra2_decode_workspace_bytes(batch, h, n_blocks, d_cb, max_seq_len))


def mlra2_decode_attn(cache: Cache, q_abs: torch.Tensor, q_rope: torch.Tensor, w_uv: torch.Tensor,
                      softmax_scale: float, out_scale: float = 1.0, out: Optional[torch.Tensor] = None,
                      out_dtype: Optional[torch.dtype] = None, lse: Optional[torch.Tensor] = None,
                      workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """MLRA-2: q_abs [batch][n_blocks][h/2][d_cb], q_rope [batch][h][d_r], w_uv [n_blocks][d_cb][(h/2)*d_h],
    lse [batch][n_blocks][h/2]; returns out [batch][h][d_h]."""
    lib = load_library()
    cs = cache.struct()
    batch, n_blocks, hb, d_cb = q_abs.shape
    h = 2 * hb
    d_h = w_uv.shape[2] // hb
    assert w_uv.shape == (n_blocks, d_cb, hb * d_h) and q_rope.shape[:2] == (batch, h)
    if out is None:
        out = torch.empty((batch, h, d_h), dtype=out_dtype or q_abs.dtype, device=q_abs.device)
    if workspace is None:
        need = mlra2_decode_workspace_bytes(batch, h, n_blocks, d_cb, cache.max_seq_len)
        workspace = torch.empty(need, dtype=torch.uint8, device=q_abs.device)
    _check(lib.mlra2_decode_attn(ctypes.byref(cs), batch, h, d_h, _ptr(q_abs), _ptr(q_rope), _ptr(w_uv),
                                 float(softmax_scale), float(out_scale), _ptr(out), _dt(out.dtype), _ptr(lse),
                                 _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
           "mlra2_decode_attn")
    return out


@dataclass
class PreWeights:
    """Projection weights of the pre-attention (struct mlra_pre_weights): device tensors and scalars."""

    w_dq: torch.Tensor       # [d][d_cq]
    w_dkv: torch.Tensor      # [d][n_blocks*d_cb]
    w_kr: torch.Tensor       # [d][d_r]
    w_uq: torch.Tensor       # [d_cq][h*d_h]
    w_qr: torch.Tensor       # [d_cq][h*d_r]
    h: int
    alpha_q: float
    alpha_kv: float
    gain_q: Optional[torch.Tensor] = None
    gain_kv: Optional[torch.Tensor] = None
    eps: float = 1e-6
    rope_base: float = 10000.0

    def struct(self) -> _PreWeightsStruct:
        d, d_cq = self.w_dq.shape
        d_h = self.w_uq.shape[1] // self.h
        assert self.w_uq.shape == (d_cq, self.h * d_h) and self.w_dkv.shape[0] == d and self.w_kr.shape[0] == d
        for t in (self.w_dkv, self.w_kr, self.w_uq, self.w_qr):
            assert t.dtype == self.w_dq.dtype
        gp = lambda t: None if t is None else t.data_ptr()
        return _PreWeightsStruct(_ptr(self.w_dq), _ptr(self.w_dkv), _ptr(self.w_kr), _ptr(self.w_uq),
                                 _ptr(self.w_qr), _ptr(self.gain_q), _ptr(self.gain_kv), d, d_cq, self.h, d_h,
                                 _dt(self.w_dq.dtype), self.alpha_q, self.alpha_kv, self.eps, self.rope_base)


def mlra_pre_attention_workspace_bytes(batch, d, d_cq, n_blocks, d_cb, d_r, h, d_h, dtype) -> int:
    return int(load_library().mlra_pre_attention_workspace_bytes(batch, d, d_cq, n_blocks, d_cb, d_r, h, d_h,
                                                                  _dt(dtype)))


def mlra_pre_attention(cache: Cache, weights: PreWeights, hidden: torch.Tensor, positions: torch.Tensor,
                       q_nope: Optional[torch.Tensor] = None, q_rope: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None, stream=None):
    """Projects the new token of every sequence, stores its cache row and returns (q_nope, q_rope)."""
    lib = load_library()
    cs, ws = cache.struct(), weights.struct()
    batch, d = hidden.shape
    assert d == ws.d and hidden.dtype == weights.w_dq.dtype and positions.dtype == torch.int32
    if q_nope is None:
        q_nope = torch.empty((batch, ws.h, ws.d_h), dtype=hidden.dtype, device=hidden.device)
    if q_rope is None:
        q_rope = torch.empty((batch, ws.h, cs.d_r), dtype=hidden.dtype, device=hidden.device)
    if workspace is None:
        need = mlra_pre_attention_workspace_bytes(batch, d, ws.d_cq, cs.n_blocks, cs.d_cb, cs.d_r, ws.h, ws.d_h,
                                                  hidden.dtype)
        workspace = torch.empty(need, dtype=torch.uint8, device=hidden.device)
    _check(lib.mlra_pre_attention(ctypes.byref(cs), ctypes.byref(ws), batch, _ptr(hidden), _ptr(positions),
                                  _ptr(q_nope), _ptr(q_rope), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream(stream)),
           "mlra_pre_attention")
    return q_nope, q_rope


def gqa_decode_workspace_bytes(batch: int, h: int, d_h: int, max_seq_len: int) -> int:
    return int(load_library().gqa_decode_workspace_bytes(batch, h, d_h, max_seq_len))


def gqa_decode_attn(k_pool: torch.Tensor, v_pool: torch.Tensor, page_table: torch.Tensor, seq_lens: torch.Tensor,
                    q: torch.Tensor, softmax_scale: float, out: Optional[torch.Tensor] = None,
                    out_dtype: Optional[torch.dtype] = None, workspace: Optional[torch.Tensor] = None,
                    stream=None) -> torch.Tensor:
    lib = load_library()
    P, g, ps, d_h = k_pool.shape
    batch, h, _ = q.shape
    max_pages = int(page_table.shape[1])
    if out is None:
        out = torch.empty((batch, h, d_h), dtype=out_dtype or q.dtype, device=q.device)
    if workspace is None:
        workspace = torch.empty(gqa_decode_workspace_bytes(batch, h, d_h, max_pages * ps), dtype=torch.uint8,
                                device=q.device)
    _check(lib.gqa_decode_attn(_ptr(k_pool), _ptr(v_pool), _ptr(page_table), _ptr(seq_lens), P, ps, max_pages,
                               batch, h, g, d_h, _dt(k_pool.dtype), _ptr(q), float(softmax_scale), _ptr(out),
                               _dt(out.dtype), _ptr(workspace), workspace.numel() * workspace.element_size(),
                               _stream(stream)), "gqa_decode_attn")
    return out


DECODE_KERNELS = ("generic", "mfma", "mfma-paired", "mfma-gla", "mfma-mla")


def mlra_decode_plan_info(batch: int, h: int, d_h: int, groups: int, n_blocks: int, d_cb: int, d_r: int,
                          page_size: int, max_seq_len: int, dtype: torch.dtype) -> dict:
    """Which kernels and which context split a decode call of this shape takes (host logic only)."""
    info = (ctypes.c_int32 * 6)()
    _check(load_library().mlra_decode_plan_info(batch, h, d_h, groups, n_blocks, d_cb, d_r, page_size, max_seq_len,
                                                _dt(dtype), info), "mlra_decode_plan_info")
    return {"kernel": DECODE_KERNELS[info[0]], "chunk_slots": info[1], "chunk_tokens": info[2],
            "target_chunks": info[3], "single_if_uniform": bool(info[4]), "merge_mfma": bool(info[5])}


def mlra_kernel_timing_begin(max_calls: int) -> None:
    _check(load_library().mlra_kernel_timing_begin(int(max_calls)), "mlra_kernel_timing_begin")


def mlra_kernel_timing_end():
    """Returns (main kernel ms, epilogue kernel ms, calls measured), averages over the calls."""
    a, b, n = ctypes.c_double(), ctypes.c_double(), ctypes.c_int32()
    _check(load_library().mlra_kernel_timing_end(ctypes.byref(a), ctypes.byref(b), ctypes.byref(n)),
           "mlra_kernel_timing_end")
    return a.value, b.value, n.value


def mlra_probe_stream_read(src: torch.Tensor, sink: torch.Tensor, workgroups: int, stream=None) -> None:
    """Plain streaming read of the whole tensor `src` (see include/mlra.h); sink: int32/uint32 [workgroups]."""
    assert sink.numel() >= workgroups and sink.element_size() == 4
    _check(load_library().mlra_probe_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink),
                                                 int(workgroups), _stream(stream)), "mlra_probe_stream_read")


def mlra_probe_shader_clock(out: torch.Tensor, spin_us: int, stream=None) -> None:
    """out: int64 [2] on the device; receives {shader cycles, 10 ns ticks} of a spin of about spin_us microseconds."""
    assert out.dtype == torch.int64 and out.numel() >= 2
    _check(load_library().mlra_probe_shader_clock(_ptr(out), int(spin_us), _stream(stream)), "mlra_probe_shader_clock")
