"""Thin ctypes binding of ``libhstu_attn.so`` (C ABI: include/hstu_attn.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch supplies device memory and streams.  There is no CPU fallback:
importing this module without the built library raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# HSTU_ATTN_LIB lets a developer point the binding at another build of the same library
LIB_PATH = os.environ.get("HSTU_ATTN_LIB") or os.path.join(_HERE, "libhstu_attn.so")

HSTU_BF16, HSTU_FP32 = 0, 1
HSTU_OK = 0


class HstuError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


class HstuAttnParams(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("num_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("total_tokens", ctypes.c_int32), ("max_seqlen", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("row_stride_q", ctypes.c_int64), ("row_stride_k", ctypes.c_int64),
        ("row_stride_v", ctypes.c_int64), ("row_stride_o", ctypes.c_int64),
        ("seq_offsets", ctypes.c_void_p), ("seq_offsets_host", ctypes.c_void_p), ("num_targets", ctypes.c_void_p),
        ("local_window", ctypes.c_int32), ("global_prefix", ctypes.c_int32),
        ("alpha", ctypes.c_float), ("inv_n", ctypes.c_float),
        ("rab_table", ctypes.c_void_p), ("rab_bounds", ctypes.c_void_p), ("num_buckets", ctypes.c_int32),
        ("d_rab_table", ctypes.c_void_p), ("query_tail", ctypes.c_int32), ("reuse_schedule", ctypes.c_int32),
    ]


class HstuLayerParams(ctypes.Structure):
    _fields_ = [
        ("attn", HstuAttnParams), ("embed_dim", ctypes.c_int32), ("norm_eps", ctypes.c_float),
        ("gated_norm_eps", ctypes.c_float), ("norm_w", ctypes.c_void_p), ("w1", ctypes.c_void_p),
        ("gated_norm_w", ctypes.c_void_p), ("w2", ctypes.c_void_p),
        ("w1_q", ctypes.c_void_p), ("w1_scale", ctypes.c_void_p), ("w2_q", ctypes.c_void_p), ("w2_scale", ctypes.c_void_p),
    ]


class HstuLbslConfig(ctypes.Structure):
    _fields_ = [("world_size", ctypes.c_int32), ("warmup_steps", ctypes.c_int32), ("recal_interval", ctypes.c_int32),
                ("sl_len", ctypes.c_int32), ("gamma", ctypes.c_double)]


class HstuLbslState(ctypes.Structure):
    _fields_ = [("step", ctypes.c_int64), ("target", ctypes.c_double), ("rank_load", ctypes.c_void_p)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2602_16986_amd.build` "
                          "(or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz, i32, i64, f32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    pp = ctypes.POINTER(HstuAttnParams)
    lib.hstu_status_string.restype = ctypes.c_char_p
    lib.hstu_status_string.argtypes = [ctypes.c_int]
    lib.hstu_attn_workspace_bytes.restype = sz
    lib.hstu_attn_workspace_bytes.argtypes = [pp, ctypes.c_int]
    lib.hstu_attn_fwd.restype = ctypes.c_int
    lib.hstu_attn_fwd.argtypes = [pp, vp, vp, vp, vp, vp, sz, vp]
    lib.hstu_attn_bwd.restype = ctypes.c_int
    lib.hstu_attn_bwd.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.hstu_attn_schedule_stats.restype = ctypes.c_int
    lib.hstu_attn_schedule_stats.argtypes = [pp, vp, ctypes.c_int, ctypes.POINTER(ctypes.c_int64)]
    lib.hstu_gated_norm_fwd.restype = ctypes.c_int
    lib.hstu_gated_norm_fwd.argtypes = [i64, i32, i32, vp, vp, vp, vp, f32, vp, vp, vp, vp]
    lib.hstu_gated_norm_bwd_workspace_bytes.restype = sz
    lib.hstu_gated_norm_bwd_workspace_bytes.argtypes = [i64, i32]
    lib.hstu_gated_norm_bwd.restype = ctypes.c_int
    lib.hstu_gated_norm_bwd.argtypes = [i64, i32, i32, vp, vp, vp, vp, vp, f32, vp, vp, vp, vp, vp, sz, vp]
    lib.hstu_gated_norm_bwd_static_max_bytes.restype = sz
    lib.hstu_gated_norm_bwd_static_max_bytes.argtypes = []
    lib.hstu_gated_norm_bwd_static.restype = ctypes.c_int
    lib.hstu_gated_norm_bwd_static.argtypes = [i64, i32, i32, vp, vp, vp, vp, vp, f32, vp, vp, vp, vp, vp]
    lib.hstu_truncate_offsets.restype = ctypes.c_int
    lib.hstu_truncate_offsets.argtypes = [i32, i32, vp, vp, vp, vp]
    lib.hstu_truncate_fwd.restype = ctypes.c_int
    lib.hstu_truncate_fwd.argtypes = [i32, vp, vp, i64, vp, i64, vp, i64, i64, vp]
    lib.hstu_truncate_bwd.restype = ctypes.c_int
    lib.hstu_truncate_bwd.argtypes = [i32, i64, vp, vp, i64, vp, i64, vp, i64, vp]
    lp = ctypes.POINTER(HstuLayerParams)
    lib.hstu_layer_workspace_bytes.restype = sz
    lib.hstu_layer_workspace_bytes.argtypes = [lp, ctypes.c_int]
    lib.hstu_layer_fwd.restype = ctypes.c_int
    lib.hstu_layer_fwd.argtypes = [lp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.hstu_layer_bwd.restype = ctypes.c_int
    lib.hstu_layer_bwd.argtypes = [lp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.hstu_layer_gemm_tunings.restype = ctypes.c_int64
    lib.hstu_layer_gemm_tunings.argtypes = []
    lib.hstu_norm_quant_fp8.restype = ctypes.c_int
    lib.hstu_norm_quant_fp8.argtypes = [i64, i32, i32, vp, vp, vp, vp, f32, vp, vp, vp, vp, vp]
    lib.hstu_fp8_gemm_bias2d.restype = ctypes.c_int
    lib.hstu_fp8_gemm_bias2d.argtypes = [i64, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    cp, sp = ctypes.POINTER(HstuLbslConfig), ctypes.POINTER(HstuLbslState)
    lib.hstu_lbsl_weight.restype = ctypes.c_double
    lib.hstu_lbsl_weight.argtypes = [i32, i32]
    lib.hstu_lbsl_expected_load.restype = ctypes.c_double
    lib.hstu_lbsl_expected_load.argtypes = [i32, i32, ctypes.c_double]
    lib.hstu_lbsl_init.restype = ctypes.c_int
    lib.hstu_lbsl_init.argtypes = [cp, sp]
    lib.hstu_lbsl_step.restype = ctypes.c_int
    lib.hstu_lbsl_step.argtypes = [cp, sp, vp, vp, vp, vp, vp, vp]
    lib.hstu_lbsl_fit_gamma.restype = ctypes.c_int
    lib.hstu_lbsl_fit_gamma.argtypes = [i32, vp, vp, ctypes.POINTER(ctypes.c_double)]
    lib.hstu_profile_enable.restype = ctypes.c_int
    lib.hstu_profile_enable.argtypes = [ctypes.c_int]
    lib.hstu_profile_read.restype = ctypes.c_int
    lib.hstu_profile_read.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_float)]
    return lib


_lib = _load()
EXPORTS = ["hstu_attn_workspace_bytes", "hstu_attn_fwd", "hstu_attn_bwd", "hstu_gated_norm_fwd",
           "hstu_gated_norm_bwd_workspace_bytes", "hstu_gated_norm_bwd", "hstu_status_string",
           "hstu_gated_norm_bwd_static_max_bytes", "hstu_gated_norm_bwd_static",
           "hstu_attn_schedule_stats", "hstu_profile_enable", "hstu_profile_read",
           "hstu_truncate_offsets", "hstu_truncate_fwd", "hstu_truncate_bwd",
           "hstu_layer_workspace_bytes", "hstu_layer_fwd", "hstu_layer_bwd", "hstu_layer_gemm_tunings",
           "hstu_norm_quant_fp8", "hstu_fp8_gemm_bias2d",
           "hstu_lbsl_weight", "hstu_lbsl_expected_load", "hstu_lbsl_init", "hstu_lbsl_step", "hstu_lbsl_fit_gamma"]


def status_string(status: int) -> str:
    return _lib.hstu_status_string(int(status)).decode()


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return HSTU_BF16
    if t.dtype == torch.float32:
        return HSTU_FP32
    raise HstuError(-3, f"dtype {t.dtype}")


class AttnProblem:
    """Owns an ``hstu_attn_params`` struct and keeps the tensors it points to alive."""

    def __init__(self, q, k, v, out_like, seq_offsets, *, max_seqlen, seq_offsets_host=None, num_targets=None,
                 local_window=-1, global_prefix=0, alpha=1.0, inv_n=1.0, rab_table=None, rab_bounds=None,
                 d_rab_table=None, query_tail=0, reuse_schedule=False):
        T, H, d = q.shape
        self._keep = (seq_offsets, num_targets, rab_table, rab_bounds, d_rab_table)
        self._host = None if seq_offsets_host is None else np.ascontiguousarray(seq_offsets_host, dtype=np.int32)
        p = HstuAttnParams()
        p.batch = int(seq_offsets.shape[0]) - 1
        p.num_heads, p.head_dim, p.total_tokens, p.max_seqlen = H, d, T, int(max_seqlen)
        p.dtype = _dtype_code(q)
        for name, t in (("q", q), ("k", k), ("v", v), ("o", out_like)):
            assert T == 0 or (t.stride(2) == 1 and t.stride(1) == d), "head stride must be d, features contiguous"
            setattr(p, f"row_stride_{name}", t.stride(0) if T > 0 else H * d)
        p.seq_offsets = _ptr(seq_offsets)
        p.seq_offsets_host = None if self._host is None else self._host.ctypes.data
        p.num_targets = _ptr(num_targets)
        p.local_window, p.global_prefix = int(local_window), int(global_prefix)
        p.alpha, p.inv_n = float(alpha), float(inv_n)
        p.rab_table, p.rab_bounds = _ptr(rab_table), _ptr(rab_bounds)
        p.num_buckets = 0 if rab_bounds is None else int(rab_bounds.shape[0])
        p.d_rab_table = _ptr(d_rab_table)          # fp32 [H, num_buckets] output of hstu_attn_bwd, or None
        p.query_tail = int(query_tail)             # forward only: compute the last rows of every sequence only
        p.reuse_schedule = int(bool(reuse_schedule))   # the workspace still holds this entry point's work lists for this batch
        self.params = p

    def ref(self):
        return ctypes.byref(self.params)


def hstu_attn_workspace_bytes(prob: AttnProblem, for_backward: bool) -> int:
    return int(_lib.hstu_attn_workspace_bytes(prob.ref(), 1 if for_backward else 0))


def new_workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def hstu_attn_fwd(prob: AttnProblem, q, k, v, out, workspace: torch.Tensor, stream=None) -> None:
    st = _lib.hstu_attn_fwd(prob.ref(), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(workspace), workspace.numel(),
                            _stream(stream))
    if st != HSTU_OK:
        raise HstuError(st, "hstu_attn_fwd")


def hstu_attn_bwd(prob: AttnProblem, q, k, v, dout, dq, dk, dv, workspace: torch.Tensor, stream=None) -> None:
    st = _lib.hstu_attn_bwd(prob.ref(), _ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv),
                            _ptr(workspace), workspace.numel(), _stream(stream))
    if st != HSTU_OK:
        raise HstuError(st, "hstu_attn_bwd")


def hstu_attn_schedule_stats(prob: AttnProblem, workspace: torch.Tensor, for_backward: bool = False):
    out = (ctypes.c_int64 * 3)()
    st = _lib.hstu_attn_schedule_stats(prob.ref(), _ptr(workspace), 1 if for_backward else 0, out)
    if st != HSTU_OK:
        raise HstuError(st, "hstu_attn_schedule_stats")
    return {"items": int(out[0]), "tiles": int(out[1]), "dense_tiles": int(out[2])}


def hstu_gated_norm_fwd(attn, u, gamma, beta, eps, y, mean=None, rstd=None, stream=None) -> None:
    T = attn.shape[0]
    D = attn.numel() // T if T else int(np.prod(attn.shape[1:]))
    st = _lib.hstu_gated_norm_fwd(T, D, _dtype_code(attn), _ptr(attn), _ptr(u), _ptr(gamma), _ptr(beta), float(eps),
                                  _ptr(y), _ptr(mean), _ptr(rstd), _stream(stream))
    if st != HSTU_OK:
        raise HstuError(st, "hstu_gated_norm_fwd")


def hstu_gated_norm_bwd_workspace_bytes(T: int, D: int) -> int:
    return int(_lib.hstu_gated_norm_bwd_workspace_bytes(T, D))


def hstu_gated_norm_bwd(dy, attn, u, gamma, beta, eps, dattn, du, dgamma, dbeta, workspace, stream=None) -> None:
    T = attn.shape[0]
    D = attn.numel() // T if T else int(np.prod(attn.shape[1:]))
    st = _lib.hstu_gated_norm_bwd(T, D, _dtype_code(attn), _ptr(dy), _ptr(attn), _ptr(u), _ptr(gamma), _ptr(beta),
                                  float(eps), _ptr(dattn), _ptr(du), _ptr(dgamma), _ptr(dbeta), _ptr(workspace),
                                  workspace.numel(), _stream(stream))
    if st != HSTU_OK:
        raise HstuError(st, "hstu_gated_norm_bwd")


def hstu_gated_norm_bwd_static_max_bytes() -> int:
    return int(_lib.hstu_gated_norm_bwd_static_max_bytes())


def hstu_gated_norm_bwd_static(dy, attn, u, gamma, beta, eps, dattn, du, dgamma, dbeta, stream=None) -> None:
    T = attn.shape[0]
    D = attn.numel() // T if T else int(np.prod(attn.shape[1:]))
    st = _lib.hstu_gated_norm_bwd_static(T, D, _dtype_code(attn), _ptr(dy), _ptr(attn), _ptr(u), _ptr(gamma), _ptr(beta),
                                         float(eps), _ptr(dattn), _ptr(du), _ptr(dgamma), _ptr(dbeta), _stream(stream))
    if st != HSTU_OK:
        raise HstuError(st, "hstu_gated_norm_bwd_static")


def _row_geometry(t: torch.Tensor):
    """(row bytes, row stride in bytes) of a tensor of rows (dim 0) that are contiguous inside."""
    assert t.dim() >= 2, "expected [rows, ...]"
    inner = int(np.prod(t.shape[1:]))
    expect = 1
    for size, stride in zip(reversed(t.shape[1:]), reversed(t.stride()[1:]) if t.numel() else ()):
        assert size == 1 or stride == expect, "rows must be contiguous inside"
        expect *= size
    stride = t.stride(0) if t.shape[0] > 1 else inner
    return inner * t.element_size(), stride * t.element_size()


def hstu_truncate_offsets(seq_offsets, keep: int, num_targets, out_offsets, stream=None) -> None:
    st = _lib.hstu_truncate_offsets(int(seq_offsets.shape[0]) - 1, int(keep), _ptr(seq_offsets), _ptr(num_targets),
                                    _ptr(out_offsets), _stream(stream))
    if st != HSTU_OK:
        raise HstuError(st, "hstu_truncate_offsets")


def hstu_truncate_fwd(seq_offsets, out_offsets, x, y, stream=None) -> None:
    """y[r] = r-th surviving row of x; y.shape[0] is the capacity in rows."""
    if x.shape[0] == 0 or y.shape[0] == 0:
        return                                   # nothing survives / nowhere to put it
    row_bytes, xs = _row_geometry(x)
    rb2, ys = _row_geometry(y)
    assert rb2 == row_bytes
    st = _lib.hstu_truncate_fwd(int(seq_offsets.shape[0]) - 1, _ptr(seq_offsets), _ptr(out_offsets), row_bytes, _ptr(x), xs,
                                _ptr(y), ys, int(y.shape[0]), _stream(stream))
    if st != HSTU_OK:
        raise HstuError(st, "hstu_truncate_fwd")


def hstu_truncate_bwd(seq_offsets, out_offsets, dy, dx, stream=None) -> None:
    """dx (all T rows) = gradient rows of the survivors, zero elsewhere."""
    row_bytes, xs = _row_geometry(dx)
    _, ys = _row_geometry(dy)
    st = _lib.hstu_truncate_bwd(int(seq_offsets.shape[0]) - 1, int(dx.shape[0]), _ptr(seq_offsets), _ptr(out_offsets),
                                row_bytes, _ptr(dy), ys, _ptr(dx), xs, _stream(stream))
    if st != HSTU_OK:
        raise HstuError(st, "hstu_truncate_bwd")


class LayerProblem:
    """Owns an ``hstu_layer_params`` struct (bf16 layer) and keeps the tensors it points to alive."""

    def __init__(self, *, num_heads, head_dim, embed_dim, total_tokens, seq_offsets, max_seqlen, norm_w, w1, gated_norm_w,
                 w2, num_targets=None, local_window=-1, global_prefix=0, alpha=1.0, inv_n=1.0, rab_table=None,
                 rab_bounds=None, d_rab_table=None, norm_eps=1e-5, gated_norm_eps=1e-5, w1_q=None, w1_scale=None, w2_q=None,
                 w2_scale=None):
        hd = num_heads * head_dim
        assert w1.dtype == torch.bfloat16 and w2.dtype == torch.bfloat16 and w1.is_contiguous() and w2.is_contiguous()
        assert tuple(w1.shape) == (4 * hd, embed_dim) and tuple(w2.shape) == (embed_dim, hd)
        assert norm_w.dtype == torch.float32 and gated_norm_w.dtype == torch.float32
        self._keep = (seq_offsets, num_targets, rab_table, rab_bounds, d_rab_table, norm_w, w1, gated_norm_w, w2, w1_q, w1_scale,
                      w2_q, w2_scale)
        p = HstuLayerParams()
        a = p.attn
        a.batch = int(seq_offsets.shape[0]) - 1
        a.num_heads, a.head_dim, a.total_tokens, a.max_seqlen = num_heads, head_dim, int(total_tokens), int(max_seqlen)
        a.dtype = HSTU_BF16
        a.row_stride_q = a.row_stride_k = a.row_stride_v = 4 * hd      # ignored by the layer entry points
        a.row_stride_o = hd
        a.seq_offsets, a.seq_offsets_host, a.num_targets = _ptr(seq_offsets), None, _ptr(num_targets)
        a.local_window, a.global_prefix = int(local_window), int(global_prefix)
        a.alpha, a.inv_n = float(alpha), float(inv_n)
        a.rab_table, a.rab_bounds = _ptr(rab_table), _ptr(rab_bounds)
        a.num_buckets = 0 if rab_bounds is None else int(rab_bounds.shape[0])
        a.d_rab_table = _ptr(d_rab_table)
        p.embed_dim, p.norm_eps, p.gated_norm_eps = int(embed_dim), float(norm_eps), float(gated_norm_eps)
        p.norm_w, p.w1, p.gated_norm_w, p.w2 = _ptr(norm_w), _ptr(w1), _ptr(gated_norm_w), _ptr(w2)
        p.w1_q, p.w1_scale, p.w2_q, p.w2_scale = _ptr(w1_q), _ptr(w1_scale), _ptr(w2_q), _ptr(w2_scale)   # optional FP8 forward
        self.params = p

    def ref(self):
        return ctypes.byref(self.params)


def hstu_layer_workspace_bytes(prob: LayerProblem, for_backward: bool) -> int:
    return int(_lib.hstu_layer_workspace_bytes(prob.ref(), 1 if for_backward else 0))


def hstu_layer_fwd(prob: LayerProblem, z, out, u_saved, attn_saved, mean, rstd, workspace, stream=None) -> None:
    st = _lib.hstu_layer_fwd(prob.ref(), _ptr(z), _ptr(out), _ptr(u_saved), _ptr(attn_saved), _ptr(mean), _ptr(rstd),
                             _ptr(workspace), workspace.numel(), _stream(stream))
    if st != HSTU_OK:
        raise HstuError(st, "hstu_layer_fwd")


def hstu_layer_bwd(prob: LayerProblem, z, u_saved, attn_saved, mean, rstd, dout, dz, d_norm_w, d_w1, d_gated_norm_w, d_w2,
                   workspace, stream=None) -> None:
    st = _lib.hstu_layer_bwd(prob.ref(), _ptr(z), _ptr(u_saved), _ptr(attn_saved), _ptr(mean), _ptr(rstd), _ptr(dout),
                             _ptr(dz), _ptr(d_norm_w), _ptr(d_w1), _ptr(d_gated_norm_w), _ptr(d_w2), _ptr(workspace),
                             workspace.numel(), _stream(stream))
    if st != HSTU_OK:
        raise HstuError(st, "hstu_layer_bwd")


def hstu_layer_gemm_tunings() -> int:
    """How many times the layer's GEMMs have timed candidate kernels (and blocked the host) in this process."""
    return int(_lib.hstu_layer_gemm_tunings())


def hstu_lbsl_weight(n: int, sl_len: int) -> float:
    return float(_lib.hstu_lbsl_weight(int(n), int(sl_len)))


def hstu_lbsl_expected_load(n: int, sl_len: int, gamma: float) -> float:
    return float(_lib.hstu_lbsl_expected_load(int(n), int(sl_len), float(gamma)))


class Lbsl:
    """Load-Balanced Stochastic Length over simulated ranks (hstu_lbsl_init / hstu_lbsl_step); host arrays are numpy."""

    def __init__(self, world_size: int, warmup_steps: int, recal_interval: int, sl_len: int, gamma: float):
        self.cfg = HstuLbslConfig(int(world_size), int(warmup_steps), int(recal_interval), int(sl_len), float(gamma))
        self.rank_load = np.zeros(max(int(world_size), 1), dtype=np.float64)
        self.state = HstuLbslState(0, 0.0, self.rank_load.ctypes.data)
        st = _lib.hstu_lbsl_init(ctypes.byref(self.cfg), ctypes.byref(self.state))
        if st != HSTU_OK:
            raise HstuError(st, "hstu_lbsl_init")

    @property
    def target(self) -> float:
        return float(self.state.target)

    @property
    def step_no(self) -> int:
        return int(self.state.step)

    def step(self, rank_offsets, lengths, uniforms):
        """One step for every rank.  Returns (new_lengths int32[total], unsampled uint8[total], realised_load float64[R])."""
        off = np.ascontiguousarray(rank_offsets, dtype=np.int32)
        lens = np.ascontiguousarray(lengths, dtype=np.int32)
        us = np.ascontiguousarray(uniforms, dtype=np.float64)
        if off.shape[0] != self.cfg.world_size + 1 or lens.shape != us.shape or (off.size and int(off[-1]) != lens.shape[0]):
            raise HstuError(-2, "hstu_lbsl_step (array shapes)")
        new = np.empty_like(lens)
        keep = np.empty(lens.shape[0], dtype=np.uint8)
        real = np.empty(self.cfg.world_size, dtype=np.float64)
        st = _lib.hstu_lbsl_step(ctypes.byref(self.cfg), ctypes.byref(self.state), off.ctypes.data, lens.ctypes.data, us.ctypes.data,
                                 new.ctypes.data, keep.ctypes.data, real.ctypes.data)
        if st != HSTU_OK:
            raise HstuError(st, "hstu_lbsl_step")
        return new, keep, real


def hstu_lbsl_fit_gamma(lengths, times) -> float:
    ls = np.ascontiguousarray(lengths, dtype=np.float64)
    ts = np.ascontiguousarray(times, dtype=np.float64)
    out = ctypes.c_double(0.0)
    st = _lib.hstu_lbsl_fit_gamma(int(ls.shape[0]), ls.ctypes.data, ts.ctypes.data, ctypes.byref(out))
    if st != HSTU_OK or ls.shape != ts.shape:
        raise HstuError(st if st != HSTU_OK else -2, "hstu_lbsl_fit_gamma")
    return float(out.value)


def hstu_norm_quant_fp8(a, u, gamma, beta, eps, q, q_scale, mean=None, rstd=None, stream=None) -> None:
    """q (uint8 [T, D]) and q_scale (fp32 [T]) of the (gated) norm of a; gamma None: plain row-wise quantisation."""
    T = a.shape[0]
    D = a.numel() // T if T else int(np.prod(a.shape[1:]))
    st = _lib.hstu_norm_quant_fp8(T, D, _dtype_code(a), _ptr(a), _ptr(u), _ptr(gamma), _ptr(beta), float(eps), _ptr(q),
                                  _ptr(q_scale), _ptr(mean), _ptr(rstd), _stream(stream))
    if st != HSTU_OK:
        raise HstuError(st, "hstu_norm_quant_fp8")


def hstu_fp8_gemm_bias2d(a_q, a_scale, b_q, b_scale, c, d, stream=None) -> None:
    """d [M, N] bf16 = a_scale[m] b_scale[n] (a_q [M, K] b_q [N, K]^T) + c [M, N] (bf16 or None); codes as uint8."""
    M, K = a_q.shape
    N = b_q.shape[0]
    assert b_q.shape[1] == K and tuple(d.shape) == (M, N) and a_q.is_contiguous() and b_q.is_contiguous() and d.is_contiguous()
    assert c is None or (tuple(c.shape) == (M, N) and c.is_contiguous())
    st = _lib.hstu_fp8_gemm_bias2d(M, N, K, _ptr(a_q), _ptr(a_scale), _ptr(b_q), _ptr(b_scale), _ptr(c), _ptr(d),
                                   _stream(stream))
    if st != HSTU_OK:
        raise HstuError(st, "hstu_fp8_gemm_bias2d")


def hstu_profile_enable(on: bool) -> None:
    st = _lib.hstu_profile_enable(1 if on else 0)
    if st != HSTU_OK:
        raise HstuError(st, "hstu_profile_enable")


def hstu_profile_read(max_entries: int = 64):
    """[(kernel name, milliseconds)] for the launches since the last read; waits for them to finish."""
    names = (ctypes.c_char_p * max_entries)()
    ms = (ctypes.c_float * max_entries)()
    n = _lib.hstu_profile_read(max_entries, names, ms)
    if n < 0:
        raise HstuError(n, "hstu_profile_read")
    return [(names[i].decode(), float(ms[i])) for i in range(n)]
