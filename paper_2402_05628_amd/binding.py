"""ctypes binding of librepquant.so: argument marshalling only.

Every function here takes torch tensors that already live on the GPU (PyTorch is used for device
memory and streams, nothing else), fills the matching C descriptor of include/repquant.h and calls
the entry point of the same name.  There is no CPU fallback: if the library is missing the import
fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librepquant.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "librepquant.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
        "(or python paper_2402_05628_amd/_build.py) first; there is no fallback path")

lib = C.CDLL(LIB_PATH)

RQ_OK = 0
NORM_LAYERNORM, NORM_RMSNORM = 0, 1
ACT_NONE, ACT_GELU, ACT_SILU_GATED = 0, 1, 2
MASK_NONE, MASK_CAUSAL = 0, 1
W_I8_BAKED, W_I8_CENTERED, W_U4, B_ACT_I8 = 0, 1, 2, 3
STEP_NAMES = ["ln1", "qkv", "qk", "softmax", "pv", "proj", "ln2", "fc1", "fc2", "aux"]

i32, i64, f32, f64, vp = C.c_int32, C.c_int64, C.c_float, C.c_double, C.c_void_p


class FoldDesc(C.Structure):
    _fields_ = [("D", i32), ("D_out", i32), ("s_ch", vp), ("z_ch", vp), ("gamma", vp), ("beta", vp), ("W", vp),
                ("b", vp), ("s_log", f32), ("s_tilde", vp), ("z_tilde", vp), ("gamma_t", vp), ("beta_t", vp),
                ("W_t", vp), ("b_t", vp), ("s_log_pair", vp)]


class WqDesc(C.Structure):
    _fields_ = [("N", i32), ("K", i32), ("bits", i32), ("format", i32), ("gate_up_rows", i32), ("W", vp),
                ("bias", vp), ("w_out", vp), ("s_w", vp), ("z_w", vp), ("colsum_w", vp), ("bias_out", vp)]


class LnDesc(C.Structure):
    _fields_ = [("T", i64), ("D", i32), ("norm_kind", i32), ("eps", f64), ("x", vp), ("ldx", i64),
                ("gamma_t", vp), ("beta_t", vp), ("s_tilde", f32), ("z_tilde", i32), ("bits", i32),
                ("store_off", i32), ("q", vp), ("ldq", i64), ("rowsum", vp)]


class GemmDesc(C.Structure):
    _fields_ = [("M", i64), ("N", i32), ("K", i32), ("A", vp), ("lda", i64), ("a_off", i32), ("z_a", i32),
                ("s_a", f32), ("B", vp), ("ldb", i64), ("b_format", i32), ("s_b", vp), ("z_b", vp),
                ("colsum_b", vp), ("rowsum_a", vp), ("b_off", i32), ("z_b_scalar", i32), ("bias", vp),
                ("act", i32), ("residual", vp), ("ldr", i64), ("out_acc", vp), ("ldacc", i64),
                ("out_f32", vp), ("ldf", i64), ("out_q", vp), ("ldq", i64), ("bits_o", i32), ("n_seg", i32),
                ("seg_len", i32), ("s_o", f32 * 4), ("z_o", i32 * 4), ("off_o", i32 * 4),
                ("batch_outer", i64), ("batch_inner", i32), ("a_stride_outer", i64), ("a_stride_inner", i64),
                ("b_stride_outer", i64), ("b_stride_inner", i64), ("acc_stride_group", i64), ("causal", i32)]


class SoftmaxDesc(C.Structure):
    _fields_ = [("G", i64), ("H", i32), ("Nq", i32), ("Nk", i32), ("ld", i64), ("acc", vp),
                ("logit_scale", f64), ("bias", vp), ("mask", i32), ("s_log", f32), ("bits", i32), ("codes", vp)]


class PvDesc(C.Structure):
    _fields_ = [("batch", i64), ("H", i32), ("Nq", i32), ("Nk", i32), ("d_head", i32), ("ld", i64), ("codes", vp),
                ("V", vp), ("ldv", i64), ("s_log", f32), ("s_v", f32), ("z_v", i32), ("v_off", i32),
                ("bits_p", i32), ("mask", i32), ("out_f32", vp), ("ldf", i64), ("out_q", vp), ("ldq", i64),
                ("s_o", f32), ("z_o", i32), ("off_o", i32), ("bits_o", i32)]


class QLinear(C.Structure):
    _fields_ = [("N", i32), ("K", i32), ("bits", i32), ("format", i32), ("w", vp), ("s_w", vp), ("z_w", vp),
                ("colsum_w", vp), ("bias", vp)]


class BlockParams(C.Structure):
    _fields_ = [("D", i32), ("H", i32), ("Dm", i32), ("norm_kind", i32), ("act", i32), ("mask", i32),
                ("bits_a", i32), ("bits_p", i32), ("eps", f64),
                ("ln1_gamma_t", vp), ("ln1_beta_t", vp), ("ln1_s", f32), ("ln1_z", i32),
                ("qkv", QLinear),
                ("s_q", f32), ("s_k", f32), ("s_v", f32), ("z_q", i32), ("z_k", i32), ("z_v", i32),
                ("rel_bias", vp), ("s_log", f32), ("s_o", f32), ("z_o", i32),
                ("proj", QLinear),
                ("ln2_gamma_t", vp), ("ln2_beta_t", vp), ("ln2_s", f32), ("ln2_z", i32),
                ("fc1", QLinear), ("s_h", f32), ("z_h", i32), ("fc2", QLinear)]


class BlockRaw(C.Structure):
    _fields_ = [("D", i32), ("H", i32), ("Dm", i32), ("norm_kind", i32), ("act", i32), ("mask", i32),
                ("bits_w", i32), ("bits_a", i32), ("bits_p", i32), ("eps", f64),
                ("ln1_gamma", vp), ("ln1_beta", vp), ("ln2_gamma", vp), ("ln2_beta", vp),
                ("w_qkv", vp), ("b_qkv", vp), ("w_proj", vp), ("b_proj", vp), ("w_fc1", vp), ("b_fc1", vp),
                ("w_fc2", vp), ("b_fc2", vp),
                ("ln1_clip_up", vp), ("ln1_clip_lo", vp), ("ln2_clip_up", vp), ("ln2_clip_lo", vp),
                ("rel_bias", vp), ("s_log", f32)]


def _sig(name, restype, argtypes):
    fn = getattr(lib, name)
    fn.restype = restype
    fn.argtypes = argtypes
    return fn


_rq_create = _sig("rq_create", i32, [C.POINTER(vp), C.c_int, vp])
_rq_destroy = _sig("rq_destroy", None, [vp])
_rq_last_error = _sig("rq_last_error", C.c_char_p, [vp])
_rq_store_offset = _sig("rq_store_offset", i32, [i32, i32])
_rq_ln_quant = _sig("rq_ln_quant", i32, [vp, C.POINTER(LnDesc)])


class RqError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__("rq status %d: %s" % (status, msg))
        self.status = status


def _p(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def store_offset(bits: int, z: int) -> int:
    return int(_rq_store_offset(bits, z))


class Context:
    """rq_ctx bound to a torch device and stream (device=None: host-only validation context)."""

    def __init__(self, device: Optional[int] = 0, stream: Optional[torch.cuda.Stream] = None):
        self._h = vp()
        if device is None:
            dev, st = -1, None
        else:
            dev = int(device)
            st = (stream or torch.cuda.current_stream(dev)).cuda_stream
        rc = _rq_create(C.byref(self._h), dev, st)
        if rc != RQ_OK:
            raise RqError(rc, _rq_last_error(None).decode())

    def close(self):
        if self._h:
            _rq_destroy(self._h)
            self._h = vp()

    def __del__(self):  # pragma: no cover
        try:
            self.close()
        except Exception:
            pass

    def check(self, rc: int):
        if rc != RQ_OK:
            raise RqError(rc, _rq_last_error(self._h).decode())

    @property
    def handle(self):
        return self._h


def rq_ln_quant(ctx: Context, x: torch.Tensor, gamma_t: torch.Tensor, beta_t: Optional[torch.Tensor], s_tilde: float,
                z_tilde: int, bits: int, q: torch.Tensor, norm_kind: int = NORM_LAYERNORM, eps: float = 1e-6,
                store_off: Optional[int] = None, rowsum: Optional[torch.Tensor] = None) -> int:
    """Fills rq_ln_desc and calls rq_ln_quant; returns the storage offset used."""
    off = store_offset(bits, z_tilde) if store_off is None else store_off
    d = LnDesc(T=x.shape[0], D=x.shape[1], norm_kind=norm_kind, eps=eps, x=_p(x), ldx=x.stride(0),
               gamma_t=_p(gamma_t), beta_t=_p(beta_t), s_tilde=s_tilde, z_tilde=z_tilde, bits=bits, store_off=off,
               q=_p(q), ldq=q.stride(0), rowsum=_p(rowsum))
    ctx.check(_rq_ln_quant(ctx.handle, C.byref(d)))
    return off
