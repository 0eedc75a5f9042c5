"""Thin ctypes binding of liblq.so: argument marshalling only, same names as include/lq.h.

PyTorch is used for device memory and the current stream, nothing else: every step of the
path runs in the library's kernels.  Importing this module fails loudly when the HIP library
has not been built (``python paper_2604_18117_amd/build.py``); there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liblq.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(f"{_LIB_PATH} is missing: build it with `python paper_2604_18117_amd/build.py`")
_lib = C.CDLL(_LIB_PATH)

LQ_OK = 0
LQ_ERR_NULL, LQ_ERR_SHAPE, LQ_ERR_UNSUPPORTED, LQ_ERR_ALIGN, LQ_ERR_BUFFER_TOO_SMALL, LQ_ERR_DEVICE, LQ_ERR_STALE_BLOB = range(1, 8)
LQ_BLOB_PACKED, LQ_BLOB_ACT = 1, 2
LQ_INT4, LQ_INT6, LQ_INT8, LQ_MXFP4_E2M1, LQ_FP8_E4M3, LQ_MXFP8_E4M3, LQ_MXINT4, LQ_MXINT8, LQ_MXFP6_E2M3 = range(9)
LQ_F32, LQ_BF16 = 0, 1
LQ_FLAG_SMOOTH = 1
_INT_FMT = {4: LQ_INT4, 6: LQ_INT6, 8: LQ_INT8}


class lq_config(C.Structure):
    _fields_ = [("N", C.c_int64), ("K", C.c_int64), ("rank", C.c_int32), ("main_w", C.c_int32),
                ("main_a", C.c_int32), ("main_w_group", C.c_int32), ("main_a_group", C.c_int32),
                ("br_w", C.c_int32), ("br_a", C.c_int32), ("residual_from_quantized", C.c_int32),
                ("x_dtype", C.c_int32), ("flags", C.c_int32)]


class lq_act_debug(C.Structure):
    _fields_ = [("xb", C.c_void_p), ("sxb", C.c_void_p), ("accT", C.c_void_p), ("T", C.c_void_p),
                ("xbe", C.c_void_p)]


class lq_fwd_debug(C.Structure):
    _fields_ = [("acc", C.c_void_p), ("acc2", C.c_void_p), ("y32", C.c_void_p)]


class lq_weights_view(C.Structure):
    _fields_ = [("pq", C.c_void_p), ("sw", C.c_void_p), ("pe", C.c_void_p), ("lq", C.c_void_p),
                ("sl", C.c_void_p), ("rq", C.c_void_p), ("sr", C.c_void_p), ("le", C.c_void_p), ("re", C.c_void_p)]


class lq_act_view(C.Structure):
    _fields_ = [("xq", C.c_void_p), ("sx", C.c_void_p), ("xe", C.c_void_p), ("tq", C.c_void_p),
                ("st", C.c_void_p), ("te", C.c_void_p)]


class lq_adam(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float)]


class lq_calib_view(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("L", "R", "mL", "vL", "mR", "vR", "gL", "gR", "E")]


class lq_cayley(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta", C.c_float), ("eps", C.c_float), ("q", C.c_float), ("s", C.c_int32),
                ("grad_scale", C.c_float)]


class lq_rot_view(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("Omega", "Mom", "G", "E1", "E2")]


EXPORTS = ["lq_status_string", "lq_packed_sizes", "lq_pack_weights", "lq_verify_blob", "lq_set_smoothing", "lq_act_sizes", "lq_quantize_act",
           "lq_linear_lowrank_fwd", "lq_handoff_sizes", "lq_linear_lowrank_fwd_handoff", "lq_branch_from_codes",
           "lq_unpack_weights", "lq_unpack_act", "lq_calib_sizes", "lq_calib_init", "lq_calib_step",
           "lq_calib_unpack", "lq_rot_sizes", "lq_rot_init", "lq_rot_step", "lq_rot_step_static", "lq_rot_apply", "lq_rot_unpack"]

_lib.lq_calib_sizes.argtypes = [C.POINTER(lq_config), C.POINTER(C.c_size_t)]
_lib.lq_calib_init.argtypes = [C.POINTER(lq_config), C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
_lib.lq_calib_step.argtypes = [C.POINTER(lq_config), C.c_void_p, C.c_void_p, C.c_size_t, C.c_int32, C.POINTER(lq_adam),
                               C.c_void_p, C.c_void_p]
_lib.lq_calib_unpack.argtypes = [C.POINTER(lq_config), C.c_void_p, C.POINTER(lq_calib_view), C.c_void_p]
_lib.lq_rot_sizes.argtypes = [C.POINTER(lq_config), C.POINTER(C.c_size_t)]
_lib.lq_rot_init.argtypes = [C.POINTER(lq_config), C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
_lib.lq_rot_step.argtypes = [C.POINTER(lq_config), C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.POINTER(lq_cayley),
                             C.c_void_p, C.c_void_p]
_lib.lq_rot_step_static.argtypes = _lib.lq_rot_step.argtypes
_lib.lq_rot_apply.argtypes = [C.POINTER(lq_config), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
_lib.lq_rot_unpack.argtypes = [C.POINTER(lq_config), C.c_void_p, C.POINTER(lq_rot_view), C.c_void_p]
_lib.lq_status_string.restype = C.c_char_p
_lib.lq_status_string.argtypes = [C.c_int]
_lib.lq_packed_sizes.argtypes = [C.POINTER(lq_config), C.POINTER(C.c_size_t)]
_lib.lq_act_sizes.argtypes = [C.POINTER(lq_config), C.c_int64, C.POINTER(C.c_size_t)]
_lib.lq_pack_weights.argtypes = [C.POINTER(lq_config), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                 C.c_size_t, C.c_void_p]
_lib.lq_verify_blob.argtypes = [C.POINTER(lq_config), C.c_int32, C.c_void_p, C.c_size_t, C.c_int64, C.c_void_p]
_lib.lq_set_smoothing.argtypes = [C.POINTER(lq_config), C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
_lib.lq_quantize_act.argtypes = [C.POINTER(lq_config), C.c_void_p, C.c_size_t, C.c_void_p, C.c_int64, C.c_int64,
                                 C.c_void_p, C.c_size_t, C.POINTER(lq_act_debug), C.c_void_p]
_lib.lq_linear_lowrank_fwd.argtypes = [C.POINTER(lq_config), C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_int64,
                                       C.c_void_p, C.c_int64, C.POINTER(lq_fwd_debug), C.c_void_p]
_lib.lq_handoff_sizes.argtypes = [C.POINTER(lq_config), C.c_int64, C.POINTER(C.c_size_t)]
_lib.lq_linear_lowrank_fwd_handoff.argtypes = [C.POINTER(lq_config), C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_int64,
                                               C.c_void_p, C.c_int64, C.POINTER(lq_config), C.c_void_p, C.c_size_t, C.c_void_p,
                                               C.c_size_t, C.c_void_p]
_lib.lq_branch_from_codes.argtypes = [C.POINTER(lq_config), C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_int64,
                                      C.c_void_p, C.c_size_t, C.c_void_p]
_lib.lq_unpack_weights.argtypes = [C.POINTER(lq_config), C.c_void_p, C.POINTER(lq_weights_view), C.c_void_p]
_lib.lq_unpack_act.argtypes = [C.POINTER(lq_config), C.c_void_p, C.c_int64, C.POINTER(lq_act_view), C.c_void_p]


class LqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lq_status_string(status)} (status {status})")


def lq_status_string(status: int) -> str:
    return _lib.lq_status_string(int(status)).decode()


def _check(st: int, where: str):
    if st != LQ_OK:
        raise LqError(st, where)


def raw():
    """The ctypes library handle (for tests of the error paths, which need no GPU)."""
    return _lib


def make_config(N: int, K: int, rank: int, family: str = "int", group: int = 64, br_w_bits: int = 8,
                br_a_bits: int = 8, x_dtype: str = "bf16", residual_from_quantized: bool = True,
                smooth: bool = False, a_group: int = 0) -> lq_config:
    """a_group (INT family): 0 = one main activation scale per token; 64 = SINT4 blocks (FP16 scale per 64
    values along K) for both operands of the main product."""
    if family == "int":
        return lq_config(N, K, rank, LQ_INT4, LQ_INT4, group, a_group, _INT_FMT[br_w_bits], _INT_FMT[br_a_bits],
                         1 if residual_from_quantized else 0, LQ_BF16 if x_dtype == "bf16" else LQ_F32,
                         LQ_FLAG_SMOOTH if smooth else 0)
    fl = LQ_FLAG_SMOOTH if smooth else 0
    if family in ("mx", "mxb"):  # "mxb": block-scaled branch (MXFP8e4, or MXFP6e2 at 6 bits) instead of fp32-scaled E4M3
        br = (LQ_MXFP6_E2M3 if br_w_bits == 6 else LQ_MXFP8_E4M3) if family == "mxb" else LQ_FP8_E4M3
        return lq_config(N, K, rank, LQ_MXFP4_E2M1, LQ_MXFP4_E2M1, 32, 32, br, br,
                         1 if residual_from_quantized else 0, LQ_BF16 if x_dtype == "bf16" else LQ_F32, fl)
    if family == "mxi":          # MXINT4 main; MXINT8 branch activations; MXINT8 or MXINT4 branch weights
        return lq_config(N, K, rank, LQ_MXINT4, LQ_MXINT4, 32, 32, LQ_MXINT8 if br_w_bits == 8 else LQ_MXINT4, LQ_MXINT8,
                         1 if residual_from_quantized else 0, LQ_BF16 if x_dtype == "bf16" else LQ_F32, fl)
    raise ValueError(family)


def config_for_layer(layer, smooth: bool = False) -> lq_config:
    return make_config(layer.N, layer.K, layer.r, layer.family, layer.g, layer.br_w_bits, layer.br_a_bits,
                       layer.x_dtype, smooth=smooth, a_group=layer.a_group)


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def lq_packed_sizes(cfg: lq_config) -> int:
    n = C.c_size_t(0)
    _check(_lib.lq_packed_sizes(C.byref(cfg), C.byref(n)), "lq_packed_sizes")
    return int(n.value)


def lq_set_smoothing(cfg: lq_config, packed: torch.Tensor, gamma: torch.Tensor) -> None:
    """gamma: K fp32 CUDA values > 0; stores their reciprocals in the blob (layer packed with smooth=True)."""
    assert gamma.is_cuda and gamma.dtype == torch.float32 and gamma.is_contiguous() and gamma.numel() == cfg.K
    _check(_lib.lq_set_smoothing(C.byref(cfg), _ptr(gamma), _ptr(packed), packed.numel(), C.c_void_p(_stream())),
           "lq_set_smoothing")


def lq_verify_blob(cfg: lq_config, kind: int, blob: torch.Tensor, M: int = 0) -> None:
    """Raises LqError(LQ_ERR_STALE_BLOB) when the blob's header does not belong to cfg (and M).  Synchronises the stream."""
    _check(_lib.lq_verify_blob(C.byref(cfg), kind, _ptr(blob), blob.numel(), M, C.c_void_p(_stream())), "lq_verify_blob")


def lq_act_sizes(cfg: lq_config, M: int) -> int:
    n = C.c_size_t(0)
    _check(_lib.lq_act_sizes(C.byref(cfg), M, C.byref(n)), "lq_act_sizes")
    return int(n.value)


def lq_pack_weights(cfg: lq_config, W: torch.Tensor, L: Optional[torch.Tensor], R: Optional[torch.Tensor],
                    packed: Optional[torch.Tensor] = None) -> torch.Tensor:
    """W (N x K), L (N x r), R (r x K): fp32 CUDA tensors, contiguous.  Returns the packed blob."""
    assert W.is_cuda and W.dtype == torch.float32 and W.is_contiguous() and tuple(W.shape) == (cfg.N, cfg.K)
    for t in (L, R):
        assert t is None or (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous())
    if cfg.rank:  # the library reads N x r and r x K values: the tensors must hold them
        assert tuple(L.shape) == (cfg.N, cfg.rank) and tuple(R.shape) == (cfg.rank, cfg.K), "factor shapes must match cfg"
    if packed is None:
        packed = torch.empty(lq_packed_sizes(cfg), dtype=torch.uint8, device=W.device)
    _check(_lib.lq_pack_weights(C.byref(cfg), _ptr(W), _ptr(L), _ptr(R), _ptr(packed), packed.numel(),
                                C.c_void_p(_stream())), "lq_pack_weights")
    return packed


@dataclass
class ActDebug:
    xb: torch.Tensor
    sxb: torch.Tensor
    accT: torch.Tensor
    T: torch.Tensor
    xbe: Optional[torch.Tensor] = None


def lq_quantize_act(cfg: lq_config, packed: torch.Tensor, X: torch.Tensor, act: Optional[torch.Tensor] = None,
                    debug: bool = False):
    """X: M x K CUDA tensor (fp32 or bf16, row stride may exceed K).  Returns the activation blob
    (and the parity taps when debug=True)."""
    assert X.is_cuda and X.dim() == 2 and X.stride(1) == 1 and X.shape[1] == cfg.K
    assert X.dtype == (torch.bfloat16 if cfg.x_dtype == LQ_BF16 else torch.float32)
    assert packed is None or packed.numel() >= lq_packed_sizes(cfg)
    M = X.shape[0]
    if act is None:
        act = torch.empty(lq_act_sizes(cfg, M), dtype=torch.uint8, device=X.device)
    dbg = None
    taps = None
    if debug:
        r = max(cfg.rank, 1)
        taps = ActDebug(torch.zeros((M, cfg.K), dtype=torch.int8, device=X.device),
                        torch.zeros(M, dtype=torch.float32, device=X.device),
                        torch.zeros((M, r), dtype=torch.int32, device=X.device),
                        torch.zeros((M, r), dtype=torch.float32, device=X.device),
                        torch.zeros((M, cfg.K // 32), dtype=torch.uint8, device=X.device))
        dbg = lq_act_debug(taps.xb.data_ptr(), taps.sxb.data_ptr(), taps.accT.data_ptr(), taps.T.data_ptr(),
                           taps.xbe.data_ptr())
    _check(_lib.lq_quantize_act(C.byref(cfg), _ptr(packed), 0 if packed is None else packed.numel(), _ptr(X), M, X.stride(0),
                                _ptr(act), act.numel(),
                                C.byref(dbg) if dbg is not None else None, C.c_void_p(_stream())),
           "lq_quantize_act")
    return (act, taps) if debug else act


@dataclass
class FwdDebug:
    acc: Optional[torch.Tensor]
    acc2: torch.Tensor
    y32: torch.Tensor


def lq_linear_lowrank_fwd(cfg: lq_config, packed: torch.Tensor, act: torch.Tensor, M: int,
                          Y: Optional[torch.Tensor] = None, debug: bool = False, debug_acc: bool = True):
    """Returns Y (M x N bf16); with debug=True also the taps (acc only if debug_acc)."""
    if Y is None:
        Y = torch.empty((M, cfg.N), dtype=torch.bfloat16, device=act.device)
    assert Y.is_cuda and Y.dtype == torch.bfloat16 and Y.stride(1) == 1 and Y.shape == (M, cfg.N)
    dbg = None
    taps = None
    if debug:
        G = cfg.K // cfg.main_w_group
        taps = FwdDebug(torch.zeros((M, cfg.N, G), dtype=torch.int32, device=act.device) if debug_acc else None,
                        torch.zeros((M, cfg.N), dtype=torch.int32, device=act.device),
                        torch.zeros((M, cfg.N), dtype=torch.float32, device=act.device))
        dbg = lq_fwd_debug(taps.acc.data_ptr() if debug_acc else None, taps.acc2.data_ptr(), taps.y32.data_ptr())
    _check(_lib.lq_linear_lowrank_fwd(C.byref(cfg), _ptr(packed), packed.numel(), _ptr(act), act.numel(), M, _ptr(Y), Y.stride(0),
                                      C.byref(dbg) if dbg is not None else None, C.c_void_p(_stream())),
           "lq_linear_lowrank_fwd")
    return (Y, taps) if debug else Y


def lq_handoff_sizes(next_cfg: lq_config, M: int) -> int:
    n = C.c_size_t(0)
    _check(_lib.lq_handoff_sizes(C.byref(next_cfg), M, C.byref(n)), "lq_handoff_sizes")
    return int(n.value)


def lq_linear_lowrank_fwd_handoff(cfg: lq_config, packed: torch.Tensor, act: torch.Tensor, M: int, next_cfg: lq_config,
                                  act_next: Optional[torch.Tensor] = None, codes: Optional[torch.Tensor] = None,
                                  Y: Optional[torch.Tensor] = None):
    """The forward plus the quantized hand-off to a next layer (K = this N).  Returns (act_next, codes); Y (M x N bf16)
    is written only when given."""
    if act_next is None:
        act_next = torch.empty(lq_act_sizes(next_cfg, M), dtype=torch.uint8, device=act.device)
    if codes is None:
        codes = torch.empty(lq_handoff_sizes(next_cfg, M), dtype=torch.uint8, device=act.device)
    if Y is not None:
        assert Y.is_cuda and Y.dtype == torch.bfloat16 and Y.stride(1) == 1 and Y.shape == (M, cfg.N)
    _check(_lib.lq_linear_lowrank_fwd_handoff(C.byref(cfg), _ptr(packed), packed.numel(), _ptr(act), act.numel(), M, _ptr(Y),
                                              Y.stride(0) if Y is not None else 0,
                                              C.byref(next_cfg), _ptr(act_next), act_next.numel(), _ptr(codes), codes.numel(),
                                              C.c_void_p(_stream())), "lq_linear_lowrank_fwd_handoff")
    return act_next, codes


def lq_branch_from_codes(next_cfg: lq_config, packed_next: torch.Tensor, codes: torch.Tensor, M: int,
                         act_next: torch.Tensor) -> torch.Tensor:
    """Completes act_next (the consumer's intermediate codes and scales) from the hand-off codes."""
    _check(_lib.lq_branch_from_codes(C.byref(next_cfg), _ptr(packed_next), 0 if packed_next is None else packed_next.numel(),
                                     _ptr(codes), codes.numel(), M, _ptr(act_next),
                                     act_next.numel(), C.c_void_p(_stream())), "lq_branch_from_codes")
    return act_next


@dataclass
class WeightsView:
    pq: torch.Tensor
    sw: Optional[torch.Tensor]
    pe: Optional[torch.Tensor]
    lq: torch.Tensor
    sl: torch.Tensor
    rq: torch.Tensor
    sr: torch.Tensor
    le: Optional[torch.Tensor] = None
    re: Optional[torch.Tensor] = None


def lq_unpack_weights(cfg: lq_config, packed: torch.Tensor) -> WeightsView:
    dev = packed.device
    N, K, r = cfg.N, cfg.K, cfg.rank
    mx = cfg.main_w in (LQ_MXFP4_E2M1, LQ_MXINT4)
    v = WeightsView(torch.zeros((N, K), dtype=torch.int8, device=dev),
                    None if mx else torch.zeros((N, K // cfg.main_w_group), dtype=torch.float32, device=dev),
                    torch.zeros((N, K // 32), dtype=torch.uint8, device=dev) if mx else None,
                    torch.zeros((N, max(r, 1)), dtype=torch.int8, device=dev),
                    torch.zeros(N, dtype=torch.float32, device=dev),
                    torch.zeros((max(r, 1), K), dtype=torch.int8, device=dev),
                    torch.zeros(max(r, 1), dtype=torch.float32, device=dev),
                    torch.zeros((N, max(r // 32, 1)), dtype=torch.uint8, device=dev),
                    torch.zeros((max(r, 1), K // 32), dtype=torch.uint8, device=dev))
    view = lq_weights_view(v.pq.data_ptr(), v.sw.data_ptr() if v.sw is not None else None,
                           v.pe.data_ptr() if v.pe is not None else None, v.lq.data_ptr(), v.sl.data_ptr(),
                           v.rq.data_ptr(), v.sr.data_ptr(), v.le.data_ptr(), v.re.data_ptr())
    _check(_lib.lq_unpack_weights(C.byref(cfg), _ptr(packed), C.byref(view), C.c_void_p(_stream())),
           "lq_unpack_weights")
    return v


@dataclass
class ActView:
    xq: torch.Tensor
    sx: Optional[torch.Tensor]
    xe: Optional[torch.Tensor]
    tq: torch.Tensor
    st: torch.Tensor
    te: Optional[torch.Tensor] = None


def lq_unpack_act(cfg: lq_config, act: torch.Tensor, M: int) -> ActView:
    dev = act.device
    K, r = cfg.K, cfg.rank
    mx = cfg.main_w in (LQ_MXFP4_E2M1, LQ_MXINT4)
    v = ActView(torch.zeros((M, K), dtype=torch.int8, device=dev),
                None if mx else torch.zeros((M, K // 64) if cfg.main_a_group == 64 else M, dtype=torch.float32, device=dev),
                torch.zeros((M, K // 32), dtype=torch.uint8, device=dev) if mx else None,
                torch.zeros((M, max(r, 1)), dtype=torch.int8, device=dev),
                torch.zeros(M, dtype=torch.float32, device=dev),
                torch.zeros((M, max(r // 32, 1)), dtype=torch.uint8, device=dev))
    view = lq_act_view(v.xq.data_ptr(), v.sx.data_ptr() if v.sx is not None else None,
                       v.xe.data_ptr() if v.xe is not None else None, v.tq.data_ptr(), v.st.data_ptr(),
                       v.te.data_ptr())
    _check(_lib.lq_unpack_act(C.byref(cfg), _ptr(act), M, C.byref(view), C.c_void_p(_stream())), "lq_unpack_act")
    return v


# ---- data-free calibration of the factors (argument marshalling only) -------------------------------------------------

def lq_calib_sizes(cfg: lq_config) -> int:
    n = C.c_size_t(0)
    _check(_lib.lq_calib_sizes(C.byref(cfg), C.byref(n)), "lq_calib_sizes")
    return int(n.value)


def lq_calib_init(cfg: lq_config, L: torch.Tensor, R: torch.Tensor, state: Optional[torch.Tensor] = None) -> torch.Tensor:
    """L (N x r), R (r x K): fp32 CUDA, contiguous (paper's sign: Q1(W + L R) - W ~ L R).  Returns the state blob."""
    for t in (L, R):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
    assert tuple(L.shape) == (cfg.N, cfg.rank) and tuple(R.shape) == (cfg.rank, cfg.K), "factor shapes must match cfg"
    if state is None:
        state = torch.empty(lq_calib_sizes(cfg), dtype=torch.uint8, device=L.device)
    _check(_lib.lq_calib_init(C.byref(cfg), _ptr(L), _ptr(R), _ptr(state), state.numel(), C.c_void_p(_stream())),
           "lq_calib_init")
    return state


def lq_calib_step(cfg: lq_config, W: torch.Tensor, state: torch.Tensor, step: int, lr: float = 1e-4, beta1: float = 0.9,
                  beta2: float = 0.999, eps: float = 1e-8, loss: Optional[torch.Tensor] = None) -> None:
    """One Adam step (step counts from 1); `loss`: optional 1-element fp32 CUDA tensor that receives the loss before the update."""
    assert W.is_cuda and W.dtype == torch.float32 and W.is_contiguous() and tuple(W.shape) == (cfg.N, cfg.K)
    ad = lq_adam(lr, beta1, beta2, eps)
    _check(_lib.lq_calib_step(C.byref(cfg), _ptr(W), _ptr(state), state.numel(), step, C.byref(ad), _ptr(loss),
                              C.c_void_p(_stream())), "lq_calib_step")


def lq_calib_unpack(cfg: lq_config, state: torch.Tensor, names=("L", "R")) -> dict:
    """Copies of the named parts of the state: L, R, mL, vL, mR, vR, gL, gR, E."""
    N, K, r = cfg.N, cfg.K, cfg.rank
    shapes = {"L": (N, r), "R": (r, K), "mL": (N, r), "vL": (N, r), "mR": (r, K), "vR": (r, K), "gL": (N, r), "gR": (r, K),
              "E": (N, K)}
    out = {k: torch.empty(shapes[k], dtype=torch.float32, device=state.device) for k in names}
    view = lq_calib_view(**{k: (out[k].data_ptr() if k in out else None) for k in shapes})
    _check(_lib.lq_calib_unpack(C.byref(cfg), _ptr(state), C.byref(view), C.c_void_p(_stream())), "lq_calib_unpack")
    return out


# ---- rotation of the calibrated factors (argument marshalling only) ---------------------------------------------------

def lq_rot_sizes(cfg: lq_config) -> int:
    n = C.c_size_t(0)
    _check(_lib.lq_rot_sizes(C.byref(cfg), C.byref(n)), "lq_rot_sizes")
    return int(n.value)


def _check_factors(cfg: lq_config, L: torch.Tensor, R: torch.Tensor) -> None:
    for t in (L, R):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
    assert tuple(L.shape) == (cfg.N, cfg.rank) and tuple(R.shape) == (cfg.rank, cfg.K), "factor shapes must match cfg"


def lq_rot_init(cfg: lq_config, Omega0: Optional[torch.Tensor] = None, Mom0: Optional[torch.Tensor] = None,
                state: Optional[torch.Tensor] = None, device="cuda") -> torch.Tensor:
    """Omega0, Mom0: r x r fp32 CUDA, contiguous, or None for the identity / zero.  Returns the state blob."""
    for t in (Omega0, Mom0):
        assert t is None or (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and tuple(t.shape) == (cfg.rank, cfg.rank))
    if state is None:
        state = torch.empty(lq_rot_sizes(cfg), dtype=torch.uint8, device=device)
    _check(_lib.lq_rot_init(C.byref(cfg), _ptr(Omega0), _ptr(Mom0), _ptr(state), state.numel(), C.c_void_p(_stream())),
           "lq_rot_init")
    return state


def lq_rot_step(cfg: lq_config, L: torch.Tensor, R: torch.Tensor, state: torch.Tensor, lr: float = 0.5, beta: float = 0.9,
                eps: float = 1e-8, q: float = 0.5, s: int = 2, grad_scale: float = 1.0,
                loss: Optional[torch.Tensor] = None) -> None:
    """One Cayley-SGD step on Omega; `loss`: optional 1-element fp32 CUDA tensor that receives the loss before the update."""
    _check_factors(cfg, L, R)
    opt = lq_cayley(lr, beta, eps, q, s, grad_scale)
    _check(_lib.lq_rot_step(C.byref(cfg), _ptr(L), _ptr(R), _ptr(state), state.numel(), C.byref(opt), _ptr(loss),
                            C.c_void_p(_stream())), "lq_rot_step")


def lq_rot_step_static(cfg: lq_config, L: torch.Tensor, R: torch.Tensor, state: torch.Tensor, lr: float = 0.5,
                       beta: float = 0.9, eps: float = 1e-8, q: float = 0.5, s: int = 2, grad_scale: float = 1.0,
                       loss: Optional[torch.Tensor] = None) -> None:
    """lq_rot_step with the step's partial results in the library's per-GPU array (allocates nothing, sizes nothing)."""
    _check_factors(cfg, L, R)
    opt = lq_cayley(lr, beta, eps, q, s, grad_scale)
    _check(_lib.lq_rot_step_static(C.byref(cfg), _ptr(L), _ptr(R), _ptr(state), state.numel(), C.byref(opt), _ptr(loss),
                                   C.c_void_p(_stream())), "lq_rot_step_static")


def lq_rot_apply(cfg: lq_config, L: torch.Tensor, R: torch.Tensor, state: torch.Tensor):
    """(L Omega, Omega^T R) as new fp32 tensors, for lq_pack_weights."""
    _check_factors(cfg, L, R)
    Lr, Rr = torch.empty_like(L), torch.empty_like(R)
    _check(_lib.lq_rot_apply(C.byref(cfg), _ptr(L), _ptr(R), _ptr(state), _ptr(Lr), _ptr(Rr), C.c_void_p(_stream())),
           "lq_rot_apply")
    return Lr, Rr


def lq_rot_unpack(cfg: lq_config, state: torch.Tensor, names=("Omega",)) -> dict:
    """Copies of the named parts of the state: Omega, Mom, G, E1, E2."""
    N, K, r = cfg.N, cfg.K, cfg.rank
    shapes = {"Omega": (r, r), "Mom": (r, r), "G": (r, r), "E1": (N, r), "E2": (r, K)}
    out = {k: torch.empty(shapes[k], dtype=torch.float32, device=state.device) for k in names}
    view = lq_rot_view(**{k: (out[k].data_ptr() if k in out else None) for k in shapes})
    _check(_lib.lq_rot_unpack(C.byref(cfg), _ptr(state), C.byref(view), C.c_void_p(_stream())), "lq_rot_unpack")
    return out
