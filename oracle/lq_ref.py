"""ctypes front-end of the CPU oracle (TEST INFRASTRUCTURE, not part of the product).

Only tests, the smoke check and the bench's cpu_baseline leg may import this module.
It loads ``liblq_oracle.so`` (built from ``lq_oracle.c`` by ``oracle/build.py``) and hands
numpy arrays to it.  It never touches the HIP library or its Python binding.

Orientation (paper Fig. 1, Eq. 5): X is M x K, W is N x K, L is N x r, R is r x K, Y is M x N.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# (LQ_ORACLE_LIB: another build of the same source, e.g. the sanitizer-instrumented one the test suite runs the pins on)
_LIB_PATH = os.environ.get("LQ_ORACLE_LIB") or os.path.join(_HERE, "liblq_oracle.so")
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError("oracle library missing: run `python oracle/build.py`")
        _lib = C.CDLL(_LIB_PATH)
        _lib.lqo_e2m1_decode.restype = C.c_float
        _lib.lqo_e2m1_decode.argtypes = [C.c_uint8]
        _lib.lqo_e4m3_decode.restype = C.c_float
        _lib.lqo_e4m3_decode.argtypes = [C.c_uint8]
        _lib.lqo_e8m0_decode.restype = C.c_double
        _lib.lqo_e8m0_decode.argtypes = [C.c_uint8]
        _lib.lqo_e2m3_decode.restype = C.c_float
        _lib.lqo_e2m3_decode.argtypes = [C.c_uint8]
        _lib.lqo_e2m3_encode.restype = C.c_uint8
        _lib.lqo_e2m3_encode.argtypes = [C.c_float]
        _lib.lqo_e2m1_encode.restype = C.c_uint8
        _lib.lqo_e2m1_encode.argtypes = [C.c_float]
        _lib.lqo_e4m3_encode.restype = C.c_uint8
        _lib.lqo_e4m3_encode.argtypes = [C.c_float]
        _lib.lqo_bf16_rne.restype = C.c_uint16
        _lib.lqo_bf16_rne.argtypes = [C.c_float]
        _lib.lqo_num_threads.restype = C.c_int
        _lib.lqo_f16_round.restype = C.c_float
        _lib.lqo_f16_round.argtypes = [C.c_float]
    return _lib


def _p(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


QMAX = {4: 7, 6: 31, 8: 127}


def num_threads() -> int:
    return int(lib().lqo_num_threads())


# ---------------------------------------------------------------------------------------
# element-level entry points (used by the pins)
# ---------------------------------------------------------------------------------------

def quant_int(v, qmax: int):
    """One vector, one scale: (codes int8, scale float32)."""
    v = _f32(v).ravel()
    q = np.empty(v.size, np.int8)
    s = np.empty(1, np.float32)
    lib().lqo_quant_int(_p(v), C.c_int64(v.size), C.c_int(qmax), _p(q), _p(s))
    return q, s[0]


def f16_round(f: float) -> float:
    return float(lib().lqo_f16_round(C.c_float(f)))


def quant_sint4(v):
    """SINT4 blocks: n values (n % 64 == 0) -> (codes int8 [n], FP16-valued scales float32 [n/64])."""
    v = _f32(v).ravel()
    assert v.size % 64 == 0
    q = np.empty(v.size, np.int8)
    s = np.empty(v.size // 64, np.float32)
    lib().lqo_quant_sint4(_p(v), C.c_int64(v.size), _p(q), _p(s))
    return q, s


def smooth(X, gamma):
    """Activation smoothing: X[m, k] * fl(1 / gamma[k]) in fp32 (the input every other entry point then sees)."""
    X = _f32(X)
    g = _f32(gamma).ravel()
    assert g.size == X.shape[1] and np.all(g > 0)
    out = np.empty_like(X)
    lib().lqo_smooth(C.c_int64(X.shape[0]), C.c_int64(X.shape[1]), _p(X), _p(g), _p(out))
    return out


def quant_mxfp4(v):
    """One row of K values (K % 32 == 0): (E2M1 codes uint8 [K], E8M0 bytes uint8 [K/32])."""
    v = _f32(v).ravel()
    assert v.size % 32 == 0
    c = np.empty(v.size, np.uint8)
    e = np.empty(v.size // 32, np.uint8)
    lib().lqo_quant_mxfp4(_p(v), C.c_int64(v.size), _p(c), _p(e))
    return c, e


def quant_fp8(v):
    v = _f32(v).ravel()
    c = np.empty(v.size, np.uint8)
    s = np.empty(1, np.float32)
    lib().lqo_quant_fp8(_p(v), C.c_int64(v.size), _p(c), _p(s))
    return c, s[0]


def e2m1_decode(codes):
    return np.array([lib().lqo_e2m1_decode(int(c)) for c in np.asarray(codes).ravel()],
                    np.float32).reshape(np.shape(codes))


def e4m3_decode(codes):
    return np.array([lib().lqo_e4m3_decode(int(c)) for c in np.asarray(codes).ravel()],
                    np.float32).reshape(np.shape(codes))


def e2m3_decode(codes):
    codes = np.asarray(codes, np.uint8)
    return np.array([lib().lqo_e2m3_decode(int(c) & 63) for c in codes.ravel()], np.float32).reshape(codes.shape)


def e2m3_encode(u: float) -> int:
    return int(lib().lqo_e2m3_encode(float(u)))


def e8m0_decode(codes):
    return np.array([lib().lqo_e8m0_decode(int(c)) for c in np.asarray(codes).ravel()],
                    np.float64).reshape(np.shape(codes))


def e2m1_encode(u: float) -> int:
    return int(lib().lqo_e2m1_encode(C.c_float(u)))


def e4m3_encode(u: float) -> int:
    return int(lib().lqo_e4m3_encode(C.c_float(u)))


def bf16_rne(f: float) -> int:
    return int(lib().lqo_bf16_rne(C.c_float(f)))


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


# ---------------------------------------------------------------------------------------
# INT family
# ---------------------------------------------------------------------------------------

@dataclass
class PackedInt:
    N: int
    K: int
    r: int
    g: int
    sint4: bool      # SINT4 blocks: g == 64, FP16-valued scales
    pq: np.ndarray   # N x K int8 in [-7,7]
    sw: np.ndarray   # N x G float32
    lq: np.ndarray   # N x r int8
    sl: np.ndarray   # N float32
    rq: np.ndarray   # r x K int8
    sr: np.ndarray   # r float32
    P: np.ndarray    # N x K float32 residual before Q1


def pack_int(W, L, R, g: int, br_w_bits: int, residual_from_quantized: bool = True,
             sint4_blocks: bool = False) -> PackedInt:
    W = _f32(W)
    N, K = W.shape
    r = 0 if L is None else int(np.shape(L)[1])
    assert K % g == 0 and (g == 64 or not sint4_blocks)
    Lc = _f32(L) if r else np.zeros((N, 0), np.float32)
    Rc = _f32(R) if r else np.zeros((0, K), np.float32)
    G = K // g
    out = PackedInt(N, K, r, g, bool(sint4_blocks), np.empty((N, K), np.int8), np.empty((N, G), np.float32),
                    np.empty((N, r), np.int8), np.ones(N, np.float32),
                    np.empty((r, K), np.int8), np.ones(r, np.float32),
                    np.empty((N, K), np.float32))
    lib().lqo_pack_int(C.c_int64(N), C.c_int64(K), C.c_int(r), C.c_int(g),
                       C.c_int(QMAX[br_w_bits]), C.c_int(1 if residual_from_quantized else 0),
                       _p(W), _p(Lc), _p(Rc), _p(out.pq), _p(out.sw), _p(out.lq), _p(out.sl),
                       _p(out.rq), _p(out.sr), _p(out.P), C.c_int(1 if sint4_blocks else 0))
    return out


@dataclass
class ActInt:
    M: int
    xq: np.ndarray    # M x K int8 in [-7,7]
    sx: np.ndarray    # M, or M x K/64 with SINT4 blocks
    xb: np.ndarray    # M x K int8
    sxb: np.ndarray   # M
    accT: np.ndarray  # M x r int32
    T: np.ndarray     # M x r float32
    tq: np.ndarray    # M x r int8
    st: np.ndarray    # M


def quantize_act_int(X, pk: PackedInt, br_a_bits: int) -> ActInt:
    """Main activation scales follow the packed weights: SINT4 blocks for both operands or for neither."""
    X = _f32(X)
    M, K = X.shape
    assert K == pk.K
    r = pk.r
    out = ActInt(M, np.empty((M, K), np.int8), np.empty((M, K // 64) if pk.sint4 else M, np.float32),
                 np.zeros((M, K), np.int8), np.ones(M, np.float32),
                 np.zeros((M, r), np.int32), np.zeros((M, r), np.float32),
                 np.zeros((M, r), np.int8), np.ones(M, np.float32))
    lib().lqo_quantize_act_int(C.c_int64(M), C.c_int64(K), C.c_int(r), C.c_int(QMAX[br_a_bits]),
                               _p(X), _p(pk.rq), _p(pk.sr), _p(out.xq), _p(out.sx), _p(out.xb),
                               _p(out.sxb), _p(out.accT), _p(out.T), _p(out.tq), _p(out.st),
                               C.c_int(64 if pk.sint4 else 0))
    return out


@dataclass
class FwdOut:
    acc: Optional[np.ndarray]    # M x N x G int32 (INT only, optional)
    acc2: Optional[np.ndarray]   # M x N int32 (INT only, optional)
    ymain: np.ndarray            # M x N float32
    ybr: np.ndarray              # M x N float32
    y32: np.ndarray              # M x N float32
    Y: np.ndarray                # M x N uint16 (bf16 bits)


def fwd_int(pk: PackedInt, act: ActInt, want_acc: bool = False) -> FwdOut:
    M, N, K, r, g = act.M, pk.N, pk.K, pk.r, pk.g
    G = K // g
    acc = np.empty((M, N, G), np.int32) if want_acc else None
    acc2 = np.empty((M, N), np.int32) if want_acc else None
    out = FwdOut(acc, acc2, np.empty((M, N), np.float32), np.empty((M, N), np.float32),
                 np.empty((M, N), np.float32), np.empty((M, N), np.uint16))
    lib().lqo_fwd_int(C.c_int64(M), C.c_int64(N), C.c_int64(K), C.c_int(r), C.c_int(g),
                      _p(act.xq), _p(act.sx), _p(pk.pq), _p(pk.sw), _p(act.tq), _p(act.st),
                      _p(pk.lq), _p(pk.sl), _p(acc), _p(acc2), _p(out.ymain), _p(out.ybr),
                      _p(out.y32), _p(out.Y), C.c_int(64 if pk.sint4 else 0))
    return out


# ---------------------------------------------------------------------------------------
# MX family
# ---------------------------------------------------------------------------------------

@dataclass
class PackedMx:
    N: int
    K: int
    r: int
    pc: np.ndarray   # N x K uint8 E2M1 codes
    pe: np.ndarray   # N x K/32 uint8 E8M0
    l8: np.ndarray   # N x r uint8 E4M3
    sl: np.ndarray
    r8: np.ndarray   # r x K uint8 E4M3
    sr: np.ndarray
    P: np.ndarray


def pack_mx(W, L, R, residual_from_quantized: bool = True) -> PackedMx:
    W = _f32(W)
    N, K = W.shape
    r = 0 if L is None else int(np.shape(L)[1])
    assert K % 32 == 0
    Lc = _f32(L) if r else np.zeros((N, 0), np.float32)
    Rc = _f32(R) if r else np.zeros((0, K), np.float32)
    out = PackedMx(N, K, r, np.empty((N, K), np.uint8), np.empty((N, K // 32), np.uint8),
                   np.empty((N, r), np.uint8), np.ones(N, np.float32),
                   np.empty((r, K), np.uint8), np.ones(r, np.float32), np.empty((N, K), np.float32))
    lib().lqo_pack_mx(C.c_int64(N), C.c_int64(K), C.c_int(r),
                      C.c_int(1 if residual_from_quantized else 0), _p(W), _p(Lc), _p(Rc),
                      _p(out.pc), _p(out.pe), _p(out.l8), _p(out.sl), _p(out.r8), _p(out.sr),
                      _p(out.P))
    return out


@dataclass
class ActMx:
    M: int
    xc: np.ndarray    # M x K uint8 E2M1
    xe: np.ndarray    # M x K/32 uint8 E8M0
    xb8: np.ndarray   # M x K uint8 E4M3
    sxb: np.ndarray
    T: np.ndarray     # M x r float32
    tq8: np.ndarray   # M x r uint8 E4M3
    st: np.ndarray


def quantize_act_mx(X, pk: PackedMx) -> ActMx:
    X = _f32(X)
    M, K = X.shape
    r = pk.r
    out = ActMx(M, np.empty((M, K), np.uint8), np.empty((M, K // 32), np.uint8),
                np.zeros((M, K), np.uint8), np.ones(M, np.float32), np.zeros((M, r), np.float32),
                np.zeros((M, r), np.uint8), np.ones(M, np.float32))
    lib().lqo_quantize_act_mx(C.c_int64(M), C.c_int64(K), C.c_int(r), _p(X), _p(pk.r8), _p(pk.sr),
                              _p(out.xc), _p(out.xe), _p(out.xb8), _p(out.sxb), _p(out.T),
                              _p(out.tq8), _p(out.st))
    return out


def fwd_mx(pk: PackedMx, act: ActMx) -> FwdOut:
    M, N, K, r = act.M, pk.N, pk.K, pk.r
    out = FwdOut(None, None, np.empty((M, N), np.float32), np.empty((M, N), np.float32),
                 np.empty((M, N), np.float32), np.empty((M, N), np.uint16))
    lib().lqo_fwd_mx(C.c_int64(M), C.c_int64(N), C.c_int64(K), C.c_int(r), _p(act.xc), _p(act.xe),
                     _p(pk.pc), _p(pk.pe), _p(act.tq8), _p(act.st), _p(pk.l8), _p(pk.sl),
                     _p(out.ymain), _p(out.ybr), _p(out.y32), _p(out.Y))
    return out


# ---------------------------------------------------------------------------------------
# MXB family: MXFP4 main, MXFP8e4 (block-scaled E4M3) branch
# ---------------------------------------------------------------------------------------

def quant_mxfp8(v):
    v = _f32(v).ravel()
    assert v.size % 32 == 0
    codes = np.empty(v.size, np.uint8)
    e = np.empty(v.size // 32, np.uint8)
    lib().lqo_quant_mxfp8(_p(v), C.c_int64(v.size), _p(codes), _p(e))
    return codes, e


def quant_mxfp6(v):
    v = _f32(v).ravel()
    assert v.size % 32 == 0
    codes = np.empty(v.size, np.uint8)
    e = np.empty(v.size // 32, np.uint8)
    lib().lqo_quant_mxfp6(_p(v), C.c_int64(v.size), _p(codes), _p(e))
    return codes, e


def mxb_decode(codes, elem: int):
    """Element values of a block-scaled FP branch: E4M3 (elem 8) or E2M3 (elem 6)."""
    return e4m3_decode(codes) if elem == 8 else e2m3_decode(codes)


@dataclass
class PackedMxb:
    N: int
    K: int
    r: int
    pc: np.ndarray   # N x K uint8 E2M1 codes
    pe: np.ndarray   # N x K/32 uint8 E8M0
    l8: np.ndarray   # N x r uint8 E4M3
    le: np.ndarray   # N x r/32 uint8 E8M0
    r8: np.ndarray   # r x K uint8 E4M3
    re: np.ndarray   # r x K/32 uint8 E8M0
    P: np.ndarray
    elem: int = 8    # 8: E4M3 elements (MXFP8e4); 6: E2M3 elements (MXFP6e2), same field names


def pack_mxb(W, L, R, residual_from_quantized: bool = True, elem: int = 8) -> PackedMxb:
    W = _f32(W)
    N, K = W.shape
    r = 0 if L is None else int(np.shape(L)[1])
    assert K % 32 == 0 and r % 32 == 0
    Lc = _f32(L) if r else np.zeros((N, 0), np.float32)
    Rc = _f32(R) if r else np.zeros((0, K), np.float32)
    out = PackedMxb(N, K, r, np.empty((N, K), np.uint8), np.empty((N, K // 32), np.uint8),
                    np.empty((N, r), np.uint8), np.empty((N, r // 32), np.uint8),
                    np.empty((r, K), np.uint8), np.empty((r, K // 32), np.uint8), np.empty((N, K), np.float32), elem)
    (lib().lqo_pack_mxb if elem == 8 else lib().lqo_pack_mxb6)(C.c_int64(N), C.c_int64(K), C.c_int(r), C.c_int(1 if residual_from_quantized else 0),
                       _p(W), _p(Lc), _p(Rc), _p(out.pc), _p(out.pe), _p(out.l8), _p(out.le), _p(out.r8),
                       _p(out.re), _p(out.P))
    return out


@dataclass
class ActMxb:
    M: int
    xc: np.ndarray    # M x K uint8 E2M1
    xe: np.ndarray    # M x K/32 uint8 E8M0
    xb8: np.ndarray   # M x K uint8 E4M3
    xbe: np.ndarray   # M x K/32 uint8 E8M0
    T: np.ndarray     # M x r float32
    tq8: np.ndarray   # M x r uint8 E4M3
    te: np.ndarray    # M x r/32 uint8 E8M0


def quantize_act_mxb(X, pk: PackedMxb) -> ActMxb:
    X = _f32(X)
    M, K = X.shape
    r = pk.r
    out = ActMxb(M, np.empty((M, K), np.uint8), np.empty((M, K // 32), np.uint8), np.zeros((M, K), np.uint8),
                 np.zeros((M, K // 32), np.uint8), np.zeros((M, r), np.float32), np.zeros((M, r), np.uint8),
                 np.zeros((M, r // 32), np.uint8))
    (lib().lqo_quantize_act_mxb if pk.elem == 8 else lib().lqo_quantize_act_mxb6)(C.c_int64(M), C.c_int64(K), C.c_int(r), _p(X), _p(pk.r8), _p(pk.re),
                               _p(out.xc), _p(out.xe), _p(out.xb8), _p(out.xbe), _p(out.T), _p(out.tq8),
                               _p(out.te))
    return out


def fwd_mxb(pk: PackedMxb, act: ActMxb) -> FwdOut:
    M, N, K, r = act.M, pk.N, pk.K, pk.r
    out = FwdOut(None, None, np.empty((M, N), np.float32), np.empty((M, N), np.float32),
                 np.empty((M, N), np.float32), np.empty((M, N), np.uint16))
    (lib().lqo_fwd_mxb if pk.elem == 8 else lib().lqo_fwd_mxb6)(C.c_int64(M), C.c_int64(N), C.c_int64(K), C.c_int(r), _p(act.xc), _p(act.xe),
                      _p(pk.pc), _p(pk.pe), _p(act.tq8), _p(act.te), _p(pk.l8), _p(pk.le),
                      _p(out.ymain), _p(out.ybr), _p(out.y32), _p(out.Y))
    return out


# ---------------------------------------------------------------------------------------
# MXI family: MXINT4 main, MXINT8 / MXINT4 branch
# ---------------------------------------------------------------------------------------

def quant_mxint(v, bits: int):
    v = _f32(v).ravel()
    assert v.size % 32 == 0 and bits in (4, 8)
    codes = np.empty(v.size, np.int8)
    e = np.empty(v.size // 32, np.uint8)
    lib().lqo_quant_mxint(_p(v), C.c_int64(v.size), C.c_int(bits), _p(codes), _p(e))
    return codes, e


def mxint_scale(e8m0, bits: int):
    """Value of one code step of a block: 2^(byte - 127 - (bits - 2)), as float64."""
    return np.ldexp(1.0, np.asarray(e8m0).astype(np.int64) - 127 - (bits - 2))


@dataclass
class PackedMxi:
    N: int
    K: int
    r: int
    bw_bits: int
    pq: np.ndarray   # N x K int8 (4-bit codes)
    pe: np.ndarray   # N x K/32 uint8 E8M0
    lq: np.ndarray   # N x r int8
    le: np.ndarray   # N x r/32 uint8
    rq: np.ndarray   # r x K int8
    re: np.ndarray   # r x K/32 uint8
    P: np.ndarray


def pack_mxi(W, L, R, bw_bits: int = 8, residual_from_quantized: bool = True) -> PackedMxi:
    W = _f32(W)
    N, K = W.shape
    r = 0 if L is None else int(np.shape(L)[1])
    assert K % 32 == 0 and r % 32 == 0 and bw_bits in (4, 8)
    Lc = _f32(L) if r else np.zeros((N, 0), np.float32)
    Rc = _f32(R) if r else np.zeros((0, K), np.float32)
    out = PackedMxi(N, K, r, bw_bits, np.empty((N, K), np.int8), np.empty((N, K // 32), np.uint8),
                    np.empty((N, r), np.int8), np.empty((N, r // 32), np.uint8),
                    np.empty((r, K), np.int8), np.empty((r, K // 32), np.uint8), np.empty((N, K), np.float32))
    lib().lqo_pack_mxi(C.c_int64(N), C.c_int64(K), C.c_int(r), C.c_int(bw_bits),
                       C.c_int(1 if residual_from_quantized else 0), _p(W), _p(Lc), _p(Rc), _p(out.pq), _p(out.pe),
                       _p(out.lq), _p(out.le), _p(out.rq), _p(out.re), _p(out.P))
    return out


@dataclass
class ActMxi:
    M: int
    xq: np.ndarray    # M x K int8 (4-bit codes)
    xe: np.ndarray    # M x K/32 uint8
    xb: np.ndarray    # M x K int8
    xbe: np.ndarray   # M x K/32 uint8
    T: np.ndarray     # M x r float32
    tq: np.ndarray    # M x r int8
    te: np.ndarray    # M x r/32 uint8


def quantize_act_mxi(X, pk: PackedMxi) -> ActMxi:
    X = _f32(X)
    M, K = X.shape
    r = pk.r
    out = ActMxi(M, np.empty((M, K), np.int8), np.empty((M, K // 32), np.uint8), np.zeros((M, K), np.int8),
                 np.zeros((M, K // 32), np.uint8), np.zeros((M, r), np.float32), np.zeros((M, r), np.int8),
                 np.zeros((M, r // 32), np.uint8))
    lib().lqo_quantize_act_mxi(C.c_int64(M), C.c_int64(K), C.c_int(r), C.c_int(pk.bw_bits), _p(X), _p(pk.rq),
                               _p(pk.re), _p(out.xq), _p(out.xe), _p(out.xb), _p(out.xbe), _p(out.T), _p(out.tq),
                               _p(out.te))
    return out


def handoff_mxi(Y_bits, pk_next: PackedMxi) -> ActMxi:
    """Quantized hand-off between two linears (Section 4.5: activations move between layers in the MX formats instead
    of 16 bits).  The reading taken: the next layer's activation codes are those of its own activation step applied to
    the bf16 value this layer would have stored, Q(bf16_rne(y)) -- so a fused epilogue that emits codes instead of
    bf16 changes no bit of the two-call path.  Y_bits: M x N uint16 (bf16 bits), N = pk_next.K."""
    return quantize_act_mxi(bf16_bits_to_f32(np.asarray(Y_bits, np.uint16)), pk_next)


def fwd_mxi(pk: PackedMxi, act: ActMxi) -> FwdOut:
    M, N, K, r = act.M, pk.N, pk.K, pk.r
    out = FwdOut(None, None, np.empty((M, N), np.float32), np.empty((M, N), np.float32),
                 np.empty((M, N), np.float32), np.empty((M, N), np.uint16))
    lib().lqo_fwd_mxi(C.c_int64(M), C.c_int64(N), C.c_int64(K), C.c_int(r), C.c_int(pk.bw_bits), _p(act.xq),
                      _p(act.xe), _p(pk.pq), _p(pk.pe), _p(act.tq), _p(act.te), _p(pk.lq), _p(pk.le),
                      _p(out.ymain), _p(out.ybr), _p(out.y32), _p(out.Y))
    return out


# ---------------------------------------------------------------------------------------
# data-free calibration of the factors (Eq. 4, App. B.2)
# ---------------------------------------------------------------------------------------

@dataclass
class CalibState:
    """fp32 state of the optimisation: factors (paper's sign: Q1(W + L R) - W ~ L R) and Adam moments."""
    L: np.ndarray
    R: np.ndarray
    mL: np.ndarray
    vL: np.ndarray
    mR: np.ndarray
    vR: np.ndarray
    step: int = 0


def calib_init(L, R) -> CalibState:
    L, R = _f32(L).copy(), _f32(R).copy()
    return CalibState(L, R, np.zeros_like(L), np.zeros_like(L), np.zeros_like(R), np.zeros_like(R), 0)


@dataclass
class CalibOut:
    loss: float          # mean squared error before this step's update
    E: np.ndarray        # N x K  deq(Q1(W + L R)) - (W + L R)
    gL: np.ndarray       # N x r
    gR: np.ndarray       # r x K


Q1_KINDS = {"int": 0, "sint4": 1, "mxfp4": 2, "mxint4": 3}


def calib_step(W, st: CalibState, g: int = 64, sint4_blocks: bool = False, lr: float = 1e-4, beta1: float = 0.9,
               beta2: float = 0.999, eps: float = 1e-8, q1: Optional[str] = None) -> CalibOut:
    """One Adam step; updates `st` in place and returns the loss / error / gradients it was computed from.
    q1: main quantiser, "int" (groups of g, fp32 scales; the default), "sint4", "mxfp4" or "mxint4"."""
    kind = Q1_KINDS[q1] if q1 is not None else (1 if sint4_blocks else 0)
    if kind:
        g = 64 if kind == 1 else 32
    W = _f32(W)
    N, K = W.shape
    r = st.L.shape[1]
    assert st.L.shape == (N, r) and st.R.shape == (r, K) and K % g == 0
    st.step += 1
    out = CalibOut(0.0, np.empty((N, K), np.float32), np.empty((N, r), np.float32), np.empty((r, K), np.float32))
    loss = C.c_double(0.0)
    lib().lqo_calib_step(C.c_int64(N), C.c_int64(K), C.c_int(r), C.c_int(g), C.c_int(kind), _p(W),
                         _p(st.L), _p(st.R), _p(st.mL), _p(st.vL), _p(st.mR), _p(st.vR), C.c_int(st.step),
                         C.c_double(lr), C.c_double(beta1), C.c_double(beta2), C.c_double(eps), _p(out.E), _p(out.gL),
                         _p(out.gR), C.byref(loss))
    out.loss = float(loss.value)
    return out


# ---------------------------------------------------------------------------------------
# rotation of the factors before quantisation (Section 3.3, Eq. 6-7)
# ---------------------------------------------------------------------------------------

@dataclass
class RotState:
    """fp32 state of the rotation search: the orthogonal matrix and the optimiser's momentum."""
    Omega: np.ndarray
    Mom: np.ndarray


def rot_init(r: int, Omega=None, Mom=None) -> RotState:
    return RotState(np.eye(r, dtype=np.float32) if Omega is None else _f32(Omega).copy(),
                    np.zeros((r, r), np.float32) if Mom is None else _f32(Mom).copy())


@dataclass
class RotOut:
    loss: float          # Eq. 7 before this step's update
    E1: np.ndarray       # N x r   deq(Q2(L Omega)) - L Omega
    E2: np.ndarray       # r x K   deq(Q2(Omega^T R)) - Omega^T R
    G: np.ndarray        # r x r   Euclidean gradient used by the step


Q2_KINDS = {"int": 0, "fp8": 1, "mxfp8": 2, "mxfp6": 3, "mxint": 4}


def rot_step(L, R, st: RotState, bits: int = 8, lr: float = 0.5, beta: float = 0.9, eps: float = 1e-8, q: float = 0.5,
             s: int = 2, grad_scale: float = 1.0, q2: str = "int") -> RotOut:
    """One Cayley-SGD step on Omega; updates `st` in place.  q2: the format of Q2 ("int": per-row symmetric integers of
    `bits`; "fp8": E4M3 with a per-row fp32 scale; "mxfp8", "mxfp6", "mxint" (of `bits`): blocks of 32 along the row)."""
    L, R = _f32(L), _f32(R)
    N, r = L.shape
    K = R.shape[1]
    assert R.shape[0] == r and st.Omega.shape == (r, r) and st.Mom.shape == (r, r)
    out = RotOut(0.0, np.empty((N, r), np.float32), np.empty((r, K), np.float32), np.empty((r, r), np.float32))
    loss = C.c_double(0.0)
    kind = Q2_KINDS[q2]
    lib().lqo_rot_step(C.c_int64(N), C.c_int64(K), C.c_int(r), C.c_int(kind), C.c_int(2 ** (bits - 1) - 1 if kind == 0 else bits),
                       _p(L), _p(R), _p(st.Omega),
                       _p(st.Mom), C.c_double(lr), C.c_double(beta), C.c_double(eps), C.c_double(q), C.c_int(s),
                       C.c_double(grad_scale), _p(out.E1), _p(out.E2), _p(out.G), C.byref(loss))
    out.loss = float(loss.value)
    return out


def rot_apply(L, R, Omega):
    """(L Omega, Omega^T R) in the fp32 arithmetic the loss quantises."""
    L, R, Omega = _f32(L), _f32(R), _f32(Omega)
    N, r = L.shape
    K = R.shape[1]
    Lr, Rr = np.empty((N, r), np.float32), np.empty((r, K), np.float32)
    lib().lqo_rot_apply(C.c_int64(N), C.c_int64(K), C.c_int(r), _p(L), _p(R), _p(Omega), _p(Lr), _p(Rr))
    return Lr, Rr
