"""Host-side checks of the C ABI (no GPU): the library loads, exports every symbol the header
declares, reports sizes, and rejects bad arguments before launching anything."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lq():
    if not os.path.exists(os.path.join(ROOT, "paper_2604_18117_amd", "liblq.so")):
        from paper_2604_18117_amd import build
        build.build()
    from paper_2604_18117_amd import binding
    return binding


def test_exports_every_declared_symbol(lq):
    header = open(os.path.join(ROOT, "include", "lq.h")).read()
    declared = set(re.findall(r"\b(lq_[a-z_0-9]+)\s*\(", header))
    assert declared == set(lq.EXPORTS)
    for name in declared:
        assert getattr(lq.raw(), name) is not None


def test_status_strings(lq):
    seen = {lq.lq_status_string(s) for s in range(8)}
    assert len(seen) == 8 and "ok" in seen


def test_sizes_follow_the_layout(lq):
    cfg = lq.make_config(3456, 1152, 32, "int", 64, 8, 8)
    pb = lq.lq_packed_sizes(cfg)
    # header 256 + codes N*K*6/8 (4-bit codes in 6-bit fields) + scales N*G*4 + lq N*32 + sl N*4 + rq r*K + sr r*4, each section 256-aligned
    parts = [256, 3456 * 1152 * 3 // 4, 3456 * 18 * 4, 3456 * 32, 3456 * 4, 32 * 1152, 32 * 4]
    assert pb == sum((x + 255) // 256 * 256 for x in parts)
    ab = lq.lq_act_sizes(cfg, 8192)
    parts = [256, 8192 * 1152 * 3 // 4, 8192 * 4, 8192 * 32, 8192 * 4]
    assert ab == sum((x + 255) // 256 * 256 for x in parts)
    # M is padded to a multiple of 32 rows
    assert lq.lq_act_sizes(cfg, 1) == lq.lq_act_sizes(cfg, 32) < lq.lq_act_sizes(cfg, 33)


def _cfg(lq, **kw):
    base = dict(N=128, K=256, rank=32, family="int", group=64, br_w_bits=8, br_a_bits=8)
    base.update(kw)
    return lq.make_config(base["N"], base["K"], base["rank"], base["family"], base["group"],
                          base["br_w_bits"], base["br_a_bits"])


@pytest.mark.parametrize("kw,status", [
    (dict(N=100), "LQ_ERR_SHAPE"), (dict(K=96), "LQ_ERR_SHAPE"), (dict(rank=24), "LQ_ERR_SHAPE"),
    (dict(group=32), "LQ_ERR_SHAPE"), (dict(K=192, group=128), "LQ_ERR_SHAPE"), (dict(N=0), "LQ_ERR_SHAPE"),
])
def test_shape_contract(lq, kw, status):
    n = C.c_size_t(0)
    cfg = _cfg(lq, **kw)
    assert lq.raw().lq_packed_sizes(C.byref(cfg), C.byref(n)) == getattr(lq, status)


def test_unsupported_combinations(lq):
    n = C.c_size_t(0)
    cfg = _cfg(lq)
    cfg.br_a = lq.LQ_INT4           # branch activations narrower than 6 bits are not a defined regime
    assert lq.raw().lq_packed_sizes(C.byref(cfg), C.byref(n)) == lq.LQ_ERR_UNSUPPORTED
    cfg = _cfg(lq)
    cfg.main_a = lq.LQ_INT8
    assert lq.raw().lq_packed_sizes(C.byref(cfg), C.byref(n)) == lq.LQ_ERR_UNSUPPORTED
    cfg = _cfg(lq)
    cfg.flags = 2                   # unknown flag bits are rejected
    assert lq.raw().lq_packed_sizes(C.byref(cfg), C.byref(n)) == lq.LQ_ERR_UNSUPPORTED
    cfg = _cfg(lq)
    cfg.main_a_group = 32           # INT activations: one scale per token, or SINT4 blocks of 64
    assert lq.raw().lq_packed_sizes(C.byref(cfg), C.byref(n)) == lq.LQ_ERR_UNSUPPORTED


def test_sint4_block_contract(lq):
    raw = lq.raw()
    n0, n1 = C.c_size_t(0), C.c_size_t(0)
    cfg = _cfg(lq)
    cfg.main_a_group = 64           # SINT4 blocks for both main operands: one block size for both
    assert raw.lq_packed_sizes(C.byref(cfg), C.byref(n1)) == lq.LQ_OK
    assert raw.lq_packed_sizes(C.byref(_cfg(lq)), C.byref(n0)) == lq.LQ_OK
    assert n0.value == n1.value     # a weight block scale takes a dword either way
    cfg.main_w_group = 128
    assert raw.lq_packed_sizes(C.byref(cfg), C.byref(n1)) == lq.LQ_ERR_UNSUPPORTED
    cfg = _cfg(lq, K=5696)
    cfg.main_a_group = 64           # K beyond 5632: the forward's LDS copy of a tile's token scales would not fit
    assert raw.lq_packed_sizes(C.byref(cfg), C.byref(n1)) == lq.LQ_ERR_UNSUPPORTED
    cfg = _cfg(lq, N=1 << 24, K=4608)
    cfg.main_a_group = 64           # 2^24 channels x 72 blocks x 4 bytes: beyond the 32-bit offsets of the scale stream
    assert raw.lq_packed_sizes(C.byref(cfg), C.byref(n1)) == lq.LQ_ERR_UNSUPPORTED
    # activation blob: K/64 scales per token (in whole 128-token tiles) instead of one
    cfg = _cfg(lq, K=256)
    cfg.main_a_group = 64
    assert raw.lq_act_sizes(C.byref(cfg), 100, C.byref(n1)) == lq.LQ_OK
    assert raw.lq_act_sizes(C.byref(_cfg(lq, K=256)), 100, C.byref(n0)) == lq.LQ_OK
    assert n1.value - n0.value == 4 * 128 * 4 - 128 * 4


def test_mx_family_contract(lq):
    n = C.c_size_t(0)
    raw = lq.raw()
    for fam in ("mx", "mxb"):
        assert raw.lq_packed_sizes(C.byref(_cfg(lq, family=fam, K=256)), C.byref(n)) == lq.LQ_OK
        # an odd number of 64-chunks is padded to whole 128-stages inside the blobs: K = 192 takes the room of K = 256
        assert lq.lq_packed_sizes(_cfg(lq, family=fam, K=192)) == lq.lq_packed_sizes(_cfg(lq, family=fam, K=256))
        assert lq.lq_act_sizes(_cfg(lq, family=fam, K=192), 100) == lq.lq_act_sizes(_cfg(lq, family=fam, K=256), 100)
        assert raw.lq_packed_sizes(C.byref(_cfg(lq, family=fam, K=160)), C.byref(n)) == lq.LQ_ERR_SHAPE
    # blocks of 32 along the rank: a block-scaled branch has no rank 16
    assert raw.lq_packed_sizes(C.byref(_cfg(lq, family="mx", rank=16)), C.byref(n)) == lq.LQ_OK
    assert raw.lq_packed_sizes(C.byref(_cfg(lq, family="mxb", rank=16)), C.byref(n)) == lq.LQ_ERR_SHAPE
    cfg = _cfg(lq, family="mxb")
    cfg.br_a = lq.LQ_FP8_E4M3       # both branch operands share one format
    assert raw.lq_packed_sizes(C.byref(cfg), C.byref(n)) == lq.LQ_ERR_UNSUPPORTED
    # MXFP6e2 branch: 32 six-bit codes sit in a 32-byte operand slot, so the sizes equal the 8-bit ones
    c6, c8 = _cfg(lq, family="mxb", br_w_bits=6, K=256), _cfg(lq, family="mxb", K=256)
    assert c6.br_w == c6.br_a == lq.LQ_MXFP6_E2M3
    assert lq.lq_packed_sizes(c6) == lq.lq_packed_sizes(c8) and lq.lq_act_sizes(c6, 100) == lq.lq_act_sizes(c8, 100)
    assert raw.lq_packed_sizes(C.byref(_cfg(lq, family="mxb", br_w_bits=6, rank=16)), C.byref(n)) == lq.LQ_ERR_SHAPE
    # codes N*K/2, E8M0 dwords per (32 rows, quad of 64-chunks, lane), lq N*64, one scale dword per
    # (channel, rank half), rq r*K, one scale dword per (128-chunk, 16 rank rows, lane) (+4)
    cfg = lq.make_config(3456, 1152, 32, "mxb")
    parts = [256, 3456 * 1152 // 2, 3456 // 32 * 5 * 256, 3456 * 64, 3456 * 8, 32 * 1152, 9 * 2 * 256 + 4]
    assert lq.lq_packed_sizes(cfg) == sum((x + 255) // 256 * 256 for x in parts)


def test_argument_errors_before_any_launch(lq):
    raw = lq.raw()
    cfg = _cfg(lq)
    good = C.c_void_p(1 << 20)       # fake, suitably aligned addresses: never dereferenced on these paths
    odd = C.c_void_p((1 << 20) + 4)
    pb, ab = lq.lq_packed_sizes(cfg), lq.lq_act_sizes(cfg, 64)
    assert raw.lq_packed_sizes(None, None) == lq.LQ_ERR_NULL
    assert raw.lq_pack_weights(C.byref(cfg), None, good, good, good, pb, None) == lq.LQ_ERR_NULL
    assert raw.lq_pack_weights(C.byref(cfg), good, None, good, good, pb, None) == lq.LQ_ERR_NULL
    assert raw.lq_pack_weights(C.byref(cfg), good, good, good, odd, pb, None) == lq.LQ_ERR_ALIGN
    assert raw.lq_pack_weights(C.byref(cfg), good, good, good, good, pb - 1, None) == lq.LQ_ERR_BUFFER_TOO_SMALL
    assert raw.lq_quantize_act(C.byref(cfg), good, pb, None, 64, 256, good, ab, None, None) == lq.LQ_ERR_NULL
    assert raw.lq_quantize_act(C.byref(cfg), None, 0, good, 64, 256, good, ab, None, None) == lq.LQ_ERR_NULL
    assert raw.lq_quantize_act(C.byref(cfg), good, pb, good, -1, 256, good, ab, None, None) == lq.LQ_ERR_SHAPE
    # an empty batch is a successful no-op on every per-call entry point: nothing launched, pointers not examined
    assert raw.lq_quantize_act(C.byref(cfg), None, 0, None, 0, 256, None, 0, None, None) == lq.LQ_OK
    assert raw.lq_linear_lowrank_fwd(C.byref(cfg), None, 0, None, 0, 0, None, 128, None, None) == lq.LQ_OK
    assert raw.lq_unpack_act(C.byref(cfg), None, 0, None, None) == lq.LQ_OK
    zero = C.c_size_t(99)
    assert raw.lq_act_sizes(C.byref(cfg), 0, C.byref(zero)) == lq.LQ_OK and zero.value == 0
    assert raw.lq_act_sizes(C.byref(cfg), -1, C.byref(zero)) == lq.LQ_ERR_SHAPE
    assert raw.lq_quantize_act(C.byref(cfg), good, pb, good, 64, 255, good, ab, None, None) == lq.LQ_ERR_SHAPE
    assert raw.lq_quantize_act(C.byref(cfg), good, pb, good, 64, 260, good, ab, None, None) == lq.LQ_ERR_ALIGN
    assert raw.lq_quantize_act(C.byref(cfg), good, pb, odd, 64, 256, good, ab, None, None) == lq.LQ_ERR_ALIGN
    assert raw.lq_quantize_act(C.byref(cfg), good, pb, good, 64, 256, good, ab - 1, None, None) == lq.LQ_ERR_BUFFER_TOO_SMALL
    assert raw.lq_linear_lowrank_fwd(C.byref(cfg), good, pb, good, ab, 64, None, 128, None, None) == lq.LQ_ERR_NULL
    assert raw.lq_linear_lowrank_fwd(C.byref(cfg), good, pb, good, ab, 64, good, 64, None, None) == lq.LQ_ERR_SHAPE
    assert raw.lq_linear_lowrank_fwd(C.byref(cfg), good, pb, good, ab, 64, good, 132, None, None) == lq.LQ_ERR_ALIGN
    # row strides beyond 2^22 elements do not fit the 32-bit offsets of the output's buffer stores
    assert raw.lq_linear_lowrank_fwd(C.byref(cfg), good, pb, good, ab, 64, good, (1 << 22) + 8, None, None) == lq.LQ_ERR_SHAPE
    assert raw.lq_linear_lowrank_fwd(C.byref(cfg), good, pb, good, ab, 64, odd, 128, None, None) == lq.LQ_ERR_ALIGN
    # a blob smaller than the configuration (or the token count) needs is refused before any launch
    assert raw.lq_linear_lowrank_fwd(C.byref(cfg), good, pb - 1, good, ab, 64, good, 128, None, None) == lq.LQ_ERR_BUFFER_TOO_SMALL
    assert raw.lq_linear_lowrank_fwd(C.byref(cfg), good, pb, good, ab - 1, 64, good, 128, None, None) == lq.LQ_ERR_BUFFER_TOO_SMALL
    assert raw.lq_linear_lowrank_fwd(C.byref(cfg), good, pb, good, lq.lq_act_sizes(cfg, 32), 64, good, 128, None, None) == lq.LQ_ERR_BUFFER_TOO_SMALL
    assert raw.lq_quantize_act(C.byref(cfg), good, pb - 1, good, 64, 256, good, ab, None, None) == lq.LQ_ERR_BUFFER_TOO_SMALL
    assert raw.lq_unpack_weights(C.byref(cfg), None, None, None) == lq.LQ_ERR_NULL
    assert raw.lq_unpack_act(C.byref(cfg), good, 64, None, None) == lq.LQ_ERR_NULL
    # K beyond the register-resident row of the activation kernels is accepted (long rows are streamed); a wrong row
    # stride is still caught first
    for fam in ("int", "mx"):
        big = _cfg(lq, K=8192, family=fam, group=64 if fam == "int" else 32)
        assert raw.lq_act_sizes(C.byref(big), 64, C.byref(C.c_size_t(0))) == lq.LQ_OK
        assert raw.lq_quantize_act(C.byref(big), good, 1 << 40, good, 64, 8000, good, 1 << 30, None, None) == lq.LQ_ERR_SHAPE


def test_mxi_contract(lq):
    n = C.c_size_t(0)
    raw = lq.raw()
    assert raw.lq_packed_sizes(C.byref(_cfg(lq, family="mxi", K=192)), C.byref(n)) == lq.LQ_OK     # K % 64 only
    assert raw.lq_packed_sizes(C.byref(_cfg(lq, family="mxi", rank=16)), C.byref(n)) == lq.LQ_ERR_SHAPE
    assert raw.lq_packed_sizes(C.byref(_cfg(lq, family="mxi", br_w_bits=4, rank=128)), C.byref(n)) == lq.LQ_OK
    cfg = _cfg(lq, family="mxi")
    cfg.br_a = lq.LQ_MXINT4          # branch activations stay at 8 bits
    assert raw.lq_packed_sizes(C.byref(cfg), C.byref(n)) == lq.LQ_ERR_UNSUPPORTED
    cfg = _cfg(lq, family="mxi")
    cfg.main_a = lq.LQ_MXFP4_E2M1    # no mixing of integer and floating-point formats within a layer (Section 4.1)
    assert raw.lq_packed_sizes(C.byref(cfg), C.byref(n)) == lq.LQ_ERR_UNSUPPORTED
    # 4-bit codes N*K/2, scale dwords per (32 rows, quad of chunks, lane), bf16 factors with one byte per block
    cfg = lq.make_config(3456, 1152, 64, "mxi")
    parts = [256, 3456 * 1152 // 2, 3456 // 32 * 5 * 256, 3456 * 64 * 2, 3456 * 2 + 4, 64 * 1152 * 2, 64 * 36 + 4]
    assert lq.lq_packed_sizes(cfg) == sum((x + 255) // 256 * 256 for x in parts)
    # the block-local scales need no register-resident row: K is not limited
    good = C.c_void_p(1 << 20)
    big = _cfg(lq, family="mxi", K=8192)
    assert raw.lq_quantize_act(C.byref(big), good, 1 << 40, good, 64, 8000, good, 1 << 30, None, None) == lq.LQ_ERR_SHAPE
    assert raw.lq_act_sizes(C.byref(big), 64, C.byref(n)) == lq.LQ_OK


def test_rank_96(lq):
    # rank 96 = the 6-bit point of a 512-bit budget (rank 85) padded; not with the fp32-scaled FP8 branch (8-bit only)
    n = C.c_size_t(0)
    raw = lq.raw()
    for fam, kw in (("mxb", {}), ("mxb", dict(br_w_bits=6)), ("mxi", {}), ("int", dict(br_w_bits=6, br_a_bits=6))):
        assert raw.lq_packed_sizes(C.byref(_cfg(lq, family=fam, rank=96, **kw)), C.byref(n)) == lq.LQ_OK
    assert raw.lq_packed_sizes(C.byref(_cfg(lq, family="mx", rank=96)), C.byref(n)) == lq.LQ_ERR_SHAPE


def test_smoothing_contract(lq):
    raw = lq.raw()
    n = C.c_size_t(0)
    good = C.c_void_p(1 << 20)
    plain, sm = _cfg(lq), lq.make_config(128, 256, 32, smooth=True)
    assert sm.flags == lq.LQ_FLAG_SMOOTH
    # one more section: K reciprocals
    assert lq.lq_packed_sizes(sm) == lq.lq_packed_sizes(plain) + 256 * 4
    pb = lq.lq_packed_sizes(sm)
    assert raw.lq_set_smoothing(C.byref(plain), good, good, pb, None) == lq.LQ_ERR_UNSUPPORTED
    assert raw.lq_set_smoothing(C.byref(sm), None, good, pb, None) == lq.LQ_ERR_NULL
    assert raw.lq_set_smoothing(C.byref(sm), good, good, pb - 1, None) == lq.LQ_ERR_BUFFER_TOO_SMALL
    assert raw.lq_set_smoothing(C.byref(sm), good, C.c_void_p((1 << 20) + 8), pb, None) == lq.LQ_ERR_ALIGN
    # the activation kernel needs the blob even without a branch
    sm0 = lq.make_config(128, 256, 0, smooth=True)
    assert raw.lq_quantize_act(C.byref(sm0), None, 0, good, 64, 256, good, 1 << 20, None, None) == lq.LQ_ERR_NULL
    # no K limit with smoothing either (long rows are streamed)
    assert raw.lq_packed_sizes(C.byref(lq.make_config(128, 4608, 32, smooth=True)), C.byref(n)) == lq.LQ_OK
    for fam, bits in (("mx", 8), ("mxb", 8), ("mxb", 6), ("mxi", 8), ("mxi", 4)):
        K = 4608
        a, b = lq.make_config(128, K, 32, fam, 32, bits, 8, smooth=True), lq.make_config(128, K, 32, fam, 32, bits, 8)
        assert a.flags == lq.LQ_FLAG_SMOOTH
        assert lq.lq_packed_sizes(a) == lq.lq_packed_sizes(b) + K * 4


def test_rotation_contract(lq):
    raw = lq.raw()
    n = C.c_size_t(0)
    good = C.c_void_p(1 << 20)
    cfg = lq.make_config(128, 256, 32)
    assert raw.lq_rot_sizes(C.byref(cfg), C.byref(n)) == lq.LQ_OK
    r, N, K = 32, 128, 256
    # Omega, momentum, gradient, E1, E2, row maxima, loss partials, 64 gradient partials, 3 scratch matrices (256-byte aligned each)
    a256 = lambda x: (x + 255) // 256 * 256
    want = 3 * a256(r * r * 4) + a256(N * r * 4) + a256(r * K * 4) + a256(1 * 4 * r * 4) + a256((1 + r * 1) * 4) + \
        a256(64 * r * r * 4) + a256(3 * r * r * 4)
    assert n.value == want
    opt = lq.lq_cayley(0.5, 0.9, 1e-8, 0.5, 2, 1.0)
    sb = n.value
    assert raw.lq_rot_init(C.byref(cfg), None, None, None, sb, None) == lq.LQ_ERR_NULL
    assert raw.lq_rot_init(C.byref(cfg), None, None, good, sb - 1, None) == lq.LQ_ERR_BUFFER_TOO_SMALL
    assert raw.lq_rot_init(C.byref(cfg), None, None, C.c_void_p((1 << 20) + 64), sb, None) == lq.LQ_ERR_ALIGN
    assert raw.lq_rot_step(C.byref(cfg), None, good, good, sb, C.byref(opt), None, None) == lq.LQ_ERR_NULL
    assert raw.lq_rot_step(C.byref(cfg), good, good, good, sb, None, None, None) == lq.LQ_ERR_NULL
    assert raw.lq_rot_step(C.byref(cfg), good, C.c_void_p((1 << 20) + 4), good, sb, C.byref(opt), None, None) == lq.LQ_ERR_ALIGN
    assert raw.lq_rot_step(C.byref(cfg), good, good, good, sb - 1, C.byref(opt), None, None) == lq.LQ_ERR_BUFFER_TOO_SMALL
    for bad in (lq.lq_cayley(0.0, 0.9, 1e-8, 0.5, 2, 1.0), lq.lq_cayley(0.5, 1.0, 1e-8, 0.5, 2, 1.0), lq.lq_cayley(0.5, 0.9, 0.0, 0.5, 2, 1.0),
                lq.lq_cayley(0.5, 0.9, 1e-8, 1.0, 2, 1.0), lq.lq_cayley(0.5, 0.9, 1e-8, 0.5, 17, 1.0), lq.lq_cayley(0.5, 0.9, 1e-8, 0.5, -1, 1.0),
                lq.lq_cayley(0.5, 0.9, 1e-8, 0.5, 2, 0.0)):
        assert raw.lq_rot_step(C.byref(cfg), good, good, good, sb, C.byref(bad), None, None) == lq.LQ_ERR_UNSUPPORTED
    assert raw.lq_rot_apply(C.byref(cfg), good, good, good, None, good, None) == lq.LQ_ERR_NULL
    assert raw.lq_rot_unpack(C.byref(cfg), good, None, None) == lq.LQ_ERR_NULL
    # every family's branch format; the state is sized by the caller's K (2240 = 35 chunks of 64, padded only inside packed blobs)
    for fam in ("mx", "mxb", "mxi"):
        assert raw.lq_rot_sizes(C.byref(lq.make_config(128, 256, 32, fam, 32)), C.byref(n)) == lq.LQ_OK and n.value == want
    a, b = lq.lq_rot_sizes(lq.make_config(128, 2240, 32, "mxb", 32)), lq.lq_rot_sizes(lq.make_config(128, 2240, 32))
    assert a == b
    # a branch to rotate
    assert raw.lq_rot_sizes(C.byref(lq.make_config(128, 256, 0)), C.byref(n)) == lq.LQ_ERR_SHAPE


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "single-GPU" in r.stderr


def test_calibration_contract(lq):
    raw = lq.raw()
    n = C.c_size_t(0)
    cfg = _cfg(lq)                                 # N 128, K 256, rank 32
    assert raw.lq_calib_sizes(C.byref(cfg), C.byref(n)) == lq.LQ_OK
    # factors, two moments and a gradient per factor, the N x K error matrix, a loss partial per wavefront, partials of grad_R
    nl, nr = 128 * 32 * 4, 32 * 256 * 4
    parts = [nl, nr, nl, nl, nr, nr, nl, nr, 128 * 256 * 4, 128 // 16 * 1 * 4 * 4, 8 * nr]   # K 256: 4 groups = one workgroup column; grad_R partials over 8 row ranges
    assert n.value == sum((x + 255) // 256 * 256 for x in parts)
    for fam in ("mx", "mxi"):                       # K 256 = four 64-chunks: the same workgroup grid, the same size
        m = C.c_size_t(0)
        assert raw.lq_calib_sizes(C.byref(_cfg(lq, family=fam)), C.byref(m)) == lq.LQ_OK and m.value == n.value
    assert raw.lq_calib_sizes(C.byref(_cfg(lq, rank=0)), C.byref(n)) == lq.LQ_ERR_SHAPE
    good, odd = C.c_void_p(1 << 20), C.c_void_p((1 << 20) + 4)
    sb = lq.lq_calib_sizes(cfg)
    ad = lq.lq_adam(1e-4, 0.9, 0.999, 1e-8)
    assert raw.lq_calib_init(C.byref(cfg), None, good, good, sb, None) == lq.LQ_ERR_NULL
    assert raw.lq_calib_init(C.byref(cfg), good, good, odd, sb, None) == lq.LQ_ERR_ALIGN
    assert raw.lq_calib_init(C.byref(cfg), good, good, good, sb - 1, None) == lq.LQ_ERR_BUFFER_TOO_SMALL
    assert raw.lq_calib_step(C.byref(cfg), None, good, sb, 1, C.byref(ad), None, None) == lq.LQ_ERR_NULL
    assert raw.lq_calib_step(C.byref(cfg), good, good, sb, 1, None, None, None) == lq.LQ_ERR_NULL
    assert raw.lq_calib_step(C.byref(cfg), good, good, sb, 0, C.byref(ad), None, None) == lq.LQ_ERR_SHAPE
    assert raw.lq_calib_step(C.byref(cfg), good, good, sb - 1, 1, C.byref(ad), None, None) == lq.LQ_ERR_BUFFER_TOO_SMALL
    assert raw.lq_calib_step(C.byref(cfg), good, odd, sb, 1, C.byref(ad), None, None) == lq.LQ_ERR_ALIGN
    bad = lq.lq_adam(1e-4, 1.0, 0.999, 1e-8)       # beta1 must be below 1
    assert raw.lq_calib_step(C.byref(cfg), good, good, sb, 1, C.byref(bad), None, None) == lq.LQ_ERR_UNSUPPORTED
    bad = lq.lq_adam(0.0, 0.9, 0.999, 1e-8)
    assert raw.lq_calib_step(C.byref(cfg), good, good, sb, 1, C.byref(bad), None, None) == lq.LQ_ERR_UNSUPPORTED
    assert raw.lq_calib_unpack(C.byref(cfg), good, None, None) == lq.LQ_ERR_NULL


def test_handoff_contract(lq):
    """Quantized hand-off: integer MX family on both sides, the consumer's K = the producer's N; every error is
    reported before any launch (no GPU needed)."""
    raw = lq.raw()
    n = C.c_size_t(0)
    prod = lq.make_config(320, 256, 32, "mxi", 32, 8, 8)
    cons = lq.make_config(128, 320, 64, "mxi", 32, 8, 8)
    assert raw.lq_handoff_sizes(C.byref(cons), 100, C.byref(n)) == lq.LQ_OK
    al = lambda x: (x + 255) // 256 * 256
    assert n.value == al(128 * 320) + al(128 * 10)          # Mp = 128 rows: one code byte per value, one scale byte per 32
    assert raw.lq_handoff_sizes(C.byref(_cfg(lq)), 100, C.byref(n)) == lq.LQ_ERR_UNSUPPORTED        # INT family
    assert raw.lq_handoff_sizes(C.byref(_cfg(lq, family="mx", K=256)), 100, C.byref(n)) == lq.LQ_ERR_UNSUPPORTED
    assert raw.lq_handoff_sizes(None, 100, C.byref(n)) == lq.LQ_ERR_NULL
    fake = C.c_void_p(0x1000)     # aligned, never dereferenced: the checks below fail first
    big = 1 << 40
    call = lambda p, c, **kw: raw.lq_linear_lowrank_fwd_handoff(
        C.byref(p), kw.get("packed", fake), kw.get("pb", big), fake, kw.get("ab", big), kw.get("M", 100), kw.get("Y", None), 0,
        C.byref(c), kw.get("act_next", fake), kw.get("anb", big), kw.get("codes", fake), kw.get("cb", big), None)
    assert call(prod, lq.make_config(128, 256, 64, "mxi", 32, 8, 8)) == lq.LQ_ERR_SHAPE          # K of the consumer != N
    assert call(_cfg(lq, N=320), cons) == lq.LQ_ERR_UNSUPPORTED                                  # producer outside the family
    assert call(prod, cons, packed=None) == lq.LQ_ERR_NULL
    assert call(prod, cons, codes=None) == lq.LQ_ERR_NULL
    assert call(prod, cons, act_next=C.c_void_p(0x1010)) == lq.LQ_ERR_ALIGN
    assert call(prod, cons, anb=16) == lq.LQ_ERR_BUFFER_TOO_SMALL
    assert call(prod, cons, cb=16) == lq.LQ_ERR_BUFFER_TOO_SMALL
    assert call(prod, cons, pb=lq.lq_packed_sizes(prod) - 1) == lq.LQ_ERR_BUFFER_TOO_SMALL       # the producer's own blobs
    assert call(prod, cons, ab=lq.lq_act_sizes(prod, 100) - 1) == lq.LQ_ERR_BUFFER_TOO_SMALL
    assert call(prod, cons, M=0) == lq.LQ_OK                                                     # an empty batch
    br = lambda c, **kw: raw.lq_branch_from_codes(C.byref(c), kw.get("packed", fake), kw.get("pb", big), kw.get("codes", fake),
                                                  kw.get("cb", big), kw.get("M", 100), fake, kw.get("anb", big), None)
    assert br(cons, packed=None) == lq.LQ_ERR_NULL
    assert br(cons, cb=16) == lq.LQ_ERR_BUFFER_TOO_SMALL
    assert br(cons, pb=64) == lq.LQ_ERR_BUFFER_TOO_SMALL
    assert br(_cfg(lq)) == lq.LQ_ERR_UNSUPPORTED
    assert br(lq.make_config(128, 320, 0, "mxi", 32, 8, 8), packed=None) == lq.LQ_OK             # rank 0: nothing to do


def test_verify_blob_contract(lq):
    raw = lq.raw()
    cfg = _cfg(lq)
    fake = C.c_void_p(0x1000)
    assert raw.lq_verify_blob(C.byref(cfg), lq.LQ_BLOB_PACKED, None, 1 << 30, 0, None) == lq.LQ_ERR_NULL
    assert raw.lq_verify_blob(C.byref(cfg), 3, fake, 1 << 30, 0, None) == lq.LQ_ERR_UNSUPPORTED
    assert raw.lq_verify_blob(C.byref(cfg), lq.LQ_BLOB_ACT, fake, 1 << 30, 0, None) == lq.LQ_ERR_SHAPE
    assert raw.lq_verify_blob(C.byref(cfg), lq.LQ_BLOB_PACKED, C.c_void_p(0x1008), 1 << 30, 0, None) == lq.LQ_ERR_ALIGN
    assert raw.lq_verify_blob(C.byref(cfg), lq.LQ_BLOB_PACKED, fake, 64, 0, None) == lq.LQ_ERR_BUFFER_TOO_SMALL
    assert raw.lq_verify_blob(C.byref(_cfg(lq, N=100)), lq.LQ_BLOB_PACKED, fake, 1 << 30, 0, None) == lq.LQ_ERR_SHAPE
