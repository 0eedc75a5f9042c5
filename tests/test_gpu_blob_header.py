"""Blob headers on the GPU, through the C-ABI: every kernel that fills a blob writes its header, lq_verify_blob accepts
the configuration (and token count) the blob was written for and reports LQ_ERR_STALE_BLOB for any other."""
import dataclasses

import pytest
import torch

from paper_2604_18117_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _status(lq, fn, *a, **k):
    try:
        fn(*a, **k)
        return lq.LQ_OK
    except lq.LqError as e:
        return e.status


def _dev(a):
    return None if a is None else torch.from_numpy(a).cuda()


CASES = [
    ("c2_qkv", dict(M=70, K=256, N=320, r=32)),      # INT family, per-token activation scales
    ("c2s_qkv", dict(M=70, K=256, N=320, r=32)),     # SINT4 blocks on both operands
    ("c4_qkv", dict(M=70, K=320, N=192, r=64)),      # 6-bit branch
    ("c5_qkv", dict(M=70, K=256, N=320, r=32)),      # MXFP4 main, fp32-scaled FP8 branch
    ("c5b_qkv", dict(M=70, K=256, N=320, r=32)),     # MXFP8e4 branch
    ("c5i_qkv", dict(M=70, K=256, N=320, r=32)),     # MXINT4 main, MXINT8 branch
]


@pytest.mark.parametrize("name,shape", [c for c in CASES if c[0] in wl.LAYERS])
def test_headers_written_and_checked(name, shape):
    from paper_2604_18117_amd import binding as lq
    layer = wl.shrink(wl.LAYERS[name], **shape)
    X, W, L, R = wl.make_inputs(layer)
    cfg = lq.config_for_layer(layer)
    packed = torch.full((lq.lq_packed_sizes(cfg),), 0xFF, dtype=torch.uint8, device="cuda")
    assert _status(lq, lq.lq_verify_blob, cfg, lq.LQ_BLOB_PACKED, packed) == lq.LQ_ERR_STALE_BLOB   # nothing written yet
    lq.lq_pack_weights(cfg, _dev(W), _dev(L), _dev(R), packed=packed)
    lq.lq_verify_blob(cfg, lq.LQ_BLOB_PACKED, packed)
    M = layer.M
    act = torch.full((lq.lq_act_sizes(cfg, M),), 0xFF, dtype=torch.uint8, device="cuda")
    assert _status(lq, lq.lq_verify_blob, cfg, lq.LQ_BLOB_ACT, act, M) == lq.LQ_ERR_STALE_BLOB
    lq.lq_quantize_act(cfg, packed, wl.to_dev_x(X, layer.x_dtype), act=act)
    lq.lq_verify_blob(cfg, lq.LQ_BLOB_ACT, act, M)
    # the wrong kind, another token count, and every single-field change of the configuration that still sizes within the blob
    assert _status(lq, lq.lq_verify_blob, cfg, lq.LQ_BLOB_ACT, packed, 1) == lq.LQ_ERR_STALE_BLOB
    assert _status(lq, lq.lq_verify_blob, cfg, lq.LQ_BLOB_ACT, act, M - 1) == lq.LQ_ERR_STALE_BLOB
    others = [dataclasses.replace(layer, N=layer.N - 64), dataclasses.replace(layer, K=layer.K - 64)]
    if layer.r == 64:
        others.append(dataclasses.replace(layer, r=32))
    if layer.family == "int":
        others.append(dataclasses.replace(layer, br_w_bits=4 if layer.br_w_bits != 4 else 8))
    for o in others:
        ocfg = lq.config_for_layer(o)
        if _status(lq, lq.lq_packed_sizes, ocfg) == lq.LQ_OK and lq.lq_packed_sizes(ocfg) <= packed.numel():
            assert _status(lq, lq.lq_verify_blob, ocfg, lq.LQ_BLOB_PACKED, packed) == lq.LQ_ERR_STALE_BLOB, o
    # the forward still consumes the blobs (the header shifts every section by 256 bytes)
    Y = lq.lq_linear_lowrank_fwd(cfg, packed, act, M)
    torch.cuda.synchronize()
    assert torch.isfinite(Y.float()).all()


def test_handoff_writes_the_consumers_header():
    from paper_2604_18117_amd import binding as lq
    M = 70
    l1 = wl.Layer("p", M, 128, 192, 32, "mxi", 32, 8, 8, "bf16", seed=3)
    l2 = wl.Layer("c", M, 192, 64, 32, "mxi", 32, 8, 8, "bf16", seed=4)
    X, W1, L1, R1 = wl.make_inputs(l1)
    _, W2, L2, R2 = wl.make_inputs(l2)
    cfg1, cfg2 = lq.config_for_layer(l1), lq.config_for_layer(l2)
    pk1 = lq.lq_pack_weights(cfg1, _dev(W1), _dev(L1), _dev(R1))
    act1 = lq.lq_quantize_act(cfg1, pk1, wl.to_dev_x(X, "bf16"))
    act2 = torch.full((lq.lq_act_sizes(cfg2, M),), 0xFF, dtype=torch.uint8, device="cuda")
    codes = torch.full((lq.lq_handoff_sizes(cfg2, M),), 0xFF, dtype=torch.uint8, device="cuda")
    lq.lq_linear_lowrank_fwd_handoff(cfg1, pk1, act1, M, cfg2, act2, codes)
    lq.lq_verify_blob(cfg2, lq.LQ_BLOB_ACT, act2, M)
    assert _status(lq, lq.lq_verify_blob, cfg1, lq.LQ_BLOB_ACT, act2, M) == lq.LQ_ERR_STALE_BLOB
