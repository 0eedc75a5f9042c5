"""The per-call path (activation step + forward) recorded into a HIP graph: two kernel nodes, no
memset nodes, no allocation.  Every replay must give the eager result, also with other work and
synchronisations between the replays and with new contents in the same input buffer."""
import numpy as np
import pytest
import torch

from paper_2604_18117_amd import binding as lq
from paper_2604_18117_amd import workloads as wl
from tests.gpu_util import to_dev_x

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("family,g,bits", [("int", 64, 8), ("int", 128, 8), ("sint4", 64, 8), ("mx", 32, 8), ("mxb", 32, 8),
                                           ("mxb", 32, 6), ("mxi", 32, 8)])
def test_graph_replays_match_eager(family, g, bits):
    ag = 64 if family == "sint4" else 0      # "sint4": INT family with SINT4 blocks for both main operands
    family = "int" if ag else family
    layer = wl.Layer("t", 700, 512, 640, 32, family, g, bits, 8 if family == "mxi" else bits, "bf16", outlier_scale=10.0,
                     n_outliers=4, seed=11, a_group=ag)
    X, W, L, R = wl.make_inputs(layer)
    cfg = lq.config_for_layer(layer)
    packed = lq.lq_pack_weights(cfg, torch.from_numpy(W).cuda(), torch.from_numpy(L).cuda(), torch.from_numpy(R).cuda())
    M = layer.M
    rng = np.random.default_rng(5)
    inputs = [to_dev_x(X if i == 0 else X[rng.permutation(M)] * np.float32(0.5 + i), "bf16") for i in range(3)]
    # eager results
    eager = []
    for Xi in inputs:
        act = lq.lq_quantize_act(cfg, packed, Xi)
        eager.append(lq.lq_linear_lowrank_fwd(cfg, packed, act, M).clone())
    torch.cuda.synchronize()
    # capture on a side stream with static buffers
    Xs = inputs[0].clone()
    act = torch.empty(lq.lq_act_sizes(cfg, M), dtype=torch.uint8, device="cuda")
    Y = torch.empty((M, layer.N), dtype=torch.bfloat16, device="cuda")
    graph = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        lq.lq_quantize_act(cfg, packed, Xs, act=act)          # warm-up outside the capture
        lq.lq_linear_lowrank_fwd(cfg, packed, act, M, Y=Y)
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=s):
        lq.lq_quantize_act(cfg, packed, Xs, act=act)
        lq.lq_linear_lowrank_fwd(cfg, packed, act, M, Y=Y)
    for rep in range(6):
        i = rep % 3
        Xs.copy_(inputs[i])
        Y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y.view(torch.int16), eager[i].view(torch.int16)), f"replay {rep}"
        # eager work of the same library between replays
        a2 = lq.lq_quantize_act(cfg, packed, inputs[(i + 1) % 3])
        y2 = lq.lq_linear_lowrank_fwd(cfg, packed, a2, M)
        torch.cuda.synchronize()
        assert torch.equal(y2.view(torch.int16), eager[(i + 1) % 3].view(torch.int16))


@pytest.mark.parametrize("family,bits", [("mx", 8), ("mxb", 8), ("mxb", 6), ("mxi", 8), ("mxi", 4), ("sint4", 8)])
def test_strided_views_and_determinism(family, bits):
    """X and Y as column slices of wider tensors (row strides beyond K and N); repeated calls give identical bits."""
    ag = 64 if family == "sint4" else 0
    family = "int" if ag else family
    layer = wl.Layer("t", 130, 384, 192, 32, family, 64 if ag else 32, bits, 8 if family == "mxi" else bits, "bf16", seed=13,
                     a_group=ag)
    X, W, L, R = wl.make_inputs(layer)
    cfg = lq.config_for_layer(layer)
    packed = lq.lq_pack_weights(cfg, torch.from_numpy(W).cuda(), torch.from_numpy(L).cuda(), torch.from_numpy(R).cuda())
    Xd = to_dev_x(X, "bf16")
    ref = lq.lq_linear_lowrank_fwd(cfg, packed, lq.lq_quantize_act(cfg, packed, Xd), layer.M)
    wide = torch.zeros((layer.M, layer.K + 64), dtype=torch.bfloat16, device="cuda")
    wide[:, :layer.K] = Xd
    wide[:, layer.K:] = 1e4                                     # must never be read into a block
    Ywide = torch.zeros((layer.M, layer.N + 8), dtype=torch.bfloat16, device="cuda")
    act = lq.lq_quantize_act(cfg, packed, wide[:, :layer.K])
    lq.lq_linear_lowrank_fwd(cfg, packed, act, layer.M, Y=Ywide[:, :layer.N])
    torch.cuda.synchronize()
    assert torch.equal(Ywide[:, :layer.N].view(torch.int16), ref.view(torch.int16)) and not Ywide[:, layer.N:].any()
    for _ in range(3):
        again = lq.lq_linear_lowrank_fwd(cfg, packed, lq.lq_quantize_act(cfg, packed, Xd), layer.M)
        assert torch.equal(again.view(torch.int16), ref.view(torch.int16))
