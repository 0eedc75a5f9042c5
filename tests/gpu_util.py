"""Helpers of the GPU parity tests: run one layer through the HIP library and the CPU oracle."""
from dataclasses import dataclass

import numpy as np
import torch

from paper_2604_18117_amd import workloads as wl


to_dev_x = wl.to_dev_x
bf16_to_bits = wl.bf16_to_bits


@dataclass
class GpuRun:
    cfg: object
    packed: torch.Tensor
    act: torch.Tensor
    Y: torch.Tensor
    wv: object = None
    av: object = None
    adbg: object = None
    fdbg: object = None


def run_gpu(layer, X, W, L, R, debug=True, debug_acc=True, gamma=None):
    """gamma: smoothing vector (K fp32 values): the layer is packed with fused smoothing and the activation kernel
    divides X by it."""
    from paper_2604_18117_amd import binding as lq
    cfg = lq.config_for_layer(layer, smooth=gamma is not None)
    Wd = torch.from_numpy(W).cuda()
    Ld = torch.from_numpy(L).cuda() if layer.r else None
    Rd = torch.from_numpy(R).cuda() if layer.r else None
    Xd = to_dev_x(X, layer.x_dtype)
    # both blobs start as 0xFF bytes (NaN patterns as floats): a kernel that reads a section nobody wrote (e.g. branch
    # scales at rank 0) then shows up as NaN instead of passing on memory that happened to be zero
    packed = lq.lq_pack_weights(cfg, Wd, Ld, Rd, packed=torch.full((lq.lq_packed_sizes(cfg),), 0xFF, dtype=torch.uint8, device="cuda"))
    if gamma is not None:
        lq.lq_set_smoothing(cfg, packed, torch.from_numpy(np.ascontiguousarray(gamma, np.float32)).cuda())
    M = X.shape[0]
    if debug and layer.family in ("mx", "mxb", "mxi"):
        debug_acc = False
    # the output starts as a bit pattern the path never produces (a NaN): a tile the grid skipped would keep it
    Y0 = torch.full((M, layer.N), -1, dtype=torch.int16, device="cuda").view(torch.bfloat16)
    act0 = torch.full((lq.lq_act_sizes(cfg, M),), 0xFF, dtype=torch.uint8, device="cuda")
    if debug:
        act, adbg = lq.lq_quantize_act(cfg, packed, Xd, act=act0, debug=True)
        Y, fdbg = lq.lq_linear_lowrank_fwd(cfg, packed, act, M, Y=Y0, debug=True, debug_acc=debug_acc)
        out = GpuRun(cfg, packed, act, Y, lq.lq_unpack_weights(cfg, packed), lq.lq_unpack_act(cfg, act, M),
                     adbg, fdbg)
    else:
        act = lq.lq_quantize_act(cfg, packed, Xd, act=act0)
        Y = lq.lq_linear_lowrank_fwd(cfg, packed, act, M, Y=Y0)
        out = GpuRun(cfg, packed, act, Y)
    torch.cuda.synchronize()
    assert not bool((Y.view(torch.int16) == -1).any()), "an output element was never written"
    return out


def run_oracle_int(oracle, layer, X, W, L, R, want_acc=True):
    pk = oracle.pack_int(W, L if layer.r else None, R if layer.r else None, layer.g, layer.br_w_bits,
                         sint4_blocks=layer.a_group == 64)
    act = oracle.quantize_act_int(X, pk, layer.br_a_bits)
    out = oracle.fwd_int(pk, act, want_acc=want_acc)
    return pk, act, out


def n(t):
    return t.cpu().numpy()
