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
    # ... followed by guard rows of the same pattern: the forward drops rows past M in hardware (range-checked buffer
    # stores) and must leave them alone
    GUARD = 40
    Yall = torch.full((M + GUARD, layer.N), -1, dtype=torch.int16, device="cuda").view(torch.bfloat16)
    Y0 = Yall[:M]
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
    assert bool((Yall[M:].view(torch.int16) == -1).all()), "the forward wrote past the last token row"
    return out


def run_oracle_int(oracle, layer, X, W, L, R, want_acc=True):
    pk = oracle.pack_int(W, L if layer.r else None, R if layer.r else None, layer.g, layer.br_w_bits,
                         sint4_blocks=layer.a_group == 64)
    act = oracle.quantize_act_int(X, pk, layer.br_a_bits)
    out = oracle.fwd_int(pk, act, want_acc=want_acc)
    return pk, act, out


def n(t):
    return t.cpu().numpy()


def check_bf16_against_oracle(oracle, Yb, y_gpu, out, bound, what=""):
    """The bf16 output against an oracle result `out` whose fp32 value the kernel's own fp32 value `y_gpu` has already
    been shown to match within `bound` (fp32 accumulation in the matrix core against the oracle's fp64 sum).
    Rule (a reading of "max relative error <= 2e-3" for a bf16 output, whose own rounding step is 2^-8 .. 2^-7 relative):
    the stored bits are the nearest-even rounding of the kernel's fp32 value; where they differ from the oracle's bits
    (a "flip") the two fp32 values straddle a rounding boundary, so the difference is exactly one bf16 step (unless the
    result cancels to less than the accumulation bound itself); everything else is within 2e-3 relative.  The number of flips is reported, and on outputs of at least 1000 elements their rate
    must stay below 2e-3 (measured: ~3e-5; a kernel that reorders sums grossly would show up here first)."""
    want = ((y_gpu.view(np.uint32) + 0x7FFF + ((y_gpu.view(np.uint32) >> 16) & 1)) >> 16).astype(np.uint16)
    assert np.array_equal(Yb, want), "Y is not bf16_rne(y32)"
    Yf = oracle.bf16_bits_to_f32(Yb).astype(np.float64)
    Yo = oracle.bf16_bits_to_f32(out.Y).astype(np.float64)
    tau = 1e-3 * np.sqrt(np.mean(out.y32.astype(np.float64) ** 2)) + 1e-300
    rel = np.abs(Yf - Yo) / np.maximum(np.abs(out.y32), tau)
    flips = Yb != out.Y
    assert np.all(rel[~flips] <= 2e-3)
    if flips.any():
        yg, yo, bf = y_gpu[flips].astype(np.float64), out.y32[flips].astype(np.float64), bound[flips]
        assert np.all(np.abs(yg - yo) <= bf)
        # two roundings (half a bf16 step each, at most 2^-8 relative) of values within the bound of each other
        assert np.all(np.abs(Yf[flips] - Yo[flips]) <= bf + 2.0 ** -8 * (np.abs(yg) + np.abs(yo)))
        # where the bound is far below a bf16 step the difference is exactly one step of the grid (results that cancel
        # to almost nothing, e.g. an all-zero channel of W whose main product and branch cancel, sit on a finer grid
        # than the bound and may land several steps apart)
        a, b = Yb[flips].astype(np.int64), out.Y[flips].astype(np.int64)
        same_sign = (a >> 15) == (b >> 15)
        one_step = np.where(same_sign, np.abs(a - b) == 1, ((a & 0x7FFF) + (b & 0x7FFF)) <= 1)
        fine = bf <= 2.0 ** -10 * np.abs(yo)
        assert np.all(one_step[fine]), "a bf16 difference of more than one step"
    if flips.size >= 1000:
        assert flips.mean() <= 2e-3, f"bf16 flip rate {flips.mean()}"
    if flips.any():
        print(f"[parity{what}] bf16 flips against the oracle: {int(flips.sum())} of {flips.size}")


def check_end_to_end(oracle, Yb, y_gpu, out_alone, bound_acc, D, Labs, what=""):
    """The kernel's result against the oracle run ALONE (its own re-quantised intermediate), end to end.
    bound_acc: the fp32-accumulation bound on y; D (M x r): |dequantised intermediate of the GPU - of the oracle|,
    itself already checked against its derived bound (half a code step on either side plus the accumulation bound
    of T); Labs (N x r): |dequantised L|.  Then |y_gpu - y32_oracle| <= bound_acc + sum_j D[m,j] |L[n,j]|, and the
    stored bf16 value is within half a bf16 step (2^-8 relative) of y_gpu."""
    tot = bound_acc + D @ Labs.T
    err = np.abs(y_gpu.astype(np.float64) - out_alone.y32.astype(np.float64))
    assert np.all(err <= tot), f"end-to-end y32 max excess {np.max(err / tot)}"
    Yf = oracle.bf16_bits_to_f32(Yb).astype(np.float64)
    e2 = np.abs(Yf - out_alone.y32.astype(np.float64))
    assert np.all(e2 <= tot + 2.0 ** -8 * np.abs(y_gpu.astype(np.float64)) + 1e-300), "end-to-end bf16 output"
    tau = 1e-3 * np.sqrt(np.mean(out_alone.y32.astype(np.float64) ** 2)) + 1e-300
    rel = e2 / np.maximum(np.abs(out_alone.y32), tau)
    print(f"[parity{what}] end to end vs the oracle alone: max |Y - y32| / max(|y32|, tau) = {rel.max():.3e}, "
          f"share above 2e-3: {np.mean(rel > 2e-3):.2e} (bf16's own rounding step is 3.9e-3 .. 7.8e-3)")
