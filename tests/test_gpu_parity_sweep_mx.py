"""Seeded sweeps over small shapes around the tile edges for the block-scaled families (MX, MXB, MXI), each compared by
its family's own parity routine (codes and scale bytes bit-exact, floating-point results to the family's bound)."""
import numpy as np
import pytest

from paper_2604_18117_amd import workloads as wl
from tests.smoothing import smoothing_vector
from tests import test_gpu_parity_mx as t_mx
from tests import test_gpu_parity_mxb as t_mxb
from tests import test_gpu_parity_mxi as t_mxi

pytestmark = pytest.mark.gpu

EDGE_M = [1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 257]


@pytest.mark.parametrize("family", ["mx", "mxb8", "mxb6", "mxi8", "mxi4"])
def test_seeded_shape_sweep(oracle, family):
    rng = np.random.default_rng(sum(map(ord, family)))
    for it in range(20):
        M = int(rng.choice(EDGE_M))
        K = 64 * int(rng.integers(1, 12))        # odd multiples of 64 included (padded to whole 128-stages inside the blobs)
        N = 64 * int(rng.integers(1, 10)) if it % 8 else 64 * int(rng.integers(10, 40))
        xd = "bf16" if rng.integers(0, 2) else "f32"
        if family == "mx":
            r = int(rng.choice([0, 16, 32, 64, 128]))
            layer, cmp = wl.Layer("t", M, K, N, r, "mx", 32, 8, 8, xd, seed=200 + it), t_mx._compare
        elif family.startswith("mxb"):
            r, e = int(rng.choice([0, 32, 64, 96, 128])), int(family[-1])
            layer, cmp = wl.Layer("t", M, K, N, r, "mxb", 32, e, e, xd, seed=200 + it), t_mxb._compare
        else:
            r, bw = int(rng.choice([0, 32, 64, 96, 128])), int(family[-1])
            layer, cmp = wl.Layer("t", M, K, N, r, "mxi", 32, bw, 8, xd, seed=200 + it), t_mxi._compare
        X, W, L, R = wl.make_inputs(layer)
        try:
            cmp(oracle, layer, X, W, L, R)
        except AssertionError as e:
            raise AssertionError(f"{family}: M={M} K={K} N={N} r={r} {xd}: {e}") from e


@pytest.mark.parametrize("family", ["mx", "mxb8", "mxb6", "mxi8", "mxi4"])
@pytest.mark.parametrize("M,K,N,r,xd", [(200, 1152, 320, 32, "bf16"), (77, 2304, 64, 64, "f32"), (33, 256, 64, 0, "bf16")])
def test_fused_smoothing(oracle, family, M, K, N, r, xd):
    """Activation smoothing (Section 3.4; App. A.1) fused into the MX families' activation kernels: the GPU gets the raw X
    and the smoothing vector, the oracle quantises the smoothed input; same bars as without smoothing."""
    base = wl.shrink(wl.LAYERS["c2_qkv"], M=M, K=K, N=N, r=r)           # outlier channels for the vector to tame
    kw = dict(base.__dict__, x_dtype=xd, seed=M + K, g=32)
    if family == "mx":
        layer, cmp = wl.Layer(**dict(kw, family="mx", br_w_bits=8, br_a_bits=8)), t_mx._compare
    elif family.startswith("mxb"):
        e = int(family[-1])
        layer, cmp = wl.Layer(**dict(kw, family="mxb", br_w_bits=e, br_a_bits=e)), t_mxb._compare
    else:
        layer, cmp = wl.Layer(**dict(kw, family="mxi", br_w_bits=int(family[-1]), br_a_bits=8)), t_mxi._compare
    X, W, L, R = wl.make_inputs(layer)
    gamma = smoothing_vector(X, W)
    Ws = (W.astype(np.float64) * gamma).astype(np.float32)            # the caller folds gamma into W before packing
    cmp(oracle, layer, X, Ws, L, R, gamma=gamma)
    # the vector did change the codes: the unsmoothed run differs
    from tests.gpu_util import n, run_gpu
    a = run_gpu(layer, X, Ws, L, R, debug=True, debug_acc=False)
    b = run_gpu(layer, X, Ws, L, R, debug=True, debug_acc=False, gamma=gamma)
    assert not np.array_equal(n(a.av.xq), n(b.av.xq))
