"""The entry point for callers that cannot allocate (lq_rot_step_static: the rotation step with its partial results in
the library's per-GPU array) against lq_rot_step, through the C-ABI: same kernels, so every output is compared bit for
bit, on two calls in a row of which the second is the smaller problem (the array then still holds the first call's
partials), then a few more steps along both trajectories."""
import ctypes as C

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

PARTS = ("Omega", "Mom", "G", "E1", "E2")


def _case(N, K, r, seed):
    rng = np.random.default_rng(seed)
    L = (rng.standard_normal((N, r)) * 0.05).astype(np.float32)
    R = (rng.standard_normal((r, K)) * 0.05).astype(np.float32)
    L[:, 3] *= 8.0
    R[5, :] *= 8.0
    X0 = np.linalg.qr(rng.standard_normal((r, r)))[0].astype(np.float32)
    M0 = (rng.standard_normal((r, r)) * 1e-3).astype(np.float32)
    return L, R, X0, M0


def _d(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _persistent_bytes(N, K, r):
    al = lambda x: (x + 255) // 256 * 256
    return 3 * al(r * r * 4) + al(N * r * 4) + al(r * K * 4)


def _run_pair(lq, cfg, L, R, X0, M0, steps, opt):
    """`steps` steps through each entry point from the same start; returns both sets of outputs and losses."""
    Ld, Rd = _d(L), _d(R)
    out = []
    for static in (False, True):
        if static:   # only the persistent sections: no room for partial results in this blob
            state = torch.full((_persistent_bytes(cfg.N, cfg.K, cfg.rank),), 0xFF, dtype=torch.uint8, device="cuda")
            full = lq.lq_rot_init(cfg, _d(X0), _d(M0))
            state.copy_(full[:state.numel()])
        else:
            state = lq.lq_rot_init(cfg, _d(X0), _d(M0))
        loss = torch.zeros(steps, dtype=torch.float32, device="cuda")
        for t in range(steps):
            (lq.lq_rot_step_static if static else lq.lq_rot_step)(cfg, Ld, Rd, state, loss=loss[t:t + 1], **opt)
        torch.cuda.synchronize()
        if static:   # the views read the leading sections only
            full = torch.zeros(lq.lq_rot_sizes(cfg), dtype=torch.uint8, device="cuda")
            full[:state.numel()] = state
            state = full
        got = {k: v.cpu().numpy() for k, v in lq.lq_rot_unpack(cfg, state, PARTS).items()}
        out.append((got, loss.cpu().numpy()))
    return out


def test_static_scratch_step_equals_the_workspace_step():
    from paper_2604_18117_amd import binding as lq
    opt = dict(lr=0.5, grad_scale=1e3)
    # first call: the larger problem; second call: a smaller one (its partials cover only part of what the first left)
    for (N, K, r, bits, fam, seed) in [(1152, 2240, 64, 6, "int", 1), (320, 256, 32, 8, "int", 2), (256, 384, 32, 8, "mxb", 3)]:
        cfg = lq.make_config(N, K, r, fam, 64 if fam == "int" else 32, bits, 8)
        L, R, X0, M0 = _case(N, K, r, seed)
        (ref, lref), (got, lgot) = _run_pair(lq, cfg, L, R, X0, M0, 1, opt)
        for k in PARTS:
            assert np.array_equal(ref[k], got[k]), f"{k} differs at N={N} K={K} r={r}"
        assert np.array_equal(lref, lgot)
        assert np.isfinite(got["Omega"]).all() and np.isfinite(lgot).all()
    # a few steps along the trajectory
    cfg = lq.make_config(512, 512, 32, "int", 64, 4, 8)
    L, R, X0, M0 = _case(512, 512, 32, 7)
    (ref, lref), (got, lgot) = _run_pair(lq, cfg, L, R, X0, M0, 5, opt)
    for k in PARTS:
        assert np.array_equal(ref[k], got[k]), k
    assert np.array_equal(lref, lgot) and lref[-1] < lref[0]


def test_static_scratch_limits_and_errors():
    from paper_2604_18117_amd import binding as lq
    raw = lq.raw()
    r = 128                                      # partial results of rank 128 exceed the library's array
    cfg = lq.make_config(256, 256, r, "int", 64, 8, 8)
    L, R, X0, M0 = _case(256, 256, r, 5)
    state = lq.lq_rot_init(cfg, _d(X0), _d(M0))
    with pytest.raises(lq.LqError) as e:
        lq.lq_rot_step_static(cfg, _d(L), _d(R), state)
    assert e.value.status == lq.LQ_ERR_UNSUPPORTED
    cfg = lq.make_config(256, 256, 32, "int", 64, 8, 8)
    L, R, X0, M0 = _case(256, 256, 32, 5)
    state = lq.lq_rot_init(cfg, _d(X0), _d(M0))
    opt = lq.lq_cayley(0.5, 0.9, 1e-8, 0.5, 2, 1.0)
    small = _persistent_bytes(256, 256, 32) - 256
    st = raw.lq_rot_step_static(C.byref(cfg), C.c_void_p(_d(L).data_ptr()), C.c_void_p(_d(R).data_ptr()),
                                C.c_void_p(state.data_ptr()), small, C.byref(opt), None, None)
    assert st == lq.LQ_ERR_BUFFER_TOO_SMALL
