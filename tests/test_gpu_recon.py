"""The two solvers of the HIP library (leap_sirt, leap_least_squares_descent) against the solver oracle driven by the
projector oracles, and their stability over a thousand iterations.

Tolerance: every iteration applies A and A^T once (relative error <= 1e-5 each, measured ~3e-7) and the iteration is a
contraction, so errors do not grow geometrically; 30 iterations are held to 1e-4 relative L2 against the double
oracle (measured ~1e-6)."""
import numpy as np
import pytest

from synthetic import config, reduced, standard_volume
from synthetic.configs import CONE_CURVED

pytestmark = pytest.mark.gpu


def rel_l2(got, ref):
    return float(np.linalg.norm(np.asarray(got, np.float64) - ref) / np.linalg.norm(ref))


def setup(cfg, number, orc):
    x_true = standard_volume(number, cfg)
    y = orc.project(cfg, x_true).astype(np.float32)
    A = lambda x: orc.project(cfg, x.astype(np.float32))
    AT = lambda s: orc.backproject(cfg, s.astype(np.float32))
    return x_true, y, A, AT


CASES = [
    ("c2_div8_sf", 2, lambda: reduced(config(2), 8, nviews=24), "sf"),
    ("c3_div8_sf", 3, lambda: reduced(config(3), 8, nviews=30).replace(shift_u=0.123), "sf"),
    ("c3_div8_siddon", 3, lambda: reduced(config(3), 8, nviews=30).replace(shift_u=0.123), "siddon"),
    ("c3_div8_curved_sf", 3, lambda: reduced(config(3), 8, nviews=30).replace(shift_u=0.123, geom=CONE_CURVED), "sf"),
]


@pytest.mark.parametrize("name,number,make,model", CASES, ids=[c[0] for c in CASES])
def test_solvers_match_the_oracle_iteration(oracle_mod, name, number, make, model):
    import torch
    from oracle import recon_oracle as ro
    from paper_2307_05801_amd import Geometry, recon
    cfg = make()
    orc = oracle_mod if model == "sf" else oracle_mod.siddon
    x_true, y, A, AT = setup(cfg, number, orc)
    print(f"[gpu] recon {name}", flush=True)
    geo = Geometry(cfg, model=model)
    yt = torch.from_numpy(y).cuda()
    iters = 30
    x_sirt = recon.sirt(geo, yt, iters).cpu().numpy()
    x_sirt_nn = recon.sirt(geo, yt, iters, relaxation=1.5, nonneg=True).cpu().numpy()
    x_ls = recon.least_squares_descent(geo, yt, iters).cpu().numpy()
    geo.close()
    zero = np.zeros(cfg.vol_shape)
    e1 = rel_l2(x_sirt, ro.sirt(A, AT, y, zero, iters))
    e2 = rel_l2(x_sirt_nn, ro.sirt(A, AT, y, zero, iters, relaxation=1.5, nonneg=True))
    e3 = rel_l2(x_ls, ro.least_squares_descent(A, AT, y, zero, iters))
    print(f"{name}: sirt {e1:.2e}  sirt(nonneg, 1.5) {e2:.2e}  descent {e3:.2e}")
    assert max(e1, e2, e3) <= 1e-4
    # and they reconstruct: the data residual has dropped by an order of magnitude
    assert np.linalg.norm(A(x_ls.astype(np.float64)) - y) < 0.1 * np.linalg.norm(y)


@pytest.mark.parametrize("model", ["sf", "siddon"])
def test_a_thousand_iterations_stay_stable(oracle_mod, model):
    """The reason for a matched pair: the data residual keeps falling (never rises) over 1000 SIRT iterations and 1000
    descent steps, continued in chunks from the previous iterate."""
    import torch
    from paper_2307_05801_amd import Geometry, recon
    cfg = reduced(config(3), 8, nviews=30).replace(shift_u=0.123)
    x_true = standard_volume(3, cfg)
    print(f"[gpu] recon 1000 iterations {model}", flush=True)
    geo = Geometry(cfg, model=model)
    y = geo.project(torch.from_numpy(x_true).cuda())
    for solver in (recon.sirt, recon.least_squares_descent):
        x = torch.zeros(cfg.vol_shape, device="cuda")
        res = [float(torch.linalg.vector_norm(geo.project(x) - y))]
        for _ in range(10):
            x = solver(geo, y, 100, x0=x)
            res.append(float(torch.linalg.vector_norm(geo.project(x) - y)))
        print(f"{model} {solver.__name__}: residual {res[0]:.3e} -> {res[1]:.3e} -> {res[-1]:.3e}")
        assert all(np.isfinite(res)) and all(b <= a * (1 + 1e-6) for a, b in zip(res, res[1:])), res
        assert res[-1] < 0.02 * res[0]
    geo.close()


def test_argument_checks(oracle_mod):
    import torch
    from paper_2307_05801_amd import Geometry, binding as B
    cfg = reduced(config(3), 16, nviews=4)
    geo = Geometry(cfg)
    n = B.leap_recon_workspace_floats(geo.handle)
    assert n >= 2 * cfg.nviews * cfg.nrows * cfg.ncols + 2 * cfg.nx * cfg.ny * cfg.nz
    y = torch.zeros(cfg.sino_shape, device="cuda")
    x = torch.zeros(cfg.vol_shape, device="cuda")
    w = torch.empty(n, device="cuda")
    with pytest.raises(B.LeapError):
        B.leap_sirt(geo.handle, y.data_ptr(), x.data_ptr(), 0, 1)
    with pytest.raises(B.LeapError):
        B.leap_sirt(geo.handle, y.data_ptr(), x.data_ptr(), w.data_ptr(), -1)
    B.leap_sirt(geo.handle, y.data_ptr(), x.data_ptr(), w.data_ptr(), 0)      # zero iterations: x untouched
    torch.cuda.synchronize()
    assert float(x.abs().max()) == 0.0
    geo.close()
