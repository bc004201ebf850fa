"""GPU parity with DDIM as the heads' sampler (appendix on other diffusion samplers): the
whole path against the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import csd_oracle as O
from paper_2411_11925_amd import synth as S
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def B():
    from paper_2411_11925_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return binding


def _t(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


@pytest.mark.parametrize("dtype,eta,tau,tol", [("f32", 1.0, 1.0, H.F32_TOL), ("f32", 0.5, 0.9, H.F32_TOL),
                                               ("bf16", 0.8, 1.0, H.BF16_TOL)])
def test_ddim_whole_path_against_the_oracle(B, dtype, eta, tau, tol):
    wl = S.WORKLOADS["tiny"].with_(gamma=3, gemm_dtype=dtype, out_scale=0.02)
    G, gamma, D, off, seed = 80, 3, 16, 2 ** 32 + 128, wl.seed
    oq, op, blobs = H.oracle_heads(wl, 0.05, ddim_eta=eta)
    dq, dp = H.device_heads(B, wl, blobs, dtype, ddim_eta=eta)
    zq, zp = wl.conds(256)
    zq, zp = zq[:G * gamma], zp[:G * gamma]
    so, _ = O.denoise_lockstep(oq, op, zq, zp, seed=seed, row_offset=off, tau=tau)
    sg = B.csd_denoise_lockstep(dq, dp, _t(zq), _t(zp), G, gamma, seed, off, tau)
    n_g, ell_g, mask_g = B.csd_verify(sg, G, gamma, D, seed, off, tau)
    tok_g, nout_g, trips_g, flags_g = B.csd_resample(sg, n_g, G, gamma, D, seed, off, tau, 256)
    torch.cuda.synchronize()
    mu_p, lv_p, mu_q, lv_q, x0, ls = O.split_summary(so, D)
    g = O.split_summary(sg.cpu().numpy(), D)
    assert H.rel_err(g[4], x0) < tol and H.rel_err(g[0], mu_p) < tol and H.rel_err(g[2], mu_q) < tol
    # fixed, equal variances: log sigma^2 is the schedule's and the Sigma factor is exactly 1
    assert np.max(np.abs(g[1] - lv_p)) < 1e-5 and np.max(np.abs(g[3] - lv_q)) < 1e-5
    assert np.all(ls == 0.0) and np.all(g[5] == 0.0)
    if dtype == "f32":
        n_o, ell_o, mask_o, log_u = O.verify(so, G, gamma, seed, off, tau)
        tok_o, nout_o, trips_o, flags_o, rec = O.resample(so, n_o, G, gamma, seed, off, tau, 256)
        exempt, ok = H.decisions_match(mask_g.cpu().numpy(), ell_o, log_u, gamma)
        for gi in range(G):
            if rec[gi] and any(abs(u - a) < 1e-3 * max(a, 1e-6) for a, u in rec[gi]):
                ok[gi] = False
        assert ok.mean() > 0.8 and 0.0 < mask_o.mean() < 1.0          # both outcomes occur
        assert np.array_equal(n_g.cpu().numpy()[ok], n_o[ok]) and np.array_equal(nout_g.cpu().numpy()[ok], nout_o[ok])
        assert np.array_equal(trips_g.cpu().numpy()[ok], trips_o[ok])
        assert H.rel_err(tok_g.cpu().numpy()[ok], tok_o[ok]) < tol
    dq.free(); dp.free()


def test_ddim_eta_one_is_the_ddpm_posterior_on_the_device(B):
    """A head whose v output is pinned to -1 (zero v rows in the output layer, bias -1) takes
    the DDPM path's variance to its lower end beta~_t, which is DDIM with eta = 1: the two
    samplers must then walk the same trajectory."""
    wl = S.WORKLOADS["tiny"]
    shape = wl.target
    blob = S.head_weights(shape, 5, 0.05, 0.05)
    off, lay = 0, {}
    for name, shp in S.param_layout(shape):
        lay[name] = (off, shp); off += int(np.prod(shp))
    o, shp = lay["out.w"]; w = blob[o:o + shp[0] * shp[1]].reshape(shp); w[16:] = 0.0
    o, shp = lay["out.b"]; blob[o + 16:o + 32] = -1.0
    T = wl.n_steps
    h_ddpm = B.csd_init_head(B.make_cfg(16, 64, 128, 2, T, B.CSD_F32, eps_skip_gain=1.0), blob)
    h_ddim = B.csd_init_head(B.make_cfg(16, 64, 128, 2, T, B.CSD_F32, eps_skip_gain=1.0, ddim_eta=1.0), blob)
    z, _ = wl.conds(64)
    a = B.csd_sample(h_ddpm, _t(z), 3, 10).cpu().numpy()
    b = B.csd_sample(h_ddim, _t(z), 3, 10).cpu().numpy()
    assert H.rel_err(b, a) < 1e-4
    with pytest.raises(B.CsdError):
        B.csd_init_head(B.make_cfg(16, 64, 128, 2, T, B.CSD_F32, ddim_eta=0.0), blob)     # eta must be > 0
    h_ddpm.free(); h_ddim.free()
