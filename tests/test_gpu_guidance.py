"""GPU parity with classifier-free guidance in the heads (conditional and unconditional
vector per row, eps_hat = eps_u + s (eps_c - eps_u)), through the C ABI against the oracle."""
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


def _pairs(wl, n_rows, seed_shift):
    """[n_rows, 2, C]: conditional vectors from the workload, unconditional ones from another block."""
    zq, zp = wl.conds(n_rows)
    uq, up = wl.conds(n_rows, 64 * (1000 + seed_shift))
    return np.stack([zq, uq], 1).astype(np.float32), np.stack([zp, up], 1).astype(np.float32)


@pytest.mark.parametrize("dtype,scale,tol", [("f32", 1.5, H.F32_TOL), ("f32", 3.0, H.F32_TOL), ("bf16", 2.0, H.BF16_TOL)])
def test_guided_whole_path_against_the_oracle(B, dtype, scale, tol):
    wl = S.WORKLOADS["tiny"].with_(gamma=3, gemm_dtype=dtype, out_scale=0.02)
    G, gamma, D, off, seed, tau = 70, 3, 16, 128, wl.seed, 1.0
    tb, db, ds = wl.heads(0.05)
    ocfg = lambda: O.HeadCfg(16, 64, 128, 2, wl.n_steps, eps_skip_gain=wl.eps_skip_gain, cfg_scale=scale)
    oq, op = O.Head(ocfg(), db), O.Head(ocfg(), tb)
    dq, dp = H.device_heads(B, wl, (db, ds, tb), dtype)
    B.csd_set_guidance(dq, True, scale); B.csd_set_guidance(dp, True, scale)
    zq, zp = _pairs(wl, 256, 1)
    zq, zp = zq[:G * gamma], zp[:G * gamma]
    so, _ = O.denoise_lockstep(oq, op, zq, zp, seed=seed, row_offset=off, tau=tau)
    sg = B.csd_denoise_lockstep(dq, dp, _t(zq), _t(zp), G, gamma, seed, off, tau)
    n_g, ell_g, mask_g = B.csd_verify(sg, G, gamma, D, seed, off, tau)
    tok_g, nout_g, trips_g, flags_g = B.csd_resample(sg, n_g, G, gamma, D, seed, off, tau, 256)
    torch.cuda.synchronize()
    mu_p, lv_p, mu_q, lv_q, x0, ls = O.split_summary(so, D)
    g = O.split_summary(sg.cpu().numpy(), D)
    assert H.rel_err(g[4], x0) < tol and H.rel_err(g[0], mu_p) < tol and H.rel_err(g[2], mu_q) < tol
    assert np.max(np.abs(g[5] - ls)) < tol * 10 * max(1.0, np.abs(ls).max())
    if dtype == "f32":
        n_o, ell_o, mask_o, log_u = O.verify(so, G, gamma, seed, off, tau)
        tok_o, nout_o, trips_o, flags_o, rec = O.resample(so, n_o, G, gamma, seed, off, tau, 256)
        exempt, ok = H.decisions_match(mask_g.cpu().numpy(), ell_o, log_u, gamma)
        for gi in range(G):
            if rec[gi] and any(abs(u - a) < 1e-3 * max(a, 1e-6) for a, u in rec[gi]):
                ok[gi] = False
        assert ok.mean() > 0.8 and 0.0 < mask_o.mean() < 1.0
        assert np.array_equal(n_g.cpu().numpy()[ok], n_o[ok]) and np.array_equal(nout_g.cpu().numpy()[ok], nout_o[ok])
        assert H.rel_err(tok_g.cpu().numpy()[ok], tok_o[ok]) < tol
    # the split-phase route with guidance leaves the same bits
    summ = torch.zeros_like(sg)
    zq4 = zq.reshape(G, gamma, 2, -1)
    for i in range(gamma):
        B.csd_denoise_draft(dq, _t(zq4[:, i]), G, gamma, i, seed, off, tau, summ)
    B.csd_denoise_target(dp, dq, _t(zp), G, gamma, seed, off, tau, summ)
    assert torch.equal(summ, sg)
    dq.free(); dp.free()


def test_guidance_special_cases_on_the_device(B):
    """scale 1 equals the unguided head fed the conditional vectors; equal vectors make the
    scale irrelevant; switching guidance off restores the plain head."""
    wl = S.WORKLOADS["mar256"]
    shape = wl.target
    blob = S.bf16_round(S.head_weights(shape, 9, 0.002))
    mk = lambda: B.make_cfg(16, shape.cond_dim, shape.width, shape.n_blocks, 20, B.CSD_BF16, eps_skip_gain=1.0)
    h = B.csd_init_head(mk(), blob)
    R = 300
    zq, zp = wl.conds(320)
    zc, zu = zq[:R], zp[:R]
    plain = B.csd_sample(h, _t(zc), 5, 64)
    B.csd_set_guidance(h, True, 1.0)
    g1 = B.csd_sample(h, _t(np.stack([zc, zu], 1)), 5, 64)
    assert H.rel_err(g1.cpu().numpy(), plain.cpu().numpy()) < 1e-4       # eps_u + 1 * (eps_c - eps_u) rounds in fp32
    B.csd_set_guidance(h, True, 2.5)
    same = B.csd_sample(h, _t(np.stack([zc, zc], 1)), 5, 64)
    assert H.rel_err(same.cpu().numpy(), plain.cpu().numpy()) < 1e-5
    guided = B.csd_sample(h, _t(np.stack([zc, zu], 1)), 5, 64)
    assert H.rel_err(guided.cpu().numpy(), plain.cpu().numpy()) > 1e-3   # guidance does something
    B.csd_set_guidance(h, False)
    assert torch.equal(B.csd_sample(h, _t(zc), 5, 64), plain)
    with pytest.raises(B.CsdError):
        B.csd_set_guidance(h, True, float("nan"))
    h.free()
