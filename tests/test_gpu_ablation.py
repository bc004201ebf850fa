"""GPU parity of the three path-ratio calculations the paper compares (Table 1: single path,
two paths without alignment, two paths with alignment) and of the token distance of the
alignment ablation (Theorem 1), through the C ABI against the oracle."""
import math

import numpy as np
import pytest
import torch

from oracle import csd_oracle as O
from paper_2411_11925_amd import synth as S
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
MODES = [O.RATIO_ALIGNED, O.RATIO_UNALIGNED, O.RATIO_SINGLE_PATH]


@pytest.fixture(scope="module")
def B():
    from paper_2411_11925_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    assert (binding.CSD_RATIO_ALIGNED, binding.CSD_RATIO_UNALIGNED, binding.CSD_RATIO_SINGLE_PATH) == tuple(MODES)
    assert binding.CSD_STREAM_TRAJ_P == O.STREAM_TRAJ_P
    return binding


def _t(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _dist_tol(dist_o, tok_o, tol, D):
    """|d(dist2)| when each of the two tokens moves by at most tol * (rms of the token row) per
    element: 2 sqrt(dist2) |delta| + |delta|^2 with |delta| <= 2 tol rms sqrt(D)."""
    delta = 2 * tol * np.sqrt((tok_o ** 2).mean(axis=1)) * math.sqrt(D)
    return 2 * np.sqrt(dist_o) * delta + delta ** 2


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("G,gamma,tau,row_offset", [(37, 3, 0.9, 2 ** 32 + 64), (300, 2, 1.0, 0)])
def test_ratio_modes_against_the_oracle_f32(B, mode, G, gamma, tau, row_offset):
    wl = S.WORKLOADS["tiny"].with_(gamma=gamma)
    D, R = 16, G * gamma
    oq, op, blobs = H.oracle_heads(wl, 0.05)
    dq, dp = H.device_heads(B, wl, blobs)
    zq, zp = wl.conds((R + 63) // 64 * 64)
    zq, zp = zq[:R], zp[:R]
    want, dist_o = O.denoise_ablation(oq, op, zq, zp, wl.seed, row_offset, tau, mode)
    got, dist_g = B.csd_denoise_ablation(dq, dp, _t(zq), _t(zp), G, gamma, wl.seed, row_offset, tau, mode)
    got, dist_g = got.cpu().numpy(), dist_g.cpu().numpy()
    mu_p, lv_p, mu_q, lv_q, x0, lr = O.split_summary(want, D)
    g = O.split_summary(got, D)
    for k in (0, 2, 4):
        assert H.rel_err(g[k], (mu_p, lv_p, mu_q, lv_q, x0)[k]) < H.F32_TOL
    assert np.max(np.abs(g[1] - lv_p)) < 1e-4 and np.max(np.abs(g[3] - lv_q)) < 1e-4
    # the sum of 2(T-1) log-densities of magnitude ~D each, in fp32
    assert np.max(np.abs(g[5] - lr)) < H.F32_TOL * 10 * max(1.0, np.abs(lr).max())
    assert np.all(np.abs(dist_g - dist_o) <= _dist_tol(dist_o, x0, H.F32_TOL, D) + 1e-12)
    if mode != O.RATIO_ALIGNED:
        assert np.abs(lr).max() > 1.0                          # the exponents are really there
    # decisions from this ratio: csd_verify applies unchanged
    n_o, ell_o, mask_o, log_u = O.verify(want, G, gamma, wl.seed, row_offset, tau)
    n_g, ell_g, mask_g = B.csd_verify(_t(got), G, gamma, D, wl.seed, row_offset, tau)
    H.decisions_match(mask_g.cpu().numpy(), ell_o, log_u, gamma)
    dq.free(); dp.free()


@pytest.mark.parametrize("dtype,G,gamma", [("f32", 37, 3), ("bf16", 2100, 4)])
def test_aligned_mode_is_the_lockstep_call_bit_for_bit(B, dtype, G, gamma):
    """(the second case is cut into row chunks)"""
    wl = S.WORKLOADS["tiny"].with_(gamma=gamma, gemm_dtype=dtype)
    R = G * gamma
    _, _, blobs = H.oracle_heads(wl, 0.05)
    dq, dp = H.device_heads(B, wl, blobs, dtype)
    zq, zp = wl.conds((R + 63) // 64 * 64)
    zq, zp = _t(zq[:R]), _t(zp[:R])
    lock = B.csd_denoise_lockstep(dq, dp, zq, zp, G, gamma, wl.seed, 128, 0.9)
    abl, _ = B.csd_denoise_ablation(dq, dp, zq, zp, G, gamma, wl.seed, 128, 0.9, B.CSD_RATIO_ALIGNED)
    assert torch.equal(lock, abl)
    dq.free(); dp.free()


@pytest.mark.parametrize("mode", [O.RATIO_UNALIGNED, O.RATIO_SINGLE_PATH])
def test_ratio_modes_at_the_workload_shape_bf16(B, mode):
    """mar256 at 16384 rows (two row chunks per head, the configuration bench.py times) against
    the oracle on sampled 64-row blocks, the oracle fed the bf16-rounded weights.  Tolerances:
    tokens and means as everywhere in the bf16 path.  The ratio before the last step: without
    alignment it is a sum of log-variances and of the noise norms, which the device regenerates
    bit for bit, so it keeps the bf16 tolerance relative to its size; on the single path it is
    built from (x^q_{t-1} - mu^p_t)/sigma^p_t, the difference of the two heads' outputs in units
    of sigma, into which the bf16 rounding of either head enters with the same 1/sigma gain -
    it is compared to 5 % of its spread over the block plus the bf16 tolerance."""
    wl = S.WORKLOADS["mar256"]
    gamma, D, seed, R = wl.gamma, 16, wl.seed, 16384
    G = R // gamma
    oq, op, blobs = H.oracle_heads(wl)
    dq, dp = H.device_heads(B, wl, blobs)
    zq, zp = wl.conds(R)
    got, dist_g = B.csd_denoise_ablation(dq, dp, _t(zq), _t(zp), G, gamma, seed, 0, 1.0, mode)
    torch.cuda.synchronize()
    got, dist_g = got.cpu().numpy(), dist_g.cpu().numpy()
    assert np.all(np.isfinite(got)) and np.all(np.isfinite(dist_g)) and np.all(dist_g >= 0)
    for r0 in (0, 8192 - 64, 8192, 16384 - 64):                 # both sides of the chunk boundary
        zq_s, zp_s = wl.conds(64, r0)
        want, dist_o = O.denoise_ablation(oq, op, zq_s, zp_s, seed, r0, 1.0, mode)
        blk = got[r0:r0 + 64]
        assert H.rel_err(blk[:, 4 * D:5 * D], want[:, 4 * D:5 * D]) < H.BF16_TOL
        assert H.rel_err(blk[:, 0:D], want[:, 0:D]) < H.BF16_TOL
        lr = want[:, -1]
        if mode == O.RATIO_UNALIGNED:
            assert np.max(np.abs(blk[:, -1] - lr)) < H.BF16_TOL * max(1.0, np.abs(lr).max())
        else:
            assert np.max(np.abs(blk[:, -1] - lr)) < 0.05 * lr.std() + H.BF16_TOL
        assert np.all(np.abs(dist_g[r0:r0 + 64] - dist_o) <= _dist_tol(dist_o, want[:, 4 * D:5 * D], H.BF16_TOL, D) + 1e-12)
    dq.free(); dp.free()


def test_structure_of_the_comparison_on_device(B):
    """On the device at scale: alignment raises the acceptance and shrinks the token distance
    (the alignment ablation; Theorem 1 says by 2 tr sqrt(Sigma^q Sigma^p) per step)."""
    wl = S.WORKLOADS["mar256"]
    gamma, D, R = wl.gamma, 16, 4096
    G = R // gamma
    _, _, blobs = H.oracle_heads(wl)
    dq, dp = H.device_heads(B, wl, blobs)
    zq, zp = wl.conds(R)
    acc, dist = {}, {}
    for mode in MODES:
        summ, d2 = B.csd_denoise_ablation(dq, dp, _t(zq), _t(zp), G, gamma, wl.seed, 0, 1.0, mode)
        _, _, mask = B.csd_verify(summ, G, gamma, D, wl.seed)
        acc[mode], dist[mode] = float(mask.float().mean()), float(d2.mean())
    assert acc[O.RATIO_ALIGNED] > 0.2 and acc[O.RATIO_ALIGNED] > 10 * acc[O.RATIO_UNALIGNED]
    assert dist[O.RATIO_ALIGNED] < 0.01 * dist[O.RATIO_UNALIGNED]
    dq.free(); dp.free()


def test_ablation_bad_calls(B):
    wl = S.WORKLOADS["tiny"]
    _, _, blobs = H.oracle_heads(wl)
    dq, dp = H.device_heads(B, wl, blobs)
    z = torch.zeros((8, 64), device=DEV)
    with pytest.raises(B.CsdError):
        B.csd_denoise_ablation(dq, dp, z, z, 4, 2, 1, 0, 1.0, 3)                      # unknown mode
    with pytest.raises(B.CsdError) as e:
        B.csd_denoise_ablation(dq, dp, z, z, 4, 2, 1, 0, 1.0, B.CSD_RATIO_SINGLE_PATH,
                               workspace=torch.empty(B.csd_workspace_bytes(dq, dp, 8), dtype=torch.uint8, device=DEV))
    assert "workspace" in str(e.value)                                                # the stored path does not fit
    assert B.csd_ablation_workspace_bytes(dq, dp, 8, B.CSD_RATIO_SINGLE_PATH) > B.csd_ablation_workspace_bytes(dq, dp, 8, 0)
    s, d = B.csd_denoise_ablation(dq, dp, torch.zeros((0, 64), device=DEV), torch.zeros((0, 64), device=DEV), 0, 2, 1, 0, 1.0, 1)
    assert s.shape[0] == 0 and d.numel() == 0
    dq.free(); dp.free()


@pytest.mark.parametrize("mode", [O.RATIO_UNALIGNED, O.RATIO_SINGLE_PATH])
def test_ratio_modes_with_guidance_and_ddim_f32(B, mode):
    """The comparison modes on heads that use the DDIM sampler and classifier-free guidance (two
    head rows per trajectory row; the stored path and the own final sample have one row each)."""
    wl = S.WORKLOADS["tiny"].with_(gamma=2, out_scale=0.02)
    G, gamma, D, off, seed, tau, scale, eta = 45, 2, 16, 64, wl.seed, 0.9, 1.5, 0.7
    R = G * gamma
    tb, db, ds = wl.heads(0.05)
    ocfg = lambda: O.HeadCfg(16, 64, 128, 2, wl.n_steps, eps_skip_gain=wl.eps_skip_gain, cfg_scale=scale,
                             sampler="ddim", ddim_eta=eta)
    oq, op = O.Head(ocfg(), db), O.Head(ocfg(), tb)
    dq, dp = H.device_heads(B, wl, (db, ds, tb), "f32", ddim_eta=eta)
    B.csd_set_guidance(dq, True, scale); B.csd_set_guidance(dp, True, scale)
    zq, zp = wl.conds(128)
    uq, up = wl.conds(128, 64 * 2000)
    zq2 = np.stack([zq, uq], 1).astype(np.float32)[:R]
    zp2 = np.stack([zp, up], 1).astype(np.float32)[:R]
    want, dist_o = O.denoise_ablation(oq, op, zq2, zp2, seed, off, tau, mode)
    got, dist_g = B.csd_denoise_ablation(dq, dp, _t(zq2), _t(zp2), G, gamma, seed, off, tau, mode)
    got, dist_g = got.cpu().numpy(), dist_g.cpu().numpy()
    assert H.rel_err(got[:, 4 * D:5 * D], want[:, 4 * D:5 * D]) < H.F32_TOL
    assert H.rel_err(got[:, 0:D], want[:, 0:D]) < H.F32_TOL
    lr = want[:, -1]
    assert np.max(np.abs(got[:, -1] - lr)) < H.F32_TOL * 10 * max(1.0, np.abs(lr).max())
    assert np.all(np.abs(dist_g - dist_o) <= _dist_tol(dist_o, want[:, 4 * D:5 * D], H.F32_TOL, D) + 1e-12)
    dq.free(); dp.free()
