"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on
identical seeded inputs.  fp32 path: tokens within 1e-4 relative, decisions
bit-exact outside |log u - log ratio| < 1e-3."""
import math

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


# ------------------------------------------------------------------ RNG ----
@pytest.mark.parametrize("seed,row_offset,slot,stream", [
    (0, 0, 0, 0), (0x5EED0001, 0, 10, 0), (2 ** 63 + 12345, 2 ** 32 - 100, 99, 2),
    (77, 2 ** 40 + 3, 65535, 3), (1, 5, 1023, 0)])
def test_rng_bit_identity(B, seed, row_offset, slot, stream):
    n = 20000
    got = B.csd_rng_normals(seed, row_offset, n, slot, stream, 16).cpu().numpy()
    rows = (np.arange(n, dtype=np.uint64) + np.uint64(row_offset))
    want = O.normals(seed, rows, slot, stream, 16).astype(np.float32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    gu = B.csd_rng_uniforms(seed, row_offset, n, slot, stream).cpu().numpy()
    wu = O.uniforms(seed, rows, slot, stream).astype(np.float32)
    assert np.array_equal(gu.view(np.uint32), wu.view(np.uint32))
    for cols in (4, 8):
        g = B.csd_rng_normals(seed, row_offset, 64, slot, stream, cols).cpu().numpy()
        assert np.array_equal(g, want[:64, :cols])


# ----------------------------------------------------- head forward (fp32) ----
@pytest.mark.parametrize("shape,T,R,gain", [
    (S.HeadShape(16, 64, 128, 2), 10, 131, 1.0),
    (S.HeadShape(8, 40, 192, 3), 7, 77, 0.0),
    (S.HeadShape(4, 8, 64, 1), 3, 5, 0.5),
    (S.HeadShape(16, 768, 1024, 6), 100, 70, 1.0)])
def test_head_eval_f32(B, shape, T, R, gain):
    blob = S.head_weights(shape, 21, out_scale=0.8, bias_std=0.2)
    oh = O.Head(O.HeadCfg(shape.token_dim, shape.cond_dim, shape.width, shape.n_blocks, T, eps_skip_gain=gain), blob)
    dh = B.csd_init_head(B.make_cfg(shape.token_dim, shape.cond_dim, shape.width, shape.n_blocks, T,
                                    B.CSD_F32, eps_skip_gain=gain), blob)
    rng = np.random.default_rng(5)
    x = rng.normal(size=(R, shape.token_dim)).astype(np.float32) * 1.5
    z = rng.normal(size=(R, shape.cond_dim)).astype(np.float32)
    for t in sorted({1, 2, T}):
        got = B.csd_head_eval(dh, _t(x), _t(z), t).cpu().numpy()
        eh, v = oh.forward(x.astype(np.float64), t, oh.cond_embed(z.astype(np.float64)))
        assert H.rel_err(got, np.concatenate([eh, v], 1)) < H.F32_TOL
    dh.free()


# ------------------------------------------------- verify, given summaries ----
def _oracle_run(wl, n_groups, bias_std=0.05, tau=1.0, row_offset=0):
    drf, tgt, blobs = H.oracle_heads(wl, bias_std)
    R = n_groups * wl.gamma
    zq, zp = wl.conds(((R + 63) // 64) * 64)
    zq, zp = zq[:R], zp[:R]
    summ, _ = O.denoise_lockstep(drf, tgt, zq, zp, wl.seed, row_offset=row_offset, tau=tau)
    return summ, zq, zp, blobs


@pytest.mark.parametrize("gamma,tau,row_offset", [(2, 1.0, 0), (4, 0.9, 2 ** 33), (5, 1.0, 64), (64, 1.0, 0), (1, 1.2, 0)])
def test_verify_and_resample_given_oracle_summary(B, gamma, tau, row_offset):
    wl = S.WORKLOADS["tiny"].with_(gamma=gamma)
    G = 600 // gamma + 1
    summ, _, _, _ = _oracle_run(wl, G, tau=tau, row_offset=row_offset)
    s32 = summ.astype(np.float32)
    D, seed = 16, wl.seed
    # the oracle sees exactly the fp32 summary the device gets
    n_o, ell_o, mask_o, log_u = O.verify(s32.astype(np.float64), G, gamma, seed, row_offset, tau)
    n_g, ell_g, mask_g = B.csd_verify(_t(s32), G, gamma, D, seed, row_offset, tau)
    n_g, ell_g, mask_g = n_g.cpu().numpy(), ell_g.cpu().numpy(), mask_g.cpu().numpy()
    fin = np.isfinite(ell_o)
    assert np.max(np.abs(ell_g[fin] - ell_o[fin]) / np.maximum(1.0, np.abs(ell_o[fin]))) < 1e-4
    exempt, ok = H.decisions_match(mask_g, ell_o, log_u, gamma)
    assert np.array_equal(n_g[ok], n_o[ok]) and ok.mean() > 0.9
    assert 0.05 < mask_o.mean() < 0.95 or gamma == 64
    # resample from the oracle's n so that both sides work on the same rows
    tok_o, nout_o, trips_o, flags_o, rec = O.resample(s32.astype(np.float64), n_o, G, gamma, seed, row_offset, tau, 64)
    tok_g, nout_g, trips_g, flags_g = B.csd_resample(_t(s32), _t(n_o), G, gamma, D, seed, row_offset, tau, 64)
    tok_g, nout_g, trips_g, flags_g = (a.cpu().numpy() for a in (tok_g, nout_g, trips_g, flags_g))
    assert np.array_equal(nout_g, nout_o)
    # a group is comparable unless one of its trials sat within the band of its threshold
    cmp_ = np.ones(G, dtype=bool)
    for g in range(G):
        if rec[g]:
            cmp_[g] = not any(abs(u - a) < 1e-3 * max(a, 1e-6) for a, u in rec[g])
    assert cmp_.mean() > 0.9
    assert np.array_equal(trips_g[cmp_], trips_o[cmp_]) and np.array_equal(flags_g[cmp_], flags_o[cmp_].astype(np.int32))
    assert H.rel_err(tok_g[cmp_], tok_o[cmp_]) < 1e-5
    assert (trips_o > 1).any() or gamma == 64


def test_resample_cap_and_nan_flags(B):
    D, G, gamma = 16, 9, 3
    s = np.zeros((G * gamma, 5 * D + 1), dtype=np.float32)
    s[:, 4 * D:5 * D] = 1.0
    s[:, -1] = -0.5                      # p = q and Sigma < 1: alpha_s = 0 everywhere, never accepts
    n_acc = np.array([0, 1, 2, 3, 0, 1, 2, 3, 0], dtype=np.int32)
    s[8 * gamma, 2 * D] = np.nan         # group 8: NaN in mu_q of its first rejected row
    for cap in (1, 3, 4, 5, 8, 9):
        tok, n_out, trips, flags = (a.cpu().numpy() for a in B.csd_resample(_t(s), _t(n_acc), G, gamma, D, 3, 0, 1.0, cap))
        want_tok, want_n, want_trips, want_flags, _ = O.resample(s.astype(np.float64), n_acc, G, gamma, 3, 0, 1.0, cap)
        assert np.array_equal(n_out, want_n) and np.array_equal(trips, want_trips)
        assert np.array_equal(flags, want_flags.astype(np.int32))
        assert np.all(flags[n_acc < gamma] & B.CSD_FLAG_CAP) and flags[8] & B.CSD_FLAG_NONFINITE
        assert H.rel_err(tok[:8], want_tok[:8]) < 1e-5


# --------------------------------------------------------- end to end, fp32 ----
def _end_to_end(B, wl, n_groups, tol, bias_std=0.05, tau=1.0, row_offset=0, dtype=None, check_decisions=True):
    summ_o, zq, zp, blobs = _oracle_run(wl, n_groups, bias_std, tau, row_offset)
    dq, dp = H.device_heads(B, wl, blobs, dtype)
    G, gamma, D, seed = n_groups, wl.gamma, 16, wl.seed
    summ_g = B.csd_denoise_lockstep(dq, dp, _t(zq), _t(zp), G, gamma, seed, row_offset, tau)
    n_g, ell_g, mask_g = B.csd_verify(summ_g, G, gamma, D, seed, row_offset, tau)
    tok_g, nout_g, trips_g, flags_g = B.csd_resample(summ_g, n_g, G, gamma, D, seed, row_offset, tau, 256)
    torch.cuda.synchronize()
    sg = summ_g.cpu().numpy()
    mu_p, lv_p, mu_q, lv_q, x0, ls = O.split_summary(summ_o, D)
    gmu_p, glv_p, gmu_q, glv_q, gx0, gls = O.split_summary(sg, D)
    assert H.rel_err(gx0, x0) < tol, "draft tokens"
    assert H.rel_err(gmu_p, mu_p) < tol and H.rel_err(gmu_q, mu_q) < tol
    assert np.max(np.abs(glv_p - lv_p)) < tol * 10 and np.max(np.abs(glv_q - lv_q)) < tol * 10
    assert np.max(np.abs(gls - ls)) < tol * 10 * max(1.0, np.abs(ls).max())
    n_o, ell_o, mask_o, log_u = O.verify(summ_o, G, gamma, seed, row_offset, tau)
    res = dict(accept=float(mask_o.mean()), agree=float((mask_g.cpu().numpy() == mask_o).mean()))
    if check_decisions:
        exempt, ok = H.decisions_match(mask_g.cpu().numpy(), ell_o, log_u, gamma)
        assert np.array_equal(n_g.cpu().numpy()[ok], n_o[ok])
        tok_o, nout_o, trips_o, flags_o, rec = O.resample(summ_o, n_o, G, gamma, seed, row_offset, tau, 256)
        for g in range(G):
            if rec[g] and any(abs(u - a) < 1e-3 * max(a, 1e-6) for a, u in rec[g]):
                ok[g] = False
        assert ok.mean() > 0.8
        assert np.array_equal(nout_g.cpu().numpy()[ok], nout_o[ok])
        assert np.array_equal(trips_g.cpu().numpy()[ok], trips_o[ok])
        assert H.rel_err(tok_g.cpu().numpy()[ok], tok_o[ok]) < tol
        res["groups_compared"] = float(ok.mean())
    dq.free(); dp.free()
    return res


@pytest.mark.parametrize("n_groups,gamma,tau,row_offset", [(1, 2, 1.0, 0), (150, 2, 1.0, 0), (67, 3, 0.9, 2 ** 32 + 64)])
def test_tiny_workload_end_to_end_f32(B, n_groups, gamma, tau, row_offset):
    wl = S.WORKLOADS["tiny"].with_(gamma=gamma)
    res = _end_to_end(B, wl, n_groups, H.F32_TOL, tau=tau, row_offset=row_offset)
    if n_groups > 50:
        assert 0.1 < res["accept"] < 0.9


def test_plain_eps_prediction_end_to_end_f32(B):
    """No input-output skip: trajectories grow by 1/sqrt(abar_T); tokens still match
    to 1e-4 relative (decisions are not compared: log-ratios are ~ -1e5)."""
    wl = S.WORKLOADS["tiny"].with_(eps_skip_gain=0.0, out_scale=1.0)
    _end_to_end(B, wl, 64, H.F32_TOL, check_decisions=False)


def test_identical_heads_accept_everything(B):
    wl = S.WORKLOADS["tiny"].with_(gamma=4)
    tb, _, _ = wl.heads(0.05)
    cfg = lambda: B.make_cfg(16, 64, 128, 2, wl.n_steps, B.CSD_F32, eps_skip_gain=1.0)
    hq, hp = B.csd_init_head(cfg(), tb), B.csd_init_head(cfg(), tb)
    zq, _ = wl.conds(128)
    z = _t(zq[:80])
    summ = B.csd_denoise_lockstep(hq, hp, z, z, 20, 4, 9)
    n, ell, mask = B.csd_verify(summ, 20, 4, 16, 9)
    assert torch.all(ell == 0) and torch.all(mask == 1) and torch.all(n == 4)
    tok, n_out, trips, flags = B.csd_resample(summ, n, 20, 4, 16, 9)
    assert torch.all(n_out == 4) and torch.all(trips == 0) and torch.all(flags == 0)
    assert torch.equal(tok[:, :4].reshape(80, 16), summ[:, 64:80]) and torch.all(tok[:, 4] == 0)
    hq.free(); hp.free()


def test_split_calls_reproduce_one_call(B):
    """Rows are keyed by the global row index: two half-size calls equal one call."""
    wl = S.WORKLOADS["tiny"].with_(gamma=2)
    _, _, blobs = H.oracle_heads(wl, 0.05)
    dq, dp = H.device_heads(B, wl, blobs)
    zq, zp = wl.conds(128)
    full = B.csd_denoise_lockstep(dq, dp, _t(zq), _t(zp), 64, 2, wl.seed)
    a = B.csd_denoise_lockstep(dq, dp, _t(zq[:64]), _t(zp[:64]), 32, 2, wl.seed, 0)
    b = B.csd_denoise_lockstep(dq, dp, _t(zq[64:]), _t(zp[64:]), 32, 2, wl.seed, 64)
    assert torch.equal(full, torch.cat([a, b]))
    again = B.csd_denoise_lockstep(dq, dp, _t(zq), _t(zp), 64, 2, wl.seed)
    assert torch.equal(full, again)              # run-to-run determinism
    dq.free(); dp.free()


def test_empty_and_bad_calls(B):
    wl = S.WORKLOADS["tiny"]
    _, _, blobs = H.oracle_heads(wl)
    dq, dp = H.device_heads(B, wl, blobs)
    z = torch.empty((0, 64), device=DEV)
    s = B.csd_denoise_lockstep(dq, dp, z, z, 0, 2, 1)
    assert s.shape == (0, 81)
    n, ell, mask = B.csd_verify(s, 0, 2, 16, 1)
    assert n.numel() == 0
    ws = torch.empty(256, dtype=torch.uint8, device=DEV)
    zz = torch.zeros((4, 64), device=DEV)
    with pytest.raises(B.CsdError) as e:
        B.csd_denoise_lockstep(dq, dp, zz, zz, 2, 2, 1, workspace=ws)
    assert e.value.code == B.CSD_EINVAL and "workspace" in str(e.value)
    with pytest.raises(B.CsdError):
        B.csd_head_eval(dq, torch.zeros((4, 16), device=DEV), zz, 11)
    dq.free(); dp.free()


# ------------------------------------------------------------- bf16 MFMA ----
def _bf16(a):
    return torch.from_numpy(S.bf16_round(a)).to(DEV).to(torch.bfloat16)


@pytest.mark.parametrize("M,N,K", [(1, 64, 64), (70, 128, 192), (300, 192, 128), (515, 256, 1024),
                                   (2048 + 37, 768, 256), (4096, 1024, 1024),
                                   # more tiles than CUs (several tiles per persistent workgroup), ragged
                                   # last row of tiles, tile counts that do and do not divide by 8
                                   (8192 + 100, 3072, 512), (16384, 2304, 192),
                                   # very wide N: column-panel tile order (18 N-tiles: panels of 9; 1 and 2 rows per XCD)
                                   (2048, 4608, 256), (4096, 4608, 320)])
def test_gemm_bf16_all_epilogues(B, M, N, K):
    rng = np.random.default_rng(M + N + K)
    A = S.bf16_round(rng.normal(size=(M, K)).astype(np.float32))
    W = S.bf16_round((rng.normal(size=(N, K)) / math.sqrt(K)).astype(np.float32))
    bias = rng.normal(size=N).astype(np.float32)
    gate = S.bf16_round(rng.normal(size=(M, N)).astype(np.float32))
    h0 = rng.normal(size=(M, N)).astype(np.float32)
    ref = A.astype(np.float64) @ W.astype(np.float64).T + bias
    tol = 2e-5 * math.sqrt(K)      # fp32 accumulation of K bf16 products
    out = B.csd_gemm_bf16(_bf16(A), _bf16(W), _t(bias), 0, out_f32=True).cpu().numpy()
    assert np.max(np.abs(out - ref)) < tol
    out = B.csd_gemm_bf16(_bf16(A), _bf16(W), _t(bias), 0).float().cpu().numpy()
    assert np.max(np.abs(out - ref) / (1 + np.abs(ref))) < 5e-3          # bf16 store
    out = B.csd_gemm_bf16(_bf16(A), _bf16(W), _t(bias), 1, out_f32=True).cpu().numpy()
    assert np.max(np.abs(out - O.silu(ref))) < tol
    out = B.csd_gemm_bf16(_bf16(A), _bf16(W), _t(bias), 1).float().cpu().numpy()
    assert np.max(np.abs(out - O.silu(ref)) / (1 + np.abs(ref))) < 5e-3  # bf16 store
    h = _t(h0.copy())
    B.csd_gemm_bf16(_bf16(A), _bf16(W), _t(bias), 2, C=h, gate=_bf16(gate))
    assert np.max(np.abs(h.cpu().numpy() - (h0 + gate.astype(np.float64) * ref))) < tol * 4


@pytest.mark.parametrize("shape,T,R", [
    (S.HeadShape(16, 64, 128, 2), 10, 131),
    (S.HeadShape(8, 40, 192, 3), 7, 300),
    (S.HeadShape(16, 768, 1024, 6), 100, 2100),
    (S.HeadShape(16, 768, 768, 6), 100, 515)])
def test_head_eval_bf16(B, shape, T, R):
    blob = S.bf16_round(S.head_weights(shape, 21, out_scale=0.8, bias_std=0.2))
    oh = O.Head(O.HeadCfg(shape.token_dim, shape.cond_dim, shape.width, shape.n_blocks, T, eps_skip_gain=1.0), blob)
    dh = B.csd_init_head(B.make_cfg(shape.token_dim, shape.cond_dim, shape.width, shape.n_blocks, T,
                                    B.CSD_BF16, eps_skip_gain=1.0), blob)
    rng = np.random.default_rng(5)
    x = rng.normal(size=(R, shape.token_dim)).astype(np.float32) * 1.5
    z = rng.normal(size=(R, shape.cond_dim)).astype(np.float32)
    for t in sorted({1, T}):
        got = B.csd_head_eval(dh, _t(x), _t(z), t).cpu().numpy()
        eh, v = oh.forward(x.astype(np.float64), t, oh.cond_embed(z.astype(np.float64)))
        want = np.concatenate([eh, v], 1)
        # one head evaluation is an intermediate, not a token: its worst element may sit a
        # little above the token tolerance (narrow heads average fewer roundings); the
        # root-mean-square error stays well below it
        assert H.rel_err(got, want) < 1.5 * H.BF16_TOL
        assert np.sqrt(np.mean((got - want) ** 2) / np.mean(want ** 2)) < 0.5 * H.BF16_TOL
    dh.free()


@pytest.mark.parametrize("out_scale", [0.05, 1.0])
def test_tiny_workload_end_to_end_bf16(B, out_scale):
    """bf16 MFMA path against the oracle fed the bf16-rounded weights: tokens within
    2e-2; decisions are reported by the bench, not gated (log-ratios amplify
    trajectory error by 1/sigma_1^2)."""
    wl = S.WORKLOADS["tiny"].with_(gamma=2, gemm_dtype="bf16", out_scale=out_scale)
    res = _end_to_end(B, wl, 150, H.BF16_TOL, dtype="bf16", check_decisions=False)
    assert res["agree"] > (0.8 if out_scale < 0.5 else 0.0)


# ------------------------------------------- full-size runs, bench configuration ----
def _sampled_rows_check(B, wl, R, sample_blocks, tol, check_decisions):
    """Run the whole path at R rows in the launch configuration bench.py times (default
    chains and tile choice), then recompute sampled 64-row blocks one by one on the
    oracle (rows are keyed by their global index) and compare."""
    gamma, D, seed = wl.gamma, 16, wl.seed
    G = R // gamma
    drf, tgt, blobs = H.oracle_heads(wl)
    dq, dp = H.device_heads(B, wl, blobs)
    zq, zp = wl.conds(R)
    summ = B.csd_denoise_lockstep(dq, dp, _t(zq), _t(zp), G, gamma, seed)
    n_g, ell_g, mask_g = B.csd_verify(summ, G, gamma, D, seed)
    tok_g, nout_g, trips_g, flags_g = B.csd_resample(summ, n_g, G, gamma, D, seed)
    torch.cuda.synchronize()
    sg, n_g, mask_g = summ.cpu().numpy(), n_g.cpu().numpy(), mask_g.cpu().numpy()
    tok_g, nout_g, trips_g = tok_g.cpu().numpy(), nout_g.cpu().numpy(), trips_g.cpu().numpy()
    # properties that hold at any size
    assert np.all(np.isfinite(sg))
    assert np.all((n_g >= 0) & (n_g <= gamma)) and np.all(nout_g == np.minimum(n_g + 1, gamma))
    first_rej = np.where(mask_g.reshape(G, gamma).all(1), gamma, np.argmin(mask_g.reshape(G, gamma), axis=1))
    assert np.array_equal(n_g, first_rej)
    assert np.all((trips_g > 0) == (n_g < gamma))
    for g in range(0, G, max(1, G // 50)):
        assert np.array_equal(tok_g[g, :n_g[g]], sg[g * gamma: g * gamma + n_g[g], 4 * D:5 * D])
        assert np.all(tok_g[g, nout_g[g]:] == 0)
    again = B.csd_denoise_lockstep(dq, dp, _t(zq), _t(zp), G, gamma, seed)
    assert torch.equal(again, summ)                      # run-to-run determinism at full size
    agree = []
    for r0 in sample_blocks:
        zq_s, zp_s = wl.conds(64, r0)
        assert np.array_equal(zq_s, zq[r0:r0 + 64])
        s_o, _ = O.denoise_lockstep(drf, tgt, zq_s, zp_s, seed, row_offset=r0)
        assert H.rel_err(sg[r0:r0 + 64, 4 * D:5 * D], s_o[:, 4 * D:5 * D]) < tol, "tokens of rows %d.." % r0
        assert H.rel_err(sg[r0:r0 + 64, 0:D], s_o[:, 0:D]) < tol
        n_o, ell_o, mask_o, log_u = O.verify(s_o, 64 // gamma, gamma, seed, r0)
        agree.append((mask_g[r0:r0 + 64].astype(bool) == mask_o.astype(bool)).mean())
        if check_decisions:
            H.decisions_match(mask_g[r0:r0 + 64], ell_o, log_u, gamma)
    dq.free(); dp.free()
    return float(np.mean(agree)), float(mask_g.mean())


def test_mar256_full_size_bf16_sampled_rows(B):
    wl = S.WORKLOADS["mar256"]
    R = wl.rows_total
    agree, acc = _sampled_rows_check(B, wl, R, [0, 8192 - 64, 8192, R - 64], H.BF16_TOL, check_decisions=False)
    assert agree > 0.9 and 0.15 < acc < 0.7


def test_mar256_latency_shape_f32(B):
    """One verify step of the 256x256-shaped workload (64 images x 4 draft tokens) in fp32:
    tokens to 1e-4 and decisions bit-exact outside the band."""
    wl = S.WORKLOADS["mar256"].with_(gemm_dtype="f32")
    _sampled_rows_check(B, wl, wl.rows_per_verify_step, [0, 192], H.F32_TOL, check_decisions=True)


def test_large_head_bf16_sampled_rows(B):
    wl = S.WORKLOADS["large"]
    _sampled_rows_check(B, wl, 2048 + 256, [0, 2048], H.BF16_TOL, check_decisions=False)


def test_reject_heavy_ragged_rows_bf16(B):
    """gamma = 8, a row count that is no multiple of any tile (ragged tail)."""
    wl = S.WORKLOADS["reject"]
    _sampled_rows_check(B, wl, 8 * 300, [0, 2304], H.BF16_TOL, check_decisions=False)


# ------------------------------------------------- schedules given as tables ----
def test_table_schedule_and_unequal_schedules_f32(B):
    """CSD_TABLE with the cosine schedule's own alpha_bar reproduces CSD_COSINE; a draft on a
    different (linear-beta) schedule than the target exercises the schedule part of log Sigma
    (the difference of the two heads' log sigma^2 at v = 0), against the oracle."""
    wl = S.WORKLOADS["tiny"].with_(gamma=2)
    tb, db, ds = wl.heads(0.05)
    T, G, gamma, D = wl.n_steps, 40, 2, 16
    zq, zp = wl.conds(128)
    zq, zp = zq[:G * gamma], zp[:G * gamma]
    cos = O.cosine_schedule(T)
    mk = lambda ab: B.make_cfg(16, 64, 128, 2, T, B.CSD_F32, alpha_bar=ab, eps_skip_gain=wl.eps_skip_gain)
    hq_c, hp_c = B.csd_init_head(mk(None), db), B.csd_init_head(mk(None), tb)
    hq_t, hp_t = B.csd_init_head(mk(cos.abar), db), B.csd_init_head(mk(cos.abar), tb)
    a = B.csd_denoise_lockstep(hq_c, hp_c, _t(zq), _t(zp), G, gamma, 5).cpu().numpy()
    b = B.csd_denoise_lockstep(hq_t, hp_t, _t(zq), _t(zp), G, gamma, 5).cpu().numpy()
    assert H.rel_err(b[:, 4 * D:5 * D], a[:, 4 * D:5 * D]) < 1e-5 and np.max(np.abs(a[:, -1] - b[:, -1])) < 1e-4
    # draft on a linear-beta schedule
    beta = np.linspace(1e-3, 0.35, T)
    abar_lin = np.concatenate([[1.0], np.cumprod(1.0 - beta)])
    lin = O.schedule_from_abar(abar_lin)
    ocfg = O.HeadCfg(16, 64, 128, 2, T, eps_skip_gain=wl.eps_skip_gain)
    oq, op = O.Head(ocfg, db, lin), O.Head(ocfg, tb, cos)
    want, _ = O.denoise_lockstep(oq, op, zq, zp, seed=5)
    hq_l = B.csd_init_head(mk(abar_lin), db)
    got = B.csd_denoise_lockstep(hq_l, hp_c, _t(zq), _t(zp), G, gamma, 5).cpu().numpy()
    mu_p, lv_p, mu_q, lv_q, x0, ls = O.split_summary(want, D)
    g = O.split_summary(got, D)
    assert H.rel_err(g[4], x0) < H.F32_TOL and H.rel_err(g[2], mu_q) < H.F32_TOL
    assert np.max(np.abs(g[3] - lv_q)) < 1e-3 and np.max(np.abs(g[1] - lv_p)) < 1e-3
    assert np.abs(ls).max() > 1.0                      # the schedule part is really there
    assert np.max(np.abs(g[5] - ls)) < H.F32_TOL * 10 * max(1.0, np.abs(ls).max())
    # and the split-phase route carries the same reference difference
    summ = torch.zeros((G * gamma, 5 * D + 1), device=DEV)
    for i in range(gamma):
        B.csd_denoise_draft(hq_l, _t(zq.reshape(G, gamma, -1)[:, i]), G, gamma, i, 5, 0, 1.0, summ)
    B.csd_denoise_target(hp_c, hq_l, _t(zp), G, gamma, 5, 0, 1.0, summ)
    assert np.array_equal(summ.cpu().numpy(), got)
    with pytest.raises(B.CsdError):                    # alpha_bar must decrease strictly from 1
        B.csd_init_head(mk(np.concatenate([[1.0], np.full(T, 0.5)])), db)
    for h in (hq_c, hp_c, hq_t, hp_t, hq_l):
        h.free()


# ------------------------------------------------------------ the stated limits ----
@pytest.mark.parametrize("shape,T,R,dtype", [
    (S.HeadShape(4, 8, 4096, 1), 2, 70, "f32"),        # widest head, smallest token and cond dims
    (S.HeadShape(4, 8, 4096, 1), 2, 300, "bf16"),
    (S.HeadShape(8, 16384, 64, 2), 3, 33, "f32"),      # largest cond dim, narrowest head
    (S.HeadShape(16, 64, 64, 64), 2, 40, "f32"),       # deepest head
    (S.HeadShape(16, 24, 320, 3), 5, 129, "bf16")])    # width that is no multiple of 256 or 192
def test_heads_at_the_limits_of_the_interface(B, shape, T, R, dtype):
    blob = S.head_weights(shape, 31, out_scale=0.3, bias_std=0.1)
    if dtype == "bf16":
        blob = S.bf16_round(blob)
    oh = O.Head(O.HeadCfg(shape.token_dim, shape.cond_dim, shape.width, shape.n_blocks, T, eps_skip_gain=1.0), blob)
    dh = B.csd_init_head(B.make_cfg(shape.token_dim, shape.cond_dim, shape.width, shape.n_blocks, T,
                                    B.CSD_BF16 if dtype == "bf16" else B.CSD_F32, eps_skip_gain=1.0), blob)
    rng = np.random.default_rng(8)
    z = rng.normal(size=(R, shape.cond_dim)).astype(np.float32)
    want = O.sample(oh, z, 77, 5, 1.0)
    got = B.csd_sample(dh, _t(z), 77, 5).cpu().numpy()
    assert H.rel_err(got, want) < (1.5 * H.BF16_TOL if dtype == "bf16" else H.F32_TOL)
    dh.free()


def test_longest_schedule_f32(B):
    """T = 4096 denoising steps (the interface's limit) with a tiny head: the step indexing,
    the noise slots and the log Sigma accumulation hold over the whole range."""
    shape, T, G, gamma = S.HeadShape(4, 8, 64, 1), 4096, 6, 2
    tb = S.head_weights(shape, 41, out_scale=0.02, bias_std=0.05)
    db = S.perturbed_copy(tb, shape, 42, 0.05, 0.02)
    ocfg = O.HeadCfg(4, 8, 64, 1, T, eps_skip_gain=1.0)
    oq, op = O.Head(ocfg, db), O.Head(ocfg, tb)
    mk = lambda: B.make_cfg(4, 8, 64, 1, T, B.CSD_F32, eps_skip_gain=1.0)
    dq, dp = B.csd_init_head(mk(), db), B.csd_init_head(mk(), tb)
    zq, zp = S.cond_vectors(G * gamma, 8, 4, add_std=0.1)
    want, _ = O.denoise_lockstep(oq, op, zq, zp, seed=3, row_offset=2 ** 40)
    got = B.csd_denoise_lockstep(dq, dp, _t(zq), _t(zp), G, gamma, 3, 2 ** 40).cpu().numpy()
    D = 4
    assert H.rel_err(got[:, 4 * D:5 * D], want[:, 4 * D:5 * D]) < 3 * H.F32_TOL      # 4096 fp32 steps
    assert np.max(np.abs(got[:, -1] - want[:, -1])) < 1e-3 * max(1.0, np.abs(want[:, -1]).max())
    dq.free(); dp.free()
