"""GPU parity of the split-phase form of Alg. 1 (draft head per position, target head on
all positions, target-only sampling, bonus token), through the C ABI against the oracle."""
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


def _split_on_device(B, dq, dp, zq, zp, G, gamma, seed, row_offset, tau, D=16):
    summ = torch.full((G * gamma, 5 * D + 1), float("nan"), device=DEV)
    zq3 = zq.reshape(G, gamma, -1)
    for i in range(gamma):
        B.csd_denoise_draft(dq, _t(zq3[:, i]), G, gamma, i, seed, row_offset, tau, summ)
    B.csd_denoise_target(dp, dq, _t(zp), G, gamma, seed, row_offset, tau, summ)
    return summ


@pytest.mark.parametrize("dtype,G,gamma,tau,row_offset", [
    ("f32", 37, 3, 0.9, 2 ** 32 + 64), ("f32", 1, 1, 1.0, 0), ("bf16", 150, 4, 1.0, 128)])
def test_split_phase_equals_lockstep_bit_for_bit(B, dtype, G, gamma, tau, row_offset):
    """gamma draft calls of G rows and one target call of G*gamma rows leave exactly the
    summary of one lockstep call (same counters, same arithmetic per row)."""
    wl = S.WORKLOADS["tiny"].with_(gamma=gamma, gemm_dtype=dtype)
    _, _, blobs = H.oracle_heads(wl, 0.05)
    dq, dp = H.device_heads(B, wl, blobs, dtype)
    zq, zp = wl.conds((G * gamma + 63) // 64 * 64)
    zq, zp = zq[:G * gamma], zp[:G * gamma]
    lock = B.csd_denoise_lockstep(dq, dp, _t(zq), _t(zp), G, gamma, wl.seed, row_offset, tau)
    split = _split_on_device(B, dq, dp, zq, zp, G, gamma, wl.seed, row_offset, tau)
    torch.cuda.synchronize()
    assert torch.equal(lock, split)
    dq.free(); dp.free()


@pytest.mark.parametrize("name,G", [("mar256", 64), ("mar256", 2100)])
def test_split_phase_at_the_workload_shapes_bf16(B, name, G):
    """The real per-verify-step shape (64 images x gamma 4: draft calls of 64 rows, one target
    call of 256) and a many-image shape whose target call is cut into row chunks: both leave
    the lockstep summary bit for bit (which the full-size tests pin to the oracle)."""
    wl = S.WORKLOADS[name]
    gamma = wl.gamma
    _, _, blobs = H.oracle_heads(wl)
    dq, dp = H.device_heads(B, wl, blobs)
    R = G * gamma
    zq, zp = wl.conds((R + 63) // 64 * 64)
    zq, zp = zq[:R], zp[:R]
    lock = B.csd_denoise_lockstep(dq, dp, _t(zq), _t(zp), G, gamma, wl.seed, 0, 1.0)
    split = _split_on_device(B, dq, dp, zq, zp, G, gamma, wl.seed, 0, 1.0)
    torch.cuda.synchronize()
    assert torch.equal(lock, split)
    dq.free(); dp.free()


def test_split_phase_against_the_oracle_f32(B):
    wl = S.WORKLOADS["tiny"].with_(gamma=3)
    G, gamma, D, tau, off = 21, 3, 16, 0.95, 192
    oq, op, blobs = H.oracle_heads(wl, 0.05)
    dq, dp = H.device_heads(B, wl, blobs)
    zq, zp = wl.conds(64)
    zq, zp = zq[:G * gamma], zp[:G * gamma]
    want = np.zeros((G * gamma, 5 * D + 1))
    for i in range(gamma):
        O.denoise_draft(oq, zq.reshape(G, gamma, -1)[:, i], gamma, i, wl.seed, off, tau, want)
    O.denoise_target(op, zp, wl.seed, off, tau, want)
    got = _split_on_device(B, dq, dp, zq, zp, G, gamma, wl.seed, off, tau).cpu().numpy()
    mu_p, lv_p, mu_q, lv_q, x0, ls = O.split_summary(want, D)
    g = O.split_summary(got, D)
    assert H.rel_err(g[4], x0) < H.F32_TOL and H.rel_err(g[0], mu_p) < H.F32_TOL and H.rel_err(g[2], mu_q) < H.F32_TOL
    assert np.max(np.abs(g[5] - ls)) < H.F32_TOL * 10 * max(1.0, np.abs(ls).max())
    dq.free(); dp.free()


@pytest.mark.parametrize("dtype,tol", [("f32", H.F32_TOL), ("bf16", H.BF16_TOL)])
def test_sample_and_bonus_stream_against_the_oracle(B, dtype, tol):
    """Target-only sampling on the trajectory stream and on the bonus stream (keyed by the
    global group index) against the oracle's sampler."""
    wl = S.WORKLOADS["tiny"].with_(gemm_dtype=dtype)
    oq, op, blobs = H.oracle_heads(wl, 0.05)
    dq, dp = H.device_heads(B, wl, blobs, dtype)
    _, zp = wl.conds(128)
    z = zp[:70]
    for stream, off in ((O.STREAM_BONUS, 2 ** 33 + 5), (O.STREAM_TRAJ, 0)):
        want = O.sample(op, z, wl.seed, off, 0.9, stream)
        got = B.csd_sample(dp, _t(z), wl.seed, off, stream, 0.9).cpu().numpy()
        assert H.rel_err(got, want) < tol
    a = B.csd_sample(dp, _t(z), wl.seed, 7, B.CSD_STREAM_BONUS)
    b = B.csd_sample(dp, _t(z), wl.seed, 7, B.CSD_STREAM_TRAJ)
    assert not torch.equal(a, b)
    # the lockstep draft token of a row is the plain draft sample of that row (same counters)
    zq, _ = wl.conds(128)
    summ = B.csd_denoise_lockstep(dq, dp, _t(zq[:70]), _t(zp[:70]), 35, 2, wl.seed, 64)
    assert torch.equal(summ[:, 64:80], B.csd_sample(dq, _t(zq[:70]), wl.seed, 64))
    with pytest.raises(B.CsdError):
        B.csd_sample(dp, _t(z), wl.seed, 0, 2)          # not a trajectory stream
    dq.free(); dp.free()


def test_append_bonus_matches_the_oracle(B):
    rng = np.random.default_rng(3)
    G, gamma, D = 300, 4, 16
    tokens = rng.normal(size=(G, gamma + 1, D)).astype(np.float32)
    n_accept = rng.integers(0, gamma + 1, size=G).astype(np.int32)
    n_out = np.where(n_accept == gamma, gamma, n_accept + 1).astype(np.int32)
    bonus = rng.normal(size=(G, D)).astype(np.float32)
    want_tok, want_n = tokens.copy(), n_out.copy()
    O.append_bonus(want_tok, want_n, n_accept, bonus, gamma)
    t, n = _t(tokens), _t(n_out)
    B.csd_append_bonus(t, n, _t(n_accept), _t(bonus), gamma)
    assert np.array_equal(t.cpu().numpy(), want_tok) and np.array_equal(n.cpu().numpy(), want_n)
    assert (n_accept == gamma).sum() > 20


def test_autoregressive_style_round_against_the_oracle(B):
    """One verify window the way Alg. 1 runs it: draft positions one by one, target on all,
    accept test, resampling, bonus token from p_{gamma+1} - decisions and emitted tokens
    against the oracle (groups inside the 1e-3 decision band excepted)."""
    wl = S.WORKLOADS["tiny"].with_(gamma=3, out_scale=0.02)      # high acceptance: many bonus tokens
    G, gamma, D, tau, off = 96, 3, 16, 1.0, 0
    seed = wl.seed
    oq, op, blobs = H.oracle_heads(wl, 0.05)
    dq, dp = H.device_heads(B, wl, blobs)
    zq, zp = wl.conds(G * gamma)
    _, zb = wl.conds(128, 4096)                                   # cond vectors of position gamma+1
    zb = zb[:G]
    # oracle
    so = np.zeros((G * gamma, 5 * D + 1))
    for i in range(gamma):
        O.denoise_draft(oq, zq.reshape(G, gamma, -1)[:, i], gamma, i, seed, off, tau, so)
    O.denoise_target(op, zp, seed, off, tau, so)
    n_o, ell_o, mask_o, log_u = O.verify(so, G, gamma, seed, off, tau)
    tok_o, nout_o, trips_o, flags_o, rec = O.resample(so, n_o, G, gamma, seed, off, tau, 256)
    bonus_o = O.sample(op, zb, seed, off // gamma, tau, O.STREAM_BONUS)
    O.append_bonus(tok_o, nout_o, n_o, bonus_o, gamma)
    # device
    sg = _split_on_device(B, dq, dp, zq, zp, G, gamma, seed, off, tau)
    n_g, ell_g, mask_g = B.csd_verify(sg, G, gamma, D, seed, off, tau)
    tok_g, nout_g, trips_g, flags_g = B.csd_resample(sg, n_g, G, gamma, D, seed, off, tau, 256)
    bonus_g = B.csd_sample(dp, _t(zb), seed, off // gamma, B.CSD_STREAM_BONUS, tau)
    B.csd_append_bonus(tok_g, nout_g, n_g, bonus_g, gamma)
    torch.cuda.synchronize()
    exempt, ok = H.decisions_match(mask_g.cpu().numpy(), ell_o, log_u, gamma)
    for g in range(G):
        if rec[g] and any(abs(u - a) < 1e-3 * max(a, 1e-6) for a, u in rec[g]):
            ok[g] = False
    assert ok.mean() > 0.8
    assert np.array_equal(n_g.cpu().numpy()[ok], n_o[ok])
    assert np.array_equal(nout_g.cpu().numpy()[ok], nout_o[ok])
    assert H.rel_err(tok_g.cpu().numpy()[ok], tok_o[ok]) < H.F32_TOL
    assert (nout_o == gamma + 1).sum() >= 5 and (nout_o <= gamma).sum() >= 5     # both branches exercised
    dq.free(); dp.free()


def test_split_phase_bad_calls(B):
    wl = S.WORKLOADS["tiny"]
    _, _, blobs = H.oracle_heads(wl)
    dq, dp = H.device_heads(B, wl, blobs)
    summ = torch.zeros((8, 81), device=DEV)
    z = torch.zeros((4, 64), device=DEV)
    with pytest.raises(B.CsdError):
        B.csd_denoise_draft(dq, z, 4, 2, 2, 1, 0, 1.0, summ)            # position out of range
    with pytest.raises(B.CsdError) as e:
        B.csd_denoise_draft(dq, z, 4, 2, 0, 1, 0, 1.0, summ, workspace=torch.empty(256, dtype=torch.uint8, device=DEV))
    assert "workspace" in str(e.value)
    with pytest.raises(B.CsdError):
        B.csd_denoise_target(dp, dq, torch.zeros((8, 64), device=DEV), 4, 2, 1, 0, 0.0, summ)   # temperature
    B.csd_denoise_draft(dq, torch.zeros((0, 64), device=DEV), 0, 2, 0, 1, 0, 1.0, torch.zeros((0, 81), device=DEV))
    dq.free(); dp.free()


def test_bonus_sample_beside_the_target_call_on_a_second_stream(B):
    """Two calls that need one chain each (no row chunks) may run at the same time on two
    streams of default priority with their own workspaces: same bits as one after the other."""
    wl = S.WORKLOADS["mar256"]
    G, gamma, D = 64, wl.gamma, 16
    _, _, blobs = H.oracle_heads(wl)
    dq, dp = H.device_heads(B, wl, blobs)
    zq, zp = wl.conds(G * gamma)
    zb = _t(zp[:G])
    summ_a = torch.zeros((G * gamma, 5 * D + 1), device=DEV)
    for i in range(gamma):
        B.csd_denoise_draft(dq, _t(zq.reshape(G, gamma, -1)[:, i]), G, gamma, i, wl.seed, 0, 1.0, summ_a)
    summ_b = summ_a.clone()
    B.csd_denoise_target(dp, dq, _t(zp), G, gamma, wl.seed, 0, 1.0, summ_a)
    bonus_a = B.csd_sample(dp, zb, wl.seed, 0, B.CSD_STREAM_BONUS)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    ws_t = torch.empty(B.csd_workspace_bytes(None, dp, G * gamma), dtype=torch.uint8, device=DEV)
    ws_b = torch.empty(B.csd_workspace_bytes(dp, None, G), dtype=torch.uint8, device=DEV)
    bonus_b = torch.empty((G, D), device=DEV)
    zp_d = _t(zp)
    for _ in range(3):
        fork = torch.cuda.Event(); fork.record()
        side.wait_event(fork)
        B.csd_sample(dp, zb, wl.seed, 0, B.CSD_STREAM_BONUS, 1.0, tokens=bonus_b, workspace=ws_b, stream=side)
        join = torch.cuda.Event(); join.record(side)
        s2 = summ_b.clone()
        B.csd_denoise_target(dp, dq, zp_d, G, gamma, wl.seed, 0, 1.0, s2, workspace=ws_t)
        torch.cuda.current_stream().wait_event(join)
        torch.cuda.synchronize()
        assert torch.equal(s2, summ_a) and torch.equal(bonus_b, bonus_a)
    dq.free(); dp.free()
