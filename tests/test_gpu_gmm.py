"""GPU parity of the mixture-of-Gaussians output heads (the appendix on other forms of the
output distribution): draft sampling, accept test and acceptance-rejection resampling with
explicit densities, through the C ABI against the oracle."""
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
    assert binding.CSD_STREAM_GMM_PICK == O.STREAM_GMM_PICK
    return binding


def _dev(m):
    return tuple(torch.from_numpy(np.ascontiguousarray(a)).to(DEV) for a in m)


@pytest.mark.parametrize("G,gamma,K,D,seed,row_offset", [
    (300, 4, 8, 16, 5, 0), (37, 3, 1, 4, 6, 2 ** 32 + 64), (1, 1, 64, 8, 7, 128), (1000, 8, 5, 16, 8, 64)])
def test_gmm_path_against_the_oracle(B, G, gamma, K, D, seed, row_offset):
    R = G * gamma
    mp, mq = S.mixture_pair(R, K, D, seed)
    dp, dq = _dev(mp), _dev(mq)
    # draft tokens: the component pick is integer work on fp32 sums (bit-exact), the token is fp32 arithmetic
    x_o = O.gmm_draft_sample(*mq, seed, row_offset)
    x_g = B.csd_gmm_draft_sample(dq, seed, row_offset)
    assert H.rel_err(x_g.cpu().numpy(), x_o) < 1e-5
    # accept test on the device's own tokens (so that both sides judge the same points)
    xs = x_g.cpu().numpy().astype(np.float64)
    n_o, ell_o, mask_o, log_u = O.gmm_verify(xs, *mp, *mq, G, gamma, seed, row_offset)
    n_g, ell_g, mask_g = B.csd_gmm_verify(x_g, dp, dq, G, gamma, seed, row_offset)
    ell_g = ell_g.cpu().numpy()
    assert np.max(np.abs(ell_g - ell_o)) < 1e-4 * max(1.0, np.abs(ell_o).max())
    exempt, ok = H.decisions_match(mask_g.cpu().numpy(), ell_o, log_u, gamma)
    # resampling, given the oracle's n_accept (decisions inside the band may differ)
    tok_o, nout_o, trips_o, flags_o, rec = O.gmm_resample(xs, n_o, *mp, *mq, G, gamma, seed, row_offset, 256)
    n_dev = torch.from_numpy(n_o).to(DEV)
    tok_g, nout_g, trips_g, flags_g = B.csd_gmm_resample(x_g, n_dev, dp, dq, G, gamma, seed, row_offset, 256)
    torch.cuda.synchronize()
    clear = np.ones(G, dtype=bool)
    for g in range(G):
        if rec[g] and any(abs(u - a) < 1e-3 * max(a, 1e-6) for a, u in rec[g]):
            clear[g] = False
    assert clear.mean() > 0.9
    assert np.array_equal(nout_g.cpu().numpy(), nout_o)
    assert np.array_equal(trips_g.cpu().numpy()[clear], trips_o[clear])
    assert np.array_equal(flags_g.cpu().numpy()[clear].astype(np.uint32), flags_o[clear])
    assert H.rel_err(tok_g.cpu().numpy()[clear], tok_o[clear]) < 1e-5
    if K > 1 and G >= 300:
        assert 0.05 < mask_o.mean() < 0.95 and (trips_o > 1).sum() > 10            # both branches, several trips
    assert np.array_equal(n_g.cpu().numpy()[ok], n_o[ok])


def test_gmm_identical_mixtures_accept_everything(B):
    G, gamma, K, D = 200, 4, 6, 16
    mp, _ = S.mixture_pair(G * gamma, K, D, 3)
    dp = _dev(mp)
    x = B.csd_gmm_draft_sample(dp, 11)
    n, ell, mask = B.csd_gmm_verify(x, dp, dp, G, gamma, 11)
    assert torch.all(ell == 0) and torch.all(mask == 1) and torch.all(n == gamma)
    tok, n_out, trips, flags = B.csd_gmm_resample(x, n, dp, dp, G, gamma, 11)
    assert torch.all(n_out == gamma) and torch.all(trips == 0) and torch.all(flags == 0)
    assert torch.equal(tok[:, :gamma].reshape(G * gamma, D), x)


def test_gmm_rows_are_keyed_by_the_global_row(B):
    """Two half-size calls equal one call (counters are global rows)."""
    G, gamma, K, D, seed = 128, 2, 4, 8, 21
    R = G * gamma
    mp, mq = S.mixture_pair(R, K, D, seed)
    dp, dq = _dev(mp), _dev(mq)
    x = B.csd_gmm_draft_sample(dq, seed, 64)
    n, ell, mask = B.csd_gmm_verify(x, dp, dq, G, gamma, seed, 64)
    tok, n_out, trips, flags = B.csd_gmm_resample(x, n, dp, dq, G, gamma, seed, 64)
    h = R // 2
    half = lambda m, a, b: tuple(t[a:b].contiguous() for t in m)
    for a, b in ((0, h), (h, R)):
        xa = B.csd_gmm_draft_sample(half(dq, a, b), seed, 64 + a)
        assert torch.equal(xa, x[a:b])
        na, ella, maska = B.csd_gmm_verify(xa, half(dp, a, b), half(dq, a, b), G // 2, gamma, seed, 64 + a)
        assert torch.equal(ella, ell[a:b]) and torch.equal(na, n[a // gamma:b // gamma])
        toka, nouta, _, _ = B.csd_gmm_resample(xa, na, half(dp, a, b), half(dq, a, b), G // 2, gamma, seed, 64 + a)
        assert torch.equal(toka, tok[a // gamma:b // gamma]) and torch.equal(nouta, n_out[a // gamma:b // gamma])


def test_gmm_bad_calls(B):
    mp, mq = S.mixture_pair(8, 3, 16, 1)
    dp, dq = _dev(mp), _dev(mq)
    x = B.csd_gmm_draft_sample(dq, 1)
    lib = B._lib
    p = lambda t: t.data_ptr()
    assert lib.csd_gmm_verify(p(x), *[p(t) for t in dp], *[p(t) for t in dq], 4, 2, 65, 16, 1, 0, None, None, None, None) == B.CSD_EINVAL
    assert b"n_components" in lib.csd_last_error()
    assert lib.csd_gmm_verify(p(x), *[p(t) for t in dp], *[p(t) for t in dq], 4, 2, 3, 12, 1, 0, None, None, None, None) == B.CSD_EINVAL
    assert lib.csd_gmm_verify(p(x), *[p(t) for t in dp], *[p(t) for t in dq], 4, 2, 3, 16, 1, 0, None, None, None, None) == B.CSD_EINVAL
    assert b"NULL" in lib.csd_last_error()
    n = torch.zeros(4, dtype=torch.int32, device=DEV)
    with pytest.raises(B.CsdError):
        B.csd_gmm_resample(x, n, dp, dq, 4, 2, 1, 0, 0)                       # max_trips
    # a zero-weight component is never drawn and does not disturb the density
    pi0 = dq[0].clone(); pi0[:, 1] = 0
    x0 = B.csd_gmm_draft_sample((pi0, dq[1], dq[2]), 5)
    two = (pi0[:, [0, 2]].contiguous(), dq[1][:, [0, 2]].contiguous(), dq[2][:, [0, 2]].contiguous())
    assert torch.equal(x0, B.csd_gmm_draft_sample(two, 5))
    _, ell_a, _ = B.csd_gmm_verify(x0, dp, (pi0, dq[1], dq[2]), 4, 2, 5)
    p2 = (dp[0][:, [0, 2]].contiguous(), dp[1][:, [0, 2]].contiguous(), dp[2][:, [0, 2]].contiguous())
    pz = dp[0].clone(); pz[:, 1] = 0
    _, ell_b, _ = B.csd_gmm_verify(x0, (pz, dp[1], dp[2]), (pi0, dq[1], dq[2]), 4, 2, 5)
    _, ell_c, _ = B.csd_gmm_verify(x0, p2, two, 4, 2, 5)
    assert torch.allclose(ell_b, ell_c, atol=1e-5) and not torch.allclose(ell_a, ell_b, atol=1e-3)
