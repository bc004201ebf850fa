"""Shared plumbing of the GPU parity tests: build the same heads on both sides and
compare results under the stated tolerances (fp32 path 1e-4, bf16 path 2e-2 on tokens,
decisions exact outside a 1e-3 band of the log-ratio)."""
from __future__ import annotations

import numpy as np

from oracle import csd_oracle as O
from paper_2411_11925_amd import synth as S

F32_TOL = 1e-4     # fp32 path vs fp64 oracle (the benchmark spec)
BF16_TOL = 2e-2    # bf16-MFMA path vs fp64 oracle fed the bf16-rounded weights
BAND = 1e-3        # decisions are exempt where |log u - log ratio| < BAND


def oracle_heads(wl: S.Workload, bias_std: float = 0.0, ddim_eta: float | None = None):
    tb, db, ds = wl.heads(bias_std)
    samp = dict(sampler="ddim", ddim_eta=ddim_eta) if ddim_eta is not None else {}
    mk = lambda sh: O.HeadCfg(sh.token_dim, sh.cond_dim, sh.width, sh.n_blocks, wl.n_steps,
                              eps_skip_gain=wl.eps_skip_gain, **samp)
    return O.Head(mk(ds), db), O.Head(mk(wl.target), tb), (db, ds, tb)


def device_heads(B, wl: S.Workload, blobs, dtype: str | None = None, ddim_eta: float | None = None):
    db, ds, tb = blobs
    gd = B.CSD_BF16 if (dtype or wl.gemm_dtype) == "bf16" else B.CSD_F32
    mk = lambda sh: B.make_cfg(sh.token_dim, sh.cond_dim, sh.width, sh.n_blocks, wl.n_steps, gd,
                               eps_skip_gain=wl.eps_skip_gain, ddim_eta=ddim_eta)
    return B.csd_init_head(mk(ds), db), B.csd_init_head(mk(wl.target), tb)


def rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max over elements of |got-want| / max(|want|, rms of want's row)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if want.size == 0:
        return 0.0
    w2 = want.reshape(want.shape[0], -1)
    scale = np.maximum(np.abs(w2), np.sqrt((w2 ** 2).mean(axis=1, keepdims=True)) + 1e-30)
    return float(np.max(np.abs(got.reshape(w2.shape) - w2) / scale))


def decisions_match(mask_gpu, ell_oracle, log_u, gamma):
    """Bit-exact accept mask outside the band; returns (exempt_rows, group_is_comparable).
    A group stays comparable only if no exempt row sits at or before its first
    rejected row (oracle's view)."""
    ell = np.asarray(ell_oracle)
    exempt = np.abs(log_u - ell) < BAND
    want = log_u <= ell
    bad = (np.asarray(mask_gpu).astype(bool) != want) & ~exempt
    assert not bad.any(), "accept decisions differ outside the band at rows %s" % np.nonzero(bad)[0][:10]
    G = ell.shape[0] // gamma
    ok = np.ones(G, dtype=bool)
    for g in range(G):
        w = want[g * gamma:(g + 1) * gamma]
        first = int(np.argmin(w)) if not w.all() else gamma - 1
        ok[g] = not exempt[g * gamma: g * gamma + first + 1].any()
    return exempt, ok
