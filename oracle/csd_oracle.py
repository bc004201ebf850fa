"""fp64 CPU oracle for continuous speculative decoding (arxiv 2411.11925).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain reference that the
HIP path is compared with.  It shares no code with the HIP library: nothing
under ``paper_2411_11925_amd/`` imports it and it imports nothing from there.
Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may call it.

What it computes, in the paper's order and notation (numpy, float64):

  * the reverse-diffusion head sampler for a draft model q and a target model p
    run in lockstep with the SAME reparameterisation noise eps_t (Sec. 3.2,
    "denoising trajectory alignment"; App. A.2),
  * per-step Gaussian transition log-densities N(x_{t-1}; mu_t, Sigma_t)
    (Eq. 3) accumulated over t = T..2 into log(Sigma) of Eq. 6, in both the
    full form (difference of log-densities) and the simplified form (half the
    difference of log-determinants),
  * the accept test of Alg. 1 with ratio Sigma * p(x0|x1^p) / q(x0|x1^q)
    (Eq. 7) and the first-reject scan,
  * acceptance-rejection resampling from max(0, p - q)/Z with the threshold of
    Corollary 1 (Eq. 8-10; Alg. 1 repeat-until loop), proposal p(.|x1^p),
  * the same accept test and resampling for mixture-of-Gaussians output heads
    (the appendix on other forms of the output distribution), where p(x) and
    q(x) are explicit.

The diffusion head itself is not defined by the paper ("a neural network with
parameter theta", Sec. 3.1); the adaLN residual MLP used here is this build's
own definition (written out in class Head below).  Its forward pass therefore has
no pin against the paper: PARITY UNPINNED against the paper for `head_forward`
(it is pinned by internal invariants and an independent scalar-loop
re-implementation in the tests).

Random numbers: Philox-4x32-10 (Salmon et al., SC'11) keyed by the call seed,
countered by (global row, slot | stream << 16, block).  Uniforms take 23 bits;
normals are Box-Muller evaluated by a fixed sequence of IEEE fp32 operations
(no fused multiply-add), so that a device implementing the same sequence gets
the same bit patterns.  The oracle promotes them to float64 before use.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

LOG_2PI = math.log(2.0 * math.pi)

STREAM_TRAJ = 0      # slot T is x_T, slot t-1 is eps_t for t = T..1
STREAM_ACCEPT_U = 1  # slot 0: the uniform r_i of the accept test
STREAM_RESAMPLE_N = 2  # slot k: proposal noise of resampling trial k
STREAM_RESAMPLE_U = 3  # slot k: uniform of resampling trial k
STREAM_BONUS = 4     # trajectory noise of the target-only sample x ~ p_{gamma+1}, keyed by the global GROUP index
STREAM_TRAJ_P = 5    # the target's own trajectory noise when the two paths are NOT aligned (ablation), slots as stream 0
STREAM_GMM_PICK = 6  # mixture heads: the uniform that picks a component; slot 0: the draft's sample, slot 1+k: resampling trial k

# how the path ratio before the final step is formed (Table 1 of the paper)
RATIO_ALIGNED = 0      # p(Y_p)/q(Y_q), eps^p_t = eps^q_t: the method
RATIO_UNALIGNED = 1    # p(Y_p)/q(Y_q), independent noise in the two paths
RATIO_SINGLE_PATH = 2  # p(Y)/q(Y), both densities on the draft's path (Eq. 2)


# --------------------------------------------------------------------------
# Noise schedule (DDPM, cosine; Nichol & Dhariwal's learned-range variance)
# --------------------------------------------------------------------------
@dataclass
class Schedule:
    T: int
    beta: np.ndarray            # [T+1], beta[0] unused (0)
    alpha: np.ndarray           # [T+1], alpha[0] = 1
    abar: np.ndarray            # [T+1], abar[0] = 1
    beta_tilde: np.ndarray      # [T+1], posterior variance, beta_tilde[1] = 0
    log_beta: np.ndarray        # [T+1], entry 0 unused
    log_beta_tilde_clip: np.ndarray  # [T+1], entry 1 replaced by entry 2


def schedule_from_abar(abar: np.ndarray) -> Schedule:
    """Every per-step constant of the sampler from abar_0..abar_T (abar_0 = 1)."""
    abar = np.asarray(abar, dtype=np.float64)
    T = abar.shape[0] - 1
    alpha = np.ones(T + 1)
    beta = np.zeros(T + 1)
    bt = np.zeros(T + 1)
    for t in range(1, T + 1):
        alpha[t] = abar[t] / abar[t - 1]
        beta[t] = 1.0 - alpha[t]
        bt[t] = beta[t] * (1.0 - abar[t - 1]) / (1.0 - abar[t])
    log_beta = np.zeros(T + 1)
    log_beta[1:] = np.log(beta[1:])
    lbt = np.zeros(T + 1)
    if T >= 2:
        lbt[2:] = np.log(bt[2:])
        lbt[1] = lbt[2]          # posterior variance is 0 at t = 1: clipped
    else:
        lbt[1] = log_beta[1]
    return Schedule(T, beta, alpha, abar, bt, log_beta, lbt)


def cosine_schedule(T: int) -> Schedule:
    """Native T-step cosine schedule: abar(t) ~ cos^2(((t/T)+s)/(1+s) * pi/2),
    s = 0.008, betas clipped at 0.999, abar the running product of the
    clipped alphas."""
    def f(t):
        return math.cos(((t / T) + 0.008) / 1.008 * math.pi / 2.0) ** 2
    abar = np.ones(T + 1)
    for t in range(1, T + 1):
        b = min(1.0 - f(t) / f(t - 1), 0.999)
        abar[t] = abar[t - 1] * (1.0 - b)
    return schedule_from_abar(abar)


# --------------------------------------------------------------------------
# Philox-4x32-10 and the fp32 uniform / normal transforms
# --------------------------------------------------------------------------
_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85
_MASK32 = np.uint64(0xFFFFFFFF)


def philox4x32_10(c0, c1, c2, c3, k0: int, k1: int):
    """Ten rounds of Philox-4x32 on arrays of counters (uint32 each)."""
    c0 = np.asarray(c0, dtype=np.uint64) & _MASK32
    c1 = np.asarray(c1, dtype=np.uint64) & _MASK32
    c2 = np.asarray(c2, dtype=np.uint64) & _MASK32
    c3 = np.asarray(c3, dtype=np.uint64) & _MASK32
    c0, c1, c2, c3 = np.broadcast_arrays(c0, c1, c2, c3)
    k0 &= 0xFFFFFFFF
    k1 &= 0xFFFFFFFF
    for _ in range(10):
        p0 = _PHILOX_M0 * c0            # 64-bit products of 32-bit values
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK32
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0), lo1,
                          hi0 ^ c3 ^ np.uint64(k1), lo0)
        k0 = (k0 + _PHILOX_W0) & 0xFFFFFFFF
        k1 = (k1 + _PHILOX_W1) & 0xFFFFFFFF
    return (c0.astype(np.uint32), c1.astype(np.uint32),
            c2.astype(np.uint32), c3.astype(np.uint32))


def uniform23(x: np.ndarray) -> np.ndarray:
    """(x >> 9 + 1/2) * 2^-23 in (0,1); every step is exact in fp32."""
    k = (np.asarray(x, dtype=np.uint32) >> np.uint32(9)).astype(np.float32)
    return (k + np.float32(0.5)) * np.float32(2.0 ** -23)


def _log_u_f32(u: np.ndarray) -> np.ndarray:
    """ln(u) for fp32 u in (0,1) by the fixed fp32 operation sequence of the
    generator spec: split u = m 2^e, fold m into (sqrt(1/2), sqrt(2)], then
    ln m = 2 s (1 + s^2 P(s^2)),  s = (m-1)/(m+1)."""
    f32 = np.float32
    bits = u.view(np.uint32)
    e = (bits >> np.uint32(23)).astype(np.int32) - 127
    m = ((bits & np.uint32(0x007FFFFF)) | np.uint32(0x3F800000)).view(np.float32)
    big = m > f32(1.41421354)
    m = np.where(big, m * f32(0.5), m)
    e = np.where(big, e + 1, e)
    s = (m - f32(1.0)) / (m + f32(1.0))
    s2 = s * s
    p = f32(1.0 / 9.0)
    p = p * s2 + f32(1.0 / 7.0)
    p = p * s2 + f32(0.2)
    p = p * s2 + f32(1.0 / 3.0)
    w = s2 * p + f32(1.0)
    lnm = (f32(2.0) * s) * w
    return e.astype(np.float32) * f32(0.693147182) + lnm


def _sincos_quarter_f32(g: np.ndarray):
    """sin and cos of (pi/2) g for fp32 g in (0, 1/2] (Taylor, Horner, fp32)."""
    f32 = np.float32
    y = g * f32(1.57079637)
    y2 = y * y
    ps = f32(1.0 / 362880.0)
    ps = ps * y2 + f32(-1.0 / 5040.0)
    ps = ps * y2 + f32(1.0 / 120.0)
    ps = ps * y2 + f32(-1.0 / 6.0)
    ps = ps * y2 + f32(1.0)
    sn = y * ps
    pc = f32(-1.0 / 3628800.0)
    pc = pc * y2 + f32(1.0 / 40320.0)
    pc = pc * y2 + f32(-1.0 / 720.0)
    pc = pc * y2 + f32(1.0 / 24.0)
    pc = pc * y2 + f32(-0.5)
    cs = pc * y2 + f32(1.0)
    return sn, cs


def normal_pair_f32(xa: np.ndarray, xb: np.ndarray):
    """Box-Muller on two 32-bit words -> two fp32 standard normals."""
    f32 = np.float32
    xa = np.asarray(xa, dtype=np.uint32)
    xb = np.asarray(xb, dtype=np.uint32)
    u1 = uniform23(xa)
    r = np.sqrt(f32(-2.0) * _log_u_f32(u1))
    kb = xb >> np.uint32(9)                       # 23 bits: a fraction of a turn
    quad = (kb >> np.uint32(21)).astype(np.int32)  # which quarter turn
    j = (kb & np.uint32(0x001FFFFF)).astype(np.float32)
    f = (j + f32(0.5)) * f32(2.0 ** -21)          # position inside the quarter
    hi = f > f32(0.5)
    g = np.where(hi, f32(1.0) - f, f)
    sn, cs = _sincos_quarter_f32(g)
    sn, cs = np.where(hi, cs, sn), np.where(hi, sn, cs)
    c = np.select([quad == 0, quad == 1, quad == 2], [cs, -sn, -cs], sn)
    s = np.select([quad == 0, quad == 1, quad == 2], [sn, cs, -sn], -cs)
    return (r * c).astype(np.float32), (r * s).astype(np.float32)


def _counter_words(rows: np.ndarray, slot: int, stream: int, blk):
    rows = np.asarray(rows, dtype=np.uint64)
    c0 = rows & _MASK32
    c1 = rows >> np.uint64(32)
    c2 = np.uint64((slot & 0xFFFF) | (stream << 16))
    return c0, c1, c2, np.asarray(blk, dtype=np.uint64)


def normals(seed: int, rows, slot: int, stream: int, D: int) -> np.ndarray:
    """[len(rows), D] standard normals (fp32 values held in float64).
    Element d = 4 b + j comes from block b of the row's counter: words (0,1)
    give elements j = 0,1 and words (2,3) give j = 2,3."""
    assert D % 4 == 0 and 0 <= slot < 65536
    rows = np.asarray(rows, dtype=np.uint64)
    out = np.empty((rows.shape[0], D), dtype=np.float64)
    for b in range(D // 4):
        c0, c1, c2, c3 = _counter_words(rows, slot, stream, b)
        w0, w1, w2, w3 = philox4x32_10(c0, c1, c2, c3,
                                       seed & 0xFFFFFFFF, seed >> 32)
        n0, n1 = normal_pair_f32(w0, w1)
        n2, n3 = normal_pair_f32(w2, w3)
        out[:, 4 * b + 0] = n0
        out[:, 4 * b + 1] = n1
        out[:, 4 * b + 2] = n2
        out[:, 4 * b + 3] = n3
    return out


def uniforms(seed: int, rows, slot: int, stream: int) -> np.ndarray:
    """One uniform in (0,1) per row: word 0 of block 0."""
    c0, c1, c2, c3 = _counter_words(rows, slot, stream, 0)
    w0, _, _, _ = philox4x32_10(c0, c1, c2, c3, seed & 0xFFFFFFFF, seed >> 32)
    return uniform23(w0).astype(np.float64)


# --------------------------------------------------------------------------
# The diffusion head (this build's definition; see module docstring)
# --------------------------------------------------------------------------
TIME_FEATURES = 256


@dataclass
class HeadCfg:
    token_dim: int      # D
    cond_dim: int       # C
    width: int          # W
    n_blocks: int       # L
    n_steps: int        # T
    ln_eps: float = 1e-6
    t_scale: float | None = None    # default 1000 / T
    eps_skip_gain: float = 0.0      # eps_hat = gain * sqrt(1-abar_t) * x_t + o[:D]
    sampler: str = "ddpm"           # "ddpm" (Eq. 3, learned-range variance) | "ddim" (App., other samplers)
    ddim_eta: float = 1.0           # DDIM: sigma_t^2 = eta^2 * beta~_t
    cfg_scale: float | None = None  # classifier-free guidance: z then holds (cond, uncond) per row


def head_param_shapes(cfg: HeadCfg):
    """(name, shape) of every tensor in the packed fp32 weight blob, in order.
    Matrices are [out, in] row-major; each bias follows its matrix."""
    D, C, W, L = cfg.token_dim, cfg.cond_dim, cfg.width, cfg.n_blocks
    s = [("t1.w", (W, TIME_FEATURES)), ("t1.b", (W,)),
         ("t2.w", (W, W)), ("t2.b", (W,)),
         ("cond.w", (W, C)), ("cond.b", (W,)),
         ("in.w", (W, D)), ("in.b", (W,))]
    for l in range(L):
        s += [(f"blk{l}.mod.w", (3 * W, W)), (f"blk{l}.mod.b", (3 * W,)),
              (f"blk{l}.fc1.w", (W, W)), (f"blk{l}.fc1.b", (W,)),
              (f"blk{l}.fc2.w", (W, W)), (f"blk{l}.fc2.b", (W,))]
    s += [("fmod.w", (2 * W, W)), ("fmod.b", (2 * W,)),
          ("out.w", (2 * D, W)), ("out.b", (2 * D,))]
    return s


def silu(a):
    return a / (1.0 + np.exp(-a))


def layernorm(h, eps):
    """No affine; biased variance over the feature axis."""
    m = h.mean(axis=-1, keepdims=True)
    v = ((h - m) ** 2).mean(axis=-1, keepdims=True)
    return (h - m) / np.sqrt(v + eps)


def sincos_features(tval: float) -> np.ndarray:
    """256 sinusoidal features of a scalar time: [cos(t w_i), sin(t w_i)],
    w_i = 10000^(-i/128), i = 0..127."""
    half = TIME_FEATURES // 2
    w = np.exp(-math.log(10000.0) * np.arange(half, dtype=np.float64) / half)
    a = tval * w
    return np.concatenate([np.cos(a), np.sin(a)])


class Head:
    """Unpacked float64 copy of one head's weights, its schedule and its
    per-step time embedding E_t[t], t = 1..T."""

    def __init__(self, cfg: HeadCfg, blob: np.ndarray, sched: Schedule | None = None):
        self.cfg = cfg
        self.sched = sched if sched is not None else cosine_schedule(cfg.n_steps)
        assert self.sched.T == cfg.n_steps
        blob = np.asarray(blob)
        self.p = {}
        off = 0
        for name, shape in head_param_shapes(cfg):
            n = int(np.prod(shape))
            self.p[name] = blob[off:off + n].astype(np.float64).reshape(shape)
            off += n
        assert off == blob.shape[0], "weight blob size does not match the config"
        t_scale = cfg.t_scale if cfg.t_scale is not None else 1000.0 / cfg.n_steps
        self.time_emb = np.zeros((cfg.n_steps + 1, cfg.width))
        for t in range(1, cfg.n_steps + 1):
            f = sincos_features(t_scale * (t - 1))
            a = silu(self.p["t1.w"] @ f + self.p["t1.b"])
            self.time_emb[t] = self.p["t2.w"] @ a + self.p["t2.b"]

    def cond_embed(self, z):
        """e = W_c z + b_c, once per row (it does not depend on t).  With guidance z is
        [R, 2, C] (the conditional vector, then the unconditional one) and e [R, 2, W]."""
        z = np.asarray(z, dtype=np.float64)
        if self.cfg.cfg_scale is not None:
            z = z.reshape(z.shape[0], 2, self.cfg.cond_dim)
        return z @ self.p["cond.w"].T + self.p["cond.b"]

    def forward(self, x, t: int, e):
        """(eps_hat, v) = Head(x_t, t, z) for a batch of rows.  x [R,D], e = cond_embed(z).
        With classifier-free guidance (scale s): the head is evaluated with the conditional
        and with the unconditional vector on the same x_t,
        eps_hat = eps_u + s (eps_c - eps_u), and v is the conditional one."""
        if self.cfg.cfg_scale is not None:
            eh_c, v_c = self._forward(x, t, e[:, 0])
            eh_u, _ = self._forward(x, t, e[:, 1])
            return eh_u + self.cfg.cfg_scale * (eh_c - eh_u), v_c
        return self._forward(x, t, e)

    def _forward(self, x, t: int, e):
        p, cfg = self.p, self.cfg
        W, D = cfg.width, cfg.token_dim
        s = silu(self.time_emb[t] + e)
        h = x @ p["in.w"].T + p["in.b"]
        for l in range(cfg.n_blocks):
            mod = s @ p[f"blk{l}.mod.w"].T + p[f"blk{l}.mod.b"]
            sh, sc, g = mod[:, :W], mod[:, W:2 * W], mod[:, 2 * W:]
            u = layernorm(h, cfg.ln_eps) * (1.0 + sc) + sh
            u = silu(u @ p[f"blk{l}.fc1.w"].T + p[f"blk{l}.fc1.b"])
            u = u @ p[f"blk{l}.fc2.w"].T + p[f"blk{l}.fc2.b"]
            h = h + g * u
        mod = s @ p["fmod.w"].T + p["fmod.b"]
        sh, sc = mod[:, :W], mod[:, W:]
        o = (layernorm(h, cfg.ln_eps) * (1.0 + sc) + sh) @ p["out.w"].T + p["out.b"]
        eps_hat = o[:, :D]
        if cfg.eps_skip_gain != 0.0:
            eps_hat = eps_hat + cfg.eps_skip_gain * math.sqrt(1.0 - self.sched.abar[t]) * x
        return eps_hat, o[:, D:]


# --------------------------------------------------------------------------
# Gaussian transition (Eq. 3) and its log-density
# --------------------------------------------------------------------------
def head_transition(head: "Head", x, t: int, eps_hat, v):
    """(mu_t, log sigma_t^2) of the head's sampler: Eq. 3 (DDPM) or the DDIM step."""
    if head.cfg.sampler == "ddim":
        return ddim_transition_params(head.sched, x, t, eps_hat, head.cfg.ddim_eta)
    assert head.cfg.sampler == "ddpm"
    return transition_params(head.sched, x, t, eps_hat, v)


def transition_params(sched: Schedule, x, t: int, eps_hat, v):
    """mu_theta(x_t,t) and log of the diagonal of Sigma_theta(x_t,t):
    mu = (x_t - beta_t/sqrt(1-abar_t) eps_hat)/sqrt(alpha_t);
    log sigma^2 = f log beta_t + (1-f) log beta_tilde_t(clipped), f = (v+1)/2."""
    mu = (x - sched.beta[t] / math.sqrt(1.0 - sched.abar[t]) * eps_hat) / math.sqrt(sched.alpha[t])
    f = (v + 1.0) / 2.0
    logvar = f * sched.log_beta[t] + (1.0 - f) * sched.log_beta_tilde_clip[t]
    return mu, logvar


def ddim_transition_params(sched: Schedule, x, t: int, eps_hat, eta: float):
    """The DDIM reverse step as a Gaussian p(x_{t-1}|x_t) (appendix on other samplers; the
    published DDIM update): with x0_hat = (x_t - sqrt(1-abar_t) eps_hat)/sqrt(abar_t),
      mu = sqrt(abar_{t-1}) x0_hat + sqrt(1 - abar_{t-1} - sigma_t^2) eps_hat,
      sigma_t^2 = eta^2 (1-abar_{t-1})/(1-abar_t) (1 - abar_t/abar_{t-1}) = eta^2 beta~_t,
    the variance is fixed (the head's v is not used).  At t = 1 beta~_1 = 0 is replaced by
    beta~_2 as in the DDPM path (the final step has to be a density), and the coefficient of
    eps_hat under the root is clamped at 0."""
    var = eta * eta * math.exp(sched.log_beta_tilde_clip[t])
    x0_hat = (x - math.sqrt(1.0 - sched.abar[t]) * eps_hat) / math.sqrt(sched.abar[t])
    mu = math.sqrt(sched.abar[t - 1]) * x0_hat + math.sqrt(max(0.0, 1.0 - sched.abar[t - 1] - var)) * eps_hat
    return mu, np.full_like(np.asarray(x, dtype=np.float64), math.log(var))


def gaussian_logpdf(x, mu, logvar, tau: float = 1.0):
    """log N(x; mu, diag(tau^2 exp(logvar))), summed over the last axis."""
    ls2 = logvar + 2.0 * math.log(tau)
    return -0.5 * np.sum((x - mu) ** 2 / np.exp(ls2) + ls2 + LOG_2PI, axis=-1)


# --------------------------------------------------------------------------
# Lockstep denoising on an aligned trajectory (Sec. 3.2, App. A.2, Alg. 1)
# --------------------------------------------------------------------------
def summary_width(D: int) -> int:
    return 5 * D + 1


def denoise_lockstep(draft: Head, target: Head, z_q, z_p, seed: int,
                     row_offset: int = 0, tau: float = 1.0,
                     noise: np.ndarray | None = None, return_trace: bool = False):
    """Run both heads from x_T = eps_T down to t = 1 with shared eps_t.

    Returns summary [R, 5D+1] = [mu^p_1 | logvar^p_1 | mu^q_1 | logvar^q_1 |
    x_0 (draft sample) | log Sigma] and a dict with
      log_sigma_full : sum_{t=2..T} [log p(x^p_{t-1}|x^p_t) - log q(x^q_{t-1}|x^q_t)]
                       from the Gaussian pdfs themselves (Eq. 3, Eq. 6 left side)
      dist2          : ||x^q_0' - x^p_0'||^2 of the two models' own final samples.
    `noise` ([T+1, R, D], slot-indexed) replaces the Philox stream if given."""
    D, T = draft.cfg.token_dim, draft.cfg.n_steps
    assert target.cfg.token_dim == D and target.cfg.n_steps == T
    z_q = np.asarray(z_q, dtype=np.float64)
    z_p = np.asarray(z_p, dtype=np.float64)
    R = z_q.shape[0]
    rows = row_offset + np.arange(R, dtype=np.uint64)

    def eps(slot, stream=STREAM_TRAJ):
        if noise is not None:
            return np.asarray(noise[slot], dtype=np.float64)
        return normals(seed, rows, slot, stream, D)

    e_q = draft.cond_embed(z_q)
    e_p = target.cond_embed(z_p)
    x_q = eps(T)
    x_p = x_q.copy()                      # p(x_T^p) = q(x_T^q): same start
    log_sigma = np.zeros(R)               # Eq. 6, simplified form
    log_sigma_full = np.zeros(R)          # Eq. 6, from the pdfs
    trace = [] if return_trace else None
    for t in range(T, 0, -1):
        eh_q, v_q = draft.forward(x_q, t, e_q)
        eh_p, v_p = target.forward(x_p, t, e_p)
        mu_q, lv_q = head_transition(draft, x_q, t, eh_q, v_q)
        mu_p, lv_p = head_transition(target, x_p, t, eh_p, v_p)
        eps_t = eps(t - 1)
        xn_q = mu_q + tau * np.exp(0.5 * lv_q) * eps_t
        xn_p = mu_p + tau * np.exp(0.5 * lv_p) * eps_t
        if return_trace:
            trace.append(dict(t=t, x_q=x_q, x_p=x_p, mu_q=mu_q, mu_p=mu_p,
                              lv_q=lv_q, lv_p=lv_p, eh_q=eh_q, eh_p=eh_p))
        if t >= 2:
            log_sigma += 0.5 * np.sum(lv_q - lv_p, axis=-1)
            log_sigma_full += (gaussian_logpdf(xn_p, mu_p, lv_p, tau)
                               - gaussian_logpdf(xn_q, mu_q, lv_q, tau))
            x_q, x_p = xn_q, xn_p
        else:
            x0 = xn_q                      # the draft token that gets verified
            summary = np.concatenate(
                [mu_p, lv_p, mu_q, lv_q, x0, log_sigma[:, None]], axis=1)
            extras = dict(log_sigma_full=log_sigma_full,
                          dist2=np.sum((xn_q - xn_p) ** 2, axis=-1),
                          x0_p=xn_p)
            if return_trace:
                extras["trace"] = trace
            return summary, extras
    raise AssertionError("T must be >= 1")


# --------------------------------------------------------------------------
# The three path ratios the paper compares (Table 1; the appendix on the
# approximation of the ratio; the alignment ablation table)
# --------------------------------------------------------------------------
def denoise_ablation(draft: Head, target: Head, z_q, z_p, seed: int, row_offset: int = 0,
                     tau: float = 1.0, mode: int = RATIO_ALIGNED):
    """Both heads from x_T to t = 1 with the path ratio formed in one of three ways.

    RATIO_ALIGNED      two paths Y_p, Y_q driven by the same noise (Sec. 3.2): the method.
    RATIO_UNALIGNED    two paths with independent noise: the target draws x_T^p and every
                       eps^p_t from STREAM_TRAJ_P, the draft from STREAM_TRAJ as always.
    RATIO_SINGLE_PATH  one path, the draft's: the target head is evaluated at the draft's
                       x_t and its density at the draft's x_{t-1} (Eq. 2).
    In all three the token x_0 is the draft's and is shared (Eq. 4).

    Returns (summary, dist2).  summary [R, 5D+1] has the layout of denoise_lockstep; its
    last column is the log of the ratio over everything before the final step,
      log p(x_T^p) - log q(x_T^q) + sum_{t=2..T} [log p(x^p_{t-1}|x^p_t) - log q(x^q_{t-1}|x^q_t)]
    from the Gaussian densities themselves (Eq. 3; with x^p = x^q in the single-path mode),
    so that log_ratio(), verify() and resample() apply unchanged.  dist2 [R] is
    ||x^q_0 - x^p_0||^2 between the two heads' own final samples (the distance of the
    alignment ablation; Theorem 1): x^p_0 = mu^p_1 + tau sigma^p_1 eps^p_1."""
    assert mode in (RATIO_ALIGNED, RATIO_UNALIGNED, RATIO_SINGLE_PATH)
    D, T = draft.cfg.token_dim, draft.cfg.n_steps
    assert target.cfg.token_dim == D and target.cfg.n_steps == T
    z_q = np.asarray(z_q, dtype=np.float64)
    z_p = np.asarray(z_p, dtype=np.float64)
    R = z_q.shape[0]
    rows = row_offset + np.arange(R, dtype=np.uint64)
    stream_p = STREAM_TRAJ_P if mode == RATIO_UNALIGNED else STREAM_TRAJ
    e_q = draft.cond_embed(z_q)
    e_p = target.cond_embed(z_p)
    x_q = normals(seed, rows, T, STREAM_TRAJ, D)
    x_p = normals(seed, rows, T, stream_p, D)
    zero = np.zeros((R, D))
    log_r = gaussian_logpdf(x_p, zero, zero) - gaussian_logpdf(x_q, zero, zero)   # 0 unless the starts differ
    for t in range(T, 0, -1):
        if mode == RATIO_SINGLE_PATH:
            x_p = x_q                      # the target looks at the draft's state
        eh_q, v_q = draft.forward(x_q, t, e_q)
        eh_p, v_p = target.forward(x_p, t, e_p)
        mu_q, lv_q = head_transition(draft, x_q, t, eh_q, v_q)
        mu_p, lv_p = head_transition(target, x_p, t, eh_p, v_p)
        xn_q = mu_q + tau * np.exp(0.5 * lv_q) * normals(seed, rows, t - 1, STREAM_TRAJ, D)
        xn_p = mu_p + tau * np.exp(0.5 * lv_p) * normals(seed, rows, t - 1, stream_p, D)
        if t >= 2:
            at_p = xn_q if mode == RATIO_SINGLE_PATH else xn_p
            log_r = log_r + gaussian_logpdf(at_p, mu_p, lv_p, tau) - gaussian_logpdf(xn_q, mu_q, lv_q, tau)
            x_q, x_p = xn_q, xn_p
        else:
            summary = np.concatenate([mu_p, lv_p, mu_q, lv_q, xn_q, log_r[:, None]], axis=1)
            return summary, np.sum((xn_q - xn_p) ** 2, axis=-1)
    raise AssertionError("T must be >= 1")


# --------------------------------------------------------------------------
# Split-phase form of Alg. 1: the draft head position by position as the draft
# AR model advances, then the target head on all positions at once
# --------------------------------------------------------------------------
def head_trajectory(head: Head, z, global_rows, seed: int, tau: float = 1.0,
                    stream: int = STREAM_TRAJ):
    """One head alone from x_T = eps_T to x_0 for the rows `global_rows` (the
    counters that key the noise).  Returns mu_1, logvar_1, x_0 and
    1/2 sum_{t=2..T} sum_d log sigma^2_{t,d} (this head's half of Eq. 6)."""
    D, T = head.cfg.token_dim, head.cfg.n_steps
    z = np.asarray(z, dtype=np.float64)
    rows = np.asarray(global_rows, dtype=np.uint64)
    e = head.cond_embed(z)
    x = normals(seed, rows, T, stream, D)
    half = np.zeros(z.shape[0])
    for t in range(T, 0, -1):
        eh, v = head.forward(x, t, e)
        mu, lv = head_transition(head, x, t, eh, v)
        xn = mu + tau * np.exp(0.5 * lv) * normals(seed, rows, t - 1, stream, D)
        if t >= 2:
            half += 0.5 * np.sum(lv, axis=-1)
            x = xn
        else:
            return dict(mu1=mu, lv1=lv, x0=xn, half_logvar=half)
    raise AssertionError("T must be >= 1")


def denoise_draft(draft: Head, z_q_pos, gamma: int, position: int, seed: int,
                  row_offset: int, tau: float, summary: np.ndarray):
    """Draft phase for ONE position (0-based) of every group (Alg. 1, the loop
    "for i = 1..gamma: x_i ~ q_i").  z_q_pos: [G, C].  Fills, in the rows
    g*gamma + position of `summary` ([G*gamma, 5D+1], in place): mu^q_1,
    logvar^q_1, the draft token x_0, and the draft's half of log Sigma in the
    last column.  Noise counters are the same global rows as in the lockstep form."""
    D = draft.cfg.token_dim
    G = np.asarray(z_q_pos).shape[0]
    local = np.arange(G, dtype=np.int64) * gamma + position
    tr = head_trajectory(draft, z_q_pos, row_offset + local.astype(np.uint64), seed, tau)
    summary[local, 2 * D:3 * D] = tr["mu1"]
    summary[local, 3 * D:4 * D] = tr["lv1"]
    summary[local, 4 * D:5 * D] = tr["x0"]
    summary[local, 5 * D] = tr["half_logvar"]
    return tr["x0"]


def denoise_target(target: Head, z_p, seed: int, row_offset: int, tau: float,
                   summary: np.ndarray):
    """Target phase for all R = G*gamma rows at once (Alg. 1, "compute
    p_1..p_gamma in parallel", with the draft's eps_t regenerated from the
    counters).  z_p: [R, C].  Fills mu^p_1, logvar^p_1 and turns the last
    column into log Sigma = (draft half) - (target half)  (Eq. 6)."""
    D = target.cfg.token_dim
    R = np.asarray(z_p).shape[0]
    tr = head_trajectory(target, z_p, row_offset + np.arange(R, dtype=np.uint64), seed, tau)
    summary[:, 0:D] = tr["mu1"]
    summary[:, D:2 * D] = tr["lv1"]
    summary[:, 5 * D] = summary[:, 5 * D] - tr["half_logvar"]


def sample(head: Head, z, seed: int, row_offset: int = 0, tau: float = 1.0,
           stream: int = STREAM_TRAJ):
    """Plain sampling x_0 ~ head(.|z) for rows row_offset.. (target-only mode:
    pre-filling, and the token from p_{gamma+1} that Alg. 1 returns when all
    gamma drafts are accepted; that one uses STREAM_BONUS and group indices)."""
    R = np.asarray(z).shape[0]
    return head_trajectory(head, z, row_offset + np.arange(R, dtype=np.uint64), seed, tau, stream)["x0"]


def append_bonus(tokens, n_out, n_accept, bonus, gamma: int):
    """Groups whose gamma drafts were all accepted also emit the target's own
    sample for position gamma+1 (Alg. 1, last line).  In place; returns n_out."""
    tokens = np.asarray(tokens); n_out = np.asarray(n_out)
    full = np.asarray(n_accept) == gamma
    tokens[full, gamma, :] = np.asarray(bonus)[full]
    n_out[full] = gamma + 1
    return n_out


def split_summary(summary, D: int):
    s = np.asarray(summary, dtype=np.float64)
    return (s[:, 0:D], s[:, D:2 * D], s[:, 2 * D:3 * D], s[:, 3 * D:4 * D],
            s[:, 4 * D:5 * D], s[:, 5 * D])


# --------------------------------------------------------------------------
# Accept test and first-reject scan (Alg. 1; Eq. 7)
# --------------------------------------------------------------------------
def log_ratio(summary, D: int, tau: float = 1.0):
    """log of Sigma * p(x0|x1^p) / q(x0|x1^q) per row."""
    mu_p, lv_p, mu_q, lv_q, x0, ls = split_summary(summary, D)
    return ls + gaussian_logpdf(x0, mu_p, lv_p, tau) - gaussian_logpdf(x0, mu_q, lv_q, tau)


def verify(summary, n_groups: int, gamma: int, seed: int, row_offset: int = 0,
           tau: float = 1.0, D: int | None = None, u: np.ndarray | None = None):
    """n_accept[g] = number of leading rows of group g with r_i <= ratio_i.
    Returns (n_accept int32 [G], log_ratio [R], mask uint8 [R], log_u [R])."""
    summary = np.asarray(summary, dtype=np.float64)
    if D is None:
        D = (summary.shape[1] - 1) // 5
    R = n_groups * gamma
    assert summary.shape[0] == R
    ell = log_ratio(summary, D, tau)
    ell = np.where(np.isfinite(ell), ell, -np.inf)
    if u is None:
        rows = row_offset + np.arange(R, dtype=np.uint64)
        u = uniforms(seed, rows, 0, STREAM_ACCEPT_U)
    log_u = np.log(u)
    mask = (log_u <= ell)
    n_acc = np.full(n_groups, gamma, dtype=np.int32)
    for g in range(n_groups):
        for i in range(gamma):
            if not mask[g * gamma + i]:
                n_acc[g] = i
                break
    return n_acc, ell, mask.astype(np.uint8), log_u


# --------------------------------------------------------------------------
# Acceptance-rejection resampling from max(0, p - q)/Z (Sec. 3.3, Cor. 1)
# --------------------------------------------------------------------------
FLAG_CAP = 1        # max_trips reached: last proposal emitted
FLAG_NONFINITE = 2  # a non-finite log-ratio was met and treated as alpha_s = 0


def resample_threshold(x, mu_p, lv_p, mu_q, lv_q, log_sigma, tau: float = 1.0):
    """alpha_s = max(0, Sigma p(x|x1^p) - q(x|x1^q)) / (Sigma p(x|x1^p))
    evaluated as max(0, 1 - exp(a)), a = log q - log Sigma - log p."""
    a = gaussian_logpdf(x, mu_q, lv_q, tau) - log_sigma - gaussian_logpdf(x, mu_p, lv_p, tau)
    return np.where(a < 0.0, -np.expm1(np.minimum(a, 0.0)), 0.0), a


def resample(summary, n_accept, n_groups: int, gamma: int, seed: int,
             row_offset: int = 0, tau: float = 1.0, max_trips: int = 1024,
             D: int | None = None):
    """For each group with n < gamma: at the first rejected row, propose
    x' = mu^p_1 + tau sigma^p_1 eps'_k and accept when eps_k <= alpha_s
    (trial k = 0, 1, ...; all groups still looping take trial k together).
    Emits tokens [G, gamma+1, D] = [x_1..x_n, x'] (unused slots 0),
    n_out [G] (n+1, or gamma when everything was accepted), trips [G], flags [G],
    and per-group lists of (alpha_s, u) per trial for tolerance-band checks."""
    summary = np.asarray(summary, dtype=np.float64)
    if D is None:
        D = (summary.shape[1] - 1) // 5
    mu_p, lv_p, mu_q, lv_q, x0, ls = split_summary(summary, D)
    n_accept = np.asarray(n_accept, dtype=np.int64)
    tokens = np.zeros((n_groups, gamma + 1, D))
    n_out = np.full(n_groups, gamma, dtype=np.int32)
    trips = np.zeros(n_groups, dtype=np.int32)
    flags = np.zeros(n_groups, dtype=np.uint32)
    records = [None] * n_groups
    for g in range(n_groups):
        n = int(n_accept[g])
        tokens[g, :n] = x0[g * gamma: g * gamma + n]
    pending = np.nonzero(n_accept < gamma)[0]          # groups that resample
    for g in pending:
        records[g] = []
    n_out[pending] = n_accept[pending] + 1
    for k in range(max_trips):
        if pending.size == 0:
            break
        j = pending * gamma + n_accept[pending]        # first rejected row of each
        rows = (row_offset + j).astype(np.uint64)
        e = normals(seed, rows, k, STREAM_RESAMPLE_N, D)
        xp = mu_p[j] + tau * np.exp(0.5 * lv_p[j]) * e
        a_s, a = resample_threshold(xp, mu_p[j], lv_p[j], mu_q[j], lv_q[j], ls[j], tau)
        bad = np.isnan(a)                              # +-inf are handled by the formula
        a_s = np.where(bad, 0.0, a_s)
        flags[pending[bad]] |= FLAG_NONFINITE
        uk = uniforms(seed, rows, k, STREAM_RESAMPLE_U)
        tokens[pending, n_accept[pending]] = xp        # last proposal so far
        trips[pending] = k + 1
        for i, g in enumerate(pending):
            records[g].append((float(a_s[i]), float(uk[i])))
        pending = pending[~(uk <= a_s)]
    flags[pending] |= FLAG_CAP                          # never accepted within max_trips
    return tokens, n_out, trips, flags, records


# --------------------------------------------------------------------------
# Mixture-of-Gaussians output heads (the appendix on other forms of the output
# distribution): p(x) = sum_k pi_k N(x; mu_k, Sigma_k), diagonal Sigma_k.  The
# densities are explicit, so the accept test uses p(x)/q(x) itself and the
# modified distribution max(0, p - q)/Z is sampled by acceptance-rejection with
# proposal p and threshold max(0, p(x) - q(x))/p(x).
# A mixture is (pi [R,K] >= 0, not necessarily summing to 1; mu [R,K,D]; logvar [R,K,D]).
# --------------------------------------------------------------------------
def gmm_logpdf(x, pi, mu, logvar):
    """log sum_k (pi_k / sum pi) N(x; mu_k, diag exp(logvar_k)) per row, by log-sum-exp."""
    x = np.asarray(x, dtype=np.float64); pi = np.asarray(pi, dtype=np.float64)
    mu = np.asarray(mu, dtype=np.float64); logvar = np.asarray(logvar, dtype=np.float64)
    comp = -0.5 * np.sum((x[:, None, :] - mu) ** 2 / np.exp(logvar) + logvar + LOG_2PI, axis=-1)   # [R,K]
    with np.errstate(divide="ignore"):
        a = comp + np.log(pi) - np.log(np.sum(pi, axis=1, keepdims=True))
    m = np.max(a, axis=1, keepdims=True)
    return (m + np.log(np.sum(np.exp(a - m), axis=1, keepdims=True)))[:, 0]


def gmm_pick(pi, u):
    """Component of each row for the uniform u: the first k whose running sum of pi reaches
    u * sum(pi).  The sums are taken in fp32, left to right, and compared in fp32, so that
    a device doing the same additions picks the same component."""
    pi32 = np.asarray(pi, dtype=np.float32)
    R, K = pi32.shape
    total = np.zeros(R, dtype=np.float32)
    for k in range(K):
        total = total + pi32[:, k]
    thr = np.asarray(u, dtype=np.float32) * total
    run = np.zeros(R, dtype=np.float32)
    pick = np.full(R, K - 1, dtype=np.int64)
    done = np.zeros(R, dtype=bool)
    for k in range(K):
        run = run + pi32[:, k]
        hit = (~done) & (run >= thr)
        pick[hit] = k
        done |= hit
    return pick


def gmm_sample(pi, mu, logvar, u, eps):
    """x = mu_k + sigma_k eps with k = gmm_pick(pi, u)."""
    k = gmm_pick(pi, u)
    r = np.arange(k.shape[0])
    mu = np.asarray(mu, dtype=np.float64); logvar = np.asarray(logvar, dtype=np.float64)
    return mu[r, k] + np.exp(0.5 * logvar[r, k]) * eps, k


def gmm_draft_sample(pi_q, mu_q, logvar_q, seed: int, row_offset: int = 0):
    """The draft tokens x_i ~ q_i: component from STREAM_GMM_PICK slot 0, noise from
    STREAM_TRAJ slot 0 (the counters of the row's final reverse step in the diffusion form)."""
    R, K, D = np.asarray(mu_q).shape
    rows = row_offset + np.arange(R, dtype=np.uint64)
    x, _ = gmm_sample(pi_q, mu_q, logvar_q, uniforms(seed, rows, 0, STREAM_GMM_PICK),
                      normals(seed, rows, 0, STREAM_TRAJ, D))
    return x


def gmm_verify(x, pi_p, mu_p, logvar_p, pi_q, mu_q, logvar_q, n_groups: int, gamma: int, seed: int,
               row_offset: int = 0):
    """Accept test r_i <= p_i(x_i)/q_i(x_i) and first-reject scan (Alg. 1 with explicit densities).
    Returns (n_accept [G], log_ratio [R], mask [R], log_u [R])."""
    R = n_groups * gamma
    ell = gmm_logpdf(x, pi_p, mu_p, logvar_p) - gmm_logpdf(x, pi_q, mu_q, logvar_q)
    ell = np.where(np.isfinite(ell), ell, -np.inf)
    rows = row_offset + np.arange(R, dtype=np.uint64)
    log_u = np.log(uniforms(seed, rows, 0, STREAM_ACCEPT_U))
    mask = log_u <= ell
    n_acc = np.full(n_groups, gamma, dtype=np.int32)
    for g in range(n_groups):
        for i in range(gamma):
            if not mask[g * gamma + i]:
                n_acc[g] = i
                break
    return n_acc, ell, mask.astype(np.uint8), log_u


def gmm_resample(x, n_accept, pi_p, mu_p, logvar_p, pi_q, mu_q, logvar_q, n_groups: int, gamma: int,
                 seed: int, row_offset: int = 0, max_trips: int = 1024):
    """At the first rejected row of each group: propose x' ~ p (component from STREAM_GMM_PICK
    slot 1+k, noise from STREAM_RESAMPLE_N slot k) and keep it when the uniform of
    STREAM_RESAMPLE_U slot k is <= alpha_s = max(0, p(x') - q(x'))/p(x').  Emits as resample():
    tokens [G, gamma+1, D], n_out, trips, flags, per-group (alpha_s, u) records."""
    x = np.asarray(x, dtype=np.float64)
    D = x.shape[1]
    n_accept = np.asarray(n_accept, dtype=np.int64)
    pi_p = np.asarray(pi_p); mu_p = np.asarray(mu_p); logvar_p = np.asarray(logvar_p)
    pi_q = np.asarray(pi_q); mu_q = np.asarray(mu_q); logvar_q = np.asarray(logvar_q)
    tokens = np.zeros((n_groups, gamma + 1, D))
    n_out = np.full(n_groups, gamma, dtype=np.int32)
    trips = np.zeros(n_groups, dtype=np.int32)
    flags = np.zeros(n_groups, dtype=np.uint32)
    records = [None] * n_groups
    for g in range(n_groups):
        tokens[g, :int(n_accept[g])] = x[g * gamma: g * gamma + int(n_accept[g])]
    pending = np.nonzero(n_accept < gamma)[0]
    for g in pending:
        records[g] = []
    n_out[pending] = n_accept[pending] + 1
    for k in range(max_trips):
        if pending.size == 0:
            break
        j = pending * gamma + n_accept[pending]
        rows = (row_offset + j).astype(np.uint64)
        xp, _ = gmm_sample(pi_p[j], mu_p[j], logvar_p[j], uniforms(seed, rows, 1 + k, STREAM_GMM_PICK),
                           normals(seed, rows, k, STREAM_RESAMPLE_N, D))
        a = gmm_logpdf(xp, pi_q[j], mu_q[j], logvar_q[j]) - gmm_logpdf(xp, pi_p[j], mu_p[j], logvar_p[j])
        bad = np.isnan(a)
        a_s = np.where(a < 0.0, -np.expm1(np.minimum(a, 0.0)), 0.0)
        a_s = np.where(bad, 0.0, a_s)
        flags[pending[bad]] |= FLAG_NONFINITE
        uk = uniforms(seed, rows, k, STREAM_RESAMPLE_U)
        tokens[pending, n_accept[pending]] = xp
        trips[pending] = k + 1
        for i, g in enumerate(pending):
            records[g].append((float(a_s[i]), float(uk[i])))
        pending = pending[~(uk <= a_s)]
    flags[pending] |= FLAG_CAP
    return tokens, n_out, trips, flags, records
