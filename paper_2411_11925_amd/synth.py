"""Seeded synthetic inputs: head weights, conditioning vectors, workload table.

This module only draws inputs.  It holds none of the method's arithmetic (no
schedule, no head forward, no densities, no RNG of the sampler) and imports
neither the HIP binding nor the oracle, so both sides can be fed from it.

The workloads stand in for the paper's MAR / xAR / Harmon runs (ImageNet
256x256 with 256 AR tokens per image, 512x512 with 1024; Sec. 4.1): same
shapes, random weights, Gaussian conditioning vectors.  No dataset item or
checkpoint is used.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

TIME_FEATURES = 256


@dataclass(frozen=True)
class HeadShape:
    token_dim: int
    cond_dim: int
    width: int
    n_blocks: int


def param_layout(h: HeadShape):
    """(name, shape, fan_in) of each tensor of the packed fp32 blob, in order.
    Matrices are [out, in] row-major and each bias follows its matrix."""
    D, C, W, L = h.token_dim, h.cond_dim, h.width, h.n_blocks
    out = [("t1.w", (W, TIME_FEATURES)), ("t1.b", (W,)),
           ("t2.w", (W, W)), ("t2.b", (W,)),
           ("cond.w", (W, C)), ("cond.b", (W,)),
           ("in.w", (W, D)), ("in.b", (W,))]
    for l in range(L):
        out += [(f"blk{l}.mod.w", (3 * W, W)), (f"blk{l}.mod.b", (3 * W,)),
                (f"blk{l}.fc1.w", (W, W)), (f"blk{l}.fc1.b", (W,)),
                (f"blk{l}.fc2.w", (W, W)), (f"blk{l}.fc2.b", (W,))]
    out += [("fmod.w", (2 * W, W)), ("fmod.b", (2 * W,)),
            ("out.w", (2 * D, W)), ("out.b", (2 * D,))]
    return out


def n_params(h: HeadShape) -> int:
    return sum(int(np.prod(s)) for _, s in param_layout(h))


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & (2**64 - 1), stream]))


def head_weights(h: HeadShape, seed: int, out_scale: float = 1.0,
                 bias_std: float = 0.0) -> np.ndarray:
    """Matrices ~ N(0, 1/fan_in) (the output layer scaled by `out_scale`),
    biases ~ N(0, bias_std^2).  Returns the packed fp32 blob."""
    g = _rng(seed, 16)
    parts = []
    for name, shape in param_layout(h):
        n = int(np.prod(shape))
        if len(shape) == 2:
            std = 1.0 / np.sqrt(shape[1])
            if name == "out.w":
                std *= out_scale
            parts.append((g.standard_normal(n) * std).astype(np.float32))
        else:
            b = g.standard_normal(n) * bias_std
            if name == "out.b":
                b *= out_scale
            parts.append(b.astype(np.float32))
    return np.concatenate(parts)


def perturbed_copy(blob: np.ndarray, h: HeadShape, seed: int, rel_std: float = 0.05,
                   out_scale: float = 1.0) -> np.ndarray:
    """blob + N(0, rel_std^2 / fan_in) on every matrix (biases unchanged); the
    output layer's perturbation is scaled by `out_scale` like the layer itself."""
    g = _rng(seed, 17)
    out = blob.astype(np.float32).copy()
    off = 0
    for name, shape in param_layout(h):
        n = int(np.prod(shape))
        if len(shape) == 2:
            std = rel_std / np.sqrt(shape[1]) * (out_scale if name == "out.w" else 1.0)
            out[off:off + n] += (g.standard_normal(n) * std).astype(np.float32)
        off += n
    return out


def bf16_round(a: np.ndarray) -> np.ndarray:
    """fp32 array rounded to the nearest bf16-representable value (ties to even)."""
    b = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    b = (b + np.uint64(0x7FFF) + ((b >> np.uint64(16)) & np.uint64(1))) & np.uint64(0xFFFF0000)
    return b.astype(np.uint32).view(np.float32).reshape(np.shape(a))


def cond_vectors(n_rows: int, cond_dim: int, seed: int, rho: float | None = None,
                 add_std: float | None = None):
    """z_q ~ N(0,I).  With `rho`: z_p = rho z_q + sqrt(1-rho^2) N(0,I);
    with `add_std`: z_p = z_q + N(0, add_std^2)."""
    g = _rng(seed, 18)
    z_q = g.standard_normal((n_rows, cond_dim))
    n = g.standard_normal((n_rows, cond_dim))
    if rho is not None:
        z_p = rho * z_q + np.sqrt(1.0 - rho * rho) * n
    else:
        z_p = z_q + (add_std if add_std is not None else 0.0) * n
    return z_q.astype(np.float32), z_p.astype(np.float32)


@dataclass(frozen=True)
class Workload:
    name: str
    target: HeadShape
    draft: HeadShape | None      # None: draft = perturbed copy of the target
    n_steps: int                 # T
    batch: int                   # images decoded together = groups per verify step
    gamma: int                   # draft tokens per verify step
    tokens_per_image: int
    rho: float | None            # cond correlation (None: additive 0.1 noise)
    out_scale: float             # std multiplier of the output layer (acceptance knob)
    eps_skip_gain: float         # input-to-output skip of the head: eps_hat = gain*sqrt(1-abar_t)*x_t + o
    gemm_dtype: str              # "f32" | "bf16"
    seed: int

    @property
    def rows_per_verify_step(self) -> int:
        return self.batch * self.gamma

    @property
    def rows_total(self) -> int:
        return self.batch * self.tokens_per_image

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)

    def heads(self, bias_std: float = 0.0, round_bf16: bool | None = None):
        """(target_blob, draft_blob, draft_shape) for this workload."""
        tb = head_weights(self.target, self.seed, self.out_scale, bias_std)
        if self.draft is None:
            ds = self.target
            db = perturbed_copy(tb, self.target, self.seed + 1, 0.05, self.out_scale)
        else:
            ds = self.draft
            db = head_weights(self.draft, self.seed + 1, self.out_scale, bias_std)
        if round_bf16 if round_bf16 is not None else (self.gemm_dtype == "bf16"):
            tb, db = bf16_round(tb), bf16_round(db)
        return tb, db, ds

    def conds(self, n_rows: int, row_offset: int = 0):
        """Conditioning vectors for global rows [row_offset, row_offset+n_rows).
        Rows are drawn in blocks of 64 keyed by the block index, so any
        block-aligned slice of the workload can be regenerated alone."""
        C = self.target.cond_dim
        assert row_offset % 64 == 0
        zq = np.empty((n_rows, C), dtype=np.float32)
        zp = np.empty((n_rows, C), dtype=np.float32)
        for b0 in range(0, n_rows, 64):
            n = min(64, n_rows - b0)
            blk = (row_offset + b0) // 64
            q, p = cond_vectors(64, C, self.seed * 1000003 + blk, rho=self.rho,
                                add_std=None if self.rho is not None else 0.1)
            zq[b0:b0 + n], zp[b0:b0 + n] = q[:n], p[:n]
        return zq, zp


_SEED = 0x5EED0000

WORKLOADS = {
    # tiny case the oracle finishes in seconds
    "tiny": Workload("tiny", HeadShape(16, 64, 128, 2), None, 10, 1, 2, 256,
                     None, 0.05, 1.0, "f32", _SEED + 1),
    # 256x256-shaped head (MAR-like: 256 tokens per image)
    "mar256": Workload("mar256", HeadShape(16, 768, 1024, 6), HeadShape(16, 768, 768, 6),
                       100, 64, 4, 256, 0.9, 0.002, 1.0, "bf16", _SEED + 2),
    # larger head
    "large": Workload("large", HeadShape(16, 1024, 1280, 8), HeadShape(16, 1024, 1024, 6),
                      100, 128, 4, 256, 0.9, 0.002, 1.0, "bf16", _SEED + 3),
    # 512x512-shaped: 1024 tokens per image
    "mar512": Workload("mar512", HeadShape(16, 1024, 1280, 8), HeadShape(16, 1024, 1024, 6),
                       100, 32, 8, 1024, 0.9, 0.002, 1.0, "bf16", _SEED + 4),
    # rejection-heavy stress case
    "reject": Workload("reject", HeadShape(16, 768, 1024, 6), HeadShape(16, 768, 768, 6),
                       100, 256, 8, 256, 0.5, 0.002, 1.0, "bf16", _SEED + 5),
}


def mixture_pair(n_rows: int, n_components: int, token_dim: int, seed: int, shift: float = 0.3,
                 row_offset: int = 0):
    """Parameters of a target and a draft mixture-of-Gaussians head for rows
    [row_offset, row_offset + n_rows): ((pi_p, mu_p, logvar_p), (pi_q, mu_q, logvar_q)), fp32,
    pi [n, K] unnormalised positive weights, mu / logvar [n, K, D].  The draft is the target
    with its means moved by `shift` standard deviations, its variances widened or narrowed
    by up to 35 % and its weights re-drawn around the target's - the kind of disagreement
    a smaller model has with a larger one.  Rows are drawn in blocks of 64 keyed by the
    block index, like the conditioning vectors."""
    assert row_offset % 64 == 0
    K, D = n_components, token_dim
    out = [np.empty((n_rows, K), np.float32), np.empty((n_rows, K, D), np.float32), np.empty((n_rows, K, D), np.float32),
           np.empty((n_rows, K), np.float32), np.empty((n_rows, K, D), np.float32), np.empty((n_rows, K, D), np.float32)]
    for b0 in range(0, n_rows, 64):
        n = min(64, n_rows - b0)
        g = _rng(seed * 1000003 + (row_offset + b0) // 64, 23)
        pi_p = g.uniform(0.2, 1.0, size=(64, K))
        mu_p = g.normal(size=(64, K, D))
        lv_p = g.uniform(-2.5, -0.5, size=(64, K, D))
        pi_q = pi_p * g.uniform(0.6, 1.4, size=(64, K))
        mu_q = mu_p + shift * np.exp(0.5 * lv_p) * g.normal(size=(64, K, D))
        lv_q = lv_p + g.uniform(-0.3, 0.3, size=(64, K, D))
        for dst, src in zip(out, (pi_p, mu_p, lv_p, pi_q, mu_q, lv_q)):
            dst[b0:b0 + n] = src[:n]
    return tuple(out[:3]), tuple(out[3:])
