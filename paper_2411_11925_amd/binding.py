"""ctypes binding of libcsd.so: argument marshalling only.

Every function has the name and meaning of its C entry point in include/csd.h;
all computation happens in the HIP kernels of the library.  PyTorch supplies
device memory and the stream.  Importing this module fails if the library has
not been built (python -m paper_2411_11925_amd.build): there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import (POINTER, Structure, byref, c_char_p, c_double, c_float, c_int, c_int32,
                    c_int64, c_size_t, c_uint64, c_void_p)

import numpy as np
import torch  # loaded first so that the library binds to the HIP runtime torch uses

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcsd.so")
if not os.path.exists(LIB_PATH):
    raise ImportError("libcsd.so is missing: run `python -m paper_2411_11925_amd.build` "
                      "(the HIP library is required; there is no CPU fallback)")
_lib = ctypes.CDLL(LIB_PATH)

CSD_OK, CSD_EINVAL, CSD_ENOMEM, CSD_EHIP, CSD_EUNSUPPORTED = 0, -1, -2, -3, -4
CSD_F32, CSD_BF16 = 0, 1
CSD_COSINE, CSD_TABLE = 0, 1
CSD_STREAM_TRAJ, CSD_STREAM_ACCEPT_U, CSD_STREAM_RESAMPLE_N, CSD_STREAM_RESAMPLE_U = 0, 1, 2, 3
CSD_STREAM_BONUS = 4
CSD_STREAM_TRAJ_P = 5
CSD_STREAM_GMM_PICK = 6
CSD_RATIO_ALIGNED, CSD_RATIO_UNALIGNED, CSD_RATIO_SINGLE_PATH = 0, 1, 2
CSD_SAMPLER_DDPM, CSD_SAMPLER_DDIM = 0, 1
CSD_FLAG_CAP, CSD_FLAG_NONFINITE = 1, 2

EXPORTS = ["csd_param_count", "csd_init_head", "csd_free_head", "csd_set_guidance", "csd_workspace_bytes",
           "csd_denoise_lockstep", "csd_ablation_workspace_bytes", "csd_denoise_ablation", "csd_denoise_draft", "csd_denoise_target", "csd_sample",
           "csd_verify", "csd_resample", "csd_append_bonus", "csd_gmm_draft_sample", "csd_gmm_verify", "csd_gmm_resample", "csd_head_eval",
           "csd_rng_normals", "csd_rng_uniforms", "csd_gemm_bf16", "csd_profile_enable", "csd_profile_read", "csd_last_error"]


class csd_head_cfg_t(Structure):
    _fields_ = [("token_dim", c_int32), ("cond_dim", c_int32), ("width", c_int32),
                ("n_blocks", c_int32), ("n_steps", c_int32), ("gemm_dtype", c_int32),
                ("schedule", c_int32), ("sampler", c_int32), ("alpha_bar", POINTER(c_double)),
                ("ln_eps", c_float), ("t_scale", c_float), ("eps_skip_gain", c_float),
                ("ddim_eta", c_float)]


_lib.csd_last_error.restype = c_char_p
_lib.csd_last_error.argtypes = []
_lib.csd_param_count.restype = c_size_t
_lib.csd_param_count.argtypes = [POINTER(csd_head_cfg_t)]
_lib.csd_init_head.restype = c_int
_lib.csd_init_head.argtypes = [POINTER(csd_head_cfg_t), c_void_p, c_size_t, c_int, POINTER(c_void_p)]
_lib.csd_free_head.restype = None
_lib.csd_free_head.argtypes = [c_void_p]
_lib.csd_set_guidance.restype = c_int
_lib.csd_set_guidance.argtypes = [c_void_p, c_int32, c_float]
_lib.csd_workspace_bytes.restype = c_size_t
_lib.csd_workspace_bytes.argtypes = [c_void_p, c_void_p, c_int64]
_lib.csd_denoise_lockstep.restype = c_int
_lib.csd_denoise_lockstep.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int32, c_uint64,
                                      c_uint64, c_float, c_void_p, c_void_p, c_size_t, c_void_p]
_lib.csd_ablation_workspace_bytes.restype = c_size_t
_lib.csd_ablation_workspace_bytes.argtypes = [c_void_p, c_void_p, c_int64, c_int32]
_lib.csd_denoise_ablation.restype = c_int
_lib.csd_denoise_ablation.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int32, c_uint64,
                                      c_uint64, c_float, c_int32, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
_lib.csd_denoise_draft.restype = c_int
_lib.csd_denoise_draft.argtypes = [c_void_p, c_void_p, c_int64, c_int32, c_int32, c_uint64, c_uint64, c_float,
                                   c_void_p, c_void_p, c_size_t, c_void_p]
_lib.csd_denoise_target.restype = c_int
_lib.csd_denoise_target.argtypes = [c_void_p, c_void_p, c_void_p, c_int64, c_int32, c_uint64, c_uint64, c_float,
                                    c_void_p, c_void_p, c_size_t, c_void_p]
_lib.csd_sample.restype = c_int
_lib.csd_sample.argtypes = [c_void_p, c_void_p, c_int64, c_uint64, c_uint64, c_int32, c_float, c_void_p, c_void_p,
                            c_size_t, c_void_p]
_lib.csd_append_bonus.restype = c_int
_lib.csd_append_bonus.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int32, c_int32, c_void_p]
_lib.csd_verify.restype = c_int
_lib.csd_verify.argtypes = [c_void_p, c_int64, c_int32, c_int32, c_uint64, c_uint64, c_float,
                            c_void_p, c_void_p, c_void_p, c_void_p]
_lib.csd_resample.restype = c_int
_lib.csd_resample.argtypes = [c_void_p, c_void_p, c_int64, c_int32, c_int32, c_uint64, c_uint64, c_float,
                              c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
_lib.csd_gmm_draft_sample.restype = c_int
_lib.csd_gmm_draft_sample.argtypes = [c_void_p, c_void_p, c_void_p, c_int64, c_int32, c_int32, c_uint64, c_uint64, c_void_p, c_void_p]
_lib.csd_gmm_verify.restype = c_int
_lib.csd_gmm_verify.argtypes = [c_void_p] * 7 + [c_int64, c_int32, c_int32, c_int32, c_uint64, c_uint64, c_void_p, c_void_p,
                                                 c_void_p, c_void_p]
_lib.csd_gmm_resample.restype = c_int
_lib.csd_gmm_resample.argtypes = [c_void_p] * 8 + [c_int64, c_int32, c_int32, c_int32, c_uint64, c_uint64, c_int32, c_void_p,
                                                   c_void_p, c_void_p, c_void_p, c_void_p]
_lib.csd_head_eval.restype = c_int
_lib.csd_head_eval.argtypes = [c_void_p, c_void_p, c_void_p, c_int32, c_int64, c_void_p, c_void_p,
                               c_size_t, c_void_p]
_lib.csd_rng_normals.restype = c_int
_lib.csd_rng_normals.argtypes = [c_uint64, c_uint64, c_int64, c_int32, c_int32, c_int32, c_void_p, c_void_p]
_lib.csd_rng_uniforms.restype = c_int
_lib.csd_rng_uniforms.argtypes = [c_uint64, c_uint64, c_int64, c_int32, c_int32, c_void_p, c_void_p]


_lib.csd_gemm_bf16.restype = c_int
_lib.csd_gemm_bf16.argtypes = [c_void_p, c_void_p, c_void_p, c_int64, c_int32, c_int32, c_int32, c_int32,
                               c_void_p, c_void_p, c_void_p]


_lib.csd_profile_enable.restype = c_int
_lib.csd_profile_enable.argtypes = [c_int32]
_lib.csd_profile_read.restype = c_int
_lib.csd_profile_read.argtypes = [POINTER(c_double), POINTER(c_int64), POINTER(c_double), POINTER(c_double)]


class CsdError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__("libcsd error %d: %s" % (code, csd_last_error()))


def csd_last_error() -> str:
    return (_lib.csd_last_error() or b"").decode()


def _check(rc: int):
    if rc != CSD_OK:
        raise CsdError(rc)


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def make_cfg(token_dim, cond_dim, width, n_blocks, n_steps, gemm_dtype=CSD_F32, alpha_bar=None,
             ln_eps=0.0, t_scale=0.0, eps_skip_gain=0.0, ddim_eta=None):
    """ddim_eta=None: the DDPM sampler; a positive value: DDIM with sigma_t^2 = eta^2 beta~_t."""
    cfg = csd_head_cfg_t(token_dim, cond_dim, width, n_blocks, n_steps, gemm_dtype,
                         CSD_COSINE if alpha_bar is None else CSD_TABLE,
                         CSD_SAMPLER_DDPM if ddim_eta is None else CSD_SAMPLER_DDIM, None,
                         ln_eps, t_scale, eps_skip_gain, 0.0 if ddim_eta is None else ddim_eta)
    if alpha_bar is not None:
        arr = np.ascontiguousarray(alpha_bar, dtype=np.float64)
        cfg._keep = arr
        cfg.alpha_bar = arr.ctypes.data_as(POINTER(c_double))
    return cfg


def csd_param_count(cfg: csd_head_cfg_t) -> int:
    return int(_lib.csd_param_count(byref(cfg)))


class Head:
    """Owner of a csd_head_t*; freed with csd_free_head."""

    def __init__(self, handle: int, cfg: csd_head_cfg_t, device: int):
        self.handle, self.cfg, self.device = handle, cfg, device
        self.reps = 1          # conditioning vectors per row: 2 with classifier-free guidance

    def free(self):
        if self.handle:
            _lib.csd_free_head(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def csd_init_head(cfg: csd_head_cfg_t, weights_host: np.ndarray, device: int = 0) -> Head:
    w = np.ascontiguousarray(weights_host, dtype=np.float32)
    out = c_void_p()
    _check(_lib.csd_init_head(byref(cfg), w.ctypes.data, w.size, device, byref(out)))
    return Head(out.value, cfg, device)


def csd_free_head(head: Head):
    head.free()


def csd_set_guidance(head: Head, enabled: bool, scale: float = 1.0):
    _check(_lib.csd_set_guidance(head.handle, 1 if enabled else 0, scale))
    head.reps = 2 if enabled else 1


def csd_workspace_bytes(draft: Head | None, target: Head | None, n_rows: int) -> int:
    return int(_lib.csd_workspace_bytes(draft.handle if draft else None, target.handle if target else None, n_rows))


def _workspace(draft, target, n_rows, device):
    n = csd_workspace_bytes(draft, target, n_rows)
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device), n


def csd_denoise_lockstep(draft: Head, target: Head, z_q: torch.Tensor, z_p: torch.Tensor, n_groups: int,
                         gamma: int, seed: int, row_offset: int = 0, temperature: float = 1.0,
                         summary: torch.Tensor | None = None, workspace: torch.Tensor | None = None,
                         stream=None) -> torch.Tensor:
    R, D = n_groups * gamma, draft.cfg.token_dim
    assert z_q.is_cuda and z_p.is_cuda and z_q.dtype == torch.float32 and z_p.dtype == torch.float32
    assert z_q.is_contiguous() and z_p.is_contiguous()
    assert z_q.numel() == R * draft.reps * draft.cfg.cond_dim and z_p.numel() == R * target.reps * target.cfg.cond_dim
    if summary is None:
        summary = torch.empty((R, 5 * D + 1), dtype=torch.float32, device=z_q.device)
    assert summary.is_contiguous() and tuple(summary.shape) == (R, 5 * D + 1) and summary.dtype == torch.float32
    if workspace is None:
        workspace, _ = _workspace(draft, target, R, z_q.device)
    _check(_lib.csd_denoise_lockstep(draft.handle, target.handle, _ptr(z_q), _ptr(z_p), n_groups, gamma,
                                     seed, row_offset, temperature, _ptr(summary), _ptr(workspace),
                                     workspace.numel(), _stream(stream)))
    return summary


def csd_ablation_workspace_bytes(draft: Head, target: Head, n_rows: int, ratio_mode: int) -> int:
    return int(_lib.csd_ablation_workspace_bytes(draft.handle, target.handle, n_rows, ratio_mode))


def csd_denoise_ablation(draft: Head, target: Head, z_q: torch.Tensor, z_p: torch.Tensor, n_groups: int,
                         gamma: int, seed: int, row_offset: int, temperature: float, ratio_mode: int,
                         summary: torch.Tensor | None = None, dist2: torch.Tensor | None = None,
                         workspace: torch.Tensor | None = None, stream=None):
    """Returns (summary, dist2)."""
    R, D = n_groups * gamma, draft.cfg.token_dim
    assert z_q.is_cuda and z_p.is_cuda and z_q.dtype == torch.float32 and z_p.dtype == torch.float32
    assert z_q.is_contiguous() and z_p.is_contiguous()
    assert z_q.numel() == R * draft.reps * draft.cfg.cond_dim and z_p.numel() == R * target.reps * target.cfg.cond_dim
    if summary is None:
        summary = torch.empty((R, 5 * D + 1), dtype=torch.float32, device=z_q.device)
    if dist2 is None:
        dist2 = torch.empty((R,), dtype=torch.float32, device=z_q.device)
    assert summary.is_contiguous() and tuple(summary.shape) == (R, 5 * D + 1) and summary.dtype == torch.float32
    assert dist2.is_contiguous() and dist2.numel() == R and dist2.dtype == torch.float32
    if workspace is None:
        n = csd_ablation_workspace_bytes(draft, target, R, ratio_mode)
        workspace = torch.empty(max(n, 256), dtype=torch.uint8, device=z_q.device)
    _check(_lib.csd_denoise_ablation(draft.handle, target.handle, _ptr(z_q), _ptr(z_p), n_groups, gamma, seed,
                                     row_offset, temperature, ratio_mode, _ptr(summary), _ptr(dist2), _ptr(workspace),
                                     workspace.numel(), _stream(stream)))
    return summary, dist2


def csd_denoise_draft(draft: Head, z_q: torch.Tensor, n_groups: int, gamma: int, position: int, seed: int,
                      row_offset: int, temperature: float, summary: torch.Tensor,
                      workspace: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    D = draft.cfg.token_dim
    assert z_q.is_cuda and z_q.dtype == torch.float32 and z_q.is_contiguous()
    assert z_q.numel() == n_groups * draft.reps * draft.cfg.cond_dim
    assert summary.is_cuda and summary.is_contiguous() and summary.dtype == torch.float32
    assert tuple(summary.shape) == (n_groups * gamma, 5 * D + 1)
    if workspace is None:
        workspace, _ = _workspace(draft, None, n_groups, z_q.device)
    _check(_lib.csd_denoise_draft(draft.handle, _ptr(z_q), n_groups, gamma, position, seed, row_offset, temperature,
                                  _ptr(summary), _ptr(workspace), workspace.numel(), _stream(stream)))
    return summary


def csd_denoise_target(target: Head, draft: Head, z_p: torch.Tensor, n_groups: int, gamma: int, seed: int,
                       row_offset: int, temperature: float, summary: torch.Tensor,
                       workspace: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    R, D = n_groups * gamma, target.cfg.token_dim
    assert z_p.is_cuda and z_p.dtype == torch.float32 and z_p.is_contiguous()
    assert z_p.numel() == R * target.reps * target.cfg.cond_dim
    assert summary.is_cuda and summary.is_contiguous() and summary.dtype == torch.float32
    assert tuple(summary.shape) == (R, 5 * D + 1)
    if workspace is None:
        workspace, _ = _workspace(None, target, R, z_p.device)
    _check(_lib.csd_denoise_target(target.handle, draft.handle, _ptr(z_p), n_groups, gamma, seed, row_offset,
                                   temperature, _ptr(summary), _ptr(workspace), workspace.numel(), _stream(stream)))
    return summary


def csd_sample(head: Head, z: torch.Tensor, seed: int, row_offset: int = 0, rng_stream: int = CSD_STREAM_TRAJ,
               temperature: float = 1.0, tokens: torch.Tensor | None = None,
               workspace: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    n, D = z.shape[0], head.cfg.token_dim
    assert z.is_cuda and z.dtype == torch.float32 and z.is_contiguous()
    assert z.numel() == n * head.reps * head.cfg.cond_dim
    if tokens is None:
        tokens = torch.empty((n, D), dtype=torch.float32, device=z.device)
    assert tokens.is_cuda and tokens.is_contiguous() and tokens.dtype == torch.float32 and tuple(tokens.shape) == (n, D)
    if workspace is None:
        workspace, _ = _workspace(head, None, n, z.device)
    _check(_lib.csd_sample(head.handle, _ptr(z), n, seed, row_offset, rng_stream, temperature, _ptr(tokens),
                           _ptr(workspace), workspace.numel(), _stream(stream)))
    return tokens


def csd_append_bonus(tokens: torch.Tensor, n_out: torch.Tensor, n_accept: torch.Tensor, bonus: torch.Tensor,
                     gamma: int, stream=None):
    G, D = n_accept.numel(), bonus.shape[1]
    assert tokens.is_cuda and tokens.is_contiguous() and tokens.dtype == torch.float32
    assert tuple(tokens.shape) == (G, gamma + 1, D) and tuple(bonus.shape) == (G, D)
    assert bonus.is_cuda and bonus.is_contiguous() and bonus.dtype == torch.float32
    assert n_out.dtype == torch.int32 and n_accept.dtype == torch.int32 and n_out.numel() == G
    _check(_lib.csd_append_bonus(_ptr(tokens), _ptr(n_out), _ptr(n_accept), _ptr(bonus), G, gamma, D, _stream(stream)))
    return tokens, n_out


def csd_verify(summary: torch.Tensor, n_groups: int, gamma: int, token_dim: int, seed: int,
               row_offset: int = 0, temperature: float = 1.0, want_log_ratio: bool = True,
               want_mask: bool = True, stream=None):
    R = n_groups * gamma
    assert summary.is_cuda and summary.is_contiguous() and summary.dtype == torch.float32
    assert tuple(summary.shape) == (R, 5 * token_dim + 1)
    dev = summary.device
    n_accept = torch.empty(n_groups, dtype=torch.int32, device=dev)
    log_ratio = torch.empty(R, dtype=torch.float32, device=dev) if want_log_ratio else None
    mask = torch.empty(R, dtype=torch.uint8, device=dev) if want_mask else None
    _check(_lib.csd_verify(_ptr(summary), n_groups, gamma, token_dim, seed, row_offset, temperature,
                           _ptr(n_accept), _ptr(log_ratio), _ptr(mask), _stream(stream)))
    return n_accept, log_ratio, mask


def csd_resample(summary: torch.Tensor, n_accept: torch.Tensor, n_groups: int, gamma: int, token_dim: int,
                 seed: int, row_offset: int = 0, temperature: float = 1.0, max_trips: int = 1024, stream=None):
    R = n_groups * gamma
    assert summary.is_cuda and summary.is_contiguous() and summary.dtype == torch.float32
    assert tuple(summary.shape) == (R, 5 * token_dim + 1)
    assert n_accept.is_cuda and n_accept.dtype == torch.int32 and n_accept.numel() == n_groups
    dev = summary.device
    tokens = torch.empty((n_groups, gamma + 1, token_dim), dtype=torch.float32, device=dev)
    n_out = torch.empty(n_groups, dtype=torch.int32, device=dev)
    trips = torch.empty(n_groups, dtype=torch.int32, device=dev)
    flags = torch.empty(n_groups, dtype=torch.int32, device=dev)
    _check(_lib.csd_resample(_ptr(summary), _ptr(n_accept), n_groups, gamma, token_dim, seed, row_offset,
                             temperature, max_trips, _ptr(tokens), _ptr(n_out), _ptr(trips), _ptr(flags),
                             _stream(stream)))
    return tokens, n_out, trips, flags


def _mix(m, R):
    """(pi [R,K], mu [R,K,D], logvar [R,K,D]) -> checked, with K and D."""
    pi, mu, lv = m
    K, D = mu.shape[1], mu.shape[2]
    for t, shape in ((pi, (R, K)), (mu, (R, K, D)), (lv, (R, K, D))):
        assert t.is_cuda and t.is_contiguous() and t.dtype == torch.float32 and tuple(t.shape) == shape
    return K, D


def csd_gmm_draft_sample(mix_q, seed: int, row_offset: int = 0, stream=None) -> torch.Tensor:
    R = mix_q[0].shape[0]
    K, D = _mix(mix_q, R)
    x = torch.empty((R, D), dtype=torch.float32, device=mix_q[0].device)
    _check(_lib.csd_gmm_draft_sample(_ptr(mix_q[0]), _ptr(mix_q[1]), _ptr(mix_q[2]), R, K, D, seed, row_offset, _ptr(x),
                                     _stream(stream)))
    return x


def csd_gmm_verify(x: torch.Tensor, mix_p, mix_q, n_groups: int, gamma: int, seed: int, row_offset: int = 0, stream=None):
    """Returns (n_accept, log_ratio, accept_mask)."""
    R = n_groups * gamma
    K, D = _mix(mix_p, R)
    assert _mix(mix_q, R) == (K, D)
    assert x.is_cuda and x.is_contiguous() and x.dtype == torch.float32 and tuple(x.shape) == (R, D)
    dev = x.device
    n_accept = torch.empty(n_groups, dtype=torch.int32, device=dev)
    log_ratio = torch.empty(R, dtype=torch.float32, device=dev)
    mask = torch.empty(R, dtype=torch.uint8, device=dev)
    _check(_lib.csd_gmm_verify(_ptr(x), *[_ptr(t) for t in mix_p], *[_ptr(t) for t in mix_q], n_groups, gamma, K, D, seed,
                               row_offset, _ptr(n_accept), _ptr(log_ratio), _ptr(mask), _stream(stream)))
    return n_accept, log_ratio, mask


def csd_gmm_resample(x: torch.Tensor, n_accept: torch.Tensor, mix_p, mix_q, n_groups: int, gamma: int, seed: int,
                     row_offset: int = 0, max_trips: int = 1024, stream=None):
    """Returns (tokens [G, gamma+1, D], n_out, trips, flags)."""
    R = n_groups * gamma
    K, D = _mix(mix_p, R)
    assert _mix(mix_q, R) == (K, D)
    assert x.is_cuda and x.is_contiguous() and x.dtype == torch.float32 and tuple(x.shape) == (R, D)
    assert n_accept.is_cuda and n_accept.dtype == torch.int32 and n_accept.numel() == n_groups
    dev = x.device
    tokens = torch.empty((n_groups, gamma + 1, D), dtype=torch.float32, device=dev)
    n_out = torch.empty(n_groups, dtype=torch.int32, device=dev)
    trips = torch.empty(n_groups, dtype=torch.int32, device=dev)
    flags = torch.empty(n_groups, dtype=torch.int32, device=dev)
    _check(_lib.csd_gmm_resample(_ptr(x), _ptr(n_accept), *[_ptr(t) for t in mix_p], *[_ptr(t) for t in mix_q], n_groups,
                                 gamma, K, D, seed, row_offset, max_trips, _ptr(tokens), _ptr(n_out), _ptr(trips),
                                 _ptr(flags), _stream(stream)))
    return tokens, n_out, trips, flags


def csd_head_eval(head: Head, x: torch.Tensor, z: torch.Tensor, t: int, workspace: torch.Tensor | None = None,
                  stream=None) -> torch.Tensor:
    R, D = x.shape[0], head.cfg.token_dim
    assert x.is_cuda and z.is_cuda and x.dtype == torch.float32 and z.dtype == torch.float32
    assert x.is_contiguous() and z.is_contiguous()
    assert tuple(x.shape) == (R, D) and z.numel() == R * head.reps * head.cfg.cond_dim
    out = torch.empty((R, 2 * D), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace, _ = _workspace(head, None, R, x.device)
    _check(_lib.csd_head_eval(head.handle, _ptr(x), _ptr(z), t, R, _ptr(out), _ptr(workspace),
                              workspace.numel(), _stream(stream)))
    return out


def csd_rng_normals(seed: int, row_offset: int, n_rows: int, slot: int, stream_id: int, n_cols: int,
                    device="cuda:0", stream=None) -> torch.Tensor:
    out = torch.empty((n_rows, n_cols), dtype=torch.float32, device=device)
    _check(_lib.csd_rng_normals(seed, row_offset, n_rows, slot, stream_id, n_cols, _ptr(out), _stream(stream)))
    return out


def csd_rng_uniforms(seed: int, row_offset: int, n_rows: int, slot: int, stream_id: int,
                     device="cuda:0", stream=None) -> torch.Tensor:
    out = torch.empty(n_rows, dtype=torch.float32, device=device)
    _check(_lib.csd_rng_uniforms(seed, row_offset, n_rows, slot, stream_id, _ptr(out), _stream(stream)))
    return out


def csd_gemm_bf16(A: torch.Tensor, B: torch.Tensor, bias: torch.Tensor, epilogue: int = 0, out_f32: bool = False,
                  C: torch.Tensor | None = None, gate: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """A [M,K], B [N,K], gate [M,N]: torch.bfloat16 on the device; bias fp32 [N]."""
    M, K = A.shape
    N = B.shape[0]
    assert A.dtype == torch.bfloat16 and B.dtype == torch.bfloat16 and bias.dtype == torch.float32
    assert A.is_contiguous() and B.is_contiguous() and B.shape[1] == K and bias.numel() == N
    if epilogue == 2:
        assert C is not None and C.dtype == torch.float32 and gate is not None and gate.dtype == torch.bfloat16
        assert gate.is_contiguous() and tuple(gate.shape) == (M, N)
    elif C is None:
        C = torch.empty((M, N), dtype=torch.float32 if out_f32 else torch.bfloat16, device=A.device)
    assert C.is_contiguous() and tuple(C.shape) == (M, N)
    _check(_lib.csd_gemm_bf16(_ptr(A), _ptr(B), _ptr(bias), M, N, K, epilogue,
                              1 if C.dtype == torch.float32 else 0, _ptr(C), _ptr(gate), _stream(stream)))
    return C


def csd_profile_enable(max_launches: int):
    _check(_lib.csd_profile_enable(max_launches))


def csd_profile_read():
    """(sum of event-to-event milliseconds, launches timed, sum of algorithmic flops,
    sum of first-workgroup-start to last-workgroup-end milliseconds or 0.0)."""
    ms, n, fl, dev = c_double(), c_int64(), c_double(), c_double()
    _check(_lib.csd_profile_read(byref(ms), byref(n), byref(fl), byref(dev)))
    return ms.value, n.value, fl.value, dev.value
