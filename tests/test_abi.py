"""Host-side checks that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2411_11925_amd import binding
    return binding


def test_every_declared_symbol_is_exported(B):
    text = open(os.path.join(ROOT, "include", "csd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(csd_[a-z_0-9]+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert getattr(lib, name) is not None


def test_param_count_matches_generator(B):
    from paper_2411_11925_amd import synth as S
    for shape in (S.HeadShape(16, 64, 128, 2), S.HeadShape(16, 768, 1024, 6), S.HeadShape(8, 40, 192, 3)):
        cfg = B.make_cfg(shape.token_dim, shape.cond_dim, shape.width, shape.n_blocks, 10)
        assert B.csd_param_count(cfg) == S.n_params(shape)


@pytest.mark.parametrize("kw", [dict(token_dim=5), dict(width=100), dict(cond_dim=12), dict(n_blocks=0),
                                dict(n_steps=0), dict(gemm_dtype=7), dict(n_steps=5000)])
def test_invalid_configs_are_rejected(B, kw):
    base = dict(token_dim=16, cond_dim=64, width=128, n_blocks=2, n_steps=10)
    base.update(kw)
    cfg = B.make_cfg(**base)
    assert B.csd_param_count(cfg) == 0
    assert B.csd_last_error() != ""
    with pytest.raises(B.CsdError) as e:
        B.csd_init_head(cfg, np.zeros(4, dtype=np.float32))
    assert e.value.code == B.CSD_EINVAL


def test_argument_errors_without_device_work(B):
    lib = B._lib
    # verify / resample / rng validate shapes before any HIP call
    assert lib.csd_verify(None, 4, 0, 16, 0, 0, 1.0, None, None, None, None) == B.CSD_EINVAL
    assert lib.csd_verify(None, 4, 65, 16, 0, 0, 1.0, None, None, None, None) == B.CSD_EINVAL
    assert lib.csd_verify(None, 4, 4, 5, 0, 0, 1.0, None, None, None, None) == B.CSD_EINVAL
    assert lib.csd_verify(None, 4, 4, 16, 0, 0, 0.0, None, None, None, None) == B.CSD_EINVAL
    assert lib.csd_verify(None, 4, 4, 16, 0, 0, 1.0, None, None, None, None) == B.CSD_EINVAL   # NULL buffers
    assert "NULL" in B.csd_last_error()
    assert lib.csd_verify(None, 0, 4, 16, 0, 0, 1.0, None, None, None, None) == B.CSD_OK       # empty: no-op
    assert lib.csd_resample(None, None, 4, 4, 16, 0, 0, 1.0, 0, None, None, None, None, None) == B.CSD_EINVAL
    assert lib.csd_resample(None, None, 4, 4, 16, 0, 0, 1.0, 70000, None, None, None, None, None) == B.CSD_EINVAL
    assert lib.csd_resample(None, None, 0, 4, 16, 0, 0, 1.0, 8, None, None, None, None, None) == B.CSD_OK
    assert lib.csd_rng_normals(1, 0, 8, 0, 0, 6, None, None) == B.CSD_EINVAL
    assert lib.csd_rng_normals(1, 0, 8, 70000, 0, 8, None, None) == B.CSD_EINVAL
    assert lib.csd_rng_uniforms(1, 0, 0, 0, 0, None, None) == B.CSD_OK
    assert lib.csd_denoise_lockstep(None, None, None, None, 1, 1, 0, 0, 1.0, None, None, 0, None) == B.CSD_EINVAL
    assert lib.csd_head_eval(None, None, None, 1, 1, None, None, 0, None) == B.CSD_EINVAL
    assert lib.csd_denoise_draft(None, None, 1, 1, 0, 0, 0, 1.0, None, None, 0, None) == B.CSD_EINVAL
    assert lib.csd_denoise_target(None, None, None, 1, 1, 0, 0, 1.0, None, None, 0, None) == B.CSD_EINVAL
    assert lib.csd_sample(None, None, 1, 0, 0, 0, 1.0, None, None, 0, None) == B.CSD_EINVAL
    assert lib.csd_set_guidance(None, 1, 1.0) == B.CSD_EINVAL
    assert lib.csd_gmm_draft_sample(None, None, None, 4, 2, 16, 0, 0, None, None) == B.CSD_EINVAL
    assert lib.csd_gmm_verify(None, None, None, None, None, None, None, 4, 2, 2, 16, 0, 0, None, None, None, None) == B.CSD_EINVAL
    assert lib.csd_gmm_resample(None, None, None, None, None, None, None, None, 4, 2, 2, 16, 0, 0, 8, None, None, None, None, None) == B.CSD_EINVAL
    assert lib.csd_append_bonus(None, None, None, None, 4, 0, 16, None) == B.CSD_EINVAL
    assert lib.csd_append_bonus(None, None, None, None, 4, 4, 5, None) == B.CSD_EINVAL
    assert lib.csd_append_bonus(None, None, None, None, 4, 4, 16, None) == B.CSD_EINVAL      # NULL buffers
    assert lib.csd_append_bonus(None, None, None, None, 0, 4, 16, None) == B.CSD_OK          # empty: no-op
    assert lib.csd_workspace_bytes(None, None, 10) == 0
    assert lib.csd_ablation_workspace_bytes(None, None, 10, 2) == 0
    assert lib.csd_denoise_ablation(None, None, None, None, 1, 1, 0, 0, 1.0, 0, None, None, None, 0, None) == B.CSD_EINVAL
    assert b"NULL head" in lib.csd_last_error()
    lib.csd_free_head(None)


def test_bench_refuses_more_than_one_gpu():
    """The path has no cross-GPU step and every box has one GPU: bench.py says so and exits."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)
