"""Benchmark of the hot path: verified tokens/s of denoise + verify + resample.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload mar256] [--dtype bf16]

A step is one pass of the whole hot path (csd_denoise_lockstep, csd_verify,
csd_resample) over all rows of the workload, inputs resident in HBM.  Prints one
JSON line with the throughput, the roofline of the dominant kernel (the modulation
GEMM, timed by hipEvents inside the timed region) and the fp64 oracle timed on a
bounded row sample on the host cores.  One GPU only.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"bf16": 2500.0, "f32": 157.3}     # MI355X dense peak, TFLOP/s


def head_flops_per_row_step(sh):
    W, L, D = sh.width, sh.n_blocks, sh.token_dim
    return (10 * L + 4) * W * W + 6 * D * W


def measured_traffic(workload, dtype, rows):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter
    summary of this same workload (profiles/), or None if there is none for it."""
    path = os.path.join(ROOT, "profiles", "%s_%s_mod_gemm_traffic.txt" % (workload, dtype))
    if not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        if ":" in line and not line.startswith("#"):
            k, v = line.split(":", 1)
            try:
                vals[k.strip()] = float(v.split()[0])
            except (ValueError, IndexError):
                pass
    if vals.get("rows_per_step") != rows or "traffic_bytes_per_launch" not in vals:
        return None
    return vals["traffic_bytes_per_launch"]


def gmm_bench(a, np, torch, B, S):
    """Mixture-of-Gaussians heads (the appendix on other forms of the output distribution): the whole
    path is three row kernels over the mixture parameters, bound by HBM.  One JSON line."""
    K, D, gamma, seed, dev = a.gmm_components, 16, 4, 1234, "cuda:0"
    R = (a.rows or (1 << 20)) // gamma * gamma
    G = R // gamma
    base_p, base_q = S.mixture_pair(4096, K, D, seed)           # tiled: 4096 distinct rows
    rep = (R + 4095) // 4096
    tile = lambda m: tuple(torch.from_numpy(t).to(dev).repeat((rep,) + (1,) * (t.ndim - 1))[:R].contiguous() for t in m)
    mp, mq = tile(base_p), tile(base_q)

    def step():
        x = B.csd_gmm_draft_sample(mq, seed)
        n, ell, mask = B.csd_gmm_verify(x, mp, mq, G, gamma, seed)
        return x, n, mask, B.csd_gmm_resample(x, n, mp, mq, G, gamma, seed)

    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(a.steps):
        x, n, mask, (tok, n_out, trips, flags) = step()
    e1.record(); torch.cuda.synchronize()
    ms = e0.elapsed_time(e1)
    # the accept test alone (the dominant kernel: it reads both mixtures of every row once)
    v0, v1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    v0.record()
    for _ in range(a.steps):
        B.csd_gmm_verify(x, mp, mq, G, gamma, seed)
    v1.record(); torch.cuda.synchronize()
    v_ms = v0.elapsed_time(v1) / a.steps
    alg = R * (2 * K * (1 + 2 * D) + D) * 4 + R * 5 + G * 4       # both mixtures + x in; log-ratio, mask, n out
    res = {"metric": "verified tokens/sec (mixture heads: draft sample + accept test + resample)",
           "value": R * a.steps / (ms / 1e3), "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
           "ms_per_step": ms / a.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
           "data": "synthetic",
           "config": {"workload": "mixture heads: K=%d components, D=%d, rows/step=%d (gamma=%d)" % (K, D, R, gamma)},
           "acceptance": {"row_accept_rate": float(mask.float().mean()), "resample_trips_mean":
                          float(trips[trips > 0].float().mean()) if bool((trips > 0).any()) else 0.0,
                          "resample_trips_max": int(trips.max()), "cap_flags": int((flags & 1).sum())},
           "roofline": {"bound": "hbm", "kernel": "accept test over both mixtures", "achieved": alg / (v_ms / 1e3) / 1e9,
                        "peak": 8000.0, "unit": "GB/s", "frac": alg / (v_ms / 1e3) / 1e9 / 8000.0,
                        "avg_launch_ms": v_ms, "algorithmic_bytes_per_launch": alg, "traffic": None}}
    if a.oracle_rows > 0:
        from oracle import csd_oracle as O
        nr = min(a.oracle_rows * 64 // gamma * gamma, 4096, R)
        sl = lambda m: tuple(t[:nr] for t in m)
        t0 = time.perf_counter()
        xo = O.gmm_draft_sample(*sl(base_q), seed)
        n_o, ell_o, mask_o, log_u = O.gmm_verify(xo, *sl(base_p), *sl(base_q), nr // gamma, gamma, seed)
        O.gmm_resample(xo, n_o, *sl(base_p), *sl(base_q), nr // gamma, gamma, seed)
        dt = time.perf_counter() - t0
        clear = np.abs(log_u - ell_o) >= 1e-3
        res["cpu_baseline"] = {"value": nr / dt, "unit": "tokens/s", "cores": 1, "kind": "oracle",
                               "sample": "first %d rows, fp64 numpy oracle, %.1f s" % (nr, dt)}
        res["parity_on_sample"] = {"rows": nr, "token_max_abs_err": float(np.max(np.abs(x[:nr].cpu().numpy() - xo))),
                                   "decision_agreement_outside_band":
                                       float((mask[:nr].cpu().numpy().astype(bool) == (log_u <= ell_o))[clear].mean())}
    print(json.dumps(res))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="mar256")
    ap.add_argument("--dtype", default=None, choices=[None, "bf16", "f32"])
    ap.add_argument("--rows", type=int, default=0, help="rows per step (default: the whole workload)")
    ap.add_argument("--oracle-rows", type=int, default=128, help="rows of the CPU-oracle sample (0: skip)")
    ap.add_argument("--ddim-eta", type=float, default=None, help="use the DDIM sampler with this eta (default: DDPM)")
    ap.add_argument("--cfg-scale", type=float, default=None,
                    help="classifier-free guidance with this scale in both heads (two conditioning vectors per row)")
    ap.add_argument("--temperature", type=float, default=1.0, help="sampler temperature tau (scales sigma_t in both heads)")
    ap.add_argument("--ratio-mode", default=None, choices=[None, "aligned", "unaligned", "single_path"],
                    help="form the path ratio as in the paper's comparison of calculation approaches "
                         "(csd_denoise_ablation) instead of the method's lockstep call")
    ap.add_argument("--gmm-components", type=int, default=0,
                    help="measure the mixture-of-Gaussians head path instead (draft sample + accept test + resampling "
                         "with this many components per mixture; --rows rows, default 2^20)")
    ap.add_argument("--no-latency-shape", action="store_true", help="skip the split-phase latency-shape figure")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the timed steps, copy 256 MiB device to device once (a kernel of known "
                         "traffic, to scale rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py measures one GPU: every box of this build has one MI355X and the path has no "
                 "cross-GPU step (rows shard by group with replicated weights); run with --gpus 1")

    import numpy as np
    import torch
    from paper_2411_11925_amd import binding as B
    from paper_2411_11925_amd import synth as S

    if a.gmm_components > 0:
        return gmm_bench(a, np, torch, B, S)
    wl = S.WORKLOADS[a.workload]
    dtype = a.dtype or wl.gemm_dtype
    wl = wl.with_(gemm_dtype=dtype)
    R = a.rows or wl.rows_total
    gamma, D = wl.gamma, wl.target.token_dim
    G = R // gamma
    R = G * gamma
    dev = "cuda:0"
    tb, db, ds = wl.heads()
    gd = B.CSD_BF16 if dtype == "bf16" else B.CSD_F32
    mk = lambda sh: B.make_cfg(sh.token_dim, sh.cond_dim, sh.width, sh.n_blocks, wl.n_steps, gd,
                               eps_skip_gain=wl.eps_skip_gain, ddim_eta=a.ddim_eta)
    h_q, h_p = B.csd_init_head(mk(ds), db), B.csd_init_head(mk(wl.target), tb)
    zq_h, zp_h = wl.conds(((R + 63) // 64) * 64)
    reps = 1
    if a.cfg_scale is not None:
        # unconditional vectors: the workload's vectors of another block of rows
        uq_h, up_h = wl.conds(((R + 63) // 64) * 64, 64 * (1 << 20))
        zq_h, zp_h = np.stack([zq_h, uq_h], 1), np.stack([zp_h, up_h], 1)
        B.csd_set_guidance(h_q, True, a.cfg_scale); B.csd_set_guidance(h_p, True, a.cfg_scale)
        reps = 2
        a.no_latency_shape = True
    z_q, z_p = torch.from_numpy(zq_h[:R]).to(dev), torch.from_numpy(zp_h[:R]).to(dev)
    ratio_mode = {None: None, "aligned": B.CSD_RATIO_ALIGNED, "unaligned": B.CSD_RATIO_UNALIGNED,
                  "single_path": B.CSD_RATIO_SINGLE_PATH}[a.ratio_mode]
    n_ws = B.csd_workspace_bytes(h_q, h_p, R)
    if ratio_mode is not None:
        n_ws = max(n_ws, B.csd_ablation_workspace_bytes(h_q, h_p, R, ratio_mode))
        a.no_latency_shape = True
    ws = torch.empty(n_ws, dtype=torch.uint8, device=dev)
    summary = torch.empty((R, 5 * D + 1), dtype=torch.float32, device=dev)
    dist2 = torch.empty((R,), dtype=torch.float32, device=dev)

    tau = a.temperature

    def step():
        if ratio_mode is None:
            B.csd_denoise_lockstep(h_q, h_p, z_q, z_p, G, gamma, wl.seed, 0, tau, summary, ws)
        else:
            B.csd_denoise_ablation(h_q, h_p, z_q, z_p, G, gamma, wl.seed, 0, tau, ratio_mode, summary, dist2, ws)
        n_acc, ell, mask = B.csd_verify(summary, G, gamma, D, wl.seed, 0, tau)
        out = B.csd_resample(summary, n_acc, G, gamma, D, wl.seed, 0, tau)
        return n_acc, ell, mask, out

    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    launches_per_step = 2 * wl.n_steps          # one stacked modulation GEMM per head, step and row chunk
    B.csd_profile_enable(min(4 * a.steps * launches_per_step + 16, 1 << 18))   # up to 4 row chunks per call
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(a.steps):
        n_acc, ell, mask, (tokens, n_out, trips, flags) = step()
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = ev0.elapsed_time(ev1)
    k_ms, k_n, k_flops, k_ms_dev = B.csd_profile_read()
    B.csd_profile_enable(0)
    # the same kernel alone on the chip (same shapes, back to back on one stream), for
    # comparison with the in-situ figure, whose launches share the chip with other chains
    iso = None
    if dtype == "bf16":
        m_iso = R // 2 if R >= 8192 else R
        tot_ms, tot_fl = 0.0, 0.0
        for sh in (wl.target, ds):
            n_mod = 3 * sh.n_blocks * sh.width
            A_ = torch.randn(m_iso, sh.width, device=dev).bfloat16()
            W_ = (torch.randn(n_mod, sh.width, device=dev) / sh.width ** 0.5).bfloat16()
            b_ = torch.zeros(n_mod, device=dev)
            C_ = torch.empty(m_iso, n_mod, device=dev, dtype=torch.bfloat16)
            for _ in range(3):
                B.csd_gemm_bf16(A_, W_, b_, 0, C=C_)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                B.csd_gemm_bf16(A_, W_, b_, 0, C=C_)
            e1.record(); torch.cuda.synchronize()
            tot_ms += e0.elapsed_time(e1) / 20
            tot_fl += 2.0 * m_iso * n_mod * sh.width
            del A_, W_, b_, C_
        iso = tot_fl / (tot_ms / 1e3) / 1e12
    if a.calibration_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    flops_row = reps * (wl.n_steps * (head_flops_per_row_step(wl.target) + head_flops_per_row_step(ds))
                        + 2 * wl.target.cond_dim * (wl.target.width + ds.width))
    tokens_per_s = R * a.steps / (ms / 1e3)
    achieved = (k_flops / k_n) / (k_ms / k_n / 1e3) / 1e12 if k_n else 0.0
    peak = PEAK[dtype]
    # modulation GEMM per launch (all L blocks of a head at once): reads s [M,W] and the stacked
    # weights [3LW,W], writes [M,3LW]; bf16 = 2 bytes.  Averages over the two heads' launches.
    esz = 2 if dtype == "bf16" else 4
    lw2 = wl.target.n_blocks * wl.target.width ** 2 + ds.n_blocks * ds.width ** 2
    lw1 = wl.target.n_blocks * wl.target.width + ds.n_blocks * ds.width
    m_launch = k_flops / k_n / (3 * lw2) if k_n else 0          # mean rows per launch
    alg_bytes = esz * (m_launch * (wl.target.width + ds.width) / 2 + 3 * lw2 / 2
                       + m_launch * 3 * lw1 / 2) if k_n else None
    mask_h, trips_h, nacc_h = mask.cpu().numpy(), trips.cpu().numpy(), n_acc.cpu().numpy()
    res = {
        "metric": "verified tokens/sec (denoise+verify+resample)", "value": tokens_per_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms / a.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": "%s: target %dx%d, draft %dx%d, C=%d, T=%d, rows/step=%d (G=%d, gamma=%d)" % (
            wl.name, wl.target.n_blocks, wl.target.width, ds.n_blocks, ds.width, wl.target.cond_dim,
            wl.n_steps, R, G, gamma), "rows_per_step": R, "gamma": gamma, "out_scale": wl.out_scale,
            "eps_skip_gain": wl.eps_skip_gain,
            "sampler": "ddpm" if a.ddim_eta is None else "ddim(eta=%g)" % a.ddim_eta,
            "cfg_scale": a.cfg_scale, "ratio_mode": a.ratio_mode, "temperature": tau},
        "wall_s": wall,
        "whole_path": {"algorithmic_TFLOP_per_s": flops_row * R * a.steps / (ms / 1e3) / 1e12,
                       "frac_of_peak": flops_row * R * a.steps / (ms / 1e3) / 1e12 / peak,
                       "GFLOP_per_row": flops_row / 1e9},
        "acceptance": {"row_accept_rate": float(mask_h.mean()), "mean_accepted_prefix": float(nacc_h.mean()),
                       "resample_trips_mean": float(trips_h[trips_h > 0].mean()) if (trips_h > 0).any() else 0.0,
                       "resample_trips_max": int(trips_h.max()), "cap_flags": int((flags.cpu().numpy() & 1).sum())},
        "roofline": {"bound": "mfma" if dtype == "bf16" else "alu", "kernel": "modulation GEMM of all L blocks [M,W]x[W,3LW]",
                     "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                     "launches_timed": k_n, "avg_launch_ms": k_ms / k_n if k_n else None,
                     "on_device": None if not (k_n and k_ms_dev > 0) else {
                         "achieved": (k_flops / k_n) / (k_ms_dev / k_n / 1e3) / 1e12,
                         "frac": (k_flops / k_n) / (k_ms_dev / k_n / 1e3) / 1e12 / peak,
                         "avg_launch_ms": k_ms_dev / k_n,
                         "note": "same launches, from the first workgroup's start to the last one's end (device clock); "
                                 "agrees with the event bracket: with four chains on the chip a launch really runs that "
                                 "long, its workgroups sharing the CUs with the other chains' kernels"},
                     "algorithmic_bytes_per_launch": alg_bytes,
                     "alone_on_chip": None if iso is None else {"achieved": iso, "frac": iso / peak,
                                                                 "note": "same kernel and shapes, no other chain running"},
                     "traffic": measured_traffic(wl.name, dtype, R)},
    }

    if ratio_mode is not None:
        ell_h = ell.cpu().numpy().astype(np.float64)
        res["ratio_comparison"] = {"mode": a.ratio_mode, "mean_log_ratio": float(ell_h.mean()),
                                   "median_ratio": float(np.exp(np.median(ell_h))),
                                   "row_accept_rate": float(mask_h.mean()),
                                   "mean_token_distance2": float(dist2.double().mean().item())}

    # Secondary figure: one verify window the way an autoregressive loop runs Alg. 1 (split-phase
    # calls at the per-step shape: gamma draft calls of `batch` rows, one target call of batch*gamma
    # rows, accept test, resampling, bonus token).  Launch-latency bound; reported, not the metric.
    if not a.no_latency_shape:
        Gl = wl.batch
        Rl = Gl * gamma
        zq3 = z_q[:Rl].reshape(Gl, gamma, -1)
        zq_pos = [zq3[:, i].contiguous() for i in range(gamma)]
        zb = z_p[:Gl].contiguous()                  # stands in for the cond vectors of position gamma+1
        summ_l = torch.empty((Rl, 5 * D + 1), dtype=torch.float32, device=dev)

        # The target's conditioning vectors for positions 1..gamma+1 come from one pass of the target
        # transformer, so the bonus sample (position gamma+1) is independent of the verification of
        # positions 1..gamma: it runs on a second stream (default priority) beside the target call.
        side = torch.cuda.Stream()
        ws_b = torch.empty(max(B.csd_workspace_bytes(h_p, None, Gl), 256), dtype=torch.uint8, device=dev)
        bonus = torch.empty((Gl, D), dtype=torch.float32, device=dev)
        ev_fork, ev_join = torch.cuda.Event(), torch.cuda.Event()

        def window():
            main = torch.cuda.current_stream()
            for i in range(gamma):
                B.csd_denoise_draft(h_q, zq_pos[i], Gl, gamma, i, wl.seed, 0, 1.0, summ_l, ws)
            ev_fork.record(main)
            side.wait_event(ev_fork)
            B.csd_sample(h_p, zb, wl.seed, 0, B.CSD_STREAM_BONUS, 1.0, tokens=bonus, workspace=ws_b, stream=side)
            ev_join.record(side)
            B.csd_denoise_target(h_p, h_q, z_p[:Rl], Gl, gamma, wl.seed, 0, 1.0, summ_l, ws)
            na, _, _ = B.csd_verify(summ_l, Gl, gamma, D, wl.seed, want_log_ratio=False, want_mask=False)
            tok, no, _, _ = B.csd_resample(summ_l, na, Gl, gamma, D, wl.seed)
            main.wait_event(ev_join)
            B.csd_append_bonus(tok, no, na, bonus, gamma)
            return no
        window(); torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 3
        e0.record()
        for _ in range(reps):
            n_emit = window()
        e1.record(); torch.cuda.synchronize()
        ms_w = e0.elapsed_time(e1) / reps
        res["latency_shape"] = {"what": "one verify window, split-phase calls: %d draft calls of %d rows, one target "
                                        "call of %d rows, verify, resample; the bonus sample of %d rows runs on a second stream beside "
                                        "the target call" % (gamma, Gl, Rl, Gl),
                                "ms_per_window": ms_w, "verified_tokens_per_s": Rl / (ms_w / 1e3),
                                "emitted_tokens_per_s": float(n_emit.sum().item()) / (ms_w / 1e3),
                                "head_passes": (gamma + 2) * wl.n_steps}

    if a.oracle_rows > 0:
        from oracle import csd_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count()
        n = min(a.oracle_rows // gamma * gamma, R)
        samp = dict(sampler="ddim", ddim_eta=a.ddim_eta) if a.ddim_eta is not None else {}
        if a.cfg_scale is not None:
            samp["cfg_scale"] = a.cfg_scale
        ocfg = lambda sh: O.HeadCfg(sh.token_dim, sh.cond_dim, sh.width, sh.n_blocks, wl.n_steps,
                                    eps_skip_gain=wl.eps_skip_gain, **samp)
        t0 = time.perf_counter()
        o_q, o_p = O.Head(ocfg(ds), db), O.Head(ocfg(wl.target), tb)
        t_init = time.perf_counter() - t0
        t0 = time.perf_counter()
        if ratio_mode is None:
            s_o, _ = O.denoise_lockstep(o_q, o_p, zq_h[:n], zp_h[:n], wl.seed, 0, tau)
        else:
            s_o, _ = O.denoise_ablation(o_q, o_p, zq_h[:n], zp_h[:n], wl.seed, 0, tau, ratio_mode)
        n_o, ell_o, mask_o, log_u = O.verify(s_o, n // gamma, gamma, wl.seed, 0, tau)
        O.resample(s_o, n_o, n // gamma, gamma, wl.seed, 0, tau)
        dt = time.perf_counter() - t0
        x_g, x_o = summary[:n].cpu().numpy()[:, 4 * D:5 * D], s_o[:, 4 * D:5 * D]
        clear = np.abs(log_u - ell_o) >= 1e-3
        res["cpu_baseline"] = {"value": n / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
                               "sample": "first %d rows of the same workload, fp64 numpy oracle, %.1f s "
                                         "(+%.1f s set-up)" % (n, dt, t_init)}
        res["parity_on_sample"] = {
            "rows": n, "token_max_err_over_rms": float(np.max(np.abs(x_g - x_o)) / np.sqrt(np.mean(x_o ** 2))),
            "decision_agreement": float((mask_h[:n].astype(bool) == (log_u <= ell_o)).mean()),
            "decision_agreement_outside_band": float((mask_h[:n].astype(bool) == (log_u <= ell_o))[clear].mean()),
            "oracle_row_accept_rate": float(mask_o.mean())}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
