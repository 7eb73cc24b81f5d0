"""Benchmark: ADMM module-iterations on one OPT-6.7B-shaped FFN module resident on one MI355X.

A step is one full inner iteration of the per-module ADMM subproblem (score -> top-k -> Gram ->
fc2 refit -> fc1 refit -> a-update -> z-update -> objective) over all T calibration tokens, with
every input already resident in HBM.  Prints ONE JSON line (see the keys below).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_F16_TFLOPS = 2500.0   # MI355X dense fp16/bf16 MFMA
PEAK_HBM_GBS = 8000.0



def measured_traffic(workload: str, kernel_class: str):
    """HBM bytes per launch of a kernel class (GB) from the tracked summary of the two rocprofv3 --pmc runs
    (profiles/traffic_<workload>.json, written by paper_2510_03246_amd.profile_summary; hardware counters cannot be read
    inside this process).  The file carries the hash of the kernel sources it was measured on: with other sources
    the figure is stale and None is returned, with a note."""
    from paper_2510_03246_amd import profile_summary
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.json")
    if not os.path.exists(path):
        return None, f"no {os.path.relpath(path, ROOT)}"
    js = json.load(open(path))
    entry = js.get("classes", {}).get(kernel_class)
    if entry is None:
        return None, f"class not in {os.path.relpath(path, ROOT)}"
    if js.get("sources_sha256") != profile_summary.sources_hash():
        return None, (f"{os.path.relpath(path, ROOT)} was measured on other kernel sources ({entry['traffic_gb']:.1f} GB per launch "
                      "there); rerun the --pmc profile")
    return entry["traffic_gb"], js.get("unit", "GB per launch")


def cpu_baseline(cfg_name: str, sample_tokens: int, score_mode: str = "wanda", timed_iters: int = 2):
    """The oracle as it stands, timed on the host cores on a bounded token sample of the same module: one warm-up
    iteration, then `timed_iters` timed ones.  The oracle's a-update factors the full f x f system, a cost that does
    not depend on the token count; it is timed separately (the same library solve on the same matrix with a single
    right-hand side) so that the per-token rate can be read beside the sample's rate."""
    import numpy as np
    import torch

    from oracle import strp_oracle as orc
    from paper_2510_03246_amd import inputs

    full = inputs.CONFIGS[cfg_name]
    cfg = inputs.with_tokens(full, sample_tokens)
    m = inputs.make_ffn_module(cfg, 0, 0, "cpu")
    st = orc.module_init(*(m[n].double().numpy() for n in ("W1hat", "W2hat", "X")))
    k = cfg.f - int(round(cfg.rbar * cfg.f))
    mode = {"wanda": orc.WANDA, "lemma": orc.LEMMA, "gain": orc.GAIN}[score_mode]
    orc.admm_step(st, k, 1.0, 1.0, mode, select=True)                      # warm-up
    times = []
    for _ in range(timed_iters):
        t0 = time.perf_counter()
        orc.admm_step(st, k, 1.0, 1.0, mode, select=True)
        times.append(time.perf_counter() - t0)
    dt = sum(times) / len(times)
    lhs = st.W2.T @ st.W2 + np.eye(cfg.f)
    t0 = time.perf_counter()
    np.linalg.solve(lhs, np.ones((cfg.f, 1)))
    t_fixed = time.perf_counter() - t0
    per_token = max(dt - t_fixed, 1e-9) / sample_tokens
    return dict(value=sample_tokens / dt, unit="calib tokens/s", cores=torch.get_num_threads(), kind="oracle",
                seconds_per_iteration=dt, token_independent_seconds=t_fixed,
                tokens_per_s_without_the_token_independent_part=1.0 / per_token,
                projected_tokens_per_s_at_32768_tokens=32768.0 / (t_fixed + per_token * 32768.0),
                sample=f"oracle ADMM iterations (fp64 numpy) on {cfg_name} d={cfg.d} f={cfg.f} k={k} with {sample_tokens} of "
                       f"the {full.T} tokens: 1 warm-up + {timed_iters} timed, {dt:.1f} s each, of which {t_fixed:.1f} s is the "
                       f"f x f factorisation of the a-update (independent of the token count)")


def select_stress(ctx, torch):
    """Multi-block top-k (one threshold over a long score vector): algorithmic bytes 4n (scores) + n (mask) + 4k (indices)."""
    res = {}
    for name, n in (("2^26 scores", 1 << 26), ("48 x 28672 scores", 48 * 28672)):
        g = torch.Generator(device="cuda").manual_seed(n)
        score = torch.randn(n, generator=g, device="cuda") ** 2
        k = int(0.3 * n)
        ctx.strp_mask_topk(score, k)                      # warm-up (also sizes the workspace)
        torch.cuda.synchronize()
        ctx.profile_enable(True)
        reps = 5
        for _ in range(reps):
            ctx.strp_mask_topk(score, k)
        torch.cuda.synchronize()
        prof = ctx.profile_read()
        ctx.profile_enable(False)
        ms = prof["topk"]["ms"] / reps
        gb = (5.0 * n + 4.0 * k) / 1e9
        res[name] = dict(n=n, k=k, ms=ms, achieved_gbs=gb / (ms * 1e-3), frac_hbm=gb / (ms * 1e-3) / PEAK_HBM_GBS)
        del score
    return res


def head_variant(ctx, torch, inputs, strp, cfg):
    """Head pruning of one attention output projection at the workload's width (units = heads of d/heads channels):
    group-summed scores, top-k heads, Gram of the kept channels of C, refit of W_O[:, S].  One pass = the four calls."""
    d, g, T = cfg.d, cfg.d // cfg.heads, cfg.T
    m = inputs.make_head_module(cfg, 0, 0, "cuda")
    WO, Cm = m["WOhat"], m["C"]
    kh = cfg.heads - int(round(cfg.rbar * cfg.heads))
    Y = torch.empty((d, Cm.shape[1]), dtype=torch.float32, device="cuda")
    for t0 in range(0, T, 32768):                              # dense target W_O C (harness, not timed)
        Y[:, t0:t0 + 32768] = WO.float() @ Cm[:, t0:t0 + 32768].float()
    score = torch.empty(cfg.heads, dtype=torch.float32, device="cuda")
    energies = torch.zeros(1, dtype=torch.float64, device="cuda")
    W = torch.empty((d, d), device="cuda")
    lam = 0.01 * float((Cm[:, :T].float() ** 2).sum().item()) / d

    def one_pass():
        ctx.strp_score_alloc(Cm, T, strp.WANDA, score, energies, 0, 1, group=g, What=WO)
        mask, idx, tau = ctx.strp_mask_topk(score, kh, g)
        G = ctx.strp_gram(Cm, T, idx=idx)
        ctx.strp_refit(strp.SIDE_FC2, G, lam, Y, Cm, T, idx, W)
        return idx

    idx = one_pass()
    torch.cuda.synchronize()
    if ctx.poll() != strp.OK:
        raise RuntimeError("head variant: device status word not clean")
    ctx.profile_enable(True)
    reps = 3
    t0 = time.perf_counter()
    for _ in range(reps):
        one_pass()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / reps
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    s = int(idx.numel())
    return dict(heads=cfg.heads, head_dim=g, kept_heads=kh, kept_channels=s, ms_per_pass=ms, tokens_per_s=T / (ms * 1e-3),
                algorithmic_tflops=(s * (s + 1.0) * T + 2.0 * d * s * T) / (ms * 1e-3) / 1e12,
                kernels={n: dict(ms=v["ms"] / reps, launches=v["launches"] // reps) for n, v in
                         sorted(prof.items(), key=lambda kv: -kv[1]["ms"])})


def stream_modules(ctx, torch, inputs, strp, cfg, mod, params, n_modules, iters):
    """Modules one after another on the one resident state: the next module's weights and calibration input come from
    pinned host memory on a second stream while the current module iterates (double-buffered staging)."""
    from paper_2510_03246_amd import stream

    host = []
    for layer in range(n_modules):
        m = inputs.make_ffn_module(cfg, layer, 0, "cuda")
        host.append(stream.pin(m))
        del m
    streamer = stream.ModuleStreamer(host)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    losses = []
    for layer, buf in streamer:
        mod.rebind_inputs(buf["W1hat"], buf["W2hat"], buf["X"])
        mod.init(params)
        for it in range(iters):
            rep = mod.step(params, report=(it == iters - 1))
        losses.append(rep.J_ridge)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    copy_ms = streamer.copy_ms()
    return dict(modules=n_modules, iterations_per_module=iters, seconds=dt, seconds_per_module=dt / n_modules,
                host_to_device_bytes_per_module=streamer.bytes_per_module, copy_ms_per_module=sum(copy_ms) / n_modules,
                copy_gbs=streamer.bytes_per_module / (sum(copy_ms) / n_modules * 1e-3) / 1e9,
                staging_bytes=streamer.staging_bytes, objective_per_module=losses,
                peak_allocated=torch.cuda.max_memory_allocated())


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="opt6.7b")
    ap.add_argument("--tokens", type=int, default=0, help="override T (0: the configuration's 128 x 2048)")
    ap.add_argument("--score-mode", default="wanda", choices=("wanda", "lemma", "gain"),
                    help="unit score used by the select stage (the metric is quoted on wanda)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=2048,
                    help="tokens of the oracle's timed sample (8192 or 32768 give the fuller baseline; minutes of CPU time)")
    ap.add_argument("--head-variant", action="store_true",
                    help="also time head pruning of one attention output projection at the workload's width (scores per "
                         "head, top-k heads, Gram, refit of W_O); reported under \"head_variant\" in the same line")
    ap.add_argument("--stream-modules", type=int, default=0,
                    help="also run this many modules one after another on the resident state, their weights and calibration "
                         "input streamed from pinned host memory beside the compute; reported under \"stream_modules\"")
    ap.add_argument("--stream-iters", type=int, default=3, help="ADMM iterations per streamed module")
    ap.add_argument("--select-stress", action="store_true",
                    help="also time the multi-block top-k on 2^26 synthetic scores and on the 48 x 28672 scores of the "
                         "largest configuration (one global threshold); reported under \"select_stress\" in the same line")
    ap.add_argument("--no-mfma-ceiling", action="store_true",
                    help="skip the sustained-rate measurement of the fp16 matrix-core instruction (register-only, and fed from "
                         "LDS with random data in the GEMM's wavefront shape; under two seconds, outside the timed region) "
                         "that is reported under \"mfma_ceiling\"")
    ap.add_argument("--dump-launches", default="",
                    help="write the library's per-launch records of the timed region (kernel class names in enqueue order) "
                         "to this JSON file, for paper_2510_03246_amd.profile_summary")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="before the timed region run one elementwise copy kernel that reads 1 GiB and writes 1 GiB, "
                         "as the known-size reference for scaling hardware byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs the per-module ADMM path on ONE GPU (modules and token shards would be "
              "spread over more GPUs by the caller); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2510_03246_amd import inputs, strp

    cfg = inputs.CONFIGS[args.workload]
    if args.tokens:
        cfg = inputs.with_tokens(cfg, args.tokens)
    k = cfg.f - int(round(cfg.rbar * cfg.f))
    dev = "cuda"
    m = inputs.make_ffn_module(cfg, 0, 0, dev)
    ctx = strp.Context(0)
    mod = strp.FFNModule(ctx, m["W1hat"], m["W2hat"], m["X"], cfg.T, k_max=k)
    mode = {"wanda": strp.WANDA, "lemma": strp.LEMMA, "gain": strp.GAIN}[args.score_mode]
    params = strp.Params(1.0, 1.0, 0.01, mode, 1, k, 0)
    mod.init(params)
    for _ in range(args.warmup):
        mod.step(params, report=False)
    torch.cuda.synchronize()
    if ctx.poll() != strp.OK:
        raise RuntimeError("device status word not clean after warm-up")

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.mul(src, 1.0)      # one elementwise kernel: 2^30 bytes in, 2^30 bytes out
        torch.cuda.synchronize()
        del src, dst

    ctx.profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        rep = mod.step(params, report=(i == args.steps - 1))
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = ctx.profile_read()
    if args.dump_launches:
        with open(args.dump_launches, "w") as f:
            json.dump({"workload": args.workload, "steps": args.steps,
                       "launches": [name for name, _, _, _ in ctx.profile_launches()]}, f)
    ctx.profile_enable(False)
    if rep.status != strp.OK:
        raise RuntimeError(f"device status {rep.status} in the timed region")

    ms_per_step = 1e3 * dt / args.steps
    tokens_per_s = cfg.T * args.steps / dt
    # dominant kernel class by time inside the timed region (HIP events on the library's stream)
    dom_name, dom = max(prof.items(), key=lambda kv: kv[1]["ms"])
    is_gemm = dom_name.startswith("gemm")
    avg_ms = dom["ms"] / dom["launches"]
    traffic, traffic_note = measured_traffic(args.workload, dom_name)
    if is_gemm:
        # class name gemm_h<p>x<q>_<epilogue>: p, q = fp16 planes per operand; a p x q product issues
        # p*q - (1 if p == q == 2) MFMA passes per algorithmic multiply-add (hi*hi + hi*lo + lo*hi)
        npp, npq = int(dom_name[6]), int(dom_name[8])
        passes = npp * npq - (1 if npp * npq == 4 else 0)
        achieved = dom["flops"] / dom["launches"] / (avg_ms * 1e-3) / 1e12
        roof = dict(bound="mfma", kernel=dom_name, achieved=achieved, peak=PEAK_F16_TFLOPS, unit="TFLOP/s",
                    frac=achieved / PEAK_F16_TFLOPS, traffic=traffic, traffic_unit=traffic_note,
                    algorithmic_gb=dom["bytes"] / dom["launches"] / 1e9, avg_ms=avg_ms,
                    launches_per_step=dom["launches"] / args.steps, mfma_passes=passes,
                    executed=achieved * passes, executed_frac=achieved * passes / PEAK_F16_TFLOPS)
    else:
        achieved = dom["bytes"] / dom["launches"] / (avg_ms * 1e-3) / 1e9
        roof = dict(bound="hbm", kernel=dom_name, achieved=achieved, peak=PEAK_HBM_GBS, unit="GB/s",
                    frac=achieved / PEAK_HBM_GBS, traffic=traffic, traffic_unit=traffic_note,
                    avg_ms=avg_ms, launches_per_step=dom["launches"] / args.steps)
    kernels = {n: dict(ms_per_step=v["ms"] / args.steps, launches=v["launches"] // args.steps,
                       tflops=v["flops"] / max(v["ms"], 1e-9) / 1e9, gbs=v["bytes"] / max(v["ms"], 1e-9) / 1e6)
               for n, v in sorted(prof.items(), key=lambda kv: -kv[1]["ms"])}
    out = {
        "metric": "ADMM module-iterations/s (calib tokens/s) at OPT-6.7B shape; % MFMA peak",
        "value": tokens_per_s, "unit": "calib tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "dtype_detail": "fp32 values as two fp16 planes on the fp16 matrix cores (hi*hi + hi*lo + lo*hi), "
                                        "fp32 accumulation; fp64 for the ridge factorisations and solves", "data": "synthetic",
        "config": {"workload": f"{cfg.name} FFN module: d={cfg.d} f={cfg.f} T={cfg.T} keep k={k} "
                               f"({cfg.rbar:.0%} pruned), {args.score_mode.upper()} score, re-select every iteration, alpha=beta=1",
                   "module_iterations_per_s": args.steps / dt, "objective_J": rep.J_ridge},
        "roofline": roof,
        "kernels": kernels,
    }
    # device memory of the one resident module (the footprint that stays fixed while the model grows in depth)
    state_bytes = sum(t.numel() * t.element_size() for t in (mod.Z, mod.A, mod.Z0, mod.Y, mod.W1, mod.W2, mod.H, mod.cholH,
                                                              mod.n2, mod.score, mod.mask, mod.idx, mod.scalars))
    input_bytes = sum(t.numel() * t.element_size() for t in (m["X"], m["W1hat"], m["W2hat"]))
    model_weight_bytes = cfg.L * 12 * cfg.d * cfg.d * 2     # 4 d^2 attention + 8 d^2 FFN per layer, bf16
    out["device_memory"] = {"unit": "bytes", "module_inputs": input_bytes, "module_state": state_bytes,
                            "plane_cache": mod.cache.numel(), "workspace": ctx.ws.numel() if ctx.ws is not None else 0,
                            "peak_allocated": torch.cuda.max_memory_allocated(),
                            "resident_weights_of_this_module": m["W1hat"].numel() * 2 * m["W1hat"].element_size(),
                            "all_weights_of_the_model_bf16": model_weight_bytes}
    if args.select_stress:
        out["select_stress"] = select_stress(ctx, torch)
    if args.stream_modules:
        out["stream_modules"] = stream_modules(ctx, torch, inputs, strp, cfg, mod, params, args.stream_modules, args.stream_iters)
    if args.head_variant:
        out["head_variant"] = head_variant(ctx, torch, inputs, strp, cfg)
    if not args.no_mfma_ceiling:
        from paper_2510_03246_amd import bench_probe
        out["mfma_ceiling"] = {"unit": "TFLOP/s", "register_operands": bench_probe.mfma_rate(0),
                               "register_operands_random_data": bench_probe.mfma_rate(2),
                               "lds_fed_random_data": bench_probe.mfma_rate(1),
                               "lds_fed_random_data_32x32x16": bench_probe.mfma_rate(3),
                               "instruction": "v_mfma_f32_16x16x32_f16 (the pipelined GEMM's); the last entry is the same "
                                              "loop on v_mfma_f32_32x32x16_f16"}
        if roof.get("executed"):
            roof["executed_frac_of_lds_fed_ceiling"] = roof["executed"] / out["mfma_ceiling"]["lds_fed_random_data"]
    if not args.no_cpu_baseline:
        del mod, m
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(args.workload, args.cpu_sample_tokens, args.score_mode)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
