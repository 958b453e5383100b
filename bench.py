#!/usr/bin/env python3
"""Benchmark of the ADMM-Q layer solver hot path on one MI355X.

A "step" is one pass of the whole hot path over one synthetic layer: Hessian accumulation over all
calibration tokens, then admmq_quantize_layer (damping, scaling, factorisation, T ADMM iterations,
pair-swap local search).  Inputs are resident in HBM before the timed region starts.  Prints ONE JSON
line.  `value` is ADMM iterations per second over the ADMM loop alone, counting the T-1 iterations that run the
W-update products (the first iteration's W-update returns the dense weights and is skipped); the layer time and
the Hessian time are reported beside it.  The oracle (float64 NumPy) is timed on the host on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import synth_inputs as si  # noqa: E402

PEAK_FP32_MFMA_TFLOPS = 157.3      # MI355X dense fp32 matrix peak
PEAK_BF16_MFMA_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak (the fp16 peak is the same)
PEAK_HBM_GBS = 8000.0              # MI355X HBM3E peak
# HBM bytes per launch from two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch, both
# calibrated at 1.00 against plain fill / copy kernels of known size).  These are figures of those counter runs
# (fewer tokens and iterations than the timed run: counters perturb timing), not of the run timed here.
PMC_TRAFFIC_FROM = {"cfg2": "profiles/cfg2_hbm_traffic_pmc.txt (rocprofv3 --pmc, 16384 tokens, 6 iterations)"}
PMC_TRAFFIC_BYTES = {
    "cfg2": {"gemm": (227176.3 + 65536.0) * 1024, "project": (65784.5 + 131104.0) * 1024,
             "gemm_project": (262509.7 + 131080.0) * 1024,
             # the opt-in products (profiles/bench_cfg2_fast_products_kernel_trace.txt): product kernel + operand split
             "gemm_f16x3": (238850.1 + 83968.0 + 32909.4 + 65536.1) * 1024},
}


def make_inputs(cfg, tokens, torch):
    """X (bf16 or fp32) and W0 on the device, generated chunk by chunk by the shared seeded generator."""
    dt = torch.bfloat16 if cfg.x_dtype == "bf16" else torch.float32
    X = torch.empty((tokens, cfg.n), dtype=dt, device="cuda")
    row = 0
    for _, xc in si.iter_x_chunks(cfg, tokens):
        t = torch.from_numpy(xc.view(np.int16) if cfg.x_dtype == "bf16" else xc)
        if cfg.x_dtype == "bf16":
            X[row:row + xc.shape[0]].view(torch.int16).copy_(t, non_blocking=False)
        else:
            X[row:row + xc.shape[0]].copy_(t)
        row += xc.shape[0]
        if (row // xc.shape[0]) % 32 == 0:
            print(f"[bench] inputs: {row} of {tokens} rows generated", file=sys.stderr, flush=True)
    W0 = torch.from_numpy(si.layer_weights(cfg)).cuda()
    return X, W0


def cpu_baseline(cfg, sample_cols=1024, sample_iters=8, sample_tokens=8192):
    """The float64 oracle, untouched, on a bounded sample of the same workload."""
    from oracle import admmq_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([d.get("num_threads", 1) for d in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    t0 = time.perf_counter()
    chunks = [si.chunk_as_f64(cfg, xc) for _, xc in si.iter_x_chunks(cfg, min(sample_tokens, cfg.tokens))]
    H = orc.hessian(chunks)
    t_h = time.perf_counter() - t0
    W0 = si.layer_weights(cfg, p_slice=sample_cols).astype(np.float64)
    Hd, _ = orc.damp_hessian(H)
    grid = orc.Grid.fit(W0, cfg.bits, cfg.group_size)
    t0 = time.perf_counter()
    d, Hs, Ws = orc.scale_problem(Hd, W0)
    np.linalg.eigh(Hs)
    t_eig = time.perf_counter() - t0
    # the oracle's admm() factorises by itself: two runs that differ only in their number of iterations,
    # the extra iterations of the longer one are what is timed
    t0 = time.perf_counter()
    orc.admm(Hd, W0, grid, T=2)
    t_short = time.perf_counter() - t0
    t0 = time.perf_counter()
    orc.admm(Hd, W0, grid, T=2 + sample_iters)
    t_long = time.perf_counter() - t0
    t_admm = t_long - t_short
    if t_admm <= 0.05 * t_long:                      # the difference drowned in the factorisation's jitter
        t_admm = float("nan")
    its_slice = sample_iters / t_admm
    its_full = its_slice * sample_cols / cfg.p      # the loop is linear in the number of columns
    # local search (Sec. 3.5): one round of a bounded number of batches on the round-to-nearest codes of the slice
    ls_batches = 96
    k_rtn, _ = orc.rtn(W0, grid)
    G0 = Hd @ (W0 - grid.dequant(k_rtn))             # the gradient product is set-up, not part of a batch
    t0 = time.perf_counter()
    ls = orc.local_search(Hd, W0, k_rtn, grid, rounds=1, batches_per_round=ls_batches, pairs_per_batch=64,
                          seed=cfg.seed, G=G0)
    t_ls = time.perf_counter() - t0
    ls_slice = ls_batches / t_ls
    return {
        "phases": {"hessian_tokens_per_s": min(sample_tokens, cfg.tokens) / t_h, "eig_s": t_eig,
                   "admm_iterations_per_s": None if its_full != its_full else its_full,
                   "local_search_batches_per_s": ls_slice * sample_cols / cfg.p,
                   "local_search_sample": f"{ls_batches} batches of 64 pairs on {sample_cols} columns: "
                                          f"{ls_slice:.1f} batches/s, {ls.moves} applied; scaled by {sample_cols}/{cfg.p}"},
        "value": None if its_full != its_full else its_full, "unit": "ADMM iterations/s", "cores": int(cores), "kind": "oracle",
        "sample": (f"{cfg.name}: first {sample_cols} of {cfg.p} columns, {sample_iters} of {cfg.T} iterations (a run of "
                   f"{2 + sample_iters} minus a run of 2), "
                   f"H from the first {min(sample_tokens, cfg.tokens)} tokens; measured {its_slice:.3f} it/s on the "
                   f"slice, scaled by {sample_cols}/{cfg.p}; eigh({cfg.n}) {t_eig:.1f} s, "
                   f"Hessian {min(sample_tokens, cfg.tokens) / t_h:.0f} tokens/s"),
        "eig_s": t_eig,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg2", choices=sorted(si.CONFIGS))
    ap.add_argument("--tokens", type=int, default=0, help="truncate the calibration set (0 = the workload's N)")
    ap.add_argument("--iters", type=int, default=0, help="ADMM iterations (0 = the workload's T)")
    ap.add_argument("--ls-rounds", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fast-products", action="store_true",
                    help="time the opt-in split-fp16 W-update products instead of the fp32 ones (not the headline)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path would shard over output columns without "
              "communication, but no multi-GPU path is built); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2605_11222_amd as admmq

    cfg = si.CONFIGS[args.workload]
    tokens = args.tokens or cfg.tokens
    T = args.iters or cfg.T
    torch.cuda.set_device(0)
    t0 = time.perf_counter()
    X, W0 = make_inputs(cfg, tokens, torch)
    torch.cuda.synchronize()
    gen_s = time.perf_counter() - t0
    H = torch.empty((cfg.n, cfg.n), dtype=torch.float32, device="cuda")
    ctx = admmq.Context(0)
    if args.fast_products:
        ctx.set_fast_products(True)
    sched = admmq.Schedule(T=T, ls_rounds=args.ls_rounds, seed=cfg.seed)

    def step(profile):
        H.zero_()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ctx.accumulate_hessian(H, X)
        e1.record()
        # (the objective values are reports, not steps of the method: the timed calls leave them out, and one
        # untimed call below evaluates them for the same codes)
        out = ctx.quantize_layer(H, W0, cfg.bits, cfg.group_size, sched, want_stats=True, profile=profile,
                                 objectives=False)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1), out

    for w in range(args.warmup):
        step(False)
        print(f"[bench] warm-up step {w + 1} of {args.warmup} done", file=sys.stderr, flush=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    hs, stats = [], []
    for _ in range(args.steps):
        h_ms, out_timed = step(True)
        hs.append(h_ms)
        stats.append(out_timed[3])
        print(f"[bench] timed step {len(hs)} of {args.steps} done", file=sys.stderr, flush=True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = 1e3 * wall / args.steps

    mean = lambda f: float(np.mean([f(s) for s in stats]))
    admm_ms = mean(lambda s: s.ms_admm)
    its = (T - 1) / (admm_ms * 1e-3) if T > 1 else T / (admm_ms * 1e-3)
    n, p = cfg.n, cfg.p
    gemm_ms = mean(lambda s: s.ms_gemm / max(s.n_gemm, 1))
    # the timed steps run the projection pass as the epilogue of eq. 7's second product wherever they can; the
    # stand-alone pass is timed in one extra layer pass that keeps it a launch of its own in every iteration
    fused_n = mean(lambda s: s.n_gemm_project)
    fused_ms = mean(lambda s: s.ms_gemm_project / max(s.n_gemm_project, 1))
    proj_launches = mean(lambda s: s.n_project)
    if fused_n > 0:
        os.environ["ADMMQ_FUSE_PROJECTION"] = "0"
        out_obj = ctx.quantize_layer(H, W0, cfg.bits, cfg.group_size, sched, want_stats=True, profile=True)
        apart = out_obj[3]
        del os.environ["ADMMQ_FUSE_PROJECTION"]
        proj_ms = apart.ms_project / max(apart.n_project, 1)
    else:
        apart = None
        out_obj = ctx.quantize_layer(H, W0, cfg.bits, cfg.group_size, sched, want_stats=True)
        proj_ms = mean(lambda s: s.ms_project / max(s.n_project, 1))
    # the untimed call above also evaluated the objectives; its codes must be those of the timed calls
    obj = out_obj[3]
    same_codes = bool(torch.equal(out_obj[0], out_timed[0]))
    tri_ms = mean(lambda s: s.ms_tridiag / max(s.n_tridiag, 1))
    lsa_ms = mean(lambda s: s.ms_ls_apply / max(s.n_ls_apply, 1))
    gemm_tf = 2.0 * n * n * p / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    proj_gbs = 16.0 * n * p / (proj_ms * 1e-3) / 1e9 if proj_ms > 0 else 0.0
    lsa_gbs = 8.0 * n * p / (lsa_ms * 1e-3) / 1e9 if lsa_ms > 0 else 0.0    # one read + one write of G per flush
    # the search apart from its flushes (group kernels, their launch gaps and the one gradient product), per batch:
    # an upper bound of a batch's time in the group kernel, priced against the bytes an evaluation has to touch
    # (pairs x 2 rows x p columns x (4 B of G + 1 B of codes))
    ls_flushes = mean(lambda s: s.n_ls_apply)
    groups_per_round = -(-(-(-n // 2)) // 16)
    ls_batches_run = (ls_flushes / groups_per_round) * (-(-n // 2)) if groups_per_round > 0 else 0.0
    ls_rest_ms = mean(lambda s: s.ms_local_search) - ls_flushes * lsa_ms
    ls_batch_us = ls_rest_ms * 1e3 / ls_batches_run if ls_batches_run > 0 else 0.0
    ls_eval_gbs = 64 * 2 * p * 5.0 / (ls_batch_us * 1e-6) / 1e9 if ls_batch_us > 0 else 0.0
    hess_ms = float(np.mean(hs))
    hess_tf = tokens * n * (n + 1) / (hess_ms * 1e-3) / 1e12
    # bf16 activations in whole 256-channel tiles are multiplied on the bf16 matrix cores (exact products, fp32
    # accumulation) and priced against that peak; anything else goes through the fp32 product
    hess_bf16 = cfg.x_dtype == "bf16" and n % 256 == 0 and os.environ.get("ADMMQ_HESSIAN_BF16", "1") != "0"
    hess_peak = PEAK_BF16_MFMA_TFLOPS if hess_bf16 else PEAK_FP32_MFMA_TFLOPS

    # what a plain streaming kernel of the library reaches on this machine: 1 GiB copied (1 GiB read + 1 GiB written)
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    ctx.stream_copy(dst, src)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(10):
        ctx.stream_copy(dst, src)
    c1.record()
    torch.cuda.synchronize()
    copy_gbs = 10 * 2.0 * (1 << 30) / (c0.elapsed_time(c1) * 1e-3) / 1e9
    assert torch.equal(dst, src)
    del src, dst

    line = {
        "metric": "layer quantize time (s) & ADMM iters/s, 4096x4096 W3; % fp32 MFMA peak",
        "value": its, "unit": "ADMM iterations/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: n={n} p={p} tokens={tokens} W{cfg.bits} group={cfg.group_size or 'per-channel'} "
                               f"T={T} ls_rounds={args.ls_rounds}",
                   "iterations_counted": f"{max(T - 1, 1)} of {T}: those that run the two W-update products"},
        "layer_quantize_time_s": mean(lambda s: s.ms_total) * 1e-3,
        "phases_s": {"hessian": hess_ms * 1e-3, "setup": mean(lambda s: s.ms_setup) * 1e-3,
                     "factorise": mean(lambda s: s.ms_factor) * 1e-3, "admm": admm_ms * 1e-3,
                     "local_search": mean(lambda s: s.ms_local_search) * 1e-3},
        "objective": {"j_damp": obj.j_damp, "j_damp_admm": obj.j_damp_admm,
                      "j_damp_rtn": obj.j_damp_rtn, "j_recon": obj.j_recon,
                      "ls_moves": stats[-1].ls_moves,
                      "evaluated_in": "one untimed call after the timed ones (four products of the Hessian with an "
                                      "error matrix that are no part of the method)",
                      "same_codes_as_the_timed_calls": same_codes},
        "roofline": {"kernel": "gemm_tn (W-update, 2 launches per iteration)" if fused_n == 0 else
                               "gemm_tn (W-update, first product of an iteration; the second, which carries the "
                               "projection pass as its epilogue, is under roofline_product_with_projection)",
                     "bound": "mfma",
                     "achieved": gemm_tf, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": gemm_tf / PEAK_FP32_MFMA_TFLOPS,
                     "traffic": PMC_TRAFFIC_BYTES.get(cfg.name, {}).get("gemm"),
                     "traffic_from": PMC_TRAFFIC_FROM.get(cfg.name),
                     "ms_per_launch": gemm_ms, "flop_per_launch": 2.0 * n * n * p},
        "roofline_projection": {"kernel": "project_dual", "bound": "hbm", "achieved": proj_gbs, "peak": PEAK_HBM_GBS,
                                "unit": "GB/s", "frac": proj_gbs / PEAK_HBM_GBS,
                                "traffic": PMC_TRAFFIC_BYTES.get(cfg.name, {}).get("project"),
                                "traffic_from": PMC_TRAFFIC_FROM.get(cfg.name),
                                "ms_per_launch": proj_ms, "bytes_per_launch": 16.0 * n * p,
                                "copy_kernel_GBs": copy_gbs, "frac_of_copy_kernel": proj_gbs / copy_gbs,
                                "copy_kernel": "admmq_stream_copy of 1 GiB (2 GiB moved), mean of 10 launches "
                                               "between events, in this run",
                                "measured_in": ("the timed steps" if apart is None else
                                                "one extra layer pass with ADMMQ_FUSE_PROJECTION=0 (the pass as a "
                                                f"launch of its own in all {apart.n_project} iterations: ADMM "
                                                f"{apart.ms_admm * 1e-3:.4f} s); the timed steps launch it "
                                                f"{proj_launches:.0f} times per layer and run it {fused_n:.0f} times as "
                                                "the epilogue of the second product")},
        "roofline_product_with_projection": None if fused_n == 0 else {
            "kernel": "gemm_tn with eqs. 8-10 as its epilogue (second product of an iteration: W stays in registers)",
            "bound": "mfma", "achieved": 2.0 * n * n * p / (fused_ms * 1e-3) / 1e12, "peak": PEAK_FP32_MFMA_TFLOPS,
            "unit": "TFLOP/s", "frac": 2.0 * n * n * p / (fused_ms * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS,
            "ms_per_launch": fused_ms, "flop_per_launch": 2.0 * n * n * p,
            "epilogue_bytes_per_launch": 16.0 * n * p, "launches_per_layer": fused_n,
            "traffic": PMC_TRAFFIC_BYTES.get(cfg.name, {}).get("gemm_project"),
            "traffic_from": PMC_TRAFFIC_FROM.get(cfg.name)},
        "roofline_ls_flush": {"kernel": "ls_flush_rows (gradient correction, once per 16 batches)", "bound": "hbm",
                              "achieved": lsa_gbs, "peak": PEAK_HBM_GBS,
                              "unit": "GB/s", "frac": lsa_gbs / PEAK_HBM_GBS, "ms_per_launch": lsa_ms},
        "roofline_ls_group": None if ls_batches_run <= 0 else {
            "kernel": "ls_group (evaluate eq. 11, choose, apply: one launch per 16 batches)", "bound": "hbm",
            "achieved": ls_eval_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ls_eval_gbs / PEAK_HBM_GBS,
            "us_per_batch": ls_batch_us, "batches": ls_batches_run,
            "measured_as": "search time minus its flushes, over the batches run (includes launch gaps and the "
                           "gradient product): an upper bound of the kernel's own time per batch",
            "what_bounds_it": "not the bytes: a batch is one exchange of sums between all blocks plus the vector "
                              "instructions between a winner's arrival and the next sums; vector ALU busy 61 % of "
                              "the kernel (profiles/ls_group_cfg2_pmc.txt)"},
        "roofline_hessian": {"kernel": ("hessian_bf16 + sym_reduce (bf16 matrix cores, lower triangle)" if hess_bf16
                                        else "gemm_tn + sym_reduce (fp32 matrix cores, lower triangle)"),
                             "bound": "mfma", "achieved": hess_tf, "peak": hess_peak, "unit": "TFLOP/s",
                             "frac": hess_tf / hess_peak, "ms_per_call": hess_ms},
        "middle_solve_ms_per_launch": tri_ms,
        "factor_form": "band16" if cfg.n >= 4096 and os.environ.get("ADMMQ_FACTOR", "")[:1] != "t" or os.environ.get("ADMMQ_FACTOR", "")[:1] == "b" else "tridiagonal",
        "input_generation_s": gen_s,
    }
    # informational, outside the timed region and not part of `value`: the same layer with the opt-in stopping
    # rule (stop once the codes have been unchanged for 8 iterations); the timed steps above run all T iterations
    early_out = ctx.quantize_layer(H, W0, cfg.bits, cfg.group_size,
                                   admmq.Schedule(T=T, ls_rounds=args.ls_rounds, seed=cfg.seed, quiet_stop=8),
                                   objectives=False)
    early = early_out[3]
    early_same = bool(torch.equal(early_out[0], out_timed[0]))
    line["with_quiet_stop_8"] = {"iterations_run": early.iters_done, "layer_quantize_time_s": early.ms_total * 1e-3,
                                 "admm_s": early.ms_admm * 1e-3, "j_damp": obj.j_damp if early_same else None,
                                 "same_codes_as_full_run": early_same}
    del early_out
    # informational as well: the same layer with the opt-in split-fp16 W-update products (fp16 matrix cores, three
    # exact products of 22-bit operand pairs accumulated in fp32); the headline above is the fp32 products
    if not args.fast_products and admmq.fast_products_bytes(n, p) > 0:
        ctx.set_fast_products(True)
        # (one untimed pass first, which also evaluates the objective; the large workloads do without, and their one
        # pass carries the objective evaluations in its time)
        f_obj = None
        if n <= 8192:
            f_obj = ctx.quantize_layer(H, W0, cfg.bits, cfg.group_size, sched, want_stats=True, profile=False)[3]
        fs = [ctx.quantize_layer(H, W0, cfg.bits, cfg.group_size, sched, want_stats=True, profile=True,
                                 objectives=f_obj is None)[3]
              for _ in range(2 if n <= 8192 else 1)]
        if f_obj is None:
            f_obj = fs[-1]
        fq = ctx.quantize_layer(H, W0, cfg.bits, cfg.group_size,
                                admmq.Schedule(T=T, ls_rounds=args.ls_rounds, seed=cfg.seed, quiet_stop=8),
                                objectives=False)[3]
        ctx.set_fast_products(False)
        f_admm = float(np.mean([s.ms_admm for s in fs]))
        f_gemm = float(np.mean([s.ms_gemm / max(s.n_gemm, 1) for s in fs]))
        f_tf = 2.0 * n * n * p / (f_gemm * 1e-3) / 1e12
        line["with_fast_products"] = {
            "admm_iterations_per_s": T / (f_admm * 1e-3),
            "layer_quantize_time_s": float(np.mean([s.ms_total for s in fs])) * 1e-3,
            "j_damp": f_obj.j_damp, "j_damp_relative_to_fp32_products": f_obj.j_damp / obj.j_damp - 1.0,
            "roofline": {"kernel": "split_f16 + gemm_f16x3 (W-update, 2 per iteration; operand split included)",
                         "bound": "mfma", "achieved": 3.0 * f_tf, "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                         "frac": 3.0 * f_tf / PEAK_BF16_MFMA_TFLOPS, "ms_per_product": f_gemm,
                         "traffic": PMC_TRAFFIC_BYTES.get(cfg.name, {}).get("gemm_f16x3"),
                         "executed_flop_per_product": 6.0 * n * n * p,
                         "fp32_equivalent_TFLOP/s": f_tf},
            "and_quiet_stop_8": {"iterations_run": fq.iters_done, "layer_quantize_time_s": fq.ms_total * 1e-3}}
    ctx.close()
    del X
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
