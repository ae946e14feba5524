#!/usr/bin/env python3
"""Benchmark of the ESSA hot path on one MI355X.

Workload (config.workload = c2_7b_decode): Qwen2.5-7B-shaped decode.  One "step" is one generation of the
whole hot path over one batch: K=32 seeds -> candidates (n = 28*4*2*16 = 3584, dense covariance basis) ->
singular values -> the q/k/v/o SVD-LoRA projections of 28 distinct layers (int8 per-channel weights, bf16
activations, r=16, 32 candidates x 8 sequences x 1 token = 256 rows; 822 MB of weights, more than the
256 MB Infinity Cache) -> synthetic reward -> rank-weighted CMA-ES update.  A candidate-token is one row
taken through the four projections of one layer, so a step processes 28 * 256 of them.

Prints ONE JSON line: metric, value, unit, ms_per_step, config, roofline (of the dominant kernel, timed with HIP
events on the launch stream) and cpu_baseline (the CPU oracle on a bounded sample of the same workload).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"w8a16": 2500.0, "w8a8": 5000.0}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--mode", choices=["w8a16", "w8a8"], default="w8a16", help="w8a16: bf16 activations as two int8 limbs on the int8 MFMA (default path); w8a8: one int8 limb")
    ap.add_argument("--workload", choices=["c2_7b_decode", "c3_32b_prefill", "c4_72b_decode", "c5_7b_es_iter"], default="c2_7b_decode",
                    help="c2 is the configuration the headline metric is quoted on; the others are side measurements")
    ap.add_argument("--layers", type=int, default=0, help="distinct layers cycled through (default: 28 for c2/c5, 1 for c3, 8 for c4)")
    ap.add_argument("--rows-per-cand", type=int, default=0)
    ap.add_argument("--population", type=int, default=0, help="candidates K (default: the workload's); with --rows-per-cand it sets the row count of a sweep point")
    ap.add_argument("--forward-only", action="store_true", help="time only the projections (no sampler / reward / update)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--refresh-basis", action="store_true",
                    help="time essa_cma_refresh_basis (C -> B, D) on the workload's search dimension instead of the step: cold, unchanged C, and after 17 generations of update")
    ap.add_argument("--optimizer", choices=["cma", "active", "sep", "es", "ars"], default="cma",
                    help="what samples the candidates and consumes the rewards: the (mu/mu_w, lambda)-CMA-ES of the headline (cma), the same with "
                         "negative weights (active), separable CMA-ES (sep), plain isotropic (mu, lambda)-ES (es) or ARS on K/2 antithetic pairs (ars)")
    ap.add_argument("--no-graph", action="store_true", help="issue every launch of a step from the host instead of replaying the recorded step")
    ap.add_argument("--two-pass-reward", action="store_true", help="reward as a second pass over Y instead of in the GEMM's epilogue")
    ap.add_argument("--calibrate-copy", action="store_true", help="also run one plain 256 MiB device copy (a reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU only (no sharding, no collectives); --gpus %d is not supported" % args.gpus)
        sys.exit(2)

    import numpy as np
    import torch

    import essa_workloads as wl
    import paper_2507_04453_amd as essa

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(2)
    cfg = wl.CONFIGS[args.workload]
    hidden, kv, r, K = cfg.hidden, cfg.kv, cfg.r, args.population or cfg.K
    layers = args.layers or {"c2_7b_decode": 28, "c3_32b_prefill": 1, "c4_72b_decode": 8, "c5_7b_es_iter": 28}[args.workload]
    rows_per = args.rows_per_cand or cfg.rows_per_cand
    if args.workload in ("c3_32b_prefill", "c4_72b_decode"):
        args.forward_only = True        # these configurations name the projections only
    if args.workload != "c2_7b_decode" or K != cfg.K:
        args.no_cpu_baseline = True
    quant = essa.QUANT_INT8_PERCH if cfg.quant == "int8" else essa.QUANT_INT4_G128
    R = K * rows_per
    P = layers * 4
    n = P * 2 * r
    flags = essa.COMPUTE_W8A8 if args.mode == "w8a8" else 0
    torch.cuda.set_device(0)
    # everything (the library's launches and torch's own fills) runs on one side stream, so that a step can be recorded
    stream = torch.cuda.Stream()
    torch.cuda.set_stream(stream)
    ctx = essa.Context(0, stream=stream)

    t0 = time.time()
    projs, sft_A, sft_B, vecs = [], [], [], []
    for l in range(layers):
        for pi, p in enumerate(wl.make_layer(hidden, kv, r, cfg.quant, l)):
            gp = essa.Projection(ctx, p.Wq, p.scales, p.zeros, p.A, p.B, quant)
            a, b = gp.spectrum()
            projs.append(gp)
            sft_A.append(a)
            sft_B.append(b)
            vecs.append(torch.from_numpy(wl.reward_vector(p.d_out, l, pi)).cuda())
    log("bench: %d projections set up in %.1f s" % (len(projs), time.time() - t0))
    sft_A = torch.from_numpy(np.stack(sft_A)).cuda()
    sft_B = torch.from_numpy(np.stack(sft_B)).cuda()

    def bf16(bits):
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()

    X1 = bf16(wl.make_x_bf16(R, hidden, 0)[0])
    X2 = bf16(wl.make_x_bf16(R, hidden, 1)[0])
    r2c = torch.from_numpy(wl.row2cand_interleaved(K, rows_per) if cfg.interleaved else wl.row2cand_contiguous(K, rows_per)).cuda()
    Q, d = wl.random_covariance_basis(n, 0)
    d = (d * 0.05).astype(np.float32)           # offsets of the order of 1% of a singular value
    zero = np.zeros(n, np.float32)
    kind = {"cma": essa.OPT_CMA, "active": essa.OPT_ACTIVE_CMA, "sep": essa.OPT_SEP_CMA, "es": essa.OPT_ES, "ars": essa.OPT_ARS}[args.optimizer]
    if kind in (essa.OPT_CMA, essa.OPT_ACTIVE_CMA):
        cma = essa.CmaState(ctx, n, 0.32, None, kind=kind)
        C0 = ((Q.astype(np.float64) * d.astype(np.float64) ** 2) @ Q.astype(np.float64).T).astype(np.float32)
        blob0 = essa.CmaState.pack_blob(n, 0, 0.32, zero, zero, zero, d, C0, Q, kind=kind)
        cma.import_blob(blob0)
    elif kind == essa.OPT_SEP_CMA:
        cma = essa.CmaState(ctx, n, 0.32, None, kind=kind)
        cma.import_blob(essa.CmaState.pack_blob(n, 0, 0.32, zero, zero, zero, d, (d.astype(np.float64) ** 2).astype(np.float32), kind=kind))
    else:       # isotropic: the same overall scale of the offsets in one step size
        cma = essa.CmaState(ctx, n, 0.32 * 0.05, None, kind=kind, ars_alpha=0.01, ars_top=K // 4)
    seeds = torch.arange(1, (K // 2 if kind == essa.OPT_ARS else K) + 1, dtype=torch.int32, device="cuda")
    theta = torch.empty(K, n, device="cuda")
    sA = torch.empty(K, P, r, device="cuda")
    sB = torch.empty(K, P, r, device="cuda")
    F = torch.zeros(K, device="cuda")
    Ys = [torch.empty(R, p.d_out, device="cuda", dtype=torch.bfloat16) for p in projs[:4]]
    items = []
    for l in range(layers):
        it = []
        for pi in range(4):
            j = l * 4 + pi
            it.append((projs[j], X2 if pi == 3 else X1, r2c, sA[:, j, :], sB[:, j, :], Ys[pi]))
        items.append(it)

    # argument blocks marshalled once; the reward share of every output tile is added by the GEMM's epilogue
    groups = [essa.ForwardGroup(items[l], vecs[l * 4:l * 4 + 4]) for l in range(layers)]
    rowpart = torch.empty(sum(g.blocks for g in groups), R, device="cuda")

    def forward_all(with_reward):
        if with_reward and not args.two_pass_reward:
            b = 0
            for l in range(layers):
                b = essa.essa_svdlora_forward_reward_group(ctx, groups[l], None, rowpart, b, flags)
            essa.essa_reward_finish(ctx, rowpart, b, r2c, F)
            return
        for l in range(layers):
            essa.essa_svdlora_forward_group(ctx, groups[l], flags)
            if with_reward:
                essa.essa_reward_accumulate_group(ctx, Ys, vecs[l * 4:l * 4 + 4], r2c, F)

    def step():
        if args.forward_only:
            forward_all(False)
            return
        essa.essa_sample_candidates(ctx, cma, seeds, theta, None)
        essa.essa_theta_to_sigma(ctx, r, sft_A, sft_B, theta, sA, sB)
        F.zero_()
        forward_all(True)
        essa.essa_cmaes_update(ctx, cma, seeds, F, None)

    if args.refresh_basis and kind != essa.OPT_CMA:
        raise SystemExit("bench.py --refresh-basis times the eigendecomposition of the default optimizer's covariance")
    if args.refresh_basis:
        # off the per-generation path: the eigendecomposition of the covariance, timed on its own
        def refresh():
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            sweeps, off = cma.refresh_basis(ctx)
            torch.cuda.synchronize()
            return {"sweeps": sweeps, "off": off, "ms": 1e3 * (time.perf_counter() - t0)}
        cma.import_blob(essa.CmaState.pack_blob(n, 0, 0.32, zero, zero, zero, np.ones(n, np.float32), C0, np.eye(n, dtype=np.float32)))
        out = {"metric": "essa_cma_refresh_basis", "n": n, "cold": refresh(), "unchanged": refresh()}
        gen = torch.Generator(device="cuda")
        gen.manual_seed(0)
        for g in range(17):
            sd = torch.arange(1 + g * K, 1 + (g + 1) * K, dtype=torch.int32, device="cuda")
            essa.essa_cmaes_update(ctx, cma, sd, torch.randn(K, device="cuda", generator=gen), None)
        out["after_17_generations"] = refresh()
        print(json.dumps(out))
        return
    if args.calibrate_copy:
        src = torch.ones(64 * 1024 * 1024, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)           # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    if args.forward_only:   # sigma must exist
        essa.essa_sample_candidates(ctx, cma, seeds, theta, None)
        essa.essa_theta_to_sigma(ctx, r, sft_A, sft_B, theta, sA, sB)
    for _ in range(max(args.warmup, 1)):
        step()
    torch.cuda.synchronize()
    # a step is a fixed sequence of launches on fixed buffers: record it once (HIP graph), replay it K times.  The
    # replay runs every kernel of the step; only the host's per-launch work is saved.
    run_step = step
    graph = None
    if not args.no_graph:
        ctx.graph_begin()
        step()
        graph = ctx.graph_end()
        run_step = graph.launch
        for _ in range(max(args.warmup, 1)):
            run_step()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    enqueue = time.perf_counter() - t0      # host time to issue the K steps (the GPU runs behind it)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # the same K steps once more with the library's HIP events around every GEMM launch (on its own stream):
    # the events cost a few percent of a step, so they stay out of the region that `value` is taken from
    ctx.profile_enable(True)
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed_profiled = time.perf_counter() - t1
    gemm_ms, gemm_launches = ctx.profile_read()
    ctx.profile_enable(False)
    ms_per_step = 1e3 * elapsed / args.steps
    value = layers * R / (elapsed / args.steps)

    # per-stage times (outside the timed region, events on the library's stream = torch's current stream)
    def timed(fn, reps=20):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    breakdown = {
        "forward_28_layers_ms": timed(lambda: forward_all(False), 5),
        "forward_plus_reward_ms": timed(lambda: forward_all(True), 5),
        "sample_ms": timed(lambda: essa.essa_sample_candidates(ctx, cma, seeds, theta, None)),
        "theta_to_sigma_ms": timed(lambda: essa.essa_theta_to_sigma(ctx, r, sft_A, sft_B, theta, sA, sB)),
        "update_ms": timed(lambda: essa.essa_cmaes_update(ctx, cma, seeds, F, None)),
    }

    # roofline of the dominant kernel (the fused-dequant MFMA GEMM, one launch per layer)
    dsum = sum(p.d_out for p in projs[:4])
    flops_per_launch = 2.0 * R * sum(p.d_out * (p.d_in + r) for p in projs[:4])
    wbytes = (lambda p: p.d_out * p.d_in + 4 * p.d_out) if cfg.quant == "int8" else (lambda p: p.d_out * p.d_in // 2 + 4 * p.d_out * (p.d_in // 128))
    # weights once + scales + U_B, two distinct X in, four Y out, rank-space vectors
    bytes_per_launch = sum(wbytes(p) + 2 * 2 * r * p.d_out for p in projs[:4]) \
        + 2 * R * hidden * (1 if args.mode == "w8a8" else 2) + 2 * R * dsum + 4 * R * 2 * r * 2
    avg_s = (gemm_ms / max(gemm_launches, 1)) * 1e-3
    t_mfma = flops_per_launch / (MFMA_PEAK_TFLOPS[args.mode] * 1e12)
    t_hbm = bytes_per_launch / (HBM_PEAK_GBS * 1e9)
    if t_mfma >= t_hbm:
        ach = flops_per_launch / avg_s / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": MFMA_PEAK_TFLOPS[args.mode], "unit": "TFLOP/s", "frac": ach / MFMA_PEAK_TFLOPS[args.mode], "traffic": None}
    else:
        ach = bytes_per_launch / avg_s / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "traffic": None}
    # HBM-side bytes per GEMM launch from rocprofv3 --pmc (profiles/c2_7b_decode_gemm_i8_hbm_traffic.md: reads scaled by the
    # factor a plain 256 MiB copy gives, 2.0; writes 1.0); measured for the default workload and mode only
    if args.workload == "c2_7b_decode" and args.mode == "w8a16" and rows_per == cfg.rows_per_cand and K == cfg.K:
        roof["traffic"] = 74.8e6
    # the library takes its 128 x 256 tile once the group fills the chip twice over with such tiles (int8 weights)
    big_tiles = -(-R // 128) * sum(-(-(-(-p.d_out // 32)) // 8) for p in projs[:4])
    # ... and, for 4-bit weights, its 64 x 256 tile once that gives every CU a workgroup
    q4_tiles = -(-R // 64) * sum(-(-(-(-p.d_out // 32)) // 8) for p in projs[:4])
    kernel = "gemm_i8_big_kernel" if (cfg.quant == "int8" and big_tiles >= 512) else ("gemm_q4_wide_kernel" if (cfg.quant != "int8" and q4_tiles >= 256) else "gemm_i8_kernel")
    roof.update({"kernel": kernel, "avg_launch_us": avg_s * 1e6, "launches": gemm_launches,
                 "flops_per_launch": flops_per_launch, "bytes_per_launch": bytes_per_launch,
                 "achieved_GBs": bytes_per_launch / avg_s / 1e9, "achieved_TFLOPs": flops_per_launch / avg_s / 1e12})

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, R, rows_per, args.mode)

    out = {
        "metric": "candidate-tokens/s through batched SVD-LoRA projections", "value": value, "unit": "candidate-tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if args.mode == "w8a16" else "int8", "data": "synthetic",
        "config": {"workload": args.workload, "layers": layers, "hidden": hidden, "kv": kv, "rank": r, "population": K,
                   "rows": R, "weights": "int8 per-channel" if cfg.quant == "int8" else "int4 g128 asymmetric", "activations": "bf16",
                   "mode": args.mode, "optimizer": args.optimizer,
                   "step": "forward only" if args.forward_only else "sample + sigma + %d layers x (q,k,v,o) + reward + update" % layers},
        "roofline": roof, "cpu_baseline": cpu, "breakdown_ms": breakdown,
        "ms_per_step_with_events": 1e3 * elapsed_profiled / args.steps,
        "host_enqueue_ms_per_step": 1e3 * enqueue / args.steps,
        "launches": "recorded step replayed (HIP graph)" if graph is not None else "issued one by one",
    }
    print(json.dumps(out), flush=True)


def cpu_baseline(cfg, R, rows_per, mode):
    """The oracle as it stands, timed on this machine's host cores on one layer of the same workload."""
    import numpy as np

    import essa_workloads as wl
    import oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        threads = 1
    K = cfg.K
    xv1 = wl.make_x_bf16(R, cfg.hidden, 0)[1]
    xv2 = wl.make_x_bf16(R, cfg.hidden, 1)[1]
    r2c = wl.row2cand_contiguous(K, rows_per)
    n_layers, dt = 0, 0.0
    while dt < 12.0 and n_layers < cfg.layers:      # about 10-30 s of oracle work
        prepared = []
        for pi, p in enumerate(wl.make_layer(cfg.hidden, cfg.kv, cfg.r, cfg.quant, n_layers)):
            # set-up (SVD, dequantisation) is not timed, as on the GPU side
            W = orc.dequant_int8(p.Wq, p.scales)
            f = orc.thin_svd_factors(p.A, p.B)
            dA, dB = wl.sigma_perturbation(K, 1, cfg.r, cfg.sigma_step, n_layers * 4 + pi)
            prepared.append((p, W, f, (f["S_A"][None] + dA[:, 0]), (f["S_B"][None] + dB[:, 0])))
        t0 = time.perf_counter()
        for p, W, f, sA, sB in prepared:
            xv = xv2 if p.name == "o" else xv1
            if mode == "w8a8":
                orc.svdlora_forward_w8a8(p.Wq, p.scales, f, xv, r2c, sA, sB)
            else:
                orc.svdlora_forward(W, f, xv, r2c, sA, sB)
        dt += time.perf_counter() - t0
        n_layers += 1
    return {"value": n_layers * R / dt, "unit": "candidate-tokens/s", "cores": threads, "kind": "oracle",
            "sample": "the first %d layers (q,k,v,o each) of c2_7b_decode, all %d rows, candidate weights W + B_k A_k formed "
                      "explicitly in fp64, forward only; %.1f s" % (n_layers, R, dt)}


if __name__ == "__main__":
    main()
