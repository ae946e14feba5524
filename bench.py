#!/usr/bin/env python3
"""Benchmark of the ESSA hot path on one MI355X.

Headline workload (config.workload = c2_7b_decode): Qwen2.5-7B-shaped decode.  One "step" is one generation of the
whole hot path over one batch: K=32 seeds -> candidates (n = 28*4*2*16 = 3584, dense covariance basis) ->
singular values -> the q/k/v/o SVD-LoRA projections of 28 distinct layers (int8 per-channel weights, bf16
activations, r=16, 32 candidates x 8 sequences x 1 token = 256 rows; 822 MB of weights, more than the
256 MB Infinity Cache) -> synthetic reward -> rank-weighted CMA-ES update.  A candidate-token is one row
taken through the four projections of one layer, so a step processes 28 * 256 of them.

Prints ONE JSON line: metric, value, unit, ms_per_step, config, roofline (of the dominant kernel, timed with HIP
events on the launch stream) and cpu_baseline (the CPU oracle on a bounded sample of the same workload).  The same
line carries, under "workloads", a short record of the other three full-size configurations (32B-shaped prefill,
72B-shaped 4-bit decode over all 80 layers, the full iteration at 32768 rows), each with its own step time, dominant
kernel, time per launch, algorithmic flops and bytes per launch and roofline fraction, and, under "row_sweep", the
forward of one 7B-shaped layer at 8 ... 512 rows (the HBM-bound side of the decode shapes).
"""
import argparse
import hashlib
import json
import os
import re
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# the default path multiplies on the int8 MFMA, one pass per limb: two passes cost what one bf16 pass would, so its
# algorithmic flops are priced at the bf16 figure (2.5 PFLOP/s); the one-limb mode at the int8 figure
MFMA_PEAK_TFLOPS = {"w8a16": 2500.0, "w8a8": 5000.0}
INT8_PEAK_TOPS = 5000.0
WORKLOADS = ["c2_7b_decode", "c3_32b_prefill", "c4_72b_decode", "c5_7b_es_iter"]
DEFAULT_LAYERS = {"c2_7b_decode": 28, "c3_32b_prefill": 1, "c4_72b_decode": 80, "c5_7b_es_iter": 28}
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "c2_7b_decode_gemm_hbm_traffic.md")
KERNEL_SOURCES = ["kernels_stream.hip"]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kernel_source_digest():
    """sha256 of the sources of the forward's GEMM and prep kernels: what a stored counter reading is valid for."""
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2507_04453_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def stored_traffic():
    """HBM-side bytes per GEMM launch of the headline workload from the tracked rocprofv3 --pmc summary, or None when
    the summary was taken with other kernel sources than the ones in this tree (a stale reading is not reported)."""
    try:
        text = open(TRAFFIC_FILE).read()
    except OSError:
        return None
    m_b = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", text, re.M)
    m_d = re.search(r"^kernel_source_sha256_16:\s*([0-9a-f]{16})", text, re.M)
    if not m_b or not m_d or m_d.group(1) != kernel_source_digest():
        return None
    return float(m_b.group(1))


class Bench:
    """Everything that lives on the GPU for one workload, and the timed step."""

    def __init__(self, essa, torch, np, wl, ctx, name, args, layers=None, population=None, rows_per=None, projs=None):
        self.essa, self.torch, self.np, self.wl, self.ctx, self.name, self.args = essa, torch, np, wl, ctx, name, args
        cfg = wl.CONFIGS[name]
        self.cfg = cfg
        self.hidden, self.kv, self.r = cfg.hidden, cfg.kv, cfg.r
        self.K = population or cfg.K
        self.layers = layers or DEFAULT_LAYERS[name]
        self.rows_per = rows_per or cfg.rows_per_cand
        self.forward_only = args.forward_only or name in ("c3_32b_prefill", "c4_72b_decode")   # these name the projections only
        self.quant = essa.QUANT_INT8_PERCH if cfg.quant == "int8" else essa.QUANT_INT4_G128
        self.R = self.K * self.rows_per
        self.P = self.layers * 4
        self.n = self.P * 2 * self.r
        self.flags = essa.COMPUTE_W8A8 if args.mode == "w8a8" else 0
        self.owns_projs = projs is None
        self._setup(projs)

    def _setup(self, projs):
        essa, torch, np, wl, ctx, cfg = self.essa, self.torch, self.np, self.wl, self.ctx, self.cfg
        t0 = time.time()
        if projs is None:
            # host set-up (random weights, SVDs, repacking, upload) of the layers in parallel: ctypes drops the GIL
            def make(l):
                out = []
                for pi, p in enumerate(wl.make_layer(self.hidden, self.kv, self.r, cfg.quant, l)):
                    out.append(essa.Projection(ctx, p.Wq, p.scales, p.zeros, p.A, p.B, self.quant))
                return out
            with ThreadPoolExecutor(max_workers=8) as ex:
                projs = [gp for layer in ex.map(make, range(self.layers)) for gp in layer]
            log("bench[%s]: %d projections set up in %.1f s" % (self.name, len(projs), time.time() - t0))
        self.projs = projs[:self.P]
        spectra = [gp.spectrum() for gp in self.projs]
        self.sft_A = torch.from_numpy(np.stack([a for a, _ in spectra])).cuda()
        self.sft_B = torch.from_numpy(np.stack([b for _, b in spectra])).cuda()
        self.vecs = [torch.from_numpy(wl.reward_vector(gp.d_out, j // 4, j % 4)).cuda() for j, gp in enumerate(self.projs)]

        def bf16(bits):
            return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()

        R, K, n, r, P = self.R, self.K, self.n, self.r, self.P
        self.X1 = bf16(wl.make_x_bf16(R, self.hidden, 0)[0])
        self.X2 = bf16(wl.make_x_bf16(R, self.hidden, 1)[0])
        self.r2c = torch.from_numpy(wl.row2cand_interleaved(K, self.rows_per) if cfg.interleaved else wl.row2cand_contiguous(K, self.rows_per)).cuda()
        kind = {"cma": essa.OPT_CMA, "active": essa.OPT_ACTIVE_CMA, "sep": essa.OPT_SEP_CMA, "es": essa.OPT_ES, "ars": essa.OPT_ARS}[self.args.optimizer]
        if self.forward_only and kind in (essa.OPT_CMA, essa.OPT_ACTIVE_CMA):
            kind = essa.OPT_SEP_CMA            # only sigma has to exist: no n x n state for the forward-only configurations
        self.kind = kind
        zero = np.zeros(n, np.float32)
        if kind in (essa.OPT_CMA, essa.OPT_ACTIVE_CMA):
            Q, d = wl.random_covariance_basis(n, 0)
            d = (d * 0.05).astype(np.float32)           # offsets of the order of 1% of a singular value
            self.cma = essa.CmaState(ctx, n, 0.32, None, kind=kind)
            self.C0 = ((Q.astype(np.float64) * d.astype(np.float64) ** 2) @ Q.astype(np.float64).T).astype(np.float32)
            self.cma.import_blob(essa.CmaState.pack_blob(n, 0, 0.32, zero, zero, zero, d, self.C0, Q, kind=kind))
            self.Q, self.d = Q, d
        elif kind == essa.OPT_SEP_CMA:
            g = np.random.default_rng(0)
            d = (0.05 * np.exp(g.uniform(np.log(0.5), np.log(2.0), size=n))).astype(np.float32)
            self.cma = essa.CmaState(ctx, n, 0.32, None, kind=kind)
            self.cma.import_blob(essa.CmaState.pack_blob(n, 0, 0.32, zero, zero, zero, d, (d.astype(np.float64) ** 2).astype(np.float32), kind=kind))
        else:       # isotropic: the same overall scale of the offsets in one step size
            self.cma = essa.CmaState(ctx, n, 0.32 * 0.05, None, kind=kind, ars_alpha=0.01, ars_top=K // 4)
        self.seeds = torch.arange(1, (K // 2 if kind == essa.OPT_ARS else K) + 1, dtype=torch.int32, device="cuda")
        self.theta = torch.empty(K, n, device="cuda")
        self.sA = torch.empty(K, P, r, device="cuda")
        self.sB = torch.empty(K, P, r, device="cuda")
        self.F = torch.zeros(K, device="cuda")
        self.Ys = [torch.empty(R, gp.d_out, device="cuda", dtype=torch.bfloat16) for gp in self.projs[:4]]
        items = []
        for l in range(self.layers):
            it = []
            for pi in range(4):
                j = l * 4 + pi
                it.append((self.projs[j], self.X2 if pi == 3 else self.X1, self.r2c, self.sA[:, j, :], self.sB[:, j, :], self.Ys[pi]))
            items.append(it)
        # argument blocks marshalled once; the reward share of every output tile is added by the GEMM's epilogue
        self.groups = [essa.ForwardGroup(items[l], self.vecs[l * 4:l * 4 + 4]) for l in range(self.layers)]
        self.rowpart = torch.empty(sum(g.blocks for g in self.groups), R, device="cuda")

    # ------------------------------------------------------------------------------------------ the step
    def forward_all(self, with_reward):
        essa, ctx = self.essa, self.ctx
        if with_reward and not self.args.two_pass_reward:
            b = 0
            for l in range(self.layers):
                b = essa.essa_svdlora_forward_reward_group(ctx, self.groups[l], None, self.rowpart, b, self.flags)
            essa.essa_reward_finish(ctx, self.rowpart, b, self.r2c, self.F)
            return
        for l in range(self.layers):
            essa.essa_svdlora_forward_group(ctx, self.groups[l], self.flags)
            if with_reward:
                essa.essa_reward_accumulate_group(ctx, self.Ys, self.vecs[l * 4:l * 4 + 4], self.r2c, self.F)

    def sample(self):
        self.essa.essa_sample_candidates(self.ctx, self.cma, self.seeds, self.theta, None)

    def to_sigma(self):
        self.essa.essa_theta_to_sigma(self.ctx, self.r, self.sft_A, self.sft_B, self.theta, self.sA, self.sB)

    def update(self):
        self.essa.essa_cmaes_update(self.ctx, self.cma, self.seeds, self.F, None)

    def step(self):
        if self.forward_only:
            self.forward_all(False)
            return
        self.sample()
        self.to_sigma()
        self.F.zero_()
        self.forward_all(True)
        self.update()

    # ------------------------------------------------------------------------------------------ timing
    def run(self, steps, warmup, with_breakdown=True):
        torch, ctx, args = self.torch, self.ctx, self.args
        if self.forward_only:   # sigma must exist
            self.sample()
            self.to_sigma()
        for _ in range(max(warmup, 1)):
            self.step()
        torch.cuda.synchronize()
        # a step is a fixed sequence of launches on fixed buffers: record it once (HIP graph), replay it K times.  The
        # replay runs every kernel of the step; only the host's per-launch work is saved.
        run_step = self.step
        graph = None
        if not args.no_graph:
            ctx.graph_begin()
            self.step()
            graph = ctx.graph_end()
            run_step = graph.launch
            for _ in range(max(warmup, 1)):
                run_step()
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            run_step()
        enqueue = time.perf_counter() - t0      # host time to issue the K steps (the GPU runs behind it)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        # the same K steps once more with the library's HIP events around every GEMM launch (on its own stream):
        # the events cost a few percent of a step, so they stay out of the region that `value` is taken from
        ctx.profile_enable(True)
        t1 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        elapsed_profiled = time.perf_counter() - t1
        gemm_ms, gemm_launches = ctx.profile_read()
        ctx.profile_enable(False)
        res = {"ms_per_step": 1e3 * elapsed / steps, "value": self.layers * self.R / (elapsed / steps),
               "ms_per_step_with_events": 1e3 * elapsed_profiled / steps, "host_enqueue_ms_per_step": 1e3 * enqueue / steps,
               "launches": "recorded step replayed (HIP graph)" if graph is not None else "issued one by one",
               "roofline": self.roofline(gemm_ms, gemm_launches)}
        if with_breakdown:
            res["breakdown_ms"] = self.breakdown()
        if graph is not None:
            graph.close()
        return res

    def timed(self, fn, reps=20):
        """events on the library's stream (= torch's current stream)"""
        torch = self.torch
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    def breakdown(self):
        reps = 5 if self.R <= 1024 else 2
        out = {"forward_%d_layers_ms" % self.layers: self.timed(lambda: self.forward_all(False), reps)}
        if not self.forward_only:
            out["forward_plus_reward_ms"] = self.timed(lambda: self.forward_all(True), reps)
            out["sample_ms"] = self.timed(self.sample)
            out["theta_to_sigma_ms"] = self.timed(self.to_sigma)
            out["update_ms"] = self.timed(self.update)
        return out

    def roofline(self, gemm_ms, gemm_launches):
        """of the dominant kernel: the fused-dequant MFMA GEMM, one launch per layer"""
        cfg, R, r, mode = self.cfg, self.R, self.r, self.args.mode
        projs = self.projs[:4]
        dsum = sum(p.d_out for p in projs)
        flops_per_launch = 2.0 * R * sum(p.d_out * (p.d_in + r) for p in projs)
        wbytes = (lambda p: p.d_out * p.d_in + 4 * p.d_out) if cfg.quant == "int8" else (lambda p: p.d_out * p.d_in // 2 + 4 * p.d_out * (p.d_in // 128))
        # weights once + scales + U_B, two distinct X in, four Y out, rank-space vectors
        bytes_per_launch = sum(wbytes(p) + 2 * 2 * r * p.d_out for p in projs) \
            + 2 * R * self.hidden * (1 if mode == "w8a8" else 2) + 2 * R * dsum + 4 * R * 2 * r * 2
        avg_s = (gemm_ms / max(gemm_launches, 1)) * 1e-3
        t_mfma = flops_per_launch / (MFMA_PEAK_TFLOPS[mode] * 1e12)
        t_hbm = bytes_per_launch / (HBM_PEAK_GBS * 1e9)
        if t_mfma >= t_hbm:
            ach = flops_per_launch / avg_s / 1e12
            roof = {"bound": "mfma", "achieved": ach, "peak": MFMA_PEAK_TFLOPS[mode], "unit": "TFLOP/s", "frac": ach / MFMA_PEAK_TFLOPS[mode], "traffic": None}
        else:
            ach = bytes_per_launch / avg_s / 1e9
            roof = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "traffic": None}
        if self.name == "c2_7b_decode" and mode == "w8a16" and self.rows_per == cfg.rows_per_cand and self.K == cfg.K:
            roof["traffic"] = stored_traffic()
        limbs = 1 if mode == "w8a8" else 2
        roof.update({"kernel": self.kernel_name(), "avg_launch_us": avg_s * 1e6, "launches": gemm_launches,
                     "flops_per_launch": flops_per_launch, "bytes_per_launch": bytes_per_launch,
                     "achieved_GBs": bytes_per_launch / avg_s / 1e9, "achieved_TFLOPs": flops_per_launch / avg_s / 1e12,
                     "frac_of_hbm": bytes_per_launch / avg_s / 1e9 / HBM_PEAK_GBS,
                     # the unit the contraction really runs on: int8 MFMA, `limbs` passes over the weights
                     "int8_mfma": {"passes": limbs, "executed_TOPs": limbs * flops_per_launch / avg_s / 1e12, "peak_TOPs": INT8_PEAK_TOPS,
                                   "frac_executed": limbs * flops_per_launch / avg_s / 1e12 / INT8_PEAK_TOPS,
                                   "frac_algorithmic": flops_per_launch / avg_s / 1e12 / INT8_PEAK_TOPS}})
        return roof

    def kernel_name(self):
        """which GEMM the library's launcher picks for this group (its rules, restated)"""
        projs, R = self.projs[:4], self.R
        col256 = sum(-(-(-(-p.d_out // 32)) // 8) for p in projs)
        if self.cfg.quant == "int8":
            if -(-R // 128) * col256 >= 512:
                return "gemm_i8_big_kernel"
            return "gemm_i8_stream_kernel" if R <= 64 else "gemm_i8_kernel"
        return "gemm_q4_wide_kernel" if -(-R // 64) * col256 >= 256 else "gemm_i8_kernel<Q4>"

    def config(self):
        cfg = self.cfg
        return {"workload": self.name, "layers": self.layers, "hidden": self.hidden, "kv": self.kv, "rank": self.r, "population": self.K,
                "rows": self.R, "weights": "int8 per-channel" if cfg.quant == "int8" else "int4 g128 asymmetric", "activations": "bf16",
                "mode": self.args.mode, "optimizer": self.args.optimizer,
                "step": "forward only" if self.forward_only else "sample + sigma + %d layers x (q,k,v,o) + reward + update" % self.layers}

    def close(self, keep_projs=False):
        self.cma.close()
        self.groups = None
        if self.owns_projs and not keep_projs:
            for gp in self.projs:
                gp.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--mode", choices=["w8a16", "w8a8"], default="w8a16", help="w8a16: bf16 activations as two int8 limbs on the int8 MFMA (default path); w8a8: one int8 limb")
    ap.add_argument("--workload", choices=WORKLOADS, default="c2_7b_decode",
                    help="c2 is the configuration the headline metric is quoted on; the others are side measurements")
    ap.add_argument("--layers", type=int, default=0, help="distinct layers cycled through (default: 28 for c2/c5, 1 for c3, 80 for c4)")
    ap.add_argument("--rows-per-cand", type=int, default=0)
    ap.add_argument("--population", type=int, default=0, help="candidates K (default: the workload's); with --rows-per-cand it sets the row count of a sweep point")
    ap.add_argument("--forward-only", action="store_true", help="time only the projections (no sampler / reward / update)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-side-workloads", action="store_true", help="only the workload named by --workload: no `workloads` and no `row_sweep` in the line")
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
    torch.cuda.set_device(0)
    # everything (the library's launches and torch's own fills) runs on one side stream, so that a step can be recorded
    stream = torch.cuda.Stream()
    torch.cuda.set_stream(stream)
    ctx = essa.Context(0, stream=stream)
    headline = args.workload == "c2_7b_decode" and not args.population and not args.rows_per_cand and not args.layers
    side = headline and not args.no_side_workloads and args.mode == "w8a16" and args.optimizer == "cma" and not args.forward_only \
        and not args.refresh_basis and not args.two_pass_reward

    main_b = Bench(essa, torch, np, wl, ctx, args.workload, args, layers=args.layers or None, population=args.population or None,
                   rows_per=args.rows_per_cand or None)
    if args.refresh_basis:
        if main_b.kind != essa.OPT_CMA:
            raise SystemExit("bench.py --refresh-basis times the eigendecomposition of the default optimizer's covariance")
        refresh_basis_report(main_b, essa, torch, np)
        return
    if args.calibrate_copy:
        src = torch.ones(64 * 1024 * 1024, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)           # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    res = main_b.run(args.steps, args.warmup)

    cpu = None
    if headline and not args.no_cpu_baseline:
        cpu = cpu_baseline(main_b.cfg, main_b.R, main_b.rows_per, args.mode)

    out = {
        "metric": "candidate-tokens/s through batched SVD-LoRA projections", "value": res["value"], "unit": "candidate-tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if args.mode == "w8a16" else "int8", "data": "synthetic",
        "config": main_b.config(), "roofline": res["roofline"], "cpu_baseline": cpu, "breakdown_ms": res["breakdown_ms"],
        "ms_per_step_with_events": res["ms_per_step_with_events"], "host_enqueue_ms_per_step": res["host_enqueue_ms_per_step"],
        "launches": res["launches"],
    }
    if side:
        out["row_sweep"] = row_sweep(essa, torch, np, wl, ctx, args, main_b.projs)
        out["workloads"] = side_workloads(essa, torch, np, wl, ctx, args, main_b, not args.no_cpu_baseline)
    print(json.dumps(out), flush=True)


def side_record(b, res):
    roof = res["roofline"]
    rec = {"config": b.config(), "value": res["value"], "unit": "candidate-tokens/s", "ms_per_step": res["ms_per_step"], "launches": res["launches"],
           "kernel": roof["kernel"], "avg_launch_us": roof["avg_launch_us"], "gemm_launches_timed": roof["launches"],
           "flops_per_launch": roof["flops_per_launch"], "bytes_per_launch": roof["bytes_per_launch"], "bound": roof["bound"],
           "peak": roof["peak"], "peak_unit": roof["unit"], "achieved": roof["achieved"], "frac": roof["frac"], "frac_of_hbm": roof["frac_of_hbm"],
           "int8_mfma": roof["int8_mfma"]}
    if "breakdown_ms" in res:
        rec["breakdown_ms"] = res["breakdown_ms"]
    return rec


def side_workloads(essa, torch, np, wl, ctx, args, main_b, with_cpu):
    """c3, c4 (all 80 layers) and c5 at their full sizes, a few steps each; c5 shares the 7B-shaped layers of the headline."""
    out = {}
    # c5 first: it reuses the headline's 112 projections
    b = Bench(essa, torch, np, wl, ctx, "c5_7b_es_iter", args, projs=main_b.projs)
    res = b.run(5, 1)
    rec = side_record(b, res)
    if with_cpu:
        rec["cpu_baseline"] = cpu_baseline_search(b, wl, np)
    out["c5_7b_es_iter"] = rec
    log("bench[c5]: %.2f ms/step, %.1f us/launch, frac %.3f" % (res["ms_per_step"], rec["avg_launch_us"], rec["frac"]))
    b.close()
    main_b.close()
    del b
    torch.cuda.empty_cache()
    for name, steps in (("c3_32b_prefill", 10), ("c4_72b_decode", 5)):
        b = Bench(essa, torch, np, wl, ctx, name, args)
        res = b.run(steps, 2, with_breakdown=False)
        out[name] = side_record(b, res)
        log("bench[%s]: %.2f ms/step, %.1f us/launch, frac %.3f" % (name, res["ms_per_step"], out[name]["avg_launch_us"], out[name]["frac"]))
        b.close()
        del b
        torch.cuda.empty_cache()
    return out


def row_sweep(essa, torch, np, wl, ctx, args, projs):
    """Forward of the 7B-shaped layers (all 28, so that the weights come from HBM) at 8 ... 512 rows, forward only:
    the regime in which the decode shapes are bound by the weight stream."""
    out = []
    for rows in (8, 16, 32, 64, 128, 256, 512):
        a2 = argparse.Namespace(**vars(args))
        a2.forward_only = True
        K = 32 if rows >= 32 else rows
        b = Bench(essa, torch, np, wl, ctx, "c2_7b_decode", a2, population=K, rows_per=rows // K, projs=projs)
        res = b.run(20, 3, with_breakdown=False)
        roof = res["roofline"]
        out.append({"rows": rows, "ms_per_step": res["ms_per_step"], "kernel": roof["kernel"], "avg_launch_us": roof["avg_launch_us"],
                    "bytes_per_launch": roof["bytes_per_launch"], "flops_per_launch": roof["flops_per_launch"], "bound": roof["bound"],
                    "frac": roof["frac"], "frac_of_hbm": roof["frac_of_hbm"], "achieved_GBs": roof["achieved_GBs"]})
        b.close()
    return out


def refresh_basis_report(b, essa, torch, np):
    """off the per-generation path: the eigendecomposition of the covariance, timed on its own"""
    n, K, cma, ctx = b.n, b.K, b.cma, b.ctx
    zero = np.zeros(n, np.float32)

    def refresh():
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        sweeps, off = cma.refresh_basis(ctx)
        torch.cuda.synchronize()
        return {"sweeps": sweeps, "off": off, "ms": 1e3 * (time.perf_counter() - t0)}
    cma.import_blob(essa.CmaState.pack_blob(n, 0, 0.32, zero, zero, zero, np.ones(n, np.float32), b.C0, np.eye(n, dtype=np.float32)))
    out = {"metric": "essa_cma_refresh_basis", "n": n, "cold": refresh(), "unchanged": refresh()}
    gen = torch.Generator(device="cuda")
    gen.manual_seed(0)
    for g in range(17):
        sd = torch.arange(1 + g * K, 1 + (g + 1) * K, dtype=torch.int32, device="cuda")
        essa.essa_cmaes_update(ctx, cma, sd, torch.randn(K, device="cuda", generator=gen), None)
    out["after_17_generations"] = refresh()
    print(json.dumps(out))


def _threads():
    try:
        from threadpoolctl import threadpool_info
        return max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        return 1


def cpu_baseline(cfg, R, rows_per, mode):
    """The oracle as it stands, timed on this machine's host cores on the first layers of the same workload."""
    import numpy as np

    import essa_workloads as wl
    import oracle as orc
    threads = _threads()
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


def cpu_baseline_search(b, wl, np):
    """The oracle's sampler and update at the full iteration's size (n = 3584, K = 64, dense basis), one call each."""
    import oracle as orc
    n, K = b.n, b.K
    st = orc.cma_state_init(n, np.float32(0.32))
    st.B, st.D, st.C = b.Q.astype(np.float64), b.d.astype(np.float64), b.C0.astype(np.float64)
    seeds = list(range(1, K + 1))
    t0 = time.perf_counter()
    theta, _ = orc.sample_candidates(st.m, st.sigma, st.B, st.D, seeds)
    t_sample = time.perf_counter() - t0
    F = -np.sum(theta * theta, axis=1)
    t0 = time.perf_counter()
    orc.cma_update(st, seeds, F.astype(np.float32))
    t_update = time.perf_counter() - t0
    return {"kind": "oracle", "cores": _threads(), "sampler_ms": 1e3 * t_sample, "update_ms": 1e3 * t_update,
            "sample": "essa_sample_candidates and essa_cmaes_update of c5 (n = %d, K = %d, dense basis), one call each, fp64 numpy" % (n, K)}


if __name__ == "__main__":
    main()
