#!/usr/bin/env python3
"""Benchmark of the partial-parameter-update local step on one MI355X.

A step = one pass of the whole hot path (forward over all parameters, restricted backward, AdamW on the
trainable subset, write-back) over one batch of seeded synthetic tokens that already sit in HBM.
Workload: the 1.3B-shape decoder (24 x 2048, 16 heads of 128, SwiGLU d_ff 8192, vocab 32000), batch 8 x 2048
tokens, trainable subset = a contiguous 1/32 slice of every layer's FFN hidden units.  The same run also times the
1/8 slice and the all-parameters-trainable (full back-propagation) step from the same library as the comparison
legs, and the CPU fp64 oracle on a bounded sample.  Prints ONE JSON line.
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

HP = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
PEAK_BF16_TFLOPS = 2500.0          # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def closed_form_flops(cfg, B, S, rho, detach=False):
    """Executed matmul FLOPs per step for the FFN-slice mask (rho < 1) or the all-trainable step (rho = 1):
    forward L(8Td^2 + 4 P d + 6TdF) + 2TdV, P = causal pairs; backward per the mask.
    detach: the ablation in which only the trainable slice enters the FFN input gradient (6TdF -> 6TdF rho there)."""
    T = B * S
    d, L, F, V = cfg["d_model"], cfg["n_layers"], cfg["d_ff"], cfg["vocab"]
    P = B * S * (S + 1) // 2
    fwd = L * (8 * T * d * d + 4 * P * d + 6 * T * d * F) + 2 * T * d * V
    if rho >= 1:
        return fwd, 2 * fwd
    Fk = F // round(1 / rho)
    Fj = Fk if detach else F          # hidden units that enter the FFN input gradient
    bwd = (2 * T * d * V + L * 6 * T * d * Fk + (L - 1) * 2 * T * d * Fj + 2 * T * d * Fk + (L - 1) * 4 * T * d * Fj
           + (L - 1) * (8 * T * d * d + 8 * P * d))
    return fwd, bwd


def closed_form_flops_paper_mask(cfg, B, S, mask):
    """Executed matmul FLOPs for the paper's masks (Section "Parameter Slicing": an FFN slice of every layer plus every
    non-MLP parameter, optionally with the Q/K/V projections restricted to a head range).  The embeddings are trainable, so
    nothing of the backward is skipped: per layer the input-gradient GEMMs run over all slices and heads (6TdF + 8Td^2 + 8Pd)
    and the weight-gradient GEMMs only over the trainable row blocks (Appendix "FLOPs calculation", rho_mlp and rho_attn)."""
    assert mask["train_embed"] and mask["train_wo"] and mask["train_lm_head"]
    T = B * S
    d, L, F, V, h = cfg["d_model"], cfg["n_layers"], cfg["d_ff"], cfg["vocab"], cfg["n_heads"]
    P = B * S * (S + 1) // 2
    Fk = mask["ffn_hi"] - mask["ffn_lo"]
    nhd = (mask["head_hi"] - mask["head_lo"]) * (d // h)
    fwd = L * (8 * T * d * d + 4 * P * d + 6 * T * d * F) + 2 * T * d * V
    bwd = 4 * T * d * V + L * (6 * T * d * Fk + 6 * T * d * F + 2 * T * d * d + 2 * T * d * d + 8 * P * d + 6 * T * d * nhd + 6 * T * d * d)
    return fwd, bwd


class PowerSampler:
    """Board power as the driver reports it (hwmon `power1_input`, microwatts) sampled every 20 ms from a thread while
    the timed steps run; `power1_cap` is the board's limit.  Reported because the matrix kernels of this path run
    against that limit (their clock drops under it), so energy per step is what bounds the step time."""

    def __init__(self):
        import glob
        self.path = self.cap = None
        for hw in sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*")):
            if os.path.exists(os.path.join(hw, "power1_input")):
                self.path = os.path.join(hw, "power1_input")
                self.cap = self._read(os.path.join(hw, "power1_cap"))
                break
        self.samples = []
        self._stop = False
        self._th = None

    @staticmethod
    def _read(path):
        try:
            with open(path) as f:
                return int(f.read().strip()) / 1e6
        except (OSError, ValueError):
            return None

    def _run(self):
        while not self._stop:
            v = self._read(self.path)
            if v is not None:
                self.samples.append(v)
            time.sleep(0.02)

    def __enter__(self):
        if self.path:
            import threading
            self._th = threading.Thread(target=self._run, daemon=True)
            self._th.start()
        return self

    def __exit__(self, *exc):
        self._stop = True
        if self._th:
            self._th.join()

    def report(self, seconds_per_step):
        if not self.samples:
            return None
        mean = sum(self.samples) / len(self.samples)
        return dict(mean_w=round(mean, 1), max_w=round(max(self.samples), 1), cap_w=self.cap, samples=len(self.samples),
                    joules_per_step=round(mean * seconds_per_step, 2),
                    source="hwmon power1_input, sampled every 20 ms over the timed steps (the driver's reading is itself smoothed)")


def run_leg(torch, pp, gen, cfg, weights, mask, batches, steps, warmup, time_gemm, outer=False, seed=0, options=()):
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    torch.cuda.reset_peak_memory_stats()
    detach = bool(cfg.get("detach_jacobian"))
    m = pp.LocalStepModel({k: v for k, v in cfg.items() if k != "detach_jacobian"}, mask)
    m.load_weights(weights)
    m.set_mask()
    for key, value in options:
        m.set_option(key, value)
    if detach:
        m.set_jacobian_slices(1)
    dev = [m.upload_tokens(t, g) for t, g in batches]
    for i in range(warmup):
        m.step(*dev[i % len(dev)], HP)
    torch.cuda.synchronize()
    # headline pass: nothing but the steps between the two synchronisations
    with PowerSampler() as power:
        t0 = time.perf_counter()
        for i in range(steps):
            m.step(*dev[i % len(dev)], HP)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    loss = float(m.loss.item())
    lc = m.launch_counts()
    # second pass of the same leg with every GEMM launch bracketed by HIP events on the model's stream (per-kernel roofline)
    gt, dt_timed = None, None
    if time_gemm:
        m.set_option("time_gemm", 1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            m.step(*dev[(steps + i) % len(dev)], HP)
        torch.cuda.synchronize()
        dt_timed = time.perf_counter() - t0
        gt = m.gemm_timing()
        m.set_option("time_gemm", 0)
    cnt = m.counters()
    mem = m.memory_report()
    peak_alloc = torch.cuda.max_memory_allocated()
    outer_res = None
    if outer:
        outer_res = time_outer_step(torch, pp, gen, m, seed)
    m.close()
    del m
    return dict(seconds=dt, seconds_gemm_timed=dt_timed, loss=loss, gemm=gt, counters=cnt, launch_counts=lc, memory=mem,
                peak_alloc=peak_alloc, outer=outer_res, power=power.report(dt / steps))


def time_outer_step(torch, pp, gen, m, seed, iters=100):
    """Config 5: the node's share of the outer step on the trainable subset of the model that just ran its local
    steps (theta_l = its current bf16 weights): delta, add the on-device sum of 31 seeded N(0, 1e-4) deltas, divide by
    the count, Nesterov update (lr 0.7, momentum 0.9).  HBM-bound: 24 algorithmic bytes per element."""
    n = m.n_trainable
    theta_g = torch.from_numpy(m.get_state("p")).to(m.dev)          # fp32 global parameters ~ the masters before drift
    mom = torch.zeros(n, dtype=torch.float32, device=m.dev)
    others = torch.empty(n, dtype=torch.float32, device=m.dev)
    keys = [gen.stream_key(seed, gen.STREAM_DELTAS, j + 1) for j in range(31)]
    pp.pp_synth_delta_sum(m.h, others.data_ptr(), n, keys, 1e-4)
    opt = pp.PPOuter(0.7, 0.9, 1, 32.0)
    for _ in range(3):
        pp.pp_outer_delta(m.h, theta_g.data_ptr(), mom.data_ptr(), others.data_ptr(), opt, None)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        pp.pp_outer_delta(m.h, theta_g.data_ptr(), mom.data_ptr(), others.data_ptr(), opt, None)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    gbps = 24.0 * n / (ms * 1e-3) / 1e9
    return dict(elements=int(n), ms_per_call=round(ms, 4), algorithmic_bytes_per_elem=24, achieved_gbps=round(gbps, 1),
                peak_gbps=PEAK_HBM_GBPS, frac=round(gbps / PEAK_HBM_GBPS, 4),
                note="one call = outer_kernel (delta, normalise, Nesterov, restart of local copy incl. 4 B/elem master write) + "
                     "shadow refresh of the updated blocks; timed with events on the model's stream")


def cpu_baseline(gen, cfg, weights, seed):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload: the full model (all layers, full width),
    ONE of the batch's full-length sequences, the benchmark's FFN slice; one forward + restricted backward + AdamW.
    FLOPs per token are those of the benchmark step, so tokens/s of the sample is the value, nothing is scaled."""
    import numpy as np
    from oracle import pp_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    L_s, B_s, S_s = cfg["n_layers"], 1, cfg["seq"]
    scfg = dict(cfg)
    keep = weights
    mask = gen.ffn_slice_mask(scfg, 0, cfg["n_slices"])
    tok, tgt = gen.make_tokens(scfg, seed, step=0, batch=B_s, seq=S_s)
    tr = O.LocalTrainer(scfg, keep, mask)
    t0 = time.perf_counter()
    loss, _ = tr.step(tok, tgt, HP, restricted=True)
    dt = time.perf_counter() - t0
    f_s = sum(closed_form_flops(scfg, B_s, S_s, 1.0 / cfg["n_slices"]))
    value = B_s * S_s / dt
    return dict(value=round(value, 3), unit="tokens/s", cores=int(cores), kind="oracle",
                sample=f"fp64 numpy oracle, the whole model ({L_s} layers, full width), B={B_s} of {cfg['batch']} sequences, S={S_s}, "
                       f"rho=1/{cfg['n_slices']}: one step (forward, restricted backward, AdamW) in {dt:.2f} s for {B_s * S_s} tokens "
                       f"({f_s / dt / 1e9:.1f} GFLOP/s fp64); measured, not extrapolated",
                seconds=round(dt, 3), loss=round(float(loss), 5))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="1p3b", choices=["1p3b", "125m"])
    ap.add_argument("--legs", default="all", choices=["main", "all", "paper"],
                    help="'main' = only the headline mask; 'all' = also rho=1/8, all-trainable, recomputation, the detach ablation and the "
                         "paper's own masks; 'paper' = headline + the paper's masks")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--seed", type=int, default=1234)
    ap.add_argument("--set", action="append", default=[], metavar="KEY=INT",
                    help="library option for every leg's model (pp_set_option), e.g. --set dw_tn=0 for a same-box A/B")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run three plain 1 GiB streaming copies (torch neg kernel, out = -in): under rocprofv3 --pmc FETCH_SIZE / "
                         "WRITE_SIZE their readings give the counter scale for the HBM-traffic figures")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs one node's local step on ONE GPU (no collectives exist in it); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import pp_inputs as gen
    import paper_2509_22418_amd as pp

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    if args.calibrate:
        # streaming kernel of known size: reads 1 GiB, writes 1 GiB (shows up as torch's neg kernel)
        b = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        a = torch.empty_like(b)
        for _ in range(3):
            torch.neg(b, out=a)
        torch.cuda.synchronize()
        del a, b
    cfg = gen.make_config(args.workload)
    B, S = cfg["batch"], cfg["seq"]
    n_slices = cfg["n_slices"]
    t0 = time.perf_counter()
    weights = gen.make_weights(cfg, args.seed, threads=16)
    log(f"[bench] weights generated in {time.perf_counter() - t0:.1f} s")
    batches = [gen.make_tokens(cfg, args.seed, step=i) for i in range(4)]

    legs = [("rho=1/%d" % n_slices, gen.ffn_slice_mask(cfg, 0, n_slices), 1.0 / n_slices, cfg)]
    if args.legs == "all":
        legs.append(("rho=1/8", gen.ffn_slice_mask(cfg, 0, 8), 1.0 / 8, cfg))
        legs.append(("all-trainable", dict(all=1), 1.0, cfg))
        if n_slices == 8:
            legs.pop(1)
        # the paper's memory regime: full activation recomputation (same results bit for bit, less workspace, more time)
        legs.append(("rho=1/%d+recompute" % n_slices, gen.ffn_slice_mask(cfg, 0, n_slices), 1.0 / n_slices, dict(cfg, recompute=1)))
        # the appendix's detach-all-but-k ablation (a different, cheaper gradient that the paper reports to diverge)
        legs.append(("rho=1/%d+detach-ablation" % n_slices, gen.ffn_slice_mask(cfg, 0, n_slices), 1.0 / n_slices, dict(cfg, detach_jacobian=1)))
    if args.legs in ("all", "paper"):
        # the paper's own masks in the paper's memory regime (Table 1: "1/4 mlps" and "1/4 mlps + 1/4 heads"; full activation
        # recomputation, Experimental Setup): every non-MLP parameter trainable, so 0.5-0.8 B packed elements go through AdamW
        legs.append(("paper:1/4 mlps+recompute", gen.paper_mlp_mask(cfg, 0, 4), None, dict(cfg, recompute=1)))
        legs.append(("paper:1/4 mlps+1/4 heads+recompute", gen.paper_mlp_mask(cfg, 0, 4, slice_heads=True), None, dict(cfg, recompute=1)))
    results = {}
    outer_step = None
    for name, mask, rho, leg_cfg in legs:
        t1 = time.perf_counter()
        r = run_leg(torch, pp, gen, leg_cfg, weights, mask, batches, args.steps, args.warmup, time_gemm=True,
                    outer=(name == legs[0][0]), seed=args.seed, options=[(kv.split("=")[0], int(kv.split("=")[1])) for kv in args.set])
        if rho is None:
            fwd, bwd = closed_form_flops_paper_mask(cfg, B, S, mask)
        else:
            fwd, bwd = closed_form_flops(cfg, B, S, rho, detach=bool(leg_cfg.get("detach_jacobian")))
        ms = r["seconds"] / args.steps * 1e3
        executed = r["counters"]["flops_fwd"] + r["counters"]["flops_bwd"]
        results[name] = dict(
            tokens_per_s=round(B * S * args.steps / r["seconds"], 1), ms_per_step=round(ms, 3),
            flops_executed=executed, flops_closed_form=fwd + bwd, flops_match=bool(executed == fwd + bwd),
            step_tflops=round((fwd + bwd) / (ms * 1e-3) / 1e12, 1),
            step_mfma_frac=round((fwd + bwd) / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
            gemm_tflops=round(r["gemm"]["flops"] / (r["gemm"]["ms"] * 1e-3) / 1e12, 1) if r["gemm"]["ms"] > 0 else None,
            gemm_ms_per_step=round(r["gemm"]["ms"] / args.steps, 3), gemm_launches_per_step=r["gemm"]["launches"] // args.steps,
            ms_per_step_with_gemm_events=round(r["seconds_gemm_timed"] / args.steps * 1e3, 3),
            plain_kernel_calls=r["launch_counts"]["plain_calls"], matrix_core_calls=r["launch_counts"]["matrix_core_calls"],
            n_trainable=r["counters"]["n_trainable"], adamw_bytes=r["counters"]["adamw_bytes"],
            hbm_bytes=r["memory"], peak_allocated_gb=round(r["peak_alloc"] / 2 ** 30, 3), final_loss=round(r["loss"], 5),
            board_power=r["power"])
        if r["outer"]:
            outer_step = r["outer"]
        if r["launch_counts"]["plain_calls"]:
            raise SystemExit(f"bench.py: leg {name} ran {r['launch_counts']['plain_calls']} contraction(s) on the plain kernels; "
                             "the benchmark shapes must run on the matrix-core kernels throughout")
        log(f"[bench] leg {name}: {results[name]['tokens_per_s']} tokens/s, {ms:.2f} ms/step, "
            f"{results[name]['step_tflops']} TFLOP/s on executed FLOPs, GEMM {results[name]['gemm_tflops']} TFLOP/s "
            f"({time.perf_counter() - t1:.1f} s incl. setup)")

    main_name = legs[0][0]
    mr = results[main_name]
    gemm_ms_launch = mr["gemm_ms_per_step"] / max(mr["gemm_launches_per_step"], 1)
    roofline = dict(bound="mfma", kernel="gemm_nt_mfma_dl_kernel (all forward / dX / dW GEMM launches of the step)",
                    achieved=mr["gemm_tflops"], peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                    frac=round(mr["gemm_tflops"] / PEAK_BF16_TFLOPS, 4) if mr["gemm_tflops"] else None, traffic=None,
                    traffic_note="null on purpose: FETCH_SIZE / WRITE_SIZE sit between L2 and the fabric, so for a GEMM they count "
                                 "L2 fills served by the Infinity Cache as well (about 0.9 GB per launch on average against 0.13-0.27 GB "
                                 "of operands, profiles/hbm_traffic_1p3b_rho32_pmc.txt), not HBM bytes; for the HBM-bound kernels of "
                                 "the step the same counters equal the algorithmic bytes within 1-2 %; L2 hit rate of the GEMM instantiations 0.69-0.80 "
                                 "(profiles/l2_lds_counters_1p3b_rho32_pmc.txt)",
                    avg_launch_ms=round(gemm_ms_launch, 4), launches_per_step=mr["gemm_launches_per_step"],
                    measured_in="a second pass of the same leg with an event pair around every GEMM launch "
                                f"({mr['ms_per_step_with_gemm_events']} ms/step); the headline ms_per_step is the pass without events",
                    gemm_share_of_step_time=round(mr["gemm_ms_per_step"] / mr["ms_per_step_with_gemm_events"], 3))
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(gen, cfg, weights, args.seed)
        log(f"[bench] cpu oracle: {cpu['value']} tokens/s on {cpu['cores']} threads")

    out = {
        "metric": "local-step tokens/s at 1.3B shape on 1 GPU" if args.workload == "1p3b" else "local-step tokens/s at 125M shape on 1 GPU",
        "value": mr["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": mr["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}-shape decoder, {cfg['n_layers']}x{cfg['d_model']}, {cfg['n_heads']} heads, d_ff {cfg['d_ff']}, "
                               f"vocab {cfg['vocab']}, batch {B} x seq {S}, trainable = 1/{n_slices} FFN slice per layer (partial update), "
                               "Zipf(1.1) tokens, N(0,0.02) weights",
                   "global_batch": B, "seq_len": S, "trainable_fraction_of_ffn": f"1/{n_slices}"},
        "step_mfma_frac": mr["step_mfma_frac"], "peak_hbm_gb": mr["peak_allocated_gb"],
        "board_power": mr["board_power"],
        "roofline": roofline, "cpu_baseline": cpu, "outer_step": outer_step, "legs": results,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
