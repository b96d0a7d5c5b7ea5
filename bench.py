#!/usr/bin/env python3
"""Benchmark of the draft-graph verification step on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c3|c2|c4|c5] [--no-cpu-baseline]

One step = the whole hot path over one batch of synthetic input: embedding of G block states,
L transformer layers (shared-prefix attention + projections; the last one computes only the rows of
masked positions behind its attention), LM head reduced to top-1/confidence/unmask, next-state build
and the acceptance walk, all in one C-ABI call with weights, prefix KV and inputs already resident in
HBM, followed by the acceptance walk against the workload's planted target states (one more
one-wavefront launch).  Prints ONE JSON line; `other_configs` holds the other workload configurations
measured the same way, `decision_check` the device step's decisions against the oracle.

metric  = draft states verified per second (G / step latency), whole job on one GPU
roofline= the dominant kernel (the SwiGLU gate/up MFMA GEMM): algorithmic flop of one launch /
          its average launch duration, timed here with HIP events around back-to-back launches
          of that kernel on the same shapes and buffers the step uses
cpu_baseline = the CPU oracle (oracle/, float64 numpy) timed on this host on a bounded sample
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
LOGIT_SCALE = 8.0             # synthetic knob: random-init logits are flat, this makes ~1/3 of positions pass tau


def step_work(cfg, n_masked):
    """Algorithmic flop and HBM bytes of one step (per state per layer: 2*B*params flop + the attention's
    4*B*(P+B)*hd*Hq; weights and cached keys / values once per step; the head on the masked rows only)."""
    M = cfg.G * cfg.B
    params_layer = cfg.d * cfg.Hq * cfg.hd * 2 + cfg.d * cfg.Hkv * cfg.hd * 2 + 3 * cfg.d * cfg.F
    # the last layer computes its output projection and FFN on the masked rows only (exact: nothing else is read
    # afterwards), so the algorithmic count takes n_masked rows for that part
    params_behind_attention = cfg.d * cfg.Hq * cfg.hd + 3 * cfg.d * cfg.F
    flop = cfg.L * (2.0 * M * params_layer + 4.0 * cfg.B * (cfg.P + cfg.B) * cfg.hd * cfg.Hq * cfg.G) \
        - 2.0 * (M - n_masked) * params_behind_attention + 2.0 * n_masked * cfg.V * cfg.d
    nbytes = cfg.L * (2.0 * params_layer + 2.0 * 2 * cfg.P * cfg.Hkv * cfg.hd) + 2.0 * cfg.V * cfg.d + 2.0 * M * cfg.d
    return flop, nbytes


def build_workload(sp, synth, key, dev, seed, n_states=0):
    """Synthetic model and inputs of one workload configuration, generated on the device from the seed."""
    import numpy as np
    import torch
    cfg = synth.CONFIGS[key]
    layers = [synth.layer_weights(cfg, l, seed, device=dev) for l in range(cfg.L)]
    prefix = [synth.prefix_kv(cfg, l, seed, device=dev) for l in range(cfg.L)]
    hw = synth.head_weights(cfg, seed, device=dev)
    w_embed = synth.embed_weights(cfg, seed, device=dev)
    states, edges = synth.draft_graph(key, cfg, seed)
    if n_states:
        states = states[:n_states]
        edges = edges[(edges < n_states).all(axis=1)].reshape(-1, 2)
        cfg = cfg.scaled(G=n_states)
    # target states "sampled from seed" for the acceptance measurement: a planted path of seeded depth
    depth = int(np.random.default_rng(seed).integers(1, 5))
    planted, path = synth.planted_targets(states, edges, cfg.V, depth, seed)
    w = dict(cfg=cfg, key=key, layers=layers, prefix=prefix, hw=hw, w_embed=w_embed, states=states, edges=edges,
             planted=planted, planted_path=path)
    w["d_states"] = torch.from_numpy(states).to(dev)
    w["d_edges"] = torch.from_numpy(np.ascontiguousarray(edges)).to(dev) if len(edges) else None
    w["d_planted"] = torch.from_numpy(planted).to(dev)
    w["plan"] = sp.StepPlan(sp.cfg_from_synth(cfg), [sp.layer_weights(x) for x in layers],
                            [sp.prefix_kv(k, v) for k, v in prefix], w_embed, hw["final_norm"], hw["w_vocab"], cfg.G,
                            cfg.B, cfg.P, cfg.threshold, logit_scale=LOGIT_SCALE, device=dev, keep_hidden=False)
    w["walk_res"] = torch.empty(4, dtype=torch.int32, device=dev)
    w["walk_state"] = torch.empty(cfg.B, dtype=torch.int32, device=dev)
    return w


def one_step(sp, w):
    """The timed unit: the whole step in one call (its walk runs on the step's own next states), then the
    acceptance walk against the planted target states of the workload (one more one-wavefront launch)."""
    w["plan"].run(w["d_states"], w["d_edges"])
    sp.graph_accept(w["d_edges"], w["d_states"], w["d_planted"], 0, res=w["walk_res"], state=w["walk_state"])


def time_steps(sp, w, steps, warmup):
    import torch
    for _ in range(warmup):
        one_step(sp, w)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    w0 = time.perf_counter()
    for a, b in ev:
        a.record()
        one_step(sp, w)
        b.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - w0
    return wall * 1e3 / steps, sorted(a.elapsed_time(b) for a, b in ev)


def time_dominant_kernel(sp, w, dev, iters):
    """The gate/up SwiGLU GEMM alone: same shapes as in the step, weights rotating over the layers, HIP events on the
    launch stream around back-to-back launches."""
    import torch
    cfg, layers = w["cfg"], w["layers"]
    M = cfg.G * cfg.B
    x = torch.randn((M, cfg.d), device=dev, dtype=torch.float32).to(torch.bfloat16)
    act = torch.empty((M, cfg.F), device=dev, dtype=torch.bfloat16)
    for lw in layers[:2]:
        sp.gemm(sp.GEMM_SWIGLU, x, lw["w_gate"], lw["w_up"], out=act)
    torch.cuda.synchronize()
    k0, k1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_launch = 0
    k0.record()
    for _ in range(iters):
        for lw in layers:
            sp.gemm(sp.GEMM_SWIGLU, x, lw["w_gate"], lw["w_up"], out=act)
            n_launch += 1
    k1.record()
    torch.cuda.synchronize()
    return k0.elapsed_time(k1) / n_launch, n_launch


def weight_stream_leg(sp, w, dev):
    """The four projections of a layer alone, through spiffy_gemm with the step's shapes (QKV as one fused weight
    matrix, output and down projections with their K slices and reduction), weights rotating over eight layers:
    algorithmic bytes over time against the HBM peak.  For the workloads whose projections are weight streams."""
    import torch
    cfg, layers = w["cfg"], w["layers"][:8]
    M, d, F = cfg.G * cfg.B, cfg.d, cfg.F
    qd = cfg.Hq * cfg.hd
    x = torch.randn((M, d), device=dev, dtype=torch.float32).to(torch.bfloat16)
    xa = torch.randn((M, qd), device=dev, dtype=torch.float32).to(torch.bfloat16)
    xf = torch.randn((M, F), device=dev, dtype=torch.float32).to(torch.bfloat16)
    r = torch.randn((M, d), device=dev, dtype=torch.float32).to(torch.bfloat16)
    ws = torch.empty(4 * M * d * 4 + 256, dtype=torch.uint8, device=dev)
    wqkv = [torch.cat([lw["wq"], lw["wk"], lw["wv"]]) for lw in layers]
    legs = {
        "qkv": (lambda i: sp.gemm(sp.GEMM_STORE, x, wqkv[i], out=o_qkv), 2.0 * (wqkv[0].numel() + M * d + M * wqkv[0].shape[0])),
        "output_projection_and_reduction": (lambda i: sp.gemm(sp.GEMM_RESID, xa, layers[i]["wo"], R=r, out=o_d, workspace=ws),
                                            2.0 * (d * qd + M * qd + 2 * M * d)),
        "gate_up": (lambda i: sp.gemm(sp.GEMM_SWIGLU, x, layers[i]["w_gate"], layers[i]["w_up"], out=o_f),
                    2.0 * (2 * F * d + M * d + M * F)),
        "down_projection_and_reduction": (lambda i: sp.gemm(sp.GEMM_RESID, xf, layers[i]["w_down"], R=r, out=o_d, workspace=ws),
                                          2.0 * (d * F + M * F + 2 * M * d)),
    }
    o_qkv = torch.empty((M, wqkv[0].shape[0]), device=dev, dtype=torch.bfloat16)
    o_d = torch.empty((M, d), device=dev, dtype=torch.bfloat16)
    o_f = torch.empty((M, F), device=dev, dtype=torch.bfloat16)
    out = {}
    for name, (fn, nbytes) in legs.items():
        for i in range(len(layers)):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            for i in range(len(layers)):
                fn(i)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / (3 * len(layers))
        out[name] = {"us": us, "algorithmic_MB": nbytes / 1e6, "GBs": nbytes / us / 1e3,
                     "frac_of_hbm_peak": nbytes / us / 1e3 / PEAK_HBM_GBS}
    return out


def roofline_of(cfg, k_ms, n_launch, traffic):
    """Roofline object of the SwiGLU GEMM: against the bf16 MFMA peak, or against the HBM peak when the launch moves
    more bytes per flop than the chip's balance point (few rows: the small-block workload, --states)."""
    M = cfg.G * cfg.B
    flop_launch = 2.0 * M * cfg.d * 2 * cfg.F
    alg_bytes = 2.0 * (2 * cfg.F * cfg.d + M * cfg.d + M * cfg.F)
    achieved = flop_launch / (k_ms * 1e-3) / 1e12
    # one "launch" is one gate/up projection: a single kernel launch except where the library splits the columns over
    # two launches of the same kernel (workload c4: wide tiles over whole rounds of workgroups, narrower ones for the rest)
    r = {"kernel": "gemm_bf16_mfma_kernel<EPI_SWIGLU> (gate/up projection)", "bound": "mfma", "achieved": achieved,
         "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic,
         "algorithmic_bytes_per_launch": alg_bytes, "avg_launch_ms": k_ms, "flop_per_launch": flop_launch,
         "launches_timed": n_launch}
    if flop_launch / alg_bytes < PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
        gbs = alg_bytes / (k_ms * 1e-3) / 1e9
        r.update({"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS})
    return r


def other_config_leg(sp, synth, key, dev, seed, steps, warmup, kernel_iters, n_states=0):
    """One of the other workload configurations on the same build: the whole step and its dominant kernel, measured
    the same way as the headline; everything is freed before the next one.  n_states: only the first states of the
    workload's draft graph (the paper's own operating point is one true block and three drafts)."""
    import torch
    w = build_workload(sp, synth, key, dev, seed, n_states)
    cfg = w["cfg"]
    ms, per = time_steps(sp, w, steps, warmup)
    k_ms, n_launch = time_dominant_kernel(sp, w, dev, kernel_iters)
    n_masked = int((w["states"] == cfg.mask_id).sum())
    flop, nbytes = step_work(cfg, n_masked)
    out = {"workload": cfg.name, "G": cfg.G, "B": cfg.B, "P": cfg.P, "L": cfg.L, "ms_per_step": ms,
           "states_per_s": cfg.G / (ms * 1e-3), "step_latency_ms_p50": per[len(per) // 2],
           "step_flop": flop, "step_algorithmic_bytes": nbytes,
           "step_frac_of_bf16_peak": flop / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
           "step_frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
           "step_bound": "hbm" if nbytes / (PEAK_HBM_GBS * 1e9) > flop / (PEAK_BF16_TFLOPS * 1e12) else "mfma",
           "roofline": roofline_of(cfg, k_ms, n_launch, None if n_states else stored_traffic(key)),
           "planted_walk": walk_outcome(w)}
    if out["roofline"]["bound"] == "hbm":
        out["weight_streams"] = weight_stream_leg(sp, w, dev)
    del w
    torch.cuda.empty_cache()
    return out


def walk_outcome(w):
    res = w["walk_res"].cpu().tolist()
    own = w["plan"].out["result"].cpu().tolist()
    return {"planted_depth": len(w["planted_path"]) - 1, "accepted_depth": res[1], "accepted_node": res[0],
            "planted_path": [int(x) for x in w["planted_path"]],
            "walk_on_the_steps_own_next_states": {"accepted_node": own[0], "depth": own[1]}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="c3")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel-iters", type=int, default=5)
    ap.add_argument("--step-only", action="store_true",
                    help="skip the legs outside the timed step (drafting, decode loop, dual cache, other configurations): "
                         "for profiles")
    ap.add_argument("--states", type=int, default=0,
                    help="verify only the first G states of the workload's draft graph (the paper's own operating point "
                         "is G = 4); implies --step-only")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run plain device copies of 1 GiB (calibration of the FETCH_SIZE/WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU (no collectives, no sharding); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    if not os.path.exists(os.path.join(ROOT, "paper_2509_18085_amd", "libspiffy.so")):
        from paper_2509_18085_amd import build as _build      # nothing built yet: build; otherwise load what is there
        _build.build()
    from paper_2509_18085_amd import spiffy as sp, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    seed = synth.DEFAULT_SEED
    if args.states:
        if not 1 <= args.states <= synth.CONFIGS[args.config].G:
            sys.exit("bench.py: --states must lie in 1..%d for %s" % (synth.CONFIGS[args.config].G, args.config))
        args.step_only = True
    t0 = time.time()
    w = build_workload(sp, synth, args.config, dev, seed, args.states)
    cfg, layers, prefix, hw, w_embed = w["cfg"], w["layers"], w["prefix"], w["hw"], w["w_embed"]
    states, edges, d_states, d_edges, plan = w["states"], w["edges"], w["d_states"], w["d_edges"], w["plan"]
    torch.cuda.synchronize()
    t_setup = time.time() - t0

    if args.copy_probe:     # a copy kernel of known size: 1 GiB read, 1 GiB written per launch
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(3)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- whole step ------------------------------------------------------------------------------
    ms_per_step, per = time_steps(sp, w, args.steps, args.warmup)
    out = plan.out
    res = out["result"].cpu().tolist()
    m = states == cfg.mask_id
    n_masked = int(m.sum())

    # ---- dominant kernel in isolation: gate/up SwiGLU GEMM, same shapes, weights rotating over layers
    k_ms, n_launch = time_dominant_kernel(sp, w, dev, args.kernel_iters)
    flop_step, bytes_step = step_work(cfg, n_masked)

    line = {
        "metric": "draft_states_verified_per_s",
        "value": cfg.G / (ms_per_step * 1e-3),
        "unit": "states/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": cfg.name, "L": cfg.L, "d": cfg.d, "Hq": cfg.Hq, "Hkv": cfg.Hkv, "hd": cfg.hd,
                   "F": cfg.F, "V": cfg.V, "P": cfg.P, "B": cfg.B, "G": cfg.G, "threshold": cfg.threshold,
                   "logit_scale": LOGIT_SCALE, "n_edges": int(len(edges)), "masked_positions": n_masked,
                   "seed": seed},
        "step_latency_ms": {"p10": per[len(per) // 10], "p50": per[len(per) // 2], "p90": per[(len(per) * 9) // 10]},
        "step_flop": flop_step,
        "step_algorithmic_bytes": bytes_step,
        "step_tflops": flop_step / (ms_per_step * 1e-3) / 1e12,
        "step_frac_of_bf16_peak": flop_step / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "outcome": {"accepted_node": res[0], "depth": res[1], "unmasked": int(out["unmask"].sum().item()),
                    "planted_walk": walk_outcome(w)},
        "roofline": roofline_of(cfg, k_ms, n_launch, stored_traffic(args.config) if not args.states else None),
        "setup_s": t_setup,
    }
    if not args.states:
        line["roofline"]["traffic_source"] = ("profiles/hbm_traffic_%s_gemm_kernels.txt (rocprofv3 --pmc FETCH_SIZE / "
                                              "WRITE_SIZE, scaled by a 1 GiB copy probe; bytes per launch)" % args.config)

    # what this chip sustains on the same units with nothing in the way: a register-only MFMA loop, a read-only stream
    line["measured_peaks"] = peaks_leg(sp, dev)
    mp = line["measured_peaks"]
    line["roofline"]["frac_of_measured_peak"] = (
        line["roofline"]["achieved"] / mp["hbm_read_GBs"] if line["roofline"]["bound"] == "hbm"
        else line["roofline"]["achieved"] / mp["mfma_bf16_random_operands_tflops"])

    if not args.step_only:
        line["vendor_library_context"] = library_leg(sp, w, dev)
        line["next_step_drafting"] = drafting_leg(sp, cfg, plan, d_states, dev)
        line["decode_loop"] = decode_leg(sp, cfg, layers, prefix, hw, w_embed, dev)
        line["dual_cache_step"] = dual_cache_leg(sp, cfg, layers, prefix, hw, w_embed, d_states, d_edges, dev, seed)
        line["full_sequence_step"] = full_sequence_leg(sp, cfg, layers, prefix, hw, w_embed, d_states, d_edges, dev)
        line["calibration_subgraph_search"] = subgraph_leg(sp, dev, seed)

    if not args.no_cpu_baseline:
        plan.keep_hidden = True             # once more with the hidden states written out: the oracle's head reads them
        one_step(sp, w)
        torch.cuda.synchronize()
        line["cpu_baseline"], line["decision_check"] = cpu_baseline(cfg, layers, prefix, hw, states, edges, plan.out)

    if not args.step_only:
        # the other workload configurations, one after the other, each freed before the next; the headline stays above
        del w, layers, prefix, hw, w_embed, plan, out, d_states, d_edges
        torch.cuda.empty_cache()
        line["other_configs"] = {}
        for key in ("c2", "c4", "c5"):
            if key != args.config:
                line["other_configs"][key] = other_config_leg(sp, synth, key, dev, seed, 10, 2, 2)
        # the paper's own operating point (D* = 3: the true block and three drafts) at the headline model shape
        line["other_configs"]["c3_four_states"] = other_config_leg(sp, synth, "c3", dev, seed, 10, 2, 2, n_states=4)
        # and the vanilla pass (one state): every projection is a weight stream, the regime of the HBM roofline
        line["other_configs"]["c3_one_state"] = other_config_leg(sp, synth, "c3", dev, seed, 10, 2, 2, n_states=1)
    print(json.dumps(line))


def library_leg(sp, w, dev):
    """Context, not a target and not on the product path: the image's GEMM library (torch.matmul, bf16) on the
    projection shapes of this workload, weights rotating over four layers, beside the same projections through
    spiffy_gemm.  The library computes the bare products: no SwiGLU, no residual, no K-slice reduction."""
    import torch
    cfg, layers = w["cfg"], w["layers"][:4]
    M, d, F, qd = cfg.G * cfg.B, cfg.d, cfg.F, cfg.Hq * cfg.hd
    x = torch.randn((M, d), device=dev, dtype=torch.float32).to(torch.bfloat16)
    xa = torch.randn((M, qd), device=dev, dtype=torch.float32).to(torch.bfloat16)
    xf = torch.randn((M, F), device=dev, dtype=torch.float32).to(torch.bfloat16)
    r = torch.randn((M, d), device=dev, dtype=torch.float32).to(torch.bfloat16)
    ws = torch.empty(4 * M * d * 4 + 256, dtype=torch.uint8, device=dev)
    wqkv = [torch.cat([lw["wq"], lw["wk"], lw["wv"]]) for lw in layers]
    wgu = [torch.cat([lw["w_gate"], lw["w_up"]]) for lw in layers]
    o_qkv = torch.empty((M, wqkv[0].shape[0]), device=dev, dtype=torch.bfloat16)
    o_gu = torch.empty((M, 2 * F), device=dev, dtype=torch.bfloat16)
    o_d = torch.empty((M, d), device=dev, dtype=torch.bfloat16)
    o_f = torch.empty((M, F), device=dev, dtype=torch.bfloat16)
    pairs = {
        "qkv": (lambda i: torch.matmul(x, wqkv[i].t(), out=o_qkv), lambda i: sp.gemm(sp.GEMM_STORE, x, wqkv[i], out=o_qkv)),
        "output_projection": (lambda i: torch.matmul(xa, layers[i]["wo"].t(), out=o_d),
                              lambda i: sp.gemm(sp.GEMM_RESID, xa, layers[i]["wo"], R=r, out=o_d, workspace=ws)),
        "gate_up": (lambda i: torch.matmul(x, wgu[i].t(), out=o_gu),
                    lambda i: sp.gemm(sp.GEMM_SWIGLU, x, layers[i]["w_gate"], layers[i]["w_up"], out=o_f)),
        "down_projection": (lambda i: torch.matmul(xf, layers[i]["w_down"].t(), out=o_d),
                            lambda i: sp.gemm(sp.GEMM_RESID, xf, layers[i]["w_down"], R=r, out=o_d, workspace=ws)),
    }

    def timed(fn):
        for i in range(len(layers)):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(4):
            for i in range(len(layers)):
                fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (4 * len(layers))

    out = {}
    for rd in range(2):                 # interleaved: the second pass is the one reported (clocks settled)
        for name, (lib_fn, own_fn) in pairs.items():
            out[name] = {"library_us": timed(lib_fn), "spiffy_gemm_us": timed(own_fn)}
    out["note"] = ("torch.matmul (the image's GEMM library) against spiffy_gemm on the same shapes and weights; the library "
                   "computes the bare product, spiffy_gemm includes the SwiGLU epilogue or the residual and the reduction "
                   "of its K slices")
    return out


def peaks_leg(sp_unused, dev):
    """Measured peaks beside the published ones: dense bf16 matrix instructions on register operands (all zero, and
    pseudo-random in (-1, 1): the chip clocks lower when the operands switch), one read-only pass over 4 GiB, and a
    device-to-device copy of 1 GiB (bytes read + bytes written)."""
    import torch
    from paper_2509_18085_amd import probe as sp      # libspiffy_probe.so: not part of the verification library
    sink = torch.empty(1024, dtype=torch.float32, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def mfma(rand):
        sp.probe_mfma(20000, rand, sink)
        torch.cuda.synchronize()
        e0.record()
        flop = sp.probe_mfma(100000, rand, sink)
        e1.record()
        torch.cuda.synchronize()
        return flop / (e0.elapsed_time(e1) * 1e-3) / 1e12

    out = {"mfma_bf16_zero_operands_tflops": mfma(False), "mfma_bf16_random_operands_tflops": mfma(True)}
    src = torch.empty(4 << 30, dtype=torch.uint8, device=dev).fill_(1)
    sink32 = torch.zeros(1, dtype=torch.int32, device=dev)
    sp.probe_hbm_read(src, sink32)
    torch.cuda.synchronize()
    e0.record()
    n = 0
    for _ in range(3):
        n += sp.probe_hbm_read(src, sink32)
    e1.record()
    torch.cuda.synchronize()
    out["hbm_read_GBs"] = n / (e0.elapsed_time(e1) * 1e-3) / 1e9
    a, b = src[:1 << 30], src[1 << 30:2 << 30]
    b.copy_(a)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(3):
        b.copy_(a)
    e1.record()
    torch.cuda.synchronize()
    out["hbm_copy_GBs"] = 3 * 2.0 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9
    out["note"] = ("register-only v_mfma_f32_32x32x16_bf16 loop on every SIMD (spiffy_probe_mfma) and a read-only pass over "
                   "4 GiB (spiffy_probe_hbm_read), both from libspiffy_probe.so; published peaks: 2500 TFLOP/s, 8000 GB/s")
    return out


def drafting_leg(sp, cfg, plan, d_states, dev, iters=50):
    """Not part of the timed step: latency of building and pruning the next step's draft graph on the
    device (spiffy_draft_prune) from the accepted node's top-1 rows, G-1 formulas 'the s most confident
    positions' pruned to (G-1)/2."""
    import numpy as np
    import torch
    D = cfg.G - 1
    formulas = [[(i, 1) for i in range(1, (n % cfg.B) + 2)] for n in range(D)]
    off = torch.tensor(np.cumsum([0] + [len(f) for f in formulas]).astype(np.int32), device=dev)
    pairs = torch.tensor(np.array([p for f in formulas for p in f], np.int32).reshape(-1, 2), device=dev)
    sets = [set()] + [set(f) for f in formulas]
    e = [(a, c) for a in range(D + 1) for c in range(1, D + 1) if a != c and sets[a] < sets[c]]
    edges = torch.tensor(np.array(e, np.int32).reshape(-1, 2), device=dev) if e else None
    node = int(plan.out["result"][0].item())
    state = plan.out["accepted_state"]
    tok = plan.out["argmax"][node].reshape(cfg.B, 1).contiguous()
    prob = plan.out["conf"][node].reshape(cfg.B, 1).contiguous()
    d_star = max(1, D // 2)
    for _ in range(3):
        out = sp.draft_prune(state, cfg.mask_id, tok, prob, off, pairs, edges, d_star)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        out = sp.draft_prune(state, cfg.mask_id, tok, prob, off, pairs, edges, d_star)
    e1.record()
    torch.cuda.synchronize()
    draft_us = e0.elapsed_time(e1) * 1e3 / iters
    # drafting source with vocabulary ranks up to 3: top-3 rows of the accepted node from what the head left
    scfg = plan.cfg
    for _ in range(3):
        sp.head_topk(scfg, plan.w_vocab, d_states, 3, LOGIT_SCALE, plan.workspace, result=plan.out["result"],
                     after_step=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(iters):
        sp.head_topk(scfg, plan.w_vocab, d_states, 3, LOGIT_SCALE, plan.workspace, result=plan.out["result"],
                     after_step=True)
    e1.record()
    torch.cuda.synchronize()
    return {"draft_prune_us": draft_us, "head_top3_us": e0.elapsed_time(e1) * 1e3 / iters, "formulas": D, "d_star": d_star,
            "edges_in": len(e), "kept_nodes": int(out["counts"][0].item()), "edges_out": int(out["counts"][1].item()),
            "note": "includes the binding's output allocations; one 64-lane kernel launch"}


def decode_leg(sp, cfg, layers, prefix, hw, w_embed, dev, n_blocks=8):
    """Not part of the timed step: a whole generation of n_blocks blocks (256 tokens at B = 32) with the host loop
    of speculative block decoding (Alg. 1) on the same model: per forward pass verify -> top-K -> draft/prune,
    with G-1 formulas 'the s most confident positions', all kept; a finished block is committed to the prefix
    cache and the next one starts.  The same generation with vanilla decoding (one state per pass) beside it."""
    import time
    import torch
    from paper_2509_18085_amd import decode
    cap = cfg.P + n_blocks * cfg.B

    def caches():
        ck, cv = [], []
        for k, v in prefix:
            kk = torch.zeros((cfg.Hkv, cap, cfg.hd), dtype=k.dtype, device=dev)
            vv = torch.zeros_like(kk)
            kk[:, :cfg.P] = k
            vv[:, :cfg.P] = v
            ck.append(kk)
            cv.append(vv)
        return ck, cv

    def run(graph, d_star, replay=False):
        ck, cv = caches()
        dec = decode.BlockDecoder(sp.cfg_from_synth(cfg), layers, ck, cv, cfg.P, w_embed, hw["final_norm"], hw["w_vocab"],
                                  cfg.B, cfg.threshold, logit_scale=LOGIT_SCALE, graph=graph, d_star=d_star, device=dev,
                                  graph_replay=replay)
        block0 = torch.full((cfg.B,), cfg.mask_id, dtype=torch.int32, device=dev)
        dec.decode_block(block0, max_steps=2)                   # warm-up (nothing is committed)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        g = dec.generate(n_blocks)
        torch.cuda.synchronize()
        return g, (time.perf_counter() - t0) * 1e3, dec

    D = cfg.G - 1
    graph = decode.DraftGraph([[(i, 1) for i in range(1, (n % cfg.B) + 2)] for n in range(D)], device=dev)
    g, ms, dec = run(graph, D)
    v, v_ms, _ = run(None, 0)
    vr, vr_ms, vr_dec = run(None, 0, replay=True)      # the same vanilla generation, passes replayed from HIP graphs
    nfe, v_nfe = sum(g["nfe"]), sum(v["nfe"])
    states = sum(sum(x) for x in g["n_states"])
    block = torch.randint(0, cfg.V - 1, (cfg.B,), dtype=torch.int32, device=dev)
    dec.P -= cfg.B                                              # time the commit on the last slot again
    dec.plan.set_prefix_len(dec.P)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    dec.plan.commit_block(block)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(3):
        dec.plan.commit_block(block)
    e1.record()
    torch.cuda.synchronize()
    # the first pass of a block, with the previous block's commit as a pass of its own and folded in
    dec.P -= cfg.B
    dec.plan.set_prefix_len(dec.P)
    one = torch.full((1, cfg.B), cfg.mask_id, dtype=torch.int32, device=dev)

    def separate():
        dec.plan.commit_block(block)
        dec.plan.set_prefix_len(dec.P + cfg.B)
        dec.plan.run(one, None)
        dec.plan.set_prefix_len(dec.P)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / 3

    sep_ms, fused_ms = timed(separate), timed(lambda: dec.plan.run_commit(block, one, None))
    tokens = n_blocks * cfg.B
    return {"blocks": n_blocks, "tokens": tokens, "forward_passes": nfe, "states_verified": states, "ms": ms,
            "ms_per_forward_pass": ms / max(1, nfe), "tokens_per_s": tokens / (ms * 1e-3), "states_per_s": states / (ms * 1e-3),
            "accepted_drafts": int(sum(sum(d) for d in g["depths"])),
            "vanilla": {"forward_passes": v_nfe, "ms": v_ms, "ms_per_forward_pass": v_ms / max(1, v_nfe),
                        "tokens_per_s": tokens / (v_ms * 1e-3)},
            "same_tokens_as_vanilla": bool((g["tokens"] == v["tokens"]).all()),
            "vanilla_passes_from_hip_graphs": {"forward_passes": sum(vr["nfe"]), "graph_launches": vr_dec.graph_launches,
                                               "ms": vr_ms, "tokens_per_s": tokens / (vr_ms * 1e-3),
                                               "same_tokens_as_eager": bool((vr["tokens"] == v["tokens"]).all())},
            "commit_block_ms": e0.elapsed_time(e1) / 3,
            "block_start_ms": {"commit_then_first_pass": sep_ms, "one_fused_pass": fused_ms},
            "note": "each time includes the commits (folded into the next block's first pass, the last one a pass of its own), top-K, drafting, pruning and the host reads of the accept result; "
                    "a block's first pass has one state, later passes one state per formula that the remaining MASK "
                    "positions can still build; random weights: drafts built from the previous distribution are rarely "
                    "accepted, so the ratio of the two times is mostly the cost of verifying up to G-1 drafts per pass; "
                    "acceptance rates are a property of trained weights"}


def dual_cache_leg(sp, cfg, layers, prefix, hw, w_embed, d_states, d_edges, dev, seed, S=224, steps=5):
    """Not part of the timed step: the same step with a dual cache (Sec. 4.3 / App. A.2), S fixed keys /
    values of the tokens after the block in every layer (S = 224: a 256-token generation, first block)."""
    import time
    import torch
    from paper_2509_18085_amd import synth
    cap = cfg.P + cfg.B + S
    pf = []
    for l, (k, v) in enumerate(prefix):
        sk, sv = synth.suffix_kv(cfg, l, S, seed, device=dev)
        kk = torch.zeros((cfg.Hkv, cap, cfg.hd), dtype=k.dtype, device=dev)
        vv = torch.zeros_like(kk)
        kk[:, :cfg.P], vv[:, :cfg.P] = k, v
        kk[:, cfg.P + cfg.B:], vv[:, cfg.P + cfg.B:] = sk, sv
        pf.append(sp.prefix_kv(kk, vv, cfg.P, S))
    plan = sp.StepPlan(sp.cfg_from_synth(cfg), [sp.layer_weights(w) for w in layers], pf, w_embed, hw["final_norm"],
                       hw["w_vocab"], cfg.G, cfg.B, cfg.P, cfg.threshold, logit_scale=LOGIT_SCALE, device=dev)
    for _ in range(2):
        plan.run(d_states, d_edges)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        plan.run(d_states, d_edges)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    return {"suffix_rows": S, "ms_per_step": ms, "states_per_s": cfg.G / (ms * 1e-3)}


def subgraph_leg(sp, dev, seed, n_levels=15, D=10, iters=3):
    """Not part of the timed step: the optimal-subgraph search of the offline calibration (Alg. 2 part 3) on a
    synthetic candidate graph of n_levels x 3 nodes; every C(N, D) node set is tried."""
    import math
    import torch
    from paper_2509_18085_amd import synth
    count, level, edges, _ = synth.candidate_graph(n_levels, seed=seed)
    N = len(count)
    c, l, e = (torch.from_numpy(x).to(dev) for x in (count, level, edges))
    out = sp.subgraph_search(c, l, e, D)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        out = sp.subgraph_search(c, l, e, D, workspace=out["_workspace"])
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    sets = math.comb(N, D)
    # per tried set: one 64-bit add, two 64-bit ANDs, one OR, one zero test, one 64-bit compare = 10 32-bit
    # integer lane operations; peak = 256 CUs x 64 lanes x 2.4 GHz
    ops, peak = 10.0 * sets, 256 * 64 * 2.4e9
    return {"nodes": N, "edges": int(len(edges)), "D": D, "sets_tried": sets, "ms": ms, "sets_per_s": sets / (ms * 1e-3),
            "connected_sets": int(out["n_connected"].item()), "best_sum": int(out["best_sum"].item()),
            "roofline": {"kernel": "sg_search_kernel", "bound": "alu", "achieved": ops / (ms * 1e-3) / 1e12,
                         "peak": peak / 1e12, "unit": "Top/s (int32 lane operations)",
                         "frac": ops / (ms * 1e-3) / peak, "traffic": None}}


def full_sequence_leg(sp, cfg, layers, prefix, hw, w_embed, d_states, d_edges, dev, S=224, steps=5):
    """Not part of the timed step: the step of a full-sequence model that caches only the prefix (Sec. 4.3, Fig. 4):
    the S true tokens after the block are recomputed in the call (S more rows through every layer) and every
    draft attends to their fresh keys / values."""
    import time
    import torch
    cap = cfg.P + cfg.B + S
    pf = []
    for k, v in prefix:
        kk = torch.zeros((cfg.Hkv, cap, cfg.hd), dtype=k.dtype, device=dev)
        vv = torch.zeros_like(kk)
        kk[:, :cfg.P], vv[:, :cfg.P] = k, v
        pf.append(sp.prefix_kv(kk, vv, cfg.P))
    plan = sp.SeqStepPlan(sp.cfg_from_synth(cfg), [sp.layer_weights(w) for w in layers], pf, w_embed, hw["final_norm"],
                          hw["w_vocab"], cfg.G, cfg.B, S, cfg.P, cfg.threshold, logit_scale=LOGIT_SCALE, device=dev)
    suffix = torch.full((S,), cfg.mask_id, dtype=torch.int32, device=dev)
    for _ in range(2):
        plan.run(d_states, suffix, d_edges)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        plan.run(d_states, suffix, d_edges)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    out = {"suffix_rows": S, "rows_per_layer": cfg.G * cfg.B + S, "ms_per_step": ms, "states_per_s": cfg.G / (ms * 1e-3)}

    # what three draft blocks add to a forward pass in this regime (the paper's own operating point, D* = 3): the step
    # with the true block alone against the step with three drafts beside it
    def timed(g):
        st, ed = d_states[:g].contiguous(), None
        for _ in range(2):
            plan.run(st, suffix, ed)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            plan.run(st, suffix, ed)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    ms1, ms4 = timed(1), timed(4)
    out["three_drafts_vs_none"] = {
        "ms_true_block_only": ms1, "ms_with_three_drafts": ms4, "ratio": ms4 / ms1,
        "note": "for context, not the same measurement: the paper's Table 4 has 1.2485 for LLaDA-8B on an A100 with its whole "
                "sequence in the forward pass and attention through a dense mask"}
    del plan, pf

    # a whole generation in this regime: S / B + 1 blocks, the MASK tokens behind the current block recomputed in
    # every pass; vanilla decoding with and without the commit pass standing in for the next block's first pass
    from paper_2509_18085_amd import decode
    n_blocks = S // cfg.B + 1

    def generate(reuse):
        ck, cv = [], []
        for k, v in prefix:
            kk = torch.zeros((cfg.Hkv, cfg.P + n_blocks * cfg.B, cfg.hd), dtype=k.dtype, device=dev)
            vv = torch.zeros_like(kk)
            kk[:, :cfg.P], vv[:, :cfg.P] = k, v
            ck.append(kk)
            cv.append(vv)
        dec = decode.BlockDecoder(sp.cfg_from_synth(cfg), layers, ck, cv, cfg.P, w_embed, hw["final_norm"], hw["w_vocab"],
                                  cfg.B, cfg.threshold, logit_scale=LOGIT_SCALE, device=dev, seq_S0=S,
                                  reuse_commit_pass=reuse)
        dec.decode_block(torch.full((cfg.B,), cfg.mask_id, dtype=torch.int32, device=dev), max_steps=1)   # warm-up
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        g = dec.generate(n_blocks)
        torch.cuda.synchronize()
        return g, (time.perf_counter() - t0) * 1e3

    g0, ms0 = generate(False)
    g1, ms1 = generate(True)
    out["vanilla_generation"] = {
        "blocks": n_blocks, "tokens": n_blocks * cfg.B,
        "first_pass_of_its_own": {"forward_passes": sum(g0["nfe"]) + n_blocks - 1, "ms": ms0},
        "first_pass_from_the_commit_pass": {"forward_passes": sum(g1["nfe"]) + n_blocks - 1, "ms": ms1},
        "tokens_that_differ": int((g0["tokens"] != g1["tokens"]).sum()),
        "note": "forward passes include the commit pass of every block but the last; the two ways compute the same "
                "function with different bf16 rounding, and with random weights (flat logits, confidences next to each "
                "other) near-ties fall either way, so the token sequences part at the first such tie"}
    return out


def stored_traffic(config):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary
    (counters cannot be collected from inside this process); None if there is none for the workload."""
    for name in ("hbm_traffic_%s_gemm_kernels.txt" % config, "hbm_traffic_%s_kernels.txt" % config):
        try:
            for ln in open(os.path.join(ROOT, "profiles", name)):
                if ln.startswith("traffic_bytes_per_launch_swiglu_gemm:"):
                    return float(ln.split(":")[1])
        except OSError:
            pass
    return None


def cpu_baseline(cfg, layers, prefix, hw, states, edges, gpu_out):
    """The oracle as it stands, on this host, on a bounded sample of the same workload: the first
    layers on all G states + the head on all G states + the walk, scaled to the full depth.
    A baseline for context, not a target.  The head runs on the device step's own final hidden states, so its
    decisions are the ones the step had to take: the second result counts how they compare (near-ties, near-threshold
    confidences, excluded states, mismatches; then the same against the plain oracle that does not round the
    normalised row to bf16, at the literal 1e-3 margin)."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import spiffy_oracle as O

    f64 = lambda t: t.detach().cpu().double().numpy()
    n_layers = min(cfg.L, 10)          # about 10 s of host work at the headline configuration
    rng = np.random.default_rng(0)
    x = rng.standard_normal((cfg.G, cfg.B, cfg.d))
    t_layers = 0.0
    for l in range(n_layers):
        w = {k: f64(v) for k, v in layers[l].items()}
        pk, pv = f64(prefix[l][0]), f64(prefix[l][1])
        t0 = time.perf_counter()
        x = O.verify_layer(w, pk, pv, x, n_q_heads=cfg.Hq, n_kv_heads=cfg.Hkv, head_dim=cfg.hd, pos0=cfg.P,
                           rms_eps=cfg.rms_eps, rope_base=cfg.rope_base)
        t_layers += time.perf_counter() - t0
        del w, pk, pv
    wv, fn = f64(hw["w_vocab"]), f64(hw["final_norm"])
    hid = f64(gpu_out["hidden"])
    t0 = time.perf_counter()
    amax, conf, unmask, margin, tgt = O.decode_head(hid, fn, wv, states, cfg.mask_id, cfg.threshold, rms_eps=cfg.rms_eps,
                                                    logit_scale=LOGIT_SCALE, operand_dtype="bf16")
    t_head = time.perf_counter() - t0
    t0 = time.perf_counter()
    O.graph_accept(edges, states, tgt, 0)
    t_walk = time.perf_counter() - t0
    step_s = t_layers * cfg.L / n_layers + t_head + t_walk
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    base = {"value": cfg.G / step_s, "unit": "states/s", "cores": threads, "kind": "oracle",
            "sample": "oracle.verify_layer on all %d states for %d of %d layers (%.2f s), oracle.decode_head on all "
                      "states (%.2f s), oracle.graph_accept (%.4f s); layer time scaled by %d/%d"
                      % (cfg.G, n_layers, cfg.L, t_layers, t_head, t_walk, cfg.L, n_layers),
            "measured_s": t_layers + t_head + t_walk, "extrapolated_step_s": step_s}

    # ---- decisions of the device step against the oracle on the same hidden states
    g = {k: gpu_out[k].cpu().numpy() for k in ("argmax", "conf", "unmask", "target_states")}
    m = states == cfg.mask_id
    tie = 1e-3 * max(1.0, LOGIT_SCALE)
    near_tie = m & (margin < tie)
    near_tau = m & (np.abs(conf.astype(np.float64) - cfg.threshold) < 1e-4 * cfg.threshold)
    ok_state = np.ones(cfg.G, bool)
    for s in range(cfg.G):
        c = np.sort(conf[s][m[s]])[::-1]
        if near_tie[s].any() or near_tau[s].any() or (c.size > 1 and c[0] - c[1] < 1e-5 * c[0]):
            ok_state[s] = False
    clear = m & ~near_tie
    p_amax, p_conf, p_unmask, p_margin, _ = O.decode_head(hid, fn, wv, states, cfg.mask_id, cfg.threshold,
                                                          rms_eps=cfg.rms_eps, logit_scale=LOGIT_SCALE)
    lit = m & (p_margin >= 1e-3)
    far = lit & (np.abs(p_conf.astype(np.float64) - cfg.threshold) >= 2e-2 * cfg.threshold)
    node, depth = O.graph_accept(edges, states, g["target_states"], 0)[:2]
    res = gpu_out["result"].cpu().tolist()
    check = {"masked": int(m.sum()), "logit_scale": LOGIT_SCALE, "tie_margin": tie,
             "near_tie": int(near_tie.sum()), "near_tie_literal_1e_3": int((m & (margin < 1e-3)).sum()),
             "near_threshold": int(near_tau.sum()), "excluded_states": int((~ok_state).sum()),
             "mismatches": {"argmax_outside_near_ties": int((g["argmax"] != amax)[clear].sum()),
                            "unmask_in_compared_states": int((g["unmask"] != unmask)[ok_state].sum()),
                            "next_state_in_compared_states": int((g["target_states"] != tgt)[ok_state].sum()),
                            "conf_max_rel_err": float(np.max(np.abs(g["conf"][m] - conf[m]) / np.maximum(conf[m], 1e-30))),
                            "walk_on_own_next_states": int([res[0], res[1]] != [node, depth])},
             "plain_float64_oracle": {"argmax_mismatch_outside_1e_3": int((g["argmax"] != p_amax)[lit].sum()),
                                      "unmask_mismatch_away_from_tau": int((g["unmask"] != p_unmask)[far].sum()),
                                      "conf_max_rel_err": float(np.max(np.abs(g["conf"][m] - p_conf[m]) / np.maximum(p_conf[m], 1e-30)))},
             "note": "oracle.decode_head on the device step's own final hidden states; first block: operands rounded to "
                     "bf16 as on the matrix cores (the gated comparison of the tests), second: no rounding"}
    return base, check


if __name__ == "__main__":
    main()
