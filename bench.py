#!/usr/bin/env python3
"""Benchmark of the RoM layer forward pass (all hot-path stages, one call of rom_layer_forward per
step) on one MI355X, on seeded synthetic inputs shaped like the paper's 1.3B-active / 16K-context
model (d_model 2048, 8 experts top-1, L = 16384).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2] [--no-cpu-baseline]

Inputs and weights are resident in HBM before the timed region starts.  Per-stage durations come
from HIP events the library records on the launch stream inside the timed region.
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
# plain-ALU ceiling for fp32: 256 CUs x 4 SIMDs x 16 lanes x 2 flop (FMA) x 2.4 GHz, no packed math
PEAK_ALU_FP32_TFLOPS = 78.6
# HBM bytes per in_proj launch at cfg2 from rocprofv3 FETCH_SIZE (x2.0 copy-kernel calibration) +
# WRITE_SIZE (x1.0): see profiles/forward_cfg2_hbm_traffic.md
TRAFFIC_IN_PROJ_CFG2_BYTES = (992 + 256) * 2 ** 20


def stage_model(cfg):
    """Algorithmic work per forward call and per stage: flops for the contractions (routed rows
    only, padding never counts), bytes for the bandwidth stages."""
    N = cfg.batch * cfg.seq_len
    S = N * cfg.top_k
    Dm, De, R, Ds = cfg.d_model, cfg.d_inner, cfg.dt_rank, cfg.d_state
    b = 2 if cfg.dtype == "bf16" else 4
    Sx = S if cfg.routed_xdt else N
    return {
        "route": ("hbm", N * Dm * b),                                   # read x once
        "permute": ("hbm", 5 * S * 4),
        "in_proj": ("mfma", 2.0 * S * Dm * 2 * De),
        "conv": ("hbm", 2 * N * De * b),                                # read x branch, write u
        "x_proj": ("mfma", 2.0 * Sx * De * (R + 2 * Ds)),
        "dt_proj": ("mfma", 2.0 * Sx * R * De),
        # read u, dt, z, write g per (token, channel) + B, C per token
        "scan_gate": ("hbm", 4 * N * De * b + N * 2 * Ds * 4),
        "out_proj": ("mfma", 2.0 * S * De * Dm),
        "combine": ("hbm", (1 + cfg.top_k) * N * Dm * b if cfg.top_k > 1 else 0),
    }


def cpu_baseline(cfg, sample_tokens):
    """The oracle as it stands, timed on this machine's host cores on a prefix of the same workload."""
    import numpy as np
    from dataclasses import replace
    from oracle import rom_oracle as O
    from rom_synth import make_input, make_weights
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    sub = replace(cfg, batch=1, seq_len=min(sample_tokens, cfg.seq_len))
    w = make_weights(sub)
    x = make_input(cfg)[:1, :sub.seq_len]
    t0 = time.perf_counter()
    O.rom_layer_forward(x, w, sub.top_k, sub.gate_mode)
    dt = time.perf_counter() - t0
    return {"value": sub.seq_len / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"first {sub.seq_len} tokens of sequence 0 of {cfg.name}, numpy fp64 oracle, "
                      f"{dt:.1f} s wall"}


def decode_step_rate(n_steps=512):
    """rom_step on the recurrent-decode workload (cfg4): 256 sequences, 512 consecutive steps,
    states carried on the device.  Reported next to the headline number, not part of it."""
    import torch
    from paper_2506_18145_amd import RomLayer
    from rom_synth import get_config, make_states, make_step_inputs, make_weights
    cfg = get_config("cfg4")
    layer = RomLayer(cfg, make_weights(cfg), device="cuda:0")
    cs, ss = make_states(cfg)
    cs, ss = layer.to_device(cs, typed=False), layer.to_device(ss, typed=False)
    xs = layer.to_device(make_step_inputs(cfg, 64))
    out = torch.empty_like(xs[0])
    for i in range(16):
        layer.step(xs[i], cs, ss, out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(n_steps):
        layer.step(xs[i % 64], cs, ss, out)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # algorithmic HBM bytes per step: every expert's weights once + fp32 state read and written
    De, Dm, R, E = cfg.d_inner, cfg.d_model, cfg.dt_rank, cfg.n_experts
    w_bytes = 2 * E * (2 * De * Dm + (R + 32) * De + De * R + Dm * De)
    s_bytes = 2 * 4 * cfg.batch * De * (16 + 3)
    return {"workload": "cfg4: 256 sequences x %d steps, d_model=2048, E=8, top-1, bf16" % n_steps,
            "us_per_step": dt / n_steps * 1e6, "tokens_per_s": cfg.batch * n_steps / dt,
            "bound": "hbm", "achieved_gbs": (w_bytes + s_bytes) / (dt / n_steps) / 1e9,
            "frac": (w_bytes + s_bytes) / (dt / n_steps) / 1e9 / PEAK_HBM_GBS}


def device_weights(cfg, seed):
    """One layer's parameters drawn on the GPU (same shapes and distributions as
    rom_synth.make_weights; a 48-layer stack would take minutes to draw on the host)."""
    import math
    import torch
    g = torch.Generator(device="cuda:0")
    g.manual_seed(seed)
    E, Ex = cfg.n_experts, cfg.n_experts_xdt
    Dm, De, Ds, k, R = cfg.d_model, cfg.d_inner, cfg.d_state, cfg.d_conv, cfg.dt_rank
    t = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32

    def normal(shape, std):
        return (torch.randn(shape, generator=g, device="cuda:0", dtype=torch.float32) * std).to(t)

    def uniform(shape, lo, hi):
        return torch.rand(shape, generator=g, device="cuda:0", dtype=torch.float32) * (hi - lo) + lo

    lim = 1.0 / math.sqrt(k)
    tau = torch.exp(uniform((De,), math.log(1e-3), math.log(1e-1)))
    return {
        "w_router": normal((E, Dm), 0.02), "b_router": None,
        "w_in": normal((E, 2 * De, Dm), cfg.weight_std),
        "conv_w": uniform((De, k), -lim, lim), "conv_b": uniform((De,), -lim, lim),
        "w_x": normal((Ex, R + 2 * Ds, De), cfg.weight_std), "w_dt": normal((Ex, De, R), cfg.weight_std),
        "dt_bias": tau + torch.log(-torch.expm1(-tau)),
        "A_log": torch.log(torch.arange(1, Ds + 1, device="cuda:0", dtype=torch.float32)).repeat(De, 1),
        "D": torch.ones(De, device="cuda:0"), "w_out": normal((E, Dm, De), cfg.weight_std),
        "norm_w": torch.ones(Dm, device="cuda:0"),
    }


def stack_rate(cfg, n_layers, steps, warmup):
    """n_layers pre-norm residual blocks of the workload's shape (the paper's 1.3B-active model is 48
    layers of d_model 2048), one rom_stack_forward call per step; embedding and output head are
    not part of it.  Every layer has its own weights, so nothing is served from a cache."""
    import torch
    from paper_2506_18145_amd import RomLayer, RomStack
    from rom_synth import make_input
    layers = [RomLayer(cfg, device_weights(cfg, 7000 + j), device="cuda:0") for j in range(n_layers)]
    stack = RomStack(layers, eps=1e-5, fold_in_place=True)
    x = layers[0].to_device(make_input(cfg))
    out = torch.empty_like(x)
    for _ in range(warmup):
        stack.forward(x, out=out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        stack.forward(x, out=out)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    finite = bool(torch.isfinite(out.float()).all().item())
    n_tok = cfg.batch * cfg.seq_len
    w_bytes = sum(v.numel() * v.element_size() for ly in layers for v in ly.weights.values() if v is not None)
    return {"workload": f"{n_layers} blocks (RMSNorm + RoM layer + skip) of {cfg.name}'s shape, one sequence of "
                        f"{cfg.seq_len} tokens", "n_layers": n_layers, "ms_per_forward": dt * 1e3,
            "ms_per_layer": dt * 1e3 / n_layers, "tokens_per_s": n_tok / dt, "weights_gib": w_bytes / 2 ** 30,
            "output_finite": finite}


def ffn_moe_rate(cfg, d_ff, steps, warmup):
    """The FFN-MoE layer that follows a RoM layer and reuses its routing decision (appendix Eq. (14),
    (15)): pre-norm, SwiGLU experts of width d_ff, skip; on the grouping rom_route leaves behind."""
    import torch
    from paper_2506_18145_amd import RomFfnMoe, RomLayer
    from rom_synth import make_input, make_weights
    g = torch.Generator(device="cuda:0")
    g.manual_seed(4242)
    t = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    E, Dm = cfg.n_experts, cfg.d_model
    normal = lambda shape: (torch.randn(shape, generator=g, device="cuda:0") * cfg.weight_std).to(t)
    layer = RomLayer(cfg, make_weights(cfg), device="cuda:0")
    ffn = RomFfnMoe(layer, d_ff, {"w_gate_up": normal((E, 2 * d_ff, Dm)), "w_down": normal((E, Dm, d_ff)),
                                  "norm_w": torch.ones(Dm, device="cuda:0")})
    x = layer.to_device(make_input(cfg)).view(-1, Dm)
    routing = layer.route(x)
    out = torch.empty_like(x)
    for _ in range(warmup):
        ffn.forward(x, routing, pre_norm=True, add_skip=True, out=out)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        ffn.forward(x, routing, pre_norm=True, add_skip=True, out=out)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    n_tok = x.shape[0]
    flops = 6.0 * n_tok * cfg.top_k * Dm * d_ff
    return {"workload": f"{cfg.name}'s tokens and routing, SwiGLU experts d_ff={d_ff}, pre-norm + skip",
            "ms_per_call": ms, "tokens_per_s": n_tok / (ms * 1e-3), "bound": "mfma",
            "achieved_tflops": flops / (ms * 1e-3) / 1e12, "frac": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}


def hybrid_stack_rate(cfg, n_layers, d_ff, steps, warmup):
    """n_layers RoM blocks, each followed by an FFN-MoE block on its routing decision (the appendix's
    RoM + FFN-MoE hybrid without its attention layers), one rom_hybrid_stack_forward call per step."""
    import torch
    from paper_2506_18145_amd import RomFfnMoe, RomHybridStack, RomLayer
    from rom_synth import make_input
    g = torch.Generator(device="cuda:0")
    g.manual_seed(99)
    t = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    E, Dm = cfg.n_experts, cfg.d_model
    normal = lambda shape: (torch.randn(shape, generator=g, device="cuda:0") * cfg.weight_std).to(t)
    layers = [RomLayer(cfg, device_weights(cfg, 8000 + j), device="cuda:0") for j in range(n_layers)]
    ffns = []
    for ly in layers:
        f = RomFfnMoe(ly, d_ff, {"w_gate_up": normal((E, 2 * d_ff, Dm)), "w_down": normal((E, Dm, d_ff)),
                                 "norm_w": torch.ones(Dm, device="cuda:0")})
        f.packed(True, drop_plain=True)
        ffns.append(f)
    stack = RomHybridStack(layers, ffns, eps=1e-5, ffn_pre_norm=True, fold_in_place=True)
    x = layers[0].to_device(make_input(cfg))
    for _ in range(warmup):
        out = stack.forward(x)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        out = stack.forward(x)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    return {"workload": f"{n_layers} x (RoM block + FFN-MoE block, d_ff={d_ff}) of {cfg.name}'s shape, one sequence of "
                        f"{cfg.seq_len} tokens", "ms_per_forward": dt * 1e3, "ms_per_pair": dt * 1e3 / n_layers,
            "tokens_per_s": cfg.batch * cfg.seq_len / dt, "output_finite": bool(torch.isfinite(out.float()).all().item())}


def time_forward(cfg, steps, warmup, calibrate_copy=False):
    """K timed calls of rom_layer_forward on resident inputs.  Returns (ms per call, ms per call
    without the stage events, per-stage dict)."""
    import torch
    from paper_2506_18145_amd import RomLayer, rom_layer_forward, rom_profile_collect, rom_profile_enable
    from rom_synth import make_input, make_weights

    layer = RomLayer(cfg, make_weights(cfg), device="cuda:0")
    x = layer.to_device(make_input(cfg))
    B, L = cfg.batch, cfg.seq_len
    out = torch.empty_like(x)
    ws = layer.workspace(B, L)

    def step():
        rom_layer_forward(layer.dims, layer.weights, x, B, L, None, None, out, None, None, ws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()

    # timed region: K calls, stage events recorded by the library on the same stream
    rom_profile_enable(steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    stage_ms, n_calls = rom_profile_collect()
    rom_profile_enable(0)

    # the same K calls without the event records, for the record-keeping overhead
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed_plain = time.perf_counter() - t1

    # load-balance statistics (Eq. (16)) from the logits and counts the last call left behind
    lg, ct = layer.ws_view("logits", B, L), layer.ws_view("counts", B, L)
    from paper_2506_18145_amd import rom_balance_stats
    stats = layer.balance_stats(lg, ct, 1e-3)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(50):
        rom_balance_stats(layer.dims, lg, ct, B * L, 1e-3, stats[0], stats[1], stats[2], ws)
    e1.record()
    torch.cuda.synchronize()
    counts = ct.cpu().tolist()
    balance = {"us_per_call": e0.elapsed_time(e1) * 1e3 / 50, "loss_term_alpha_1e-3": float(stats[2].cpu()[0]),
               "max_over_mean_count": max(counts) / (sum(counts) / len(counts))}

    if calibrate_copy:
        src = torch.ones(1 << 29, dtype=torch.bfloat16, device="cuda:0")     # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    n_tok = B * L
    stages = {}
    for name, (bound, work) in stage_model(cfg).items():
        avg_ms = stage_ms[name] / max(n_calls, 1)
        if avg_ms <= 0 or work == 0:
            stages[name] = {"ms": avg_ms}
            continue
        if bound == "mfma":
            ach = work / (avg_ms * 1e-3) / 1e12
            stages[name] = {"ms": avg_ms, "bound": "mfma", "achieved_tflops": ach,
                            "frac": ach / PEAK_BF16_TFLOPS}
        else:
            ach = work / (avg_ms * 1e-3) / 1e9
            stages[name] = {"ms": avg_ms, "bound": "hbm", "achieved_gbs": ach, "frac": ach / PEAK_HBM_GBS}
    # the scan is bound by plain ALU issue, not by HBM: also report it against the fp32 vector peak
    # (7 flops per (token, channel, state): dt*A, exp, dt*u*B, fma (2), C*h, one add of the reduction)
    if stages["scan_gate"].get("ms", 0) > 0:
        fl = 7.0 * n_tok * cfg.d_inner * cfg.d_state
        ach = fl / (stages["scan_gate"]["ms"] * 1e-3) / 1e12
        stages["scan_gate"].update({"alu_tflops": ach, "alu_frac": ach / PEAK_ALU_FP32_TFLOPS})
    return elapsed * 1e3 / steps, elapsed_plain * 1e3 / steps, stages, balance


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg2", choices=["cfg1", "cfg2", "cfg3"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=16384)
    ap.add_argument("--no-step", action="store_true",
                    help="skip the extra rom_step measurement (256 sequences x 512 steps, cfg4)")
    ap.add_argument("--no-shared-xdt", action="store_true",
                    help="skip the extra measurement of the shared x/dt variant of the workload")
    ap.add_argument("--no-ffn", action="store_true", help="skip the extra FFN-MoE layer measurement")
    ap.add_argument("--stack-layers", type=int, default=48,
                    help="layers of the extra whole-stack measurement (0 = skip it)")
    ap.add_argument("--hybrid-layers", type=int, default=0,
                    help="also time a stack of this many (RoM block + FFN-MoE block) pairs (0 = skip)")
    ap.add_argument("--only-step", action="store_true",
                    help="run only the rom_step measurement and print its JSON object (for profiling)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 1 GiB device copies (a kernel of known traffic, for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.only_step:
        print(json.dumps({"decode_step": decode_step_rate()}))
        return

    from dataclasses import replace
    from rom_synth import get_config

    cfg = get_config(args.workload)
    B, L = cfg.batch, cfg.seq_len
    n_tok = B * L
    ms_per_step, ms_plain, stages, balance = time_forward(cfg, args.steps, args.warmup, args.calibrate_copy)
    dom = stages["in_proj"]
    roofline = {"kernel": "in_proj grouped GEMM (gemm_bf16_dma_kernel<256, 4, 2, 0>)", "bound": "mfma",
                "achieved": dom.get("achieved_tflops"), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": dom.get("frac"),
                "traffic": TRAFFIC_IN_PROJ_CFG2_BYTES if cfg.name == "cfg2" else None}

    result = {
        "metric": "RoM layer fwd tokens/s at d=2048,L=16K; % MFMA peak (GEMM), % HBM BW (scan)",
        "value": n_tok / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_without_stage_events": ms_plain,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: RoM layer forward, B={B}, L={L}, d_model={cfg.d_model}, "
                               f"d_inner={cfg.d_inner}, d_state={cfg.d_state}, dt_rank={cfg.dt_rank}, "
                               f"E={cfg.n_experts}, top_k={cfg.top_k}, routed x/dt, bf16",
                   "tokens_per_step": n_tok},
        "roofline": roofline,
        "stages": stages,
    }
    result["balance_stats"] = balance

    def extra(name, fn):
        """A leg beside the headline measurement: its failure must not cost the headline line."""
        try:
            result[name] = fn()
        except Exception as exc:                      # reported, not hidden: the leg's object says what failed
            result[name] = {"error": f"{type(exc).__name__}: {exc}"}

    if not args.no_shared_xdt:
        # the paper's default variant (Sec. 4.3, design choices): x and dt projections shared by all experts, so
        # those two stages are plain GEMMs; same shapes and inputs otherwise
        def shared_leg():
            shared = replace(cfg, name=cfg.name + "-shared-xdt", routed_xdt=False)
            ms_s, _, stages_s, _ = time_forward(shared, max(args.steps // 2, 1), args.warmup)
            return {"workload": f"{cfg.name} with one shared x/dt projection (E_x = 1)", "ms_per_step": ms_s,
                    "tokens_per_s": n_tok / (ms_s * 1e-3), "stages_ms": {k: v["ms"] for k, v in stages_s.items()}}
        extra("shared_xdt_variant", shared_leg)
    if not args.no_ffn:
        extra("ffn_moe", lambda: ffn_moe_rate(cfg, 2 * cfg.d_model, 20, 20))
    if args.hybrid_layers > 0:
        extra("hybrid_stack_forward", lambda: hybrid_stack_rate(cfg, args.hybrid_layers, 2 * cfg.d_model, 3, 1))
    if args.stack_layers > 0:
        extra("stack_forward", lambda: stack_rate(cfg, args.stack_layers, 3, 1))
    if not args.no_step:
        extra("decode_step", decode_step_rate)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, args.cpu_sample_tokens)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
