#!/usr/bin/env python3
"""Benchmark of the RoM layer forward pass (all hot-path stages, one call of rom_layer_forward per
step) on one MI355X, on seeded synthetic inputs shaped like the paper's 1.3B-active / 16K-context
model (d_model 2048, 8 experts top-1, L = 16384).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2] [--no-cpu-baseline]

Inputs and weights are resident in HBM before the timed region starts.  The timed calls carry HIP
events around the dominant kernel (the in projection) only; the per-stage breakdown comes from a
second pass with an event at every stage boundary.  Beside the headline: HBM traffic of the
dominant kernel from two rocprofv3 counter runs of this script, forward timings of the two other
layer configurations, the load-balance statistics, the shared x/dt variant, forward + backward of
the layer, RoM on a Mamba2 and on a Gated DeltaNet layer of the same width, a 48-block stack, the FFN-MoE layer, the
recurrent step and the CPU oracle's rate
(--help lists the switches that skip them; --probe prints issue-rate measurements instead).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA (published, at the nominal 2.4 GHz)
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E (published)
# fp32 vector peak: 256 CUs x 4 SIMDs x 32 lanes per clock x 2 flop (FMA) x 2.4 GHz = 157.3 TFLOP/s, the
# published figure.  It needs no packed math: a SIMD issues one 64-lane fp32 FMA every two clocks
# (measured here: 2.3 clocks per wavefront instruction with four or more wavefronts per SIMD; a
# lone wavefront gets one every 5 clocks, a DPP instruction costs 4.2, v_exp_f32 8.2).
PEAK_ALU_FP32_TFLOPS = 157.3
ALU_PEAK_NOTE = ("fp32 vector peak 157.3 TFLOP/s = 256 CU x 4 SIMD x 32 lanes/clk x 2 flop x 2.4 GHz (published; "
                 "reached without packed-fp32 instructions, which this build never emits)")
NOMINAL_CLOCK_GHZ = 2.4
# shader clock under the in projection's load, from GRBM_GUI_ACTIVE of that kernel over its duration
# (profiles/forward_cfg2_hbm_traffic.md: 1.06e6 cycles per XCD in 0.543 ms): the published peaks
# assume 2.4 GHz, the chip sustains less under a bf16 GEMM of N(0,1)-like operands
COUNTER_CLOCK_GHZ_GEMM = 1.95
DOMINANT_KERNEL = "gemm_bf16_dma_kernel<256, 4, 2, 0, false>"     # the in projection at top-1
DOMINANT_STAGE = "in_proj"


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
    # backward of the same layer (forward recomputation with the pre-activations kept, then the adjoint)
    d_out = torch.randn(x.shape, generator=g, device="cuda:0").to(t)
    for _ in range(3):
        ffn.backward(x, routing, d_out, pre_norm=True, add_skip=True)
    e0.record()
    n_bwd = max(3, steps // 4)
    for _ in range(n_bwd):
        d_x, _, _ = ffn.backward(x, routing, d_out, pre_norm=True, add_skip=True)
    e1.record()
    torch.cuda.synchronize()
    ms_bwd = e0.elapsed_time(e1) / n_bwd
    # one training step of the hybrid pair of the appendix: RoM block forward, FFN-MoE block forward on its
    # routing decision, then the two backward calls (the FFN's gate gradient handed to the block)
    B, L = cfg.batch, cfg.seq_len
    x3 = x.view(B, L, Dm)
    names = ("offsets", "perm", "inv_perm", "gate")

    def pair_step():
        mid = layer.block_forward_train(x3, eps=1e-5)
        r = {k: layer.train_routing_view(k, B, L) for k in names}
        ffn.forward_train(mid.view(-1, Dm), r, pre_norm=True, add_skip=True, out=out)
        d_mid, d_gate_ffn, _ = ffn.backward(mid.view(-1, Dm), r, d_out, pre_norm=True, add_skip=True, saved=True)
        return layer.block_backward(x3, d_mid.view(B, L, Dm), eps=1e-5, d_gate_ffn=d_gate_ffn, saved=True)[0]

    for _ in range(2):
        pair_step()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(n_bwd):
        d_xp = pair_step()
    e1.record()
    torch.cuda.synchronize()
    ms_pair = e0.elapsed_time(e1) / n_bwd
    return {"workload": f"{cfg.name}'s tokens and routing, SwiGLU experts d_ff={d_ff}, pre-norm + skip",
            "hybrid_pair_training_step": {
                "workload": "rom_block_forward_train + rom_ffn_moe_forward_train + rom_ffn_moe_backward_saved + "
                            "rom_block_backward_saved (activations kept between forward and backward), no optimizer",
                "ms_per_step": ms_pair, "tokens_per_s": n_tok / (ms_pair * 1e-3),
                "gradients_finite": bool(torch.isfinite(d_xp.float()).all().item())},
            "ms_per_call": ms, "tokens_per_s": n_tok / (ms * 1e-3), "bound": "mfma",
            "achieved_tflops": flops / (ms * 1e-3) / 1e12, "frac": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "backward": {"workload": "rom_ffn_moe_backward: forward recomputation + gradients w.r.t. x, the gate weights, "
                                     "the norm scale and both expert weights",
                         "ms_per_call": ms_bwd, "tokens_per_s": n_tok / (ms_bwd * 1e-3),
                         "gemm_tflops": 3.0 * flops / (ms_bwd * 1e-3) / 1e12,     # recomputed forward + four adjoint GEMMs = 3 x forward
                         "gradients_finite": bool(torch.isfinite(d_x.float()).all().item())}}


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


def _median(v):
    v = sorted(v)
    n = len(v)
    return 0.0 if n == 0 else (v[n // 2] if n % 2 else 0.5 * (v[n // 2 - 1] + v[n // 2]))


def time_forward(cfg, steps, warmup, with_balance=True):
    """K timed calls of rom_layer_forward on resident inputs, bracketed by synchronize.  Every call
    sits between two events on the launch stream, and the library records events around the dominant
    stage (the in projection) alone: an event between two kernels costs several microseconds of
    launch overlap, and nine of them per call made the timed calls 5 % slower than undisturbed ones.
    The per-stage breakdown comes from a second pass of K calls with an event at every stage
    boundary; a third pass runs the same K calls with no library events at all.  Returns a dict:
    median and mean milliseconds per call, the wall-clock means of the three passes, and per-stage
    medians with achieved rates (the dominant stage's from the timed region)."""
    import torch
    from paper_2506_18145_amd import (STAGE_NAMES, RomLayer, rom_layer_forward, rom_profile_collect_calls,
                                      rom_profile_enable, rom_profile_select)
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

    # timed region: K calls; events on the launch stream (torch's current stream is the one the
    # binding hands to the library) around every call and, inside the library, around the in projection
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    rom_profile_select(1 << STAGE_NAMES.index(DOMINANT_STAGE))
    rom_profile_enable(steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    evs[0].record()
    for i in range(steps):
        step()
        evs[i + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    per_call = [evs[i].elapsed_time(evs[i + 1]) for i in range(steps)]
    dominant_calls = rom_profile_collect_calls(steps)

    # second pass: the same K calls with an event at every stage boundary, for the breakdown
    rom_profile_select(0xFFFFFFFF)
    rom_profile_enable(steps)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed_all_events = time.perf_counter() - t2
    calls = rom_profile_collect_calls(steps)
    rom_profile_enable(0)
    for c, d in zip(calls, dominant_calls):
        c[DOMINANT_STAGE] = d[DOMINANT_STAGE]         # the dominant stage as it ran in the timed region

    # third pass: no library events at all
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed_plain = time.perf_counter() - t1

    res = {"ms_median": _median(per_call), "ms_mean_wall": elapsed * 1e3 / steps,
           "ms_mean_wall_without_stage_events": elapsed_plain * 1e3 / steps,
           "ms_mean_wall_all_stage_events": elapsed_all_events * 1e3 / steps, "ms_min": min(per_call),
           "ms_max": max(per_call)}

    if with_balance:
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
        res["balance"] = {"us_per_call": e0.elapsed_time(e1) * 1e3 / 50, "loss_term_alpha_1e-3": float(stats[2].cpu()[0]),
                          "max_over_mean_count": max(counts) / (sum(counts) / len(counts)),
                          "counts": counts}

    n_tok = B * L
    stages = {}
    for name, (bound, work) in stage_model(cfg).items():
        ms = _median([c[name] for c in calls]) if calls else 0.0
        if ms <= 0 or work == 0:
            stages[name] = {"ms": ms}
            continue
        if bound == "mfma":
            ach = work / (ms * 1e-3) / 1e12
            stages[name] = {"ms": ms, "bound": "mfma", "achieved_tflops": ach, "frac": ach / PEAK_BF16_TFLOPS}
        else:
            ach = work / (ms * 1e-3) / 1e9
            stages[name] = {"ms": ms, "bound": "hbm", "achieved_gbs": ach, "frac": ach / PEAK_HBM_GBS}
    # the scan is bound by plain ALU issue, not by HBM: also report it against the fp32 vector peak
    # (7 flops per (token, channel, state): dt*A, exp, dt*u*B, fma (2), C*h, one add of the reduction)
    if stages["scan_gate"].get("ms", 0) > 0:
        fl = 7.0 * n_tok * cfg.d_inner * cfg.d_state
        ach = fl / (stages["scan_gate"]["ms"] * 1e-3) / 1e12
        stages["scan_gate"].update({"alu_tflops": ach, "alu_frac": ach / PEAK_ALU_FP32_TFLOPS,
                                    "alu_peak_tflops": PEAK_ALU_FP32_TFLOPS})
    # the two narrow projections move far more bytes than their flops can hide: the x projection reads all
    # of u for 160 output columns, the dt projection writes all of dt from 128 input columns.  Next to their
    # MFMA fraction, their algorithmic HBM bytes against the HBM peak.
    b = 2 if cfg.dtype == "bf16" else 4
    Sx = n_tok * cfg.top_k if cfg.routed_xdt else n_tok
    narrow = {"x_proj": Sx * cfg.d_inner * b + Sx * (cfg.dt_rank + 2 * cfg.d_state) * 4,
              "dt_proj": Sx * cfg.dt_rank * b + n_tok * cfg.d_inner * b}
    for name, nbytes in narrow.items():
        if stages[name].get("ms", 0) > 0:
            gbs = nbytes / (stages[name]["ms"] * 1e-3) / 1e9
            stages[name].update({"hbm_gbs": gbs, "hbm_frac": gbs / PEAK_HBM_GBS})
    res["stages"] = stages
    return res


def backward_rate(cfg, steps, warmup):
    """rom_layer_backward on the workload (activation recomputation: the call runs the forward pass
    into its workspace, then the backward pass)."""
    import numpy as np
    import torch
    from paper_2506_18145_amd import RomLayer
    from rom_synth import make_input, make_weights
    layer = RomLayer(cfg, make_weights(cfg), device="cuda:0")
    x = layer.to_device(make_input(cfg))
    g = torch.Generator(device="cuda:0")
    g.manual_seed(77)
    d_out = torch.randn(x.shape, generator=g, device="cuda:0").to(x.dtype)
    for _ in range(warmup):
        layer.backward(x, d_out)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    evs[0].record()
    for i in range(steps):
        d_x, grads = layer.backward(x, d_out)
        evs[i + 1].record()
    torch.cuda.synchronize()
    ms = _median([evs[i].elapsed_time(evs[i + 1]) for i in range(steps)])
    # a training step: the caller's own forward pass on the backward workspace, then the backward
    # pass on the activations it left (rom_layer_backward_saved: no recomputation)
    torch.cuda.synchronize()
    evs[0].record()
    for i in range(steps):
        layer.forward_for_backward(x)
        d_x, grads = layer.backward(x, d_out, saved=True)
        evs[i + 1].record()
    torch.cuda.synchronize()
    ms_step = _median([evs[i].elapsed_time(evs[i + 1]) for i in range(steps)])
    # the pre-norm residual block's backward (materialised norm, layer forward + backward on it, norm adjoint + skip)
    for _ in range(2):
        layer.block_backward(x, d_out)
    torch.cuda.synchronize()
    evs[0].record()
    for i in range(steps):
        d_xb, _ = layer.block_backward(x, d_out)
        evs[i + 1].record()
    torch.cuda.synchronize()
    ms_block = _median([evs[i].elapsed_time(evs[i + 1]) for i in range(steps)])
    n_tok = cfg.batch * cfg.seq_len
    S = n_tok * cfg.top_k
    Sx = S if cfg.routed_xdt else n_tok
    gemm = 2.0 * S * cfg.d_model * 2 * cfg.d_inner + 2.0 * Sx * cfg.d_inner * (cfg.dt_rank + 2 * cfg.d_state) \
        + 2.0 * Sx * cfg.dt_rank * cfg.d_inner + 2.0 * S * cfg.d_inner * cfg.d_model
    finite = bool(torch.isfinite(d_x.float()).all().item()) and all(bool(torch.isfinite(v).all().item()) for v in grads.values())
    return {"workload": f"{cfg.name}: rom_layer_backward (forward recomputation + backward of one layer), gradients "
                        "w.r.t. x and all parameters; training_step = rom_layer_forward + rom_layer_backward_saved",
            "ms_per_call": ms, "tokens_per_s": n_tok / (ms * 1e-3),
            "ms_per_training_step": ms_step, "training_tokens_per_s": n_tok / (ms_step * 1e-3),
            "ms_per_block_backward_call": ms_block,
            "gemm_tflops_forward_plus_backward": 3.0 * gemm / (ms * 1e-3) / 1e12, "gradients_finite": finite}


def mamba2_rate(steps, warmup):
    """RoM on a Mamba2 layer (Sec. 5.2, Table 3) at the headline layer's size: rom_mamba2_forward on
    B=1, L=16384, d_model 2048, 64 heads of 64 channels, state size 128, 8 experts top-1."""
    import torch
    from paper_2506_18145_amd import (RomMamba2Layer, rom_profile_collect_calls, rom_profile_enable,
                                      rom_profile_select, STAGE_NAMES)
    from rom_synth import get_mamba2_config, make_mamba2_input, make_mamba2_weights
    cfg = get_mamba2_config("m2_cfg2")
    layer = RomMamba2Layer(cfg, make_mamba2_weights(cfg), device="cuda:0")
    x = layer.to_device(make_mamba2_input(cfg))
    for _ in range(warmup):
        layer.forward(x)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    evs[0].record()
    for i in range(steps):
        layer.forward(x)
        evs[i + 1].record()
    torch.cuda.synchronize()
    ms = _median([evs[i].elapsed_time(evs[i + 1]) for i in range(steps)])
    # a second pass with an event at every stage boundary
    rom_profile_select(0xFFFFFFFF)
    rom_profile_enable(steps)
    for _ in range(steps):
        layer.forward(x)
    torch.cuda.synchronize()
    per_call = rom_profile_collect_calls(steps)
    rom_profile_enable(0)
    names = {"dt_proj": "rms_norm", "scan_gate": "ssd_scan_gate"}
    stages = {}
    for nm in STAGE_NAMES:
        vals = [c[nm] for c in per_call if c[nm] > 0]
        if vals:
            stages[names.get(nm, nm)] = _median(vals)
    n_tok = cfg.n_tokens
    S = n_tok * cfg.top_k
    gemm = 2.0 * S * cfg.d_model * cfg.d_in_proj + 2.0 * S * cfg.d_inner * cfg.d_model
    # the recurrence per chunk of 64 steps and head: scores, scores x inputs, C x state, state update
    ssd = n_tok / 64.0 * cfg.n_heads * 2.0 * (64 * 64 * cfg.d_state + 64 * 64 * 64 + 2 * 64 * cfg.d_state * 64)
    out = {"workload": f"{cfg.name}: RoM on Mamba2, B={cfg.batch}, L={cfg.seq_len}, d_model={cfg.d_model}, "
                       f"d_inner={cfg.d_inner}, headdim={cfg.headdim}, d_state={cfg.d_state}, E={cfg.n_experts}, "
                       f"top_k={cfg.top_k}, bf16",
           "ms_per_call": ms, "tokens_per_s": n_tok / (ms * 1e-3), "stages_ms": stages,
           "gemm_tflops": gemm / (ms * 1e-3) / 1e12}
    # the recurrent form: one new token for each of 256 sequences, states updated in place
    n_seq = 256
    xs = layer.to_device(make_mamba2_input(cfg)[0, :n_seq].copy())
    cs_shape, ss_shape = layer.state_shapes(n_seq)
    cs = torch.zeros(cs_shape, device="cuda:0")
    ss = torch.zeros(ss_shape, device="cuda:0")
    out_step = torch.empty_like(xs)
    for _ in range(10):
        layer.step(xs, cs, ss, out=out_step)
    torch.cuda.synchronize()
    n_steps = 50
    evs[0].record()
    for _ in range(n_steps):
        layer.step(xs, cs, ss, out=out_step)
    evs[1].record()
    torch.cuda.synchronize()
    ms_step = evs[0].elapsed_time(evs[1]) / n_steps
    w_bytes = 2.0 * cfg.n_experts * (cfg.d_in_proj * cfg.d_model + cfg.d_model * cfg.d_inner)
    s_bytes = 2.0 * 4.0 * n_seq * cfg.n_heads * cfg.d_state * cfg.headdim
    out["decode_step"] = {"workload": f"rom_mamba2_step, {n_seq} sequences", "ms_per_step": ms_step,
                          "tokens_per_s": n_seq / (ms_step * 1e-3), "bound": "hbm",
                          "algorithmic_gbytes_per_s": (w_bytes + s_bytes) / (ms_step * 1e-3) / 1e9,
                          "frac": (w_bytes + s_bytes) / (ms_step * 1e-3) / 1e9 / PEAK_HBM_GBS}
    if "in_proj" in stages:
        out["in_proj_frac_of_mfma_peak"] = 2.0 * S * cfg.d_model * cfg.d_in_proj / (stages["in_proj"] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS
    if "ssd_scan_gate" in stages:
        t = stages["ssd_scan_gate"] * 1e-3
        # algorithmic bytes of the recurrence: x, B, C, dt, z read once, the gated output written once
        byt = n_tok * 2.0 * (cfg.d_inner * 3 + 2 * cfg.d_state + cfg.n_heads)
        out["ssd_scan"] = {"ms": stages["ssd_scan_gate"], "tflops": ssd / t / 1e12, "gbytes_per_s": byt / t / 1e9,
                           "frac_of_hbm_peak": byt / t / 1e9 / PEAK_HBM_GBS}
    return out


def gdn_rate(steps, warmup):
    """RoM on a Gated DeltaNet layer (Sec. 5.2, Table 3): rom_gdn_forward on d_model 2048, 32 heads of
    64 key and 64 value channels, 8 experts top-1 - the 16K-token sequence, and the same number of
    tokens as 8 sequences of 2048 (the recurrence is parallel over sequences x heads only)."""
    import torch
    from dataclasses import replace as dc_replace
    from paper_2506_18145_amd import (RomGdnLayer, rom_profile_collect_calls, rom_profile_enable, rom_profile_select,
                                      STAGE_NAMES)
    from rom_synth import get_gdn_config, make_gdn_input, make_gdn_weights
    out = {}
    for label, cfg in (("one_sequence", get_gdn_config("gdn_cfg2")),
                       ("eight_sequences", dc_replace(get_gdn_config("gdn_cfg2"), batch=8, seq_len=2048))):
        layer = RomGdnLayer(cfg, make_gdn_weights(cfg), device="cuda:0")
        x = layer.to_device(make_gdn_input(cfg))
        for _ in range(warmup):
            layer.forward(x)
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        torch.cuda.synchronize()
        evs[0].record()
        for i in range(steps):
            layer.forward(x)
            evs[i + 1].record()
        torch.cuda.synchronize()
        ms = _median([evs[i].elapsed_time(evs[i + 1]) for i in range(steps)])
        rom_profile_select(0xFFFFFFFF)
        rom_profile_enable(steps)
        for _ in range(steps):
            layer.forward(x)
        torch.cuda.synchronize()
        per_call = rom_profile_collect_calls(steps)
        rom_profile_enable(0)
        stages = {}
        for nm in STAGE_NAMES:
            vals = [c[nm] for c in per_call if c[nm] > 0]
            if vals:
                stages["delta_rule_norm_gate" if nm == "scan_gate" else nm] = _median(vals)
        out[label] = {"workload": f"{cfg.name}: B={cfg.batch}, L={cfg.seq_len}, d_model={cfg.d_model}, heads={cfg.n_heads}, "
                                  f"d_k={cfg.d_k}, d_v={cfg.d_v}, E={cfg.n_experts}, top_k={cfg.top_k}, bf16",
                      "ms_per_call": ms, "tokens_per_s": cfg.n_tokens / (ms * 1e-3), "stages_ms": stages}
        if label == "eight_sequences":
            # the recurrent form: one new token for each of 256 sequences, states updated in place
            n_seq = 256
            xs = layer.to_device(make_gdn_input(cfg)[0, :n_seq].copy())
            cs_shape, ss_shape = layer.state_shapes(n_seq)
            cs = torch.zeros(cs_shape, device="cuda:0")
            ss = torch.zeros(ss_shape, device="cuda:0")
            out_step = torch.empty_like(xs)
            for _ in range(10):
                layer.step(xs, cs, ss, out=out_step)
            torch.cuda.synchronize()
            evs[0].record()
            for _ in range(50):
                layer.step(xs, cs, ss, out=out_step)
            evs[1].record()
            torch.cuda.synchronize()
            ms_step = evs[0].elapsed_time(evs[1]) / 50
            w_bytes = 2.0 * cfg.n_experts * (cfg.d_in_proj * cfg.d_model + cfg.d_model * cfg.d_vt)
            s_bytes = 2.0 * 4.0 * n_seq * cfg.n_heads * cfg.d_k * cfg.d_v
            out["decode_step"] = {"workload": f"rom_gdn_step, {n_seq} sequences", "ms_per_step": ms_step,
                                  "tokens_per_s": n_seq / (ms_step * 1e-3), "bound": "hbm",
                                  "algorithmic_gbytes_per_s": (w_bytes + s_bytes) / (ms_step * 1e-3) / 1e9,
                                  "frac": (w_bytes + s_bytes) / (ms_step * 1e-3) / 1e9 / PEAK_HBM_GBS}
        del layer, x
    return out


def config_leg(name, steps, warmup):
    """The same measurement on another of the paper-shaped workloads (beside the headline one)."""
    from rom_synth import get_config
    cfg = get_config(name)
    r = time_forward(cfg, steps, warmup, with_balance=True)
    n_tok = cfg.batch * cfg.seq_len
    gemm = {k: v for k, v in r["stages"].items() if v.get("bound") == "mfma"}
    fl = sum(v["achieved_tflops"] * v["ms"] for v in gemm.values())
    ms = sum(v["ms"] for v in gemm.values())
    return {"workload": f"{cfg.name}: B={cfg.batch}, L={cfg.seq_len}, d_model={cfg.d_model}, E={cfg.n_experts}, "
                        f"top_k={cfg.top_k}, bf16", "ms_per_step": r["ms_median"], "tokens_per_s": n_tok / (r["ms_median"] * 1e-3),
            "gemm_frac_of_mfma_peak": (fl / ms / PEAK_BF16_TFLOPS) if ms > 0 else None,
            "scan_frac_of_hbm_peak": r["stages"]["scan_gate"].get("frac"),
            "expert_counts_max_over_mean": r["balance"]["max_over_mean_count"], "stages": r["stages"]}


# ------------------------------------------------------------------ HBM traffic of the dominant kernel
def traffic_child(workload):
    """Runs under rocprofv3 --pmc: a few forward calls and a few copies of known size."""
    import torch
    from paper_2506_18145_amd import RomLayer, rom_layer_forward, rom_profile_copy
    from rom_synth import get_config, make_input, make_weights
    cfg = get_config(workload)
    layer = RomLayer(cfg, make_weights(cfg), device="cuda:0")
    x = layer.to_device(make_input(cfg))
    B, L = cfg.batch, cfg.seq_len
    out = torch.empty_like(x)
    ws = layer.workspace(B, L)
    for _ in range(3):
        rom_layer_forward(layer.dims, layer.weights, x, B, L, None, None, out, None, None, ws)
    src = torch.ones(TRAFFIC_COPY_BYTES, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    for _ in range(3):
        rom_profile_copy(src, dst)
    torch.cuda.synchronize()


TRAFFIC_COPY_BYTES = 1 << 29      # 512 MiB read + 512 MiB written by the calibration copy


def measure_traffic(workload):
    """HBM bytes per launch of the dominant kernel from two rocprofv3 --pmc runs of this script
    (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch), each reading scaled by what the same counter
    shows for the library's plain copy kernel of known size.  Runs the profiler as child processes
    BEFORE this process touches the GPU.  Returns (bytes or None, detail dict)."""
    import csv
    import glob
    import shutil
    import subprocess
    import tempfile
    prof = shutil.which("rocprofv3") or "/opt/rocm/bin/rocprofv3"
    if not os.path.exists(prof):
        return None, {"note": "rocprofv3 not found"}
    detail = {"command": "rocprofv3 --pmc <FETCH_SIZE|WRITE_SIZE> -d <tmp> -o p --output-format csv -- python3 bench.py "
                         f"--traffic-child --workload {workload}", "copy_bytes": TRAFFIC_COPY_BYTES}
    total = 0.0
    for counter in ("FETCH_SIZE", "WRITE_SIZE"):
        tmp = tempfile.mkdtemp(prefix="rom_pmc_", dir="/tmp")
        try:
            env = dict(os.environ, TMPDIR="/tmp")
            cmd = [prof, "--pmc", counter, "-d", tmp, "-o", "p", "--output-format", "csv", "--", "python3",
                   os.path.join(ROOT, "bench.py"), "--traffic-child", "--workload", workload]
            run = subprocess.run(cmd, cwd="/tmp", env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=240)
            files = glob.glob(os.path.join(tmp, "**", "*counter_collection.csv"), recursive=True)
            if run.returncode != 0 or not files:
                return None, dict(detail, note=f"{counter} run failed (rc {run.returncode})")
            kern, copy = [], []
            for path in files:
                for row in csv.DictReader(open(path)):
                    if row.get("Counter_Name") != counter:
                        continue
                    if DOMINANT_KERNEL in row["Kernel_Name"]:
                        kern.append(float(row["Counter_Value"]))
                    elif "calib_copy_kernel" in row["Kernel_Name"]:
                        copy.append(float(row["Counter_Value"]))
            if not kern or not copy:
                return None, dict(detail, note=f"{counter}: kernel rows not found")
            kern_kib, copy_kib = sum(kern) / len(kern), sum(copy) / len(copy)
            factor = (TRAFFIC_COPY_BYTES / 1024.0) / copy_kib
            detail[counter] = {"kernel_kib_per_dispatch": kern_kib, "copy_kib_per_dispatch": copy_kib, "scale": factor}
            total += kern_kib * 1024.0 * factor
        except Exception as exc:      # a profiler problem must not cost the benchmark line
            return None, dict(detail, note=f"{counter}: {type(exc).__name__}: {exc}")
        finally:
            shutil.rmtree(tmp, ignore_errors=True)
    return total, detail


def probe_rates():
    """Issue rates of this chip as a wavefront sees them (ns and clocks at 2.4 GHz per instruction and
    wavefront, at 1 / 2 / 4 / 8 wavefronts per SIMD), and the pipelined scan's tile without its memory
    traffic.  Prints one JSON object."""
    import torch
    from paper_2506_18145_amd import rom_probe
    scratch = torch.empty(256 * 8 * 256, dtype=torch.float32, device="cuda:0")

    def run(kind, p0, p1, waves, iters):
        rom_probe(kind, p0, p1, 256 * waves, 8, scratch)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        rom_probe(kind, p0, p1, 256 * waves, iters, scratch)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)

    out = {"note": "ns per instruction (or scan step) and wavefront; clk = ns x 2.4; waves = wavefronts per SIMD"}
    ops = {0: "v_fma_f32", 1: "v_exp_f32", 2: "v_mov_b32_dpp"}
    for op, name in ops.items():
        for chains in (1, 8):
            row = {}
            for waves in (1, 2, 4, 8):
                ns = run(0, op, chains, waves, 20000) * 1e6 / (20000 * 64)
                row[f"waves={waves}"] = {"ns": round(ns, 3), "clk": round(ns * 2.4, 2), "simd_clk_per_inst": round(ns * 2.4 / waves, 2)}
            out[f"{name}, {'dependent chain' if chains == 1 else '8 independent chains'}"] = row
    parts = {(3, 0): "scan tile: decay/input + FMA chain", (6, 0): "scan tile: FMA chain + reduction/gate",
             (7, 0): "scan tile: all three stages, registers only", (7, 1): "scan tile: all + LDS reads",
             (7, 2): "scan tile: all + LDS reads + barrier"}
    for (p0, p1), name in parts.items():
        row = {}
        for blocks in (1, 2):
            ns = run(1, p0, p1, blocks, 256) * 1e6 / (256 * 64)
            row[f"blocks_per_cu={blocks}"] = {"ns_per_step": round(ns, 2), "clk_per_step": round(ns * 2.4, 1)}
        out[name] = row
    print(json.dumps(out, indent=1))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=50,
                    help="untimed calls before the timed ones (the first dozens of calls after an idle spell run up to 4 %% slower: clocks still ramping)")
    ap.add_argument("--workload", default="cfg2", choices=["cfg1", "cfg2", "cfg3"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=16384)
    ap.add_argument("--no-step", action="store_true",
                    help="skip the extra rom_step measurement (256 sequences x 512 steps, cfg4)")
    ap.add_argument("--no-shared-xdt", action="store_true",
                    help="skip the extra measurement of the shared x/dt variant of the workload")
    ap.add_argument("--no-ffn", action="store_true", help="skip the extra FFN-MoE layer measurement")
    ap.add_argument("--no-backward", action="store_true", help="skip the extra backward-pass measurement")
    ap.add_argument("--no-mamba2", action="store_true", help="skip the RoM-on-Mamba2 layer measurement")
    ap.add_argument("--no-gdn", action="store_true", help="skip the RoM-on-Gated-DeltaNet layer measurement")
    ap.add_argument("--no-configs", action="store_true", help="skip the legs on the other paper-shaped workloads")
    ap.add_argument("--no-traffic", action="store_true",
                    help="skip the two rocprofv3 counter runs that measure the dominant kernel's HBM traffic")
    ap.add_argument("--stack-layers", type=int, default=48,
                    help="layers of the extra whole-stack measurement (0 = skip it)")
    ap.add_argument("--hybrid-layers", type=int, default=0,
                    help="also time a stack of this many (RoM block + FFN-MoE block) pairs (0 = skip)")
    ap.add_argument("--only-step", action="store_true",
                    help="run only the rom_step measurement and print its JSON object (for profiling)")
    ap.add_argument("--traffic-child", action="store_true", help=argparse.SUPPRESS)
    ap.add_argument("--probe", action="store_true",
                    help="print the chip's measured instruction issue rates and the scan tile's compute-only time, then exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.traffic_child:
        traffic_child(args.workload)
        return
    if args.probe:
        probe_rates()
        return
    if args.only_step:
        print(json.dumps({"decode_step": decode_step_rate()}))
        return

    # counter runs first: they are child processes of a parent that has not touched the GPU yet
    traffic, traffic_detail = (None, {"note": "skipped (--no-traffic)"}) if args.no_traffic else measure_traffic(args.workload)

    from dataclasses import replace
    from rom_synth import get_config

    cfg = get_config(args.workload)
    B, L = cfg.batch, cfg.seq_len
    n_tok = B * L
    r = time_forward(cfg, args.steps, args.warmup)
    stages = r["stages"]
    dom = stages["in_proj"]
    clock_ratio = COUNTER_CLOCK_GHZ_GEMM / NOMINAL_CLOCK_GHZ
    roofline = {"kernel": f"in_proj grouped GEMM ({DOMINANT_KERNEL})", "bound": "mfma",
                "achieved": dom.get("achieved_tflops"), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": dom.get("frac"),
                "traffic": traffic, "traffic_detail": traffic_detail,
                "algorithmic_bytes": (n_tok * cfg.top_k * cfg.d_model + cfg.n_experts * 2 * cfg.d_inner * cfg.d_model
                                      + n_tok * cfg.top_k * 2 * cfg.d_inner) * 2,
                "clock_ghz_nominal": NOMINAL_CLOCK_GHZ, "clock_ghz_from_counters": COUNTER_CLOCK_GHZ_GEMM,
                "peak_at_counter_clock": PEAK_BF16_TFLOPS * clock_ratio,
                "frac_at_counter_clock": (dom["frac"] / clock_ratio) if dom.get("frac") else None,
                "alu_peak_note": ALU_PEAK_NOTE}

    result = {
        "metric": "RoM layer fwd tokens/s at d=2048,L=16K; % MFMA peak (GEMM), % HBM BW (scan)",
        "value": n_tok / (r["ms_median"] * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["ms_median"],
        "ms_per_step_is": "median over the K timed calls (HIP events around every call and around the in projection "
                          "inside it, on the launch stream)",
        "ms_per_step_mean_wall": r["ms_mean_wall"],
        "ms_per_step_without_stage_events": r["ms_mean_wall_without_stage_events"],
        "ms_per_step_with_all_stage_events": r["ms_mean_wall_all_stage_events"],
        "stages_are": "medians over a second pass of K calls with an event at every stage boundary "
                      "(in_proj: from the timed region)",
        "ms_per_step_min_max": [r["ms_min"], r["ms_max"]],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: RoM layer forward, B={B}, L={L}, d_model={cfg.d_model}, "
                               f"d_inner={cfg.d_inner}, d_state={cfg.d_state}, dt_rank={cfg.dt_rank}, "
                               f"E={cfg.n_experts}, top_k={cfg.top_k}, routed x/dt, bf16",
                   "tokens_per_step": n_tok},
        "roofline": roofline,
        "stages": stages,
    }
    result["balance_stats"] = r.get("balance")

    def extra(name, fn):
        """A leg beside the headline measurement: its failure must not cost the headline line."""
        try:
            result[name] = fn()
        except Exception as exc:                      # reported, not hidden: the leg's object says what failed
            result[name] = {"error": f"{type(exc).__name__}: {exc}"}

    if not args.no_configs:
        for other in ("cfg1", "cfg3"):
            if other != cfg.name:
                extra(other, lambda other=other: config_leg(other, max(args.steps // 2, 5), args.warmup))
    if not args.no_shared_xdt:
        # the paper's default variant (Sec. 4.3, design choices): x and dt projections shared by all experts, so
        # those two stages are plain GEMMs; same shapes and inputs otherwise
        def shared_leg():
            shared = replace(cfg, name=cfg.name + "-shared-xdt", routed_xdt=False)
            rs = time_forward(shared, max(args.steps // 2, 1), args.warmup, with_balance=False)
            return {"workload": f"{cfg.name} with one shared x/dt projection (E_x = 1)", "ms_per_step": rs["ms_median"],
                    "tokens_per_s": n_tok / (rs["ms_median"] * 1e-3),
                    "stages_ms": {k: v["ms"] for k, v in rs["stages"].items()}}
        extra("shared_xdt_variant", shared_leg)
    if not args.no_backward and cfg.top_k == 1:
        extra("backward", lambda: backward_rate(cfg, 5, 2))
    if not args.no_mamba2:
        extra("mamba2_variant", lambda: mamba2_rate(10, 3))
    if not args.no_gdn:
        extra("gdn_variant", lambda: gdn_rate(5, 2))
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
