"""Shared helpers of the GPU parity tests: run the HIP path through the binding, run the oracle
on the same seeded inputs, compare under the stated tolerances."""
from __future__ import annotations

import numpy as np
import torch

from oracle import rom_oracle as O
from paper_2506_18145_amd import RomLayer
from rom_synth import make_input, make_weights

# max |gpu - ref| / max |ref| per tensor
TOL = {"fp32": 1e-4, "bf16": 2e-2}
MARGIN = 1e-5     # tokens whose top-K logit margin is below this are excluded from the exact-index check
# Per element, with a floor: max_i |gpu_i - ref_i| / (|ref_i| + rms(ref)).  The tensor-normalised
# figure above lets an error hide in small-magnitude regions next to a few large elements; this one
# holds every element to its own size, down to the tensor's rms (a plain elementwise ratio has no
# meaning at zero crossings).  An element of typical size carries the same rounding error as the
# tensor maximum does relative to itself, but the errors of the bf16 intermediates it was computed
# from scale with *their* typical size, so the ratio is a few times the normalised figure: the
# bound is 2.5 x TOL.  It is asserted for xz, u, dt_low, B/C and dt, whose elements all live on
# the scale of their tensor.  g and out are heavy-tailed (y = C.h cancels, and h spans decades
# across channels and tokens): an element whose terms are as large as the tensor's largest but
# cancel carries the largest elements' absolute error against a small value, so there the figure
# is printed only.  What is asserted for them (same bound) is the componentwise form of the
# textbook error bound of a sum, |error of sum| <= eps * sum |terms|: the oracle is run once more
# on absolute values (|u|, |B|, |C|, |D|, |h0| through the scan, then |SiLU(z)| and |W_out|; the
# inputs that are projection or conv outputs, whose own error is uniform over their tensor, enter
# at |value| + rms), which gives every element the size of the terms it was added up from - it
# follows dt, the channel and the history of the state, which is where the decades come from -
# and the error of every element of g and out is held to the tolerance at that scale.
ELEM_TOL = {"fp32": 2.5e-4, "bf16": 5e-2}


def rel_err(got, ref) -> float:
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    scale = np.max(np.abs(ref))
    return float(np.max(np.abs(got - ref)) / (scale if scale > 0 else 1.0))


def elem_err(got, ref) -> float:
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    rms = float(np.sqrt(np.mean(ref * ref)))
    if rms == 0.0:
        return float(np.max(np.abs(got - ref)))
    return float(np.max(np.abs(got - ref) / (np.abs(ref) + rms)))


def col_err(got, ref) -> float:
    """Worst column of a [rows, columns] tensor, each column normalised by its own maximum: for
    tensors whose columns live on different scales (dt spans two decades across channels)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    scale = np.max(np.abs(ref), axis=0)
    scale = np.where(scale > 0, scale, 1.0)
    return float(np.max(np.max(np.abs(got - ref), axis=0) / scale))


def term_scales(cfg, ref, w_np, idx, ssm_state):
    """Size of the terms every element of g and of the layer output is summed from: the oracle's
    scan, gate and out projection evaluated on absolute values (of the oracle's own u, dt, B, C, z
    and gate).  Returns (g_abs [N, D_e], out_abs [N, D_m])."""
    n_tok, d_e = ref["u"].shape
    bsz = cfg.batch
    length = n_tok // bsz
    r, d_s = cfg.dt_rank, cfg.d_state
    # u, B, C and z are themselves sums that cancel (conv taps, projections), with an error that is
    # uniform over their tensor: each enters at |value| + rms of its tensor
    rms = lambda v: np.sqrt(np.mean(np.square(v)))
    bm, cm = ref["xdbl"][:, r:r + d_s], ref["xdbl"][:, r + d_s:]
    b_abs = (np.abs(bm) + rms(bm)).reshape(bsz, length, d_s)
    c_abs = (np.abs(cm) + rms(cm)).reshape(bsz, length, d_s)
    u_abs = (np.abs(ref["u"]) + rms(ref["u"])).reshape(bsz, length, d_e)
    a = -np.exp(np.asarray(w_np["A_log"], np.float64))
    y_abs, _ = O.selective_scan(u_abs, ref["dt"].reshape(bsz, length, d_e), b_abs, c_abs, a,
                                np.abs(np.asarray(w_np["D"], np.float64)),
                                None if ssm_state is None else np.abs(np.asarray(ssm_state, np.float64)))
    # the gate factor SiLU(z): z is a projection output whose error is uniform over the tensor
    # (every element sums terms of one size), so its factor is floored at the tensor's rms
    z = ref["xz"][:, d_e:]
    g_abs = y_abs.reshape(n_tok, d_e) * (np.abs(O.silu(z)) + np.sqrt(np.mean(z * z)))
    w_out_abs = np.abs(np.asarray(w_np["w_out"], np.float64))
    out_abs = np.zeros((n_tok, cfg.d_model))
    for k in range(cfg.top_k):
        out_abs += ref["gate"][:, k:k + 1] * O.routed_linear(g_abs, w_out_abs, idx[:, k:k + 1])
    return g_abs, out_abs


def max_excluded(logits, top_k: int) -> int:
    """How many tokens the margin band may exempt from the exact-index check before the check
    counts as vacuous.  For continuous logits of spread sigma the density of an expert's logit
    is at most 0.4 / sigma, so a given neighbour gap is below MARGIN with probability at most
    MARGIN * E * 0.4 / sigma; K gaps per token, a factor 3 of slack, plus 2: a handful of the
    16K tokens of the paper-shaped workloads (measured: 0 or 1), a few percent only at 64
    experts with top-8 on narrow logits."""
    logits = np.asarray(logits, np.float64)
    n, e = logits.shape
    sigma = float(np.median(np.std(logits, axis=0))) if n > 1 else 1.0
    sigma = max(sigma, 1e-3)
    return 2 + int(3.0 * n * top_k * e * 0.4 * MARGIN / sigma)


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy() if t.is_floating_point() else t.detach().cpu().numpy()


def f64_weights(w):
    """Upcast once so that repeated oracle calls do not convert the big matrices again."""
    return {k: (None if v is None else np.asarray(v, np.float64)) for k, v in w.items()}


BLOCK_EPS = 1e-5


def check_routing(cfg, gpu, x_np, w_np, block=False):
    """gpu: dict of numpy arrays from the HIP path.  Returns (expert_idx to hand the oracle, n_excluded).
    block: the router sees the RMS-normalised input."""
    n_tok = gpu["expert_idx"].shape[0]
    x_r = O.rms_norm(x_np, w_np["norm_w"], BLOCK_EPS) if block else x_np
    logits = O.router_logits(x_r.reshape(n_tok, -1), w_np["w_router"], w_np.get("b_router"))
    own = O.topk_select(logits, cfg.top_k)
    close = O.topk_margin(logits, cfg.top_k) < MARGIN
    idx = gpu["expert_idx"].astype(np.int32)
    assert int(close.sum()) <= max_excluded(logits, cfg.top_k), \
        f"{int(close.sum())} of {n_tok} tokens inside the margin band"
    assert np.array_equal(idx[~close], own[~close]), "expert assignment differs outside the margin band"
    # whatever the GPU chose for the excluded tokens must still be K distinct valid experts
    assert idx.min() >= 0 and idx.max() < cfg.n_experts
    if cfg.top_k > 1:
        srt = np.sort(idx, axis=1)
        assert np.all(srt[:, 1:] != srt[:, :-1])
    counts, offsets, perm, inv_perm = O.expert_permutation(idx, cfg.n_experts)
    assert np.array_equal(gpu["counts"], counts)
    assert np.array_equal(gpu["offsets"], offsets)
    assert np.array_equal(gpu["perm"], perm)
    assert np.array_equal(gpu["inv_perm"], inv_perm)
    assert counts.sum() == n_tok * cfg.top_k
    tol = TOL[cfg.dtype]
    if "logits" in gpu:
        assert rel_err(gpu["logits"], logits) <= min(tol, 1e-4)
    gate = O.gate_weights(logits, idx, cfg.gate_mode)
    assert rel_err(gpu["gate"], gate) <= min(tol, 1e-4)
    return idx, int(close.sum())


def run_layer(cfg, conv_state=None, ssm_state=None, x_np=None, w_np=None, return_states=True, block=False):
    """block: the pre-norm residual block (rom_block_forward) instead of the bare layer."""
    w_np = make_weights(cfg) if w_np is None else w_np
    x_np = make_input(cfg) if x_np is None else x_np
    layer = RomLayer(cfg, w_np)
    x = layer.to_device(x_np)
    cs = None if conv_state is None else layer.to_device(conv_state, typed=False)
    ss = None if ssm_state is None else layer.to_device(ssm_state, typed=False)
    B, L = x.shape[0], x.shape[1]
    # the workspace sits between two canary pads: the call may touch rom_workspace_bytes() bytes only
    from paper_2506_18145_amd import rom_workspace_bytes
    need, pad = rom_workspace_bytes(layer.dims, max(B, 1), max(L, 1)), 4096
    guarded = torch.full((need + 2 * pad,), 0xA5, dtype=torch.uint8, device=layer.device)
    layer._ws = guarded[pad:pad + need]
    if block:
        out, conv_out, ssm_out = layer.block_forward(x, cs, ss, return_states=True, eps=BLOCK_EPS)
    else:
        out, conv_out, ssm_out = layer.forward(x, cs, ss, return_states=True)
    torch.cuda.synchronize()
    assert layer._ws.data_ptr() == guarded.data_ptr() + pad, "the layer replaced the guarded workspace"
    assert bool((guarded[:pad] == 0xA5).all()) and bool((guarded[pad + need:] == 0xA5).all()), \
        "a kernel wrote outside the workspace"
    gpu = {name: to_np(layer.ws_view(name, B, L)) for name in
           ("expert_idx", "gate", "counts", "offsets", "perm", "inv_perm", "logits", "xz", "u", "dt_low",
            "bc", "dt", "g")}
    gpu.update(out=to_np(out), conv_state=to_np(conv_out), ssm_state=to_np(ssm_out))
    return layer, gpu, x_np, w_np


def compare_layer(cfg, gpu, x_np, w_np, conv_state=None, ssm_state=None, stages=True, block=False):
    idx, n_excl = check_routing(cfg, gpu, x_np, w_np, block)
    if block:
        ref = O.rom_block_forward(x_np, w_np, cfg.top_k, cfg.gate_mode, BLOCK_EPS, conv_state, ssm_state,
                                  expert_idx=idx)
    else:
        ref = O.rom_layer_forward(x_np, w_np, cfg.top_k, cfg.gate_mode, conv_state, ssm_state, expert_idx=idx)
    tol = TOL[cfg.dtype]
    errs, elem, scaled = {}, {}, {}
    if stages:
        r = cfg.dt_rank
        pairs = {"xz": (gpu["xz"], ref["xz"]), "u": (gpu["u"], ref["u"]),
                 "dt_low": (gpu["dt_low"], ref["xdbl"][:, :r]), "bc": (gpu["bc"], ref["xdbl"][:, r:]),
                 "dt": (gpu["dt"], ref["dt"]), "g": (gpu["g"], ref["g"])}
        for name, (got, want) in pairs.items():
            errs[name] = rel_err(got, want)
            elem[name] = elem_err(got, want)
        errs["dt/col"] = col_err(gpu["dt"], ref["dt"])       # every channel's dt at its own scale
    errs["out"] = rel_err(gpu["out"], ref["out"])
    elem["out"] = elem_err(gpu["out"], ref["out"])
    if stages:
        g_abs, out_abs = term_scales(cfg, ref, w_np, idx, ssm_state)
        scaled["g"] = float(np.max(np.abs(np.asarray(gpu["g"], np.float64) - ref["g"]) / (g_abs + 1e-300)))
        got_out = np.asarray(gpu["out"], np.float64).reshape(out_abs.shape)
        if block:            # the skip term is exact up to the output's own rounding
            out_abs = out_abs + np.abs(np.asarray(x_np, np.float64)).reshape(out_abs.shape)
        scaled["out"] = float(np.max(np.abs(got_out - ref["out"].reshape(out_abs.shape)) / (out_abs + 1e-300)))
    if block:
        # the branch alone, so that an error in it cannot hide behind a large skip term; the
        # output's own rounding (unit roundoff of the activation type: 8 significant bits in
        # bf16, 24 in fp32, times |out|) is allowed on top
        got_branch = gpu["out"].astype(np.float64) - np.asarray(x_np, np.float64)
        ulp = 2.0 ** -8 if cfg.dtype == "bf16" else 2.0 ** -24
        slack = ulp * np.max(np.abs(ref["out"])) / np.max(np.abs(ref["branch"]))
        errs["branch"] = max(rel_err(got_branch, ref["branch"]) - slack, 0.0)
    errs["ssm_state"] = rel_err(gpu["ssm_state"], ref["ssm_state"])
    errs["conv_state"] = rel_err(gpu["conv_state"], ref["conv_state"])
    print(f"[{cfg.name}] excluded={n_excl} counts={gpu['counts'].tolist()} "
          + " ".join(f"{k}={v:.2e}" for k, v in errs.items())
          + " | per element (rms floor): " + " ".join(f"{k}={v:.2e}" for k, v in elem.items())
          + " | at the scale of the summed terms: " + " ".join(f"{k}={v:.2e}" for k, v in scaled.items()), flush=True)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, f"beyond tolerance {tol}: {bad}"
    etol = ELEM_TOL[cfg.dtype]
    bad = {k: v for k, v in elem.items() if k not in ("g", "out") and not v <= etol}
    assert not bad, f"per-element error beyond {etol}: {bad}"
    bad = {k: v for k, v in scaled.items() if not v <= etol}
    assert not bad, f"error beyond {etol} of the summed terms' size: {bad}"
    return ref, errs
