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


def rel_err(got, ref) -> float:
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    scale = np.max(np.abs(ref))
    return float(np.max(np.abs(got - ref)) / (scale if scale > 0 else 1.0))


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
    if block:
        out, conv_out, ssm_out = layer.block_forward(x, cs, ss, return_states=True, eps=BLOCK_EPS)
    else:
        out, conv_out, ssm_out = layer.forward(x, cs, ss, return_states=True)
    torch.cuda.synchronize()
    B, L = x.shape[0], x.shape[1]
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
    errs = {}
    if stages:
        r = cfg.dt_rank
        errs["xz"] = rel_err(gpu["xz"], ref["xz"])
        errs["u"] = rel_err(gpu["u"], ref["u"])
        errs["dt_low"] = rel_err(gpu["dt_low"], ref["xdbl"][:, :r])
        errs["bc"] = rel_err(gpu["bc"], ref["xdbl"][:, r:])
        errs["dt"] = rel_err(gpu["dt"], ref["dt"])
        errs["g"] = rel_err(gpu["g"], ref["g"])
    errs["out"] = rel_err(gpu["out"], ref["out"])
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
          + " ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, f"beyond tolerance {tol}: {bad}"
    return ref, errs
