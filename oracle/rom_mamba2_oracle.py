"""CPU oracle for RoM applied to a Mamba2 layer (Sec. 5.2, Table 3 and the paragraph on streamlined
SSMs; the appendix's note that deploying RoM on Mamba2 follows the logic of the original Mamba).

TEST INFRASTRUCTURE ONLY, like oracle/rom_oracle.py: plain fp64, no tiling, no chunking, no fusion.
Only tests, the smoke check and the benchmark's cpu_baseline leg may import it.

The paper prints no equations for this variant.  Readings taken here (also in the design notes):
  * The Mamba2 layer is the published one (Dao & Gu 2024, "state space duality"): ONE input
    projection produces z | x | B | C | dt; a short causal depthwise conv + SiLU runs over x | B | C;
    dt = softplus(dt + dt_bias) is one number per head; A = -exp(A_log) is one negative scalar per
    head; per head of P channels the state is a P x N matrix with
        H_t = exp(dt_t A) H_{t-1} + dt_t x_t B_t^T,      y_t = H_t C_t + D x_t;
    the output is RMSNorm(y * SiLU(z)) * norm_w (gate first, then the norm over all d_inner
    channels, eps inside the root), then the output projection.  One group: B and C are shared by
    all heads.
  * "Applied comprehensively across all major projection layers": the input projection (all five
    parts of it) and the output projection are mixtures of experts driven by ONE router decision
    per token; conv, dt_bias, A, D and the norm scale are shared.  As in Eq. (10)/(11) the routed
    input projection is an unweighted sum over the selected experts; as in Eq. (12)/(13) only the
    output projection is weighted by the router's gate.

Array layouts: w_in [E, 2*d_inner + 2*N + H, d_model] with rows z | x | B | C | dt; conv_w
[d_inner + 2*N, k], conv_b [d_inner + 2*N] over the channels x | B | C; dt_bias, A_log, D [H];
norm_w [d_inner]; w_out [E, d_model, d_inner]; router as in the Mamba variant.

Pins (tests/test_oracle_pins_mamba2.py): the scan against the pinned Mamba scan it reduces to when
every channel of a head shares dt and A, against the explicit double sum of the dual (attention-like)
form and a geometric-series closed form; the gated norm against hand values and a library norm; the
layer against a dense Mamba2 layer assembled from library routines (one expert) and against an
all-experts brute force.  Nothing here is "parity unpinned".
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from .rom_oracle import (F64, causal_conv_silu, expert_permutation, gate_weights, routed_linear,
                         router_logits, silu, softplus, topk_select)


def ssd_scan(x, dt, a, b_mat, c_mat, d_skip, h0=None):
    """Mamba2's recurrence, one step at a time.

    x [B, L, H, P]; dt [B, L, H] (positive); a [H] (negative); b_mat, c_mat [B, L, N]; d_skip [H];
    h0 [B, H, P, N] or None (zeros).
        state[b,h,p,n] <- exp(dt[b,t,h] a[h]) state[b,h,p,n] + dt[b,t,h] x[b,t,h,p] b_mat[b,t,n]
        y[b,t,h,p]      = sum_n c_mat[b,t,n] state[b,h,p,n] + d_skip[h] x[b,t,h,p]
    Returns (y, final state).
    """
    x = np.asarray(x, F64)
    dt = np.asarray(dt, F64)
    a = np.asarray(a, F64)
    b_mat = np.asarray(b_mat, F64)
    c_mat = np.asarray(c_mat, F64)
    d_skip = np.asarray(d_skip, F64)
    bsz, length, n_heads, p_dim = x.shape
    n_state = b_mat.shape[2]
    state = (np.zeros((bsz, n_heads, p_dim, n_state), F64) if h0 is None else np.array(h0, F64, copy=True))
    y = np.empty((bsz, length, n_heads, p_dim), F64)
    for t in range(length):
        decay = np.exp(dt[:, t, :] * a[None, :])                                   # [B, H]
        inject = (dt[:, t, :, None] * x[:, t, :, :])[:, :, :, None] * b_mat[:, t, None, None, :]
        state = decay[:, :, None, None] * state + inject
        y[:, t] = (state * c_mat[:, t, None, None, :]).sum(axis=3) + d_skip[None, :, None] * x[:, t]
    return y, state


def gated_rms_norm(y, z, weight, eps):
    """RMSNorm(y * SiLU(z)) * weight over the last axis (eps inside the root)."""
    v = np.asarray(y, F64) * silu(np.asarray(z, F64))
    ms = np.mean(v * v, axis=-1, keepdims=True)
    return v / np.sqrt(ms + eps) * np.asarray(weight, F64)


def rom_mamba2_forward(x, w: Dict[str, Optional[np.ndarray]], top_k: int, gate_mode: int, headdim: int,
                       eps: float = 1e-5, expert_idx=None, conv_state=None, ssm_state=None) -> Dict[str, np.ndarray]:
    """x [B, L, d_model] -> out [B, L, d_model] and the intermediates (token-major, [N, ...]).
    conv_state [B, d_inner + 2N, k-1] (the last k-1 conv inputs, oldest first) and ssm_state
    [B, H, P, N] carry a sequence across calls (None: zeros); the new ones are returned."""
    x = np.asarray(x, F64)
    bsz, length, d_m = x.shape
    n_tok = bsz * length
    xt = x.reshape(n_tok, d_m)
    n_exp = w["w_router"].shape[0]
    d_e = w["w_out"].shape[2]
    n_heads = d_e // headdim
    n_state = (w["w_in"].shape[1] - 2 * d_e - n_heads) // 2

    logits = router_logits(xt, w["w_router"], w.get("b_router"))
    idx = topk_select(logits, top_k) if expert_idx is None else np.asarray(expert_idx, np.int32)
    gate = gate_weights(logits, idx, gate_mode)
    counts, offsets, perm, inv_perm = expert_permutation(idx, n_exp)

    zxbcdt = routed_linear(xt, w["w_in"], idx)                   # unweighted sum over the chosen experts
    z = zxbcdt[:, :d_e]
    xbc_pre = zxbcdt[:, d_e:2 * d_e + 2 * n_state].reshape(bsz, length, d_e + 2 * n_state)
    dt_raw = zxbcdt[:, 2 * d_e + 2 * n_state:]
    xbc, conv_out = causal_conv_silu(xbc_pre, w["conv_w"], w.get("conv_b"), conv_state)
    xs = xbc[:, :, :d_e].reshape(bsz, length, n_heads, headdim)
    b_mat = xbc[:, :, d_e:d_e + n_state]
    c_mat = xbc[:, :, d_e + n_state:]
    dt = softplus(dt_raw + np.asarray(w["dt_bias"], F64)[None, :]).reshape(bsz, length, n_heads)
    a = -np.exp(np.asarray(w["A_log"], F64))
    y, state = ssd_scan(xs, dt, a, b_mat, c_mat, w["D"], ssm_state)
    y = y.reshape(n_tok, d_e)
    g = gated_rms_norm(y, z, w["norm_w"], eps)
    out = np.zeros((n_tok, d_m), F64)
    for k in range(top_k):                                       # gate-weighted, as Eq. (12)
        out += gate[:, k:k + 1] * routed_linear(g, w["w_out"], idx[:, k:k + 1])
    return {
        "logits": logits, "expert_idx": idx, "gate": gate, "counts": counts, "offsets": offsets,
        "perm": perm, "inv_perm": inv_perm, "zxbcdt": zxbcdt, "xbc": xbc.reshape(n_tok, -1),
        "dt": dt.reshape(n_tok, n_heads), "y": y, "g": g, "out": out.reshape(bsz, length, d_m),
        "conv_state": conv_out, "ssm_state": state,
    }


def rom_mamba2_step(x, w, top_k, gate_mode, headdim, conv_state, ssm_state, eps=1e-5, expert_idx=None):
    """One new token per sequence: x [B, d_model]; the same dict with out [B, d_model] and the updated states."""
    res = rom_mamba2_forward(np.asarray(x, F64)[:, None, :], w, top_k, gate_mode, headdim, eps, expert_idx,
                             conv_state, ssm_state)
    res["out"] = res["out"][:, 0, :]
    return res
