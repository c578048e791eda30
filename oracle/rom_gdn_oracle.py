"""CPU oracle for RoM applied to a Gated DeltaNet layer (Sec. 5.2, Table 3 and the paragraph on
streamlined SSMs).

TEST INFRASTRUCTURE ONLY, like oracle/rom_oracle.py: plain fp64, step by step, no chunking.

The paper prints no equations for this variant.  Readings taken here (also in the design notes):
  * The layer is the published Gated DeltaNet (Yang, Kautz, Hatamizadeh 2024): projections of the
    input to a gate z, queries q, keys k, values v and two numbers per head b, a; a short causal
    depthwise conv + SiLU over q | k | v; q and k are L2-normalised per head (x / sqrt(sum x^2 + 1e-6))
    and q is scaled by d_k^-1/2; beta = sigmoid(b) and the log decay g = -exp(A_log) softplus(a + dt_bias)
    are one number per head and step; per head the state S (d_v x d_k) follows the gated delta rule
        S_t = alpha_t S_{t-1} (I - beta_t k_t k_t^T) + beta_t v_t k_t^T,   alpha_t = exp(g_t),
        o_t = S_t q_t;
    the output is RMSNorm over each head's d_v channels (scale norm_w [d_v], eps inside the root)
    times SiLU(z), then the output projection.
  * "Applied comprehensively across all major projection layers": the input projection (all six
    parts, stored as one matrix with rows z | q | k | v | b | a) and the output projection are
    mixtures of experts driven by ONE router decision per token; conv, dt_bias, A_log and the norm
    scale are shared.  The routed input projection is an unweighted sum over the selected experts
    (as Eq. (10)/(11)); only the output projection is weighted by the router's gate (Eq. (12)/(13)).

Array layouts: w_in [E, 2*D_v + 2*D_k + 2*H, d_model] (D_k = H d_k, D_v = H d_v); conv_w
[2*D_k + D_v, 4], conv_b over the channels q | k | v; dt_bias, A_log [H]; norm_w [d_v];
w_out [E, d_model, D_v].

Pins (tests/test_oracle_pins_gdn.py): the recurrence against explicit products of the transition
matrices, against the linear system its chunk form solves, the delta rule's exact recall with
orthonormal keys, and the decay-only special case; the layer against a dense layer assembled
separately for one expert and a brute force over the experts.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from .rom_oracle import (F64, causal_conv_silu, expert_permutation, gate_weights, routed_linear,
                         router_logits, silu, softplus, topk_select)


def gated_delta_scan(q, k, v, beta, g, s0=None):
    """The gated delta rule, one step at a time.

    q, k [B, L, H, d_k]; v [B, L, H, d_v]; beta (in (0, 1)), g (log decay, <= 0) [B, L, H];
    s0 [B, H, d_v, d_k] or None (zeros).
        S <- exp(g_t) S;   u = beta_t (v_t - S k_t);   S <- S + u k_t^T;   o_t = S q_t
    Returns (o [B, L, H, d_v], final S).
    """
    q = np.asarray(q, F64)
    k = np.asarray(k, F64)
    v = np.asarray(v, F64)
    beta = np.asarray(beta, F64)
    g = np.asarray(g, F64)
    bsz, length, n_heads, d_k = k.shape
    d_v = v.shape[3]
    state = np.zeros((bsz, n_heads, d_v, d_k), F64) if s0 is None else np.array(s0, F64, copy=True)
    o = np.empty((bsz, length, n_heads, d_v), F64)
    for t in range(length):
        state = np.exp(g[:, t])[:, :, None, None] * state
        pred = np.einsum("bhvk,bhk->bhv", state, k[:, t])
        u = beta[:, t][:, :, None] * (v[:, t] - pred)
        state = state + u[:, :, :, None] * k[:, t][:, :, None, :]
        o[:, t] = np.einsum("bhvk,bhk->bhv", state, q[:, t])
    return o, state


def l2_normalize(x, eps=1e-6):
    """x / sqrt(sum(x^2) + eps) over the last axis."""
    x = np.asarray(x, F64)
    return x / np.sqrt(np.sum(x * x, axis=-1, keepdims=True) + eps)


def head_rms_norm_gated(o, z, weight, eps):
    """Per head: RMSNorm over the d_v channels, times weight [d_v], times SiLU(z).  o, z [..., H, d_v]."""
    o = np.asarray(o, F64)
    ms = np.mean(o * o, axis=-1, keepdims=True)
    return o / np.sqrt(ms + eps) * np.asarray(weight, F64) * silu(np.asarray(z, F64))


def rom_gdn_forward(x, w: Dict[str, Optional[np.ndarray]], top_k: int, gate_mode: int, n_heads: int, d_k: int,
                    eps: float = 1e-5, expert_idx=None, conv_state=None, ssm_state=None) -> Dict[str, np.ndarray]:
    """x [B, L, d_model] -> out [B, L, d_model] and the intermediates (token-major).  conv_state
    [B, 2 D_k + D_v, 3] and ssm_state [B, H, d_v, d_k] carry a sequence across calls (None: zeros)."""
    x = np.asarray(x, F64)
    bsz, length, d_m = x.shape
    n_tok = bsz * length
    xt = x.reshape(n_tok, d_m)
    n_exp = w["w_router"].shape[0]
    d_vt = w["w_out"].shape[2]
    d_v = d_vt // n_heads
    d_kt = n_heads * d_k

    logits = router_logits(xt, w["w_router"], w.get("b_router"))
    idx = topk_select(logits, top_k) if expert_idx is None else np.asarray(expert_idx, np.int32)
    gate = gate_weights(logits, idx, gate_mode)
    counts, offsets, perm, inv_perm = expert_permutation(idx, n_exp)

    proj = routed_linear(xt, w["w_in"], idx)                     # z | q | k | v | b | a
    z = proj[:, :d_vt]
    qkv_pre = proj[:, d_vt:2 * d_vt + 2 * d_kt].reshape(bsz, length, 2 * d_kt + d_vt)
    b_raw = proj[:, 2 * d_vt + 2 * d_kt:2 * d_vt + 2 * d_kt + n_heads]
    a_raw = proj[:, 2 * d_vt + 2 * d_kt + n_heads:]
    qkv, conv_out = causal_conv_silu(qkv_pre, w["conv_w"], w.get("conv_b"), conv_state)
    q = l2_normalize(qkv[:, :, :d_kt].reshape(bsz, length, n_heads, d_k)) * d_k ** -0.5
    k = l2_normalize(qkv[:, :, d_kt:2 * d_kt].reshape(bsz, length, n_heads, d_k))
    v = qkv[:, :, 2 * d_kt:].reshape(bsz, length, n_heads, d_v)
    beta = (1.0 / (1.0 + np.exp(-b_raw))).reshape(bsz, length, n_heads)
    g = (-np.exp(np.asarray(w["A_log"], F64))[None, :]
         * softplus(a_raw + np.asarray(w["dt_bias"], F64)[None, :])).reshape(bsz, length, n_heads)
    o, state = gated_delta_scan(q, k, v, beta, g, ssm_state)
    y = head_rms_norm_gated(o, z.reshape(bsz, length, n_heads, d_v), w["norm_w"], eps).reshape(n_tok, d_vt)
    out = np.zeros((n_tok, d_m), F64)
    for kk in range(top_k):                                      # gate-weighted, as Eq. (12)
        out += gate[:, kk:kk + 1] * routed_linear(y, w["w_out"], idx[:, kk:kk + 1])
    return {
        "logits": logits, "expert_idx": idx, "gate": gate, "counts": counts, "offsets": offsets,
        "perm": perm, "inv_perm": inv_perm, "proj": proj, "qkv": qkv.reshape(n_tok, -1),
        "q": q.reshape(n_tok, d_kt), "k": k.reshape(n_tok, d_kt), "beta": beta.reshape(n_tok, n_heads),
        "g": g.reshape(n_tok, n_heads), "o": o.reshape(n_tok, d_vt), "y": y,
        "out": out.reshape(bsz, length, d_m), "conv_state": conv_out, "ssm_state": state,
    }


def rom_gdn_step(x, w, top_k, gate_mode, n_heads, d_k, conv_state, ssm_state, eps=1e-5, expert_idx=None):
    """One new token per sequence: x [B, d_model]; the same dict with out [B, d_model] and the updated states."""
    res = rom_gdn_forward(np.asarray(x, F64)[:, None, :], w, top_k, gate_mode, n_heads, d_k, eps, expert_idx,
                          conv_state, ssm_state)
    res["out"] = res["out"][:, 0, :]
    return res
