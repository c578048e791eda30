"""CPU oracle for the Routing Mamba (RoM) layer: forward pass, recurrent step, backward pass.

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, fp64 statement of what the
layer computes, written from the paper's equations.  Only tests, the smoke
check and the benchmark's cpu_baseline leg may import it; the product path
(the HIP library and its Python binding) never does, and shares no code with it.

Every function upcasts its inputs to float64 and never rounds an intermediate.
There is no token permutation, no tiling and no fusion: routed projections are
the indicator sums of Eq. (10)/(11) evaluated expert by expert, the scan is the
per-step recurrence of Eq. (5).

Notation (paper Sec. 3.1 / Sec. 4): N tokens, D_m = d_model, D_e = d_inner,
D_s = d_state, k = d_conv, R = dt_rank, E experts, K = top-K.

Readings of the paper taken here (each is also listed in the design notes):
  * gate_mode 0 is Eq. (9) as printed (softmax over all experts, masked to the
    top-K); gate_mode 1 renormalises over the selected K (text before Eq. (9)).
  * Eq. (10)/(11): the routed in/gate projections are *unweighted* sums over
    the selected experts; only the out projection is gate-weighted (Eq. (12)).
  * Eq. (6)/(13): (Y * SiLU-gate) is formed first, then multiplied by W_out.
  * The discretised input matrix is the first-order form dt*B (not the exact
    zero-order hold printed after Eq. (4)); A-bar = exp(dt*A) is exact.
  * y gets the D*u skip term, dt = softplus(dt_proj(...) + dt_bias), the conv
    has a bias: the standard Mamba layer the paper builds on (Sec. 3.1).
  * Routed x/dt projections (the "Conv, Gate, dt, x, Out" variant of Table 1)
    are indicator sums like Eq. (11); dt_bias is one shared vector.
  * Top-K picks on logits, descending, lowest expert index on ties.
  * Eq. (16): per-layer term, F normalised by N*K, expectation over the call's tokens.
  * Eq. (14)/(15): the FFN-MoE layer takes both the TopK set and the weights R_i from the
    preceding RoM layer's router; its experts are SwiGLU MLPs with SiLU as the gate activation.
  * The pre-norm is RMSNorm with a learned scale and an eps inside the square root (the
    paper cites it without a formula or an eps); the skip adds the block's own input.
  * Backward pass (training, Sec. 5.1): reverse-mode differentiation of the equations above with
    the TopK indicator held constant; the router learns through the gate weights of Eq. (12).

Every function here is pinned by tests/test_oracle_pins.py (nothing is "parity unpinned").
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------
# Router: Eq. (9)
# --------------------------------------------------------------------------
def router_logits(x, w_router, b_router=None):
    """l[n, e] = sum_d x[n, d] * W_r[e, d] (+ b_r[e]).  x [N, D_m], w_router [E, D_m]."""
    logits = np.asarray(x, F64) @ np.asarray(w_router, F64).T
    if b_router is not None:
        logits = logits + np.asarray(b_router, F64)[None, :]
    return logits


def topk_select(logits, top_k):
    """K rounds of arg-max over the experts not yet chosen; ties go to the lowest index.

    Returns idx [N, K] int32 with column k the (k+1)-th largest logit.
    """
    work = np.asarray(logits, F64)
    n = work.shape[0]
    idx = np.empty((n, top_k), np.int32)
    rows = np.arange(n)
    chosen = np.zeros(work.shape, bool)
    for k in range(top_k):
        best = np.argmax(np.where(chosen, -np.inf, work), axis=1)   # first occurrence = lowest index
        # every expert still available sits at -inf (a masking bias): the K picks stay distinct,
        # the lowest index not yet chosen is next
        again = chosen[rows, best]
        if again.any():
            best[again] = np.argmin(chosen[again], axis=1)
        idx[:, k] = best
        chosen[rows, best] = True
    return idx


def topk_margin(logits, top_k):
    """Smallest gap between consecutive sorted logits over ranks 1..K+1 (K if K == E).

    A token whose margin is tiny may legitimately be routed differently by an
    fp32 router; parity tests exclude such tokens from the exact-index check.
    """
    s = -np.sort(-np.asarray(logits, F64), axis=1)
    hi = min(top_k + 1, s.shape[1])
    if hi < 2:
        return np.full(s.shape[0], np.inf)
    return np.min(s[:, : hi - 1] - s[:, 1:hi], axis=1)


def softmax(logits):
    z = np.asarray(logits, F64)
    z = z - z.max(axis=1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=1, keepdims=True)


def gate_weights(logits, idx, gate_mode):
    """R_i of Eq. (9) for the selected experts: gate[n, k] = P[n, idx[n, k]] (mode 0),
    divided by the sum over the K selected (mode 1)."""
    p = softmax(logits)
    g = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    if gate_mode == 1:
        g = g / g.sum(axis=1, keepdims=True)
    elif gate_mode != 0:
        raise ValueError("gate_mode must be 0 or 1")
    return g


def expert_permutation(idx, n_experts):
    """Grouping of the N*K (token, k) slots by expert, stable in slot order.

    slot s = n*K + k.  counts[e] = number of slots routed to e; offsets = exclusive
    prefix sum (offsets[E] = N*K); inv_perm[s] = offsets[e_s] + rank of s among the
    slots of the same expert in ascending s; perm = inverse of inv_perm.
    """
    flat = np.asarray(idx, np.int64).reshape(-1)
    counts = np.zeros(n_experts, np.int32)
    for e in flat:
        counts[e] += 1
    offsets = np.zeros(n_experts + 1, np.int32)
    for e in range(n_experts):
        offsets[e + 1] = offsets[e] + counts[e]
    cursor = offsets[:-1].astype(np.int64).copy()
    inv_perm = np.empty(flat.size, np.int32)
    perm = np.empty(flat.size, np.int32)
    for s, e in enumerate(flat):
        pos = cursor[e]
        cursor[e] += 1
        inv_perm[s] = pos
        perm[pos] = s
    return counts, offsets, perm, inv_perm


def balance_stats(logits, idx, n_experts, alpha=1.0):
    """One layer's term of the auxiliary load-balance loss, Eq. (16) (appendix on load balance).

    F[i]     = (slots routed to expert i) / (N * K): the fraction of the dispatched (token, k)
               slots that expert i receives, so that sum_i F[i] = 1 for every K
    P_bar[i] = mean over the N tokens of softmax(logits[n, :])[i]  (the full softmax over all
               E experts, the expectation of Eq. (16) taken over the tokens of the call)
    loss     = alpha * E * sum_i F[i] * P_bar[i]

    The model-level loss is the sum of this term over the layers.  Readings: the equation's
    inner index runs over the experts (its printed upper limit N is the number of experts, as the
    text below it says); F is normalised by N*K rather than N; no routing jitter is applied.
    Returns (F [E], P_bar [E], loss) in float64.
    """
    logits = np.asarray(logits, F64)
    idx = np.asarray(idx)
    n, k = idx.shape
    frac = np.zeros(n_experts, F64)
    p_bar = np.zeros(n_experts, F64)
    for i in range(n_experts):
        frac[i] = np.count_nonzero(idx == i) / float(n * k)
    p = softmax(logits)
    for i in range(n_experts):
        p_bar[i] = p[:, i].sum() / float(n)
    loss = alpha * n_experts * float(np.dot(frac, p_bar))
    return frac, p_bar, loss


# --------------------------------------------------------------------------
# Routed projections: Eq. (10), (11), (13)
# --------------------------------------------------------------------------
def routed_linear(inp, w, idx):
    """out[n, :] = sum_i 1[i in idx[n, :]] * inp[n, :] @ w[i].T     (Eq. (11) pattern)

    inp [N, D_in], w [E, D_out, D_in], idx [N, K].  With E == 1 (shared module)
    every token uses w[0] once.
    """
    inp = np.asarray(inp, F64)
    n_exp = w.shape[0]
    out = np.zeros((inp.shape[0], w.shape[1]), F64)
    if n_exp == 1:
        return inp @ np.asarray(w[0], F64).T
    for i in range(n_exp):
        rows = np.nonzero((idx == i).any(axis=1))[0]
        if rows.size:
            out[rows] += inp[rows] @ np.asarray(w[i], F64).T
    return out


def silu(v):
    return v / (1.0 + np.exp(-v))


def softplus(v):
    # log(1 + exp(v)), written so that large |v| neither overflows nor loses digits
    return np.maximum(v, 0.0) + np.log1p(np.exp(-np.abs(v)))


# --------------------------------------------------------------------------
# Short causal depthwise convolution + SiLU: Eq. (2)
# --------------------------------------------------------------------------
def causal_conv_silu(h, conv_w, conv_b=None, conv_state=None):
    """u[b, t, i] = SiLU(conv_b[i] + sum_j conv_w[i, j] * h[b, t-(k-1)+j, i]).

    h [B, L, D_e]; conv_w [D_e, k]; taps that reach before t = 0 read
    conv_state [B, D_e, k-1] (oldest first) or zero.
    Returns (u, new_conv_state) with new_conv_state the last k-1 inputs.
    """
    h = np.asarray(h, F64)
    bsz, length, d_e = h.shape
    k = conv_w.shape[1]
    cw = np.asarray(conv_w, F64)
    hist = (np.zeros((bsz, k - 1, d_e), F64) if conv_state is None
            else np.asarray(conv_state, F64).transpose(0, 2, 1))
    ext = np.concatenate([hist, h], axis=1)            # [B, k-1+L, D_e]; ext[:, k-1+t] = h[:, t]
    c = np.zeros((bsz, length, d_e), F64)
    if conv_b is not None:
        c += np.asarray(conv_b, F64)[None, None, :]
    for j in range(k):
        c += cw[None, None, :, j] * ext[:, j:j + length, :]
    new_state = ext[:, length:, :].transpose(0, 2, 1).copy()   # last k-1 rows, [B, D_e, k-1]
    return silu(c), new_state


# --------------------------------------------------------------------------
# Selective scan: Eq. (5) with A-bar = exp(dt*A), B-bar*u = dt*B*u, plus D skip
# --------------------------------------------------------------------------
def selective_scan(u, dt, b_mat, c_mat, a, d_skip, h0=None):
    """Per-step recurrence, one step at a time.

    u, dt [B, L, D_e]; b_mat, c_mat [B, L, D_s]; a [D_e, D_s] (negative); d_skip [D_e];
    h0 [B, D_e, D_s] or None (zeros).
        h[b,i,n] <- exp(dt[b,t,i]*a[i,n]) * h[b,i,n] + dt[b,t,i]*b_mat[b,t,n]*u[b,t,i]
        y[b,t,i]  = sum_n c_mat[b,t,n]*h[b,i,n] + d_skip[i]*u[b,t,i]
    Returns (y, h_final).
    """
    u = np.asarray(u, F64)
    dt = np.asarray(dt, F64)
    b_mat = np.asarray(b_mat, F64)
    c_mat = np.asarray(c_mat, F64)
    a = np.asarray(a, F64)
    d_skip = np.asarray(d_skip, F64)
    bsz, length, d_e = u.shape
    h = (np.zeros((bsz, d_e, a.shape[1]), F64) if h0 is None else np.array(h0, F64, copy=True))
    y = np.empty((bsz, length, d_e), F64)
    for t in range(length):
        decay = np.exp(dt[:, t, :, None] * a[None, :, :])
        h = decay * h + (dt[:, t, :] * u[:, t, :])[:, :, None] * b_mat[:, t, None, :]
        y[:, t, :] = (h * c_mat[:, t, None, :]).sum(axis=2) + d_skip[None, :] * u[:, t, :]
    return y, h


# --------------------------------------------------------------------------
# The layer: Eq. (9)-(13) over Eq. (1)-(6)
# --------------------------------------------------------------------------
def rom_layer_forward(x, w: Dict[str, Optional[np.ndarray]], top_k: int, gate_mode: int = 0,
                      conv_state=None, ssm_state=None, expert_idx=None) -> Dict[str, np.ndarray]:
    """x [B, L, D_m] -> out [B, L, D_m] and everything in between.

    `w` uses the layouts of rom_synth.make_weights.  `expert_idx` [N, K], if given,
    replaces the oracle's own top-K decision (used only for tokens whose logits
    are too close to call in fp32).
    """
    x = np.asarray(x, F64)
    bsz, length, d_m = x.shape
    n_tok = bsz * length
    xt = x.reshape(n_tok, d_m)
    n_exp = w["w_router"].shape[0]
    d_e = w["w_out"].shape[2]
    d_s = w["A_log"].shape[1]
    r = w["w_dt"].shape[2]

    logits = router_logits(xt, w["w_router"], w.get("b_router"))
    idx = topk_select(logits, top_k) if expert_idx is None else np.asarray(expert_idx, np.int32)
    gate = gate_weights(logits, idx, gate_mode)
    counts, offsets, perm, inv_perm = expert_permutation(idx, n_exp)

    xz = routed_linear(xt, w["w_in"], idx)                       # Eq. (11) | Eq. (10) before SiLU
    h_pre = xz[:, :d_e].reshape(bsz, length, d_e)
    z = xz[:, d_e:]
    u, conv_out = causal_conv_silu(h_pre, w["conv_w"], w.get("conv_b"), conv_state)   # Eq. (2)
    ut = u.reshape(n_tok, d_e)
    xdbl = routed_linear(ut, w["w_x"], idx)                      # dt_low | B | C
    dt_low, b_mat, c_mat = xdbl[:, :r], xdbl[:, r:r + d_s], xdbl[:, r + d_s:]
    dt = softplus(routed_linear(dt_low, w["w_dt"], idx) + np.asarray(w["dt_bias"], F64)[None, :])
    a = -np.exp(np.asarray(w["A_log"], F64))
    y, ssm_out = selective_scan(u, dt.reshape(bsz, length, d_e), b_mat.reshape(bsz, length, d_s),
                                c_mat.reshape(bsz, length, d_s), a, w["D"], ssm_state)   # Eq. (5)
    g = y.reshape(n_tok, d_e) * silu(z)                          # Y * G, Eq. (10)/(13)
    out = np.zeros((n_tok, d_m), F64)
    for k in range(top_k):                                       # Eq. (12)
        out += gate[:, k:k + 1] * routed_linear(g, w["w_out"], idx[:, k:k + 1])
    return {
        "logits": logits, "expert_idx": idx, "gate": gate, "counts": counts, "offsets": offsets,
        "perm": perm, "inv_perm": inv_perm, "xz": xz, "u": ut, "xdbl": xdbl, "dt": dt,
        "y": y.reshape(n_tok, d_e), "g": g, "out": out.reshape(bsz, length, d_m),
        "conv_state": conv_out, "ssm_state": ssm_out,
    }


def rom_step(x, w, top_k, gate_mode, conv_state, ssm_state, expert_idx=None):
    """One new token per sequence: x [B, D_m]; states as in rom_layer_forward.
    Returns the same dict with out [B, D_m] and the updated states."""
    res = rom_layer_forward(np.asarray(x, F64)[:, None, :], w, top_k, gate_mode,
                            conv_state, ssm_state, expert_idx)
    res["out"] = res["out"][:, 0, :]
    return res


# --------------------------------------------------------------------------
# Pre-norm residual block and a stack of blocks (appendix, architectures overview)
# --------------------------------------------------------------------------
def rms_norm(x, weight, eps):
    """Root-mean-square layer normalisation over the last axis:
    x / sqrt(mean(x^2) + eps) * weight (the pre-norm the paper cites for every layer)."""
    x = np.asarray(x, F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(weight, F64)


def rom_block_forward(x, w, top_k, gate_mode=0, eps=1e-5, conv_state=None, ssm_state=None,
                      expert_idx=None):
    """out = x + RoM(RMSNorm(x)): the pre-norm, skip-connected layer of the appendix's
    architecture overview.  w["norm_w"] [D_m] is the norm's scale.  Returns the dict of
    rom_layer_forward (intermediates of the inner layer) with "out" the block output and
    "xn" the normalised input."""
    x = np.asarray(x, F64)
    xn = rms_norm(x, w["norm_w"], eps)
    res = rom_layer_forward(xn, w, top_k, gate_mode, conv_state, ssm_state, expert_idx)
    res["xn"] = xn
    res["branch"] = res["out"]
    res["out"] = x + res["out"]
    return res


def rom_stack_forward(x, layers, top_k, gate_mode=0, eps=1e-5, conv_states=None, ssm_states=None,
                      expert_idx=None):
    """Blocks applied one after another: layer j reads layer j-1's output.  conv_states /
    ssm_states: per-layer lists (or None for zeros); expert_idx: per-layer list (or None).
    Returns (out, per-layer result dicts)."""
    h = np.asarray(x, F64)
    results = []
    for j, w in enumerate(layers):
        res = rom_block_forward(h, w, top_k, gate_mode, eps,
                                None if conv_states is None else conv_states[j],
                                None if ssm_states is None else ssm_states[j],
                                None if expert_idx is None else expert_idx[j])
        results.append(res)
        h = res["out"]
    return h, results


# --------------------------------------------------------------------------
# FFN-MoE with the routing decision of the preceding RoM layer (appendix, Eq. (14), (15))
# --------------------------------------------------------------------------
def swiglu_expert(x, w_gate_up, w_down):
    """f(x) = W_down (SiLU(W_gate x) * (W_up x)) for one feed-forward SwiGLU expert.
    x [n, D_m]; w_gate_up [2*D_f, D_m] (rows [0, D_f) gate, rows [D_f, 2*D_f) up); w_down [D_m, D_f]."""
    x = np.asarray(x, F64)
    w_gate_up = np.asarray(w_gate_up, F64)
    d_f = w_gate_up.shape[0] // 2
    h = x @ w_gate_up.T
    return (silu(h[:, :d_f]) * h[:, d_f:]) @ np.asarray(w_down, F64).T


def ffn_moe_forward(x, w_gate_up, w_down, idx, gate, norm_w=None, eps=1e-5, skip=False):
    """Y[n] = sum_i R_i[n] * 1[i in TopK[n]] * f_i(X[n])   (Eq. (14), (15)): no router of its own,
    the experts idx [N, K] and weights gate [N, K] are those of the RoM layer in front of it.
    x [N, D_m]; w_gate_up [E, 2*D_f, D_m]; w_down [E, D_m, D_f].
    norm_w: the experts see RMSNorm(x) (pre-norm); skip: x is added to the result."""
    x = np.asarray(x, F64)
    xin = x if norm_w is None else rms_norm(x, norm_w, eps)
    idx = np.asarray(idx)
    gate = np.asarray(gate, F64)
    n_exp = np.asarray(w_gate_up).shape[0]
    y = np.zeros_like(x)
    for k in range(idx.shape[1]):
        for i in range(n_exp):
            rows = np.nonzero(idx[:, k] == i)[0]
            if rows.size:
                y[rows] += gate[rows, k:k + 1] * swiglu_expert(xin[rows], w_gate_up[i], w_down[i])
    return x + y if skip else y


# --------------------------------------------------------------------------
# Backward pass of the layer (training, Sec. 5.1): the gradient of a scalar loss with respect to
# the layer input and every parameter, given d loss / d out.  Plain reverse-mode differentiation
# of the equations above, stage by stage in reverse order.  Readings:
#   * the TopK indicator of Eq. (9) is piecewise constant: it gets no gradient; the router is
#     trained through the gate weights R_i = P_i of Eq. (12) only (straight-through selection,
#     no jitter and no SparseMixer estimator, which the paper mentions as training options only);
#   * gate_mode 1 differentiates the renormalisation over the selected K as well;
#   * initial conv / scan states are constants (no gradient flows into a previous call).
# --------------------------------------------------------------------------
def gate_weights_backward(logits, idx, gate_mode, d_gate):
    """d loss / d logits [N, E] from d loss / d gate [N, K] (Eq. (9): gate = softmax prob of the
    selected experts, mode 1: divided by their sum)."""
    p = softmax(logits)
    idx64 = np.asarray(idx, np.int64)
    d_gate = np.asarray(d_gate, F64)
    sel = np.take_along_axis(p, idx64, axis=1)                   # P of the selected experts
    if gate_mode == 1:
        s = sel.sum(axis=1, keepdims=True)
        gate = sel / s
        d_sel = (d_gate - (d_gate * gate).sum(axis=1, keepdims=True)) / s
    else:
        d_sel = d_gate
    d_p = np.zeros_like(p)
    np.put_along_axis(d_p, idx64, d_sel, axis=1)                 # K distinct experts per token
    # softmax: dl_e = P_e (dP_e - sum_j P_j dP_j)
    return p * (d_p - (p * d_p).sum(axis=1, keepdims=True))


def routed_linear_backward(inp, w, idx, d_out):
    """Backward of routed_linear: returns (d_inp [N, D_in], d_w [E, D_out, D_in])."""
    inp = np.asarray(inp, F64)
    d_out = np.asarray(d_out, F64)
    n_exp = w.shape[0]
    d_w = np.zeros(w.shape, F64)
    if n_exp == 1:
        return d_out @ np.asarray(w[0], F64), (d_out.T @ inp)[None]
    d_inp = np.zeros_like(inp)
    for i in range(n_exp):
        rows = np.nonzero((idx == i).any(axis=1))[0]
        if rows.size:
            d_inp[rows] += d_out[rows] @ np.asarray(w[i], F64)
            d_w[i] = d_out[rows].T @ inp[rows]
    return d_inp, d_w


def silu_grad(v):
    s = 1.0 / (1.0 + np.exp(-v))
    return s * (1.0 + v * (1.0 - s))


def causal_conv_silu_backward(h, conv_w, conv_b, d_u, conv_state=None):
    """Backward of causal_conv_silu: returns (d_h [B, L, D_e], d_conv_w [D_e, k], d_conv_b [D_e])."""
    h = np.asarray(h, F64)
    bsz, length, d_e = h.shape
    k = conv_w.shape[1]
    cw = np.asarray(conv_w, F64)
    hist = (np.zeros((bsz, k - 1, d_e), F64) if conv_state is None
            else np.asarray(conv_state, F64).transpose(0, 2, 1))
    ext = np.concatenate([hist, h], axis=1)
    c = np.zeros((bsz, length, d_e), F64)
    if conv_b is not None:
        c += np.asarray(conv_b, F64)[None, None, :]
    for j in range(k):
        c += cw[None, None, :, j] * ext[:, j:j + length, :]
    d_c = np.asarray(d_u, F64) * silu_grad(c)
    d_ext = np.zeros_like(ext)
    d_w = np.zeros_like(cw)
    for j in range(k):
        d_ext[:, j:j + length, :] += cw[None, None, :, j] * d_c
        d_w[:, j] = (d_c * ext[:, j:j + length, :]).sum(axis=(0, 1))
    return d_ext[:, k - 1:, :], d_w, d_c.sum(axis=(0, 1))


def selective_scan_backward(u, dt, b_mat, c_mat, a, d_skip, d_y, h0=None):
    """Backward of selective_scan (Eq. (5)): the forward recurrence is run once more keeping every
    state, then the adjoint recurrence d_h[t-1] = exp(dt_t a) d_h[t] runs backwards in time.
    Returns dict: d_u, d_dt [B, L, D_e]; d_b, d_c [B, L, D_s]; d_a [D_e, D_s]; d_d [D_e]."""
    u = np.asarray(u, F64)
    dt = np.asarray(dt, F64)
    b_mat = np.asarray(b_mat, F64)
    c_mat = np.asarray(c_mat, F64)
    a = np.asarray(a, F64)
    d_skip = np.asarray(d_skip, F64)
    d_y = np.asarray(d_y, F64)
    bsz, length, d_e = u.shape
    d_s = a.shape[1]
    h = (np.zeros((bsz, d_e, d_s), F64) if h0 is None else np.array(h0, F64, copy=True))
    states = np.empty((length + 1, bsz, d_e, d_s), F64)
    states[0] = h
    for t in range(length):
        decay = np.exp(dt[:, t, :, None] * a[None, :, :])
        h = decay * h + (dt[:, t, :] * u[:, t, :])[:, :, None] * b_mat[:, t, None, :]
        states[t + 1] = h
    d_u = d_skip[None, None, :] * d_y
    d_dt = np.zeros_like(dt)
    d_b = np.zeros_like(b_mat)
    d_c = np.zeros_like(c_mat)
    d_a = np.zeros_like(a)
    d_d = (d_y * u).sum(axis=(0, 1))
    d_h = np.zeros((bsz, d_e, d_s), F64)
    for t in range(length - 1, -1, -1):
        d_c[:, t, :] = (d_y[:, t, :, None] * states[t + 1]).sum(axis=1)
        d_h = d_h + d_y[:, t, :, None] * c_mat[:, t, None, :]          # y_t = C_t . h_t
        decay = np.exp(dt[:, t, :, None] * a[None, :, :])
        d_decay_arg = d_h * states[t] * decay                          # d / d (dt_t * a)
        d_dt[:, t, :] += (d_decay_arg * a[None, :, :]).sum(axis=2)
        d_a += (d_decay_arg * dt[:, t, :, None]).sum(axis=0)
        inj = d_h * b_mat[:, t, None, :]                               # input term dt * B * u
        d_dt[:, t, :] += inj.sum(axis=2) * u[:, t, :]
        d_u[:, t, :] += inj.sum(axis=2) * dt[:, t, :]
        d_b[:, t, :] = (d_h * (dt[:, t, :] * u[:, t, :])[:, :, None]).sum(axis=1)
        d_h = d_h * decay                                              # adjoint of h_{t-1}
    return {"d_u": d_u, "d_dt": d_dt, "d_b": d_b, "d_c": d_c, "d_a": d_a, "d_d": d_d, "d_h0": d_h}


def rom_layer_backward(x, w, top_k, gate_mode, d_out, expert_idx=None, d_gate_extra=None):
    """Gradients of the layer of rom_layer_forward (zero initial states).  d_gate_extra [N, K]: a
    gradient with respect to the gate weights that arrives from outside the layer (an FFN-MoE layer
    running on this layer's routing decision, Eq. (15)); it joins the layer's own before the router.

    x [B, L, D_m], d_out [B, L, D_m].  Returns a dict with d_x [B, L, D_m], one d_<name> per
    parameter of `w` (same shapes; d_A_log is with respect to A_log, A = -exp(A_log)), and the
    intermediate gradients d_g, d_dt (w.r.t. the softplus output), d_u, d_xz, d_gate, d_logits.
    """
    fwd = rom_layer_forward(x, w, top_k, gate_mode, expert_idx=expert_idx)
    x = np.asarray(x, F64)
    bsz, length, d_m = x.shape
    n_tok = bsz * length
    xt = x.reshape(n_tok, d_m)
    idx, gate = fwd["expert_idx"], fwd["gate"]
    d_e = w["w_out"].shape[2]
    d_s = w["A_log"].shape[1]
    r = w["w_dt"].shape[2]
    d_o = np.asarray(d_out, F64).reshape(n_tok, d_m)
    g, xz, ut, xdbl = fwd["g"], fwd["xz"], fwd["u"], fwd["xdbl"]
    z = xz[:, d_e:]

    # Eq. (12)/(13): out = sum_k gate_k * (g W_out[e_k]^T)
    d_g = np.zeros((n_tok, d_e), F64)
    d_gate = np.zeros((n_tok, top_k), F64)
    d_w_out = np.zeros(w["w_out"].shape, F64)
    for k in range(top_k):
        col = idx[:, k:k + 1]
        d_gate[:, k] = (d_o * routed_linear(g, w["w_out"], col)).sum(axis=1)
        d_gk, d_wk = routed_linear_backward(g, w["w_out"], col, gate[:, k:k + 1] * d_o)
        d_g += d_gk
        d_w_out += d_wk
    # Eq. (6)/(10): g = y * SiLU(z)
    d_y = d_g * silu(z)
    d_z = d_g * fwd["y"] * silu_grad(z)
    # Eq. (5)
    a = -np.exp(np.asarray(w["A_log"], F64))
    dt = fwd["dt"]
    sc = selective_scan_backward(ut.reshape(bsz, length, d_e), dt.reshape(bsz, length, d_e),
                                 xdbl[:, r:r + d_s].reshape(bsz, length, d_s),
                                 xdbl[:, r + d_s:].reshape(bsz, length, d_s), a, w["D"],
                                 d_y.reshape(bsz, length, d_e))
    d_dt = sc["d_dt"].reshape(n_tok, d_e)
    # dt = softplus(pre): d pre = d dt * sigmoid(pre) = d dt * (1 - exp(-dt))
    d_pre = d_dt * (1.0 - np.exp(-dt))
    d_dt_low, d_w_dt = routed_linear_backward(xdbl[:, :r], w["w_dt"], idx, d_pre)
    d_xdbl = np.concatenate([d_dt_low, sc["d_b"].reshape(n_tok, d_s), sc["d_c"].reshape(n_tok, d_s)], axis=1)
    d_u_x, d_w_x = routed_linear_backward(ut, w["w_x"], idx, d_xdbl)
    d_u = sc["d_u"].reshape(n_tok, d_e) + d_u_x
    # Eq. (2)
    d_h_pre, d_conv_w, d_conv_b = causal_conv_silu_backward(
        xz[:, :d_e].reshape(bsz, length, d_e), w["conv_w"], w.get("conv_b"), d_u.reshape(bsz, length, d_e))
    d_xz = np.concatenate([d_h_pre.reshape(n_tok, d_e), d_z], axis=1)
    # Eq. (10)/(11)
    d_x, d_w_in = routed_linear_backward(xt, w["w_in"], idx, d_xz)
    # Eq. (9): the gates
    if d_gate_extra is not None:
        d_gate = d_gate + np.asarray(d_gate_extra, F64)
    d_logits = gate_weights_backward(fwd["logits"], idx, gate_mode, d_gate)
    d_x = d_x + d_logits @ np.asarray(w["w_router"], F64)
    return {
        "d_x": d_x.reshape(bsz, length, d_m), "d_w_router": d_logits.T @ xt, "d_b_router": d_logits.sum(axis=0),
        "d_w_in": d_w_in, "d_conv_w": d_conv_w, "d_conv_b": d_conv_b, "d_w_x": d_w_x, "d_w_dt": d_w_dt,
        "d_dt_bias": d_pre.sum(axis=0), "d_A_log": sc["d_a"] * a, "d_D": sc["d_d"], "d_w_out": d_w_out,
        "d_g": d_g, "d_y": d_y, "d_z": d_z, "d_dt": d_dt, "d_pre": d_pre, "d_u": d_u, "d_u_scan": sc["d_u"].reshape(n_tok, d_e),
        "d_xdbl": d_xdbl, "d_xz": d_xz, "d_gate": d_gate, "d_logits": d_logits, "fwd": fwd,
    }


def rms_norm_backward(x, weight, eps, d_y):
    """Adjoint of rms_norm: y = x / sqrt(mean(x^2) + eps) * weight.  With r = 1 / sqrt(mean(x^2) + eps)
    and x^ = x r:  d_weight = sum over rows of d_y x^;  d_x = r (d_y weight - x^ mean_d(d_y weight x^)).
    Returns (d_x, d_weight)."""
    x = np.asarray(x, F64)
    d_y = np.asarray(d_y, F64)
    wgt = np.asarray(weight, F64)
    r = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    xh = x * r
    d_weight = (d_y * xh).reshape(-1, x.shape[-1]).sum(axis=0)
    d_xh = d_y * wgt
    d_x = r * (d_xh - xh * np.mean(d_xh * xh, axis=-1, keepdims=True))
    return d_x, d_weight


def rom_block_backward(x, w, top_k, gate_mode, d_out, eps=1e-5, expert_idx=None, d_gate_extra=None):
    """Gradients of rom_block_forward (zero initial states): the layer's backward on the normalised
    input, the norm's adjoint, and the skip connection's d_out added to d_x.  Returns the dict of
    rom_layer_backward with d_x the block's input gradient and d_norm_w [D_m] added."""
    x = np.asarray(x, F64)
    xn = rms_norm(x, w["norm_w"], eps)
    res = rom_layer_backward(xn, w, top_k, gate_mode, d_out, expert_idx, d_gate_extra)
    d_x_norm, d_norm_w = rms_norm_backward(x, w["norm_w"], eps, res["d_x"])
    res["d_xn"] = res["d_x"]
    res["d_x"] = np.asarray(d_out, F64) + d_x_norm
    res["d_norm_w"] = d_norm_w
    return res


def ffn_moe_backward(x, w_gate_up, w_down, idx, gate, d_out, norm_w=None, eps=1e-5, skip=False):
    """Gradients of ffn_moe_forward for d loss / d y = d_out [N, D_m], slot by slot:
        h = W_gu,i x~,  a = SiLU(h_gate) * h_up,  o = W_down,i a,  y += gate * o
    Returns d_x [N, D_m], d_w_gate_up [E, 2 D_f, D_m] (plain row order), d_w_down [E, D_m, D_f],
    d_gate [N, K] (to be added to the gate gradient of the RoM layer that made the routing decision)
    and, with a pre-norm, d_norm_w [D_m]."""
    x = np.asarray(x, F64)
    d_out = np.asarray(d_out, F64)
    xin = x if norm_w is None else rms_norm(x, norm_w, eps)
    idx = np.asarray(idx)
    gate = np.asarray(gate, F64)
    w_gate_up = np.asarray(w_gate_up, F64)
    w_down = np.asarray(w_down, F64)
    n_exp, d_f = w_gate_up.shape[0], w_gate_up.shape[1] // 2
    d_xin = np.zeros_like(x)
    d_wgu = np.zeros_like(w_gate_up)
    d_wd = np.zeros_like(w_down)
    d_gate = np.zeros_like(gate)
    for k in range(idx.shape[1]):
        for i in range(n_exp):
            rows = np.nonzero(idx[:, k] == i)[0]
            if not rows.size:
                continue
            h = xin[rows] @ w_gate_up[i].T
            hg, hu = h[:, :d_f], h[:, d_f:]
            sig = 1.0 / (1.0 + np.exp(-hg))
            a = hg * sig * hu
            d_gate[rows, k] = (d_out[rows] * (a @ w_down[i].T)).sum(axis=1)
            d_o = gate[rows, k:k + 1] * d_out[rows]
            d_wd[i] += d_o.T @ a
            d_a = d_o @ w_down[i]
            d_h = np.concatenate([d_a * hu * sig * (1.0 + hg * (1.0 - sig)), d_a * hg * sig], axis=1)
            d_wgu[i] += d_h.T @ xin[rows]
            d_xin[rows] += d_h @ w_gate_up[i]
    res = {"d_w_gate_up": d_wgu, "d_w_down": d_wd, "d_gate": d_gate}
    if norm_w is None:
        d_x = d_xin
    else:
        d_x, res["d_norm_w"] = rms_norm_backward(x, norm_w, eps, d_xin)
    res["d_x"] = d_x + d_out if skip else d_x
    return res
