"""Pins of the Mamba2-variant oracle (oracle/rom_mamba2_oracle.py) against things other than itself:
the pinned Mamba scan it reduces to, the explicit double sum of the dual form, closed forms, hand
values, and a dense Mamba2 layer assembled from library routines.  CPU only."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import rom_synth as S
from oracle import rom_mamba2_oracle as M
from oracle import rom_oracle as O


def _rand_scan(seed, bsz=2, length=9, n_heads=3, p_dim=4, n_state=5):
    r = np.random.default_rng(seed)
    x = r.standard_normal((bsz, length, n_heads, p_dim))
    dt = r.uniform(0.01, 0.6, (bsz, length, n_heads))
    a = -r.uniform(0.5, 4.0, n_heads)
    b = r.standard_normal((bsz, length, n_state))
    c = r.standard_normal((bsz, length, n_state))
    d = r.standard_normal(n_heads)
    return x, dt, a, b, c, d


def test_ssd_scan_reduces_to_the_mamba_scan_with_per_head_dt_and_a():
    """Every channel of a head sharing dt and A (constant over the states) is a special case of the
    Mamba recurrence of Eq. (5), whose oracle is pinned on its own."""
    x, dt, a, b, c, d = _rand_scan(1)
    bsz, length, n_heads, p_dim = x.shape
    n_state = b.shape[2]
    h0 = np.random.default_rng(2).standard_normal((bsz, n_heads, p_dim, n_state))
    y, state = M.ssd_scan(x, dt, a, b, c, d, h0)
    u = x.reshape(bsz, length, n_heads * p_dim)
    dt_ch = np.repeat(dt, p_dim, axis=2)
    a_ch = np.repeat(a, p_dim)[:, None] * np.ones((1, n_state))
    d_ch = np.repeat(d, p_dim)
    y_ref, h_ref = O.selective_scan(u, dt_ch, b, c, a_ch, d_ch, h0.reshape(bsz, n_heads * p_dim, n_state))
    np.testing.assert_allclose(y.reshape(bsz, length, -1), y_ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(state.reshape(bsz, -1, n_state), h_ref, rtol=1e-12, atol=1e-13)


def test_ssd_scan_matches_the_dual_double_sum():
    """y_t = sum_{s <= t} (C_t . B_s) exp(a sum_{r = s+1..t} dt_r) dt_s x_s + D x_t, loop by loop."""
    x, dt, a, b, c, d = _rand_scan(3, bsz=1, length=7, n_heads=2, p_dim=3, n_state=4)
    y, _ = M.ssd_scan(x, dt, a, b, c, d)
    for h in range(2):
        for t in range(7):
            acc = d[h] * x[0, t, h].copy()
            for s in range(t + 1):
                log_decay = a[h] * sum(dt[0, r, h] for r in range(s + 1, t + 1))
                acc += float(np.dot(c[0, t], b[0, s])) * np.exp(log_decay) * dt[0, s, h] * x[0, s, h]
            np.testing.assert_allclose(y[0, t, h], acc, rtol=1e-12, atol=1e-13)


def test_ssd_scan_constant_coefficients_is_a_geometric_series():
    length, dt0, a0, d0 = 12, 0.25, -1.5, 0.75
    x = np.ones((1, length, 1, 2))
    x[..., 1] = -2.0
    dt = np.full((1, length, 1), dt0)
    e0 = np.zeros((1, length, 3))
    e0[:, :, 1] = 1.0
    y, state = M.ssd_scan(x, dt, np.array([a0]), e0, 3.0 * e0, np.array([d0]))
    q = np.exp(dt0 * a0)
    for t in range(length):
        series = dt0 * (1.0 - q ** (t + 1)) / (1.0 - q)
        np.testing.assert_allclose(y[0, t, 0], np.array([1.0, -2.0]) * (3.0 * series + d0), rtol=1e-12)
    # only state column 1 is ever fed
    assert np.all(state[0, 0, :, 0] == 0.0) and np.all(state[0, 0, :, 2] == 0.0)
    np.testing.assert_allclose(state[0, 0, :, 1], np.array([1.0, -2.0]) * dt0 * (1 - q ** length) / (1 - q), rtol=1e-12)


def test_ssd_scan_state_carry_equals_unsplit():
    x, dt, a, b, c, d = _rand_scan(4, length=10)
    y, state = M.ssd_scan(x, dt, a, b, c, d)
    y1, s1 = M.ssd_scan(x[:, :4], dt[:, :4], a, b[:, :4], c[:, :4], d)
    y2, s2 = M.ssd_scan(x[:, 4:], dt[:, 4:], a, b[:, 4:], c[:, 4:], d, s1)
    np.testing.assert_allclose(np.concatenate([y1, y2], axis=1), y, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(s2, state, rtol=1e-12, atol=1e-13)


def test_gated_rms_norm_hand_values_and_library():
    # z0 with SiLU(z0) = z0 / (1 + exp(-z0)) = 1 (bisection on that formula): the gate passes y unchanged
    lo, hi = 1.0, 2.0
    for _ in range(80):
        mid = 0.5 * (lo + hi)
        lo, hi = (mid, hi) if mid / (1.0 + np.exp(-mid)) < 1.0 else (lo, mid)
    y = np.array([[3.0, -4.0]])
    one = np.full((1, 2), lo)
    np.testing.assert_allclose(M.gated_rms_norm(y, one, np.array([2.0, 0.5]), 0.0),
                               [[2.0 * 3.0 / np.sqrt(12.5), 0.5 * -4.0 / np.sqrt(12.5)]], rtol=1e-12)
    # eps sits inside the root: mean square 12.5, eps 3.5 -> divide by 4
    np.testing.assert_allclose(M.gated_rms_norm(y, one, np.ones(2), 3.5), [[0.75, -1.0]], rtol=1e-12)
    # the gate acts before the norm: gating only the first channel by SiLU(0) = 0 leaves mean square 8
    np.testing.assert_allclose(M.gated_rms_norm(y, np.array([[0.0, lo]]), np.ones(2), 0.0), [[0.0, -4.0 / np.sqrt(8.0)]],
                               rtol=1e-12)
    assert np.all(M.gated_rms_norm(y, np.zeros((1, 2)), np.ones(2), 1e-5) == 0.0)
    r = np.random.default_rng(5)
    yv, zv, wn = r.standard_normal((6, 32)), r.standard_normal((6, 32)), r.uniform(0.5, 1.5, 32)
    ref = F.rms_norm(torch.from_numpy(yv) * F.silu(torch.from_numpy(zv)), (32,), torch.from_numpy(wn), eps=1e-5)
    np.testing.assert_allclose(M.gated_rms_norm(yv, zv, wn, 1e-5), ref.numpy(), rtol=1e-12, atol=1e-13)
    # the gate is inside the norm: gating after the norm gives something else
    assert not np.allclose(M.gated_rms_norm(yv, zv, wn, 1e-5), O.rms_norm(yv, wn, 1e-5) * O.silu(zv))


def _dense_mamba2_library(x, w_in, w, w_out, cfg):
    """A dense Mamba2 layer from torch routines: linear, conv1d, a cumulative-sum form of the scan
    (per head: the attention-like matrix with the decay mask), rms_norm, linear."""
    xt = torch.from_numpy(np.asarray(x, np.float64))
    bsz, length, _ = xt.shape
    d_e, n_state, n_heads, p_dim = cfg.d_inner, cfg.d_state, cfg.n_heads, cfg.headdim
    zxbcdt = F.linear(xt, torch.from_numpy(w_in).double())
    z, xbc, dt_raw = torch.split(zxbcdt, [d_e, d_e + 2 * n_state, n_heads], dim=-1)
    conv = F.conv1d(xbc.transpose(1, 2), torch.from_numpy(w["conv_w"]).double()[:, None, :],
                    torch.from_numpy(w["conv_b"]).double(), padding=cfg.d_conv - 1, groups=cfg.d_conv_ch)
    xbc = F.silu(conv[:, :, :length].transpose(1, 2))
    xs, b_mat, c_mat = torch.split(xbc, [d_e, n_state, n_state], dim=-1)
    xs = xs.reshape(bsz, length, n_heads, p_dim)
    dt = F.softplus(dt_raw + torch.from_numpy(w["dt_bias"]).double())
    a = -torch.exp(torch.from_numpy(w["A_log"]).double())
    cum = torch.cumsum(dt * a, dim=1)                                         # [B, L, H]
    seg = cum[:, :, None, :] - cum[:, None, :, :]                             # [B, t, s, H]
    causal = torch.tril(torch.ones(length, length, dtype=torch.bool))
    decay = torch.where(causal[None, :, :, None], torch.exp(torch.where(causal[None, :, :, None], seg, torch.zeros_like(seg))),
                        torch.zeros_like(seg))
    scores = torch.einsum("btn,bsn->bts", c_mat, b_mat)[:, :, :, None] * decay * dt[:, None, :, :]
    y = torch.einsum("btsh,bshp->bthp", scores, xs) + torch.from_numpy(w["D"]).double()[None, None, :, None] * xs
    g = F.rms_norm(y.reshape(bsz, length, d_e) * F.silu(z), (d_e,), torch.from_numpy(w["norm_w"]).double(), eps=1e-5)
    return F.linear(g, torch.from_numpy(w_out).double()).numpy()


def _tiny_cfg(**kw):
    base = dict(batch=2, seq_len=11, d_model=24, d_inner=32, d_state=6, headdim=8, n_experts=3, top_k=1,
                gate_mode=0, dtype="fp32", weight_std=0.3)
    base.update(kw)
    return S.Mamba2Config("tiny", 30, **base)


def test_single_expert_is_the_dense_mamba2_layer():
    cfg = _tiny_cfg(n_experts=1)
    w = S.make_mamba2_weights(cfg)
    x = S.make_mamba2_input(cfg)
    res = M.rom_mamba2_forward(x, w, 1, 0, cfg.headdim)
    ref = _dense_mamba2_library(x, w["w_in"][0], w, w["w_out"][0], cfg)
    # one expert: its softmax gate is 1
    np.testing.assert_allclose(res["gate"], 1.0, rtol=0, atol=0)
    np.testing.assert_allclose(res["out"], ref, rtol=1e-9, atol=1e-11)


@pytest.mark.parametrize("top_k,gate_mode", [(1, 0), (2, 1), (3, 0)])
def test_layer_is_the_dense_layer_with_per_token_mixed_projections(top_k, gate_mode):
    """Brute force over the experts: the routed input projection of a token is the plain sum of its
    chosen experts' projections, the output is the gate-weighted sum of their output projections;
    everything between is the dense layer's.  Assembled here token by token."""
    cfg = _tiny_cfg(top_k=top_k, gate_mode=gate_mode, seq_len=7, batch=1)
    w = S.make_mamba2_weights(cfg)
    x = S.make_mamba2_input(cfg).astype(np.float64)
    res = M.rom_mamba2_forward(x, w, top_k, gate_mode, cfg.headdim)
    xt = x.reshape(-1, cfg.d_model)
    logits = xt @ w["w_router"].astype(np.float64).T
    order = np.argsort(-logits, axis=1, kind="stable")[:, :top_k]
    assert np.array_equal(np.sort(order, axis=1), np.sort(res["expert_idx"], axis=1))
    prob = np.exp(logits - logits.max(axis=1, keepdims=True))
    prob /= prob.sum(axis=1, keepdims=True)
    # per-token mixed input projection, then the dense pipeline with an identity "output projection"
    w_in_tok = np.stack([sum(w["w_in"][e].astype(np.float64) for e in order[n]) for n in range(xt.shape[0])])
    zxbcdt = np.einsum("nd,nod->no", xt, w_in_tok)
    d_e, n_state, n_heads = cfg.d_inner, cfg.d_state, cfg.n_heads
    np.testing.assert_allclose(res["zxbcdt"], zxbcdt, rtol=1e-10, atol=1e-12)
    # the middle of the layer on these projections: reuse the library form with w_in = identity on zxbcdt
    eye_cfg = S.Mamba2Config("eye", 31, 1, cfg.seq_len, cfg.d_in_proj, d_e, n_state, cfg.headdim, 1, 1, 0, dtype="fp32")
    g = _dense_mamba2_library(zxbcdt[None], np.eye(cfg.d_in_proj), w, np.eye(d_e), eye_cfg)[0]
    np.testing.assert_allclose(res["g"], g, rtol=1e-9, atol=1e-11)
    out = np.zeros((xt.shape[0], cfg.d_model))
    for n in range(xt.shape[0]):
        sel = order[n]
        wts = prob[n, sel] / (prob[n, sel].sum() if gate_mode == 1 else 1.0)
        for e, wt in zip(sel, wts):
            out[n] += wt * (w["w_out"][e].astype(np.float64) @ g[n])
    np.testing.assert_allclose(res["out"][0], out, rtol=1e-9, atol=1e-11)


def test_layer_is_causal_and_sequences_are_independent():
    cfg = _tiny_cfg(top_k=2, gate_mode=1)
    w = S.make_mamba2_weights(cfg)
    x = S.make_mamba2_input(cfg).astype(np.float64)
    base = M.rom_mamba2_forward(x, w, 2, 1, cfg.headdim)["out"]
    x2 = x.copy()
    x2[0, 6:] += 1.0
    moved = M.rom_mamba2_forward(x2, w, 2, 1, cfg.headdim)["out"]
    np.testing.assert_array_equal(moved[0, :6], base[0, :6])
    np.testing.assert_array_equal(moved[1], base[1])
    assert np.abs(moved[0, 6:] - base[0, 6:]).max() > 1e-3


def test_layer_state_carry_and_step_equal_the_unsplit_run():
    """A sequence fed in two calls, or token by token through the step, gives what one call gives:
    pins the state arguments (conv history order, state layout) to the stateless layer."""
    cfg = _tiny_cfg(top_k=2, gate_mode=1, seq_len=9)
    w = S.make_mamba2_weights(cfg)
    x = S.make_mamba2_input(cfg).astype(np.float64)
    whole = M.rom_mamba2_forward(x, w, 2, 1, cfg.headdim)
    first = M.rom_mamba2_forward(x[:, :4], w, 2, 1, cfg.headdim)
    second = M.rom_mamba2_forward(x[:, 4:], w, 2, 1, cfg.headdim, conv_state=first["conv_state"],
                                  ssm_state=first["ssm_state"])
    np.testing.assert_allclose(np.concatenate([first["out"], second["out"]], axis=1), whole["out"], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(second["ssm_state"], whole["ssm_state"], rtol=1e-10, atol=1e-12)
    np.testing.assert_array_equal(second["conv_state"], whole["conv_state"])
    # the conv state is the last three inputs of the conv, oldest first
    xbc_pre = whole["zxbcdt"][:, cfg.d_inner:2 * cfg.d_inner + 2 * cfg.d_state].reshape(cfg.batch, cfg.seq_len, -1)
    np.testing.assert_array_equal(whole["conv_state"], xbc_pre[:, -3:, :].transpose(0, 2, 1))
    cs = np.zeros((cfg.batch, cfg.d_conv_ch, cfg.d_conv - 1))
    ss = np.zeros((cfg.batch, cfg.n_heads, cfg.headdim, cfg.d_state))
    for t in range(cfg.seq_len):
        res = M.rom_mamba2_step(x[:, t], w, 2, 1, cfg.headdim, cs, ss)
        cs, ss = res["conv_state"], res["ssm_state"]
        np.testing.assert_allclose(res["out"], whole["out"][:, t], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(ss, whole["ssm_state"], rtol=1e-10, atol=1e-12)


def test_mamba2_synth_shapes():
    cfg = S.get_mamba2_config("m2_cfg2")
    assert (cfg.n_heads, cfg.d_in_proj, cfg.d_conv_ch) == (64, 8512, 4352)
    small = S.get_mamba2_config("m2_small")
    w = S.make_mamba2_weights(small)
    assert w["w_in"].shape == (4, small.d_in_proj, 256) and w["conv_w"].shape == (small.d_conv_ch, 4)
    assert w["A_log"].shape == (small.n_heads,) and w["norm_w"].shape == (small.d_inner,)
    assert np.array_equal(S.round_to_bf16(w["w_in"]), w["w_in"])
    assert S.make_mamba2_input(small).shape == (2, 200, 256)
