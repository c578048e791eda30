"""Pins of the Gated-DeltaNet-variant oracle (oracle/rom_gdn_oracle.py) against things other than
itself: explicit products of transition matrices, the linear system the chunk form solves, the
delta rule's textbook properties, and a dense layer assembled separately.  CPU only."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import rom_synth as S
from oracle import rom_gdn_oracle as G
from oracle import rom_mamba2_oracle as M2


def _rand(seed, bsz=2, length=8, n_heads=2, d_k=5, d_v=4):
    r = np.random.default_rng(seed)
    q = r.standard_normal((bsz, length, n_heads, d_k))
    k = r.standard_normal((bsz, length, n_heads, d_k))
    k /= np.linalg.norm(k, axis=-1, keepdims=True)
    v = r.standard_normal((bsz, length, n_heads, d_v))
    beta = r.uniform(0.1, 0.9, (bsz, length, n_heads))
    g = -r.uniform(0.01, 1.0, (bsz, length, n_heads))
    return q, k, v, beta, g


def test_scan_matches_products_of_transition_matrices():
    """S_t = sum_i beta_i v_i k_i^T prod_{j = i+1..t} alpha_j (I - beta_j k_j k_j^T) (+ S_0 prod ...),
    with the matrix products written out."""
    q, k, v, beta, g = _rand(1, bsz=1, length=6, n_heads=1)
    s0 = np.random.default_rng(2).standard_normal((1, 1, 4, 5))
    o, s_fin = G.gated_delta_scan(q, k, v, beta, g, s0)
    eye = np.eye(5)
    for t in range(6):
        def trans(j):
            kj = k[0, j, 0]
            return np.exp(g[0, j, 0]) * (eye - beta[0, j, 0] * np.outer(kj, kj))
        s_t = s0[0, 0].copy()
        for j in range(t + 1):
            s_t = s_t @ trans(j)
        for i in range(t + 1):
            term = beta[0, i, 0] * np.outer(v[0, i, 0], k[0, i, 0])
            for j in range(i + 1, t + 1):
                term = term @ trans(j)
            s_t += term
        np.testing.assert_allclose(o[0, t, 0], s_t @ q[0, t, 0], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(s_fin[0, 0], s_t, rtol=1e-11, atol=1e-12)


def test_scan_solves_the_chunk_linear_system():
    """Inside a chunk the updates u_t obey (I + A) U = diag(beta) V - diag(beta gamma) K S_0^T with
    A[t][s] = beta_t (gamma_t / gamma_s) (k_t . k_s) for s < t and gamma the cumulative decay; outputs
    and the end state follow from U.  Solved here with a library solver."""
    q, k, v, beta, g = _rand(3, bsz=1, length=7, n_heads=1)
    s0 = np.random.default_rng(4).standard_normal((1, 1, 4, 5))
    o, s_fin = G.gated_delta_scan(q, k, v, beta, g, s0)
    kk, vv, qq, bb = k[0, :, 0], v[0, :, 0], q[0, :, 0], beta[0, :, 0]
    cum = np.cumsum(g[0, :, 0])
    gamma = np.exp(cum)
    ratio = np.exp(cum[:, None] - cum[None, :])
    a_mat = np.tril(bb[:, None] * ratio * (kk @ kk.T), -1)
    rhs = bb[:, None] * vv - (bb * gamma)[:, None] * (kk @ s0[0, 0].T)
    u = np.linalg.solve(np.eye(7) + a_mat, rhs)
    o_ref = gamma[:, None] * (qq @ s0[0, 0].T) + np.tril(ratio * (qq @ kk.T)) @ u
    np.testing.assert_allclose(o[0, :, 0], o_ref, rtol=1e-10, atol=1e-12)
    s_ref = gamma[-1] * s0[0, 0] + (u * np.exp(cum[-1] - cum)[:, None]).T @ kk
    np.testing.assert_allclose(s_fin[0, 0], s_ref, rtol=1e-10, atol=1e-12)


def test_delta_rule_recalls_exactly_with_orthonormal_keys():
    """beta = 1, no decay, orthonormal keys: writing (k_i, v_i) makes S k_i = v_i for every pair written,
    and rewriting a key replaces its value (the property that names the delta rule)."""
    d_k, d_v = 6, 3
    r = np.random.default_rng(5)
    keys, _ = np.linalg.qr(r.standard_normal((d_k, d_k)))
    vals = r.standard_normal((5, d_v))
    order = [0, 1, 2, 0, 3]                      # key 0 is written twice
    k = keys[order][None, :, None, :]
    v = vals[None, :, None, :]
    ones = np.ones((1, 5, 1))
    _, s_fin = G.gated_delta_scan(k, k, v, ones, 0.0 * ones)
    np.testing.assert_allclose(s_fin[0, 0] @ keys[1], vals[1], atol=1e-12)
    np.testing.assert_allclose(s_fin[0, 0] @ keys[2], vals[2], atol=1e-12)
    np.testing.assert_allclose(s_fin[0, 0] @ keys[3], vals[4], atol=1e-12)
    np.testing.assert_allclose(s_fin[0, 0] @ keys[0], vals[3], atol=1e-12)      # the second write won
    np.testing.assert_allclose(s_fin[0, 0] @ keys[4], 0.0, atol=1e-12)          # never written


def test_beta_zero_only_decays_and_linear_attention_limit():
    q, k, v, beta, g = _rand(6)
    s0 = np.random.default_rng(7).standard_normal((2, 2, 4, 5))
    o, s_fin = G.gated_delta_scan(q, k, v, 0.0 * beta, g, s0)
    total = np.exp(g.sum(axis=1))
    np.testing.assert_allclose(s_fin, total[:, :, None, None] * s0, rtol=1e-12)
    np.testing.assert_allclose(o[:, 0], np.einsum("bhvk,bhk->bhv", np.exp(g[:, 0])[:, :, None, None] * s0, q[:, 0]), rtol=1e-12)
    # mutually orthogonal keys never interfere: the rule reduces to decayed linear attention, which
    # is Mamba2's recurrence with dt = beta, B = k, C = q, x = v (per head; a = g / dt)
    d_k = 8
    keys, _ = np.linalg.qr(np.random.default_rng(8).standard_normal((d_k, d_k)))
    k2 = keys[:6][None, :, None, :]
    q2 = np.random.default_rng(9).standard_normal((1, 6, 1, d_k))
    v2 = np.random.default_rng(10).standard_normal((1, 6, 1, 3))
    b2 = np.full((1, 6, 1), 0.7)
    g2 = np.full((1, 6, 1), -0.7 * 0.4)
    o2, _ = G.gated_delta_scan(q2, k2, v2, b2, g2)
    y_ref, _ = M2.ssd_scan(v2, b2, np.array([-0.4]), k2[:, :, 0, :], q2[:, :, 0, :], np.zeros(1))
    np.testing.assert_allclose(o2, y_ref, rtol=1e-11, atol=1e-13)


def test_l2_and_head_norm_hand_values():
    np.testing.assert_allclose(G.l2_normalize(np.array([[3.0, 4.0]]), 0.0), [[0.6, 0.8]], rtol=1e-14)
    np.testing.assert_allclose(G.l2_normalize(np.array([[3.0, 4.0]]), 11.0), [[0.5, 4.0 / 6.0]], rtol=1e-14)
    # z0 with SiLU(z0) = 1 (bisection on z / (1 + exp(-z)) = 1)
    lo, hi = 1.0, 2.0
    for _ in range(80):
        mid = 0.5 * (lo + hi)
        lo, hi = (mid, hi) if mid / (1.0 + np.exp(-mid)) < 1.0 else (lo, mid)
    o = np.array([[[3.0, -4.0], [1.0, 1.0]]])                 # two heads of two channels
    z = np.full((1, 2, 2), lo)
    got = G.head_rms_norm_gated(o, z, np.array([2.0, 0.5]), 3.5)
    # head 0: mean square 12.5 + 3.5 -> / 4; head 1: mean square 1 + 3.5
    np.testing.assert_allclose(got[0, 0], [2.0 * 0.75, 0.5 * -1.0], rtol=1e-12)
    np.testing.assert_allclose(got[0, 1], [2.0 / np.sqrt(4.5), 0.5 / np.sqrt(4.5)], rtol=1e-12)
    # the gate acts after the norm: SiLU(0) = 0 on one channel leaves the other's value unchanged
    z[0, 0, 0] = 0.0
    got = G.head_rms_norm_gated(o, z, np.array([2.0, 0.5]), 3.5)
    np.testing.assert_allclose(got[0, 0], [0.0, -0.5], rtol=1e-12)


def _tiny_cfg(**kw):
    base = dict(batch=2, seq_len=9, d_model=24, n_heads=4, d_k=6, d_v=5, n_experts=3, top_k=1, gate_mode=0,
                dtype="fp32", weight_std=0.3)
    base.update(kw)
    return S.GdnConfig("tiny", 60, **base)


def _dense_gdn_torch(proj, w, cfg):
    """The layer between its two projections with torch routines: conv1d, normalize, sigmoid,
    softplus, and the recurrence as the solution of the whole sequence's linear system."""
    bsz, length, _ = proj.shape
    h, d_k, d_v, d_kt, d_vt = cfg.n_heads, cfg.d_k, cfg.d_v, cfg.d_kt, cfg.d_vt
    p = torch.from_numpy(proj)
    z, qkv, b_raw, a_raw = torch.split(p, [d_vt, 2 * d_kt + d_vt, h, h], dim=-1)
    conv = F.conv1d(qkv.transpose(1, 2), torch.from_numpy(w["conv_w"]).double()[:, None, :],
                    torch.from_numpy(w["conv_b"]).double(), padding=cfg.d_conv - 1, groups=cfg.d_conv_ch)
    qkv = F.silu(conv[:, :, :length].transpose(1, 2))
    q, k, v = torch.split(qkv, [d_kt, d_kt, d_vt], dim=-1)
    q = q.reshape(bsz, length, h, d_k)
    k = k.reshape(bsz, length, h, d_k)
    q = q / torch.sqrt((q * q).sum(-1, keepdim=True) + 1e-6) * d_k ** -0.5
    k = k / torch.sqrt((k * k).sum(-1, keepdim=True) + 1e-6)
    v = v.reshape(bsz, length, h, d_v)
    beta = torch.sigmoid(b_raw)
    g = -torch.exp(torch.from_numpy(w["A_log"]).double()) * F.softplus(a_raw + torch.from_numpy(w["dt_bias"]).double())
    cum = torch.cumsum(g, dim=1)                                              # [B, L, H]
    ratio = torch.exp(cum[:, :, None, :] - cum[:, None, :, :]).permute(0, 3, 1, 2)     # [B, H, t, s]
    kk = torch.einsum("bthd,bshd->bhts", k, k)
    a_mat = torch.tril(beta.permute(0, 2, 1)[:, :, :, None] * ratio * kk, -1)
    rhs = (beta[..., None] * v).permute(0, 2, 1, 3)                           # [B, H, L, d_v]
    u = torch.linalg.solve(torch.eye(length, dtype=torch.float64) + a_mat, rhs)
    qk = torch.einsum("bthd,bshd->bhts", q, k)
    o = (torch.tril(ratio * qk) @ u).permute(0, 2, 1, 3)                      # [B, L, H, d_v]
    o = F.rms_norm(o, (d_v,), torch.from_numpy(w["norm_w"]).double(), eps=1e-5)
    return (o * F.silu(z.reshape(bsz, length, h, d_v))).reshape(bsz, length, d_vt).numpy()


def test_single_expert_is_the_dense_layer():
    cfg = _tiny_cfg(n_experts=1)
    w = S.make_gdn_weights(cfg)
    x = S.make_gdn_input(cfg).astype(np.float64)
    res = G.rom_gdn_forward(x, w, 1, 0, cfg.n_heads, cfg.d_k)
    proj = x @ w["w_in"][0].astype(np.float64).T
    y = _dense_gdn_torch(proj, w, cfg)
    np.testing.assert_allclose(res["y"].reshape(y.shape), y, rtol=1e-8, atol=1e-10)
    np.testing.assert_allclose(res["out"], y @ w["w_out"][0].astype(np.float64).T, rtol=1e-8, atol=1e-10)
    assert np.all(res["beta"] > 0) and np.all(res["beta"] < 1) and np.all(res["g"] < 0)
    assert res["beta"].std() > 0.05          # the per-head logits leave the middle of the sigmoid


@pytest.mark.parametrize("top_k,gate_mode", [(1, 0), (2, 1), (3, 0)])
def test_layer_is_the_dense_layer_with_per_token_mixed_projections(top_k, gate_mode):
    cfg = _tiny_cfg(top_k=top_k, gate_mode=gate_mode, batch=1, seq_len=7)
    w = S.make_gdn_weights(cfg)
    x = S.make_gdn_input(cfg).astype(np.float64)
    res = G.rom_gdn_forward(x, w, top_k, gate_mode, cfg.n_heads, cfg.d_k)
    xt = x.reshape(-1, cfg.d_model)
    logits = xt @ w["w_router"].astype(np.float64).T
    order = np.argsort(-logits, axis=1, kind="stable")[:, :top_k]
    prob = np.exp(logits - logits.max(axis=1, keepdims=True))
    prob /= prob.sum(axis=1, keepdims=True)
    w_in_tok = np.stack([sum(w["w_in"][e].astype(np.float64) for e in order[n]) for n in range(xt.shape[0])])
    proj = np.einsum("nd,nod->no", xt, w_in_tok)
    np.testing.assert_allclose(res["proj"], proj, rtol=1e-10, atol=1e-12)
    y = _dense_gdn_torch(proj[None], w, cfg)[0]
    np.testing.assert_allclose(res["y"], y, rtol=1e-8, atol=1e-10)
    out = np.zeros((xt.shape[0], cfg.d_model))
    for n in range(xt.shape[0]):
        sel = order[n]
        wts = prob[n, sel] / (prob[n, sel].sum() if gate_mode == 1 else 1.0)
        for e, wt in zip(sel, wts):
            out[n] += wt * (w["w_out"][e].astype(np.float64) @ y[n])
    np.testing.assert_allclose(res["out"][0], out, rtol=1e-8, atol=1e-10)


def test_state_carry_equals_unsplit_and_causality():
    cfg = _tiny_cfg(top_k=2, gate_mode=1)
    w = S.make_gdn_weights(cfg)
    x = S.make_gdn_input(cfg).astype(np.float64)
    whole = G.rom_gdn_forward(x, w, 2, 1, cfg.n_heads, cfg.d_k)
    first = G.rom_gdn_forward(x[:, :4], w, 2, 1, cfg.n_heads, cfg.d_k)
    second = G.rom_gdn_forward(x[:, 4:], w, 2, 1, cfg.n_heads, cfg.d_k, conv_state=first["conv_state"],
                               ssm_state=first["ssm_state"])
    np.testing.assert_allclose(np.concatenate([first["out"], second["out"]], axis=1), whole["out"], rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(second["ssm_state"], whole["ssm_state"], rtol=1e-9, atol=1e-12)
    # token by token through the step
    cs = np.zeros((cfg.batch, cfg.d_conv_ch, cfg.d_conv - 1))
    ss = np.zeros((cfg.batch, cfg.n_heads, cfg.d_v, cfg.d_k))
    for t in range(cfg.seq_len):
        res = G.rom_gdn_step(x[:, t], w, 2, 1, cfg.n_heads, cfg.d_k, cs, ss)
        cs, ss = res["conv_state"], res["ssm_state"]
        np.testing.assert_allclose(res["out"], whole["out"][:, t], rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(ss, whole["ssm_state"], rtol=1e-9, atol=1e-12)
    x2 = x.copy()
    x2[0, 5:] += 1.0
    moved = G.rom_gdn_forward(x2, w, 2, 1, cfg.n_heads, cfg.d_k)["out"]
    np.testing.assert_array_equal(moved[0, :5], whole["out"][0, :5])
    np.testing.assert_array_equal(moved[1], whole["out"][1])


def test_gdn_synth_shapes():
    cfg = S.get_gdn_config("gdn_cfg2")
    assert (cfg.d_kt, cfg.d_vt, cfg.d_in_proj, cfg.d_conv_ch) == (2048, 2048, 8256, 6144)
    small = S.get_gdn_config("gdn_small")
    w = S.make_gdn_weights(small)
    assert w["w_in"].shape == (4, small.d_in_proj, 256) and w["norm_w"].shape == (small.d_v,)
    assert np.array_equal(S.round_to_bf16(w["w_in"]), w["w_in"])
