"""Pins for the CPU oracle: everything here checks oracle/rom_oracle.py against
something other than itself - closed forms, library routines in the special
cases that reduce to them, brute force with a different loop structure,
hand-worked fixtures and the figures the paper prints.  No GPU needed.
"""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import rom_oracle as O
from rom_synth import RomConfig, make_input, make_weights

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny_cfg(**kw):
    base = dict(name="tiny", cfg_id=77, batch=2, seq_len=9, d_model=8, d_inner=16, d_state=4,
                d_conv=4, dt_rank=2, n_experts=3, top_k=1, dtype="fp32", gate_mode=0,
                weight_std=0.5)
    base.update(kw)
    return RomConfig(**base)


def _weights(cfg, seed_shift=0):
    w = make_weights(cfg)
    # less regular A, D and a router bias so that no term can hide behind a symmetric value
    rng = np.random.default_rng(4242 + seed_shift)
    w["A_log"] = rng.uniform(-1.0, 1.0, w["A_log"].shape).astype(np.float32)
    w["D"] = rng.standard_normal(w["D"].shape).astype(np.float32)
    w["b_router"] = rng.standard_normal(cfg.n_experts).astype(np.float32)
    return w


# --------------------------------------------------------------------------
# routing
# --------------------------------------------------------------------------
def _read_golden_blocks(path):
    blocks, cur = {}, None
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("["):
                cur = line.strip("[]")
                blocks[cur] = []
            else:
                blocks[cur].append([float(v) for v in line.split()])
    return blocks


def test_routing_hand_worked_example():
    b = _read_golden_blocks(os.path.join(GOLDEN, "routing_worked_example.txt"))
    logits = np.array(b["logits"])
    idx = O.topk_select(logits, 2)
    assert idx.tolist() == np.array(b["expert_idx"], int).tolist()
    counts, offsets, perm, inv_perm = O.expert_permutation(idx, 4)
    assert counts.tolist() == [int(v) for v in b["counts"][0]]
    assert offsets.tolist() == [int(v) for v in b["offsets"][0]]
    assert perm.tolist() == [int(v) for v in b["perm"][0]]
    assert inv_perm.tolist() == [int(v) for v in b["inv_perm"][0]]


def test_topk_margin_hand_worked_example():
    """The margin decides which tokens the routing parity tests exempt from the bit-exact check,
    so it is pinned by hand-worked values (ties, the (K+1)-th gap deciding, K = E)."""
    b = _read_golden_blocks(os.path.join(GOLDEN, "routing_worked_example.txt"))
    logits = np.array(b["margin_logits"])
    for k in (1, 2, 3, 4):
        assert O.topk_margin(logits, k).tolist() == b[f"margin_k{k}"][0], f"K={k}"
    # a single expert has no neighbour to be confused with
    assert np.all(np.isinf(O.topk_margin(logits[:, :1], 1)))
    # every margin is a gap: never negative
    rng = np.random.default_rng(5)
    assert np.all(O.topk_margin(rng.standard_normal((200, 6)), 3) >= 0.0)


def test_topk_margin_is_the_perturbation_the_selection_survives():
    """What the margin means: moving every logit by less than half the margin cannot change the
    picks or their order; swapping the two logits that realise the margin (a move of exactly the
    margin) does change them.  A sign slip or an off-by-one in the rank range fails one of the two."""
    rng = np.random.default_rng(6)
    n, e = 400, 7
    logits = rng.standard_normal((n, e))
    for k in (1, 2, 4, 7):
        m = O.topk_margin(logits, k)
        assert np.all(m > 0)
        base = O.topk_select(logits, k)
        for _ in range(5):
            noise = rng.uniform(-0.499, 0.499, (n, e)) * m[:, None]
            assert np.array_equal(O.topk_select(logits + noise, k), base)
        # the two neighbours (in sorted order, among the first K+1 ranks) whose gap is the margin
        order = np.argsort(-logits, axis=1, kind="stable")
        srt = np.take_along_axis(logits, order, axis=1)
        hi = min(k + 1, e)
        gaps = srt[:, :hi - 1] - srt[:, 1:hi]
        j = np.argmin(gaps, axis=1)
        assert np.allclose(gaps[np.arange(n), j], m, rtol=0, atol=0)
        swapped = logits.copy()
        a, c = order[np.arange(n), j], order[np.arange(n), j + 1]
        swapped[np.arange(n), a], swapped[np.arange(n), c] = logits[np.arange(n), c], logits[np.arange(n), a]
        changed = np.any(O.topk_select(swapped, k) != base, axis=1)
        assert np.all(changed)
        # gaps beyond rank K+1 do not count: shrinking one of them leaves the margin alone
        if k + 2 <= e:
            squeezed = srt.copy()
            squeezed[:, k + 1] = squeezed[:, k] - 1e-9          # ranks K+1 and K+2 almost tie
            squeezed[:, k + 2:] -= 10.0
            assert np.array_equal(O.topk_margin(squeezed, k), m)


def test_topk_select_on_a_row_without_finite_order():
    """NaN logits are outside the layer's contract, but the selection must still name K distinct
    valid experts (the grouping indexes arrays with them): arg-max treats NaN as the maximum, so
    an all-NaN row yields experts 0..K-1."""
    logits = np.full((2, 5), np.nan)
    logits[1] = [0.0, -np.inf, -np.inf, -np.inf, 1.0]       # fewer finite logits than K
    idx = O.topk_select(logits, 3)
    assert idx[0].tolist() == [0, 1, 2]
    assert idx[1].tolist() == [4, 0, 1]
    assert all(len(set(r)) == 3 for r in idx.tolist())


def test_topk_matches_stable_sort():
    rng = np.random.default_rng(0)
    logits = np.round(rng.standard_normal((500, 7)) * 2) / 2     # many exact ties
    for k in (1, 2, 3, 7):
        idx = O.topk_select(logits, k)
        ref = np.argsort(-logits, axis=1, kind="stable")[:, :k]  # stable: lowest index first on ties
        assert np.array_equal(idx, ref)
        assert all(len(set(r)) == k for r in idx.tolist())


def test_router_logits_against_explicit_sum():
    rng = np.random.default_rng(1)
    x, wr, br = rng.standard_normal((5, 6)), rng.standard_normal((4, 6)), rng.standard_normal(4)
    got = O.router_logits(x, wr, br)
    for n in range(5):
        for e in range(4):
            want = sum(x[n, d] * wr[e, d] for d in range(6)) + br[e]
            assert abs(got[n, e] - want) < 1e-12


def test_gate_weights_invariants_and_values():
    rng = np.random.default_rng(2)
    logits = rng.standard_normal((64, 5)) * 3
    p = O.softmax(logits)
    assert np.allclose(p.sum(1), 1.0, atol=1e-14)
    assert np.allclose(p, torch.softmax(torch.from_numpy(logits), dim=1).numpy(), atol=1e-15)
    idx = O.topk_select(logits, 2)
    g0 = O.gate_weights(logits, idx, 0)
    g1 = O.gate_weights(logits, idx, 1)
    # mode 0: masked softmax of Eq. (9): the two largest probabilities, in order
    top2 = -np.sort(-p, axis=1)[:, :2]
    assert np.allclose(g0, top2, atol=1e-15)
    assert np.all(g0[:, 0] >= g0[:, 1])
    # mode 1: renormalised over the selected experts
    assert np.allclose(g1.sum(1), 1.0, atol=1e-14)
    assert np.allclose(g1, top2 / top2.sum(1, keepdims=True), atol=1e-15)
    # one expert: the gate is exactly one in both modes
    one = O.gate_weights(logits[:, :1], np.zeros((64, 1), np.int32), 0)
    assert np.array_equal(one, np.ones((64, 1)))
    # K = E in mode 0 is the whole softmax
    full = O.gate_weights(logits, O.topk_select(logits, 5), 0)
    assert np.allclose(full.sum(1), 1.0, atol=1e-14)


def test_permutation_invariants():
    rng = np.random.default_rng(3)
    n_tok, n_exp, k = 333, 6, 2
    logits = rng.standard_normal((n_tok, n_exp))
    idx = O.topk_select(logits, k)
    counts, offsets, perm, inv_perm = O.expert_permutation(idx, n_exp)
    assert counts.sum() == n_tok * k
    assert np.array_equal(counts, np.bincount(idx.ravel(), minlength=n_exp))
    assert offsets[0] == 0 and offsets[-1] == n_tok * k
    assert np.array_equal(np.diff(offsets), counts)
    assert sorted(perm.tolist()) == list(range(n_tok * k))
    assert np.array_equal(inv_perm[perm], np.arange(n_tok * k))
    exp_along = idx.ravel()[perm]
    assert np.all(np.diff(exp_along) >= 0)                       # grouped by expert
    for e in range(n_exp):                                       # stable inside a group
        seg = perm[offsets[e]:offsets[e + 1]]
        assert np.all(np.diff(seg) > 0)
    # equals a stable sort of the slots by expert
    assert np.array_equal(perm, np.argsort(idx.ravel(), kind="stable"))


def test_balance_stats_hand_worked_example():
    b = _read_golden_blocks(os.path.join(GOLDEN, "balance_worked_example.txt"))
    logits = np.log(np.array(b["exp_logits"]))
    idx = O.topk_select(logits, 2)
    assert idx.tolist() == np.array(b["expert_idx"], int).tolist()
    frac, p_bar, loss = O.balance_stats(logits, idx, 3, alpha=1.0)
    np.testing.assert_allclose(frac, b["F"][0], rtol=0, atol=1e-15)
    np.testing.assert_allclose(p_bar, b["P_bar"][0], rtol=0, atol=1e-15)
    assert abs(loss - b["loss"][0][0]) < 1e-15


def test_balance_stats_closed_forms_and_brute_force():
    """Eq. (16): flat router -> alpha whatever the counts; a router that spreads tokens evenly
    with near-certain choices -> alpha; a collapsed router -> alpha * E; and a token-by-token
    accumulation with math.exp on random logits."""
    import math
    E, N, alpha = 5, 40, 1e-3
    flat = np.zeros((N, E))
    frac, p_bar, loss = O.balance_stats(flat, O.topk_select(flat, 1), E, alpha)
    assert frac.tolist() == [1.0, 0, 0, 0, 0]            # ties go to expert 0
    np.testing.assert_allclose(p_bar, 1.0 / E, atol=1e-15)
    assert abs(loss - alpha) < 1e-18
    even = np.full((N, E), -60.0)
    even[np.arange(N), np.arange(N) % E] = 60.0
    frac, p_bar, loss = O.balance_stats(even, O.topk_select(even, 1), E, alpha)
    np.testing.assert_allclose(frac, 1.0 / E, atol=1e-15)
    np.testing.assert_allclose(p_bar, 1.0 / E, atol=1e-15)
    assert abs(loss - alpha) < 1e-15
    collapsed = np.full((N, E), -60.0)
    collapsed[:, 3] = 60.0
    frac, p_bar, loss = O.balance_stats(collapsed, O.topk_select(collapsed, 1), E, alpha)
    assert abs(loss - alpha * E) < 1e-15 and frac[3] == 1.0

    rng = np.random.default_rng(99)
    for K in (1, 2, 5):
        logits = rng.standard_normal((N, E)) * 2.0
        idx = O.topk_select(logits, K)
        frac, p_bar, loss = O.balance_stats(logits, idx, E, alpha)
        cnt, acc = [0] * E, [0.0] * E
        for n in range(N):
            ex = [math.exp(v) for v in logits[n]]
            tot = sum(ex)
            for e in range(E):
                acc[e] += ex[e] / tot
            for e in sorted(range(E), key=lambda e: (-logits[n, e], e))[:K]:
                cnt[e] += 1
        assert abs(sum(frac) - 1.0) < 1e-12 and abs(sum(p_bar) - 1.0) < 1e-12
        np.testing.assert_allclose(frac, [c / (N * K) for c in cnt], atol=1e-15)
        np.testing.assert_allclose(p_bar, [a / N for a in acc], atol=1e-14)
        assert abs(loss - alpha * E * sum(c / (N * K) * a / N for c, a in zip(cnt, acc))) < 1e-15
        # K = E: every expert gets every token, F is uniform and the loss is alpha again
        if K == E:
            assert abs(loss - alpha) < 1e-15
    # the counts agree with the grouping the layer uses
    counts, _, _, _ = O.expert_permutation(idx, E)
    np.testing.assert_allclose(frac, counts / float(N * 5), atol=1e-15)


def test_routing_is_per_token():
    """Permuting the tokens permutes the decisions (the router sees one token at a time)."""
    cfg = tiny_cfg(batch=1, seq_len=20, n_experts=4, top_k=2)
    w = _weights(cfg)
    x = make_input(cfg)[0]
    order = np.random.default_rng(5).permutation(x.shape[0])
    l_a = O.router_logits(x, w["w_router"], w["b_router"])
    l_b = O.router_logits(x[order], w["w_router"], w["b_router"])
    assert np.array_equal(O.topk_select(l_a, 2)[order], O.topk_select(l_b, 2))


# --------------------------------------------------------------------------
# conv
# --------------------------------------------------------------------------
def test_conv_matches_library_depthwise_conv():
    rng = np.random.default_rng(6)
    bsz, length, d_e, k = 2, 13, 5, 4
    h = rng.standard_normal((bsz, length, d_e))
    cw, cb = rng.standard_normal((d_e, k)), rng.standard_normal(d_e)
    u, state = O.causal_conv_silu(h, cw, cb)
    ht = torch.from_numpy(h).transpose(1, 2)
    ref = F.conv1d(ht, torch.from_numpy(cw)[:, None, :], torch.from_numpy(cb),
                   padding=k - 1, groups=d_e)[..., :length]
    ref = F.silu(ref).transpose(1, 2).numpy()
    assert np.allclose(u, ref, atol=1e-13)
    assert np.array_equal(state, h[:, -(k - 1):, :].transpose(0, 2, 1))


def test_conv_impulse_returns_taps_in_order():
    d_e, k, length = 3, 4, 8
    cw = np.arange(1, d_e * k + 1, dtype=float).reshape(d_e, k)
    h = np.zeros((1, length, d_e))
    h[0, 2, :] = 1.0
    u, _ = O.causal_conv_silu(h, cw, None)
    # invert SiLU on the known pre-activations instead: compare against silu(expected)
    expect = np.zeros((length, d_e))
    for j in range(k):                       # tap j multiplies the input k-1-j steps back
        expect[2 + (k - 1 - j), :] = cw[:, j]
    assert np.allclose(u[0], O.silu(expect), atol=1e-14)
    assert np.all(u[0, :2] == 0.0)           # causal: nothing before the impulse


def test_conv_state_carry_equals_unsplit():
    rng = np.random.default_rng(7)
    h = rng.standard_normal((2, 11, 4))
    cw, cb = rng.standard_normal((4, 4)), rng.standard_normal(4)
    full, st_full = O.causal_conv_silu(h, cw, cb)
    for m in (1, 2, 3, 7):
        a, st = O.causal_conv_silu(h[:, :m], cw, cb)
        b, st2 = O.causal_conv_silu(h[:, m:], cw, cb, st)
        assert np.allclose(np.concatenate([a, b], 1), full, atol=1e-14)
        assert np.allclose(st2, st_full)


# --------------------------------------------------------------------------
# scan
# --------------------------------------------------------------------------
def test_scan_constant_coefficients_closed_form():
    """dt, B, C, u constant: h_t = b (1 - a^t) / (1 - a), a = exp(dt A), b = dt B u."""
    length, dt, bb, cc, uu, dd = 40, 0.07, 0.9, -1.3, 0.6, 0.25
    a_vals = np.array([[-0.5, -2.0, -7.0]])
    y, h = O.selective_scan(np.full((1, length, 1), uu), np.full((1, length, 1), dt),
                            np.full((1, length, 3), bb), np.full((1, length, 3), cc),
                            a_vals, np.array([dd]))
    abar = np.exp(dt * a_vals[0])
    for t in range(length):
        h_t = dt * bb * uu * (1 - abar ** (t + 1)) / (1 - abar)
        assert abs(y[0, t, 0] - (cc * h_t.sum() + dd * uu)) < 1e-13
    assert np.allclose(h[0, 0], dt * bb * uu * (1 - abar ** length) / (1 - abar), atol=1e-14)


def _scan_double_sum(u, dt, bm, cm, a, d):
    """y_t = sum_{s<=t} sum_n C_t,n exp(a_n (S_t - S_s)) dt_s B_s,n u_s + d u_t, S = cumsum(dt)."""
    bsz, length, d_e = u.shape
    y = np.zeros_like(u)
    s_cum = np.cumsum(dt, axis=1)
    for b in range(bsz):
        for i in range(d_e):
            for t in range(length):
                acc = 0.0
                for s in range(t + 1):
                    w = np.exp(a[i] * (s_cum[b, t, i] - s_cum[b, s, i]))
                    acc += np.sum(cm[b, t] * w * bm[b, s]) * dt[b, s, i] * u[b, s, i]
                y[b, t, i] = acc + d[i] * u[b, t, i]
    return y


def test_scan_matches_unrolled_double_sum():
    rng = np.random.default_rng(8)
    bsz, length, d_e, d_s = 2, 12, 3, 4
    u = rng.standard_normal((bsz, length, d_e))
    dt = rng.uniform(0.01, 0.3, (bsz, length, d_e))
    bm, cm = rng.standard_normal((bsz, length, d_s)), rng.standard_normal((bsz, length, d_s))
    a, d = -rng.uniform(0.2, 3.0, (d_e, d_s)), rng.standard_normal(d_e)
    y, _ = O.selective_scan(u, dt, bm, cm, a, d)
    assert np.allclose(y, _scan_double_sum(u, dt, bm, cm, a, d), atol=1e-12)


def test_scan_impulse_response_and_linearity():
    rng = np.random.default_rng(9)
    length, d_s = 10, 3
    dt = rng.uniform(0.05, 0.2, (1, length, 1))
    bm, cm = rng.standard_normal((1, length, d_s)), rng.standard_normal((1, length, d_s))
    a = -rng.uniform(0.5, 2.0, (1, d_s))
    u = np.zeros((1, length, 1))
    u[0, 0, 0] = 1.0
    y, _ = O.selective_scan(u, dt, bm, cm, a, np.zeros(1))
    for t in range(length):
        decay = np.exp(a[0] * dt[0, 1:t + 1, 0].sum())
        assert abs(y[0, t, 0] - np.sum(cm[0, t] * decay * dt[0, 0, 0] * bm[0, 0])) < 1e-14
    u1, u2 = rng.standard_normal((1, length, 1)), rng.standard_normal((1, length, 1))
    d = np.array([0.3])
    y1, _ = O.selective_scan(u1, dt, bm, cm, a, d)
    y2, _ = O.selective_scan(u2, dt, bm, cm, a, d)
    y12, _ = O.selective_scan(2 * u1 - 3 * u2, dt, bm, cm, a, d)
    assert np.allclose(y12, 2 * y1 - 3 * y2, atol=1e-13)


def test_scan_chunked_equals_per_step():
    """Any split of the sequence with the state carried across equals the unsplit recurrence."""
    rng = np.random.default_rng(10)
    bsz, length, d_e, d_s = 2, 17, 4, 3
    u = rng.standard_normal((bsz, length, d_e))
    dt = rng.uniform(0.01, 0.3, (bsz, length, d_e))
    bm, cm = rng.standard_normal((bsz, length, d_s)), rng.standard_normal((bsz, length, d_s))
    a, d = -rng.uniform(0.2, 3.0, (d_e, d_s)), rng.standard_normal(d_e)
    h0 = rng.standard_normal((bsz, d_e, d_s))
    y_full, h_full = O.selective_scan(u, dt, bm, cm, a, d, h0)
    for cuts in ([5], [1, 2, 16], [4, 8, 12]):
        h, ys, prev = h0, [], 0
        for c in cuts + [length]:
            yc, h = O.selective_scan(u[:, prev:c], dt[:, prev:c], bm[:, prev:c], cm[:, prev:c], a, d, h)
            ys.append(yc)
            prev = c
        assert np.allclose(np.concatenate(ys, 1), y_full, atol=1e-13)
        assert np.allclose(h, h_full, atol=1e-13)


# --------------------------------------------------------------------------
# whole layer
# --------------------------------------------------------------------------
def _dense_mamba_torch(x, w):
    """Dense Mamba layer, Eq. (1)-(6), from library routines; scan by the unrolled double sum."""
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    d_e, d_s, r = w["w_out"].shape[2], w["A_log"].shape[1], w["w_dt"].shape[2]
    k = w["conv_w"].shape[1]
    xt = t(x)
    length = xt.shape[1]
    xz = F.linear(xt, t(w["w_in"][0]))
    h_pre, z = xz[..., :d_e], xz[..., d_e:]
    c = F.conv1d(h_pre.transpose(1, 2), t(w["conv_w"])[:, None, :], t(w["conv_b"]),
                 padding=k - 1, groups=d_e)[..., :length]
    u = F.silu(c).transpose(1, 2)
    xdbl = F.linear(u, t(w["w_x"][0]))
    dt = F.softplus(F.linear(xdbl[..., :r], t(w["w_dt"][0])) + t(w["dt_bias"]))
    a = -np.exp(np.asarray(w["A_log"], np.float64))
    y = _scan_double_sum(u.numpy(), dt.numpy(), xdbl[..., r:r + d_s].numpy(),
                         xdbl[..., r + d_s:].numpy(), a, np.asarray(w["D"], np.float64))
    g = t(y) * F.silu(z)
    return F.linear(g, t(w["w_out"][0])).numpy()


def test_single_expert_reduces_to_dense_mamba():
    cfg = tiny_cfg(n_experts=1, top_k=1)
    w = _weights(cfg)
    x = make_input(cfg)
    for mode in (0, 1):
        res = O.rom_layer_forward(x, w, 1, mode)
        assert np.array_equal(res["gate"], np.ones_like(res["gate"]))
        assert np.allclose(res["out"], _dense_mamba_torch(x, w), rtol=1e-11, atol=1e-13)


def _brute_force_layer(x, w, top_k, gate_mode):
    """Eq. (9)-(13) with every expert evaluated densely for every token and the router's
    indicator / weight applied afterwards; scalar loops for conv and recurrence."""
    x = np.asarray(x, np.float64)
    bsz, length, d_m = x.shape
    n_exp, d_e = w["w_router"].shape[0], w["w_out"].shape[2]
    d_s, r, k = w["A_log"].shape[1], w["w_dt"].shape[2], w["conv_w"].shape[1]
    routed_xdt = w["w_x"].shape[0] == n_exp
    f = lambda a: np.asarray(a, np.float64)
    a_mat = -np.exp(f(w["A_log"]))
    out = np.zeros((bsz, length, d_m))
    for b in range(bsz):
        ind = np.zeros((length, n_exp))
        weight = np.zeros((length, n_exp))
        for t in range(length):
            logit = [float(np.dot(f(w["w_router"])[e], x[b, t]) + w["b_router"][e]) for e in range(n_exp)]
            order = sorted(range(n_exp), key=lambda e: (-logit[e], e))[:top_k]
            m = max(logit)
            ex = [np.exp(v - m) for v in logit]
            p = [v / sum(ex) for v in ex]
            norm = sum(p[e] for e in order) if gate_mode == 1 else 1.0
            for e in order:
                ind[t, e] = 1.0
                weight[t, e] = p[e] / norm
        hz = np.zeros((length, 2 * d_e))
        for t in range(length):
            for e in range(n_exp):
                hz[t] += ind[t, e] * (f(w["w_in"][e]) @ x[b, t])
        u = np.zeros((length, d_e))
        for t in range(length):
            for i in range(d_e):
                acc = float(w["conv_b"][i])
                for j in range(k):
                    src = t - (k - 1) + j
                    if src >= 0:
                        acc += float(w["conv_w"][i, j]) * hz[src, i]
                u[t, i] = acc / (1.0 + np.exp(-acc))
        state = np.zeros((d_e, d_s))
        for t in range(length):
            xdbl = np.zeros(r + 2 * d_s)
            for e in range(n_exp if routed_xdt else 1):
                xdbl += (ind[t, e] if routed_xdt else 1.0) * (f(w["w_x"][e]) @ u[t])
            pre = np.zeros(d_e)
            for e in range(n_exp if routed_xdt else 1):
                pre += (ind[t, e] if routed_xdt else 1.0) * (f(w["w_dt"][e]) @ xdbl[:r])
            pre += f(w["dt_bias"])
            dt = np.log1p(np.exp(pre))
            bm, cm = xdbl[r:r + d_s], xdbl[r + d_s:]
            y = np.zeros(d_e)
            for i in range(d_e):
                for n in range(d_s):
                    state[i, n] = np.exp(dt[i] * a_mat[i, n]) * state[i, n] + dt[i] * bm[n] * u[t, i]
                    y[i] += cm[n] * state[i, n]
                y[i] += float(w["D"][i]) * u[t, i]
            zt = hz[t, d_e:]
            g = y * (zt / (1.0 + np.exp(-zt)))
            for e in range(n_exp):
                out[b, t] += weight[t, e] * (f(w["w_out"][e]) @ g)
    return out


@pytest.mark.parametrize("top_k,gate_mode,routed", [(1, 0, True), (2, 0, True), (2, 1, True),
                                                     (3, 1, True), (2, 1, False), (1, 0, False)])
def test_layer_matches_all_experts_brute_force(top_k, gate_mode, routed):
    cfg = tiny_cfg(batch=2, seq_len=6, d_model=4, d_inner=6, d_state=3, dt_rank=2,
                   n_experts=3, top_k=top_k, gate_mode=gate_mode, routed_xdt=routed)
    w = _weights(cfg, seed_shift=top_k)
    x = make_input(cfg)
    res = O.rom_layer_forward(x, w, top_k, gate_mode)
    ref = _brute_force_layer(x, w, top_k, gate_mode)
    assert np.allclose(res["out"], ref, rtol=1e-11, atol=1e-13)
    assert res["counts"].sum() == x.shape[0] * x.shape[1] * top_k


def test_all_experts_selected_is_dense_mixture():
    """K = E with renormalised gates: out = sum_e P_e * ((Y*G) W_out,e) with every projection
    summed over all experts - a special case that needs no routing at all."""
    cfg = tiny_cfg(batch=1, seq_len=7, n_experts=3, top_k=3, gate_mode=1)
    w = _weights(cfg)
    x = make_input(cfg)
    res = O.rom_layer_forward(x, w, 3, 1)
    w_sum = dict(w)
    for name in ("w_in", "w_x", "w_dt"):
        w_sum[name] = w[name].astype(np.float64).sum(axis=0, keepdims=True)
    w_sum["w_router"] = w["w_router"][:1]
    w_sum["b_router"] = w["b_router"][:1]
    p = O.softmax(O.router_logits(x[0], w["w_router"], w["b_router"]))
    w_sum["w_out"] = np.zeros_like(w["w_out"][:1], dtype=np.float64)
    dense = O.rom_layer_forward(x, w_sum, 1, 0)          # single "expert" = summed projections
    g = dense["g"]
    want = sum(p[:, e:e + 1] * (g @ w["w_out"][e].astype(np.float64).T) for e in range(3))
    assert np.allclose(res["out"][0], want, rtol=1e-11, atol=1e-13)


def test_causality_and_batch_independence():
    cfg = tiny_cfg(batch=3, seq_len=10, n_experts=4, top_k=2, gate_mode=1)
    w = _weights(cfg)
    x = make_input(cfg)
    base = O.rom_layer_forward(x, w, 2, 1)["out"]
    x2 = x.copy()
    x2[:, 6:, :] += 1.0
    pert = O.rom_layer_forward(x2, w, 2, 1)["out"]
    assert np.array_equal(pert[:, :6], base[:, :6])
    assert not np.allclose(pert[:, 6:], base[:, 6:])
    for b in range(3):
        alone = O.rom_layer_forward(x[b:b + 1], w, 2, 1)["out"]
        assert np.allclose(alone[0], base[b], rtol=1e-12, atol=1e-14)


def test_state_api_split_and_step():
    cfg = tiny_cfg(batch=2, seq_len=12, n_experts=3, top_k=2, gate_mode=1)
    w = _weights(cfg)
    x = make_input(cfg)
    full = O.rom_layer_forward(x, w, 2, 1)
    for m in (1, 3, 8):
        a = O.rom_layer_forward(x[:, :m], w, 2, 1)
        b = O.rom_layer_forward(x[:, m:], w, 2, 1, a["conv_state"], a["ssm_state"])
        assert np.allclose(np.concatenate([a["out"], b["out"]], 1), full["out"], rtol=1e-11, atol=1e-13)
        assert np.allclose(b["ssm_state"], full["ssm_state"], rtol=1e-11, atol=1e-13)
        assert np.allclose(b["conv_state"], full["conv_state"])
    head = O.rom_layer_forward(x[:, :-1], w, 2, 1)
    step = O.rom_step(x[:, -1], w, 2, 1, head["conv_state"], head["ssm_state"])
    assert np.allclose(step["out"], full["out"][:, -1], rtol=1e-11, atol=1e-13)
    assert np.allclose(step["ssm_state"], full["ssm_state"], rtol=1e-11, atol=1e-13)
    # a step from given states is the recurrence written out for one token
    cs = np.random.default_rng(11).standard_normal((2, cfg.d_inner, cfg.d_conv - 1))
    ss = np.random.default_rng(12).standard_normal((2, cfg.d_inner, cfg.d_state))
    st = O.rom_step(x[:, 0], w, 2, 1, cs, ss)
    window = np.concatenate([cs, st["xz"][:, :cfg.d_inner, None]], axis=2)      # [B, D_e, k]
    pre = (window * w["conv_w"][None]).sum(2) + w["conv_b"][None]
    assert np.allclose(st["u"], pre / (1 + np.exp(-pre)), rtol=1e-12)
    assert np.allclose(st["conv_state"], window[:, :, 1:])
    a_mat = -np.exp(w["A_log"].astype(np.float64))
    r, d_s = cfg.dt_rank, cfg.d_state
    h = (np.exp(st["dt"][:, :, None] * a_mat[None]) * ss
         + (st["dt"] * st["u"])[:, :, None] * st["xdbl"][:, None, r:r + d_s])
    assert np.allclose(st["ssm_state"], h, rtol=1e-12)


def test_rms_norm_against_library_and_closed_forms():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((3, 7, 24)) * 3.0
    wn = rng.uniform(0.5, 1.5, 24)
    ref = F.rms_norm(torch.from_numpy(x), (24,), torch.from_numpy(wn), eps=1e-5).numpy()
    np.testing.assert_allclose(O.rms_norm(x, wn, 1e-5), ref, rtol=1e-13, atol=1e-14)
    # a constant row c maps to sign(c) * w / sqrt(1 + eps / c^2)
    np.testing.assert_allclose(O.rms_norm(np.full((1, 24), -2.0), wn, 0.04)[0], -wn / np.sqrt(1.01), rtol=1e-14)
    # eps = 0: unit RMS for w = 1 and invariance to the input's scale
    y = O.rms_norm(x, np.ones(24), 0.0)
    np.testing.assert_allclose(np.sqrt(np.mean(y * y, axis=-1)), 1.0, rtol=1e-14)
    np.testing.assert_allclose(O.rms_norm(7.5 * x, wn, 0.0), O.rms_norm(x, wn, 0.0), rtol=1e-13)
    # rows are independent, and it is the row that is normalised (not the column)
    np.testing.assert_allclose(O.rms_norm(x[1:2, 3:4], wn, 1e-5), O.rms_norm(x, wn, 1e-5)[1:2, 3:4], rtol=1e-14)


def test_block_is_skip_plus_layer_of_normalised_input():
    """The block against its parts assembled from library routines: torch's rms_norm in front of
    a dense Mamba layer (E = 1), plus the input; with W_out = 0 the block is the identity; and
    a routed block keeps the router's view of the *normalised* input."""
    cfg = tiny_cfg(n_experts=1)
    w = _weights(cfg)
    w["norm_w"] = np.random.default_rng(8).uniform(0.5, 1.5, cfg.d_model).astype(np.float32)
    x = make_input(cfg).astype(np.float64) * 2.5
    xn = F.rms_norm(torch.from_numpy(x), (cfg.d_model,), torch.from_numpy(w["norm_w"]).double(), eps=1e-5)
    want = x + _dense_mamba_torch(xn.numpy(), w)
    got = O.rom_block_forward(x, w, 1, 0, 1e-5)
    np.testing.assert_allclose(got["out"], want, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(got["out"] - got["branch"], x, rtol=0, atol=1e-12)

    w0 = dict(w)
    w0["w_out"] = np.zeros_like(w["w_out"])
    np.testing.assert_array_equal(O.rom_block_forward(x, w0, 1, 0, 1e-5)["out"], x)

    cfg = tiny_cfg(n_experts=4, top_k=2)
    w = _weights(cfg, 3)
    w["norm_w"] = np.random.default_rng(9).uniform(0.5, 1.5, cfg.d_model).astype(np.float32)
    x = make_input(cfg).astype(np.float64)
    blk = O.rom_block_forward(x, w, 2, 1, 1e-5)
    inner = O.rom_layer_forward(O.rms_norm(x, w["norm_w"], 1e-5), w, 2, 1)
    assert blk["expert_idx"].tolist() == inner["expert_idx"].tolist()
    # scaling the block input by a positive constant leaves the branch (almost: eps) unchanged
    blk2 = O.rom_block_forward(1000.0 * x, w, 2, 1, 0.0)
    blk1 = O.rom_block_forward(x, w, 2, 1, 0.0)
    np.testing.assert_allclose(blk2["branch"], blk1["branch"], rtol=1e-9, atol=1e-12)


def test_stack_is_the_composition_of_blocks_with_per_layer_state():
    cfg = tiny_cfg(n_experts=3, top_k=1)
    layers = []
    for j in range(3):
        w = _weights(cfg, 10 + j)
        w["norm_w"] = np.random.default_rng(20 + j).uniform(0.5, 1.5, cfg.d_model).astype(np.float32)
        layers.append(w)
    x = make_input(cfg).astype(np.float64)
    out, res = O.rom_stack_forward(x, layers, 1, 0, 1e-5)
    h = x
    for j in range(3):
        h = h + O.rom_layer_forward(O.rms_norm(h, layers[j]["norm_w"], 1e-5), layers[j], 1, 0)["out"]
    np.testing.assert_allclose(out, h, rtol=1e-12, atol=1e-13)
    # prefill of a prefix, then the rest from the per-layer states, equals the unsplit run
    cut = 5
    o1, r1 = O.rom_stack_forward(x[:, :cut], layers, 1, 0, 1e-5)
    o2, _ = O.rom_stack_forward(x[:, cut:], layers, 1, 0, 1e-5, [r["conv_state"] for r in r1],
                                [r["ssm_state"] for r in r1])
    np.testing.assert_allclose(np.concatenate([o1, o2], axis=1), out, rtol=1e-10, atol=1e-12)
    # causal through the whole stack
    x2 = x.copy()
    x2[:, 6:] += 1.0
    out2, _ = O.rom_stack_forward(x2, layers, 1, 0, 1e-5)
    np.testing.assert_array_equal(out2[:, :6], out[:, :6])


def test_ffn_moe_against_library_mlp_and_brute_force():
    """Eq. (14)/(15): one expert with weight 1 is a dense SwiGLU MLP from library routines; the routed
    form equals a scalar-loop evaluation of every expert times its indicator and weight."""
    rng = np.random.default_rng(31)
    n, d_m, d_f, n_exp = 11, 6, 10, 4
    x = rng.standard_normal((n, d_m))
    wgu = rng.standard_normal((n_exp, 2 * d_f, d_m)) * 0.5
    wd = rng.standard_normal((n_exp, d_m, d_f)) * 0.5
    xt = torch.from_numpy(x)
    gate_w, up_w = torch.from_numpy(wgu[2, :d_f]), torch.from_numpy(wgu[2, d_f:])
    want = F.linear(F.silu(F.linear(xt, gate_w)) * F.linear(xt, up_w), torch.from_numpy(wd[2])).numpy()
    idx1 = np.full((n, 1), 2)
    got = O.ffn_moe_forward(x, wgu, wd, idx1, np.ones((n, 1)))
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
    # swapping the gate and up halves changes the result (SiLU sits on the first half)
    swapped = np.concatenate([wgu[:, d_f:], wgu[:, :d_f]], axis=1)
    assert np.max(np.abs(O.ffn_moe_forward(x, swapped, wd, idx1, np.ones((n, 1))) - want)) > 1e-3

    logits = rng.standard_normal((n, n_exp))
    for K, mode in ((1, 0), (2, 0), (3, 1)):
        idx = O.topk_select(logits, K)
        gate = O.gate_weights(logits, idx, mode)
        got = O.ffn_moe_forward(x, wgu, wd, idx, gate)
        want = np.zeros((n, d_m))
        for t in range(n):
            for i in range(n_exp):
                r = sum(gate[t, k] for k in range(K) if idx[t, k] == i)      # R_i * indicator
                if r == 0.0:
                    continue
                hid = [0.0] * d_f
                for f in range(d_f):
                    a = sum(wgu[i, f, d] * x[t, d] for d in range(d_m))
                    b = sum(wgu[i, d_f + f, d] * x[t, d] for d in range(d_m))
                    hid[f] = a / (1.0 + np.exp(-a)) * b
                for d in range(d_m):
                    want[t, d] += r * sum(wd[i, d, f] * hid[f] for f in range(d_f))
        np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-12)
    # pre-norm and skip: experts see the normalised rows, the raw rows are added
    nw = rng.uniform(0.5, 1.5, d_m)
    xn = F.rms_norm(xt, (d_m,), torch.from_numpy(nw), eps=1e-5).numpy()
    np.testing.assert_allclose(O.ffn_moe_forward(x, wgu, wd, idx, gate, nw, 1e-5, skip=True),
                               x + O.ffn_moe_forward(xn, wgu, wd, idx, gate), rtol=1e-12, atol=1e-13)
    # all experts identical and weights summing to one: routing cannot matter
    same_gu, same_d = np.repeat(wgu[:1], n_exp, 0), np.repeat(wd[:1], n_exp, 0)
    idx = O.topk_select(logits, 2)
    gate = O.gate_weights(logits, idx, 1)
    np.testing.assert_allclose(O.ffn_moe_forward(x, same_gu, same_d, idx, gate),
                               O.swiglu_expert(x, wgu[0], wd[0]), rtol=1e-12, atol=1e-13)


# --------------------------------------------------------------------------
# backward pass
# --------------------------------------------------------------------------
_PARAMS = ("w_router", "b_router", "w_in", "conv_w", "conv_b", "w_x", "w_dt", "dt_bias", "A_log", "D", "w_out")


def _routed_layer_torch(x, w, idx, gate_mode):
    """The layer of Eq. (9)-(13) from torch routines in float64 with a per-step loop for the
    recurrence, on a given expert choice: an implementation independent of the oracle whose
    gradients come from torch's reverse-mode differentiation."""
    bsz, length, d_m = x.shape
    n_exp, d_e = w["w_router"].shape[0], w["w_out"].shape[2]
    d_s, r, k = w["A_log"].shape[1], w["w_dt"].shape[2], w["conv_w"].shape[1]
    idx_t = torch.as_tensor(np.asarray(idx, np.int64)).reshape(bsz, length, -1)
    onehot = F.one_hot(idx_t, n_exp).to(torch.float64)                 # [B, L, K, E]
    ind = onehot.sum(dim=2)                                            # indicator 1[i in TopK]
    logits = F.linear(x, w["w_router"], w["b_router"])
    p = torch.softmax(logits, dim=-1)
    sel = torch.gather(p, -1, idx_t)
    gate = sel / sel.sum(-1, keepdim=True) if gate_mode == 1 else sel

    def routed(inp, wt, weight_per_expert):
        if wt.shape[0] == 1:
            return F.linear(inp, wt[0])
        return sum(weight_per_expert[..., e:e + 1] * F.linear(inp, wt[e]) for e in range(wt.shape[0]))

    xz = routed(x, w["w_in"], ind)
    h_pre, z = xz[..., :d_e], xz[..., d_e:]
    c = F.conv1d(h_pre.transpose(1, 2), w["conv_w"][:, None, :], w["conv_b"], padding=k - 1, groups=d_e)[..., :length]
    u = F.silu(c).transpose(1, 2)
    xdbl = routed(u, w["w_x"], ind)
    dt = F.softplus(routed(xdbl[..., :r], w["w_dt"], ind) + w["dt_bias"])
    bm, cm = xdbl[..., r:r + d_s], xdbl[..., r + d_s:]
    a = -torch.exp(w["A_log"])
    h = torch.zeros(bsz, d_e, d_s, dtype=torch.float64)
    ys = []
    for t in range(length):
        h = torch.exp(dt[:, t, :, None] * a) * h + (dt[:, t] * u[:, t])[:, :, None] * bm[:, t, None, :]
        ys.append((h * cm[:, t, None, :]).sum(-1) + w["D"] * u[:, t])
    g = torch.stack(ys, dim=1) * F.silu(z)
    weights = (onehot * gate[..., None]).sum(dim=2)                    # R_i of Eq. (12) per expert
    return sum(weights[..., e:e + 1] * F.linear(g, w["w_out"][e]) for e in range(n_exp))


@pytest.mark.parametrize("top_k,gate_mode,routed,n_exp", [(1, 0, True, 3), (2, 1, True, 4), (2, 0, False, 3),
                                                           (3, 1, True, 3), (1, 0, True, 1)])
def test_backward_matches_reverse_mode_differentiation_of_library_layer(top_k, gate_mode, routed, n_exp):
    cfg = tiny_cfg(top_k=top_k, gate_mode=gate_mode, routed_xdt=routed, n_experts=n_exp, seq_len=11)
    w = _weights(cfg, seed_shift=top_k + 10 * gate_mode)
    x = make_input(cfg)
    rng = np.random.default_rng(17)
    d_out = rng.standard_normal(x.shape)
    res = O.rom_layer_backward(x, w, top_k, gate_mode, d_out)
    idx = res["fwd"]["expert_idx"]
    tw = {k: torch.tensor(np.asarray(w[k], np.float64), requires_grad=True) for k in _PARAMS}
    tx = torch.tensor(np.asarray(x, np.float64), requires_grad=True)
    out = _routed_layer_torch(tx, tw, idx, gate_mode)
    assert np.allclose(out.detach().numpy(), res["fwd"]["out"], rtol=1e-11, atol=1e-13)
    (out * torch.tensor(d_out)).sum().backward()
    for name in _PARAMS:
        want = tw[name].grad.numpy()
        got = res["d_" + name]
        assert got.shape == want.shape, name
        assert np.max(np.abs(got - want)) <= 1e-10 * (1.0 + np.max(np.abs(want))), name
    assert np.max(np.abs(res["d_x"] - tx.grad.numpy())) <= 1e-10 * (1.0 + np.max(np.abs(tx.grad.numpy())))
    # every gradient is exercised: none of them is identically zero on this input
    assert all(np.max(np.abs(res["d_" + n])) > 1e-6 for n in _PARAMS if not (n_exp == 1 and n.endswith("router")))
    if n_exp == 1:      # one expert: the gate is 1 whatever the logits, the router gets no gradient
        assert np.max(np.abs(res["d_w_router"])) < 1e-12 and np.max(np.abs(res["d_b_router"])) < 1e-12


def test_backward_matches_central_differences_of_the_forward_oracle():
    """d/d theta of sum(out * d_out) by central differences of rom_layer_forward at a fixed expert
    choice, for sampled entries of x and of every parameter."""
    cfg = tiny_cfg(top_k=2, gate_mode=1, n_experts=4, seq_len=9)
    w = {k: (None if v is None else np.asarray(v, np.float64)) for k, v in _weights(cfg).items()}
    x = np.asarray(make_input(cfg), np.float64)
    rng = np.random.default_rng(23)
    d_out = rng.standard_normal(x.shape)
    res = O.rom_layer_backward(x, w, 2, 1, d_out)
    idx = res["fwd"]["expert_idx"]

    def loss(xx, ww):
        return float((O.rom_layer_forward(xx, ww, 2, 1, expert_idx=idx)["out"] * d_out).sum())

    eps = 1e-5
    for name in _PARAMS + ("x",):
        base = x if name == "x" else w[name]
        grad = res["d_" + name]
        scale = np.max(np.abs(grad))
        for _ in range(8):
            i = tuple(int(rng.integers(0, n)) for n in base.shape)
            plus, minus = base.copy(), base.copy()
            plus[i] += eps
            minus[i] -= eps
            if name == "x":
                fd = (loss(plus, w) - loss(minus, w)) / (2 * eps)
            else:
                fd = (loss(x, dict(w, **{name: plus})) - loss(x, dict(w, **{name: minus}))) / (2 * eps)
            assert abs(fd - grad[i]) <= 1e-6 * scale + 1e-8, (name, i, fd, grad[i])


def test_rms_norm_backward_against_library_differentiation():
    rng = np.random.default_rng(31)
    x = rng.standard_normal((3, 5, 12))
    wgt = 1.0 + 0.3 * rng.standard_normal(12)
    d_y = rng.standard_normal(x.shape)
    d_x, d_w = O.rms_norm_backward(x, wgt, 1e-5, d_y)
    tx = torch.tensor(x, requires_grad=True)
    tw = torch.tensor(wgt, requires_grad=True)
    y = F.rms_norm(tx, (12,), tw, 1e-5)
    assert np.allclose(y.detach().numpy(), O.rms_norm(x, wgt, 1e-5), rtol=1e-12, atol=1e-14)
    (y * torch.tensor(d_y)).sum().backward()
    assert np.allclose(d_x, tx.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(d_w, tw.grad.numpy(), rtol=1e-10, atol=1e-12)
    # the gradient has no component along x^ scaled by the weight-free norm: d_x . x = 0 when weight = 1
    d_x1, _ = O.rms_norm_backward(x, np.ones(12), 0.0, d_y)
    assert np.max(np.abs((d_x1 * x).sum(-1))) < 1e-12


def test_block_backward_matches_central_differences_of_the_block_forward():
    """out = x + RoM(RMSNorm(x)): d/d theta of sum(out * d_out) by central differences of
    rom_block_forward at a fixed expert choice, for sampled entries of x, of the norm's scale and of
    every parameter; and the skip alone (all-zero out projection) passes d_out through."""
    cfg = tiny_cfg(top_k=2, gate_mode=1, n_experts=4, seq_len=7)
    w = {k: (None if v is None else np.asarray(v, np.float64)) for k, v in _weights(cfg).items()}
    rng = np.random.default_rng(29)
    w["norm_w"] = 1.0 + 0.3 * rng.standard_normal(cfg.d_model)
    x = 1.7 * np.asarray(make_input(cfg), np.float64)
    d_out = rng.standard_normal(x.shape)
    res = O.rom_block_backward(x, w, 2, 1, d_out, 1e-5)
    idx = res["fwd"]["expert_idx"]
    assert np.array_equal(idx, O.rom_block_forward(x, w, 2, 1, 1e-5)["expert_idx"])

    def loss(xx, ww):
        return float((O.rom_block_forward(xx, ww, 2, 1, 1e-5, expert_idx=idx)["out"] * d_out).sum())

    eps = 1e-5
    for name in _PARAMS + ("norm_w", "x"):
        base = x if name == "x" else w[name]
        grad = res["d_" + name]
        assert grad.shape == base.shape, name
        scale = np.max(np.abs(grad))
        assert scale > 1e-6, name
        for _ in range(8):
            i = tuple(int(rng.integers(0, n)) for n in base.shape)
            plus, minus = base.copy(), base.copy()
            plus[i] += eps
            minus[i] -= eps
            if name == "x":
                fd = (loss(plus, w) - loss(minus, w)) / (2 * eps)
            else:
                fd = (loss(x, dict(w, **{name: plus})) - loss(x, dict(w, **{name: minus}))) / (2 * eps)
            assert abs(fd - grad[i]) <= 1e-6 * scale + 1e-8, (name, i, fd, grad[i])
    w0 = dict(w, w_out=np.zeros_like(w["w_out"]))
    res0 = O.rom_block_backward(x, w0, 2, 1, d_out, 1e-5, expert_idx=idx)
    assert np.array_equal(res0["d_x"], d_out) and np.max(np.abs(res0["d_norm_w"])) == 0.0


@pytest.mark.parametrize("pre_norm,skip,top_k", [(False, False, 1), (True, True, 2), (True, False, 3), (False, True, 2)])
def test_ffn_moe_backward_against_library_differentiation(pre_norm, skip, top_k):
    """The FFN-MoE layer of Eq. (14)/(15) written separately from torch routines (dense over the
    experts, masked by the routing decision), differentiated by torch, against the oracle's
    hand-written backward; the gate weights are an input here and get their own gradient."""
    rng = np.random.default_rng(41 + top_k)
    n_tok, d_m, d_f, n_exp = 23, 6, 5, 4
    x = 1.3 * rng.standard_normal((n_tok, d_m))
    wgu = 0.5 * rng.standard_normal((n_exp, 2 * d_f, d_m))
    wd = 0.5 * rng.standard_normal((n_exp, d_m, d_f))
    nw = 1.0 + 0.3 * rng.standard_normal(d_m) if pre_norm else None
    idx = np.stack([rng.permutation(n_exp)[:top_k] for _ in range(n_tok)]).astype(np.int32)
    gate = rng.uniform(0.1, 1.0, (n_tok, top_k))
    d_out = rng.standard_normal((n_tok, d_m))
    res = O.ffn_moe_backward(x, wgu, wd, idx, gate, d_out, nw, 1e-5, skip)

    tx = torch.tensor(x, requires_grad=True)
    tgu = torch.tensor(wgu, requires_grad=True)
    tdn = torch.tensor(wd, requires_grad=True)
    tg = torch.tensor(gate, requires_grad=True)
    tn = torch.tensor(nw, requires_grad=True) if pre_norm else None
    xin = F.rms_norm(tx, (d_m,), tn, 1e-5) if pre_norm else tx
    weights = torch.zeros(n_tok, n_exp, dtype=torch.float64)
    weights = weights.scatter_add(1, torch.as_tensor(idx, dtype=torch.int64), tg)      # R_i per expert (0 if not selected)
    y = torch.zeros_like(tx)
    for i in range(n_exp):
        h = F.linear(xin, tgu[i])
        y = y + weights[:, i:i + 1] * F.linear(F.silu(h[:, :d_f]) * h[:, d_f:], tdn[i])
    if skip:
        y = y + tx
    assert np.allclose(y.detach().numpy(), O.ffn_moe_forward(x, wgu, wd, idx, gate, nw, 1e-5, skip), rtol=1e-11, atol=1e-13)
    (y * torch.tensor(d_out)).sum().backward()
    pairs = [("d_x", tx), ("d_w_gate_up", tgu), ("d_w_down", tdn), ("d_gate", tg)] + ([("d_norm_w", tn)] if pre_norm else [])
    for name, t in pairs:
        want = t.grad.numpy()
        assert res[name].shape == want.shape, name
        assert np.max(np.abs(want)) > 1e-6, name
        assert np.max(np.abs(res[name] - want)) <= 1e-10 * (1.0 + np.max(np.abs(want))), name
    assert pre_norm or "d_norm_w" not in res


def test_hybrid_pair_backward_matches_central_differences():
    """A RoM block followed by an FFN-MoE block on the RoM block's routing decision and gate weights
    (Eq. (14)/(15)): the chain ffn_moe_backward -> rom_block_backward, with the FFN's gate gradient
    handed to the block, against central differences of the composed forward - for x, the router
    (which the FFN reaches through the gates only) and samples of the other parameters."""
    cfg = tiny_cfg(top_k=2, gate_mode=0, n_experts=4, seq_len=6)
    w = {k: (None if v is None else np.asarray(v, np.float64)) for k, v in _weights(cfg).items()}
    rng = np.random.default_rng(37)
    d_m, d_f = cfg.d_model, 6
    w["norm_w"] = 1.0 + 0.3 * rng.standard_normal(d_m)
    fw = {"w_gate_up": 0.5 * rng.standard_normal((4, 2 * d_f, d_m)), "w_down": 0.5 * rng.standard_normal((4, d_m, d_f)),
          "norm_w": 1.0 + 0.3 * rng.standard_normal(d_m)}
    x = 1.2 * np.asarray(make_input(cfg), np.float64)
    n_tok = x.shape[0] * x.shape[1]
    d_out = rng.standard_normal((n_tok, d_m))
    idx = O.rom_block_forward(x, w, 2, 0, 1e-5)["expert_idx"]

    def forward(xx, ww, ff):
        blk = O.rom_block_forward(xx, ww, 2, 0, 1e-5, expert_idx=idx)
        return blk, O.ffn_moe_forward(blk["out"].reshape(n_tok, d_m), ff["w_gate_up"], ff["w_down"], idx, blk["gate"],
                                      ff["norm_w"], 1e-5, skip=True)

    blk, _ = forward(x, w, fw)
    fb = O.ffn_moe_backward(blk["out"].reshape(n_tok, d_m), fw["w_gate_up"], fw["w_down"], idx, blk["gate"], d_out,
                            fw["norm_w"], 1e-5, skip=True)
    res = O.rom_block_backward(x, w, 2, 0, fb["d_x"].reshape(x.shape), 1e-5, expert_idx=idx, d_gate_extra=fb["d_gate"])
    without = O.rom_block_backward(x, w, 2, 0, fb["d_x"].reshape(x.shape), 1e-5, expert_idx=idx)
    assert np.max(np.abs(res["d_w_router"] - without["d_w_router"])) > 1e-3      # the handed-over gradient matters here

    def loss(xx, ww, ff):
        return float((forward(xx, ww, ff)[1] * d_out).sum())

    eps = 1e-5
    for name in ("x", "w_router", "b_router", "w_in", "w_out", "norm_w"):
        base = x if name == "x" else w[name]
        grad = res["d_" + name]
        scale = np.max(np.abs(grad))
        for _ in range(8):
            i = tuple(int(rng.integers(0, n)) for n in base.shape)
            plus, minus = base.copy(), base.copy()
            plus[i] += eps
            minus[i] -= eps
            if name == "x":
                fd = (loss(plus, w, fw) - loss(minus, w, fw)) / (2 * eps)
            else:
                fd = (loss(x, dict(w, **{name: plus}), fw) - loss(x, dict(w, **{name: minus}), fw)) / (2 * eps)
            assert abs(fd - grad[i]) <= 1e-6 * scale + 1e-8, (name, i, fd, grad[i])
    for name in ("w_gate_up", "w_down", "norm_w"):
        base, grad = fw[name], fb["d_" + name]
        scale = np.max(np.abs(grad))
        for _ in range(6):
            i = tuple(int(rng.integers(0, n)) for n in base.shape)
            plus, minus = base.copy(), base.copy()
            plus[i] += eps
            minus[i] -= eps
            fd = (loss(x, w, dict(fw, **{name: plus})) - loss(x, w, dict(fw, **{name: minus}))) / (2 * eps)
            assert abs(fd - grad[i]) <= 1e-6 * scale + 1e-8, (name, i, fd, grad[i])


def test_scan_backward_closed_forms():
    """Constant coefficients: y_T depends on u_s through C . a^(T-s) . dt B (+ D at s = T), so a
    one-hot d_y at time T gives that as d_u; and the adjoint state after the last step back is
    d_h0 = C a^T.  The D gradient is sum(d_y * u)."""
    length, d_e, d_s = 9, 2, 3
    rng = np.random.default_rng(31)
    a = -rng.uniform(0.2, 1.5, (d_e, d_s))
    dt0, b0, c0 = 0.3, rng.standard_normal(d_s), rng.standard_normal(d_s)
    d_skip = rng.standard_normal(d_e)
    u = rng.standard_normal((1, length, d_e))
    dt = np.full((1, length, d_e), dt0)
    bm, cm = np.tile(b0, (1, length, 1)), np.tile(c0, (1, length, 1))
    t_hot = 6
    d_y = np.zeros((1, length, d_e))
    d_y[0, t_hot, :] = 1.0
    r = O.selective_scan_backward(u, dt, bm, cm, a, d_skip, d_y)
    decay = np.exp(dt0 * a)
    for s_ in range(length):
        want = np.zeros(d_e) if s_ > t_hot else dt0 * (c0 * b0 * decay ** (t_hot - s_)).sum(axis=1)
        if s_ == t_hot:
            want = want + d_skip
        assert np.allclose(r["d_u"][0, s_], want, rtol=1e-12, atol=1e-14)
    assert np.allclose(r["d_h0"][0], c0 * decay ** (t_hot + 1), rtol=1e-12)
    assert np.allclose(r["d_d"], u[0, t_hot], rtol=1e-13)
    # d_c[t] = d_y[t] * h[t]: only the hot step has one, and it is the forward state there
    _, h_hot = O.selective_scan(u[:, :t_hot + 1], dt[:, :t_hot + 1], bm[:, :t_hot + 1], cm[:, :t_hot + 1], a, d_skip)
    assert np.allclose(r["d_c"][0, t_hot], h_hot[0].sum(axis=0), rtol=1e-12)
    assert np.all(r["d_c"][0, :t_hot] == 0) and np.all(r["d_c"][0, t_hot + 1:] == 0)


def test_gate_backward_against_library_softmax():
    rng = np.random.default_rng(37)
    logits = rng.standard_normal((50, 6)) * 2
    d_gate = rng.standard_normal((50, 3))
    idx = O.topk_select(logits, 3)
    for mode in (0, 1):
        lt = torch.tensor(logits, requires_grad=True)
        p = torch.softmax(lt, dim=1)
        sel = torch.gather(p, 1, torch.as_tensor(idx.astype(np.int64)))
        gate = sel / sel.sum(1, keepdim=True) if mode == 1 else sel
        (gate * torch.tensor(d_gate)).sum().backward()
        got = O.gate_weights_backward(logits, idx, mode, d_gate)
        assert np.allclose(got, lt.grad.numpy(), rtol=1e-11, atol=1e-14)
        assert np.allclose(got.sum(axis=1), 0.0, atol=1e-13)          # softmax is shift-invariant
        if mode == 1:    # renormalised over all E selected = constant gate: no gradient at all
            full = O.gate_weights_backward(logits, O.topk_select(logits, 6), 1, rng.standard_normal((50, 6)) * 0 + 1.0)
            assert np.max(np.abs(full)) < 1e-13


def test_softplus_and_silu_against_library():
    v = np.linspace(-40, 40, 161)
    assert np.allclose(O.softplus(v), F.softplus(torch.from_numpy(v), threshold=1e9).numpy(), rtol=1e-13)
    assert np.allclose(O.silu(v), F.silu(torch.from_numpy(v)).numpy(), rtol=1e-13, atol=1e-300)


# --------------------------------------------------------------------------
# shapes: the parameter counts the paper prints
# --------------------------------------------------------------------------
def _layer_params(d_model, n_experts):
    cfg = RomConfig("count", 99, 1, 1, d_model, 2 * d_model, 16, 4, d_model // 16, n_experts, 1,
                    "fp32", 0, routed_xdt=False)
    # shapes only: count from the layout table of rom_synth without drawing big tensors
    e, ex = cfg.n_experts, cfg.n_experts_xdt
    dm, de, ds, k, r = cfg.d_model, cfg.d_inner, cfg.d_state, cfg.d_conv, cfg.dt_rank
    total = e * 2 * de * dm + de * k + de + ex * (r + 2 * ds) * de + ex * de * r + de + de * ds + de + e * dm * de
    active = total - (e - 1) * (2 * de * dm + dm * de)
    return active + dm, total + dm            # + one pre-norm weight vector per layer


def _fmt(count):
    return f"{count / 1e9:.1f}B" if count >= 1e9 else f"{round(count / 1e6)}M"


def test_parameter_counts_match_paper_tables():
    vocab = 32000                              # Llama-2 tokenizer as in the Samba setup the paper follows
    with open(os.path.join(GOLDEN, "param_counts.txt")) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    for n_layers, d_model, active_s, total_s in rows:
        n_layers, d_model = int(n_layers), int(d_model)
        act, tot = _layer_params(d_model, 8)
        emb = vocab * d_model + d_model        # tied embedding + final norm
        active, total = n_layers * act + emb, n_layers * tot + emb
        assert _fmt(active) == active_s, (d_model, active)
        got_total = _fmt(total)
        if total_s == "10B":                   # printed with two significant digits
            assert round(total / 1e9) == 10
        else:
            assert got_total == total_s, (d_model, total)


def test_synth_shapes_follow_layout_table():
    cfg = tiny_cfg(n_experts=3, routed_xdt=True)
    w = make_weights(cfg)
    assert w["w_in"].shape == (3, 2 * cfg.d_inner, cfg.d_model)
    assert w["w_x"].shape == (3, cfg.dt_rank + 2 * cfg.d_state, cfg.d_inner)
    assert w["w_dt"].shape == (3, cfg.d_inner, cfg.dt_rank)
    assert w["w_out"].shape == (3, cfg.d_model, cfg.d_inner)
    assert make_weights(tiny_cfg(routed_xdt=False))["w_x"].shape[0] == 1
