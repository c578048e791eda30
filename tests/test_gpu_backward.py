"""Parity of the HIP backward pass (rom_layer_backward through the C ABI) with the CPU oracle's
backward on the same seeded inputs and upstream gradient: every parameter gradient and d_x,
max|gpu - ref| / max|ref| <= 1e-4 (fp32) or 2e-2 (bf16) per tensor."""
import numpy as np
import pytest
import torch

from oracle import rom_oracle as O
from paper_2506_18145_amd import RomFfnMoe, RomLayer
from rom_synth import RomConfig, get_config, make_ffn_weights, make_input, make_weights, round_to_bf16

from gpu_util import TOL, check_routing, rel_err, to_np

pytestmark = pytest.mark.gpu

PARAMS = ("w_router", "b_router", "w_in", "conv_w", "conv_b", "w_x", "w_dt", "dt_bias", "A_log", "D", "w_out")


def small_cfg(**kw):
    base = dict(name="bwd", cfg_id=150, batch=2, seq_len=301, d_model=256, d_inner=512, d_state=16, d_conv=4,
                dt_rank=16, n_experts=4, top_k=1, dtype="bf16", gate_mode=0, weight_std=0.05)
    base.update(kw)
    base["name"] = "bwd-" + "-".join(f"{k}{v}" for k, v in kw.items()) if kw else "bwd"
    return RomConfig(**base)


def _d_out(cfg, shape):
    rng = np.random.Generator(np.random.Philox(1000 * cfg.cfg_id + 99))
    d = rng.standard_normal(shape, dtype=np.float32)
    return round_to_bf16(d) if cfg.dtype == "bf16" else d


def run_backward(cfg):
    w, x = make_weights(cfg), make_input(cfg)
    if w["b_router"] is None:
        w["b_router"] = np.zeros(cfg.n_experts, np.float32)        # so that its gradient is returned
    d_out = _d_out(cfg, x.shape)
    layer = RomLayer(cfg, w)
    xd, dd = layer.to_device(x), layer.to_device(d_out)
    d_x, grads = layer.backward(xd, dd)
    d_x2, grads2 = layer.backward(xd, dd)
    torch.cuda.synchronize()
    assert torch.equal(d_x, d_x2) and all(torch.equal(grads[k], grads2[k]) for k in grads), "not deterministic"
    # the routing decision of the call's own forward pass (left in the workspace), checked as in the forward tests
    B, L = cfg.batch, cfg.seq_len
    ws_keep = layer._ws
    layer._ws = layer._bwd_ws
    gpu = {k: to_np(layer.ws_view(k, B, L)) for k in ("expert_idx", "gate", "counts", "offsets", "perm", "inv_perm", "logits")}
    layer._ws = ws_keep
    idx, n_excl = check_routing(cfg, gpu, x, w)
    ref = O.rom_layer_backward(x, w, cfg.top_k, cfg.gate_mode, d_out, expert_idx=idx)
    tol = TOL[cfg.dtype]
    errs = {"d_x": rel_err(to_np(d_x), ref["d_x"])}
    for name in PARAMS:
        errs["d_" + name] = rel_err(to_np(grads["d_" + name]), ref["d_" + name])
    scales = {k: float(np.max(np.abs(ref[k]))) for k in errs}
    print(f"[{cfg.name}] excluded={n_excl} " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    print("    max|ref|: " + " ".join(f"{k}={v:.2e}" for k, v in scales.items()), flush=True)
    # one expert, or renormalised top-1 gates: the gate is the constant 1 and the router gets no gradient
    if cfg.n_experts == 1 or (cfg.gate_mode == 1 and cfg.top_k == 1):
        for k in ("d_w_router", "d_b_router"):
            assert scales[k] < 1e-9 and float(np.max(np.abs(to_np(grads[k])))) < 1e-6
            errs.pop(k)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, f"beyond tolerance {tol}: {bad}"
    return errs


def test_backward_cfg0_tiny_fp32():
    run_backward(get_config("cfg0"))


@pytest.mark.parametrize("kw", [
    dict(),
    dict(dtype="fp32"),
    dict(routed_xdt=False),
    dict(routed_xdt=False, dtype="fp32"),
    dict(n_experts=1),
    dict(gate_mode=1),
    dict(batch=1, seq_len=5),
    dict(batch=3, seq_len=64, n_experts=16),
    dict(batch=1, seq_len=1000, d_model=128, d_inner=256, dt_rank=8, n_experts=8),
    dict(d_model=264, d_inner=528, dt_rank=24, seq_len=130),          # sizes off the tile grids
    # top-K: per-slot input gradients summed over a token's slots, gate gradient per slot, router
    # through both gate modes
    dict(top_k=2, gate_mode=1),
    dict(top_k=2, gate_mode=0, dtype="fp32"),
    dict(top_k=2, gate_mode=1, routed_xdt=False),
    dict(top_k=3, gate_mode=0, n_experts=5, dt_rank=3, dtype="fp32", seq_len=77),
    dict(top_k=4, gate_mode=1, n_experts=4, batch=1, seq_len=40),
])
def test_backward_small(kw):
    run_backward(small_cfg(**kw))


@pytest.mark.parametrize("kw", [
    dict(batch=1, seq_len=5000, d_model=512, d_inner=1024, dt_rank=32, cfg_id=160),          # 256-row GEMM tiles
    dict(batch=2, seq_len=2050, d_model=512, d_inner=1024, dt_rank=64, routed_xdt=False, cfg_id=161),
    dict(batch=1, seq_len=4999, d_model=512, d_inner=1024, dt_rank=32, cfg_id=162,
         router_bias=(0.5, 0.0, 0.0, -50.0)),                                                # an expert without tokens
    dict(batch=1, seq_len=3000, d_model=512, d_inner=1024, dt_rank=64, top_k=2, gate_mode=1, n_experts=6, cfg_id=163),
])
def test_backward_medium(kw):
    run_backward(small_cfg(**kw))


@pytest.mark.parametrize("seed", [6, 8])
def test_backward_random_long_shapes(seed):
    """Seeded random narrow layers over more than 8192 tokens (the backward's launch shapes that only
    long inputs reach: router on the matrix pipe, 256-row tiles with ragged groups, time-chunked adjoint
    scan), widths on and off the 256 grid of the big weight-gradient kernel, any top-K."""
    import random
    rng = random.Random(seed)
    for i in range(6):
        E = rng.choice([2, 3, 5, 8, 12, 16])
        B = rng.choice([1, 1, 2, 3])
        L = rng.randint(8193, 14000) // B + 1
        kw = dict(name=f"random-long-bwd-{seed}-{i}", cfg_id=1200 + i, batch=B, seq_len=L,
                  d_model=rng.choice([32 * rng.randint(2, 10), 8 * rng.randint(8, 40), 256]),
                  d_inner=rng.choice([16 * rng.randint(2, 16), 256]), d_state=16, d_conv=4,
                  dt_rank=rng.choice([3, 8, 16, 32]), n_experts=E, top_k=rng.randint(1, min(E, 3)),
                  dtype=rng.choice(["bf16", "bf16", "fp32"]), gate_mode=rng.choice([0, 1]),
                  routed_xdt=rng.choice([True, True, False]), weight_std=0.05)
        cfg = RomConfig(**kw)
        print(f"[{cfg.name}] B={B} L={L} Dm={cfg.d_model} De={cfg.d_inner} R={cfg.dt_rank} E={E} K={cfg.top_k} "
              f"{cfg.dtype} gate_mode={cfg.gate_mode} routed_xdt={cfg.routed_xdt}", flush=True)
        run_backward(cfg)


@pytest.mark.parametrize("kw", [dict(), dict(top_k=2, gate_mode=1), dict(dtype="fp32", routed_xdt=False),
                                dict(batch=1, seq_len=3000, d_model=512, d_inner=1024, dt_rank=64, top_k=2, gate_mode=1,
                                     n_experts=6, cfg_id=163)])
def test_backward_saved_matches_backward_bit_for_bit(kw):
    """rom_layer_backward_saved after the caller's own rom_layer_forward on the backward workspace gives
    the bits of rom_layer_backward (which recomputes the forward pass itself), and the forward's out is
    that of a plain forward call."""
    cfg = small_cfg(**kw)
    w, x = make_weights(cfg), make_input(cfg)
    layer = RomLayer(cfg, w)
    xd = layer.to_device(x)
    dd = layer.to_device(_d_out(cfg, x.shape))
    d_x, grads = layer.backward(xd, dd)
    out = layer.forward_for_backward(xd)
    d_x2, grads2 = layer.backward(xd, dd, saved=True)
    out_plain = layer.forward(xd)
    torch.cuda.synchronize()
    assert torch.equal(out, out_plain)
    assert torch.equal(d_x, d_x2)
    for k in grads:
        assert torch.equal(grads[k], grads2[k]), k


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3"])
def test_backward_full_size(name):
    run_backward(get_config(name))


@pytest.mark.parametrize("kw,scale", [
    (dict(cfg_id=170), 1.7),
    (dict(cfg_id=171, dtype="fp32", seq_len=77), 0.6),
    (dict(cfg_id=174, weight_std=0.1), 1.2),                      # a branch of the size of the skip term
    (dict(cfg_id=172, top_k=2, gate_mode=1, d_model=264, d_inner=528, dt_rank=24, seq_len=130), 1.3),    # off the tile grids
    (dict(cfg_id=173, batch=1, seq_len=5000, d_model=512, d_inner=1024, dt_rank=32), 1.4),                 # big-tile kernels
])
def test_block_backward(kw, scale):
    """rom_block_backward (out = x + RoM(RMSNorm(x))) against the oracle's block backward: d_x, the norm
    scale's gradient and every parameter gradient."""
    cfg = small_cfg(**kw)
    w, x = make_weights(cfg), make_input(cfg) * np.float32(scale)      # off unit RMS, so that 1/rms matters
    x = round_to_bf16(x) if cfg.dtype == "bf16" else x
    if w["b_router"] is None:
        w["b_router"] = np.zeros(cfg.n_experts, np.float32)
    rng = np.random.default_rng(cfg.cfg_id)
    w["norm_w"] = (1.0 + 0.3 * rng.standard_normal(cfg.d_model)).astype(np.float32)
    d_out = _d_out(cfg, x.shape)
    layer = RomLayer(cfg, w)
    xd, dd = layer.to_device(x), layer.to_device(d_out)
    d_x, grads = layer.block_backward(xd, dd, eps=1e-5)
    d_x2, grads2 = layer.block_backward(xd, dd, eps=1e-5)
    torch.cuda.synchronize()
    assert torch.equal(d_x, d_x2) and all(torch.equal(grads[k], grads2[k]) for k in grads), "not deterministic"
    # the expert choice of the call's own forward pass (on the normalised input), left in its workspace
    B, L = cfg.batch, cfg.seq_len
    ws_keep = layer._ws
    layer._ws = layer._blk_bwd_ws
    gpu = {k: to_np(layer.ws_view(k, B, L)) for k in ("expert_idx", "gate", "counts", "offsets", "perm", "inv_perm", "logits")}
    layer._ws = ws_keep
    # the materialised norm against the oracle's; the router normalises the raw x itself, as the forward block does
    xn = to_np(layer.block_backward_xn(B, L))
    assert rel_err(xn, O.rms_norm(x, w["norm_w"], 1e-5)) <= (2.0 ** -8 if cfg.dtype == "bf16" else 1e-6)
    idx, n_excl = check_routing(cfg, gpu, x, w, block=True)
    ref = O.rom_block_backward(x, w, cfg.top_k, cfg.gate_mode, d_out, 1e-5, expert_idx=idx)
    tol = TOL[cfg.dtype]
    errs = {"d_x": rel_err(to_np(d_x), ref["d_x"]), "d_norm_w": rel_err(to_np(grads["d_norm_w"]), ref["d_norm_w"])}
    # the norm's part of d_x alone: the skip term must not hide it
    got_branch = to_np(d_x).astype(np.float64) - np.asarray(d_out, np.float64)
    want_branch = ref["d_x"] - np.asarray(d_out, np.float64)
    ulp = 2.0 ** -8 if cfg.dtype == "bf16" else 2.0 ** -24
    slack = ulp * np.max(np.abs(ref["d_x"])) / np.max(np.abs(want_branch))
    errs["d_x-d_out"] = max(rel_err(got_branch, want_branch) - slack, 0.0)
    for name in PARAMS:
        errs["d_" + name] = rel_err(to_np(grads["d_" + name]), ref["d_" + name])
    ratio = float(np.max(np.abs(want_branch)) / np.max(np.abs(d_out)))
    print(f"[block {cfg.name}] excluded={n_excl} branch/skip={ratio:.2f} " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()),
          flush=True)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, f"beyond tolerance {tol}: {bad}"


def _pack_rows(g, d_ff):
    """Plain row order [gate 0..d_ff) | up 0..d_ff) -> the library's blocks of 8 gate + 8 up rows (axis 1)."""
    b = d_ff // 8
    gate, up = g[:, :d_ff].reshape(g.shape[0], b, 8, -1), g[:, d_ff:].reshape(g.shape[0], b, 8, -1)
    return np.concatenate([gate, up], axis=2).reshape(g.shape[0], 2 * d_ff, -1)


def _ffn_backward_case(cfg, d_ff, pre_norm, add_skip):
    w, fw, x = make_weights(cfg), make_ffn_weights(cfg, d_ff), make_input(cfg) * np.float32(1.3)
    x = round_to_bf16(x) if cfg.dtype == "bf16" else x
    layer = RomLayer(cfg, w)
    ffn = RomFfnMoe(layer, d_ff, fw, eps=1e-5)
    B, L = cfg.batch, cfg.seq_len
    N = B * L
    xd = layer.to_device(x)
    d_out = _d_out(cfg, x.shape)
    dd = layer.to_device(d_out)
    routing = layer.route(xd.view(N, -1))
    d_x, d_gate, grads = ffn.backward(xd, routing, dd, pre_norm=pre_norm, add_skip=add_skip)
    d_x2, d_gate2, grads2 = ffn.backward(xd, routing, dd, pre_norm=pre_norm, add_skip=add_skip)
    torch.cuda.synchronize()
    assert torch.equal(d_x, d_x2) and torch.equal(d_gate, d_gate2) and all(torch.equal(grads[k], grads2[k]) for k in grads)
    gpu = {k: to_np(routing[k]) for k in ("expert_idx", "gate", "counts", "offsets", "perm", "inv_perm", "logits")}
    idx, _ = check_routing(cfg, gpu, x, w)
    gate = O.gate_weights(O.router_logits(x.reshape(N, -1), w["w_router"], w.get("b_router")), idx, cfg.gate_mode)
    ref = O.ffn_moe_backward(x.reshape(N, -1), fw["w_gate_up"], fw["w_down"], idx, gate, d_out.reshape(N, -1),
                             fw["norm_w"] if pre_norm else None, 1e-5, skip=add_skip)
    errs = {"d_x": rel_err(to_np(d_x).reshape(N, -1), ref["d_x"]), "d_gate": rel_err(to_np(d_gate), ref["d_gate"]),
            "d_w_gate_up": rel_err(to_np(grads["d_w_gate_up"]), _pack_rows(ref["d_w_gate_up"], d_ff)),
            "d_w_down": rel_err(to_np(grads["d_w_down"]), ref["d_w_down"])}
    if pre_norm:
        errs["d_norm_w"] = rel_err(to_np(grads["d_norm_w"]), ref["d_norm_w"])
    if add_skip:        # the branch alone: the skip term must not hide it
        got = to_np(d_x).reshape(N, -1).astype(np.float64) - d_out.reshape(N, -1)
        want = ref["d_x"] - d_out.reshape(N, -1)
        ulp = 2.0 ** -8 if cfg.dtype == "bf16" else 2.0 ** -24
        errs["d_x-d_out"] = max(rel_err(got, want) - ulp * np.max(np.abs(ref["d_x"])) / np.max(np.abs(want)), 0.0)
    print(f"[ffn bwd {cfg.name} d_ff={d_ff} norm={pre_norm} skip={add_skip}] "
          + " ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    bad = {k: v for k, v in errs.items() if not v <= TOL[cfg.dtype]}
    assert not bad, bad


@pytest.mark.parametrize("kw,d_ff,pre_norm,add_skip", [
    (dict(cfg_id=180), 512, False, False),
    (dict(cfg_id=181), 512, True, True),
    (dict(cfg_id=182, dtype="fp32"), 272, True, True),
    (dict(cfg_id=183, dtype="fp32", top_k=2, gate_mode=1), 256, False, True),
    (dict(cfg_id=184, top_k=2, gate_mode=1), 400, True, False),
    (dict(cfg_id=185, top_k=3, gate_mode=0, n_experts=16), 512, True, True),
    (dict(cfg_id=186, batch=3, seq_len=1), 512, True, True),
    (dict(cfg_id=187, batch=1, seq_len=1500, d_model=264), 528, True, True),                       # off the tile grids
    (dict(cfg_id=188, batch=1, seq_len=5000, d_model=512, d_inner=1024, dt_rank=32), 1024, True, True),   # big-tile kernels
    (dict(cfg_id=189, batch=1, seq_len=4999, d_model=512, d_inner=1024, dt_rank=32,
          router_bias=(0.5, 0.0, 0.0, -50.0)), 768, False, True),                                  # an expert without tokens
])
def test_ffn_moe_backward(kw, d_ff, pre_norm, add_skip):
    _ffn_backward_case(small_cfg(weight_std=0.08, **kw), d_ff, pre_norm, add_skip)


def test_ffn_moe_backward_full_size():
    _ffn_backward_case(get_config("cfg2"), 4096, True, True)
    _ffn_backward_case(get_config("cfg1"), 2048, True, False)      # and a branch that no skip term can mask


@pytest.mark.parametrize("kw", [dict(cfg_id=190), dict(cfg_id=191, dtype="fp32", seq_len=90),
                                dict(cfg_id=192, top_k=2, gate_mode=1, n_experts=8)])
def test_hybrid_pair_backward_chain(kw):
    """A RoM block, then an FFN-MoE block on its routing decision (pre-norm + skip both): the training
    step's backward chain rom_ffn_moe_backward -> rom_block_backward(d_gate_ffn = the FFN's gate
    gradient), against the oracle's chain on the same expert choice.  The router's gradient is where a
    dropped or mis-scaled hand-over would show."""
    cfg = small_cfg(weight_std=0.08, **kw)
    d_ff = 384
    w, fw, x = make_weights(cfg), make_ffn_weights(cfg, d_ff), make_input(cfg)
    if w["b_router"] is None:
        w["b_router"] = np.zeros(cfg.n_experts, np.float32)
    rng = np.random.default_rng(cfg.cfg_id)
    w["norm_w"] = (1.0 + 0.3 * rng.standard_normal(cfg.d_model)).astype(np.float32)
    layer = RomLayer(cfg, w)
    ffn = RomFfnMoe(layer, d_ff, fw, eps=1e-5)
    B, L = cfg.batch, cfg.seq_len
    N = B * L
    xd = layer.to_device(x)
    d_out = _d_out(cfg, x.shape)
    dd = layer.to_device(d_out)
    # forward of the pair (the block leaves its routing decision in the layer's workspace)
    mid = layer.block_forward(xd, eps=1e-5)
    routing = {k: layer.ws_view(k, B, L).clone() for k in ("offsets", "perm", "inv_perm", "gate", "expert_idx")}
    # backward: FFN first, its input gradient and gate gradient go to the block
    d_mid, d_gate_ffn, fg = ffn.backward(mid.view(N, -1), routing, dd.view(N, -1), pre_norm=True, add_skip=True)
    d_x, grads = layer.block_backward(xd, d_mid.view(B, L, -1), eps=1e-5, d_gate_ffn=d_gate_ffn)
    torch.cuda.synchronize()
    idx = to_np(routing["expert_idx"])
    # the block backward recomputes the routing on its materialised norm: it must agree with the forward's
    ws_keep = layer._ws
    layer._ws = layer._blk_bwd_ws
    assert np.array_equal(to_np(layer.ws_view("expert_idx", B, L)), idx)
    layer._ws = ws_keep
    blk = O.rom_block_forward(x, w, cfg.top_k, cfg.gate_mode, 1e-5, expert_idx=idx)
    fb = O.ffn_moe_backward(blk["out"].reshape(N, -1), fw["w_gate_up"], fw["w_down"], idx, blk["gate"],
                            d_out.reshape(N, -1), fw["norm_w"], 1e-5, skip=True)
    ref = O.rom_block_backward(x, w, cfg.top_k, cfg.gate_mode, fb["d_x"].reshape(x.shape), 1e-5, expert_idx=idx,
                               d_gate_extra=fb["d_gate"])
    alone = O.rom_block_backward(x, w, cfg.top_k, cfg.gate_mode, fb["d_x"].reshape(x.shape), 1e-5, expert_idx=idx)
    errs = {"d_x": rel_err(to_np(d_x), ref["d_x"]), "d_norm_w": rel_err(to_np(grads["d_norm_w"]), ref["d_norm_w"]),
            "d_gate_ffn": rel_err(to_np(d_gate_ffn), fb["d_gate"]),
            "ffn d_w_down": rel_err(to_np(fg["d_w_down"]), fb["d_w_down"])}
    for name in PARAMS:
        errs["d_" + name] = rel_err(to_np(grads["d_" + name]), ref["d_" + name])
    share = float(np.max(np.abs(ref["d_w_router"] - alone["d_w_router"])) / np.max(np.abs(ref["d_w_router"])))
    print(f"[pair {cfg.name}] ffn share of d_w_router={share:.2f} " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()),
          flush=True)
    assert share > 0.1, "the FFN's gate gradient is too small here to test the hand-over"
    bad = {k: v for k, v in errs.items() if not v <= TOL[cfg.dtype]}
    assert not bad, bad


@pytest.mark.parametrize("kw", [dict(cfg_id=195), dict(cfg_id=196, top_k=2, gate_mode=1), dict(cfg_id=197, dtype="fp32", seq_len=70),
                                dict(cfg_id=199, weight_std=0.1),
                                dict(cfg_id=198, batch=1, seq_len=5000, d_model=512, d_inner=1024, dt_rank=32)])
def test_block_training_step_halves(kw):
    """rom_block_forward_train + rom_block_backward_saved: the same gradients as rom_block_backward, bit
    for bit, and an output that is the block's (against the oracle; against rom_block_forward up to the
    rounding of the materialised norm)."""
    cfg = small_cfg(**kw)
    w, x = make_weights(cfg), make_input(cfg) * np.float32(1.3)
    x = round_to_bf16(x) if cfg.dtype == "bf16" else x
    if w["b_router"] is None:
        w["b_router"] = np.zeros(cfg.n_experts, np.float32)
    layer = RomLayer(cfg, w)
    xd, dd = layer.to_device(x), layer.to_device(_d_out(cfg, x.shape))
    B, L = cfg.batch, cfg.seq_len
    d_x, grads = layer.block_backward(xd, dd, eps=1e-5)
    d_x, grads = d_x.clone(), {k: v.clone() for k, v in grads.items()}
    layer._blk_bwd_ws.fill_(0xA5)                      # nothing may survive from the call above
    out = layer.block_forward_train(xd, eps=1e-5)
    idx = to_np(layer.train_routing_view("expert_idx", B, L))
    d_x2, grads2 = layer.block_backward(xd, dd, eps=1e-5, saved=True)
    fused = layer.block_forward(xd, eps=1e-5)
    torch.cuda.synchronize()
    assert torch.equal(d_x, d_x2)
    for k in grads:
        assert torch.equal(grads[k], grads2[k]), k
    ref = O.rom_block_forward(x, w, cfg.top_k, cfg.gate_mode, 1e-5, expert_idx=idx)
    tol = TOL[cfg.dtype]
    got_branch = to_np(out).astype(np.float64) - np.asarray(x, np.float64)
    ulp = 2.0 ** -8 if cfg.dtype == "bf16" else 2.0 ** -24
    slack = ulp * np.max(np.abs(ref["out"])) / np.max(np.abs(ref["branch"]))
    errs = {"out": rel_err(to_np(out), ref["out"]), "branch": max(rel_err(got_branch, ref["branch"]) - slack, 0.0),
            "vs fused": rel_err(to_np(out), to_np(fused))}
    print(f"[train halves {cfg.name}] " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    assert all(v <= tol for v in errs.values()), errs


@pytest.mark.parametrize("kw,d_ff,pre_norm,add_skip", [
    (dict(cfg_id=200), 512, True, True),
    (dict(cfg_id=201, top_k=2, gate_mode=1), 400, True, False),
    (dict(cfg_id=202, dtype="fp32", seq_len=90), 272, False, True),
    (dict(cfg_id=203, batch=1, seq_len=5000, d_model=512, d_inner=1024, dt_rank=32), 1024, True, True),
])
def test_ffn_training_step_halves(kw, d_ff, pre_norm, add_skip):
    """rom_ffn_moe_forward_train + rom_ffn_moe_backward_saved: the gradients of rom_ffn_moe_backward bit
    for bit, and the layer's output (against the oracle and against the fused forward)."""
    cfg = small_cfg(weight_std=0.08, **kw)
    w, fw, x = make_weights(cfg), make_ffn_weights(cfg, d_ff), make_input(cfg) * np.float32(1.3)
    x = round_to_bf16(x) if cfg.dtype == "bf16" else x
    layer = RomLayer(cfg, w)
    ffn = RomFfnMoe(layer, d_ff, fw, eps=1e-5)
    N = cfg.batch * cfg.seq_len
    xd = layer.to_device(x).view(N, -1)
    dd = layer.to_device(_d_out(cfg, x.shape)).view(N, -1)
    routing = layer.route(xd)
    d_x, d_gate, grads = ffn.backward(xd, routing, dd, pre_norm=pre_norm, add_skip=add_skip)
    d_x, d_gate, grads = d_x.clone(), d_gate.clone(), {k: v.clone() for k, v in grads.items()}
    ffn._bwd_ws.fill_(0xA5)
    out = ffn.forward_train(xd, routing, pre_norm=pre_norm, add_skip=add_skip)
    d_x2, d_gate2, grads2 = ffn.backward(xd, routing, dd, pre_norm=pre_norm, add_skip=add_skip, saved=True)
    fused = ffn.forward(xd, routing, pre_norm=pre_norm, add_skip=add_skip)
    torch.cuda.synchronize()
    assert torch.equal(d_x, d_x2) and torch.equal(d_gate, d_gate2)
    for k in grads:
        assert torch.equal(grads[k], grads2[k]), k
    idx, gate = to_np(routing["expert_idx"]), to_np(routing["gate"])
    ref = O.ffn_moe_forward(x.reshape(N, -1), fw["w_gate_up"], fw["w_down"], idx, gate, fw["norm_w"] if pre_norm else None,
                            1e-5, skip=add_skip)
    errs = {"out": rel_err(to_np(out), ref), "vs fused": rel_err(to_np(out), to_np(fused))}
    print(f"[ffn train halves {cfg.name}] " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    assert all(v <= TOL[cfg.dtype] for v in errs.values()), errs
