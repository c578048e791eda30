"""GPU parity of the pre-norm residual blocks around the Mamba2 and Gated DeltaNet layers
(rom_mamba2_block_forward, rom_gdn_block_forward) against the CPU oracle: out = x + layer(RMSNorm(x)),
the oracle's norm and layer composed as written.  The branch (out - x) is compared on its own, so that
an error in it cannot hide behind the skip term; tolerance 2e-2 of the tensor maximum (bf16)."""
import numpy as np
import pytest
import torch

from gpu_util import BLOCK_EPS, TOL, check_routing, rel_err, to_np
from oracle import rom_gdn_oracle as G
from oracle import rom_mamba2_oracle as M
from oracle import rom_oracle as O
from paper_2506_18145_amd import (RomGdnLayer, RomMamba2Layer, rom_fold_norm_rows, rom_gdn_block_forward,
                                  rom_mamba2_block_forward)
from rom_synth import (get_gdn_config, get_mamba2_config, make_gdn_input, make_gdn_weights, make_mamba2_input,
                       make_mamba2_weights, round_to_bf16)

pytestmark = pytest.mark.gpu

EPS = 1e-5
ROUTING = ("expert_idx", "gate", "counts", "offsets", "perm", "inv_perm", "logits")


def _pre_norm_weight(cfg):
    rng = np.random.default_rng(1000 + cfg.cfg_id)
    return (1.0 + 0.3 * rng.standard_normal(cfg.d_model)).astype(np.float32)


def _run_block(kind, cfg, scale, with_states):
    if kind == "mamba2":
        w_np, x_np = make_mamba2_weights(cfg), make_mamba2_input(cfg)
        layer = RomMamba2Layer(cfg, w_np, eps=EPS)
    else:
        w_np, x_np = make_gdn_weights(cfg), make_gdn_input(cfg)
        layer = RomGdnLayer(cfg, w_np, eps=EPS)
    x_np = round_to_bf16(x_np * np.float32(scale))      # off unit RMS, so that the 1/rms factor matters
    pre_w = _pre_norm_weight(cfg)
    pre_w_d = torch.from_numpy(pre_w).cuda()
    x = layer.to_device(x_np)
    B, L = cfg.batch, cfg.seq_len
    cs_np = ss_np = cs = ss = None
    if with_states:
        rng = np.random.default_rng(cfg.cfg_id)
        cshape, sshape = layer.state_shapes(B)
        cs_np = rng.standard_normal(cshape).astype(np.float32)
        ss_np = (0.5 * rng.standard_normal(sshape)).astype(np.float32)
        cs, ss = torch.from_numpy(cs_np).cuda(), torch.from_numpy(ss_np).cuda()
    out, cs_out, ss_out = layer.block_forward(x, pre_w_d, BLOCK_EPS, cs, ss, return_states=True)
    torch.cuda.synchronize()
    gpu = {name: to_np(layer.ws_view(name, B, L)) for name in ROUTING}
    gpu.update(out=to_np(out), conv_state=to_np(cs_out), ssm_state=to_np(ss_out))
    # routing: the router sees the normalised input
    idx, n_excl = check_routing(cfg, gpu, x_np, dict(w_np, norm_w=pre_w), block=True)
    xn = O.rms_norm(x_np, pre_w, BLOCK_EPS)
    s0 = None if ss_np is None else ss_np.transpose(0, 1, 3, 2)      # the oracles keep the state transposed
    if kind == "mamba2":
        ref = M.rom_mamba2_forward(xn, w_np, cfg.top_k, cfg.gate_mode, cfg.headdim, EPS, expert_idx=idx,
                                   conv_state=cs_np, ssm_state=s0)
    else:
        ref = G.rom_gdn_forward(xn, w_np, cfg.top_k, cfg.gate_mode, cfg.n_heads, cfg.d_k, EPS, expert_idx=idx,
                                conv_state=cs_np, ssm_state=s0)
    branch = ref["out"]
    want = np.asarray(x_np, np.float64) + branch
    got_branch = gpu["out"].astype(np.float64) - np.asarray(x_np, np.float64)
    # the output's own rounding (2^-8 |out|) is allowed on top of the branch's tolerance
    slack = 2.0 ** -8 * np.max(np.abs(want)) / np.max(np.abs(branch))
    errs = {"out": rel_err(gpu["out"], want), "branch": max(rel_err(got_branch, branch) - slack, 0.0),
            "conv_state": rel_err(gpu["conv_state"], ref["conv_state"]),
            "ssm_state": rel_err(gpu["ssm_state"], ref["ssm_state"].transpose(0, 1, 3, 2))}
    ratio = float(np.max(np.abs(branch)) / np.max(np.abs(x_np)))
    print(f"[{kind} block {cfg.name}] B={B} L={L} K={cfg.top_k} excluded={n_excl} branch/x={ratio:.2f} "
          + " ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    assert ratio > 0.05, "the branch is too small against the skip term for this case to test it"
    bad = {k: v for k, v in errs.items() if not v <= TOL["bf16"]}
    assert not bad, bad
    return layer, x, pre_w_d, out


# weights large enough that the branch is of the size of the skip term: at the paper-like
# initialisations an error in the fused projections would hide behind x
@pytest.mark.parametrize("kind,name,over,scale,states", [
    ("mamba2", "m2_small", dict(cfg_id=60, weight_std=0.05), 1.7, False),                         # top-1: row scale and skip in the GEMMs
    ("mamba2", "m2_mid", dict(batch=1, seq_len=1100, cfg_id=61, weight_std=0.05), 0.6, True),      # top-2: slot sum and combine; segments
    ("mamba2", "m2_cfg2", dict(batch=1, seq_len=4096, cfg_id=62, weight_std=0.03), 1.3, False),    # the 256-row tiles
    ("gdn", "gdn_small", dict(cfg_id=63, weight_std=0.1), 1.7, False),
    ("gdn", "gdn_mid", dict(batch=1, seq_len=1100, cfg_id=64, weight_std=0.04), 0.6, True),
    ("gdn", "gdn_cfg2", dict(batch=1, seq_len=4096, cfg_id=65, weight_std=0.04), 1.3, False),
])
def test_variant_block_matches_oracle(kind, name, over, scale, states):
    cfg = (get_mamba2_config if kind == "mamba2" else get_gdn_config)(name, **over)
    _run_block(kind, cfg, scale, states)


@pytest.mark.parametrize("kind", ["mamba2", "gdn"])
def test_variant_block_is_the_layer_on_a_normalised_input(kind):
    """Property at any size: the block equals x + layer(RMSNorm(x)) computed by the library's own
    layer call on an input normalised beforehand, up to the rounding of that input to bf16."""
    cfg = (get_mamba2_config("m2_small", cfg_id=66, weight_std=0.05) if kind == "mamba2" else get_gdn_config("gdn_small", cfg_id=66, weight_std=0.1))
    layer, x, pre_w, out = _run_block(kind, cfg, 1.4, False)
    xf = x.float()
    xn = (xf * torch.rsqrt((xf * xf).mean(-1, keepdim=True) + BLOCK_EPS) * pre_w).to(torch.bfloat16)
    want = xf + layer.forward(xn).float()
    torch.cuda.synchronize()
    assert rel_err(to_np(out), to_np(want)) <= TOL["bf16"]


def test_fold_norm_rows_scales_the_columns():
    rng = np.random.default_rng(5)
    w = torch.from_numpy(rng.standard_normal((37, 200)).astype(np.float32)).cuda()
    s = torch.from_numpy(rng.standard_normal(200).astype(np.float32)).cuda()
    for dt, code in ((torch.float32, 0), (torch.bfloat16, 1)):
        src = w.to(dt)
        dst = torch.empty_like(src)
        rom_fold_norm_rows(code, src, s, dst, 37, 200)
        torch.cuda.synchronize()
        assert torch.equal(dst, (src.float() * s).to(dt))


@pytest.mark.parametrize("kind", ["mamba2", "gdn"])
def test_variant_block_decodes_one_token_at_a_time(kind):
    """The block call with L = 1 and the states passed as both input and output is the block's
    recurrent step: 40 steps against the oracle's block on the whole sequence."""
    if kind == "mamba2":
        cfg = get_mamba2_config("m2_small", batch=3, seq_len=40, cfg_id=67, weight_std=0.05)
        w_np, x_np = make_mamba2_weights(cfg), make_mamba2_input(cfg)
        layer = RomMamba2Layer(cfg, w_np, eps=EPS)
    else:
        cfg = get_gdn_config("gdn_small", batch=3, seq_len=40, cfg_id=67, weight_std=0.1)
        w_np, x_np = make_gdn_weights(cfg), make_gdn_input(cfg)
        layer = RomGdnLayer(cfg, w_np, eps=EPS)
    x_np = round_to_bf16(x_np * np.float32(1.3))
    pre_w = _pre_norm_weight(cfg)
    pre_w_d = torch.from_numpy(pre_w).cuda()
    x = layer.to_device(x_np)
    B, L = cfg.batch, cfg.seq_len
    cshape, sshape = layer.state_shapes(B)
    cs = torch.zeros(cshape, dtype=torch.float32, device="cuda")
    ss = torch.zeros(sshape, dtype=torch.float32, device="cuda")
    outs, idxs = [], []
    for t in range(L):
        xt = x[:, t:t + 1].contiguous()
        out = torch.empty_like(xt)
        fn = rom_mamba2_block_forward if kind == "mamba2" else rom_gdn_block_forward
        fn(layer.dims, layer.block_weights(pre_w_d), pre_w_d, BLOCK_EPS, xt, B, 1, layer.eps, cs, ss, out, cs, ss,
           layer.workspace(B, 1))
        outs.append(to_np(out)[:, 0])
        idxs.append(to_np(layer.ws_view("expert_idx", B, 1)).reshape(B, -1))
    torch.cuda.synchronize()
    got = np.stack(outs, axis=1)
    idx = np.stack(idxs, axis=1).reshape(B * L, -1)
    xn = O.rms_norm(x_np, pre_w, BLOCK_EPS)
    logits = O.router_logits(xn.reshape(B * L, -1), w_np["w_router"], w_np.get("b_router"))
    close = O.topk_margin(logits, cfg.top_k) < 1e-5
    assert np.array_equal(idx[~close], O.topk_select(logits, cfg.top_k)[~close])
    if kind == "mamba2":
        ref = M.rom_mamba2_forward(xn, w_np, cfg.top_k, cfg.gate_mode, cfg.headdim, EPS, expert_idx=idx)
    else:
        ref = G.rom_gdn_forward(xn, w_np, cfg.top_k, cfg.gate_mode, cfg.n_heads, cfg.d_k, EPS, expert_idx=idx)
    want = np.asarray(x_np, np.float64) + ref["out"]
    errs = {"out": rel_err(got, want), "conv_state": rel_err(to_np(cs), ref["conv_state"]),
            "ssm_state": rel_err(to_np(ss), ref["ssm_state"].transpose(0, 1, 3, 2))}
    print(f"[{kind} block steps] " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    assert all(v <= TOL["bf16"] for v in errs.values()), errs
