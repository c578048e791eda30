"""Workload table and seeded tensor generators for the RoM layer.

Shapes follow the paper's Mamba parameterisation (Sec. 3.1: d_e = 2 d_m,
d_r = d_m / 16, d_s = 16, k = 4) and its 8-expert top-1 models up to
d_model = 2048 at 16K context (Sec. 5.2, Table 5).  The paper's inputs are
hidden states of trained language models; seeded random tensors of the same
shapes stand in for them.

Array layouts produced here (row-major, "out-features major" like a linear
layer's weight):

    w_router [E, d_model]          b_router [E] (fp32) or None
    w_in     [E, 2*d_inner, d_model]   rows [0,d_inner) feed the conv branch,
                                       rows [d_inner, 2*d_inner) the gate branch
    conv_w   [d_inner, d_conv] (fp32)  conv_b [d_inner] (fp32)
    w_x      [E_x, dt_rank + 2*d_state, d_inner]   rows = dt_low | B | C
    w_dt     [E_x, d_inner, dt_rank]
    dt_bias  [d_inner] (fp32)   A_log [d_inner, d_state] (fp32)   D [d_inner] (fp32)
    w_out    [E, d_model, d_inner]
    norm_w   [d_model] (fp32)      scale of the pre-norm of the residual block

All arrays are returned as float32.  For bf16 workloads the tensors that the
layer stores in bf16 (x, w_router, w_in, w_x, w_dt, w_out) hold values that
are exactly representable in bf16, so the oracle (which upcasts to fp64) and
the GPU path (which receives the 16-bit patterns) see identical numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np


@dataclass(frozen=True)
class RomConfig:
    name: str
    cfg_id: int          # seed base = 1000 * cfg_id + tensor id
    batch: int
    seq_len: int         # L (for the step workload: number of consecutive steps)
    d_model: int
    d_inner: int
    d_state: int
    d_conv: int
    dt_rank: int
    n_experts: int
    top_k: int
    dtype: str           # "fp32" | "bf16"
    gate_mode: int       # 0: softmax over all experts, masked; 1: renormalised over the K selected
    routed_xdt: bool = True
    weight_std: float = 0.02
    rms_norm_x: bool = False
    router_bias: Optional[tuple] = None
    step: bool = False   # single-token recurrent workload

    @property
    def n_experts_xdt(self) -> int:
        return self.n_experts if self.routed_xdt else 1

    @property
    def n_tokens(self) -> int:
        return self.batch * (1 if self.step else self.seq_len)


# Router bias of the skewed workload.  With x ~ N(0,1) and W_r ~ N(0, 0.02) at
# d_model = 2048 the logits are ~N(0, 0.905^2); adding +5.0 to expert 0 puts it
# in (nearly) every token's top-2 (about half of all slots) and +0.92 to experts
# 1..3 gives each about a tenth of the slots; the other twelve share the rest.
_SKEW_BIAS = (5.0, 0.92, 0.92, 0.92) + (0.0,) * 12

CONFIGS: Dict[str, RomConfig] = {
    # 0: tiny fp32 correctness case
    "cfg0": RomConfig("cfg0", 0, 1, 64, 64, 128, 16, 4, 4, 4, 1, "fp32", 0),
    # 1: mid bf16 case
    "cfg1": RomConfig("cfg1", 1, 4, 4096, 1024, 2048, 16, 4, 64, 8, 1, "bf16", 0),
    # 2: headline, 1.3B-active-class layer at 16K context
    "cfg2": RomConfig("cfg2", 2, 1, 16384, 2048, 4096, 16, 4, 128, 8, 1, "bf16", 0,
                      weight_std=0.02 / float(np.sqrt(2 * 48)), rms_norm_x=True),
    # 3: skewed routing, 16 experts top-2, renormalised gates
    "cfg3": RomConfig("cfg3", 3, 2, 8192, 2048, 4096, 16, 4, 128, 16, 2, "bf16", 1,
                      router_bias=_SKEW_BIAS),
    # 4: recurrent decode, 256 sequences x 512 steps
    "cfg4": RomConfig("cfg4", 4, 256, 512, 2048, 4096, 16, 4, 128, 8, 1, "bf16", 0, step=True),
}


def get_config(name: str, **overrides) -> RomConfig:
    cfg = CONFIGS[name]
    return replace(cfg, **overrides) if overrides else cfg


# --------------------------------------------------------------------------
# bf16 storage helpers (round-to-nearest-even on the upper 16 bits of fp32)
# --------------------------------------------------------------------------
def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of `a` rounded to bf16 (nearest even). Finite inputs only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float32 array whose values are `a` rounded to bf16."""
    return (bf16_bits(a).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(cfg: RomConfig, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(1000 * cfg.cfg_id + tensor_id))


def _normal(cfg: RomConfig, tensor_id: int, shape, std: float) -> np.ndarray:
    out = _rng(cfg, tensor_id).standard_normal(shape, dtype=np.float32)
    out *= np.float32(std)
    return out


def _store(cfg: RomConfig, a: np.ndarray) -> np.ndarray:
    return round_to_bf16(a) if cfg.dtype == "bf16" else a


# tensor ids (seed = 1000 * cfg_id + id)
(_T_X, _T_WR, _T_WIN, _T_CW, _T_CB, _T_WX, _T_WDT, _T_DTB, _T_WOUT, _T_CS, _T_SS, _T_XS, _T_NORM, _T_FGU,
 _T_FDN, _T_FNORM) = range(1, 17)


def make_weights(cfg: RomConfig) -> Dict[str, Optional[np.ndarray]]:
    E, Ex = cfg.n_experts, cfg.n_experts_xdt
    Dm, De, Ds, k, R = cfg.d_model, cfg.d_inner, cfg.d_state, cfg.d_conv, cfg.dt_rank
    s = cfg.weight_std
    w: Dict[str, Optional[np.ndarray]] = {}
    w["w_router"] = _store(cfg, _normal(cfg, _T_WR, (E, Dm), 0.02))
    w["b_router"] = (np.asarray(cfg.router_bias, dtype=np.float32)
                     if cfg.router_bias is not None else None)
    w["w_in"] = _store(cfg, _normal(cfg, _T_WIN, (E, 2 * De, Dm), s))
    # The paper does not give the short-conv initialisation; uniform(-1/sqrt(k), 1/sqrt(k))
    # keeps the conv output at the scale of its input so SiLU is exercised off its linear part.
    lim = 1.0 / np.sqrt(k)
    w["conv_w"] = _rng(cfg, _T_CW).uniform(-lim, lim, (De, k)).astype(np.float32)
    w["conv_b"] = _rng(cfg, _T_CB).uniform(-lim, lim, (De,)).astype(np.float32)
    w["w_x"] = _store(cfg, _normal(cfg, _T_WX, (Ex, R + 2 * Ds, De), s))
    w["w_dt"] = _store(cfg, _normal(cfg, _T_WDT, (Ex, De, R), s))
    # dt_bias: inverse softplus of a log-uniform time step in [1e-3, 1e-1]
    tau = np.exp(_rng(cfg, _T_DTB).uniform(np.log(1e-3), np.log(1e-1), (De,)))
    w["dt_bias"] = (tau + np.log(-np.expm1(-tau))).astype(np.float32)
    w["A_log"] = np.log(np.tile(np.arange(1, Ds + 1, dtype=np.float64), (De, 1))).astype(np.float32)
    w["D"] = np.ones((De,), dtype=np.float32)
    w["w_out"] = _store(cfg, _normal(cfg, _T_WOUT, (E, Dm, De), s))
    # scale of the block's pre-norm (fp32): 1 at initialisation in any trained model; spread to
    # [0.7, 1.3] here so that a missing or misplaced scale cannot hide
    w["norm_w"] = _rng(cfg, _T_NORM).uniform(0.7, 1.3, (Dm,)).astype(np.float32)
    return w


def make_ffn_weights(cfg: RomConfig, d_ff: int) -> Dict[str, np.ndarray]:
    """Parameters of an FFN-MoE layer with cfg's experts: w_gate_up [E, 2*d_ff, d_model] (gate rows
    first), w_down [E, d_model, d_ff], norm_w [d_model] (fp32, scale of its pre-norm)."""
    E, Dm = cfg.n_experts, cfg.d_model
    return {
        "w_gate_up": _store(cfg, _normal(cfg, _T_FGU, (E, 2 * d_ff, Dm), cfg.weight_std)),
        "w_down": _store(cfg, _normal(cfg, _T_FDN, (E, Dm, d_ff), cfg.weight_std)),
        "norm_w": _rng(cfg, _T_FNORM).uniform(0.7, 1.3, (Dm,)).astype(np.float32),
    }


def make_stack_weights(cfg: RomConfig, n_layers: int):
    """Per-layer weight dicts of a stack of blocks: layer j draws from the seeds of
    cfg_id + 1000 * (j + 1), so no two layers (and no other workload) share a tensor."""
    return [make_weights(replace(cfg, cfg_id=cfg.cfg_id + 1000 * (j + 1))) for j in range(n_layers)]


def make_input(cfg: RomConfig) -> np.ndarray:
    """x [B, L, d_model] (for the step workload: the first step's [B, 1, d_model])."""
    L = 1 if cfg.step else cfg.seq_len
    x = _normal(cfg, _T_X, (cfg.batch, L, cfg.d_model), 1.0)
    if cfg.rms_norm_x:
        x /= np.sqrt(np.mean(np.square(x, dtype=np.float32), axis=-1, keepdims=True))
    return _store(cfg, x)


def make_states(cfg: RomConfig):
    """(conv_state [B, d_inner, d_conv-1], ssm_state [B, d_inner, d_state]), fp32, ~N(0,1)."""
    cs = _normal(cfg, _T_CS, (cfg.batch, cfg.d_inner, cfg.d_conv - 1), 1.0)
    ss = _normal(cfg, _T_SS, (cfg.batch, cfg.d_inner, cfg.d_state), 1.0)
    return cs, ss


def make_step_inputs(cfg: RomConfig, n_steps: Optional[int] = None) -> np.ndarray:
    """x_steps [n_steps, B, d_model]: one new token per sequence per step (no feedback)."""
    n = cfg.seq_len if n_steps is None else n_steps
    # values are drawn sequentially, so a shorter run is a prefix of a longer one
    return _store(cfg, _normal(cfg, _T_XS, (n, cfg.batch, cfg.d_model), 1.0))


# --------------------------------------------------------------------------
# RoM on a Mamba2 layer (Sec. 5.2, Table 3): shapes of the published Mamba2 layer
# (expand 2, head dimension 64, state size 128, one B/C group, conv width 4)
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Mamba2Config:
    name: str
    cfg_id: int          # seed base = 1000 * cfg_id + tensor id
    batch: int
    seq_len: int
    d_model: int
    d_inner: int
    d_state: int
    headdim: int
    n_experts: int
    top_k: int
    gate_mode: int
    dtype: str = "bf16"
    d_conv: int = 4
    weight_std: float = 0.02
    rms_norm_x: bool = False
    router_bias: Optional[tuple] = None

    @property
    def n_heads(self) -> int:
        return self.d_inner // self.headdim

    @property
    def n_tokens(self) -> int:
        return self.batch * self.seq_len

    @property
    def d_in_proj(self) -> int:          # rows of one expert's input projection: z | x | B | C | dt
        return 2 * self.d_inner + 2 * self.d_state + self.n_heads

    @property
    def d_conv_ch(self) -> int:          # channels the short conv runs over: x | B | C
        return self.d_inner + 2 * self.d_state


MAMBA2_CONFIGS: Dict[str, Mamba2Config] = {
    # small: several chunks, a ragged tail, two sequences
    "m2_small": Mamba2Config("m2_small", 20, 2, 200, 256, 512, 64, 64, 4, 1, 0),
    # mid: top-2 with renormalised gates, state size 128
    "m2_mid": Mamba2Config("m2_mid", 21, 2, 1500, 512, 1024, 128, 64, 6, 2, 1),
    # the headline layer's Mamba2 counterpart: 16K context, d_model 2048, 8 experts top-1
    "m2_cfg2": Mamba2Config("m2_cfg2", 22, 1, 16384, 2048, 4096, 128, 64, 8, 1, 0,
                            weight_std=0.02 / float(np.sqrt(2 * 48)), rms_norm_x=True),
}


def get_mamba2_config(name: str, **overrides) -> Mamba2Config:
    cfg = MAMBA2_CONFIGS[name]
    return replace(cfg, **overrides) if overrides else cfg


def make_mamba2_weights(cfg: Mamba2Config) -> Dict[str, Optional[np.ndarray]]:
    """w_router [E, d_model], b_router, w_in [E, d_in_proj, d_model] (rows z | x | B | C | dt),
    conv_w [d_conv_ch, k], conv_b [d_conv_ch], dt_bias / A_log / D [H], norm_w [d_inner],
    w_out [E, d_model, d_inner]; float32, the bf16-stored ones exactly representable in bf16."""
    E, Dm, De, H = cfg.n_experts, cfg.d_model, cfg.d_inner, cfg.n_heads
    w: Dict[str, Optional[np.ndarray]] = {}
    w["w_router"] = _store(cfg, _normal(cfg, _T_WR, (E, Dm), 0.02))
    w["b_router"] = (np.asarray(cfg.router_bias, dtype=np.float32) if cfg.router_bias is not None else None)
    w["w_in"] = _store(cfg, _normal(cfg, _T_WIN, (E, cfg.d_in_proj, Dm), cfg.weight_std))
    lim = 1.0 / np.sqrt(cfg.d_conv)
    w["conv_w"] = _rng(cfg, _T_CW).uniform(-lim, lim, (cfg.d_conv_ch, cfg.d_conv)).astype(np.float32)
    w["conv_b"] = _rng(cfg, _T_CB).uniform(-lim, lim, (cfg.d_conv_ch,)).astype(np.float32)
    # per head: time step log-uniform in [1e-3, 1e-1] (dt_bias is its inverse softplus), A uniform in [1, 16]
    tau = np.exp(_rng(cfg, _T_DTB).uniform(np.log(1e-3), np.log(1e-1), (H,)))
    w["dt_bias"] = (tau + np.log(-np.expm1(-tau))).astype(np.float32)
    w["A_log"] = np.log(_rng(cfg, _T_WDT).uniform(1.0, 16.0, (H,))).astype(np.float32)
    w["D"] = _rng(cfg, _T_WX).uniform(0.5, 1.5, (H,)).astype(np.float32)
    w["norm_w"] = _rng(cfg, _T_NORM).uniform(0.7, 1.3, (De,)).astype(np.float32)
    w["w_out"] = _store(cfg, _normal(cfg, _T_WOUT, (E, Dm, De), cfg.weight_std))
    return w


def make_mamba2_input(cfg: Mamba2Config) -> np.ndarray:
    """x [B, L, d_model]."""
    x = _normal(cfg, _T_X, (cfg.batch, cfg.seq_len, cfg.d_model), 1.0)
    if cfg.rms_norm_x:
        x /= np.sqrt(np.mean(np.square(x, dtype=np.float32), axis=-1, keepdims=True))
    return _store(cfg, x)


# --------------------------------------------------------------------------
# RoM on a Gated DeltaNet layer (Sec. 5.2, Table 3): shapes of the published layer at small scale
# (value width 2 x d_model, key width d_model, conv width 4); the paper gives none of its own
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class GdnConfig:
    name: str
    cfg_id: int          # seed base = 1000 * cfg_id + tensor id
    batch: int
    seq_len: int
    d_model: int
    n_heads: int
    d_k: int             # key / query channels per head
    d_v: int             # value channels per head
    n_experts: int
    top_k: int
    gate_mode: int
    dtype: str = "bf16"
    d_conv: int = 4
    weight_std: float = 0.02
    rms_norm_x: bool = False
    router_bias: Optional[tuple] = None

    @property
    def d_kt(self) -> int:
        return self.n_heads * self.d_k

    @property
    def d_vt(self) -> int:
        return self.n_heads * self.d_v

    @property
    def n_tokens(self) -> int:
        return self.batch * self.seq_len

    @property
    def d_in_proj(self) -> int:          # rows of one expert's input projection: z | q | k | v | b | a
        return 2 * self.d_vt + 2 * self.d_kt + 2 * self.n_heads

    @property
    def d_conv_ch(self) -> int:          # channels the short conv runs over: q | k | v
        return 2 * self.d_kt + self.d_vt


GDN_CONFIGS: Dict[str, GdnConfig] = {
    "gdn_small": GdnConfig("gdn_small", 50, 2, 200, 256, 8, 64, 64, 4, 1, 0),
    "gdn_mid": GdnConfig("gdn_mid", 51, 2, 1500, 512, 16, 64, 64, 6, 2, 1),
    # the headline layer's counterpart: 16K context, d_model 2048, 8 experts top-1
    "gdn_cfg2": GdnConfig("gdn_cfg2", 52, 1, 16384, 2048, 32, 64, 64, 8, 1, 0,
                          weight_std=0.02 / float(np.sqrt(2 * 48)), rms_norm_x=True),
}


def get_gdn_config(name: str, **overrides) -> GdnConfig:
    cfg = GDN_CONFIGS[name]
    return replace(cfg, **overrides) if overrides else cfg


def make_gdn_weights(cfg: GdnConfig) -> Dict[str, Optional[np.ndarray]]:
    """w_router [E, d_model], b_router, w_in [E, d_in_proj, d_model] (rows z | q | k | v | b | a),
    conv_w [d_conv_ch, k], conv_b, dt_bias / A_log [H], norm_w [d_v], w_out [E, d_model, D_v];
    float32, the bf16-stored ones exactly representable in bf16."""
    E, Dm, H = cfg.n_experts, cfg.d_model, cfg.n_heads
    w: Dict[str, Optional[np.ndarray]] = {}
    w["w_router"] = _store(cfg, _normal(cfg, _T_WR, (E, Dm), 0.02))
    w["b_router"] = (np.asarray(cfg.router_bias, dtype=np.float32) if cfg.router_bias is not None else None)
    w_in = _normal(cfg, _T_WIN, (E, cfg.d_in_proj, Dm), cfg.weight_std)
    # the two per-head logits are single numbers: at the projections' scale they would never leave
    # the middle of the sigmoid / softplus, so their rows are drawn ten times wider
    w_in[:, 2 * cfg.d_vt + 2 * cfg.d_kt:, :] *= 10.0
    w["w_in"] = _store(cfg, w_in)
    lim = 1.0 / np.sqrt(cfg.d_conv)
    w["conv_w"] = _rng(cfg, _T_CW).uniform(-lim, lim, (cfg.d_conv_ch, cfg.d_conv)).astype(np.float32)
    w["conv_b"] = _rng(cfg, _T_CB).uniform(-lim, lim, (cfg.d_conv_ch,)).astype(np.float32)
    # per head: time step log-uniform in [1e-3, 1e-1] (dt_bias is its inverse softplus), decay rate uniform in [1, 16]
    tau = np.exp(_rng(cfg, _T_DTB).uniform(np.log(1e-3), np.log(1e-1), (H,)))
    w["dt_bias"] = (tau + np.log(-np.expm1(-tau))).astype(np.float32)
    w["A_log"] = np.log(_rng(cfg, _T_WDT).uniform(1.0, 16.0, (H,))).astype(np.float32)
    w["norm_w"] = _rng(cfg, _T_NORM).uniform(0.7, 1.3, (cfg.d_v,)).astype(np.float32)
    w["w_out"] = _store(cfg, _normal(cfg, _T_WOUT, (E, Dm, cfg.d_vt), cfg.weight_std))
    return w


def make_gdn_input(cfg: GdnConfig) -> np.ndarray:
    """x [B, L, d_model]."""
    x = _normal(cfg, _T_X, (cfg.batch, cfg.seq_len, cfg.d_model), 1.0)
    if cfg.rms_norm_x:
        x /= np.sqrt(np.mean(np.square(x, dtype=np.float32), axis=-1, keepdims=True))
    return _store(cfg, x)
