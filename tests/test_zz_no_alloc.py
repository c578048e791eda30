"""rom_step_static (the step for callers that cannot allocate: its workspace is a static device
array of the library) against rom_step, through the C ABI: two calls in a row on carried states,
the second on fewer sequences, every output and state bit for bit."""
import numpy as np
import pytest
import torch

from paper_2506_18145_amd import RomError, RomLayer, rom_step, rom_step_static
from rom_synth import RomConfig, make_states, make_step_inputs, make_weights

pytestmark = pytest.mark.gpu


def _cfg(**kw):
    base = dict(name="static-step", cfg_id=97, batch=37, seq_len=2, d_model=256, d_inner=512, d_state=16, d_conv=4,
                dt_rank=16, n_experts=8, top_k=2, dtype="bf16", gate_mode=1, step=True, weight_std=0.05)
    base.update(kw)
    return RomConfig(**base)


@pytest.mark.parametrize("kw", [dict(), dict(dtype="fp32", top_k=1, gate_mode=0, n_experts=4),
                                dict(batch=256, d_model=2048, d_inner=4096, dt_rank=128, top_k=1, gate_mode=0,
                                     weight_std=0.02)])
def test_step_static_matches_step_on_two_calls_the_second_smaller(kw):
    cfg = _cfg(**kw)
    layer = RomLayer(cfg, make_weights(cfg))
    xs = layer.to_device(make_step_inputs(cfg, 2))            # [2, B, d_model]
    cs0, ss0 = make_states(cfg)
    B = cfg.batch
    B2 = max(1, B // 3)                                       # the second call: fewer sequences
    ref_cs, ref_ss = layer.to_device(cs0, typed=False), layer.to_device(ss0, typed=False)
    got_cs, got_ss = ref_cs.clone(), ref_ss.clone()
    ws = layer.workspace(B, 1)
    for t, n in ((0, B), (1, B2)):
        x = xs[t, :n].contiguous()
        ref_out, got_out = torch.empty_like(x), torch.full_like(x, float("nan"))
        rom_step(layer.dims, layer.weights, x, n, ref_cs[:n], ref_ss[:n], ref_out, ws)
        rom_step_static(layer.dims, layer.weights, x, n, got_cs[:n], got_ss[:n], got_out)
        torch.cuda.synchronize()
        assert torch.equal(ref_out, got_out), f"call {t}: out differs"
        assert torch.equal(ref_cs, got_cs) and torch.equal(ref_ss, got_ss), f"call {t}: states differ"
        assert bool(torch.isfinite(got_out.float()).all())


def test_step_static_refuses_what_does_not_fit():
    cfg = _cfg(batch=4096, d_model=2048, d_inner=4096, dt_rank=128)
    from paper_2506_18145_amd.binding import RomDims, _RomWeights, load_library
    import ctypes
    lib = load_library()
    d = RomDims(cfg.d_model, cfg.d_inner, 16, 4, cfg.dt_rank, cfg.n_experts, cfg.top_k, cfg.n_experts, 1, 1)
    buf = torch.zeros(1024, dtype=torch.uint8, device="cuda:0")
    a = buf.data_ptr()
    w = _RomWeights(*([a] * 11))
    assert lib.rom_step_static(ctypes.byref(d), ctypes.byref(w), a, 4096, a, a, a, None) == -5
    assert b"static" in lib.rom_strerror(-5)
    assert lib.rom_step_static(ctypes.byref(d), ctypes.byref(w), a, 0, None, None, a, None) == 0     # no-op
    assert lib.rom_step_static(ctypes.byref(d), ctypes.byref(w), a, 4, None, a, a, None) == -1
