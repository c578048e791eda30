"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
include/rom.h declares, and its argument validation / workspace planning behave as documented."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2506_18145_amd import binding
    if not os.path.exists(binding._LIB_PATH):
        from paper_2506_18145_amd.build import build_library
        build_library()
    return binding.load_library()


def _dims(**kw):
    from paper_2506_18145_amd.binding import RomDims
    base = dict(d_model=64, d_inner=128, d_state=16, d_conv=4, dt_rank=8, n_experts=4, top_k=1,
                n_experts_xdt=4, dtype=0, gate_mode=0)
    base.update(kw)
    return RomDims(**base)


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "rom.h")).read()
    names = re.findall(r"ROM_API\s+[\w\s\*]+?\b(rom_\w+)\s*\(", header)
    assert len(names) >= 9
    for name in names:
        assert hasattr(lib, name), name


def test_struct_sizes_match_header():
    from paper_2506_18145_amd import binding
    assert ctypes.sizeof(binding.RomDims) == 40
    assert ctypes.sizeof(binding._RomWeights) == 11 * ctypes.sizeof(ctypes.c_void_p)
    assert ctypes.sizeof(binding._RomWsLayout) == 14 * ctypes.sizeof(ctypes.c_size_t)
    assert ctypes.sizeof(binding._RomBlock) == 12 * ctypes.sizeof(ctypes.c_void_p)
    assert ctypes.sizeof(binding._RomFfnWeights) == 2 * ctypes.sizeof(ctypes.c_void_p)


def test_workspace_bytes_and_layout(lib):
    from paper_2506_18145_amd import binding
    d = _dims()
    small = binding.rom_workspace_bytes(d, 1, 64)
    big = binding.rom_workspace_bytes(d, 2, 64)
    assert 0 < small < big
    lay = binding.rom_workspace_layout(d, 1, 64)
    assert lay["total_bytes"] == small
    offs = [lay[k] for k in ("expert_idx", "gate", "counts", "offsets", "perm", "inv_perm", "logits",
                             "xz", "u", "dt_low", "bc", "dt", "g")]
    assert offs == sorted(offs) and len(set(offs)) == len(offs)
    assert all(o % 256 == 0 and o < small for o in offs)
    # xz holds N * 2*d_inner fp32 values before u starts
    assert lay["u"] - lay["xz"] >= 64 * 2 * 128 * 4


def test_invalid_dims_are_rejected_before_any_launch(lib):
    from paper_2506_18145_amd import binding
    assert binding.rom_workspace_bytes(_dims(d_state=8), 1, 8) == 0          # unsupported
    assert binding.rom_workspace_bytes(_dims(top_k=5), 1, 8) == 0            # K > E
    assert binding.rom_workspace_bytes(_dims(dtype=7), 1, 8) == 0
    lay = binding._RomWsLayout()
    assert lib.rom_workspace_layout(ctypes.byref(_dims(d_conv=3)), 1, 8, ctypes.byref(lay)) == -3
    assert lib.rom_workspace_layout(ctypes.byref(_dims(top_k=0)), 1, 8, ctypes.byref(lay)) == -1
    assert lib.rom_workspace_layout(ctypes.byref(_dims(n_experts_xdt=2)), 1, 8, ctypes.byref(lay)) == -1
    w = binding._RomWeights()                                                # all NULL
    d = _dims()
    # NULL weights / tensors: refused with ROM_E_INVAL, nothing is launched (no GPU here)
    assert lib.rom_layer_forward(ctypes.byref(d), ctypes.byref(w), None, 1, 8, None, None, None, None,
                                 None, None, 0, None) == -1
    assert lib.rom_route(ctypes.byref(d), ctypes.byref(w), None, 8, None, None, None, None, None, None,
                         None, None, 0, None) == -1
    assert lib.rom_step(ctypes.byref(d), ctypes.byref(w), None, 4, None, None, None, None, 0, None) == -1
    assert lib.rom_layer_forward(None, ctypes.byref(w), None, 1, 8, None, None, None, None, None, None,
                                 0, None) == -1


def test_sizes_beyond_the_supported_range_are_refused(lib):
    """More than 65535 sequences, or more than 2^30 (token, k) slots: ROM_E_UNSUPPORTED before the
    workspace is even looked at."""
    from paper_2506_18145_amd import binding
    d = _dims(top_k=2)
    buf = ctypes.create_string_buffer(4096 + 256)
    addr = (ctypes.addressof(buf) + 255) // 256 * 256
    w = binding._RomWeights(*([addr] * 11))
    fwd = lambda B, L: lib.rom_layer_forward(ctypes.byref(d), ctypes.byref(w), addr, B, L, None, None,
                                             addr + 2048, None, None, addr, 4096, None)
    assert fwd(65536, 1) == -3
    assert fwd(1, (1 << 29) + 1) == -3
    assert fwd(65535, 1) == -2 and fwd(1, 1 << 20) == -2      # in range: only the workspace is too small
    assert lib.rom_route(ctypes.byref(d), ctypes.byref(w), addr, (1 << 29) + 1, addr, addr, addr, addr, addr,
                         addr, None, addr, 4096, None) == -3


def test_error_strings_and_stage_names(lib):
    assert lib.rom_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4):
        assert len(lib.rom_strerror(code)) > 5
    from paper_2506_18145_amd.binding import STAGE_NAMES
    assert tuple(lib.rom_stage_name(i).decode() for i in range(len(STAGE_NAMES))) == STAGE_NAMES


def test_empty_input_is_a_successful_noop(lib):
    """B == 0 or L == 0 returns ROM_OK without touching any pointer (so it is safe with no GPU)."""
    from paper_2506_18145_amd import binding
    d = _dims()
    buf = ctypes.create_string_buffer(4096 + 256)
    addr = (ctypes.addressof(buf) + 255) // 256 * 256
    w = binding._RomWeights(*([addr] * 11))
    assert lib.rom_layer_forward(ctypes.byref(d), ctypes.byref(w), addr, 0, 8, None, None, addr, None,
                                 None, addr, 4096, None) == 0
    assert lib.rom_layer_forward(ctypes.byref(d), ctypes.byref(w), addr, 2, 0, None, None, addr, None,
                                 None, addr, 4096, None) == 0
    assert lib.rom_route(ctypes.byref(d), ctypes.byref(w), addr, 0, addr, addr, addr, addr, addr, addr,
                         None, addr, 4096, None) == 0
    assert lib.rom_step(ctypes.byref(d), ctypes.byref(w), addr, 0, None, None, addr, addr, 4096, None) == 0


def test_binding_refuses_to_run_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    from paper_2506_18145_amd import RomError, RomLayer
    from rom_synth import get_config, make_weights
    cfg = get_config("cfg0")
    with pytest.raises(RomError):
        RomLayer(cfg, make_weights(cfg))


def test_route_workspace_is_small_and_the_layer_workspace_an_upper_bound(lib):
    from paper_2506_18145_amd import binding
    d = _dims(dtype=1, d_model=2048, d_inner=4096, dt_rank=128, n_experts=8, n_experts_xdt=8)
    n = 16384
    need = binding.rom_route_workspace_bytes(d, n)
    assert 0 < need <= 4 * n * 8 + (1 << 20)                  # index arrays only: no activation region
    assert need <= binding.rom_workspace_bytes(d, n, 1) and need <= binding.rom_workspace_bytes(d, 1, n)
    assert binding.rom_route_workspace_bytes(_dims(top_k=9), n) == 0
    buf = ctypes.create_string_buffer(4096 + 256)
    addr = (ctypes.addressof(buf) + 255) // 256 * 256
    w = binding._RomWeights(*([addr] * 11))
    args = (addr, n, addr, addr, addr, addr, addr, addr, None, addr)
    assert lib.rom_route(ctypes.byref(d), ctypes.byref(w), *args, need - 1, None) == -2    # refused before any launch


def test_balance_stats_arguments_and_scratch_placement(lib):
    """rom_balance_stats refuses bad arguments before any launch, and the scratch it takes from the
    workspace sits between the logits and xz at an offset that depends on N, K and E only."""
    from paper_2506_18145_amd import binding
    d = _dims(n_experts=8, top_k=2, n_experts_xdt=8)
    buf = ctypes.create_string_buffer(4096 + 256)
    addr = (ctypes.addressof(buf) + 255) // 256 * 256
    call = lambda dims, lg, ct, n, ws, nbytes: lib.rom_balance_stats(
        ctypes.byref(dims), lg, ct, n, 1e-3, addr, addr, addr, ws, nbytes, None)
    assert call(d, addr, addr, 0, addr, 4096) == -1            # no tokens
    assert call(d, None, addr, 16, addr, 4096) == -1
    assert call(d, addr, None, 16, addr, 4096) == -1
    assert call(d, addr, addr, 16, None, 4096) == -1
    assert call(d, addr, addr, 16, addr + 8, 4096) == -1       # misaligned workspace
    assert call(d, addr, addr, 16, addr, 4096) == -2           # workspace too small
    assert call(_dims(top_k=9), addr, addr, 16, addr, 4096) == -1
    N, E = 1200, 8
    lays = [binding.rom_workspace_layout(d, 1, N), binding.rom_workspace_layout(d, N, 1),
            binding.rom_workspace_layout(d, 4, N // 4)]
    for lay in lays:
        assert lay["logits"] == lays[0]["logits"] and lay["xz"] == lays[0]["xz"]
        assert lay["xz"] - lay["logits"] >= N * E * 4 + 256 * E * 4


def test_block_and_stack_arguments_are_checked_before_any_launch(lib):
    from paper_2506_18145_amd import binding
    d = _dims()
    buf = ctypes.create_string_buffer(8192 + 256)
    addr = (ctypes.addressof(buf) + 255) // 256 * 256
    w = binding._RomWeights(*([addr] * 11))
    F = ctypes.c_float
    # no norm weight / negative eps / misaligned norm weight
    assert lib.rom_block_forward(ctypes.byref(d), ctypes.byref(w), None, F(1e-5), addr, 1, 8, None, None,
                                 addr + 4096, None, None, addr, 4096, None) == -1
    assert lib.rom_block_forward(ctypes.byref(d), ctypes.byref(w), addr, F(-1.0), addr, 1, 8, None, None,
                                 addr + 4096, None, None, addr, 4096, None) == -1
    assert lib.rom_block_forward(ctypes.byref(d), ctypes.byref(w), addr + 4, F(1e-5), addr, 1, 8, None, None,
                                 addr + 4096, None, None, addr, 4096, None) == -1
    # a valid call shape with a workspace that is too small, and the empty call
    assert lib.rom_block_forward(ctypes.byref(d), ctypes.byref(w), addr, F(1e-5), addr, 1, 8, None, None,
                                 addr + 4096, None, None, addr, 4096, None) == -2
    assert lib.rom_block_forward(ctypes.byref(d), ctypes.byref(w), addr, F(1e-5), addr, 0, 8, None, None,
                                 addr + 4096, None, None, addr, 4096, None) == 0
    assert lib.rom_block_step(ctypes.byref(d), ctypes.byref(w), addr, F(1e-5), addr, 4, None, None, addr + 4096,
                              addr, 4096, None) == -1                   # a step needs its states
    assert lib.rom_fold_norm(ctypes.byref(d), None, addr, addr, None) == -1
    assert lib.rom_fold_norm(ctypes.byref(_dims(d_conv=3)), addr, addr, addr, None) == -3
    blocks = (binding._RomBlock * 2)()
    for b in blocks:
        b.w = w
        b.norm_weight = addr
    call = lambda blk, n, tmp, out=addr + 4096, B=1: lib.rom_stack_forward(
        ctypes.byref(d), blk, n, F(1e-5), addr, B, 8, None, None, out, None, None, tmp, addr, 4096, None)
    assert call(blocks, 2, None) == -1                 # two layers need the scratch buffer
    assert call(blocks, 2, addr) == -1                 # ... which must not alias x
    assert call(blocks, 2, addr + 4096) == -1          # ... nor out
    assert call(blocks, 0, addr + 2048) == -1
    assert call(None, 2, addr + 2048) == -1
    assert call(blocks, 2, addr + 2048) == -2          # all pointers fine, workspace too small
    assert call(blocks, 2, addr + 2048, B=0) == 0
    blocks[1].norm_weight = None                       # a bad second layer is refused before layer 0 runs
    assert call(blocks, 2, addr + 2048) == -1
    assert lib.rom_stack_step(ctypes.byref(d), blocks, 2, F(1e-5), addr, 4, None, None, addr + 4096,
                              addr + 2048, addr, 4096, None) == -1


def test_ffn_moe_arguments_and_workspace(lib):
    from paper_2506_18145_amd import binding
    d = _dims(n_experts=4, top_k=2)
    assert binding.rom_ffn_workspace_bytes(d, 24, 8) == 0            # d_ff not a multiple of 16
    assert binding.rom_ffn_workspace_bytes(d, 0, 8) == 0
    assert binding.rom_ffn_workspace_bytes(_dims(d_state=8), 32, 8) == 0
    small, big = binding.rom_ffn_workspace_bytes(d, 32, 8), binding.rom_ffn_workspace_bytes(d, 32, 64)
    # slots x (gate|up row + activated row + per-expert output row) at least
    assert 0 < small < big and big >= 64 * 2 * (2 * 32 + 32 + 64) * 4
    buf = ctypes.create_string_buffer(8192 + 256)
    addr = (ctypes.addressof(buf) + 255) // 256 * 256
    w = binding._RomFfnWeights(addr, addr)
    F = ctypes.c_float
    call = lambda dims, d_ff, wp, x, out, n, ws, nbytes, offs=addr: lib.rom_ffn_moe_forward(
        ctypes.byref(dims), d_ff, wp, 1, F(1e-5), 1, x, n, offs, addr, addr, addr, out, ws, nbytes, None)
    assert call(d, 32, ctypes.byref(w), addr, addr + 4096, 0, addr, 4096) == 0        # no tokens
    assert call(d, 24, ctypes.byref(w), addr, addr + 4096, 8, addr, 4096) == -3
    assert call(d, 32, None, addr, addr + 4096, 8, addr, 4096) == -1
    assert call(d, 32, ctypes.byref(w), addr, addr, 8, addr, 4096) == -1              # out aliases x
    assert call(d, 32, ctypes.byref(w), addr, addr + 4096, 8, addr, 4096, offs=None) == -1
    assert call(d, 32, ctypes.byref(w), addr, addr + 4096, 8, addr + 8, 4096) == -1   # misaligned workspace
    assert call(d, 32, ctypes.byref(w), addr, addr + 4096, 8, addr, 4096) == -2       # workspace too small
    assert lib.rom_ffn_moe_forward(ctypes.byref(d), 32, ctypes.byref(w), 1, F(-1.0), 1, addr, 8, addr, addr, addr,
                                   addr, addr + 4096, addr, 4096, None) == -1         # negative eps
    assert lib.rom_ffn_pack_gate_up(ctypes.byref(d), 32, None, addr, addr + 4096, None) == -1
    assert lib.rom_ffn_pack_gate_up(ctypes.byref(d), 32, addr, None, addr, None) == -1     # not in place


def test_hybrid_stack_arguments_are_checked_before_any_launch(lib):
    from paper_2506_18145_amd import binding
    d = _dims()
    buf = ctypes.create_string_buffer(8192 + 256)
    addr = (ctypes.addressof(buf) + 255) // 256 * 256
    w = binding._RomWeights(*([addr] * 11))
    blocks = (binding._RomBlock * 2)()
    for b in blocks:
        b.w = w
        b.norm_weight = addr
    ffns = (binding._RomFfnWeights * 2)()
    ffns[1] = binding._RomFfnWeights(addr, addr)
    F = ctypes.c_float
    call = lambda fw, d_ff=32, tmp=addr + 2048, ffn_ws=addr + 6144, n=2, B=1: lib.rom_hybrid_stack_forward(
        ctypes.byref(d), d_ff, blocks, fw, 1, n, F(1e-5), addr, B, 8, None, None, addr + 4096, None, None, tmp,
        addr, 4096, ffn_ws, 1024, None)
    assert call(ffns, d_ff=24) == -3                       # d_ff not a multiple of 16
    assert call(None) == -1
    assert call(ffns, tmp=None) == -1
    assert call(ffns, ffn_ws=None) == -1                   # layer 1 has an FFN: it needs its workspace
    assert call(ffns, ffn_ws=addr) == -1                   # ... distinct from the RoM workspace
    assert call(ffns) == -2                                # everything in place, workspaces too small
    assert call(ffns, B=0) == 0
    ffns[1].w_down = None                                  # half an FFN
    assert call(ffns) == -1
