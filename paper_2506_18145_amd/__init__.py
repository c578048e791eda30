"""MI355X-native Routing Mamba (RoM) layer forward pass: Python binding over librom.so.

The binding only marshals arguments (torch tensors -> device pointers); every step of
the layer runs in the HIP kernels behind the C ABI declared in include/rom.h.
"""
from .binding import (  # noqa: F401
    RomDims,
    RomError,
    RomFfnMoe,
    RomHybridStack,
    RomLayer,
    RomStack,
    load_library,
    rom_balance_stats,
    rom_block_forward,
    rom_block_step,
    rom_ffn_pack_gate_up,
    rom_ffn_moe_forward,
    rom_ffn_workspace_bytes,
    rom_fold_norm,
    rom_hybrid_stack_forward,
    rom_stack_forward,
    rom_stack_step,
    rom_layer_forward,
    rom_layer_backward,
    rom_backward_workspace_bytes,
    rom_profile_collect,
    rom_profile_collect_calls,
    rom_profile_copy,
    rom_probe,
    rom_profile_enable,
    rom_route,
    rom_route_workspace_bytes,
    rom_step,
    rom_step_static,
    rom_workspace_bytes,
    rom_workspace_layout,
    STAGE_NAMES,
)
