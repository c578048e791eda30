"""Seeded synthetic inputs for the Routing Mamba (RoM) layer.

This module serves both the CPU oracle's tests and the HIP path's tests and
benchmark.  It only *draws and lays out numbers* (shapes, distributions,
rounding of stored values to bf16); none of the layer's arithmetic (router,
projections, convolution, scan, gating, combine) lives here.
"""
from .configs import (  # noqa: F401
    RomConfig,
    CONFIGS,
    get_config,
    make_weights,
    make_stack_weights,
    make_ffn_weights,
    make_input,
    make_states,
    make_step_inputs,
    round_to_bf16,
    bf16_bits,
    Mamba2Config,
    MAMBA2_CONFIGS,
    get_mamba2_config,
    make_mamba2_weights,
    make_mamba2_input,
    GdnConfig,
    GDN_CONFIGS,
    get_gdn_config,
    make_gdn_weights,
    make_gdn_input,
)
