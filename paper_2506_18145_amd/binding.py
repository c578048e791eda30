"""ctypes binding of librom.so.  Argument marshalling only - no arithmetic happens here."""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "librom.so")
_lib: Optional[ctypes.CDLL] = None

ROM_DTYPE_F32, ROM_DTYPE_BF16 = 0, 1
STAGE_NAMES = ("route", "permute", "in_proj", "conv", "x_proj", "dt_proj", "scan_gate", "out_proj",
               "combine")


class RomError(RuntimeError):
    pass


class RomDims(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "d_model", "d_inner", "d_state", "d_conv", "dt_rank", "n_experts", "top_k",
        "n_experts_xdt", "dtype", "gate_mode")]


class _RomWeights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in (
        "w_router", "b_router", "w_in", "conv_w", "conv_b", "w_x", "w_dt", "dt_bias", "A_log", "D",
        "w_out")]


class _RomGrads(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in (
        "d_w_router", "d_b_router", "d_w_in", "d_conv_w", "d_conv_b", "d_w_x", "d_w_dt", "d_dt_bias", "d_A_log",
        "d_D", "d_w_out")]


class _RomBlock(ctypes.Structure):
    _fields_ = [("w", _RomWeights), ("norm_weight", ctypes.c_void_p)]


class _RomFfnWeights(ctypes.Structure):
    _fields_ = [("w_gate_up", ctypes.c_void_p), ("w_down", ctypes.c_void_p)]


class _RomFfnGrads(ctypes.Structure):
    _fields_ = [("d_w_gate_up", ctypes.c_void_p), ("d_w_down", ctypes.c_void_p), ("d_norm_weight", ctypes.c_void_p)]


class _RomWsLayout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_size_t) for n in (
        "total_bytes", "expert_idx", "gate", "counts", "offsets", "perm", "inv_perm", "logits", "xz",
        "u", "dt_low", "bc", "dt", "g")]


class RomMamba2Dims(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "d_model", "d_inner", "d_state", "d_conv", "headdim", "n_experts", "top_k", "dtype", "gate_mode")]


class _RomMamba2Weights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in (
        "w_router", "b_router", "w_in", "conv_w", "conv_b", "dt_bias", "A_log", "D", "norm_w", "w_out")]


class _RomMamba2WsLayout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_size_t) for n in (
        "total_bytes", "expert_idx", "gate", "counts", "offsets", "perm", "inv_perm", "logits", "zxbcdt", "xbc",
        "yz", "g")]


class RomGdnDims(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "d_model", "n_heads", "d_k", "d_v", "d_conv", "n_experts", "top_k", "dtype", "gate_mode")]


class _RomGdnWeights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in (
        "w_router", "b_router", "w_in", "conv_w", "conv_b", "dt_bias", "A_log", "norm_w", "w_out")]


class _RomGdnWsLayout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_size_t) for n in (
        "total_bytes", "expert_idx", "gate", "counts", "offsets", "perm", "inv_perm", "logits", "proj", "qkv", "y")]


def load_library() -> ctypes.CDLL:
    """Loads librom.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RomError(f"{_LIB_PATH} is missing: build it with `python -m paper_2506_18145_amd.build` "
                       "(or __graft_entry__.build()); there is no non-HIP fallback")
    lib = ctypes.CDLL(_LIB_PATH)
    P, I64, SZ = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t
    lib.rom_workspace_bytes.restype = SZ
    lib.rom_workspace_bytes.argtypes = [ctypes.POINTER(RomDims), I64, I64]
    lib.rom_route_workspace_bytes.restype = SZ
    lib.rom_route_workspace_bytes.argtypes = [ctypes.POINTER(RomDims), I64]
    lib.rom_workspace_layout.restype = ctypes.c_int
    lib.rom_workspace_layout.argtypes = [ctypes.POINTER(RomDims), I64, I64, ctypes.POINTER(_RomWsLayout)]
    lib.rom_route.restype = ctypes.c_int
    lib.rom_route.argtypes = [ctypes.POINTER(RomDims), ctypes.POINTER(_RomWeights), P, I64,
                              P, P, P, P, P, P, P, P, SZ, P]
    lib.rom_balance_stats.restype = ctypes.c_int
    lib.rom_balance_stats.argtypes = [ctypes.POINTER(RomDims), P, P, I64, ctypes.c_float, P, P, P, P, SZ, P]
    lib.rom_layer_forward.restype = ctypes.c_int
    lib.rom_layer_forward.argtypes = [ctypes.POINTER(RomDims), ctypes.POINTER(_RomWeights), P, I64, I64,
                                      P, P, P, P, P, P, SZ, P]
    lib.rom_step.restype = ctypes.c_int
    lib.rom_step.argtypes = [ctypes.POINTER(RomDims), ctypes.POINTER(_RomWeights), P, I64, P, P, P, P, SZ, P]
    lib.rom_backward_workspace_bytes.restype = SZ
    lib.rom_backward_workspace_bytes.argtypes = [ctypes.POINTER(RomDims), I64, I64]
    lib.rom_layer_backward.restype = ctypes.c_int
    lib.rom_layer_backward.argtypes = [ctypes.POINTER(RomDims), ctypes.POINTER(_RomWeights), P, I64, I64, P, P,
                                       ctypes.POINTER(_RomGrads), P, SZ, P]
    lib.rom_layer_backward_saved.restype = ctypes.c_int
    lib.rom_layer_backward_saved.argtypes = lib.rom_layer_backward.argtypes
    lib.rom_step_static.restype = ctypes.c_int
    lib.rom_step_static.argtypes = [ctypes.POINTER(RomDims), ctypes.POINTER(_RomWeights), P, I64, P, P, P, P]
    F32 = ctypes.c_float
    lib.rom_block_backward_workspace_bytes.restype = SZ
    lib.rom_block_backward_workspace_bytes.argtypes = [ctypes.POINTER(RomDims), I64, I64]
    lib.rom_block_backward.restype = ctypes.c_int
    lib.rom_block_backward.argtypes = [ctypes.POINTER(RomDims), ctypes.POINTER(_RomWeights), P, F32, P, I64, I64, P, P, P,
                                       ctypes.POINTER(_RomGrads), P, P, SZ, P]
    lib.rom_block_backward_saved.restype = ctypes.c_int
    lib.rom_block_backward_saved.argtypes = lib.rom_block_backward.argtypes
    lib.rom_block_forward_train.restype = ctypes.c_int
    lib.rom_block_forward_train.argtypes = [ctypes.POINTER(RomDims), ctypes.POINTER(_RomWeights), P, F32, P, I64, I64, P, P,
                                            SZ, P]
    lib.rom_fold_norm.restype = ctypes.c_int
    lib.rom_fold_norm.argtypes = [ctypes.POINTER(RomDims), P, P, P, P]
    lib.rom_block_forward.restype = ctypes.c_int
    lib.rom_block_forward.argtypes = [ctypes.POINTER(RomDims), ctypes.POINTER(_RomWeights), P, F32, P, I64,
                                      I64, P, P, P, P, P, P, SZ, P]
    lib.rom_block_step.restype = ctypes.c_int
    lib.rom_block_step.argtypes = [ctypes.POINTER(RomDims), ctypes.POINTER(_RomWeights), P, F32, P, I64, P, P,
                                   P, P, SZ, P]
    lib.rom_stack_forward.restype = ctypes.c_int
    lib.rom_stack_forward.argtypes = [ctypes.POINTER(RomDims), ctypes.POINTER(_RomBlock), ctypes.c_int, F32, P,
                                      I64, I64, P, P, P, P, P, P, P, SZ, P]
    lib.rom_stack_step.restype = ctypes.c_int
    lib.rom_stack_step.argtypes = [ctypes.POINTER(RomDims), ctypes.POINTER(_RomBlock), ctypes.c_int, F32, P,
                                   I64, P, P, P, P, P, SZ, P]
    lib.rom_ffn_workspace_bytes.restype = SZ
    lib.rom_ffn_workspace_bytes.argtypes = [ctypes.POINTER(RomDims), ctypes.c_int32, I64]
    lib.rom_ffn_pack_gate_up.restype = ctypes.c_int
    lib.rom_ffn_pack_gate_up.argtypes = [ctypes.POINTER(RomDims), ctypes.c_int32, P, P, P, P]
    lib.rom_ffn_moe_forward.restype = ctypes.c_int
    lib.rom_ffn_moe_forward.argtypes = [ctypes.POINTER(RomDims), ctypes.c_int32, ctypes.POINTER(_RomFfnWeights),
                                        ctypes.c_int, F32, ctypes.c_int, P, I64, P, P, P, P, P, P, SZ, P]
    lib.rom_ffn_backward_workspace_bytes.restype = SZ
    lib.rom_ffn_backward_workspace_bytes.argtypes = [ctypes.POINTER(RomDims), ctypes.c_int32, I64]
    lib.rom_ffn_moe_backward.restype = ctypes.c_int
    lib.rom_ffn_moe_backward.argtypes = [ctypes.POINTER(RomDims), ctypes.c_int32, ctypes.POINTER(_RomFfnWeights), P, F32,
                                         ctypes.c_int, P, I64, P, P, P, P, P, P, P, ctypes.POINTER(_RomFfnGrads), P, SZ, P]
    lib.rom_ffn_moe_backward_saved.restype = ctypes.c_int
    lib.rom_ffn_moe_backward_saved.argtypes = lib.rom_ffn_moe_backward.argtypes
    lib.rom_ffn_moe_forward_train.restype = ctypes.c_int
    lib.rom_ffn_moe_forward_train.argtypes = [ctypes.POINTER(RomDims), ctypes.c_int32, ctypes.POINTER(_RomFfnWeights), P, F32,
                                              ctypes.c_int, P, I64, P, P, P, P, P, P, SZ, P]
    lib.rom_hybrid_stack_forward.restype = ctypes.c_int
    lib.rom_hybrid_stack_forward.argtypes = [ctypes.POINTER(RomDims), ctypes.c_int32, ctypes.POINTER(_RomBlock),
                                             ctypes.POINTER(_RomFfnWeights), ctypes.c_int, ctypes.c_int, F32, P,
                                             I64, I64, P, P, P, P, P, P, P, SZ, P, SZ, P]
    lib.rom_mamba2_workspace_bytes.restype = SZ
    lib.rom_mamba2_workspace_bytes.argtypes = [ctypes.POINTER(RomMamba2Dims), I64, I64]
    lib.rom_mamba2_workspace_layout.restype = ctypes.c_int
    lib.rom_mamba2_workspace_layout.argtypes = [ctypes.POINTER(RomMamba2Dims), I64, I64,
                                                ctypes.POINTER(_RomMamba2WsLayout)]
    lib.rom_mamba2_forward.restype = ctypes.c_int
    lib.rom_mamba2_forward.argtypes = [ctypes.POINTER(RomMamba2Dims), ctypes.POINTER(_RomMamba2Weights), P, I64, I64,
                                       F32, P, P, P, P, P, P, SZ, P]
    lib.rom_mamba2_block_forward.restype = ctypes.c_int
    lib.rom_mamba2_block_forward.argtypes = [ctypes.POINTER(RomMamba2Dims), ctypes.POINTER(_RomMamba2Weights), P, F32, P,
                                             I64, I64, F32, P, P, P, P, P, P, SZ, P]
    lib.rom_gdn_block_forward.restype = ctypes.c_int
    lib.rom_gdn_block_forward.argtypes = [ctypes.POINTER(RomGdnDims), ctypes.POINTER(_RomGdnWeights), P, F32, P, I64, I64,
                                          F32, P, P, P, P, P, P, SZ, P]
    lib.rom_fold_norm_rows.restype = ctypes.c_int
    lib.rom_fold_norm_rows.argtypes = [ctypes.c_int, P, P, P, I64, ctypes.c_int32, P]
    lib.rom_mamba2_step.restype = ctypes.c_int
    lib.rom_mamba2_step.argtypes = [ctypes.POINTER(RomMamba2Dims), ctypes.POINTER(_RomMamba2Weights), P, I64, F32, P, P,
                                    P, P, SZ, P]
    lib.rom_gdn_workspace_bytes.restype = SZ
    lib.rom_gdn_workspace_bytes.argtypes = [ctypes.POINTER(RomGdnDims), I64, I64]
    lib.rom_gdn_workspace_layout.restype = ctypes.c_int
    lib.rom_gdn_workspace_layout.argtypes = [ctypes.POINTER(RomGdnDims), I64, I64, ctypes.POINTER(_RomGdnWsLayout)]
    lib.rom_gdn_forward.restype = ctypes.c_int
    lib.rom_gdn_forward.argtypes = [ctypes.POINTER(RomGdnDims), ctypes.POINTER(_RomGdnWeights), P, I64, I64, F32, P, P,
                                    P, P, P, P, SZ, P]
    lib.rom_gdn_step.restype = ctypes.c_int
    lib.rom_gdn_step.argtypes = [ctypes.POINTER(RomGdnDims), ctypes.POINTER(_RomGdnWeights), P, I64, F32, P, P, P, P, SZ, P]
    lib.rom_strerror.restype = ctypes.c_char_p
    lib.rom_strerror.argtypes = [ctypes.c_int]
    lib.rom_profile_enable.restype = ctypes.c_int
    lib.rom_profile_enable.argtypes = [ctypes.c_int]
    lib.rom_profile_select.restype = ctypes.c_int
    lib.rom_profile_select.argtypes = [ctypes.c_uint]
    lib.rom_profile_collect.restype = ctypes.c_int
    lib.rom_profile_collect.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int)]
    lib.rom_profile_collect_calls.restype = ctypes.c_int
    lib.rom_profile_collect_calls.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.c_int,
                                              ctypes.POINTER(ctypes.c_int)]
    lib.rom_profile_copy.restype = ctypes.c_int
    lib.rom_profile_copy.argtypes = [P, P, SZ, P]
    lib.rom_probe.restype = ctypes.c_int
    lib.rom_probe.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, P, SZ, P]
    lib.rom_stage_name.restype = ctypes.c_char_p
    lib.rom_stage_name.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def _check(code: int, what: str) -> None:
    if code != 0:
        raise RomError(f"{what} failed: {load_library().rom_strerror(code).decode()} ({code})")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_contiguous():
        raise RomError("tensor arguments must be contiguous")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _weights_struct(w: Dict[str, Optional[torch.Tensor]]) -> _RomWeights:
    s = _RomWeights()
    for name, _ in _RomWeights._fields_:
        setattr(s, name, _ptr(w.get(name)))
    return s


def rom_workspace_bytes(dims: RomDims, B: int, L: int) -> int:
    return int(load_library().rom_workspace_bytes(ctypes.byref(dims), B, L))


def rom_route_workspace_bytes(dims: RomDims, N: int) -> int:
    return int(load_library().rom_route_workspace_bytes(ctypes.byref(dims), N))


def rom_workspace_layout(dims: RomDims, B: int, L: int) -> Dict[str, int]:
    lay = _RomWsLayout()
    _check(load_library().rom_workspace_layout(ctypes.byref(dims), B, L, ctypes.byref(lay)),
           "rom_workspace_layout")
    return {n: int(getattr(lay, n)) for n, _ in _RomWsLayout._fields_}


def rom_route(dims, weights, x, expert_idx, gate, counts, offsets, perm, inv_perm, logits, ws):
    n_tok = x.numel() // dims.d_model if dims.d_model else 0
    code = load_library().rom_route(
        ctypes.byref(dims), ctypes.byref(_weights_struct(weights)), _ptr(x), n_tok, _ptr(expert_idx),
        _ptr(gate), _ptr(counts), _ptr(offsets), _ptr(perm), _ptr(inv_perm), _ptr(logits), _ptr(ws),
        ws.numel() * ws.element_size() if ws is not None else 0, _stream())
    _check(code, "rom_route")


def rom_balance_stats(dims, logits, counts, n_tokens, alpha, frac, mean_prob, loss, ws):
    code = load_library().rom_balance_stats(
        ctypes.byref(dims), _ptr(logits), _ptr(counts), n_tokens, alpha, _ptr(frac), _ptr(mean_prob),
        _ptr(loss), _ptr(ws), ws.numel() * ws.element_size() if ws is not None else 0, _stream())
    _check(code, "rom_balance_stats")


def rom_layer_forward(dims, weights, x, B, L, conv_state_in, ssm_state_in, out, conv_state_out,
                      ssm_state_out, ws):
    code = load_library().rom_layer_forward(
        ctypes.byref(dims), ctypes.byref(_weights_struct(weights)), _ptr(x), B, L, _ptr(conv_state_in),
        _ptr(ssm_state_in), _ptr(out), _ptr(conv_state_out), _ptr(ssm_state_out), _ptr(ws),
        ws.numel() * ws.element_size() if ws is not None else 0, _stream())
    _check(code, "rom_layer_forward")


def rom_step(dims, weights, x, B, conv_state, ssm_state, out, ws):
    code = load_library().rom_step(
        ctypes.byref(dims), ctypes.byref(_weights_struct(weights)), _ptr(x), B, _ptr(conv_state),
        _ptr(ssm_state), _ptr(out), _ptr(ws), ws.numel() * ws.element_size() if ws is not None else 0,
        _stream())
    _check(code, "rom_step")


def rom_step_static(dims, weights, x, B, conv_state, ssm_state, out):
    code = load_library().rom_step_static(
        ctypes.byref(dims), ctypes.byref(_weights_struct(weights)), _ptr(x), B, _ptr(conv_state),
        _ptr(ssm_state), _ptr(out), _stream())
    _check(code, "rom_step_static")


def rom_backward_workspace_bytes(dims: RomDims, B: int, L: int) -> int:
    return int(load_library().rom_backward_workspace_bytes(ctypes.byref(dims), B, L))


def rom_layer_backward(dims, weights, x, B, L, d_out, d_x, grads, ws, saved=False):
    """grads: mapping d_<parameter> -> f32 tensor (d_b_router / d_conv_b may be missing or None).
    saved: rom_layer_backward_saved (ws holds the activations of the caller's own forward call)."""
    gs = _RomGrads()
    for name, _ in _RomGrads._fields_:
        setattr(gs, name, _ptr(grads.get(name)))
    lib = load_library()
    fn = lib.rom_layer_backward_saved if saved else lib.rom_layer_backward
    code = fn(ctypes.byref(dims), ctypes.byref(_weights_struct(weights)), _ptr(x), B, L, _ptr(d_out), _ptr(d_x),
              ctypes.byref(gs), _ptr(ws), _nbytes(ws), _stream())
    _check(code, "rom_layer_backward_saved" if saved else "rom_layer_backward")


def rom_block_backward_workspace_bytes(dims: RomDims, B: int, L: int) -> int:
    return int(load_library().rom_block_backward_workspace_bytes(ctypes.byref(dims), B, L))


def rom_block_forward_train(dims, weights, norm_weight, eps, x, B, L, out, ws):
    """The training step's forward of a block (plain weights), activations left in ws."""
    code = load_library().rom_block_forward_train(
        ctypes.byref(dims), ctypes.byref(_weights_struct(weights)), _ptr(norm_weight), eps, _ptr(x), B, L, _ptr(out),
        _ptr(ws), _nbytes(ws), _stream())
    _check(code, "rom_block_forward_train")


def rom_block_backward(dims, weights, norm_weight, eps, x, B, L, d_out, d_x, grads, d_norm_weight, ws, d_gate_ffn=None,
                       saved=False):
    """weights: the plain ones (w_in not folded); grads as for rom_layer_backward; d_gate_ffn: the gate
    gradient of an FFN-MoE layer on this block's routing decision (f32 [B*L, K]) or None; saved:
    rom_block_backward_saved (ws holds what rom_block_forward_train has just left)."""
    gs = _RomGrads()
    for name, _ in _RomGrads._fields_:
        setattr(gs, name, _ptr(grads.get(name)))
    lib = load_library()
    fn = lib.rom_block_backward_saved if saved else lib.rom_block_backward
    code = fn(ctypes.byref(dims), ctypes.byref(_weights_struct(weights)), _ptr(norm_weight), eps, _ptr(x), B, L, _ptr(d_out),
              _ptr(d_gate_ffn), _ptr(d_x), ctypes.byref(gs), _ptr(d_norm_weight), _ptr(ws), _nbytes(ws), _stream())
    _check(code, "rom_block_backward_saved" if saved else "rom_block_backward")


def _nbytes(t) -> int:
    return t.numel() * t.element_size() if t is not None else 0


def rom_fold_norm(dims, w_in, norm_weight, w_in_folded):
    _check(load_library().rom_fold_norm(ctypes.byref(dims), _ptr(w_in), _ptr(norm_weight),
                                        _ptr(w_in_folded), _stream()), "rom_fold_norm")


def rom_block_forward(dims, weights, norm_weight, eps, x, B, L, conv_state_in, ssm_state_in, out,
                      conv_state_out, ssm_state_out, ws):
    code = load_library().rom_block_forward(
        ctypes.byref(dims), ctypes.byref(_weights_struct(weights)), _ptr(norm_weight), eps, _ptr(x), B, L,
        _ptr(conv_state_in), _ptr(ssm_state_in), _ptr(out), _ptr(conv_state_out), _ptr(ssm_state_out),
        _ptr(ws), _nbytes(ws), _stream())
    _check(code, "rom_block_forward")


def rom_block_step(dims, weights, norm_weight, eps, x, B, conv_state, ssm_state, out, ws):
    code = load_library().rom_block_step(
        ctypes.byref(dims), ctypes.byref(_weights_struct(weights)), _ptr(norm_weight), eps, _ptr(x), B,
        _ptr(conv_state), _ptr(ssm_state), _ptr(out), _ptr(ws), _nbytes(ws), _stream())
    _check(code, "rom_block_step")


def make_blocks(layers):
    """Host array of rom_block for a list of (weights dict with folded w_in, norm_weight) pairs."""
    arr = (_RomBlock * len(layers))()
    for j, (w, norm_weight) in enumerate(layers):
        arr[j].w = _weights_struct(w)
        arr[j].norm_weight = _ptr(norm_weight)
    return arr


def rom_stack_forward(dims, blocks, eps, x, B, L, conv_state_in, ssm_state_in, out, conv_state_out,
                      ssm_state_out, tmp, ws):
    code = load_library().rom_stack_forward(
        ctypes.byref(dims), blocks, len(blocks), eps, _ptr(x), B, L, _ptr(conv_state_in),
        _ptr(ssm_state_in), _ptr(out), _ptr(conv_state_out), _ptr(ssm_state_out), _ptr(tmp), _ptr(ws),
        _nbytes(ws), _stream())
    _check(code, "rom_stack_forward")


def rom_stack_step(dims, blocks, eps, x, B, conv_state, ssm_state, out, tmp, ws):
    code = load_library().rom_stack_step(
        ctypes.byref(dims), blocks, len(blocks), eps, _ptr(x), B, _ptr(conv_state), _ptr(ssm_state),
        _ptr(out), _ptr(tmp), _ptr(ws), _nbytes(ws), _stream())
    _check(code, "rom_stack_step")


def rom_ffn_workspace_bytes(dims, d_ff: int, n_tokens: int) -> int:
    return int(load_library().rom_ffn_workspace_bytes(ctypes.byref(dims), d_ff, n_tokens))


def rom_ffn_pack_gate_up(dims, d_ff, w_gate_up, norm_weight, w_packed):
    _check(load_library().rom_ffn_pack_gate_up(ctypes.byref(dims), d_ff, _ptr(w_gate_up), _ptr(norm_weight),
                                               _ptr(w_packed), _stream()), "rom_ffn_pack_gate_up")


def rom_ffn_moe_forward(dims, d_ff, w_gate_up, w_down, pre_norm, eps, add_skip, x, n_tokens, offsets, perm,
                        inv_perm, gate, out, ws):
    w = _RomFfnWeights(_ptr(w_gate_up), _ptr(w_down))
    code = load_library().rom_ffn_moe_forward(
        ctypes.byref(dims), d_ff, ctypes.byref(w), int(bool(pre_norm)), eps, int(bool(add_skip)), _ptr(x),
        n_tokens, _ptr(offsets), _ptr(perm), _ptr(inv_perm), _ptr(gate), _ptr(out), _ptr(ws), _nbytes(ws),
        _stream())
    _check(code, "rom_ffn_moe_forward")


def rom_hybrid_stack_forward(dims, d_ff, blocks, ffns, ffn_pre_norm, eps, x, B, L, conv_state_in, ssm_state_in,
                             out, conv_state_out, ssm_state_out, tmp, ws, ffn_ws):
    code = load_library().rom_hybrid_stack_forward(
        ctypes.byref(dims), d_ff, blocks, ffns, int(bool(ffn_pre_norm)), len(blocks), eps, _ptr(x), B, L,
        _ptr(conv_state_in), _ptr(ssm_state_in), _ptr(out), _ptr(conv_state_out), _ptr(ssm_state_out),
        _ptr(tmp), _ptr(ws), _nbytes(ws), _ptr(ffn_ws), _nbytes(ffn_ws), _stream())
    _check(code, "rom_hybrid_stack_forward")


def rom_mamba2_workspace_bytes(dims: RomMamba2Dims, B: int, L: int) -> int:
    return int(load_library().rom_mamba2_workspace_bytes(ctypes.byref(dims), B, L))


def rom_mamba2_workspace_layout(dims: RomMamba2Dims, B: int, L: int) -> Dict[str, int]:
    lay = _RomMamba2WsLayout()
    _check(load_library().rom_mamba2_workspace_layout(ctypes.byref(dims), B, L, ctypes.byref(lay)),
           "rom_mamba2_workspace_layout")
    return {n: int(getattr(lay, n)) for n, _ in _RomMamba2WsLayout._fields_}


def _mamba2_weights_struct(weights) -> _RomMamba2Weights:
    s = _RomMamba2Weights()
    for name, _ in _RomMamba2Weights._fields_:
        setattr(s, name, _ptr(weights.get(name)))
    return s


def rom_mamba2_forward(dims, weights, x, B, L, eps, conv_state_in, ssm_state_in, out, conv_state_out, ssm_state_out,
                       ws):
    code = load_library().rom_mamba2_forward(
        ctypes.byref(dims), ctypes.byref(_mamba2_weights_struct(weights)), _ptr(x), B, L, eps, _ptr(conv_state_in),
        _ptr(ssm_state_in), _ptr(out), _ptr(conv_state_out), _ptr(ssm_state_out), _ptr(ws),
        ws.numel() * ws.element_size() if ws is not None else 0, _stream())
    _check(code, "rom_mamba2_forward")


def rom_fold_norm_rows(dtype, w, norm_weight, w_folded, n_rows, d_model):
    _check(load_library().rom_fold_norm_rows(dtype, _ptr(w), _ptr(norm_weight), _ptr(w_folded), n_rows, d_model, _stream()),
           "rom_fold_norm_rows")


def rom_mamba2_block_forward(dims, weights, norm_weight, norm_eps, x, B, L, eps, conv_state_in, ssm_state_in, out,
                             conv_state_out, ssm_state_out, ws):
    code = load_library().rom_mamba2_block_forward(
        ctypes.byref(dims), ctypes.byref(_mamba2_weights_struct(weights)), _ptr(norm_weight), norm_eps, _ptr(x), B, L, eps,
        _ptr(conv_state_in), _ptr(ssm_state_in), _ptr(out), _ptr(conv_state_out), _ptr(ssm_state_out), _ptr(ws),
        ws.numel() * ws.element_size() if ws is not None else 0, _stream())
    _check(code, "rom_mamba2_block_forward")


def rom_mamba2_step(dims, weights, x, B, eps, conv_state, ssm_state, out, ws):
    code = load_library().rom_mamba2_step(
        ctypes.byref(dims), ctypes.byref(_mamba2_weights_struct(weights)), _ptr(x), B, eps, _ptr(conv_state),
        _ptr(ssm_state), _ptr(out), _ptr(ws), ws.numel() * ws.element_size() if ws is not None else 0, _stream())
    _check(code, "rom_mamba2_step")


def rom_gdn_workspace_bytes(dims: RomGdnDims, B: int, L: int) -> int:
    return int(load_library().rom_gdn_workspace_bytes(ctypes.byref(dims), B, L))


def rom_gdn_workspace_layout(dims: RomGdnDims, B: int, L: int) -> Dict[str, int]:
    lay = _RomGdnWsLayout()
    _check(load_library().rom_gdn_workspace_layout(ctypes.byref(dims), B, L, ctypes.byref(lay)), "rom_gdn_workspace_layout")
    return {n: int(getattr(lay, n)) for n, _ in _RomGdnWsLayout._fields_}


def _gdn_weights_struct(weights) -> _RomGdnWeights:
    s = _RomGdnWeights()
    for name, _ in _RomGdnWeights._fields_:
        setattr(s, name, _ptr(weights.get(name)))
    return s


def rom_gdn_step(dims, weights, x, B, eps, conv_state, ssm_state, out, ws):
    code = load_library().rom_gdn_step(
        ctypes.byref(dims), ctypes.byref(_gdn_weights_struct(weights)), _ptr(x), B, eps, _ptr(conv_state), _ptr(ssm_state),
        _ptr(out), _ptr(ws), ws.numel() * ws.element_size() if ws is not None else 0, _stream())
    _check(code, "rom_gdn_step")


def rom_gdn_block_forward(dims, weights, norm_weight, norm_eps, x, B, L, eps, conv_state_in, ssm_state_in, out,
                          conv_state_out, ssm_state_out, ws):
    code = load_library().rom_gdn_block_forward(
        ctypes.byref(dims), ctypes.byref(_gdn_weights_struct(weights)), _ptr(norm_weight), norm_eps, _ptr(x), B, L, eps,
        _ptr(conv_state_in), _ptr(ssm_state_in), _ptr(out), _ptr(conv_state_out), _ptr(ssm_state_out), _ptr(ws),
        ws.numel() * ws.element_size() if ws is not None else 0, _stream())
    _check(code, "rom_gdn_block_forward")


def rom_gdn_forward(dims, weights, x, B, L, eps, conv_state_in, ssm_state_in, out, conv_state_out, ssm_state_out, ws):
    wstruct = _gdn_weights_struct(weights)
    code = load_library().rom_gdn_forward(
        ctypes.byref(dims), ctypes.byref(wstruct), _ptr(x), B, L, eps, _ptr(conv_state_in), _ptr(ssm_state_in), _ptr(out),
        _ptr(conv_state_out), _ptr(ssm_state_out), _ptr(ws), ws.numel() * ws.element_size() if ws is not None else 0,
        _stream())
    _check(code, "rom_gdn_forward")


def rom_profile_enable(max_calls: int) -> None:
    _check(load_library().rom_profile_enable(max_calls), "rom_profile_enable")


def rom_profile_select(stage_mask: int) -> None:
    """Time only the stages whose bit (1 << index in STAGE_NAMES) is set; the default is all."""
    _check(load_library().rom_profile_select(stage_mask & 0xFFFFFFFF), "rom_profile_select")


def rom_profile_collect():
    """Returns ({stage name: summed milliseconds}, number of recorded calls)."""
    ms = (ctypes.c_double * len(STAGE_NAMES))()
    n = ctypes.c_int(0)
    _check(load_library().rom_profile_collect(ms, ctypes.byref(n)), "rom_profile_collect")
    return {name: ms[i] for i, name in enumerate(STAGE_NAMES)}, n.value


def rom_profile_collect_calls(max_calls: int):
    """Per recorded call: {stage name: milliseconds}.  Returns a list of such dicts."""
    buf = (ctypes.c_double * (max(max_calls, 1) * len(STAGE_NAMES)))()
    n = ctypes.c_int(0)
    _check(load_library().rom_profile_collect_calls(buf, max_calls, ctypes.byref(n)), "rom_profile_collect_calls")
    k = len(STAGE_NAMES)
    return [{name: buf[c * k + i] for i, name in enumerate(STAGE_NAMES)} for c in range(n.value)]


def rom_profile_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    _check(load_library().rom_profile_copy(_ptr(src), _ptr(dst), _nbytes(src), _stream()), "rom_profile_copy")


def rom_probe(kind: int, p0: int, p1: int, n_blocks: int, iters: int, scratch: torch.Tensor) -> None:
    _check(load_library().rom_probe(kind, p0, p1, n_blocks, iters, _ptr(scratch), _nbytes(scratch), _stream()),
           "rom_probe")


class RomLayer:
    """Holds one layer's parameters on the GPU plus a workspace, and forwards to the C ABI."""

    _TORCH_DTYPE = {"fp32": torch.float32, "bf16": torch.bfloat16}

    def __init__(self, cfg, weights_np, device="cuda:0"):
        load_library()
        if not torch.cuda.is_available():
            raise RomError("RomLayer needs a GPU: librom has no CPU path")
        self.device = torch.device(device)
        self.tdtype = self._TORCH_DTYPE[cfg.dtype]
        self.dims = RomDims(cfg.d_model, cfg.d_inner, cfg.d_state, cfg.d_conv, cfg.dt_rank,
                            cfg.n_experts, cfg.top_k, cfg.n_experts_xdt,
                            ROM_DTYPE_BF16 if cfg.dtype == "bf16" else ROM_DTYPE_F32, cfg.gate_mode)
        typed = {"w_router", "w_in", "w_x", "w_dt", "w_out"}
        self.weights: Dict[str, Optional[torch.Tensor]] = {}
        for name, arr in weights_np.items():
            if arr is None:
                self.weights[name] = None
                continue
            t = arr if isinstance(arr, torch.Tensor) else torch.from_numpy(arr)   # host arrays or tensors
            t = t.to(self.tdtype) if name in typed else t.to(torch.float32)
            self.weights[name] = t.to(self.device).contiguous()
        self._ws: Optional[torch.Tensor] = None
        self._route_ws: Optional[torch.Tensor] = None
        self._bwd_ws: Optional[torch.Tensor] = None
        self._blk_bwd_ws: Optional[torch.Tensor] = None
        self._block_weights: Optional[Dict[str, Optional[torch.Tensor]]] = None

    def block_weights(self, in_place: bool = False) -> Dict[str, Optional[torch.Tensor]]:
        """The parameters the block entry points take: w_in with the pre-norm's scale folded in
        (rom_fold_norm), everything else shared with the plain layer.  in_place overwrites w_in
        (the plain layer calls are then no longer meaningful) instead of keeping a second copy."""
        if self._block_weights is None:
            if self.weights.get("norm_w") is None:
                raise RomError("this layer has no norm_w")
            folded = self.weights["w_in"] if in_place else torch.empty_like(self.weights["w_in"])
            rom_fold_norm(self.dims, self.weights["w_in"], self.weights["norm_w"], folded)
            self._block_weights = dict(self.weights)
            self._block_weights["w_in"] = folded
        return self._block_weights

    def block_forward(self, x: torch.Tensor, conv_state=None, ssm_state=None, return_states=False,
                      eps: float = 1e-5):
        B, L, _ = x.shape
        out = torch.empty_like(x)
        conv_out = ssm_out = None
        if return_states:
            f32 = dict(dtype=torch.float32, device=self.device)
            conv_out = torch.empty((B, self.dims.d_inner, self.dims.d_conv - 1), **f32)
            ssm_out = torch.empty((B, self.dims.d_inner, self.dims.d_state), **f32)
        rom_block_forward(self.dims, self.block_weights(), self.weights["norm_w"], eps, x, B, L, conv_state,
                          ssm_state, out, conv_out, ssm_out, self.workspace(max(B, 1), max(L, 1)))
        return (out, conv_out, ssm_out) if return_states else out

    def block_step(self, x: torch.Tensor, conv_state: torch.Tensor, ssm_state: torch.Tensor,
                   out: Optional[torch.Tensor] = None, eps: float = 1e-5):
        B = x.shape[0]
        if out is None:
            out = torch.empty_like(x)
        rom_block_step(self.dims, self.block_weights(), self.weights["norm_w"], eps, x, B, conv_state,
                       ssm_state, out, self.workspace(max(B, 1), 1))
        return out

    def to_device(self, arr, typed=True) -> torch.Tensor:
        t = torch.from_numpy(arr)
        return t.to(self.tdtype if typed else torch.float32).to(self.device).contiguous()

    def workspace(self, B: int, L: int) -> torch.Tensor:
        need = rom_workspace_bytes(self.dims, B, L)
        if need == 0:
            raise RomError("rom_workspace_bytes returned 0: unsupported dims")
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._ws

    def ws_view(self, name: str, B: int, L: int) -> torch.Tensor:
        """Intermediate tensor `name` of the last forward/step call with these B, L."""
        lay = rom_workspace_layout(self.dims, B, L)
        d, n = self.dims, B * L
        shapes = {
            "expert_idx": (torch.int32, (n, d.top_k)), "gate": (torch.float32, (n, d.top_k)),
            "counts": (torch.int32, (d.n_experts,)), "offsets": (torch.int32, (d.n_experts + 1,)),
            "perm": (torch.int32, (n * d.top_k,)), "inv_perm": (torch.int32, (n * d.top_k,)),
            "logits": (torch.float32, (n, d.n_experts)), "xz": (self.tdtype, (n, 2 * d.d_inner)),
            "u": (self.tdtype, (n, d.d_inner)), "dt_low": (self.tdtype, (n, d.dt_rank)),
            "bc": (torch.float32, (n, 2 * d.d_state)), "dt": (self.tdtype, (n, d.d_inner)),
            "g": (self.tdtype, (n, d.d_inner)),
        }
        dtype, shape = shapes[name]
        count = 1
        for s in shape:
            count *= s
        nbytes = count * torch.empty((), dtype=dtype).element_size()
        off = lay[name]
        return self._ws[off:off + nbytes].view(dtype).view(shape)

    def route(self, x: torch.Tensor):
        d = self.dims
        n = x.numel() // d.d_model
        i32 = dict(dtype=torch.int32, device=self.device)
        res = {
            "expert_idx": torch.empty((n, d.top_k), **i32),
            "gate": torch.empty((n, d.top_k), dtype=torch.float32, device=self.device),
            "counts": torch.empty((d.n_experts,), **i32),
            "offsets": torch.empty((d.n_experts + 1,), **i32),
            "perm": torch.empty((n * d.top_k,), **i32),
            "inv_perm": torch.empty((n * d.top_k,), **i32),
            "logits": torch.empty((n, d.n_experts), dtype=torch.float32, device=self.device),
        }
        need = rom_route_workspace_bytes(d, max(n, 1))
        if self._route_ws is None or self._route_ws.numel() < need:
            self._route_ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        rom_route(d, self.weights, x, res["expert_idx"], res["gate"], res["counts"], res["offsets"],
                  res["perm"], res["inv_perm"], res["logits"], self._route_ws)
        return res

    def balance_stats(self, logits: torch.Tensor, counts: torch.Tensor, alpha: float = 1e-3):
        """(frac [E], mean_prob [E], loss [1]) of Eq. (16) for router outputs of this layer."""
        E = self.dims.n_experts
        n = logits.numel() // E
        f32 = dict(dtype=torch.float32, device=self.device)
        frac, mean_prob, loss = torch.empty(E, **f32), torch.empty(E, **f32), torch.empty(1, **f32)
        # the call's scratch lies in front of the activation regions of a layer workspace
        need = rom_workspace_layout(self.dims, max(n, 1), 1)["xz"]
        if self._route_ws is None or self._route_ws.numel() < need:
            self._route_ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        rom_balance_stats(self.dims, logits, counts, n, alpha, frac, mean_prob, loss, self._route_ws)
        return frac, mean_prob, loss

    def forward(self, x: torch.Tensor, conv_state=None, ssm_state=None, return_states=False):
        B, L, _ = x.shape
        out = torch.empty_like(x)
        conv_out = ssm_out = None
        if return_states:
            conv_out = torch.empty((B, self.dims.d_inner, self.dims.d_conv - 1), dtype=torch.float32,
                                   device=self.device)
            ssm_out = torch.empty((B, self.dims.d_inner, self.dims.d_state), dtype=torch.float32,
                                  device=self.device)
        rom_layer_forward(self.dims, self.weights, x, B, L, conv_state, ssm_state, out, conv_out,
                          ssm_out, self.workspace(max(B, 1), max(L, 1)))
        return (out, conv_out, ssm_out) if return_states else out

    def step(self, x: torch.Tensor, conv_state: torch.Tensor, ssm_state: torch.Tensor,
             out: Optional[torch.Tensor] = None):
        B = x.shape[0]
        if out is None:
            out = torch.empty_like(x)
        rom_step(self.dims, self.weights, x, B, conv_state, ssm_state, out, self.workspace(max(B, 1), 1))
        return out

    def _backward_workspace(self, B: int, L: int) -> torch.Tensor:
        need = rom_backward_workspace_bytes(self.dims, max(B, 1), max(L, 1))
        if need == 0:
            raise RomError("rom_backward_workspace_bytes returned 0: unsupported dims")
        if self._bwd_ws is None or self._bwd_ws.numel() < need:
            self._bwd_ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._bwd_ws

    def forward_for_backward(self, x: torch.Tensor) -> torch.Tensor:
        """rom_layer_forward into the backward workspace (zero initial states): the out of a training
        step whose backward(x, d_out, saved=True) then skips the forward recomputation."""
        B, L, _ = x.shape
        out = torch.empty_like(x)
        rom_layer_forward(self.dims, self.weights, x, B, L, None, None, out, None, None, self._backward_workspace(B, L))
        return out

    def backward(self, x: torch.Tensor, d_out: torch.Tensor, saved: bool = False):
        """(d_x, {d_<parameter>: f32 tensor}) for the layer on input x and upstream gradient d_out.
        saved: the activations are those forward_for_backward(x) has just left (rom_layer_backward_saved)."""
        B, L, _ = x.shape
        self._backward_workspace(B, L)
        d_x = torch.empty_like(x)
        grads = {}
        for name, _ in _RomGrads._fields_:
            wt = self.weights.get(name[2:])
            if wt is not None:
                grads[name] = torch.empty(wt.shape, dtype=torch.float32, device=self.device)
        rom_layer_backward(self.dims, self.weights, x, B, L, d_out, d_x, grads, self._bwd_ws, saved=saved)
        return d_x, grads

    def _block_backward_workspace(self, B: int, L: int) -> torch.Tensor:
        need = rom_block_backward_workspace_bytes(self.dims, max(B, 1), max(L, 1))
        if need == 0:
            raise RomError("rom_block_backward_workspace_bytes returned 0: unsupported dims")
        if self._blk_bwd_ws is None or self._blk_bwd_ws.numel() < need:
            self._blk_bwd_ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._blk_bwd_ws

    def block_forward_train(self, x: torch.Tensor, eps: float = 1e-5) -> torch.Tensor:
        """The block's output by rom_block_forward_train (plain weights, activations kept in the block's
        backward workspace): block_backward(x, d_out, saved=True) then skips the forward recomputation.
        The routing decision of the call: train_routing_view(name, B, L)."""
        B, L, _ = x.shape
        out = torch.empty_like(x)
        rom_block_forward_train(self.dims, self.weights, self.weights["norm_w"], eps, x, B, L, out,
                                self._block_backward_workspace(B, L))
        return out

    def train_routing_view(self, name: str, B: int, L: int) -> torch.Tensor:
        keep = self._ws
        self._ws = self._blk_bwd_ws
        try:
            return self.ws_view(name, B, L)
        finally:
            self._ws = keep

    def block_backward(self, x: torch.Tensor, d_out: torch.Tensor, eps: float = 1e-5, d_gate_ffn=None, saved: bool = False):
        """(d_x, grads) of the pre-norm residual block out = x + layer(RMSNorm(x)); grads also holds
        d_norm_w.  Uses the plain weights (the fold of block_weights() is the forward's business).
        saved: the activations are those block_forward_train(x) has just left."""
        B, L, _ = x.shape
        self._block_backward_workspace(B, L)
        d_x = torch.empty_like(x)
        grads = {}
        for name, _ in _RomGrads._fields_:
            wt = self.weights.get(name[2:])
            if wt is not None:
                grads[name] = torch.empty(wt.shape, dtype=torch.float32, device=self.device)
        grads["d_norm_w"] = torch.empty(self.dims.d_model, dtype=torch.float32, device=self.device)
        rom_block_backward(self.dims, self.weights, self.weights["norm_w"], eps, x, B, L, d_out, d_x, grads,
                           grads["d_norm_w"], self._blk_bwd_ws, d_gate_ffn=d_gate_ffn, saved=saved)
        return d_x, grads

    def block_backward_xn(self, B: int, L: int) -> torch.Tensor:
        """The normalised input the last block_backward(B, L) call materialised (it follows the layer's
        backward plan in the workspace, 256-byte aligned)."""
        off = (rom_backward_workspace_bytes(self.dims, B, L) + 255) // 256 * 256
        n = B * L * self.dims.d_model
        nbytes = n * torch.empty((), dtype=self.tdtype).element_size()
        return self._blk_bwd_ws[off:off + nbytes].view(self.tdtype).view(B, L, self.dims.d_model)


class RomStack:
    """n_layers pre-norm residual blocks of one shape behind rom_stack_forward / rom_stack_step."""

    def __init__(self, layers, eps: float = 1e-5, fold_in_place: bool = True):
        if not layers:
            raise RomError("a stack needs at least one layer")
        self.layers = list(layers)
        self.dims = self.layers[0].dims
        self.device = self.layers[0].device
        self.eps = eps
        self._keep = [(ly.block_weights(in_place=fold_in_place), ly.weights["norm_w"]) for ly in self.layers]
        self.blocks = make_blocks(self._keep)
        self._tmp: Optional[torch.Tensor] = None

    def _scratch(self, like: torch.Tensor) -> Optional[torch.Tensor]:
        if len(self.layers) == 1:
            return None
        if self._tmp is None or self._tmp.shape != like.shape or self._tmp.dtype != like.dtype:
            self._tmp = torch.empty_like(like)
        return self._tmp

    def state_shapes(self, B: int):
        n, d = len(self.layers), self.dims
        return (n, B, d.d_inner, d.d_conv - 1), (n, B, d.d_inner, d.d_state)

    def forward(self, x: torch.Tensor, conv_state=None, ssm_state=None, return_states=False,
                out: Optional[torch.Tensor] = None):
        B, L, _ = x.shape
        if out is None:
            out = torch.empty_like(x)
        conv_out = ssm_out = None
        if return_states:
            cs, ss = self.state_shapes(B)
            conv_out = torch.empty(cs, dtype=torch.float32, device=self.device)
            ssm_out = torch.empty(ss, dtype=torch.float32, device=self.device)
        rom_stack_forward(self.dims, self.blocks, self.eps, x, B, L, conv_state, ssm_state, out, conv_out,
                          ssm_out, self._scratch(x), self.layers[0].workspace(max(B, 1), max(L, 1)))
        return (out, conv_out, ssm_out) if return_states else out

    def step(self, x: torch.Tensor, conv_state: torch.Tensor, ssm_state: torch.Tensor,
             out: Optional[torch.Tensor] = None):
        B = x.shape[0]
        if out is None:
            out = torch.empty_like(x)
        rom_stack_step(self.dims, self.blocks, self.eps, x, B, conv_state, ssm_state, out, self._scratch(x),
                       self.layers[0].workspace(max(B, 1), 1))
        return out


class RomFfnMoe:
    """An FFN-MoE layer (SwiGLU experts) that runs on the routing decision of a RomLayer call."""

    def __init__(self, layer, d_ff: int, weights, eps: float = 1e-5):
        # layer: a RomLayer, or a RomMamba2Layer / RomGdnLayer (their routing_dims() carry what the FFN call reads)
        dims = layer.dims if isinstance(layer.dims, RomDims) else layer.routing_dims()
        self.layer, self.dims, self.d_ff, self.eps = layer, dims, d_ff, eps
        self.device = layer.device
        conv = lambda a, dt: (a if isinstance(a, torch.Tensor) else torch.from_numpy(a)).to(dt).to(self.device).contiguous()
        self.w_gate_up = conv(weights["w_gate_up"], layer.tdtype)
        self.w_down = conv(weights["w_down"], layer.tdtype)
        self.norm_w = conv(weights["norm_w"], torch.float32) if weights.get("norm_w") is not None else None
        self._packed: Dict[bool, torch.Tensor] = {}
        self._ws: Optional[torch.Tensor] = None
        self._bwd_ws: Optional[torch.Tensor] = None

    def packed(self, pre_norm: bool, drop_plain: bool = False) -> torch.Tensor:
        """w_gate_up in the library's packed row order, with the pre-norm's scale folded in or not."""
        if pre_norm not in self._packed:
            out = torch.empty_like(self.w_gate_up)
            rom_ffn_pack_gate_up(self.dims, self.d_ff, self.w_gate_up, self.norm_w if pre_norm else None, out)
            self._packed[pre_norm] = out
            if drop_plain:
                torch.cuda.synchronize()
                self.w_gate_up = None
        return self._packed[pre_norm]

    def forward(self, x: torch.Tensor, routing, pre_norm: bool = False, add_skip: bool = False,
                out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """x [N, d_model] (or [B, L, d_model]); routing: mapping with offsets, perm, inv_perm, gate."""
        n = x.numel() // self.dims.d_model
        need = rom_ffn_workspace_bytes(self.dims, self.d_ff, max(n, 1))
        if need == 0:
            raise RomError("rom_ffn_workspace_bytes returned 0: unsupported dims or d_ff")
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        if out is None:
            out = torch.empty_like(x)
        rom_ffn_moe_forward(self.dims, self.d_ff, self.packed(bool(pre_norm)), self.w_down,
                            pre_norm, self.eps, add_skip, x, n, routing["offsets"], routing["perm"],
                            routing["inv_perm"], routing["gate"], out, self._ws)
        return out

    def _backward_workspace(self, n: int) -> torch.Tensor:
        need = rom_ffn_backward_workspace_bytes(self.dims, self.d_ff, max(n, 1))
        if need == 0:
            raise RomError("rom_ffn_backward_workspace_bytes returned 0: unsupported dims or d_ff")
        if self._bwd_ws is None or self._bwd_ws.numel() < need:
            self._bwd_ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._bwd_ws

    def forward_train(self, x: torch.Tensor, routing, pre_norm: bool = False, add_skip: bool = False,
                      out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """The layer's output by rom_ffn_moe_forward_train (unfolded packed weights, activations kept):
        backward(..., saved=True) with the same arguments then skips the forward recomputation."""
        n = x.numel() // self.dims.d_model
        if out is None:
            out = torch.empty_like(x)
        rom_ffn_moe_forward_train(self.dims, self.d_ff, self.packed(False), self.w_down, self.norm_w if pre_norm else None,
                                  self.eps, add_skip, x, n, routing["offsets"], routing["perm"], routing["inv_perm"],
                                  routing["gate"], out, self._backward_workspace(n))
        return out

    def backward(self, x: torch.Tensor, routing, d_out: torch.Tensor, pre_norm: bool = False, add_skip: bool = False,
                 saved: bool = False):
        """(d_x, d_gate [N, K], {d_w_gate_up (packed row order), d_w_down, d_norm_w}) of forward(x, routing, ...).
        saved: the activations are those forward_train(x, routing, ...) has just left."""
        n = x.numel() // self.dims.d_model
        self._backward_workspace(n)
        d_x = torch.empty_like(x)
        f32 = dict(dtype=torch.float32, device=self.device)
        d_gate = torch.empty((n, self.dims.top_k), **f32)
        grads = {"d_w_gate_up": torch.empty(self.w_down.shape[0], 2 * self.d_ff, self.dims.d_model, **f32),
                 "d_w_down": torch.empty(self.w_down.shape, **f32)}
        if pre_norm:
            grads["d_norm_w"] = torch.empty(self.dims.d_model, **f32)
        rom_ffn_moe_backward(self.dims, self.d_ff, self.packed(False), self.w_down, self.norm_w if pre_norm else None,
                             self.eps, add_skip, x, n, routing["offsets"], routing["perm"], routing["inv_perm"],
                             routing["gate"], d_out, d_x, d_gate, grads["d_w_gate_up"], grads["d_w_down"],
                             grads.get("d_norm_w"), self._bwd_ws, saved=saved)
        return d_x, d_gate, grads


def rom_ffn_backward_workspace_bytes(dims: RomDims, d_ff: int, N: int) -> int:
    return int(load_library().rom_ffn_backward_workspace_bytes(ctypes.byref(dims), d_ff, N))


def rom_ffn_moe_forward_train(dims, d_ff, w_gate_up_packed, w_down, norm_weight, eps, add_skip, x, N, offsets, perm,
                              inv_perm, gate, out, ws):
    wst = _RomFfnWeights(_ptr(w_gate_up_packed), _ptr(w_down))
    code = load_library().rom_ffn_moe_forward_train(
        ctypes.byref(dims), d_ff, ctypes.byref(wst), _ptr(norm_weight), eps, int(bool(add_skip)), _ptr(x), N, _ptr(offsets),
        _ptr(perm), _ptr(inv_perm), _ptr(gate), _ptr(out), _ptr(ws), _nbytes(ws), _stream())
    _check(code, "rom_ffn_moe_forward_train")


def rom_ffn_moe_backward(dims, d_ff, w_gate_up_packed, w_down, norm_weight, eps, add_skip, x, N, offsets, perm, inv_perm,
                         gate, d_out, d_x, d_gate, d_w_gate_up, d_w_down, d_norm_weight, ws, saved=False):
    """w_gate_up_packed: packed WITHOUT the norm's scale; norm_weight None: no pre-norm; saved:
    rom_ffn_moe_backward_saved (ws holds what rom_ffn_moe_forward_train has just left)."""
    wst = _RomFfnWeights(_ptr(w_gate_up_packed), _ptr(w_down))
    gst = _RomFfnGrads(_ptr(d_w_gate_up), _ptr(d_w_down), _ptr(d_norm_weight))
    lib_fn = load_library().rom_ffn_moe_backward_saved if saved else load_library().rom_ffn_moe_backward
    code = lib_fn(
        ctypes.byref(dims), d_ff, ctypes.byref(wst), _ptr(norm_weight), eps, int(bool(add_skip)), _ptr(x), N, _ptr(offsets),
        _ptr(perm), _ptr(inv_perm), _ptr(gate), _ptr(d_out), _ptr(d_x), _ptr(d_gate), ctypes.byref(gst), _ptr(ws),
        _nbytes(ws), _stream())
    _check(code, "rom_ffn_moe_backward_saved" if saved else "rom_ffn_moe_backward")


class RomHybridStack:
    """RoM blocks, each optionally followed by an FFN-MoE block that reuses its routing decision
    (rom_hybrid_stack_forward).  ffns: one RomFfnMoe or None per layer, all of the same d_ff."""

    def __init__(self, layers, ffns, eps: float = 1e-5, ffn_pre_norm: bool = True, fold_in_place: bool = True):
        if not layers or len(layers) != len(ffns):
            raise RomError("one (possibly None) FFN-MoE entry per layer")
        self.layers, self.ffns, self.eps, self.ffn_pre_norm = list(layers), list(ffns), eps, ffn_pre_norm
        self.dims, self.device = self.layers[0].dims, self.layers[0].device
        d_ffs = {f.d_ff for f in self.ffns if f is not None}
        if len(d_ffs) > 1:
            raise RomError("all FFN-MoE blocks of a stack share one d_ff")
        self.d_ff = d_ffs.pop() if d_ffs else 16
        self._keep = [(ly.block_weights(in_place=fold_in_place), ly.weights["norm_w"]) for ly in self.layers]
        self.blocks = make_blocks(self._keep)
        self._packed = [None if f is None else f.packed(ffn_pre_norm) for f in self.ffns]
        self.ffn_structs = (_RomFfnWeights * len(self.ffns))()
        for j, f in enumerate(self.ffns):
            if f is not None:
                self.ffn_structs[j] = _RomFfnWeights(_ptr(self._packed[j]), _ptr(f.w_down))
        self._tmp: Optional[torch.Tensor] = None
        self._ffn_ws: Optional[torch.Tensor] = None

    def forward(self, x: torch.Tensor, conv_state=None, ssm_state=None, return_states=False):
        B, L, _ = x.shape
        out = torch.empty_like(x)
        if self._tmp is None or self._tmp.shape != x.shape or self._tmp.dtype != x.dtype:
            self._tmp = torch.empty_like(x)
        need = rom_ffn_workspace_bytes(self.dims, self.d_ff, max(B * L, 1))
        if self._ffn_ws is None or self._ffn_ws.numel() < need:
            self._ffn_ws = torch.empty(max(need, 256), dtype=torch.uint8, device=self.device)
        conv_out = ssm_out = None
        if return_states:
            n, d = len(self.layers), self.dims
            conv_out = torch.empty((n, B, d.d_inner, d.d_conv - 1), dtype=torch.float32, device=self.device)
            ssm_out = torch.empty((n, B, d.d_inner, d.d_state), dtype=torch.float32, device=self.device)
        rom_hybrid_stack_forward(self.dims, self.d_ff, self.blocks, self.ffn_structs, self.ffn_pre_norm, self.eps, x,
                                 B, L, conv_state, ssm_state, out, conv_out, ssm_out, self._tmp,
                                 self.layers[0].workspace(max(B, 1), max(L, 1)), self._ffn_ws)
        return (out, conv_out, ssm_out) if return_states else out


class RomMamba2Layer:
    """Holds the parameters of one RoM-on-Mamba2 layer on the GPU plus a workspace, and forwards to
    rom_mamba2_forward."""

    def __init__(self, cfg, weights_np, device="cuda:0", eps: float = 1e-5):
        load_library()
        if not torch.cuda.is_available():
            raise RomError("RomMamba2Layer needs a GPU: librom has no CPU path")
        if cfg.dtype != "bf16":
            raise RomError("rom_mamba2_forward takes bf16 only")
        self.device = torch.device(device)
        self.tdtype = torch.bfloat16
        self.eps = eps
        self.dims = RomMamba2Dims(cfg.d_model, cfg.d_inner, cfg.d_state, cfg.d_conv, cfg.headdim, cfg.n_experts,
                                  cfg.top_k, ROM_DTYPE_BF16, cfg.gate_mode)
        typed = {"w_router", "w_in", "w_out"}
        self.weights: Dict[str, Optional[torch.Tensor]] = {}
        for name, arr in weights_np.items():
            if arr is None:
                self.weights[name] = None
                continue
            t = arr if isinstance(arr, torch.Tensor) else torch.from_numpy(arr)
            t = t.to(self.tdtype) if name in typed else t.to(torch.float32)
            self.weights[name] = t.to(self.device).contiguous()
        self._ws: Optional[torch.Tensor] = None

    def to_device(self, arr) -> torch.Tensor:
        return torch.from_numpy(arr).to(self.tdtype).to(self.device).contiguous()

    def workspace(self, B: int, L: int) -> torch.Tensor:
        need = rom_mamba2_workspace_bytes(self.dims, B, L)
        if need == 0:
            raise RomError("rom_mamba2_workspace_bytes returned 0: unsupported dims")
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._ws

    def ws_view(self, name: str, B: int, L: int) -> torch.Tensor:
        """Intermediate tensor `name` of the last forward call with these B, L."""
        lay = rom_mamba2_workspace_layout(self.dims, B, L)
        d, n = self.dims, B * L
        n_heads = d.d_inner // d.headdim
        shapes = {
            "expert_idx": (torch.int32, (n, d.top_k)), "gate": (torch.float32, (n, d.top_k)),
            "counts": (torch.int32, (d.n_experts,)), "offsets": (torch.int32, (d.n_experts + 1,)),
            "perm": (torch.int32, (n * d.top_k,)), "inv_perm": (torch.int32, (n * d.top_k,)),
            "logits": (torch.float32, (n, d.n_experts)),
            "zxbcdt": (self.tdtype, (n, 2 * d.d_inner + 2 * d.d_state + n_heads)),
            "xbc": (self.tdtype, (n, d.d_inner + 2 * d.d_state)),
            "yz": (self.tdtype, (n, d.d_inner)), "g": (self.tdtype, (n, d.d_inner)),
        }
        dtype, shape = shapes[name]
        count = 1
        for s in shape:
            count *= s
        nbytes = count * torch.empty((), dtype=dtype).element_size()
        off = lay[name]
        return self._ws[off:off + nbytes].view(dtype).view(shape)

    def state_shapes(self, B: int):
        d = self.dims
        return (B, d.d_inner + 2 * d.d_state, d.d_conv - 1), (B, d.d_inner // d.headdim, d.d_state, d.headdim)

    def routing_dims(self) -> RomDims:
        """What rom_ffn_moe_forward reads of a layer's dims (d_model, experts, top-k, dtype, gate mode), for an
        FFN-MoE layer that runs on this layer's routing decision; the Mamba-only fields hold valid placeholders."""
        d = self.dims
        return RomDims(d.d_model, 2 * d.d_model, 16, 4, max(d.d_model // 16, 1), d.n_experts, d.top_k, d.n_experts, d.dtype,
                       d.gate_mode)

    def forward(self, x: torch.Tensor, conv_state=None, ssm_state=None, return_states=False):
        B, L = int(x.shape[0]), int(x.shape[1])
        out = torch.empty_like(x)
        conv_out = ssm_out = None
        if return_states:
            cs, ss = self.state_shapes(B)
            conv_out = torch.empty(cs, dtype=torch.float32, device=self.device)
            ssm_out = torch.empty(ss, dtype=torch.float32, device=self.device)
        rom_mamba2_forward(self.dims, self.weights, x, B, L, self.eps, conv_state, ssm_state, out, conv_out, ssm_out,
                           self.workspace(max(B, 1), max(L, 1)))
        return (out, conv_out, ssm_out) if return_states else out

    def block_weights(self, pre_norm_w: torch.Tensor) -> Dict[str, Optional[torch.Tensor]]:
        """The weight set the block entry point expects: w_in with the pre-norm's scale folded into its
        columns (rom_fold_norm_rows, cached per pre-norm tensor), everything else shared."""
        key = (pre_norm_w.data_ptr(), pre_norm_w._version)
        if getattr(self, "_fold_key", None) != key:
            w_in = self.weights["w_in"]
            folded = torch.empty_like(w_in)
            rom_fold_norm_rows(self.dims.dtype, w_in, pre_norm_w, folded, w_in.shape[0] * w_in.shape[1], w_in.shape[2])
            self._folded = dict(self.weights, w_in=folded)
            self._fold_key = key
        return self._folded

    def block_forward(self, x: torch.Tensor, pre_norm_w: torch.Tensor, pre_norm_eps: float = 1e-5, conv_state=None,
                      ssm_state=None, return_states=False):
        """out = x + layer(RMSNorm(x)); pre_norm_w f32 [d_model] on the device."""
        B, L = int(x.shape[0]), int(x.shape[1])
        out = torch.empty_like(x)
        conv_out = ssm_out = None
        if return_states:
            cs, ss = self.state_shapes(B)
            conv_out = torch.empty(cs, dtype=torch.float32, device=self.device)
            ssm_out = torch.empty(ss, dtype=torch.float32, device=self.device)
        rom_mamba2_block_forward(self.dims, self.block_weights(pre_norm_w), pre_norm_w, pre_norm_eps, x, B, L, self.eps,
                                 conv_state, ssm_state, out, conv_out, ssm_out, self.workspace(max(B, 1), max(L, 1)))
        return (out, conv_out, ssm_out) if return_states else out

    def step(self, x: torch.Tensor, conv_state: torch.Tensor, ssm_state: torch.Tensor, out=None) -> torch.Tensor:
        """x [B, d_model]; the states are updated in place."""
        B = int(x.shape[0])
        out = torch.empty_like(x) if out is None else out
        rom_mamba2_step(self.dims, self.weights, x, B, self.eps, conv_state, ssm_state, out, self.workspace(max(B, 1), 1))
        return out


class RomGdnLayer:
    """Holds the parameters of one RoM-on-Gated-DeltaNet layer on the GPU plus a workspace, and forwards
    to rom_gdn_forward."""

    def __init__(self, cfg, weights_np, device="cuda:0", eps: float = 1e-5):
        load_library()
        if not torch.cuda.is_available():
            raise RomError("RomGdnLayer needs a GPU: librom has no CPU path")
        if cfg.dtype != "bf16":
            raise RomError("rom_gdn_forward takes bf16 only")
        self.device = torch.device(device)
        self.tdtype = torch.bfloat16
        self.eps = eps
        self.dims = RomGdnDims(cfg.d_model, cfg.n_heads, cfg.d_k, cfg.d_v, cfg.d_conv, cfg.n_experts, cfg.top_k,
                               ROM_DTYPE_BF16, cfg.gate_mode)
        typed = {"w_router", "w_in", "w_out"}
        self.weights: Dict[str, Optional[torch.Tensor]] = {}
        for name, arr in weights_np.items():
            if arr is None:
                self.weights[name] = None
                continue
            t = arr if isinstance(arr, torch.Tensor) else torch.from_numpy(arr)
            t = t.to(self.tdtype) if name in typed else t.to(torch.float32)
            self.weights[name] = t.to(self.device).contiguous()
        self._ws: Optional[torch.Tensor] = None

    def to_device(self, arr) -> torch.Tensor:
        return torch.from_numpy(arr).to(self.tdtype).to(self.device).contiguous()

    def workspace(self, B: int, L: int) -> torch.Tensor:
        need = rom_gdn_workspace_bytes(self.dims, B, L)
        if need == 0:
            raise RomError("rom_gdn_workspace_bytes returned 0: unsupported dims")
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._ws

    def state_shapes(self, B: int):
        d = self.dims
        return (B, 2 * d.n_heads * d.d_k + d.n_heads * d.d_v, d.d_conv - 1), (B, d.n_heads, d.d_k, d.d_v)

    def routing_dims(self) -> RomDims:
        """What rom_ffn_moe_forward reads of a layer's dims, for an FFN-MoE layer on this layer's routing decision."""
        d = self.dims
        return RomDims(d.d_model, 2 * d.d_model, 16, 4, max(d.d_model // 16, 1), d.n_experts, d.top_k, d.n_experts, d.dtype,
                       d.gate_mode)

    def ws_view(self, name: str, B: int, L: int) -> torch.Tensor:
        """Intermediate tensor `name` of the last forward call with these B, L."""
        lay = rom_gdn_workspace_layout(self.dims, B, L)
        d, n = self.dims, B * L
        dk, dv = d.n_heads * d.d_k, d.n_heads * d.d_v
        shapes = {
            "expert_idx": (torch.int32, (n, d.top_k)), "gate": (torch.float32, (n, d.top_k)),
            "counts": (torch.int32, (d.n_experts,)), "offsets": (torch.int32, (d.n_experts + 1,)),
            "perm": (torch.int32, (n * d.top_k,)), "inv_perm": (torch.int32, (n * d.top_k,)),
            "logits": (torch.float32, (n, d.n_experts)),
            "proj": (self.tdtype, (n, 2 * dv + 2 * dk + 2 * d.n_heads)),
            "qkv": (self.tdtype, (n, 2 * dk + dv)), "y": (self.tdtype, (n, dv)),
        }
        dtype, shape = shapes[name]
        count = 1
        for s in shape:
            count *= s
        nbytes = count * torch.empty((), dtype=dtype).element_size()
        off = lay[name]
        return self._ws[off:off + nbytes].view(dtype).view(shape)

    def forward(self, x: torch.Tensor, conv_state=None, ssm_state=None, return_states=False):
        B, L = int(x.shape[0]), int(x.shape[1])
        out = torch.empty_like(x)
        conv_out = ssm_out = None
        if return_states:
            cs, ss = self.state_shapes(B)
            conv_out = torch.empty(cs, dtype=torch.float32, device=self.device)
            ssm_out = torch.empty(ss, dtype=torch.float32, device=self.device)
        rom_gdn_forward(self.dims, self.weights, x, B, L, self.eps, conv_state, ssm_state, out, conv_out, ssm_out,
                        self.workspace(max(B, 1), max(L, 1)))
        return (out, conv_out, ssm_out) if return_states else out

    def block_weights(self, pre_norm_w: torch.Tensor) -> Dict[str, Optional[torch.Tensor]]:
        """The weight set the block entry point expects: w_in with the pre-norm's scale folded into its
        columns (rom_fold_norm_rows, cached per pre-norm tensor), everything else shared."""
        key = (pre_norm_w.data_ptr(), pre_norm_w._version)
        if getattr(self, "_fold_key", None) != key:
            w_in = self.weights["w_in"]
            folded = torch.empty_like(w_in)
            rom_fold_norm_rows(self.dims.dtype, w_in, pre_norm_w, folded, w_in.shape[0] * w_in.shape[1], w_in.shape[2])
            self._folded = dict(self.weights, w_in=folded)
            self._fold_key = key
        return self._folded

    def block_forward(self, x: torch.Tensor, pre_norm_w: torch.Tensor, pre_norm_eps: float = 1e-5, conv_state=None,
                      ssm_state=None, return_states=False):
        """out = x + layer(RMSNorm(x)); pre_norm_w f32 [d_model] on the device."""
        B, L = int(x.shape[0]), int(x.shape[1])
        out = torch.empty_like(x)
        conv_out = ssm_out = None
        if return_states:
            cs, ss = self.state_shapes(B)
            conv_out = torch.empty(cs, dtype=torch.float32, device=self.device)
            ssm_out = torch.empty(ss, dtype=torch.float32, device=self.device)
        rom_gdn_block_forward(self.dims, self.block_weights(pre_norm_w), pre_norm_w, pre_norm_eps, x, B, L, self.eps,
                              conv_state, ssm_state, out, conv_out, ssm_out, self.workspace(max(B, 1), max(L, 1)))
        return (out, conv_out, ssm_out) if return_states else out

    def step(self, x: torch.Tensor, conv_state: torch.Tensor, ssm_state: torch.Tensor, out=None) -> torch.Tensor:
        """x [B, d_model]; the states are updated in place."""
        B = int(x.shape[0])
        out = torch.empty_like(x) if out is None else out
        rom_gdn_step(self.dims, self.weights, x, B, self.eps, conv_state, ssm_state, out, self.workspace(max(B, 1), 1))
        return out
