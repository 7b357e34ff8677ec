"""Thin Python binding of the SSA C ABI (``include/ssa.h``): argument marshalling only.

PyTorch supplies device memory and the stream; every step of the path runs in the HIP library.  The
functions mirror the C entry points by name.  Loading fails loudly when ``lib/libssa_hip.so`` has not been
built (``python -m paper_2505_17412_amd.build``); there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libssa_hip.so")

SSA_BF16, SSA_F32 = 0, 1
ARRAYS = dict(perm=0, inv_perm=1, cmp_start=2, slc_start=3, win_start=4, slc_child_start=5, cmp_batch=6,
              slc_batch=7, tok_win=8)
EXPORTED_SYMBOLS = (
    "ssa_build_blocks", "ssa_build_blocks_1d", "ssa_blocks_counts", "ssa_blocks_max_slc_per_item", "ssa_blocks_export",
    "ssa_blocks_destroy", "ssa_workspace_bytes", "ssa_forward", "ssa_backward", "ssa_topk_from_scores",
    "ssa_error_string", "ssa_profile_enable", "ssa_profile_num_kernels", "ssa_profile_get",
    "ssa_compress_workspace_bytes", "ssa_compress_forward", "ssa_compress_backward", "ssa_forward_pooled",
    "ssa_backward_pooled", "ssa_gate_workspace_bytes", "ssa_gate_forward", "ssa_gate_backward", "ssa_gate_forward_static",
    "ssa_linear_workspace_bytes", "ssa_linear_forward", "ssa_linear_backward",
    "ssa_layer_saved_bytes", "ssa_layer_workspace_bytes", "ssa_layer_forward", "ssa_layer_backward",
)


class ssa_layer_weights_t(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("wq", "wk", "wv", "wg", "bg", "wo", "bq", "bk", "bv", "bo",
                                                 "pe_k", "wc_k", "bc_k", "pe_v", "wc_v", "bc_v")]


class ssa_layer_grads_t(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("dwq", "dwk", "dwv", "dwg", "dbg", "dwo", "dbq", "dbk", "dbv", "dbo",
                                                 "dpe_k", "dwc_k", "dbc_k", "dpe_v", "dwc_v", "dbc_v")]


class ssa_params_t(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_tokens", "n_batch", "grid", "m_cmp", "m_slc", "m_win", "topk",
                                         "n_heads_q", "n_heads_kv", "head_dim", "dtype")] + [("scale", C.c_float)]


class ssa_cmp_weights_t(C.Structure):
    _fields_ = [("pe", C.c_void_p), ("w", C.c_void_p), ("bias", C.c_void_p)]


class SSAError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {error_string(status)} ({status})")


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2505_17412_amd.build`")
        L = C.CDLL(_LIB_PATH)
        vp, i32p = C.c_void_p, C.POINTER(C.c_int32)
        L.ssa_build_blocks.argtypes = [C.POINTER(ssa_params_t), vp, vp, vp, C.POINTER(vp)]
        L.ssa_build_blocks_1d.argtypes = [C.POINTER(ssa_params_t), vp, vp, C.POINTER(vp)]
        L.ssa_blocks_counts.argtypes = [vp, i32p, i32p, i32p]
        L.ssa_blocks_max_slc_per_item.argtypes = [vp, i32p]
        L.ssa_blocks_export.argtypes = [vp, C.c_int, vp, C.c_size_t, vp]
        L.ssa_blocks_destroy.argtypes = [vp]
        L.ssa_blocks_destroy.restype = None
        L.ssa_workspace_bytes.argtypes = [C.POINTER(ssa_params_t), vp, C.c_int]
        L.ssa_workspace_bytes.restype = C.c_size_t
        L.ssa_forward.argtypes = [C.POINTER(ssa_params_t), vp] + [vp] * 8 + [vp, C.c_size_t, vp]
        L.ssa_backward.argtypes = [C.POINTER(ssa_params_t), vp] + [vp] * 12 + [vp, C.c_size_t, vp]
        L.ssa_topk_from_scores.argtypes = [C.POINTER(ssa_params_t), vp, vp, vp, vp]
        L.ssa_compress_workspace_bytes.argtypes = [C.POINTER(ssa_params_t), vp, C.c_int]
        L.ssa_compress_workspace_bytes.restype = C.c_size_t
        L.ssa_compress_forward.argtypes = [C.POINTER(ssa_params_t), vp, vp, C.POINTER(ssa_cmp_weights_t), vp, vp, C.c_size_t, vp]
        L.ssa_compress_backward.argtypes = [C.POINTER(ssa_params_t), vp, vp, C.POINTER(ssa_cmp_weights_t)] + [vp] * 5 + \
            [vp, C.c_size_t, vp]
        L.ssa_linear_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int]
        L.ssa_linear_workspace_bytes.restype = C.c_size_t
        L.ssa_linear_forward.argtypes = [C.c_int32] * 3 + [vp] * 5
        L.ssa_linear_backward.argtypes = [C.c_int32] * 3 + [vp] * 6 + [vp, C.c_size_t, vp]
        L.ssa_layer_saved_bytes.argtypes = [C.POINTER(ssa_params_t), C.POINTER(C.c_size_t)]
        L.ssa_layer_saved_bytes.restype = C.c_size_t
        L.ssa_layer_workspace_bytes.argtypes = [C.POINTER(ssa_params_t), vp, C.c_int32, C.c_int]
        L.ssa_layer_workspace_bytes.restype = C.c_size_t
        L.ssa_layer_forward.argtypes = [C.POINTER(ssa_params_t), vp, C.c_int32, vp, C.POINTER(ssa_layer_weights_t), vp, vp, C.c_size_t, vp, C.c_size_t, vp]
        L.ssa_layer_backward.argtypes = [C.POINTER(ssa_params_t), vp, C.c_int32, vp, C.POINTER(ssa_layer_weights_t), vp, vp, vp, C.POINTER(ssa_layer_grads_t), vp, C.c_size_t, vp]
        L.ssa_gate_workspace_bytes.argtypes = [C.POINTER(ssa_params_t), C.c_int32, C.c_int]
        L.ssa_gate_workspace_bytes.restype = C.c_size_t
        L.ssa_gate_forward.argtypes = [C.POINTER(ssa_params_t), C.c_int32] + [vp] * 4 + [vp, C.c_size_t, vp]
        L.ssa_gate_backward.argtypes = [C.POINTER(ssa_params_t), C.c_int32] + [vp] * 7 + [vp, C.c_size_t, vp]
        L.ssa_gate_forward_static.argtypes = [C.POINTER(ssa_params_t), C.c_int32] + [vp] * 4 + [vp]
        L.ssa_forward_pooled.argtypes = [C.POINTER(ssa_params_t), vp] + [vp] * 10 + [vp, C.c_size_t, vp]
        L.ssa_backward_pooled.argtypes = [C.POINTER(ssa_params_t), vp] + [vp] * 16 + [vp, C.c_size_t, vp]
        L.ssa_profile_enable.argtypes = [C.c_int]
        L.ssa_profile_get.argtypes = [C.c_int, C.POINTER(C.c_char_p), C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        L.ssa_error_string.argtypes = [C.c_int]
        L.ssa_error_string.restype = C.c_char_p
        _lib = L
    return _lib


def error_string(status: int) -> str:
    return lib().ssa_error_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise SSAError(status, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous(), "tensors must be contiguous"
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def make_params(n_tokens, n_batch, grid, m_cmp, m_slc, m_win, topk, n_heads_q, n_heads_kv, head_dim, dtype,
                scale: float = 0.0) -> ssa_params_t:
    code = {"bf16": SSA_BF16, "f32": SSA_F32, torch.bfloat16: SSA_BF16, torch.float32: SSA_F32}.get(dtype, dtype)
    return ssa_params_t(n_tokens, n_batch, grid, m_cmp, m_slc, m_win, topk, n_heads_q, n_heads_kv, head_dim,
                        int(code), float(scale))


class Blocks:
    """Owner of an ``ssa_blocks_t*``."""

    def __init__(self, handle: int, params: ssa_params_t):
        self.handle = handle
        self.params = params

    def counts(self) -> Tuple[int, int, int]:
        a, b, c = C.c_int32(), C.c_int32(), C.c_int32()
        _check(lib().ssa_blocks_counts(self.handle, C.byref(a), C.byref(b), C.byref(c)), "ssa_blocks_counts")
        return a.value, b.value, c.value

    def max_slc_per_item(self) -> int:
        a = C.c_int32()
        _check(lib().ssa_blocks_max_slc_per_item(self.handle, C.byref(a)), "ssa_blocks_max_slc_per_item")
        return a.value

    def export(self, name: str) -> torch.Tensor:
        nc, ns, nw = self.counts()
        p = self.params
        n = dict(perm=p.n_tokens, inv_perm=p.n_tokens, cmp_start=nc + 1, slc_start=ns + 1, win_start=nw + 1,
                 slc_child_start=ns + 1, cmp_batch=p.n_batch + 1, slc_batch=p.n_batch + 1, tok_win=p.n_tokens)[name]
        dst = torch.empty(max(n, 1), dtype=torch.int32, device="cuda")
        _check(lib().ssa_blocks_export(self.handle, ARRAYS[name], dst.data_ptr(), dst.numel() * 4, _stream()),
               "ssa_blocks_export")
        return dst[:n]

    def destroy(self) -> None:
        if self.handle:
            lib().ssa_blocks_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def ssa_build_blocks(params: ssa_params_t, coords: torch.Tensor, batch_offsets: torch.Tensor) -> Blocks:
    """coords: cuda int32 [N,3]; batch_offsets: cuda int32 [B+1]."""
    assert coords.dtype == torch.int32 and batch_offsets.dtype == torch.int32
    h = C.c_void_p()
    _check(lib().ssa_build_blocks(C.byref(params), _ptr(coords), _ptr(batch_offsets), _stream(), C.byref(h)),
           "ssa_build_blocks")
    return Blocks(h.value, params)


def ssa_build_blocks_1d(params: ssa_params_t, batch_offsets: torch.Tensor) -> Blocks:
    """Sequence partition: m_cmp / m_slc / m_win of ``params`` are block lengths in tokens; batch_offsets: cuda int32 [B+1]."""
    assert batch_offsets.dtype == torch.int32
    h = C.c_void_p()
    _check(lib().ssa_build_blocks_1d(C.byref(params), _ptr(batch_offsets), _stream(), C.byref(h)), "ssa_build_blocks_1d")
    return Blocks(h.value, params)


def ssa_workspace_bytes(params: ssa_params_t, blocks: Blocks, for_backward: bool) -> int:
    return int(lib().ssa_workspace_bytes(C.byref(params), blocks.handle, int(for_backward)))


def ssa_forward(params, blocks: Blocks, q, k, v, gates, out, lse=None, topk_idx=None, out_branch=None,
                workspace: Optional[torch.Tensor] = None) -> None:
    if workspace is None:
        workspace = torch.empty(ssa_workspace_bytes(params, blocks, False), dtype=torch.uint8, device="cuda")
    _check(lib().ssa_forward(C.byref(params), blocks.handle, _ptr(q), _ptr(k), _ptr(v), _ptr(gates), _ptr(out),
                             _ptr(lse), _ptr(topk_idx), _ptr(out_branch), _ptr(workspace), workspace.numel(),
                             _stream()), "ssa_forward")


def ssa_backward(params, blocks: Blocks, q, k, v, gates, out_branch, lse, topk_idx, dout, dq, dk, dv, dgates,
                 workspace: Optional[torch.Tensor] = None) -> None:
    if workspace is None:
        workspace = torch.empty(ssa_workspace_bytes(params, blocks, True), dtype=torch.uint8, device="cuda")
    _check(lib().ssa_backward(C.byref(params), blocks.handle, _ptr(q), _ptr(k), _ptr(v), _ptr(gates),
                              _ptr(out_branch), _ptr(lse), _ptr(topk_idx), _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv),
                              _ptr(dgates), _ptr(workspace), workspace.numel(), _stream()), "ssa_backward")


def ssa_compress_workspace_bytes(params: ssa_params_t, blocks: Blocks, for_backward: bool) -> int:
    return int(lib().ssa_compress_workspace_bytes(C.byref(params), blocks.handle, int(for_backward)))


def _weights(pe, w, bias) -> ssa_cmp_weights_t:
    return ssa_cmp_weights_t(_ptr(pe), _ptr(w), _ptr(bias))


def ssa_compress_forward(params, blocks: Blocks, x, pe, w, bias, x_cmp, workspace: Optional[torch.Tensor] = None) -> None:
    if workspace is None:
        workspace = torch.empty(ssa_compress_workspace_bytes(params, blocks, False), dtype=torch.uint8, device="cuda")
    wt = _weights(pe, w, bias)
    _check(lib().ssa_compress_forward(C.byref(params), blocks.handle, _ptr(x), C.byref(wt), _ptr(x_cmp), _ptr(workspace),
                                      workspace.numel(), _stream()), "ssa_compress_forward")


def ssa_compress_backward(params, blocks: Blocks, x, pe, w, bias, dx_cmp, dx_accum, dpe, dw, dbias,
                          workspace: Optional[torch.Tensor] = None) -> None:
    if workspace is None:
        workspace = torch.empty(ssa_compress_workspace_bytes(params, blocks, True), dtype=torch.uint8, device="cuda")
    wt = _weights(pe, w, bias)
    _check(lib().ssa_compress_backward(C.byref(params), blocks.handle, _ptr(x), C.byref(wt), _ptr(dx_cmp), _ptr(dx_accum),
                                       _ptr(dpe), _ptr(dw), _ptr(dbias), _ptr(workspace), workspace.numel(), _stream()),
           "ssa_compress_backward")


def ssa_forward_pooled(params, blocks: Blocks, q, k, v, gates, k_cmp, v_cmp, out, lse=None, topk_idx=None, out_branch=None,
                       workspace: Optional[torch.Tensor] = None) -> None:
    if workspace is None:
        workspace = torch.empty(ssa_workspace_bytes(params, blocks, False), dtype=torch.uint8, device="cuda")
    _check(lib().ssa_forward_pooled(C.byref(params), blocks.handle, _ptr(q), _ptr(k), _ptr(v), _ptr(gates), _ptr(k_cmp),
                                    _ptr(v_cmp), _ptr(out), _ptr(lse), _ptr(topk_idx), _ptr(out_branch), _ptr(workspace),
                                    workspace.numel(), _stream()), "ssa_forward_pooled")


def ssa_backward_pooled(params, blocks: Blocks, q, k, v, gates, k_cmp, v_cmp, out_branch, lse, topk_idx, dout, dq, dk, dv,
                        dgates, dk_cmp, dv_cmp, workspace: Optional[torch.Tensor] = None) -> None:
    if workspace is None:
        workspace = torch.empty(ssa_workspace_bytes(params, blocks, True), dtype=torch.uint8, device="cuda")
    _check(lib().ssa_backward_pooled(C.byref(params), blocks.handle, _ptr(q), _ptr(k), _ptr(v), _ptr(gates), _ptr(k_cmp),
                                     _ptr(v_cmp), _ptr(out_branch), _ptr(lse), _ptr(topk_idx), _ptr(dout), _ptr(dq),
                                     _ptr(dk), _ptr(dv), _ptr(dgates), _ptr(dk_cmp), _ptr(dv_cmp), _ptr(workspace),
                                     workspace.numel(), _stream()), "ssa_backward_pooled")


def ssa_gate_workspace_bytes(params: ssa_params_t, d_model: int, for_backward: bool) -> int:
    return int(lib().ssa_gate_workspace_bytes(C.byref(params), int(d_model), int(for_backward)))


def ssa_gate_forward(params, d_model: int, x, w, bias, gates, workspace: Optional[torch.Tensor] = None) -> None:
    if workspace is None:
        workspace = torch.empty(ssa_gate_workspace_bytes(params, d_model, False), dtype=torch.uint8, device="cuda")
    _check(lib().ssa_gate_forward(C.byref(params), int(d_model), _ptr(x), _ptr(w), _ptr(bias), _ptr(gates), _ptr(workspace),
                                  workspace.numel(), _stream()), "ssa_gate_forward")


def ssa_gate_forward_static(params, d_model: int, x, w, bias, gates) -> None:
    _check(lib().ssa_gate_forward_static(C.byref(params), int(d_model), _ptr(x), _ptr(w), _ptr(bias), _ptr(gates), _stream()),
           "ssa_gate_forward_static")


def ssa_gate_backward(params, d_model: int, x, w, gates, dgates, dx_accum, dw, dbias,
                      workspace: Optional[torch.Tensor] = None) -> None:
    if workspace is None:
        workspace = torch.empty(ssa_gate_workspace_bytes(params, d_model, True), dtype=torch.uint8, device="cuda")
    _check(lib().ssa_gate_backward(C.byref(params), int(d_model), _ptr(x), _ptr(w), _ptr(gates), _ptr(dgates), _ptr(dx_accum),
                                   _ptr(dw), _ptr(dbias), _ptr(workspace), workspace.numel(), _stream()), "ssa_gate_backward")


def ssa_topk_from_scores(params, blocks: Blocks, scores: torch.Tensor, topk_idx: torch.Tensor) -> None:
    assert scores.dtype == torch.float32 and topk_idx.dtype == torch.int32
    _check(lib().ssa_topk_from_scores(C.byref(params), blocks.handle, _ptr(scores), _ptr(topk_idx), _stream()),
           "ssa_topk_from_scores")


def ssa_profile_enable(on: bool) -> None:
    _check(lib().ssa_profile_enable(int(on)), "ssa_profile_enable")


def ssa_profile_get() -> dict:
    """{kernel name: (total_ms, launches)} since the last ssa_profile_enable."""
    res = {}
    for i in range(lib().ssa_profile_num_kernels()):
        name, ms, cnt = C.c_char_p(), C.c_double(), C.c_int64()
        _check(lib().ssa_profile_get(i, C.byref(name), C.byref(ms), C.byref(cnt)), "ssa_profile_get")
        if cnt.value:
            res[name.value.decode()] = (ms.value, cnt.value)
    return res


def ssa_linear_workspace_bytes(n_tokens: int, d_in: int, d_out: int, for_backward: bool) -> int:
    return int(lib().ssa_linear_workspace_bytes(n_tokens, d_in, d_out, int(for_backward)))


def ssa_linear_forward(x, w, bias, y) -> None:
    """y [N,d_out] = x [N,d_in] w[d_out,d_in]^T + bias (bf16 cuda tensors; bias may be None)."""
    n, d_in = x.shape
    _check(lib().ssa_linear_forward(n, d_in, w.shape[0], _ptr(x), _ptr(w), _ptr(bias), _ptr(y), _stream()),
           "ssa_linear_forward")


def ssa_linear_backward(x, w, dy, dx, dw, dbias=None, workspace: Optional[torch.Tensor] = None) -> None:
    n, d_in = x.shape
    d_out = w.shape[0]
    if workspace is None:
        workspace = torch.empty(max(ssa_linear_workspace_bytes(n, d_in, d_out, True), 1), dtype=torch.uint8, device="cuda")
    _check(lib().ssa_linear_backward(n, d_in, d_out, _ptr(x), _ptr(w), _ptr(dy), _ptr(dx), _ptr(dw), _ptr(dbias),
                                     _ptr(workspace), workspace.numel(), _stream()), "ssa_linear_backward")


LAYER_SAVED = ("q", "k", "v", "gates", "o", "out_branch", "lse", "topk_idx")


def ssa_layer_saved_bytes(params: ssa_params_t):
    """(bytes, {name: byte offset from the 256-byte aligned start}) of the activations the layer keeps for backward."""
    offs = (C.c_size_t * 8)()
    n = int(lib().ssa_layer_saved_bytes(C.byref(params), offs))
    return n, dict(zip(LAYER_SAVED, (int(o) for o in offs)))


def ssa_layer_workspace_bytes(params: ssa_params_t, blocks: Blocks, d_model: int, for_backward: bool) -> int:
    return int(lib().ssa_layer_workspace_bytes(C.byref(params), blocks.handle, d_model, int(for_backward)))


def _layer_struct(cls, tensors: dict):
    return cls(**{k: _ptr(tensors.get(k)) for k, _ in cls._fields_})


def ssa_layer_forward(params, blocks: Blocks, x, weights: dict, y, saved, workspace: Optional[torch.Tensor] = None) -> None:
    """weights: dict of cuda bf16 tensors wq, wk, wv, wg, bg, wo (+ optional bq, bk, bv, bo; + pe_k, wc_k, bc_k, pe_v,
    wc_v, bc_v for the learned compression module on keys and values, all six or none)."""
    d_model = x.shape[1]
    if workspace is None:
        workspace = torch.empty(max(ssa_layer_workspace_bytes(params, blocks, d_model, False), 1), dtype=torch.uint8, device="cuda")
    w = _layer_struct(ssa_layer_weights_t, weights)
    _check(lib().ssa_layer_forward(C.byref(params), blocks.handle, d_model, _ptr(x), C.byref(w), _ptr(y), _ptr(saved),
                                   saved.numel(), _ptr(workspace), workspace.numel(), _stream()), "ssa_layer_forward")


def ssa_layer_backward(params, blocks: Blocks, x, weights: dict, saved, dy, dx, grads: dict,
                       workspace: Optional[torch.Tensor] = None) -> None:
    """grads: dict of cuda float tensors dwq, dwk, dwv, dwg, dbg, dwo (+ optional dbq, dbk, dbv, dbo; + dpe_k, dwc_k,
    dbc_k, dpe_v, dwc_v, dbc_v when the module's weights are given), overwritten."""
    d_model = x.shape[1]
    if workspace is None:
        workspace = torch.empty(max(ssa_layer_workspace_bytes(params, blocks, d_model, True), 1), dtype=torch.uint8, device="cuda")
    w = _layer_struct(ssa_layer_weights_t, weights)
    g = _layer_struct(ssa_layer_grads_t, grads)
    _check(lib().ssa_layer_backward(C.byref(params), blocks.handle, d_model, _ptr(x), C.byref(w), _ptr(saved), _ptr(dy),
                                    _ptr(dx), C.byref(g), _ptr(workspace), workspace.numel(), _stream()), "ssa_layer_backward")
