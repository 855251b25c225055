"""ctypes binding of the C ABI in include/des.h.

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  torch is used for device memory and for the current stream.  There
is no fallback: if the compiled library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdes_hip.so")

DES_VANILLA, DES_SEQ, DES_VOTE = 0, 1, 2
DES_F32, DES_BF16 = 0, 1
DES_LAYOUT_ROWMAJOR, DES_LAYOUT_PACKED = 0, 1
MODES = {"vanilla": DES_VANILLA, "seq": DES_SEQ, "vote": DES_VOTE}

EXPORTS = (
    "des_coreset_capacity", "des_workspace_bytes", "des_route", "des_select_coreset",
    "des_moe_forward", "des_moe_forward_builtin_ws", "des_stack_workspace_bytes", "des_moe_stack_forward",
    "des_pack_expert_weights", "des_strerror", "des_last_hip_error",
    "des_kernel_timing_enable", "des_kernel_timing_count", "des_kernel_timing_name",
    "des_kernel_timing_read", "des_hbm_read_probe", "des_coreset_from_beta", "des_test_hooks",
    "des_attention_workspace_bytes", "des_block_attention", "des_decoder_workspace_bytes",
    "des_decoder_stack_forward",
)


DES_ROUTER_SOFTMAX, DES_ROUTER_SIGMOID = 0, 1
ROUTER_ACTS = {"softmax": DES_ROUTER_SOFTMAX, "sigmoid": DES_ROUTER_SIGMOID}
DES_GROUP_MAX, DES_GROUP_TOP2SUM = 1, 2
GROUP_SCORES = {"max": DES_GROUP_MAX, "top2sum": DES_GROUP_TOP2SUM}


class DesShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "n_seqs", "n_tokens", "hidden", "n_experts", "ffn", "ffn_shared", "top_k", "coreset",
        "k_seq", "mode", "dtype", "weight_layout", "residual", "k_route")] + [
        ("skip_beta", ctypes.c_float), ("router_act", ctypes.c_int32), ("vote_renorm", ctypes.c_int32),
        ("n_group", ctypes.c_int32), ("topk_group", ctypes.c_int32), ("group_score", ctypes.c_int32),
        ("vote_atomic", ctypes.c_int32)]


class DesAttnShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("n_heads", "n_kv_heads", "head_dim", "n_prefix", "n_suffix")]


class DesError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"des error {code}: {text}")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """The compiled library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2602_00879_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        sp = ctypes.POINTER(DesShape)
        L.des_coreset_capacity.restype = i32
        L.des_coreset_capacity.argtypes = [sp]
        L.des_workspace_bytes.restype = sz
        L.des_workspace_bytes.argtypes = [sp]
        L.des_stack_workspace_bytes.restype = sz
        L.des_stack_workspace_bytes.argtypes = [sp]
        ap = ctypes.POINTER(DesAttnShape)
        L.des_attention_workspace_bytes.restype = sz
        L.des_attention_workspace_bytes.argtypes = [sp, ap]
        L.des_decoder_workspace_bytes.restype = sz
        L.des_decoder_workspace_bytes.argtypes = [sp, ap]
        L.des_block_attention.restype = ctypes.c_int
        L.des_block_attention.argtypes = [sp, ap] + [vp] * 9 + [sz, vp]
        L.des_decoder_stack_forward.restype = ctypes.c_int
        L.des_decoder_stack_forward.argtypes = [sp, ap, i32] + [vp] * 19 + [sz, vp]
        L.des_route.restype = ctypes.c_int
        L.des_route.argtypes = [sp] + [vp] * 6
        L.des_select_coreset.restype = ctypes.c_int
        L.des_select_coreset.argtypes = [sp] + [vp] * 6
        L.des_moe_forward.restype = ctypes.c_int
        L.des_moe_forward.argtypes = [sp] + [vp] * 18 + [sz, vp]
        L.des_moe_forward_builtin_ws.restype = ctypes.c_int
        L.des_moe_forward_builtin_ws.argtypes = [sp] + [vp] * 18
        L.des_moe_stack_forward.restype = ctypes.c_int
        L.des_moe_stack_forward.argtypes = [sp, i32] + [vp] * 13 + [sz, vp]
        L.des_pack_expert_weights.restype = ctypes.c_int
        L.des_pack_expert_weights.argtypes = [vp, vp, ctypes.c_int64, i32, i32, vp]
        L.des_hbm_read_probe.restype = ctypes.c_int
        L.des_hbm_read_probe.argtypes = [vp, sz, vp, vp]
        L.des_coreset_from_beta.restype = i32
        L.des_coreset_from_beta.argtypes = [ctypes.c_double, i32]
        L.des_test_hooks.restype = ctypes.c_int
        L.des_test_hooks.argtypes = [ctypes.c_int, ctypes.c_int]
        L.des_strerror.restype = ctypes.c_char_p
        L.des_strerror.argtypes = [ctypes.c_int]
        L.des_last_hip_error.restype = ctypes.c_char_p
        L.des_last_hip_error.argtypes = []
        L.des_kernel_timing_enable.restype = ctypes.c_int
        L.des_kernel_timing_enable.argtypes = [ctypes.c_int]
        L.des_kernel_timing_count.restype = ctypes.c_int
        L.des_kernel_timing_count.argtypes = []
        L.des_kernel_timing_name.restype = ctypes.c_char_p
        L.des_kernel_timing_name.argtypes = [ctypes.c_int]
        L.des_kernel_timing_read.restype = ctypes.c_int
        L.des_kernel_timing_read.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_double),
                                             ctypes.POINTER(ctypes.c_int64)]
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().des_strerror(code).decode()


def _check(code: int) -> None:
    if code != 0:
        text = strerror(code)
        if code == -6:
            text += ": " + lib().des_last_hip_error().decode()
        raise DesError(code, text)


def make_shape(n_seqs: int, n_tokens: int, hidden: int, n_experts: int, ffn: int, top_k: int,
               coreset: int, mode, dtype, ffn_shared: int = 0, k_seq: int = 0,
               weight_layout: int = DES_LAYOUT_ROWMAJOR, residual: int = 0, k_route: int = 0,
               skip_beta: float = 0.0, router_act=0, vote_renorm: int = 0, n_group: int = 0,
               topk_group: int = 0, group_score=DES_GROUP_MAX, vote_atomic: int = 0) -> DesShape:
    if isinstance(mode, str):
        mode = MODES[mode]
    if isinstance(dtype, str):
        dtype = {"f32": DES_F32, "bf16": DES_BF16}[dtype]
    elif isinstance(dtype, torch.dtype):
        dtype = {torch.float32: DES_F32, torch.bfloat16: DES_BF16}[dtype]
    return DesShape(n_seqs, n_tokens, hidden, n_experts, ffn, ffn_shared, top_k, coreset, k_seq,
                    mode, dtype, weight_layout, residual, k_route, skip_beta,
                    ROUTER_ACTS[router_act] if isinstance(router_act, str) else router_act, vote_renorm,
                    n_group, topk_group,
                    GROUP_SCORES[group_score] if isinstance(group_score, str) else group_score, vote_atomic)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_contiguous(), "tensors handed to the library must be contiguous"
    return ctypes.c_void_p(t.data_ptr())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def des_coreset_capacity(shape: DesShape) -> int:
    return int(lib().des_coreset_capacity(ctypes.byref(shape)))


def des_workspace_bytes(shape: DesShape) -> int:
    return int(lib().des_workspace_bytes(ctypes.byref(shape)))


def des_stack_workspace_bytes(shape: DesShape) -> int:
    return int(lib().des_stack_workspace_bytes(ctypes.byref(shape)))


def des_route(shape: DesShape, x: torch.Tensor, w_router: torch.Tensor,
              router_bias: Optional[torch.Tensor], want_probs: bool = True
              ) -> Tuple[torch.Tensor, Optional[torch.Tensor]]:
    B, N, M = shape.n_seqs, shape.n_tokens, shape.n_experts
    logits = torch.empty((B, N, M), dtype=torch.float32, device=x.device)
    probs = torch.empty_like(logits) if want_probs else None
    _check(lib().des_route(ctypes.byref(shape), _ptr(x), _ptr(w_router), _ptr(router_bias),
                           _ptr(logits), _ptr(probs), _stream()))
    return logits, probs


def des_select_coreset(shape: DesShape, logits: torch.Tensor,
                       out: Optional[Dict[str, torch.Tensor]] = None) -> Dict[str, torch.Tensor]:
    """`out`: the dict of a previous call, to reuse its output tensors."""
    B, M = shape.n_seqs, shape.n_experts
    cap = des_coreset_capacity(shape)
    dev = logits.device
    out = out if out is not None else dict(
        coreset_idx=torch.empty((B, cap), dtype=torch.int32, device=dev),
        coreset_size=torch.empty((B,), dtype=torch.int32, device=dev),
        votes=torch.zeros((B, M), dtype=torch.float32, device=dev),
        k_seq_used=torch.empty((B,), dtype=torch.int32, device=dev),
    )
    _check(lib().des_select_coreset(ctypes.byref(shape), _ptr(logits), _ptr(out["coreset_idx"]),
                                    _ptr(out["coreset_size"]), _ptr(out["votes"]),
                                    _ptr(out["k_seq_used"]), _stream()))
    return out


BUILTIN_WORKSPACE_BYTES = 8 << 20   # DES_BUILTIN_WORKSPACE_BYTES of des.h


class MoeBuffers:
    """Outputs and workspace of des_moe_forward, allocated once per shape.
    with_workspace=False: outputs only (des_moe_forward_builtin_ws)."""

    def __init__(self, shape: DesShape, device, out_dtype: torch.dtype, with_workspace: bool = True):
        B, N, D, M, K = shape.n_seqs, shape.n_tokens, shape.hidden, shape.n_experts, shape.top_k
        cap = des_coreset_capacity(shape)
        nbytes = des_workspace_bytes(shape)
        if nbytes == 0:
            raise DesError(-2, "invalid shape")
        i32, f32 = torch.int32, torch.float32
        self.y = torch.empty((B, N, D), dtype=out_dtype, device=device)
        self.logits = torch.empty((B, N, M), dtype=f32, device=device)
        self.topk_idx = torch.empty((B, N, K), dtype=i32, device=device)
        self.topk_w = torch.empty((B, N, K), dtype=f32, device=device)
        self.expert_counts = torch.empty((M,), dtype=i32, device=device)
        self.n_unique = torch.empty((1,), dtype=i32, device=device)
        self.coreset_idx = torch.empty((B, cap), dtype=i32, device=device)
        self.coreset_size = torch.empty((B,), dtype=i32, device=device)
        self.workspace = (torch.empty((nbytes,), dtype=torch.uint8, device=device)
                          if with_workspace else None)


def des_moe_forward_builtin_ws(shape: DesShape, x, w_router, router_bias, w_gate, w_up, w_down,
                               shared: Optional[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]] = None,
                               buffers: Optional[MoeBuffers] = None) -> MoeBuffers:
    """des_moe_forward with the library's built-in scratch: the call itself allocates
    nothing when `buffers` (the outputs) is given."""
    b = buffers if buffers is not None else MoeBuffers(shape, x.device, x.dtype, with_workspace=False)
    sg, su, sd = shared if shared is not None else (None, None, None)
    _check(lib().des_moe_forward_builtin_ws(
        ctypes.byref(shape), _ptr(x), _ptr(w_router), _ptr(router_bias), _ptr(w_gate), _ptr(w_up),
        _ptr(w_down), _ptr(sg), _ptr(su), _ptr(sd), _ptr(b.y), _ptr(b.logits), _ptr(b.topk_idx),
        _ptr(b.topk_w), _ptr(b.expert_counts), _ptr(b.n_unique), _ptr(b.coreset_idx),
        _ptr(b.coreset_size), _stream()))
    return b


def des_moe_forward(shape: DesShape, x, w_router, router_bias, w_gate, w_up, w_down,
                    shared: Optional[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]] = None,
                    buffers: Optional[MoeBuffers] = None) -> MoeBuffers:
    b = buffers if buffers is not None else MoeBuffers(shape, x.device, x.dtype)
    sg, su, sd = shared if shared is not None else (None, None, None)
    _check(lib().des_moe_forward(
        ctypes.byref(shape), _ptr(x), _ptr(w_router), _ptr(router_bias), _ptr(w_gate), _ptr(w_up),
        _ptr(w_down), _ptr(sg), _ptr(su), _ptr(sd), _ptr(b.y), _ptr(b.logits), _ptr(b.topk_idx),
        _ptr(b.topk_w), _ptr(b.expert_counts), _ptr(b.n_unique), _ptr(b.coreset_idx),
        _ptr(b.coreset_size), _ptr(b.workspace), ctypes.c_size_t(b.workspace.numel()), _stream()))
    return b


class StackBuffers:
    def __init__(self, shape: DesShape, n_layers: int, device, out_dtype: torch.dtype):
        B, N, D, M = shape.n_seqs, shape.n_tokens, shape.hidden, shape.n_experts
        nbytes = des_stack_workspace_bytes(shape)
        if nbytes == 0:
            raise DesError(-2, "invalid shape")
        self.y = torch.empty((B, N, D), dtype=out_dtype, device=device)
        self.expert_counts = torch.empty((n_layers, M), dtype=torch.int32, device=device)
        self.n_unique = torch.empty((n_layers,), dtype=torch.int32, device=device)
        self.workspace = torch.empty((nbytes,), dtype=torch.uint8, device=device)


def des_moe_stack_forward(shape: DesShape, n_layers: int, x, w_router, router_bias, w_gate, w_up,
                          w_down, shared=None, buffers: Optional[StackBuffers] = None
                          ) -> StackBuffers:
    b = buffers if buffers is not None else StackBuffers(shape, n_layers, x.device, x.dtype)
    sg, su, sd = shared if shared is not None else (None, None, None)
    _check(lib().des_moe_stack_forward(
        ctypes.byref(shape), n_layers, _ptr(x), _ptr(w_router), _ptr(router_bias), _ptr(w_gate),
        _ptr(w_up), _ptr(w_down), _ptr(sg), _ptr(su), _ptr(sd), _ptr(b.y), _ptr(b.expert_counts),
        _ptr(b.n_unique), _ptr(b.workspace), ctypes.c_size_t(b.workspace.numel()), _stream()))
    return b


def make_attn_shape(n_heads: int, n_kv_heads: int, head_dim: int, n_prefix: int = 0,
                    n_suffix: int = 0) -> DesAttnShape:
    return DesAttnShape(n_heads, n_kv_heads, head_dim, n_prefix, n_suffix)


def des_attention_workspace_bytes(shape: DesShape, attn: DesAttnShape) -> int:
    return int(lib().des_attention_workspace_bytes(ctypes.byref(shape), ctypes.byref(attn)))


def des_decoder_workspace_bytes(shape: DesShape, attn: DesAttnShape) -> int:
    return int(lib().des_decoder_workspace_bytes(ctypes.byref(shape), ctypes.byref(attn)))


def _workspace(nbytes: int, device) -> torch.Tensor:
    if nbytes == 0:
        raise DesError(-2, "shape rejected by the library (workspace size 0)")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def des_block_attention(shape: DesShape, attn: DesAttnShape, x, wq, wk, wv, wo, k_cache=None,
                        v_cache=None, y: Optional[torch.Tensor] = None,
                        workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """The attention sub-layer of one block-parallel decoding step; returns y [B, N, D]."""
    if y is None:
        y = torch.empty_like(x)
    if workspace is None:
        workspace = _workspace(des_attention_workspace_bytes(shape, attn), x.device)
    _check(lib().des_block_attention(
        ctypes.byref(shape), ctypes.byref(attn), _ptr(x), _ptr(wq), _ptr(wk), _ptr(wv), _ptr(wo),
        _ptr(k_cache), _ptr(v_cache), _ptr(y), _ptr(workspace), ctypes.c_size_t(workspace.numel()),
        _stream()))
    return y


class DecoderBuffers:
    """Outputs and scratch of des_decoder_stack_forward."""

    def __init__(self, shape: DesShape, attn: DesAttnShape, n_layers: int, device, dtype):
        B, N, M = shape.n_seqs, shape.n_tokens, shape.n_experts
        i32 = torch.int32
        self.y = torch.empty((B, N, shape.hidden), dtype=dtype, device=device)
        self.expert_counts = torch.empty((n_layers, M), dtype=i32, device=device)
        self.n_unique = torch.empty((n_layers,), dtype=i32, device=device)
        self.workspace = _workspace(des_decoder_workspace_bytes(shape, attn), device)


def des_decoder_stack_forward(shape: DesShape, attn: DesAttnShape, n_layers: int, x, wq, wk, wv, wo,
                              k_cache, v_cache, w_router, router_bias, w_gate, w_up, w_down,
                              shared=None, buffers: Optional[DecoderBuffers] = None) -> DecoderBuffers:
    b = buffers if buffers is not None else DecoderBuffers(shape, attn, n_layers, x.device, x.dtype)
    sg, su, sd = shared if shared is not None else (None, None, None)
    _check(lib().des_decoder_stack_forward(
        ctypes.byref(shape), ctypes.byref(attn), n_layers, _ptr(x), _ptr(wq), _ptr(wk), _ptr(wv),
        _ptr(wo), _ptr(k_cache), _ptr(v_cache), _ptr(w_router), _ptr(router_bias), _ptr(w_gate),
        _ptr(w_up), _ptr(w_down), _ptr(sg), _ptr(su), _ptr(sd), _ptr(b.y), _ptr(b.expert_counts),
        _ptr(b.n_unique), _ptr(b.workspace), ctypes.c_size_t(b.workspace.numel()), _stream()))
    return b


def des_pack_expert_weights(src: torch.Tensor) -> torch.Tensor:
    """src: [..., rows, cols] bf16 row-major -> same shape, tiled layout."""
    rows, cols = src.shape[-2], src.shape[-1]
    n_mats = src.numel() // (rows * cols)
    dst = torch.empty_like(src)
    _check(lib().des_pack_expert_weights(_ptr(src), _ptr(dst), n_mats, rows, cols, _stream()))
    return dst


def des_hbm_read_probe(src: torch.Tensor, n_bytes: int, sink: torch.Tensor) -> None:
    """One bare streaming read of the first n_bytes of src (a multiple of 64 KiB)."""
    if n_bytes > src.numel() * src.element_size() or sink.numel() * sink.element_size() < 16:
        raise ValueError("read probe: n_bytes exceeds src, or sink smaller than 16 bytes")
    _check(lib().des_hbm_read_probe(_ptr(src), n_bytes, _ptr(sink), _stream()))


def des_coreset_from_beta(beta: float, n_experts: int) -> int:
    """floor(beta * M): the coreset size for a budget given as a fraction (Table 1)."""
    return int(lib().des_coreset_from_beta(float(beta), int(n_experts)))


def des_test_hooks(skip_router, max_wait_iters: int) -> None:
    """Test aid: forces the give-up path of the bounded waits ((0, 0) = normal;
    skip_router = 2: for the next fused routing launch only)."""
    _check(lib().des_test_hooks(int(skip_router), int(max_wait_iters)))


def des_kernel_timing_enable(enable: bool) -> None:
    _check(lib().des_kernel_timing_enable(1 if enable else 0))


def des_kernel_timing_read() -> Dict[str, Tuple[float, int]]:
    """{kernel name: (total ms, launches)} accumulated since timing was enabled."""
    out = {}
    for k in range(lib().des_kernel_timing_count()):
        ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
        _check(lib().des_kernel_timing_read(k, ctypes.byref(ms), ctypes.byref(n)))
        out[lib().des_kernel_timing_name(k).decode()] = (ms.value, n.value)
    return out
