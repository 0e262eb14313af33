"""Python binding of libconfu_verify.so (MI355X / gfx950 tree-verification library).

Argument marshalling only: every step of the path runs in the library's HIP kernels.
PyTorch is used for device memory and streams.  There is no CPU fallback: if the
shared library has not been built, importing the entry points raises.

    from paper_2603_08899_amd import tree_verify_attention, tree_accept
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libconfu_verify.so")

TV_OK, TV_ERR_INVALID_ARG, TV_ERR_WORKSPACE, TV_ERR_LAUNCH, TV_ERR_UNSUPPORTED = 0, 1, 2, 3, 4
TV_STATUS_BAD_PARENT, TV_STATUS_BAD_KIND, TV_STATUS_BAD_PREFIX, TV_STATUS_BAD_TOKEN = 1, 2, 4, 8
TV_STATUS_INTERNAL = 16
TV_STATUS_BAD_PATH = 32
TV_MAX_ROWS = 128
TV_PREPARED_TREE_BYTES = 2304
TV_DTYPE_F32, TV_DTYPE_BF16 = 0, 1
TV_KIND_NODE, TV_KIND_CONTEMPLATE = 0, 1
TV_RULE_GREEDY, TV_RULE_DETERMINISTIC, TV_RULE_DRAFT_WOR, TV_RULE_DRAFT_WR, TV_RULE_SAMPLE_MATCH = 0, 1, 2, 3, 4
TV_FINAL_BONUS, TV_FINAL_RESIDUAL = 0, 1

EXPORTED_SYMBOLS = (
    "tv_attention_workspace_bytes", "tv_attention_plan", "tv_prepare_tree", "tree_verify_attention",
    "tree_verify_attention_noalloc",
    "tv_accept_workspace_bytes", "tree_accept",
    "tree_commit", "contemplate_embed", "tv_embed_workspace_bytes",
    "tv_build_mask_host", "tv_error_string", "tv_version", "tv_set_wait_limit",
)


class tv_attn_desc(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32), ("dtype", ctypes.c_int32),
        ("B", ctypes.c_int32), ("M", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
        ("D", ctypes.c_int32), ("soft_len", ctypes.c_int32), ("max_prefix_len", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float),
        ("kv_token_stride", ctypes.c_int64), ("kv_head_stride", ctypes.c_int64),
        ("num_splits", ctypes.c_int32), ("wg_row_blocks", ctypes.c_int32), ("sum_prefix_len", ctypes.c_int64),
    ]


class tv_accept_desc(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32), ("B", ctypes.c_int32), ("T", ctypes.c_int32),
        ("V", ctypes.c_int32), ("C", ctypes.c_int32), ("rule", ctypes.c_int32),
        ("temperature", ctypes.c_float), ("logits_row_stride", ctypes.c_int64),
        ("logits_dtype", ctypes.c_int32), ("reserved", ctypes.c_int32),
    ]


class tv_commit_desc(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32), ("dtype", ctypes.c_int32), ("B", ctypes.c_int32), ("T", ctypes.c_int32),
        ("M", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("D", ctypes.c_int32), ("n_layers", ctypes.c_int32),
        ("kv_layer_stride", ctypes.c_int64), ("kv_token_stride", ctypes.c_int64), ("kv_head_stride", ctypes.c_int64),
        ("C", ctypes.c_int32), ("d_model", ctypes.c_int32),
    ]


class tv_embed_desc(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32), ("dtype", ctypes.c_int32), ("B", ctypes.c_int32), ("d_in", ctypes.c_int32),
        ("d_out", ctypes.c_int32), ("n_expert", ctypes.c_int32), ("k_expert", ctypes.c_int32),
        ("reserved", ctypes.c_int32),
    ]


class ConfuVerifyError(RuntimeError):
    def __init__(self, code: int, where: str):
        msg = lib().tv_error_string(code).decode() if _lib is not None else str(code)
        super().__init__(f"{where}: {msg} (code {code})")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """Loads the shared library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2603_08899_amd.build` "
                "(hipcc, gfx950). There is no CPU fallback.")
        # PyTorch ships its own copy of the HIP runtime.  If this library were loaded first it would bring in the
        # system's copy, and the process would then hold two: a device initialised through one is not visible to
        # the other ("No HIP GPUs are available" from torch after a host-only call such as tv_attention_plan).
        # Importing torch first makes both use the one torch loads.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        l = ctypes.CDLL(LIB_PATH)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        l.tv_version.restype = ctypes.c_int
        l.tv_set_wait_limit.restype = ctypes.c_int
        l.tv_set_wait_limit.argtypes = [ctypes.c_int]
        l.tv_error_string.restype = ctypes.c_char_p
        l.tv_error_string.argtypes = [ctypes.c_int]
        l.tv_build_mask_host.restype = ctypes.c_int
        l.tv_build_mask_host.argtypes = [vp, vp, ctypes.c_int, vp]
        l.tv_attention_workspace_bytes.restype = ctypes.c_int
        l.tv_attention_workspace_bytes.argtypes = [ctypes.POINTER(tv_attn_desc), ctypes.POINTER(sz)]
        l.tv_attention_plan.restype = ctypes.c_int
        l.tv_attention_plan.argtypes = [ctypes.POINTER(tv_attn_desc), ctypes.POINTER(ctypes.c_int32),
                                        ctypes.POINTER(ctypes.c_int32)]
        l.tree_verify_attention.restype = ctypes.c_int
        l.tree_verify_attention.argtypes = [ctypes.POINTER(tv_attn_desc)] + [vp] * 12 + [sz, vp]
        l.tree_verify_attention_noalloc.restype = ctypes.c_int
        l.tree_verify_attention_noalloc.argtypes = [ctypes.POINTER(tv_attn_desc)] + [vp] * 12
        l.tv_prepare_tree.restype = ctypes.c_int
        l.tv_prepare_tree.argtypes = [ctypes.c_int32, ctypes.c_int32, vp, vp, vp, sz, vp]
        l.tv_accept_workspace_bytes.restype = ctypes.c_int
        l.tv_accept_workspace_bytes.argtypes = [ctypes.POINTER(tv_accept_desc), ctypes.POINTER(sz)]
        l.tree_accept.restype = ctypes.c_int
        l.tree_accept.argtypes = [ctypes.POINTER(tv_accept_desc)] + [vp] * 14 + [sz, vp]
        l.tree_commit.restype = ctypes.c_int
        l.tree_commit.argtypes = [ctypes.POINTER(tv_commit_desc)] + [vp] * 14
        l.contemplate_embed.restype = ctypes.c_int
        l.contemplate_embed.argtypes = [ctypes.POINTER(tv_embed_desc)] + [vp] * 7 + [sz, vp]
        l.tv_embed_workspace_bytes.restype = ctypes.c_int
        l.tv_embed_workspace_bytes.argtypes = [ctypes.POINTER(tv_embed_desc), ctypes.POINTER(sz)]
        _lib = l
    return _lib


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream_handle(stream) -> Optional[int]:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream or None


def make_attn_desc(*, dtype: int, B: int, M: int, Hq: int, Hkv: int, D: int, soft_len: int,
                   max_prefix_len: int, softmax_scale: float, kv_token_stride: int = 0,
                   kv_head_stride: int = 0, num_splits: int = 0, wg_row_blocks: int = 0,
                   sum_prefix_len: int = 0) -> tv_attn_desc:
    return tv_attn_desc(ctypes.sizeof(tv_attn_desc), dtype, B, M, Hq, Hkv, D, soft_len, max_prefix_len,
                        softmax_scale, kv_token_stride, kv_head_stride, num_splits, wg_row_blocks, sum_prefix_len)


def make_accept_desc(*, B: int, T: int, V: int, C: int, rule: int, temperature: float,
                     logits_row_stride: int = 0, logits_dtype: int = 0) -> tv_accept_desc:
    return tv_accept_desc(ctypes.sizeof(tv_accept_desc), B, T, V, C, rule, temperature, logits_row_stride,
                          logits_dtype, 0)


def tv_attention_workspace_bytes(desc: tv_attn_desc) -> int:
    n = ctypes.c_size_t(0)
    rc = lib().tv_attention_workspace_bytes(ctypes.byref(desc), ctypes.byref(n))
    if rc:
        raise ConfuVerifyError(rc, "tv_attention_workspace_bytes")
    return int(n.value)


def tv_attention_plan(desc: tv_attn_desc):
    """(64-row blocks per workgroup, key ranges) the library would launch *desc with."""
    rb, n = ctypes.c_int32(0), ctypes.c_int32(0)
    rc = lib().tv_attention_plan(ctypes.byref(desc), ctypes.byref(rb), ctypes.byref(n))
    if rc:
        raise ConfuVerifyError(rc, "tv_attention_plan")
    return int(rb.value), int(n.value)


def tv_accept_workspace_bytes(desc: tv_accept_desc) -> int:
    n = ctypes.c_size_t(0)
    rc = lib().tv_accept_workspace_bytes(ctypes.byref(desc), ctypes.byref(n))
    if rc:
        raise ConfuVerifyError(rc, "tv_accept_workspace_bytes")
    return int(n.value)


def tv_set_wait_limit(polls: int) -> int:
    """Test hook: looks at another workgroup's slot before a sibling-chain workgroup computes that share itself
    (0 = default); returns the old value."""
    return int(lib().tv_set_wait_limit(int(polls)))


def tv_build_mask_host(parent, kind):
    """numpy int32[M], uint8[M] -> uint64[M, 2] ancestor bit mask (raises on a malformed tree)."""
    import numpy as np
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    kind = np.ascontiguousarray(kind, dtype=np.uint8)
    bits = np.zeros((len(parent), 2), dtype=np.uint64)
    rc = lib().tv_build_mask_host(parent.ctypes.data, kind.ctypes.data, len(parent), bits.ctypes.data)
    if rc:
        raise ConfuVerifyError(rc, "tv_build_mask_host")
    return bits


def tv_prepare_tree(parent, kind, prepared, stream=None) -> None:
    """parent int32 [B, M], kind uint8 [B, M], prepared uint8 [>= B * TV_PREPARED_TREE_BYTES] (torch CUDA tensors):
    checks the trees and writes their ancestor masks once for all layers of a verification step."""
    B, M = parent.shape
    rc = lib().tv_prepare_tree(int(B), int(M), _ptr(parent), _ptr(kind), _ptr(prepared),
                               prepared.numel() * prepared.element_size(), _stream_handle(stream))
    if rc:
        raise ConfuVerifyError(rc, "tv_prepare_tree")


def tree_verify_attention(desc: tv_attn_desc, q, k_pool, v_pool, kv_offset, prefix_len, parent, kind,
                          out, lse, status, workspace, stream=None, prepared_tree=None) -> None:
    """All tensor arguments are torch CUDA tensors (lse / workspace / prepared_tree may be None); see
    include/confu_verify.h for shapes.  Enqueues on `stream` (default: torch's current stream)."""
    rc = lib().tree_verify_attention(
        ctypes.byref(desc), _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(kv_offset), _ptr(prefix_len),
        _ptr(parent), _ptr(kind), _ptr(prepared_tree), _ptr(out), _ptr(lse), _ptr(status), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if rc:
        raise ConfuVerifyError(rc, "tree_verify_attention")


TV_NOALLOC_SCRATCH_BYTES = 16 << 20


def tree_verify_attention_noalloc(desc: tv_attn_desc, q, k_pool, v_pool, kv_offset, prefix_len, parent, kind,
                                  out, lse, status, stream=None, prepared_tree=None) -> None:
    """tree_verify_attention without a workspace: partial results live in a fixed array inside the library."""
    rc = lib().tree_verify_attention_noalloc(
        ctypes.byref(desc), _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(kv_offset), _ptr(prefix_len),
        _ptr(parent), _ptr(kind), _ptr(prepared_tree), _ptr(out), _ptr(lse), _ptr(status), _stream_handle(stream))
    if rc:
        raise ConfuVerifyError(rc, "tree_verify_attention_noalloc")


def tree_accept(desc: tv_accept_desc, target_logits, draft_logits, token, parent, uniforms, con_anchor,
                path, n_accepted, final_token, final_kind, last_node, selected_con, status, workspace,
                stream=None) -> None:
    rc = lib().tree_accept(
        ctypes.byref(desc), _ptr(target_logits), _ptr(draft_logits), _ptr(token), _ptr(parent),
        _ptr(uniforms), _ptr(con_anchor), _ptr(path), _ptr(n_accepted), _ptr(final_token),
        _ptr(final_kind), _ptr(last_node), _ptr(selected_con), _ptr(status), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if rc:
        raise ConfuVerifyError(rc, "tree_accept")


def make_commit_desc(*, dtype: int, B: int, T: int, M: int, Hkv: int, D: int, n_layers: int, kv_layer_stride: int = 0,
                     kv_token_stride: int = 0, kv_head_stride: int = 0, C: int = 0, d_model: int = 0) -> tv_commit_desc:
    return tv_commit_desc(ctypes.sizeof(tv_commit_desc), dtype, B, T, M, Hkv, D, n_layers, kv_layer_stride,
                          kv_token_stride, kv_head_stride, C, d_model)


def tree_commit(desc: tv_commit_desc, k_pool, v_pool, kv_offset, prefix_len, path, n_accepted, node_row, hidden,
                con_row, selected_con, f_out, new_prefix_len, status, stream=None) -> None:
    """Moves the accepted path's K/V rows to the front of this step's rows in every layer (in place) and, when
    `hidden` is given, gathers the future prediction of the last accepted token; see include/confu_verify.h."""
    rc = lib().tree_commit(
        ctypes.byref(desc), _ptr(k_pool), _ptr(v_pool), _ptr(kv_offset), _ptr(prefix_len), _ptr(path),
        _ptr(n_accepted), _ptr(node_row), _ptr(hidden), _ptr(con_row), _ptr(selected_con), _ptr(f_out),
        _ptr(new_prefix_len), _ptr(status), _stream_handle(stream))
    if rc:
        raise ConfuVerifyError(rc, "tree_commit")


def make_embed_desc(*, dtype: int, B: int, d_in: int, d_out: int, n_expert: int, k_expert: int) -> tv_embed_desc:
    return tv_embed_desc(ctypes.sizeof(tv_embed_desc), dtype, B, d_in, d_out, n_expert, k_expert, 0)


def tv_embed_workspace_bytes(desc: tv_embed_desc) -> int:
    n = ctypes.c_size_t(0)
    rc = lib().tv_embed_workspace_bytes(ctypes.byref(desc), ctypes.byref(n))
    if rc:
        raise ConfuVerifyError(rc, "tv_embed_workspace_bytes")
    return int(n.value)


def contemplate_embed(desc: tv_embed_desc, h, router_w, expert_emb, out, gates, chosen, workspace, stream=None) -> None:
    """Mixture-of-experts embedding of contemplate / future tokens; see include/confu_verify.h."""
    rc = lib().contemplate_embed(ctypes.byref(desc), _ptr(h), _ptr(router_w), _ptr(expert_emb), _ptr(out),
                                 _ptr(gates), _ptr(chosen), _ptr(workspace),
                                 0 if workspace is None else workspace.numel() * workspace.element_size(),
                                 _stream_handle(stream))
    if rc:
        raise ConfuVerifyError(rc, "contemplate_embed")
