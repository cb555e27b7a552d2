"""ctypes binding of libfspad.so: argument marshalling only.

Every step of the verification path runs in the HIP kernels behind the C ABI
(include/fspad.h); PyTorch is used here for device memory and the current HIP
stream, nothing else.  There is no CPU or PyTorch fallback: if the library has
not been built, every call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np
import torch

from .build import LIB_PATH

FSPAD_OK = 0
FSPAD_F32, FSPAD_BF16 = 0, 1
FSPAD_MAX_NODES = 64

_STATUS_NAMES = {0: "FSPAD_OK", 1: "FSPAD_ERR_NULL", 2: "FSPAD_ERR_SHAPE", 3: "FSPAD_ERR_TREE",
                 4: "FSPAD_ERR_DTYPE", 5: "FSPAD_ERR_WORKSPACE", 6: "FSPAD_ERR_TEMPERATURE", 7: "FSPAD_ERR_HIP"}

EXPORTS = ("fspad_tree_attn_workspace_bytes", "fspad_tree_attn",
           "fspad_tree_accept_workspace_bytes", "fspad_tree_accept_greedy", "fspad_tree_accept_greedy_static",
           "fspad_tree_accept_sample",
           "fspad_tree_accept_sample_draft_workspace_bytes", "fspad_tree_accept_sample_draft",
           "fspad_tree_accept_lm_head_workspace_bytes", "fspad_tree_accept_greedy_lm_head",
           "fspad_tree_accept_sample_lm_head",
           "fspad_kv_commit", "fspad_feature_sampler_workspace_bytes", "fspad_feature_sampler",
           "fspad_draft_layer_workspace_bytes", "fspad_draft_layer", "fspad_packed_weight_bytes", "fspad_pack_weight",
           "fspad_draft_topk_workspace_bytes", "fspad_draft_topk", "fspad_tree_build", "fspad_tree_build_mask",
           "fspad_tree_validate", "fspad_status_string")


class FspadError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib().fspad_status_string(status).decode() if _LIB is not None else ""
        super().__init__(f"{where}: {_STATUS_NAMES.get(status, status)} ({msg})")


class fspad_attn_desc(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_nodes_max", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("io_dtype", ctypes.c_int32),
                ("out_dtype", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
                ("cache_stride_batch", ctypes.c_int64), ("cache_stride_head", ctypes.c_int64),
                ("cache_stride_token", ctypes.c_int64), ("workgroups", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class fspad_draft_layer_desc(ctypes.Structure):
    _fields_ = [("attn", fspad_attn_desc), ("hidden_dim", ctypes.c_int32), ("intermediate_dim", ctypes.c_int32),
                ("rms_eps", ctypes.c_float), ("rope_theta", ctypes.c_float), ("weights_packed", ctypes.c_int32)]


class fspad_draft_layer_weights(ctypes.Structure):
    _fields_ = [(name, ctypes.c_void_p) for name in
                ("w_qkv", "w_o", "w_gate", "w_up", "w_down", "gain_attn", "gain_mlp")]


_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it first (python -m paper_2408_15562_amd.build, or "
                "__graft_entry__.build()). There is no fallback path.")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        lib.fspad_status_string.restype = ctypes.c_char_p
        lib.fspad_status_string.argtypes = [ctypes.c_int]
        lib.fspad_tree_attn_workspace_bytes.restype = sz
        lib.fspad_tree_attn_workspace_bytes.argtypes = [ctypes.POINTER(fspad_attn_desc), i32]
        lib.fspad_tree_attn.restype = ctypes.c_int
        lib.fspad_tree_attn.argtypes = [ctypes.POINTER(fspad_attn_desc)] + [vp] * 9 + [vp, sz, vp]
        lib.fspad_tree_accept_workspace_bytes.restype = sz
        lib.fspad_tree_accept_workspace_bytes.argtypes = [i32, i32, i32]
        lib.fspad_tree_accept_greedy.restype = ctypes.c_int
        lib.fspad_tree_accept_greedy.argtypes = [i32, i32, i32, vp, i64, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.fspad_tree_accept_greedy_static.restype = ctypes.c_int
        lib.fspad_tree_accept_greedy_static.argtypes = [i32, i32, i32, vp, i64, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.fspad_tree_accept_sample.restype = ctypes.c_int
        lib.fspad_tree_accept_sample.argtypes = [i32, i32, i32, vp, i64, vp, vp, vp, ctypes.c_float, vp,
                                                 vp, vp, vp, vp, vp, sz, vp]
        lib.fspad_tree_accept_sample_draft_workspace_bytes.restype = sz
        lib.fspad_tree_accept_sample_draft_workspace_bytes.argtypes = [i32, i32, i32]
        lib.fspad_tree_accept_sample_draft.restype = ctypes.c_int
        lib.fspad_tree_accept_sample_draft.argtypes = [i32, i32, i32, vp, vp, i64, vp, vp, vp, ctypes.c_float, vp,
                                                       vp, vp, vp, vp, vp, sz, vp]
        lib.fspad_tree_accept_lm_head_workspace_bytes.restype = sz
        lib.fspad_tree_accept_lm_head_workspace_bytes.argtypes = [i32, i32, i32]
        lib.fspad_tree_accept_greedy_lm_head.restype = ctypes.c_int
        lib.fspad_tree_accept_greedy_lm_head.argtypes = [i32, i32, i32, i32, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                                         vp, sz, vp]
        lib.fspad_tree_accept_sample_lm_head.restype = ctypes.c_int
        lib.fspad_tree_accept_sample_lm_head.argtypes = [i32, i32, i32, i32, vp, vp, i32, vp, vp, vp, ctypes.c_float, vp,
                                                         vp, vp, vp, vp, vp, sz, vp]
        lib.fspad_kv_commit.restype = ctypes.c_int
        lib.fspad_kv_commit.argtypes = [ctypes.POINTER(fspad_attn_desc), vp, vp, vp, vp, i32, vp, vp, vp, vp, vp]
        lib.fspad_feature_sampler_workspace_bytes.restype = sz
        lib.fspad_feature_sampler_workspace_bytes.argtypes = [i32, i32, i32]
        lib.fspad_feature_sampler.restype = ctypes.c_int
        lib.fspad_feature_sampler.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, i32, vp, vp, sz, vp]
        lib.fspad_packed_weight_bytes.restype = sz
        lib.fspad_packed_weight_bytes.argtypes = [i32, i32]
        lib.fspad_pack_weight.restype = ctypes.c_int
        lib.fspad_pack_weight.argtypes = [i32, i32, vp, vp, vp]
        lib.fspad_draft_layer_workspace_bytes.restype = sz
        lib.fspad_draft_layer_workspace_bytes.argtypes = [ctypes.POINTER(fspad_draft_layer_desc), i32]
        lib.fspad_draft_layer.restype = ctypes.c_int
        lib.fspad_draft_layer.argtypes = [ctypes.POINTER(fspad_draft_layer_desc),
                                          ctypes.POINTER(fspad_draft_layer_weights)] + [vp] * 11 + [vp, sz, vp]
        lib.fspad_draft_topk_workspace_bytes.restype = sz
        lib.fspad_draft_topk_workspace_bytes.argtypes = [i32, i32, i32]
        lib.fspad_draft_topk.restype = ctypes.c_int
        lib.fspad_draft_topk.argtypes = [i32, i32, i32, vp, i64, vp, vp, vp, sz, vp]
        lib.fspad_tree_build.restype = ctypes.c_int
        lib.fspad_tree_build.argtypes = [i32, i32, i32, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp]
        lib.fspad_tree_build_mask.restype = ctypes.c_int
        lib.fspad_tree_build_mask.argtypes = [i32, i32, vp, vp, vp]
        lib.fspad_tree_validate.restype = ctypes.c_int
        lib.fspad_tree_validate.argtypes = [i32, i32, i32, vp, vp, vp]
        _LIB = lib
    return _LIB


def library_path() -> str:
    _lib()
    return LIB_PATH


def _check(status: int, where: str):
    if status != FSPAD_OK:
        raise FspadError(status, where)


class PreparedCall:
    """One library call with its arguments already marshalled: calling it issues exactly that call
    again (same buffers, same stream). For loops that repeat a call, so that Python's argument
    checks are paid once. Holds references to every tensor and host array it points into."""

    __slots__ = ("_fn", "_where", "_args", "_keep", "result")

    def __init__(self, fn, where, args, keep, result):
        self._fn, self._where, self._args, self._keep, self.result = fn, where, args, keep, result

    def __call__(self):
        st = self._fn(*self._args)
        if st != FSPAD_OK:
            raise FspadError(st, self._where)
        return self.result


def _issue(fn, where, args, keep, result, prepare):
    call = PreparedCall(fn, where, args, keep, result)
    return call if prepare else call()


def _dev_ptr(t: Optional[torch.Tensor], name: str, dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _host_i32(a, name: str) -> np.ndarray:
    if isinstance(a, torch.Tensor):
        if a.is_cuda:
            raise ValueError(f"{name} must live on the host")
        a = a.numpy()
    return np.ascontiguousarray(a, dtype=np.int32)


def _stream_ptr(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dtype_code(dt: torch.dtype) -> int:
    if dt == torch.float32:
        return FSPAD_F32
    if dt == torch.bfloat16:
        return FSPAD_BF16
    raise FspadError(4, f"dtype {dt}")


def make_attn_desc(q: torch.Tensor, k_tree: torch.Tensor, k_cache: Optional[torch.Tensor],
                   out_dtype: Optional[torch.dtype] = None, softmax_scale: float = 0.0,
                   workgroups: int = 0) -> fspad_attn_desc:
    """Fill the descriptor from tensor shapes; cache strides are taken from k_cache."""
    B, Nmax, Hq, D = q.shape
    Hkv = k_tree.shape[2]
    d = fspad_attn_desc()
    d.batch, d.n_nodes_max, d.n_q_heads, d.n_kv_heads, d.head_dim = B, Nmax, Hq, Hkv, D
    d.io_dtype = _dtype_code(q.dtype)
    d.out_dtype = _dtype_code(out_dtype if out_dtype is not None else q.dtype)
    d.softmax_scale = float(softmax_scale)
    d.workgroups = int(workgroups)
    if k_cache is not None:
        if k_cache.stride(3) != 1:
            raise ValueError("head_dim must be contiguous in the cache")
        d.cache_stride_batch, d.cache_stride_head, d.cache_stride_token = (
            k_cache.stride(0), k_cache.stride(1), k_cache.stride(2))
    else:
        d.cache_stride_batch = d.cache_stride_head = 0
        d.cache_stride_token = D
    return d


def fspad_tree_attn_workspace_bytes(desc: fspad_attn_desc, max_kv_len: int) -> int:
    return int(_lib().fspad_tree_attn_workspace_bytes(ctypes.byref(desc), int(max_kv_len)))


def fspad_tree_attn(q: torch.Tensor, k_tree: torch.Tensor, v_tree: torch.Tensor,
                    k_cache: Optional[torch.Tensor], v_cache: Optional[torch.Tensor],
                    kv_len, n_nodes, anc_mask: torch.Tensor, out: Optional[torch.Tensor] = None,
                    workspace: Optional[torch.Tensor] = None, softmax_scale: float = 0.0,
                    out_dtype: Optional[torch.dtype] = None, stream=None,
                    desc: Optional[fspad_attn_desc] = None, prepare: bool = False, workgroups: int = 0):
    """q [B,Nmax,Hq,D]; k_tree,v_tree [B,Nmax,Hkv,D]; k_cache,v_cache [B,Hkv,Lcap,D] views (any
    batch/head/token strides); kv_len,n_nodes HOST int32 [B]; anc_mask device int64/uint64 [B,Nmax];
    workgroups: the descriptor's tuning field (0 = built-in choice), used when no desc is given.
    Returns out [B,Nmax,Hq,D]; with prepare=True a PreparedCall that issues the call each time it is called."""
    for name, t in (("q", q), ("k_tree", k_tree), ("v_tree", v_tree)):
        if not t.is_contiguous():
            raise ValueError(f"{name} must be contiguous")
    if k_cache is not None and (v_cache is None or v_cache.stride() != k_cache.stride()
                                or v_cache.dtype != q.dtype or k_cache.dtype != q.dtype):
        raise ValueError("k_cache and v_cache must share strides and the dtype of q")
    if desc is None:
        desc = make_attn_desc(q, k_tree, k_cache, out_dtype if out_dtype is not None else
                              (out.dtype if out is not None else None), softmax_scale, workgroups)
    kv_len = _host_i32(kv_len, "kv_len")
    n_nodes = _host_i32(n_nodes, "n_nodes")
    if kv_len.shape != (desc.batch,) or n_nodes.shape != (desc.batch,):
        raise ValueError("kv_len and n_nodes must have one entry per sequence")
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32 if desc.out_dtype == FSPAD_F32 else torch.bfloat16,
                          device=q.device)
    if anc_mask.dtype not in (torch.int64, torch.uint64) or not anc_mask.is_contiguous():
        raise ValueError("anc_mask must be a contiguous 64-bit integer tensor")
    if workspace is None:
        need = fspad_tree_attn_workspace_bytes(desc, int(kv_len.max(initial=0)))
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    args = (ctypes.byref(desc), _dev_ptr(q, "q"), _dev_ptr(k_tree, "k_tree"), _dev_ptr(v_tree, "v_tree"),
            _dev_ptr(k_cache, "k_cache"), _dev_ptr(v_cache, "v_cache"),
            kv_len.ctypes.data, n_nodes.ctypes.data, _dev_ptr(anc_mask, "anc_mask"), _dev_ptr(out, "out"),
            _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    keep = (desc, q, k_tree, v_tree, k_cache, v_cache, kv_len, n_nodes, anc_mask, out, workspace)
    return _issue(_lib().fspad_tree_attn, "fspad_tree_attn", args, keep, out, prepare)


def fspad_tree_accept_workspace_bytes(B: int, Nmax: int, V: int) -> int:
    return int(_lib().fspad_tree_accept_workspace_bytes(B, Nmax, V))


def _accept_outputs(B, Nmax, device, outputs):
    if outputs is not None:
        return outputs
    return (torch.empty((B, Nmax), dtype=torch.int32, device=device), torch.empty((B,), dtype=torch.int32, device=device),
            torch.empty((B, Nmax), dtype=torch.int32, device=device), torch.empty((B,), dtype=torch.int32, device=device))


def _accept_common(logits, draft_tokens, parent, n_nodes, workspace):
    if logits.dim() != 3 or logits.stride(2) != 1 or logits.stride(0) != logits.shape[1] * logits.stride(1):
        raise ValueError("logits must be [B,Nmax,V] with a uniform row stride")
    B, Nmax, V = logits.shape
    if workspace is None:
        workspace = torch.empty(fspad_tree_accept_workspace_bytes(B, Nmax, V), dtype=torch.uint8, device=logits.device)
    for name, t in (("draft_tokens", draft_tokens), ("parent", parent), ("n_nodes", n_nodes)):
        if t.dtype != torch.int32 or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous int32 device tensor")
    return B, Nmax, V, workspace


def fspad_tree_accept_greedy(logits: torch.Tensor, draft_tokens: torch.Tensor, parent: torch.Tensor,
                             n_nodes: torch.Tensor, outputs=None, workspace: Optional[torch.Tensor] = None,
                             stream=None, prepare: bool = False):
    """All tensors on the device. Returns (path [B,Nmax], path_len [B], tokens [B,Nmax], n_tokens [B]);
    with prepare=True a PreparedCall."""
    B, Nmax, V, workspace = _accept_common(logits, draft_tokens, parent, n_nodes, workspace)
    path, path_len, tokens, n_tokens = _accept_outputs(B, Nmax, logits.device, outputs)
    args = (B, Nmax, V, _dev_ptr(logits, "logits", torch.float32), logits.stride(1),
            _dev_ptr(draft_tokens, "draft_tokens"), _dev_ptr(parent, "parent"), _dev_ptr(n_nodes, "n_nodes"),
            _dev_ptr(path, "path"), _dev_ptr(path_len, "path_len"), _dev_ptr(tokens, "tokens"),
            _dev_ptr(n_tokens, "n_tokens"), _dev_ptr(workspace, "workspace"),
            workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    keep = (logits, draft_tokens, parent, n_nodes, workspace)
    return _issue(_lib().fspad_tree_accept_greedy, "fspad_tree_accept_greedy", args, keep,
                  (path, path_len, tokens, n_tokens), prepare)


def fspad_tree_accept_greedy_static(logits: torch.Tensor, draft_tokens: torch.Tensor, parent: torch.Tensor,
                                    n_nodes: torch.Tensor, outputs, stream=None, prepare: bool = False):
    """fspad_tree_accept_greedy without a workspace (the library's own fixed device array holds the
    chunk statistics) and without any allocation here either: the four output tensors are required."""
    if logits.dim() != 3 or logits.stride(2) != 1 or logits.stride(0) != logits.shape[1] * logits.stride(1):
        raise ValueError("logits must be [B,Nmax,V] with a uniform row stride")
    B, Nmax, V = logits.shape
    for name, t in (("draft_tokens", draft_tokens), ("parent", parent), ("n_nodes", n_nodes)):
        if t.dtype != torch.int32 or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous int32 device tensor")
    path, path_len, tokens, n_tokens = outputs
    args = (B, Nmax, V, _dev_ptr(logits, "logits", torch.float32), logits.stride(1),
            _dev_ptr(draft_tokens, "draft_tokens"), _dev_ptr(parent, "parent"), _dev_ptr(n_nodes, "n_nodes"),
            _dev_ptr(path, "path"), _dev_ptr(path_len, "path_len"), _dev_ptr(tokens, "tokens"),
            _dev_ptr(n_tokens, "n_tokens"), _stream_ptr(stream))
    keep = (logits, draft_tokens, parent, n_nodes, outputs)
    return _issue(_lib().fspad_tree_accept_greedy_static, "fspad_tree_accept_greedy_static", args, keep,
                  (path, path_len, tokens, n_tokens), prepare)


def fspad_tree_accept_sample(logits: torch.Tensor, draft_tokens: torch.Tensor, parent: torch.Tensor,
                             n_nodes: torch.Tensor, temperature: float, uniforms: torch.Tensor, outputs=None,
                             workspace: Optional[torch.Tensor] = None, stream=None, prepare: bool = False):
    """uniforms: device fp32 [B,2,Nmax] in [0,1). Returns (path, path_len, tokens, n_tokens); with
    prepare=True a PreparedCall."""
    B, Nmax, V, workspace = _accept_common(logits, draft_tokens, parent, n_nodes, workspace)
    if uniforms.dtype != torch.float32 or not uniforms.is_contiguous() or tuple(uniforms.shape) != (B, 2, Nmax):
        raise ValueError("uniforms must be a contiguous fp32 [B,2,Nmax] device tensor")
    path, path_len, tokens, n_tokens = _accept_outputs(B, Nmax, logits.device, outputs)
    args = (B, Nmax, V, _dev_ptr(logits, "logits", torch.float32), logits.stride(1),
            _dev_ptr(draft_tokens, "draft_tokens"), _dev_ptr(parent, "parent"), _dev_ptr(n_nodes, "n_nodes"),
            float(temperature), _dev_ptr(uniforms, "uniforms"),
            _dev_ptr(path, "path"), _dev_ptr(path_len, "path_len"), _dev_ptr(tokens, "tokens"),
            _dev_ptr(n_tokens, "n_tokens"), _dev_ptr(workspace, "workspace"),
            workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    keep = (logits, draft_tokens, parent, n_nodes, uniforms, workspace)
    return _issue(_lib().fspad_tree_accept_sample, "fspad_tree_accept_sample", args, keep,
                  (path, path_len, tokens, n_tokens), prepare)


def fspad_tree_accept_sample_draft_workspace_bytes(B: int, Nmax: int, V: int) -> int:
    return int(_lib().fspad_tree_accept_sample_draft_workspace_bytes(B, Nmax, V))


def fspad_tree_accept_sample_draft(logits: torch.Tensor, draft_logits: torch.Tensor, draft_tokens: torch.Tensor,
                                   parent: torch.Tensor, n_nodes: torch.Tensor, temperature: float,
                                   uniforms: torch.Tensor, outputs=None, workspace: Optional[torch.Tensor] = None,
                                   stream=None, prepare: bool = False):
    """logits, draft_logits fp32 [B,Nmax,V] with the same strides (vocabulary contiguous); uniforms fp32
    [B,2,Nmax]; everything on the device. Returns (path, path_len, tokens, n_tokens); with prepare=True a
    PreparedCall."""
    if workspace is None:
        workspace = torch.empty(max(16, fspad_tree_accept_sample_draft_workspace_bytes(*logits.shape)), dtype=torch.uint8,
                                device=logits.device)
    B, Nmax, V, workspace = _accept_common(logits, draft_tokens, parent, n_nodes, workspace)
    if draft_logits.dtype != torch.float32 or draft_logits.shape != logits.shape or draft_logits.stride() != logits.stride():
        raise ValueError("draft_logits must have the dtype, shape and strides of logits")
    if uniforms.dtype != torch.float32 or not uniforms.is_contiguous() or tuple(uniforms.shape) != (B, 2, Nmax):
        raise ValueError("uniforms must be a contiguous fp32 [B,2,Nmax] device tensor")
    path, path_len, tokens, n_tokens = _accept_outputs(B, Nmax, logits.device, outputs)
    args = (B, Nmax, V, _dev_ptr(logits, "logits", torch.float32), _dev_ptr(draft_logits, "draft_logits", torch.float32),
            logits.stride(1), _dev_ptr(draft_tokens, "draft_tokens"), _dev_ptr(parent, "parent"),
            _dev_ptr(n_nodes, "n_nodes"), float(temperature), _dev_ptr(uniforms, "uniforms"), _dev_ptr(path, "path"),
            _dev_ptr(path_len, "path_len"), _dev_ptr(tokens, "tokens"), _dev_ptr(n_tokens, "n_tokens"),
            _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    keep = (logits, draft_logits, draft_tokens, parent, n_nodes, uniforms, workspace)
    return _issue(_lib().fspad_tree_accept_sample_draft, "fspad_tree_accept_sample_draft", args, keep,
                  (path, path_len, tokens, n_tokens), prepare)


def fspad_tree_accept_lm_head_workspace_bytes(B: int, Nmax: int, V: int) -> int:
    return int(_lib().fspad_tree_accept_lm_head_workspace_bytes(B, Nmax, V))


def _lm_head_shapes(hidden, lm_head, packed, vocab):
    if hidden.dim() != 3 or not hidden.is_contiguous() or not lm_head.is_contiguous():
        raise ValueError("hidden must be a contiguous [B,Nmax,Hd] tensor and lm_head contiguous")
    B, Nmax, Hd = hidden.shape
    if packed and (vocab is not None or lm_head.dim() != 2):
        if vocab is None:
            raise ValueError("a flat packed lm_head needs `vocab`")
        V = int(vocab)
        if lm_head.numel() != (V + 15) // 16 * 16 * Hd:
            raise ValueError("packed lm_head does not have ceil(V/16)*16*Hd entries")
        return B, Nmax, Hd, V
    if lm_head.dim() != 2 or lm_head.shape[1] != Hd:
        raise ValueError("lm_head must be a [V,Hd] tensor with the hidden size of `hidden`")
    return B, Nmax, Hd, lm_head.shape[0]


def fspad_tree_accept_greedy_lm_head(hidden: torch.Tensor, lm_head: torch.Tensor, draft_tokens: torch.Tensor,
                                     parent: torch.Tensor, n_nodes: torch.Tensor, outputs=None, node_outputs=None,
                                     workspace: Optional[torch.Tensor] = None, stream=None, prepare: bool = False,
                                     packed: bool = False, vocab: Optional[int] = None):
    """hidden [B,Nmax,Hd] bf16, lm_head [V,Hd] bf16, both contiguous on the device (packed=True: lm_head
    is what fspad_pack_weight returned; give `vocab` when that is a flat tensor). Returns
    (path, path_len, tokens, n_tokens, node_target [B,Nmax] i32, node_top [B,Nmax] f32); with
    prepare=True a PreparedCall."""
    B, Nmax, Hd, V = _lm_head_shapes(hidden, lm_head, packed, vocab)
    for name, t in (("draft_tokens", draft_tokens), ("parent", parent), ("n_nodes", n_nodes)):
        if t.dtype != torch.int32 or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous int32 device tensor")
    if workspace is None:
        workspace = torch.empty(max(16, fspad_tree_accept_lm_head_workspace_bytes(B, Nmax, V)), dtype=torch.uint8,
                                device=hidden.device)
    path, path_len, tokens, n_tokens = _accept_outputs(B, Nmax, hidden.device, outputs)
    if node_outputs is None:
        node_outputs = (torch.empty((B, Nmax), dtype=torch.int32, device=hidden.device),
                        torch.empty((B, Nmax), dtype=torch.float32, device=hidden.device))
    node_target, node_top = node_outputs
    args = (B, Nmax, V, Hd, _dev_ptr(hidden, "hidden", torch.bfloat16), _dev_ptr(lm_head, "lm_head", torch.bfloat16),
            2 if packed else 0,
            _dev_ptr(draft_tokens, "draft_tokens"), _dev_ptr(parent, "parent"), _dev_ptr(n_nodes, "n_nodes"),
            _dev_ptr(path, "path"), _dev_ptr(path_len, "path_len"), _dev_ptr(tokens, "tokens"),
            _dev_ptr(n_tokens, "n_tokens"), _dev_ptr(node_target, "node_target", torch.int32),
            _dev_ptr(node_top, "node_top", torch.float32), _dev_ptr(workspace, "workspace"),
            workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    keep = (hidden, lm_head, draft_tokens, parent, n_nodes, workspace)
    return _issue(_lib().fspad_tree_accept_greedy_lm_head, "fspad_tree_accept_greedy_lm_head", args, keep,
                  (path, path_len, tokens, n_tokens, node_target, node_top), prepare)


def fspad_tree_accept_sample_lm_head(hidden: torch.Tensor, lm_head: torch.Tensor, draft_tokens: torch.Tensor,
                                     parent: torch.Tensor, n_nodes: torch.Tensor, temperature: float,
                                     uniforms: torch.Tensor, outputs=None, workspace: Optional[torch.Tensor] = None,
                                     stream=None, prepare: bool = False, packed: bool = False,
                                     vocab: Optional[int] = None):
    """hidden [B,Nmax,Hd] bf16, lm_head [V,Hd] bf16, uniforms fp32 [B,2,Nmax], all contiguous on the
    device (packed / vocab as for the greedy call). Returns (path, path_len, tokens, n_tokens); with
    prepare=True a PreparedCall."""
    B, Nmax, Hd, V = _lm_head_shapes(hidden, lm_head, packed, vocab)
    for name, t in (("draft_tokens", draft_tokens), ("parent", parent), ("n_nodes", n_nodes)):
        if t.dtype != torch.int32 or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous int32 device tensor")
    if uniforms.dtype != torch.float32 or not uniforms.is_contiguous() or tuple(uniforms.shape) != (B, 2, Nmax):
        raise ValueError("uniforms must be a contiguous fp32 [B,2,Nmax] device tensor")
    if workspace is None:
        workspace = torch.empty(max(16, fspad_tree_accept_lm_head_workspace_bytes(B, Nmax, V)), dtype=torch.uint8,
                                device=hidden.device)
    path, path_len, tokens, n_tokens = _accept_outputs(B, Nmax, hidden.device, outputs)
    args = (B, Nmax, V, Hd, _dev_ptr(hidden, "hidden", torch.bfloat16), _dev_ptr(lm_head, "lm_head", torch.bfloat16),
            2 if packed else 0,
            _dev_ptr(draft_tokens, "draft_tokens"), _dev_ptr(parent, "parent"), _dev_ptr(n_nodes, "n_nodes"),
            float(temperature), _dev_ptr(uniforms, "uniforms"),
            _dev_ptr(path, "path"), _dev_ptr(path_len, "path_len"), _dev_ptr(tokens, "tokens"),
            _dev_ptr(n_tokens, "n_tokens"), _dev_ptr(workspace, "workspace"),
            workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    keep = (hidden, lm_head, draft_tokens, parent, n_nodes, uniforms, workspace)
    return _issue(_lib().fspad_tree_accept_sample_lm_head, "fspad_tree_accept_sample_lm_head", args, keep,
                  (path, path_len, tokens, n_tokens), prepare)


def fspad_kv_commit(k_tree: torch.Tensor, v_tree: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                    kv_len, path: torch.Tensor, path_len: torch.Tensor,
                    kv_len_out: Optional[torch.Tensor] = None, stream=None, prepare: bool = False):
    """Appends the accepted nodes' keys/values to the cache in place. k_tree,v_tree [B,Nmax,Hkv,D];
    k_cache,v_cache [B,Hkv,Lcap,D] views; kv_len HOST int32 [B]; path [B,Nmax], path_len [B] device
    int32 (from an acceptance call). Returns kv_len_out."""
    for name, t in (("k_tree", k_tree), ("v_tree", v_tree)):
        if not t.is_contiguous():
            raise ValueError(f"{name} must be contiguous")
    if (v_cache.stride() != k_cache.stride() or v_cache.shape != k_cache.shape or k_cache.stride(3) != 1
            or k_cache.dtype != k_tree.dtype or v_cache.dtype != k_tree.dtype):
        raise ValueError("k_cache and v_cache must share shape, strides and the dtype of k_tree")
    B, Nmax, Hkv, D = k_tree.shape
    d = fspad_attn_desc()
    d.batch, d.n_nodes_max, d.n_q_heads, d.n_kv_heads, d.head_dim = B, Nmax, Hkv, Hkv, D
    d.io_dtype = d.out_dtype = _dtype_code(k_tree.dtype)
    d.cache_stride_batch, d.cache_stride_head, d.cache_stride_token = (
        k_cache.stride(0), k_cache.stride(1), k_cache.stride(2))
    kv_len = _host_i32(kv_len, "kv_len")
    if kv_len.shape != (B,):
        raise ValueError("kv_len must have one entry per sequence")
    if path.shape != (B, Nmax) or path_len.shape != (B,) or not path.is_contiguous():
        raise ValueError("path must be [B,Nmax] and path_len [B]")
    args = (ctypes.byref(d), _dev_ptr(k_tree, "k_tree"), _dev_ptr(v_tree, "v_tree"),
            _dev_ptr(k_cache, "k_cache"), _dev_ptr(v_cache, "v_cache"), int(k_cache.shape[2]),
            kv_len.ctypes.data, _dev_ptr(path, "path", torch.int32), _dev_ptr(path_len, "path_len", torch.int32),
            _dev_ptr(kv_len_out, "kv_len_out", torch.int32), _stream_ptr(stream))
    keep = (d, k_tree, v_tree, k_cache, v_cache, kv_len, path, path_len, kv_len_out)
    return _issue(_lib().fspad_kv_commit, "fspad_kv_commit", args, keep, kv_len_out, prepare)


def fspad_feature_sampler_workspace_bytes(rows: int, hidden_dim: int, intermediate_dim: int) -> int:
    return int(_lib().fspad_feature_sampler_workspace_bytes(rows, hidden_dim, intermediate_dim))


def fspad_packed_weight_bytes(n_rows: int, k: int) -> int:
    return int(_lib().fspad_packed_weight_bytes(int(n_rows), int(k)))


def fspad_pack_weight(w: torch.Tensor, stream=None) -> torch.Tensor:
    """Repack a contiguous [N,K] bf16 device matrix into the tile order the draft-side projections stream
    fastest (pass the result with packed=True). Returns a new tensor of the same shape (N a multiple of 16;
    its bytes are the tiles, not rows) or, when N is not a multiple of 16, a flat bf16 tensor."""
    N, K = w.shape
    if not w.is_contiguous() or w.dtype != torch.bfloat16:
        raise ValueError("w must be a contiguous bf16 matrix")
    need = fspad_packed_weight_bytes(N, K)
    if need == 0:
        raise FspadError(2, "fspad_pack_weight")
    out = torch.empty(need // 2, dtype=torch.bfloat16, device=w.device)
    _check(_lib().fspad_pack_weight(N, K, _dev_ptr(w, "w"), _dev_ptr(out, "packed"), _stream_ptr(stream)), "fspad_pack_weight")
    return out.view(N, K) if N % 16 == 0 else out


def fspad_feature_sampler(f: torch.Tensor, e: torch.Tensor, w_up: torch.Tensor, w_gate: torch.Tensor,
                          w_down: torch.Tensor, residual: bool = True, out: Optional[torch.Tensor] = None,
                          workspace: Optional[torch.Tensor] = None, stream=None, prepare: bool = False,
                          packed: bool = False):
    """f, e [rows,Hd]; w_up, w_gate [I,Hd]; w_down [Hd,I]; all contiguous bf16 device tensors (packed=True:
    the three weight matrices went through fspad_pack_weight). Returns eta [rows,Hd] bf16; with
    prepare=True a PreparedCall."""
    rows, Hd = f.shape
    I = w_up.shape[0]
    for name, t, shape in (("f", f, (rows, Hd)), ("e", e, (rows, Hd)), ("w_up", w_up, (I, Hd)), ("w_gate", w_gate, (I, Hd)),
                           ("w_down", w_down, (Hd, I))):
        if tuple(t.shape) != shape or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous {shape} tensor")
    if out is None:
        out = torch.empty((rows, Hd), dtype=torch.bfloat16, device=f.device)
    if workspace is None:
        workspace = torch.empty(max(16, fspad_feature_sampler_workspace_bytes(rows, Hd, I)), dtype=torch.uint8, device=f.device)
    args = (rows, Hd, I, _dev_ptr(f, "f", torch.bfloat16), _dev_ptr(e, "e", torch.bfloat16),
            _dev_ptr(w_up, "w_up", torch.bfloat16), _dev_ptr(w_gate, "w_gate", torch.bfloat16),
            _dev_ptr(w_down, "w_down", torch.bfloat16), (1 if residual else 0) | (2 if packed else 0),
            _dev_ptr(out, "eta", torch.bfloat16),
            _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    return _issue(_lib().fspad_feature_sampler, "fspad_feature_sampler", args, (f, e, w_up, w_gate, w_down, workspace),
                  out, prepare)


def fspad_draft_layer_workspace_bytes(desc: fspad_draft_layer_desc, max_kv_len: int) -> int:
    return int(_lib().fspad_draft_layer_workspace_bytes(ctypes.byref(desc), int(max_kv_len)))


_DRAFT_LAYER_WEIGHTS = ("w_qkv", "w_o", "w_gate", "w_up", "w_down", "gain_attn", "gain_mlp")


def fspad_draft_layer(eta: torch.Tensor, positions: torch.Tensor, weights: dict, k_cache: Optional[torch.Tensor],
                      v_cache: Optional[torch.Tensor], kv_len, n_nodes, anc_mask: torch.Tensor, n_q_heads: int,
                      n_kv_heads: int, head_dim: int, rms_eps: float = 1e-6, rope_theta: float = 10000.0,
                      outputs=None, workspace: Optional[torch.Tensor] = None, stream=None, prepare: bool = False,
                      packed: bool = False):
    """eta [B,Nmax,Hd] bf16; positions [B,Nmax] int32 (device); weights: dict of contiguous bf16 device
    tensors w_qkv [(Hq+2Hkv)D,Hd], w_o [Hd,HqD], w_gate, w_up [I,Hd], w_down [2Hd,I], gain_attn, gain_mlp
    [Hd] (packed=True: the five matrices went through fspad_pack_weight); k_cache, v_cache [B,Hkv,Lcap,D] views of the draft's own cache (or None); kv_len, n_nodes HOST
    int32 [B]; anc_mask device 64-bit [B,Nmax]. Returns (f_tilde, f, k_tree, v_tree): [B,Nmax,Hd] twice and
    [B,Nmax,Hkv,D] twice, bf16 (pass them as `outputs` to reuse buffers); with prepare=True a PreparedCall."""
    B, Nmax, Hd = eta.shape
    Hq, Hkv, D = int(n_q_heads), int(n_kv_heads), int(head_dim)
    I = weights["w_up"].shape[0]
    shapes = {"w_qkv": ((Hq + 2 * Hkv) * D, Hd), "w_o": (Hd, Hq * D), "w_gate": (I, Hd), "w_up": (I, Hd),
              "w_down": (2 * Hd, I), "gain_attn": (Hd,), "gain_mlp": (Hd,)}
    for name in _DRAFT_LAYER_WEIGHTS:
        t = weights[name]
        if tuple(t.shape) != shapes[name] or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous {shapes[name]} tensor")
    if not eta.is_contiguous() or not positions.is_contiguous() or tuple(positions.shape) != (B, Nmax):
        raise ValueError("eta must be contiguous and positions a contiguous [B,Nmax] tensor")
    if k_cache is not None and (v_cache is None or v_cache.stride() != k_cache.stride()
                                or v_cache.dtype != eta.dtype or k_cache.dtype != eta.dtype):
        raise ValueError("k_cache and v_cache must share strides and the dtype of eta")
    if anc_mask.dtype not in (torch.int64, torch.uint64) or not anc_mask.is_contiguous():
        raise ValueError("anc_mask must be a contiguous 64-bit integer tensor")
    desc = fspad_draft_layer_desc()
    a = desc.attn
    a.batch, a.n_nodes_max, a.n_q_heads, a.n_kv_heads, a.head_dim = B, Nmax, Hq, Hkv, D
    a.io_dtype = a.out_dtype = _dtype_code(eta.dtype)
    a.softmax_scale = 0.0
    if k_cache is not None:
        if k_cache.stride(3) != 1:
            raise ValueError("head_dim must be contiguous in the cache")
        a.cache_stride_batch, a.cache_stride_head, a.cache_stride_token = k_cache.stride(0), k_cache.stride(1), k_cache.stride(2)
    else:
        a.cache_stride_batch = a.cache_stride_head = 0
        a.cache_stride_token = D
    desc.hidden_dim, desc.intermediate_dim, desc.rms_eps, desc.rope_theta = Hd, I, float(rms_eps), float(rope_theta)
    desc.weights_packed = 1 if packed else 0
    w = fspad_draft_layer_weights()
    for name in _DRAFT_LAYER_WEIGHTS:
        setattr(w, name, _dev_ptr(weights[name], name, torch.bfloat16))
    kv_len = _host_i32(kv_len, "kv_len")
    n_nodes = _host_i32(n_nodes, "n_nodes")
    if kv_len.shape != (B,) or n_nodes.shape != (B,):
        raise ValueError("kv_len and n_nodes must have one entry per sequence")
    if outputs is None:
        outputs = (torch.empty((B, Nmax, Hd), dtype=torch.bfloat16, device=eta.device),
                   torch.empty((B, Nmax, Hd), dtype=torch.bfloat16, device=eta.device),
                   torch.empty((B, Nmax, Hkv, D), dtype=torch.bfloat16, device=eta.device),
                   torch.empty((B, Nmax, Hkv, D), dtype=torch.bfloat16, device=eta.device))
    f_tilde, f, k_tree, v_tree = outputs
    if workspace is None:
        need = fspad_draft_layer_workspace_bytes(desc, int(kv_len.max(initial=0)))
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=eta.device)
    args = (ctypes.byref(desc), ctypes.byref(w), _dev_ptr(eta, "eta", torch.bfloat16),
            _dev_ptr(positions, "positions", torch.int32), _dev_ptr(k_cache, "k_cache"), _dev_ptr(v_cache, "v_cache"),
            kv_len.ctypes.data, n_nodes.ctypes.data, _dev_ptr(anc_mask, "anc_mask"),
            _dev_ptr(k_tree, "k_tree", torch.bfloat16), _dev_ptr(v_tree, "v_tree", torch.bfloat16),
            _dev_ptr(f_tilde, "f_tilde", torch.bfloat16), _dev_ptr(f, "f", torch.bfloat16),
            _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    keep = (desc, w, eta, positions, dict(weights), k_cache, v_cache, kv_len, n_nodes, anc_mask, outputs, workspace)
    return _issue(_lib().fspad_draft_layer, "fspad_draft_layer", args, keep, outputs, prepare)


def fspad_draft_topk_workspace_bytes(rows: int, V: int, k: int) -> int:
    return int(_lib().fspad_draft_topk_workspace_bytes(rows, V, k))


def fspad_draft_topk(logits: torch.Tensor, k: int, outputs=None, workspace: Optional[torch.Tensor] = None,
                     stream=None, prepare: bool = False):
    """logits: device fp32 [rows,V] (rows may be strided, entries contiguous). Returns
    (tokens [rows,k] i32, logp [rows,k] f32); with prepare=True a PreparedCall."""
    if logits.dim() != 2 or logits.stride(1) != 1:
        raise ValueError("logits must be [rows,V] with contiguous entries")
    rows, V = logits.shape
    if workspace is None:
        workspace = torch.empty(max(16, fspad_draft_topk_workspace_bytes(rows, V, k)), dtype=torch.uint8,
                                device=logits.device)
    if outputs is None:
        outputs = (torch.empty((rows, k), dtype=torch.int32, device=logits.device),
                   torch.empty((rows, k), dtype=torch.float32, device=logits.device))
    tokens, logp = outputs
    args = (rows, V, int(k), _dev_ptr(logits, "logits", torch.float32), logits.stride(0),
            _dev_ptr(tokens, "tokens", torch.int32), _dev_ptr(logp, "logp", torch.float32),
            _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    return _issue(_lib().fspad_draft_topk, "fspad_draft_topk", args, (logits, workspace), (tokens, logp), prepare)


def fspad_tree_build(cand_parent: torch.Tensor, cand_token: torch.Tensor, cand_logp: torch.Tensor,
                     n_cand: torch.Tensor, n_keep: int, n_max: int, outputs=None, stream=None,
                     prepare: bool = False):
    """Device tensors: cand_parent, cand_token int32 [B,M], cand_logp fp32 [B,M], n_cand int32 [B].
    Returns (parent [B,n_max], draft_tokens [B,n_max], n_nodes [B], anc_mask [B,n_max] int64 bit
    pattern of the u64 words, node_cand [B,n_max]); `outputs` may bring these five tensors."""
    B, M = cand_parent.shape
    for name, t, dt in (("cand_parent", cand_parent, torch.int32), ("cand_token", cand_token, torch.int32),
                        ("cand_logp", cand_logp, torch.float32)):
        if t.dtype != dt or not t.is_contiguous() or tuple(t.shape) != (B, M):
            raise ValueError(f"{name} must be a contiguous {dt} [B,M] device tensor")
    if n_cand.dtype != torch.int32 or tuple(n_cand.shape) != (B,):
        raise ValueError("n_cand must be an int32 [B] device tensor")
    dev = cand_parent.device
    if outputs is None:
        outputs = (torch.empty((B, n_max), dtype=torch.int32, device=dev), torch.empty((B, n_max), dtype=torch.int32, device=dev),
                   torch.empty((B,), dtype=torch.int32, device=dev), torch.empty((B, n_max), dtype=torch.int64, device=dev),
                   torch.empty((B, n_max), dtype=torch.int32, device=dev))
    parent, tokens, n_nodes, mask, node_cand = outputs
    for name, t, shape in (("parent", parent, (B, n_max)), ("draft_tokens", tokens, (B, n_max)), ("n_nodes", n_nodes, (B,)),
                           ("anc_mask", mask, (B, n_max)), ("node_cand", node_cand, (B, n_max))):
        if tuple(t.shape) != shape or not t.is_contiguous() or t.dtype != (torch.int64 if name == "anc_mask" else torch.int32):
            raise ValueError(f"{name} must be a contiguous {shape} device tensor of the documented type")
    args = (B, M, int(n_max), _dev_ptr(cand_parent, "cand_parent"), _dev_ptr(cand_token, "cand_token"),
            _dev_ptr(cand_logp, "cand_logp"), _dev_ptr(n_cand, "n_cand"), int(n_keep), _dev_ptr(parent, "parent"),
            _dev_ptr(tokens, "draft_tokens"), _dev_ptr(n_nodes, "n_nodes"), _dev_ptr(mask, "anc_mask"),
            _dev_ptr(node_cand, "node_cand"), _stream_ptr(stream))
    keep = (cand_parent, cand_token, cand_logp, n_cand)
    return _issue(_lib().fspad_tree_build, "fspad_tree_build", args, keep,
                  (parent, tokens, n_nodes, mask, node_cand), prepare)


def fspad_tree_build_mask(parent, n_nodes) -> np.ndarray:
    """Host arrays in, host uint64 [B,Nmax] out."""
    parent = _host_i32(parent, "parent")
    n_nodes = _host_i32(n_nodes, "n_nodes")
    B, Nmax = parent.shape
    mask = np.zeros((B, Nmax), dtype=np.uint64)
    st = _lib().fspad_tree_build_mask(B, Nmax, parent.ctypes.data, n_nodes.ctypes.data, mask.ctypes.data)
    _check(st, "fspad_tree_build_mask")
    return mask


def fspad_tree_validate(parent, tokens, n_nodes, vocab: int) -> int:
    """Returns the status code (0 = well-formed) instead of raising."""
    parent = _host_i32(parent, "parent")
    n_nodes = _host_i32(n_nodes, "n_nodes")
    B, Nmax = parent.shape
    tok_ptr = None
    if tokens is not None:
        tokens = _host_i32(tokens, "tokens")
        tok_ptr = tokens.ctypes.data
    return int(_lib().fspad_tree_validate(B, Nmax, int(vocab), parent.ctypes.data, tok_ptr, n_nodes.ctypes.data))


def fspad_status_string(status: int) -> str:
    return _lib().fspad_status_string(int(status)).decode()
