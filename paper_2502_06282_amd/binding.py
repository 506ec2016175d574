"""ctypes binding of libjakiro_verify (argument marshalling only).

Function names and argument meaning follow include/jakiro_verify.h.  Tensors
are torch tensors on the ROCm device; torch is used for device memory and the
current stream, nothing else.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libjakiro_verify.so")

JK_BF16, JK_F32 = 0, 1
JK_GREEDY, JK_SAMPLE = 0, 1
JK_DEVERR_BAD_TREE, JK_DEVERR_BAD_TOKEN, JK_DEVERR_BAD_PAGE, JK_DEVERR_MERGE_WAIT, JK_DEVERR_WALK_WAIT = 1, 2, 4, 8, 16
JK_WORKSPACE_HEADER_BYTES = 32768
JK_HEADS_DECOUPLED, JK_HEADS_CONTRASTIVE = 0, 1
MAX_TREE = 128


class JakiroError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib().jk_status_string(status).decode()} (status {status})")


class AttnDesc(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_tree", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("q_stride_b", ctypes.c_int64), ("q_stride_t", ctypes.c_int64), ("q_stride_h", ctypes.c_int64),
        ("kc_stride_b", ctypes.c_int64), ("kc_stride_l", ctypes.c_int64), ("kc_stride_h", ctypes.c_int64),
        ("kt_stride_b", ctypes.c_int64), ("kt_stride_t", ctypes.c_int64), ("kt_stride_h", ctypes.c_int64),
        ("o_stride_b", ctypes.c_int64), ("o_stride_t", ctypes.c_int64), ("o_stride_h", ctypes.c_int64),
        ("scale", ctypes.c_float), ("dtype", ctypes.c_int32),
    ]


_lib = None

class DraftHeadsDesc(ctypes.Structure):
    """jk_draft_heads_desc"""
    _fields_ = [("rows", ctypes.c_int32), ("d_model", ctypes.c_int32), ("vocab", ctypes.c_int32),
                ("top_k", ctypes.c_int32), ("mode", ctypes.c_int32), ("temperature", ctypes.c_float),
                ("alpha", ctypes.c_float), ("beta", ctypes.c_float)]


class MoeDesc(ctypes.Structure):
    """jk_moe_desc"""
    _fields_ = [("rows", ctypes.c_int32), ("d_model", ctypes.c_int32), ("d_ff", ctypes.c_int32),
                ("n_experts", ctypes.c_int32)]


class TreeStateDesc(ctypes.Structure):
    """jk_tree_state"""
    _fields_ = [("tokens", ctypes.c_void_p), ("parent", ctypes.c_void_p), ("score", ctypes.c_void_p),
                ("q_row", ctypes.c_void_p), ("n_nodes", ctypes.c_void_p), ("max_nodes", ctypes.c_int32)]


class PagedKV(ctypes.Structure):
    """jk_paged_kv"""
    _fields_ = [("block_table", ctypes.c_void_p), ("max_blocks", ctypes.c_int32), ("page_size", ctypes.c_int32),
                ("n_pages", ctypes.c_int32), ("page_stride", ctypes.c_int64)]


EXPORTS = ("jk_tree_verify_attention_workspace", "jk_tree_verify_attention_plan", "jk_tree_verify_attention", "jk_tree_verify_attention_paged",
           "jk_commit_path_layers_paged", "jk_accept_path_workspace",
           "jk_accept_path", "jk_accept_path_greedy_static", "jk_accept_path_rows", "jk_draft_heads_workspace", "jk_draft_heads", "jk_moe_experts_workspace", "jk_moe_experts", "jk_linear_workspace", "jk_linear", "jk_tree_grow", "jk_tree_grow_tail", "jk_tree_fill_static", "jk_tree_finalize", "jk_gather_draft_probs", "jk_commit_path", "jk_commit_path_layers", "jk_workspace_init", "jk_init", "jk_set_tuning", "jk_last_device_error", "jk_stream_read_probe", "jk_validate_tree", "jk_status_string", "jk_version")


def library_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with "
                               "`python -m paper_2502_06282_amd.build` (needs hipcc)")
        l = ctypes.CDLL(_LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        l.jk_tree_verify_attention_workspace.restype = sz
        l.jk_tree_verify_attention_workspace.argtypes = [ctypes.POINTER(AttnDesc), i32]
        l.jk_tree_verify_attention.restype = i32
        l.jk_tree_verify_attention.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp, vp, i32,
                                               vp, vp, sz, vp]
        l.jk_tree_verify_attention_paged.restype = i32
        l.jk_tree_verify_attention_paged.argtypes = [ctypes.POINTER(AttnDesc), ctypes.POINTER(PagedKV), vp, vp, vp, vp, vp,
                                                     vp, vp, i32, vp, vp, sz, vp]
        l.jk_commit_path_layers_paged.restype = i32
        l.jk_commit_path_layers_paged.argtypes = [ctypes.POINTER(AttnDesc), ctypes.POINTER(PagedKV), i32, vp, vp, vp, vp,
                                                  vp, vp, i32, vp, i32, vp]
        l.jk_accept_path_workspace.restype = sz
        l.jk_accept_path_workspace.argtypes = [i32, i32, i32, i32]
        l.jk_accept_path.restype = i32
        l.jk_accept_path.argtypes = [i32, i32, i32, i32, vp, vp, vp, i32, ctypes.c_float, vp, vp, vp, vp,
                                     vp, vp, sz, vp]
        l.jk_accept_path_rows.restype = i32
        l.jk_accept_path_rows.argtypes = [i32, i32, i32, i32, vp, vp, vp, i32, ctypes.c_float, vp, ctypes.c_int64, vp,
                                          vp, vp, vp, vp, vp, sz, vp]
        l.jk_commit_path.restype = i32
        l.jk_commit_path.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp, i32, i32, vp, i32, vp]
        l.jk_commit_path_layers.restype = i32
        l.jk_commit_path_layers.argtypes = [ctypes.POINTER(AttnDesc), i32, vp, vp, vp, vp, vp, vp, i32, i32, vp, i32, vp]
        l.jk_draft_heads_workspace.restype = sz
        l.jk_draft_heads_workspace.argtypes = [i32, i32, i32]
        l.jk_draft_heads.restype = i32
        l.jk_draft_heads.argtypes = [ctypes.POINTER(DraftHeadsDesc), vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        l.jk_moe_experts_workspace.restype = sz
        l.jk_moe_experts_workspace.argtypes = [ctypes.POINTER(MoeDesc)]
        l.jk_moe_experts.restype = i32
        l.jk_moe_experts.argtypes = [ctypes.POINTER(MoeDesc), vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        l.jk_linear_workspace.restype = sz
        l.jk_linear_workspace.argtypes = [i32, i32, i32]
        l.jk_linear.restype = i32
        l.jk_linear.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
        l.jk_tree_grow.restype = i32
        l.jk_tree_grow.argtypes = [ctypes.POINTER(TreeStateDesc), i32, i32, i32, i32, i32, vp, vp, vp, vp, vp]
        l.jk_tree_grow_tail.restype = i32
        l.jk_tree_grow_tail.argtypes = [ctypes.POINTER(TreeStateDesc), i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp]
        l.jk_tree_fill_static.restype = i32
        l.jk_tree_fill_static.argtypes = [ctypes.POINTER(TreeStateDesc), i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, i32,
                                          vp, i32, vp, vp, vp]
        l.jk_tree_finalize.restype = i32
        l.jk_tree_finalize.argtypes = [ctypes.POINTER(TreeStateDesc), i32, i32, vp, vp, vp, vp, vp, vp]
        l.jk_gather_draft_probs.restype = i32
        l.jk_gather_draft_probs.argtypes = [i32, i32, i32, vp, ctypes.c_int64, vp, vp, vp]
        l.jk_workspace_init.restype = i32
        l.jk_workspace_init.argtypes = [vp, sz, vp]
        l.jk_tree_verify_attention_plan.restype = i32
        l.jk_tree_verify_attention_plan.argtypes = [ctypes.POINTER(AttnDesc), i32, ctypes.POINTER(i32)]
        l.jk_init.restype = i32
        l.jk_init.argtypes = [vp]
        l.jk_set_tuning.restype = i32
        l.jk_set_tuning.argtypes = [ctypes.c_char_p, i32]
        l.jk_last_device_error.restype = i32
        l.jk_last_device_error.argtypes = [vp]
        l.jk_stream_read_probe.restype = i32
        l.jk_stream_read_probe.argtypes = [vp, sz, vp, vp]
        l.jk_validate_tree.restype = i32
        l.jk_validate_tree.argtypes = [ctypes.POINTER(ctypes.c_int32), i32]
        l.jk_status_string.restype = ctypes.c_char_p
        l.jk_status_string.argtypes = [i32]
        l.jk_version.restype = ctypes.c_char_p
        l.jk_version.argtypes = []
        _lib = l
    return _lib


def version() -> str:
    return lib().jk_version().decode()


def validate_tree(parent) -> int:
    """Status code of jk_validate_tree for a host sequence of ints."""
    arr = (ctypes.c_int32 * len(parent))(*[int(x) for x in parent])
    return int(lib().jk_validate_tree(arr, len(parent)))


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


_initialised_devices = set()


def _stream_handle(stream) -> Optional[int]:
    """The hipStream_t of `stream` (default: torch's current stream).  The first use on a device also runs
    jk_init there (a short synchronous probe), unless that stream is being captured into a graph."""
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    handle = s.cuda_stream or None
    dev = torch.cuda.current_device()
    if dev not in _initialised_devices and not torch.cuda.is_current_stream_capturing():
        st = lib().jk_init(handle)
        if st != 0:
            raise JakiroError(st, "jk_init")
        _initialised_devices.add(dev)
    return handle


def _new_workspace(nbytes: int, device, stream):
    """A zero-filled workspace whose fill is ordered on the stream the library call will use, and which the
    caching allocator will not hand out again while that stream may still be using it."""
    import torch
    s = torch.cuda.current_stream(device) if stream is None else stream
    with torch.cuda.stream(s):
        ws = torch.zeros(nbytes, dtype=torch.uint8, device=device)
    ws.record_stream(s)
    return ws


def set_tuning(name: str, value: int) -> None:
    """jk_set_tuning: force part of a launch plan (experiments and tests)."""
    st = lib().jk_set_tuning(name.encode(), int(value))
    if st != 0:
        raise JakiroError(st, f"jk_set_tuning({name})")


def last_device_error(workspace) -> int:
    """jk_last_device_error: the sticky JK_DEVERR_* bits of an attention or acceptance workspace (synchronous)."""
    return int(lib().jk_last_device_error(_ptr(workspace)))


def _make_desc(q, k_cache, k_tree, out, scale: float) -> AttnDesc:
    import torch
    B, T, Hq, D = q.shape
    Hkv = k_tree.shape[2]
    if q.dtype == torch.bfloat16:
        dt = JK_BF16
    elif q.dtype == torch.float32:
        dt = JK_F32
    else:
        raise TypeError("q must be bfloat16 or float32")
    for t in (q, k_cache, k_tree, out):
        if t is not None and t.stride(-1) != 1 and t.shape[-1] > 1:
            raise ValueError("head_dim must be the contiguous innermost axis")
    kc = k_cache.stride() if k_cache is not None else (0, 0, 0, 1)
    return AttnDesc(B, T, Hq, Hkv, D, q.stride(0), q.stride(1), q.stride(2), kc[0], kc[1], kc[2],
                    k_tree.stride(0), k_tree.stride(1), k_tree.stride(2),
                    out.stride(0), out.stride(1), out.stride(2), float(scale), dt)


def tree_verify_attention_workspace(q, k_cache, k_tree, max_prefix_len: int, scale: float = 0.0) -> int:
    d = _make_desc(q, k_cache, k_tree, q, scale)
    return int(lib().jk_tree_verify_attention_workspace(ctypes.byref(d), int(max_prefix_len)))


def tree_verify_attention_plan(q, k_cache, k_tree, max_prefix_len: int, scale: float = 0.0) -> dict:
    """jk_tree_verify_attention_plan as a dict (wm, wn, kt, row_tiles, splits, fused)."""
    _stream_handle(None)  # (the plan depends on jk_init having run on this device)
    d = _make_desc(q, k_cache, k_tree, q, scale)
    out = (ctypes.c_int32 * 6)()
    st = lib().jk_tree_verify_attention_plan(ctypes.byref(d), int(max_prefix_len), out)
    if st != 0:
        raise JakiroError(st, "jk_tree_verify_attention_plan")
    return dict(zip(("wm", "wn", "kt", "row_tiles", "splits", "fused"), [int(v) for v in out]))


def tree_verify_attention(q, k_cache, v_cache, k_tree, v_tree, parent, prefix_len,
                          max_prefix_len: Optional[int] = None, scale: float = 0.0, out=None,
                          workspace=None, stream=None):
    """jk_tree_verify_attention.  q [B,T,Hq,D]; k_cache, v_cache [B,Lcap,Hkv,D] (same strides);
    k_tree, v_tree [B,T,Hkv,D] (same strides); parent int32 [B,T]; prefix_len int32 [B], all on
    the device.  Returns out [B,T,Hq,D] (allocated unless given).  Asynchronous on `stream`
    (default: torch's current stream)."""
    import torch
    if k_cache is not None and k_cache.shape[1] == 0:  # an empty cache has no meaningful strides
        k_cache = v_cache = None
    if max_prefix_len is None:
        max_prefix_len = 0 if k_cache is None else int(k_cache.shape[1])
    if out is None:
        out = torch.empty_like(q, memory_format=torch.contiguous_format)
    if k_cache is not None and (k_cache.stride() != v_cache.stride() or k_cache.shape != v_cache.shape):
        raise ValueError("k_cache and v_cache must share shape and strides")
    if k_tree.stride() != v_tree.stride() or k_tree.shape != v_tree.shape:
        raise ValueError("k_tree and v_tree must share shape and strides")
    if parent.dtype != torch.int32 or prefix_len.dtype != torch.int32:
        raise TypeError("parent and prefix_len must be int32")
    if not (parent.is_contiguous() and prefix_len.is_contiguous()):
        raise ValueError("parent and prefix_len must be contiguous")
    d = _make_desc(q, k_cache, k_tree, out, scale)
    need = int(lib().jk_tree_verify_attention_workspace(ctypes.byref(d), int(max_prefix_len)))
    if need == 0:
        raise JakiroError(3, "jk_tree_verify_attention_workspace")
    if workspace is None:
        workspace = _new_workspace(need, q.device, stream)
    st = lib().jk_tree_verify_attention(ctypes.byref(d), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_tree),
                                        _ptr(v_tree), _ptr(parent), _ptr(prefix_len), int(max_prefix_len),
                                        _ptr(out), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                        _stream_handle(stream))
    if st != 0:
        raise JakiroError(st, "jk_tree_verify_attention")
    return out


def accept_path_workspace(batch: int, n_tree: int, vocab: int, mode: int) -> int:
    return int(lib().jk_accept_path_workspace(batch, n_tree, vocab, mode))


def stream_read_probe(src, sink, stream=None) -> None:
    """jk_stream_read_probe over the whole tensor `src` (measurement aid)."""
    st = lib().jk_stream_read_probe(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream_handle(stream))
    if st != 0:
        raise JakiroError(st, "jk_stream_read_probe")


def workspace_init(workspace, stream=None) -> None:
    """jk_workspace_init: zero-fill a workspace tensor on `stream` (once, before its first accept_path)."""
    st = lib().jk_workspace_init(_ptr(workspace), workspace.numel() * workspace.element_size(),
                                 _stream_handle(stream))
    if st != 0:
        raise JakiroError(st, "jk_workspace_init")


def accept_path(tree_tokens, parent, target_logits, mode: int = JK_GREEDY, temperature: float = 1.0,
                draft_probs=None, uniforms=None, max_depth: Optional[int] = None, workspace=None,
                stream=None) -> Tuple["torch.Tensor", "torch.Tensor", "torch.Tensor"]:
    """jk_accept_path.  tree_tokens, parent int32 [B,N]; target_logits fp32 [B,N+1,V] contiguous;
    sampling also needs draft_probs fp32 [B,N,V] and uniforms fp32 [B,N+1].
    Returns (path [B,max_depth], accept_len [B], bonus_token [B]) int32 device tensors."""
    import torch
    B, N = tree_tokens.shape
    V = target_logits.shape[-1]
    if max_depth is None:
        max_depth = N
    for t in (tree_tokens, parent):
        if t.dtype != torch.int32 or not t.is_contiguous():
            raise TypeError("tree_tokens and parent must be contiguous int32")
    for t in (target_logits, draft_probs, uniforms):
        if t is not None and (t.dtype != torch.float32 or not t.is_contiguous()):
            raise TypeError("logits, draft_probs and uniforms must be contiguous float32")
    if target_logits.shape != (B, N + 1, V):
        raise ValueError("target_logits must be [B, N+1, V]")
    dev = tree_tokens.device
    path = torch.empty((B, max_depth), dtype=torch.int32, device=dev)
    alen = torch.empty((B,), dtype=torch.int32, device=dev)
    bonus = torch.empty((B,), dtype=torch.int32, device=dev)
    need = accept_path_workspace(B, N, V, mode)
    if need == 0:
        raise JakiroError(3, "jk_accept_path_workspace")
    if workspace is None:
        workspace = _new_workspace(need, dev, stream)
    st = lib().jk_accept_path(B, N, V, int(max_depth), _ptr(tree_tokens), _ptr(parent), _ptr(target_logits),
                              int(mode), float(temperature), _ptr(draft_probs), _ptr(uniforms), _ptr(path),
                              _ptr(alen), _ptr(bonus), _ptr(workspace),
                              workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if st != 0:
        raise JakiroError(st, "jk_accept_path")
    return path, alen, bonus


def accept_path_greedy_static(tree_tokens, parent, target_logits, out_path, out_accept_len, out_bonus_token,
                              stream=None) -> None:
    """jk_accept_path_greedy_static: greedy acceptance without a workspace (the library's built-in scratch
    buffer); the caller passes every output tensor, the call allocates nothing.  out_path int32 [B, max_depth]."""
    import torch
    B, N = tree_tokens.shape
    V = target_logits.shape[-1]
    for t in (tree_tokens, parent, out_path, out_accept_len, out_bonus_token):
        if t.dtype != torch.int32 or not t.is_contiguous():
            raise TypeError("tokens, parent and the outputs must be contiguous int32")
    if target_logits.dtype != torch.float32 or not target_logits.is_contiguous() or target_logits.shape != (B, N + 1, V):
        raise TypeError("target_logits must be contiguous float32 [B, N+1, V]")
    if out_path.dim() != 2 or out_path.shape[0] != B or out_accept_len.numel() != B or out_bonus_token.numel() != B:
        raise ValueError("outputs must be [B, max_depth], [B], [B]")
    fn = lib().jk_accept_path_greedy_static
    vp, i32 = ctypes.c_void_p, ctypes.c_int32
    fn.restype = i32
    fn.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    st = fn(B, N, V, int(out_path.shape[1]), _ptr(tree_tokens), _ptr(parent), _ptr(target_logits), _ptr(out_path),
            _ptr(out_accept_len), _ptr(out_bonus_token), _stream_handle(stream))
    if st != 0:
        raise JakiroError(st, "jk_accept_path_greedy_static")


class PreparedCall:
    """A C-ABI call with its arguments marshalled once.  `launch()` issues exactly that one
    library call on the given (default: torch's current) stream: what a decoding loop, or a
    HIP-graph capture of it, calls per step.  Holds references to every tensor it points to."""

    def __init__(self, fn, where, args, stream_index, keep):
        self._fn, self._where, self._args, self._si, self._keep = fn, where, list(args), stream_index, keep

    def launch(self, stream=None) -> None:
        self._args[self._si] = _stream_handle(stream)
        st = self._fn(*self._args)
        if st != 0:
            raise JakiroError(st, self._where)


def prepare_tree_verify_attention(q, k_cache, v_cache, k_tree, v_tree, parent, prefix_len, out, workspace,
                                  max_prefix_len: Optional[int] = None, scale: float = 0.0) -> PreparedCall:
    """Same arguments as tree_verify_attention with out and workspace given; nothing is launched."""
    if k_cache is not None and k_cache.shape[1] == 0:
        k_cache = v_cache = None
    if max_prefix_len is None:
        max_prefix_len = 0 if k_cache is None else int(k_cache.shape[1])
    d = _make_desc(q, k_cache, k_tree, out, scale)
    args = [ctypes.byref(d), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_tree), _ptr(v_tree), _ptr(parent),
            _ptr(prefix_len), int(max_prefix_len), _ptr(out), _ptr(workspace),
            workspace.numel() * workspace.element_size(), None]
    return PreparedCall(lib().jk_tree_verify_attention, "jk_tree_verify_attention", args, 12,
                        (d, q, k_cache, v_cache, k_tree, v_tree, parent, prefix_len, out, workspace))


def _commit_args(k_tree, v_tree, k_cache, v_cache, path, accept_len, prefix_len, advance):
    import torch
    B, T, Hkv, D = k_tree.shape
    if k_tree.dtype == torch.bfloat16:
        dt = JK_BF16
    elif k_tree.dtype == torch.float32:
        dt = JK_F32
    else:
        raise TypeError("k_tree must be bfloat16 or float32")
    if v_tree.stride() != k_tree.stride() or v_cache.stride() != k_cache.stride():
        raise ValueError("K and V must share strides")
    for t in (k_tree, k_cache):
        if t.stride(-1) != 1 and t.shape[-1] > 1:
            raise ValueError("head_dim must be the contiguous innermost axis")
    d = AttnDesc(B, T, Hkv, Hkv, D, 0, 0, 0, k_cache.stride(0), k_cache.stride(1), k_cache.stride(2),
                 k_tree.stride(0), k_tree.stride(1), k_tree.stride(2), 0, 0, 0, 0.0, dt)
    return d, [_ptr(k_tree), _ptr(v_tree), _ptr(k_cache), _ptr(v_cache), _ptr(path), _ptr(accept_len),
               int(path.shape[1]), int(k_cache.shape[1]), _ptr(prefix_len), 1 if advance else 0]


def commit_path(k_tree, v_tree, k_cache, v_cache, path, accept_len, prefix_len, advance: bool = True,
                stream=None) -> None:
    """jk_commit_path: copies the K/V rows of the accepted nodes path[b][:accept_len[b]] to the cache
    positions prefix_len[b]..., in place; advances prefix_len (device int32 [B]) when `advance`."""
    d, args = _commit_args(k_tree, v_tree, k_cache, v_cache, path, accept_len, prefix_len, advance)
    st = lib().jk_commit_path(ctypes.byref(d), *args, _stream_handle(stream))
    if st != 0:
        raise JakiroError(st, "jk_commit_path")


def prepare_commit_path(k_tree, v_tree, k_cache, v_cache, path, accept_len, prefix_len,
                        advance: bool = True) -> "PreparedCall":
    """Same arguments as commit_path; nothing is launched."""
    d, args = _commit_args(k_tree, v_tree, k_cache, v_cache, path, accept_len, prefix_len, advance)
    return PreparedCall(lib().jk_commit_path, "jk_commit_path", [ctypes.byref(d)] + args + [None], 11,
                        (d, k_tree, v_tree, k_cache, v_cache, path, accept_len, prefix_len))


def prepare_commit_path_layers(k_trees, v_trees, k_caches, v_caches, path, accept_len, prefix_len,
                               advance: bool = True) -> "PreparedCall":
    """jk_commit_path_layers for lists of per-layer tensors (all of one shape, dtype and stride set): builds the
    device pointer tables once; `launch()` commits every layer with one call."""
    import torch
    n = len(k_trees)
    for ts in (k_trees, v_trees, k_caches, v_caches):
        if len(ts) != n or any(t.stride() != ts[0].stride() or t.shape != ts[0].shape for t in ts):
            raise ValueError("per-layer tensors must share shape and strides")
    d, args = _commit_args(k_trees[0], v_trees[0], k_caches[0], v_caches[0], path, accept_len, prefix_len, advance)
    tables = [torch.tensor([t.data_ptr() for t in ts], dtype=torch.int64, device=path.device)
              for ts in (k_trees, v_trees, k_caches, v_caches)]
    call_args = [ctypes.byref(d), n] + [_ptr(t) for t in tables] + args[4:] + [None]
    return PreparedCall(lib().jk_commit_path_layers, "jk_commit_path_layers", call_args, 12,
                        (d, tables, list(k_trees), list(v_trees), list(k_caches), list(v_caches), path, accept_len,
                         prefix_len))


def _paged(k_pool, block_table) -> PagedKV:
    """k_pool [n_pages, page_size, Hkv, D]; block_table int32 [B, max_blocks] on the device."""
    return PagedKV(block_table.data_ptr(), int(block_table.shape[1]), int(k_pool.shape[1]), int(k_pool.shape[0]),
                   int(k_pool.stride(0)))


def _paged_desc(q, k_pool, k_tree, out, scale):
    d = _make_desc(q, None, k_tree, out, scale)
    d.kc_stride_b, d.kc_stride_l, d.kc_stride_h = 0, k_pool.stride(1), k_pool.stride(2)
    return d


def prepare_tree_verify_attention_paged(q, k_pool, v_pool, block_table, k_tree, v_tree, parent, prefix_len, out,
                                        workspace, max_prefix_len: int, scale: float = 0.0) -> "PreparedCall":
    """jk_tree_verify_attention_paged with out and workspace given; nothing is launched.  k_pool, v_pool
    [n_pages, page_size, Hkv, D] (same strides), block_table int32 [B, max_blocks]."""
    if v_pool.stride() != k_pool.stride():
        raise ValueError("K and V pools must share strides")
    d = _paged_desc(q, k_pool, k_tree, out, scale)
    pg = _paged(k_pool, block_table)
    args = [ctypes.byref(d), ctypes.byref(pg), _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(k_tree), _ptr(v_tree),
            _ptr(parent), _ptr(prefix_len), int(max_prefix_len), _ptr(out), _ptr(workspace),
            workspace.numel() * workspace.element_size(), None]
    return PreparedCall(lib().jk_tree_verify_attention_paged, "jk_tree_verify_attention_paged", args, 13,
                        (d, pg, q, k_pool, v_pool, block_table, k_tree, v_tree, parent, prefix_len, out, workspace))


def tree_verify_attention_paged(q, k_pool, v_pool, block_table, k_tree, v_tree, parent, prefix_len,
                                max_prefix_len: int, scale: float = 0.0, out=None, workspace=None, stream=None):
    """jk_tree_verify_attention_paged; returns out [B,T,Hq,D] (allocated unless given)."""
    import torch
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        d = _paged_desc(q, k_pool, k_tree, out, scale)
        need = int(lib().jk_tree_verify_attention_workspace(ctypes.byref(d), int(max_prefix_len)))
        if need == 0:
            raise JakiroError(3, "jk_tree_verify_attention_workspace")
        workspace = _new_workspace(need, q.device, stream)
    prepare_tree_verify_attention_paged(q, k_pool, v_pool, block_table, k_tree, v_tree, parent, prefix_len, out,
                                        workspace, max_prefix_len, scale).launch(stream)
    return out


def prepare_commit_path_layers_paged(k_trees, v_trees, k_pools, v_pools, block_table, path, accept_len, prefix_len,
                                     advance: bool = True) -> "PreparedCall":
    """jk_commit_path_layers_paged for lists of per-layer tree tensors and page pools (one block table)."""
    import torch
    n = len(k_trees)
    for ts in (k_trees, v_trees, k_pools, v_pools):
        if len(ts) != n or any(t.stride() != ts[0].stride() or t.shape != ts[0].shape for t in ts):
            raise ValueError("per-layer tensors must share shape and strides")
    kt, kp = k_trees[0], k_pools[0]
    B, T, Hkv, D = kt.shape
    dt = JK_BF16 if kt.dtype == torch.bfloat16 else JK_F32
    d = AttnDesc(B, T, Hkv, Hkv, D, 0, 0, 0, 0, kp.stride(1), kp.stride(2), kt.stride(0), kt.stride(1), kt.stride(2),
                 0, 0, 0, 0.0, dt)
    pg = _paged(kp, block_table)
    tables = [torch.tensor([t.data_ptr() for t in ts], dtype=torch.int64, device=path.device)
              for ts in (k_trees, v_trees, k_pools, v_pools)]
    args = [ctypes.byref(d), ctypes.byref(pg), n] + [_ptr(t) for t in tables] + \
           [_ptr(path), _ptr(accept_len), int(path.shape[1]), _ptr(prefix_len), 1 if advance else 0, None]
    return PreparedCall(lib().jk_commit_path_layers_paged, "jk_commit_path_layers_paged", args, 12,
                        (d, pg, tables, list(k_trees), list(v_trees), list(k_pools), list(v_pools), block_table, path,
                         accept_len, prefix_len))


def prepare_accept_path(tree_tokens, parent, target_logits, mode, temperature, draft_probs, uniforms, out_path,
                        out_accept_len, out_bonus_token, workspace) -> PreparedCall:
    """Same arguments as accept_path with outputs and workspace given; nothing is launched."""
    B, N = tree_tokens.shape
    V = target_logits.shape[-1]
    args = [B, N, V, int(out_path.shape[1]), _ptr(tree_tokens), _ptr(parent), _ptr(target_logits), int(mode),
            float(temperature), _ptr(draft_probs), _ptr(uniforms), _ptr(out_path), _ptr(out_accept_len),
            _ptr(out_bonus_token), _ptr(workspace), workspace.numel() * workspace.element_size(), None]
    return PreparedCall(lib().jk_accept_path, "jk_accept_path", args, 16,
                        (tree_tokens, parent, target_logits, draft_probs, uniforms, out_path, out_accept_len,
                         out_bonus_token, workspace))


def _draft_heads_args(f_top, s_top, w_head, mode, temperature, top_k, alpha, beta, logits, draft_probs,
                      topk_tokens, topk_probs, workspace):
    import torch
    R, two, d = f_top.shape
    V = w_head.shape[0]
    if two != 2 or tuple(s_top.shape) != (R, 2) or w_head.shape[1] != d:
        raise ValueError("f_top [R,2,d], s_top [R,2], w_head [V,d]")
    for t in (f_top, w_head):
        if t.dtype != torch.bfloat16 or not t.is_contiguous():
            raise TypeError("f_top and w_head must be contiguous bfloat16")
    for t in (s_top, logits, draft_probs, topk_probs):
        if t is not None and (t.dtype != torch.float32 or not t.is_contiguous()):
            raise TypeError("s_top, logits, draft_probs and topk_probs must be contiguous float32")
    if topk_tokens.dtype != torch.int32 or not topk_tokens.is_contiguous():
        raise TypeError("topk_tokens must be contiguous int32")
    desc = DraftHeadsDesc(R, d, V, int(top_k), int(mode), float(temperature), float(alpha), float(beta))
    args = [ctypes.byref(desc), _ptr(f_top), _ptr(s_top), _ptr(w_head), _ptr(logits), _ptr(draft_probs),
            _ptr(topk_tokens), _ptr(topk_probs), _ptr(workspace), workspace.numel() * workspace.element_size(), None]
    return desc, args


def draft_heads_workspace(rows: int, d_model: int, vocab: int) -> int:
    return int(lib().jk_draft_heads_workspace(int(rows), int(d_model), int(vocab)))


def draft_heads(f_top, s_top, w_head, mode: int = JK_HEADS_DECOUPLED, temperature: float = 1.0, top_k: int = 10,
                alpha: float = 0.0, beta: float = 0.0, want_probs: bool = True, stream=None, out_probs=None):
    """jk_draft_heads.  f_top bf16 [R,2,d], s_top fp32 [R,2], w_head bf16 [V,d].
    Returns (logits [R,2,V], draft_probs [R,2,V] or None, topk_tokens [R,2,k] int32, topk_probs [R,2,k]).
    `out_probs` (contiguous fp32 [R,2,V], for instance rows of a round's table of draft distributions)
    receives the distributions instead of a new tensor."""
    import torch
    R, _, d = f_top.shape
    V = w_head.shape[0]
    dev = f_top.device
    logits = torch.empty((R, 2, V), dtype=torch.float32, device=dev)
    if out_probs is not None:
        if tuple(out_probs.shape) != (R, 2, V):
            raise ValueError("out_probs must be [R, 2, V]")
        probs = out_probs
    else:
        probs = torch.empty((R, 2, V), dtype=torch.float32, device=dev) if want_probs else None
    tk = torch.empty((R, 2, int(top_k)), dtype=torch.int32, device=dev)
    tp = torch.empty((R, 2, int(top_k)), dtype=torch.float32, device=dev)
    need = draft_heads_workspace(R, d, V)
    if need == 0:
        raise JakiroError(3, "jk_draft_heads_workspace")
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    desc, args = _draft_heads_args(f_top, s_top, w_head, mode, temperature, top_k, alpha, beta, logits, probs,
                                   tk, tp, ws)
    args[-1] = _stream_handle(stream)
    st = lib().jk_draft_heads(*args)
    if st != 0:
        raise JakiroError(st, "jk_draft_heads")
    return logits, probs, tk, tp


def prepare_draft_heads(f_top, s_top, w_head, mode, temperature, top_k, alpha, beta, logits, draft_probs,
                        topk_tokens, topk_probs, workspace) -> PreparedCall:
    """jk_draft_heads with outputs and workspace given; nothing is launched."""
    desc, args = _draft_heads_args(f_top, s_top, w_head, mode, temperature, top_k, alpha, beta, logits, draft_probs,
                                   topk_tokens, topk_probs, workspace)
    return PreparedCall(lib().jk_draft_heads, "jk_draft_heads", args, 10,
                        (desc, f_top, s_top, w_head, logits, draft_probs, topk_tokens, topk_probs, workspace))


def _moe_args(u, centroids, w_gate, w_up, w_down, f_top, s_top, expert_idx, f_mix, workspace):
    import torch
    R, d = u.shape
    N, F, d2 = w_gate.shape
    if d2 != d or tuple(centroids.shape) != (N, d) or tuple(w_up.shape) != (N, F, d) or tuple(w_down.shape) != (N, d, F):
        raise ValueError("u [R,d], centroids [N,d], w_gate/w_up [N,F,d], w_down [N,d,F]")
    for t in (u, centroids, w_gate, w_up, w_down, f_top, f_mix):
        if t is not None and (t.dtype != torch.bfloat16 or not t.is_contiguous()):
            raise TypeError("features and weights must be contiguous bfloat16")
    if s_top.dtype != torch.float32 or expert_idx.dtype != torch.int32:
        raise TypeError("s_top float32, expert_idx int32")
    desc = MoeDesc(R, d, F, N)
    need = int(lib().jk_moe_experts_workspace(ctypes.byref(desc)))
    if workspace is None:
        if need == 0:
            raise JakiroError(3, "jk_moe_experts_workspace")
        workspace = torch.empty(need, dtype=torch.uint8, device=u.device)
    args = [ctypes.byref(desc), _ptr(u), _ptr(centroids), _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(f_top),
            _ptr(s_top), _ptr(expert_idx), _ptr(f_mix), _ptr(workspace), workspace.numel() * workspace.element_size(),
            None]
    return desc, args, workspace


def moe_experts_workspace(rows: int, d_model: int, d_ff: int, n_experts: int) -> int:
    return int(lib().jk_moe_experts_workspace(ctypes.byref(MoeDesc(int(rows), int(d_model), int(d_ff), int(n_experts)))))


def moe_experts(u, centroids, w_gate, w_up, w_down, want_mix: bool = True, stream=None):
    """jk_moe_experts.  Returns (f_top [R,2,d] bf16, s_top [R,2], expert_idx [R,2] int32, f_mix [R,d] bf16 or None)."""
    import torch
    R, d = u.shape
    dev = u.device
    f_top = torch.empty((R, 2, d), dtype=torch.bfloat16, device=dev)
    s_top = torch.empty((R, 2), dtype=torch.float32, device=dev)
    idx = torch.empty((R, 2), dtype=torch.int32, device=dev)
    f_mix = torch.empty((R, d), dtype=torch.bfloat16, device=dev) if want_mix else None
    desc, args, ws = _moe_args(u, centroids, w_gate, w_up, w_down, f_top, s_top, idx, f_mix, None)
    args[-1] = _stream_handle(stream)
    st = lib().jk_moe_experts(*args)
    if st != 0:
        raise JakiroError(st, "jk_moe_experts")
    return f_top, s_top, idx, f_mix


def prepare_moe_experts(u, centroids, w_gate, w_up, w_down, f_top, s_top, expert_idx, f_mix, workspace) -> PreparedCall:
    """jk_moe_experts with outputs and workspace given; nothing is launched."""
    desc, args, ws = _moe_args(u, centroids, w_gate, w_up, w_down, f_top, s_top, expert_idx, f_mix, workspace)
    return PreparedCall(lib().jk_moe_experts, "jk_moe_experts", args, 12,
                        (desc, u, centroids, w_gate, w_up, w_down, f_top, s_top, expert_idx, f_mix, ws))


class TreeState:
    """Device arrays of a growing draft tree (jk_tree_state), one set per batch."""

    def __init__(self, batch: int, max_nodes: int, device="cuda"):
        import torch
        self.batch, self.max_nodes = int(batch), int(max_nodes)
        self.tokens = torch.zeros((batch, max_nodes), dtype=torch.int32, device=device)
        self.parent = torch.full((batch, max_nodes), -1, dtype=torch.int32, device=device)
        self.score = torch.zeros((batch, max_nodes), dtype=torch.float32, device=device)
        self.q_row = torch.zeros((batch, max_nodes), dtype=torch.int32, device=device)
        self.n_nodes = torch.zeros((batch,), dtype=torch.int32, device=device)

    def reset(self) -> None:
        self.n_nodes.zero_()

    def desc(self) -> TreeStateDesc:
        return TreeStateDesc(_ptr(self.tokens), _ptr(self.parent), _ptr(self.score), _ptr(self.q_row),
                             _ptr(self.n_nodes), self.max_nodes)


def tree_grow(state: TreeState, frontier_in, cand_tokens, cand_probs, width: int, q_row_base: int, stream=None):
    """jk_tree_grow.  frontier_in int32 [B,n_front] or None (root); cand_tokens int32 / cand_probs fp32
    [B*n_front,2,k].  Returns the next frontier, int32 [B,width]."""
    import torch
    B = state.batch
    n_front = 1 if frontier_in is None else int(frontier_in.shape[1])
    rows, two, k = cand_tokens.shape
    if rows != B * n_front or two != 2 or tuple(cand_probs.shape) != (rows, 2, k):
        raise ValueError("cand_tokens / cand_probs must be [B*n_front, 2, k]")
    if cand_tokens.dtype != torch.int32 or cand_probs.dtype != torch.float32 or \
            not cand_tokens.is_contiguous() or not cand_probs.is_contiguous():
        raise TypeError("cand_tokens contiguous int32, cand_probs contiguous float32")
    if frontier_in is not None and (frontier_in.dtype != torch.int32 or not frontier_in.is_contiguous()):
        raise TypeError("frontier_in contiguous int32")
    out = torch.empty((B, int(width)), dtype=torch.int32, device=cand_tokens.device)
    d = state.desc()
    st = lib().jk_tree_grow(ctypes.byref(d), B, n_front, int(k), int(width), int(q_row_base), _ptr(frontier_in),
                            _ptr(cand_tokens), _ptr(cand_probs), _ptr(out), _stream_handle(stream))
    if st != 0:
        raise JakiroError(st, "jk_tree_grow")
    return out


def tree_grow_tail(state: TreeState, frontier_in, cand_tokens, cand_probs, k1: int, k2: int, width: int,
                   q_row_base: int, stream=None) -> None:
    """jk_tree_grow_tail: children from head 0's lists, grandchildren from head 1's (contrastive mode)."""
    B = state.batch
    n_front = 1 if frontier_in is None else int(frontier_in.shape[1])
    rows, two, k = cand_tokens.shape
    if rows != B * n_front or two != 2 or tuple(cand_probs.shape) != (rows, 2, k):
        raise ValueError("cand_tokens / cand_probs must be [B*n_front, 2, k]")
    d = state.desc()
    st = lib().jk_tree_grow_tail(ctypes.byref(d), B, n_front, int(k), int(k1), int(k2), int(width), int(q_row_base),
                                 _ptr(frontier_in), _ptr(cand_tokens), _ptr(cand_probs), _stream_handle(stream))
    if st != 0:
        raise JakiroError(st, "jk_tree_grow_tail")


def tree_fill_static(state: TreeState, frontier_in, cand_tokens, cand_probs, shape_slot, shape_expert, shape_rank,
                     next_index, q_row_base: int, stream=None):
    """jk_tree_fill_static.  shape_* int32 [n_new] device tensors; next_index int32 [n_next] or None.
    Returns (frontier_out int32 [B,n_next] or None, new_ids int32 [B,n_new])."""
    import torch
    B = state.batch
    n_front = 1 if frontier_in is None else int(frontier_in.shape[1])
    rows, two, k = cand_tokens.shape
    if rows != B * n_front or two != 2 or tuple(cand_probs.shape) != (rows, 2, k):
        raise ValueError("cand_tokens / cand_probs must be [B*n_front, 2, k]")
    n_new = int(shape_slot.numel())
    n_next = 0 if next_index is None else int(next_index.numel())
    dev = cand_tokens.device
    new_ids = torch.empty((B, n_new), dtype=torch.int32, device=dev)
    out = torch.empty((B, n_next), dtype=torch.int32, device=dev) if n_next else None
    d = state.desc()
    st = lib().jk_tree_fill_static(ctypes.byref(d), B, n_front, int(k), int(q_row_base), _ptr(frontier_in),
                                   _ptr(cand_tokens), _ptr(cand_probs), _ptr(shape_slot), _ptr(shape_expert),
                                   _ptr(shape_rank), n_new, _ptr(next_index), n_next, _ptr(out), _ptr(new_ids),
                                   _stream_handle(stream))
    if st != 0:
        raise JakiroError(st, "jk_tree_fill_static")
    return out, new_ids


def tree_finalize(state: TreeState, n_keep: int, stream=None):
    """jk_tree_finalize.  Returns (tree_tokens, parent, q_row, old_index) int32 [B,n_keep] and n_valid int32 [B]."""
    import torch
    B = state.batch
    dev = state.tokens.device
    outs = [torch.empty((B, int(n_keep)), dtype=torch.int32, device=dev) for _ in range(4)]
    n_valid = torch.empty((B,), dtype=torch.int32, device=dev)
    d = state.desc()
    st = lib().jk_tree_finalize(ctypes.byref(d), B, int(n_keep), _ptr(outs[0]), _ptr(outs[1]), _ptr(outs[2]),
                                _ptr(outs[3]), _ptr(n_valid), _stream_handle(stream))
    if st != 0:
        raise JakiroError(st, "jk_tree_finalize")
    return outs[0], outs[1], outs[2], outs[3], n_valid


def gather_draft_probs(q_all, q_row, stream=None):
    """jk_gather_draft_probs.  q_all fp32 [n_rows, V] (contiguous), q_row int32 [B, N] -> fp32 [B, N, V]."""
    import torch
    if q_all.dtype != torch.float32 or not q_all.is_contiguous() or q_row.dtype != torch.int32 or \
            not q_row.is_contiguous():
        raise TypeError("q_all contiguous float32, q_row contiguous int32")
    V = q_all.shape[-1]
    n_rows = q_all.numel() // V
    B, N = q_row.shape
    out = torch.empty((B, N, V), dtype=torch.float32, device=q_all.device)
    st = lib().jk_gather_draft_probs(B, N, V, _ptr(q_all), n_rows, _ptr(q_row), _ptr(out), _stream_handle(stream))
    if st != 0:
        raise JakiroError(st, "jk_gather_draft_probs")
    return out


def linear(x, w, residual=None, out_dtype=None, stream=None):
    """jk_linear: x bf16 [m,k], w bf16 [n,k], residual bf16 [m,n] or None -> x @ w.T (+ residual) as bf16
    (default) or float32 (out_dtype=torch.float32)."""
    import torch
    m, k = x.shape
    n = w.shape[0]
    for t in (x, w, residual):
        if t is not None and (t.dtype != torch.bfloat16 or not t.is_contiguous()):
            raise TypeError("x, w and residual must be contiguous bfloat16")
    if w.shape[1] != k or (residual is not None and tuple(residual.shape) != (m, n)):
        raise ValueError("x [m,k], w [n,k], residual [m,n]")
    f32 = out_dtype == torch.float32
    out = torch.empty((m, n), dtype=torch.float32 if f32 else torch.bfloat16, device=x.device)
    need = int(lib().jk_linear_workspace(m, n, k))
    if need == 0:
        raise JakiroError(3, "jk_linear_workspace")
    ws = torch.empty(need, dtype=torch.uint8, device=x.device)
    st = lib().jk_linear(m, n, k, _ptr(x), _ptr(w), _ptr(residual), None if f32 else _ptr(out),
                         _ptr(out) if f32 else None, _ptr(ws), need, _stream_handle(stream))
    if st != 0:
        raise JakiroError(st, "jk_linear")
    return out


def accept_path_rows(tree_tokens, parent, target_logits, q_all, q_row, uniforms, temperature: float = 1.0,
                     max_depth: Optional[int] = None, workspace=None, stream=None):
    """jk_accept_path_rows (speculative sampling): like accept_path, with node k of sequence b tested against
    q_all[q_row[b, k]] (q_all fp32 [n_rows, V] contiguous, q_row int32 [B, N]) instead of a dense draft_probs."""
    import torch
    B, N = tree_tokens.shape
    V = target_logits.shape[-1]
    if max_depth is None:
        max_depth = N
    for t in (tree_tokens, parent, q_row):
        if t.dtype != torch.int32 or not t.is_contiguous():
            raise TypeError("tree_tokens, parent and q_row must be contiguous int32")
    for t in (target_logits, q_all, uniforms):
        if t.dtype != torch.float32 or not t.is_contiguous():
            raise TypeError("logits, q_all and uniforms must be contiguous float32")
    if q_all.shape[-1] != V or tuple(q_row.shape) != (B, N):
        raise ValueError("q_all [n_rows, V], q_row [B, N]")
    dev = tree_tokens.device
    path = torch.empty((B, max_depth), dtype=torch.int32, device=dev)
    alen = torch.empty((B,), dtype=torch.int32, device=dev)
    bonus = torch.empty((B,), dtype=torch.int32, device=dev)
    need = accept_path_workspace(B, N, V, JK_SAMPLE)
    if workspace is None:
        workspace = _new_workspace(need, dev, stream)
    st = lib().jk_accept_path_rows(B, N, V, int(max_depth), _ptr(tree_tokens), _ptr(parent), _ptr(target_logits),
                                   JK_SAMPLE, float(temperature), _ptr(q_all), q_all.numel() // V, _ptr(q_row),
                                   _ptr(uniforms), _ptr(path), _ptr(alen), _ptr(bonus), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if st != 0:
        raise JakiroError(st, "jk_accept_path_rows")
    return path, alen, bonus
