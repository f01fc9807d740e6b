"""Thin ctypes binding of libapbv.so: argument marshalling only.

Every step of the hot path runs inside the HIP library; PyTorch is used here for device memory and
for the current HIP stream.  If the library has not been built the calls raise -- there is no
fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libapbv.so")
_lib = None


class ApbvError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {status_string(code)} ({code})")
        self.code = code


class ApbvTensor(ctypes.Structure):
    """Mirror of ``apbv_tensor`` in include/apbv.h."""
    _fields_ = [
        ("ptr", ctypes.c_void_p),
        ("tokens", ctypes.c_int64),
        ("stride_token", ctypes.c_int64),
        ("stride_head", ctypes.c_int64),
        ("stride_batch", ctypes.c_int64),
    ]


class ApbvAttentionItem(ctypes.Structure):
    """Mirror of ``apbv_attention_item`` in include/apbv.h."""
    _fields_ = [
        ("q_local", ApbvTensor),
        ("k_anchor", ApbvTensor), ("v_anchor", ApbvTensor),
        ("k_pass", ApbvTensor), ("v_pass", ApbvTensor),
        ("k_local", ApbvTensor), ("v_local", ApbvTensor),
        ("out", ctypes.c_void_p),
        ("lse_out", ctypes.c_void_p),
    ]


def load_library() -> ctypes.CDLL:
    """Load libapbv.so (built in-tree by ``paper_2601_21444_amd.build``); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: build the HIP library first (python -m paper_2601_21444_amd.build). "
            "There is no CPU or PyTorch fallback for the APB-V hot path.")
    lib = ctypes.CDLL(_LIB_PATH)
    lib.apbv_status_string.restype = ctypes.c_char_p
    lib.apbv_status_string.argtypes = [ctypes.c_int]
    lib.apbv_version.restype = ctypes.c_int
    lib.apbv_version.argtypes = []
    lib.apbv_compress_workspace_bytes.restype = ctypes.c_size_t
    lib.apbv_compress_workspace_bytes.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int64]
    lib.apbv_compress_kv.restype = ctypes.c_int
    lib.apbv_compress_kv.argtypes = [
        ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
        ApbvTensor, ApbvTensor, ApbvTensor, ctypes.c_int64,
        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.apbv_compress_kv_noalloc.restype = ctypes.c_int
    lib.apbv_compress_kv_noalloc.argtypes = list(lib.apbv_compress_kv.argtypes[:12]) + [ctypes.c_void_p]
    lib.apbv_compress_reduced_workspace_bytes.restype = ctypes.c_size_t
    lib.apbv_compress_reduced_workspace_bytes.argtypes = [
        ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64]
    lib.apbv_compress_kv_reduced.restype = ctypes.c_int
    lib.apbv_compress_kv_reduced.argtypes = [ctypes.c_int, ctypes.c_float] + list(lib.apbv_compress_kv.argtypes)
    lib.apbv_host_attention.restype = ctypes.c_int
    lib.apbv_host_attention.argtypes = [
        ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
        ApbvTensor, ApbvTensor, ApbvTensor, ApbvTensor, ApbvTensor, ApbvTensor, ApbvTensor,
        ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    lib.apbv_merge_lse.restype = ctypes.c_int
    lib.apbv_merge_lse.argtypes = [
        ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
        ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    lib.apbv_query_attention_workspace_bytes.restype = ctypes.c_size_t
    lib.apbv_query_attention_workspace_bytes.argtypes = [
        ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int]
    lib.apbv_query_attention.restype = ctypes.c_int
    lib.apbv_query_attention.argtypes = [
        ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
        ApbvTensor, ApbvTensor, ApbvTensor, ApbvTensor, ApbvTensor, ApbvTensor, ApbvTensor,
        ctypes.c_float, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.apbv_host_attention_group.restype = ctypes.c_int
    lib.apbv_host_attention_group.argtypes = [
        ctypes.c_int, ctypes.POINTER(ApbvAttentionItem), ctypes.c_int, ctypes.c_int, ctypes.c_int,
        ctypes.c_float, ctypes.c_void_p]
    _lib = lib
    return lib


def status_string(code: int) -> str:
    return load_library().apbv_status_string(int(code)).decode()


def apbv_version() -> int:
    return int(load_library().apbv_version())


def apbv_compress_workspace_bytes(batch: int, n_kv_heads: int, head_dim: int, L: int, l_p: int) -> int:
    return int(load_library().apbv_compress_workspace_bytes(batch, n_kv_heads, head_dim, L, l_p))


def tensor_view(t: torch.Tensor) -> Tuple[ApbvTensor, int]:
    """``[tokens, heads, d]`` or ``[batch, tokens, heads, d]`` bf16 tensor -> (apbv_tensor, batch)."""
    if t.dtype != torch.bfloat16:
        raise TypeError("expected a bfloat16 tensor")
    if t.dim() == 3:
        t = t.unsqueeze(0)
    if t.dim() != 4:
        raise ValueError("expected [tokens, heads, d] or [batch, tokens, heads, d]")
    if t.shape[1] > 0 and t.stride(3) != 1:
        raise ValueError("head_dim must be contiguous")
    b, n, _, _ = t.shape
    view = ApbvTensor(t.data_ptr() if n > 0 else None, n, t.stride(1), t.stride(2), t.stride(0))
    return view, b


def _check_buffer(t: Optional[torch.Tensor], name: str, dtype: torch.dtype, shape, device) -> None:
    """A caller-supplied output or workspace must be a dense device tensor of the right type holding at least the
    elements the library will write (``shape``: the dense shape, or a minimum element count) -- its pointer goes to
    the C ABI unchecked beyond that."""
    if t is None:
        return
    need = int(shape) if isinstance(shape, int) else int(torch.Size(shape).numel())
    if not isinstance(t, torch.Tensor) or t.dtype != dtype:
        raise TypeError(f"{name}: expected a {dtype} tensor")
    if not t.is_cuda or t.device != device:
        raise ValueError(f"{name}: must live on {device}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    if t.numel() < need:
        raise ValueError(f"{name}: holds {t.numel()} elements, {need} are written")


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


REDUCERS = {"sum": 0, "max": 1, "softmax_sum": 2}


def apbv_compress_reduced_workspace_bytes(reducer: str, batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
                                          n_q: int, L: int, l_p: int) -> int:
    return int(load_library().apbv_compress_reduced_workspace_bytes(REDUCERS[reducer], batch, n_q_heads, n_kv_heads,
                                                                    head_dim, n_q, L, l_p))


def apbv_compress_kv(q_probe: torch.Tensor, k_local: torch.Tensor, v_local: torch.Tensor, l_p: int, *,
                     reducer: str = "sum", softmax_scale: float = 0.0,
                     return_scores: bool = False, workspace: Optional[torch.Tensor] = None,
                     idx_out: Optional[torch.Tensor] = None, k_c_out: Optional[torch.Tensor] = None,
                     v_c_out: Optional[torch.Tensor] = None, scores_out: Optional[torch.Tensor] = None,
                     stream: Optional[torch.cuda.Stream] = None):
    """Compressed block (idx, K_c, V_c[, scores]) of one context block; see apbv_compress_kv in
    include/apbv.h.  Tensors are ``[tokens, heads, d]`` or batched ``[batch, tokens, heads, d]``.  A ``reducer``
    other than "sum" ("max", "softmax_sum") goes through apbv_compress_kv_reduced."""
    lib = load_library()
    batched = k_local.dim() == 4
    qv, bq = tensor_view(q_probe)
    kv, b = tensor_view(k_local)
    vv, bv = tensor_view(v_local)
    if not (bq == b == bv):
        raise ValueError("batch sizes differ")
    hq, d = q_probe.shape[-2], q_probe.shape[-1]
    hkv, L = k_local.shape[-2], k_local.shape[-3]
    dev = k_local.device
    _check_buffer(idx_out, "idx_out", torch.int32, (b, hkv, l_p), dev)
    _check_buffer(k_c_out, "k_c_out", torch.bfloat16, (b, l_p, hkv, d), dev)
    _check_buffer(v_c_out, "v_c_out", torch.bfloat16, (b, l_p, hkv, d), dev)
    _check_buffer(scores_out, "scores_out", torch.float64, (b, hkv, L), dev)
    _check_buffer(workspace, "workspace", torch.uint8, 0, dev)
    if idx_out is None:
        idx_out = torch.empty((b, hkv, l_p), dtype=torch.int32, device=dev)
    if k_c_out is None:
        k_c_out = torch.empty((b, l_p, hkv, d), dtype=torch.bfloat16, device=dev)
    if v_c_out is None:
        v_c_out = torch.empty((b, l_p, hkv, d), dtype=torch.bfloat16, device=dev)
    if return_scores and scores_out is None:
        scores_out = torch.empty((b, hkv, L), dtype=torch.float64, device=dev)
    if workspace is None:
        nbytes = max(apbv_compress_reduced_workspace_bytes(reducer, b, hq, hkv, d, q_probe.shape[-3], L, l_p), 256)
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    entry = lib.apbv_compress_kv if reducer == "sum" else lib.apbv_compress_kv_reduced
    lead = () if reducer == "sum" else (REDUCERS[reducer], float(softmax_scale))
    st = entry(
        *lead, b, hq, hkv, d, qv, kv, vv, int(l_p),
        idx_out.data_ptr() if l_p > 0 else None, k_c_out.data_ptr() if l_p > 0 else None,
        v_c_out.data_ptr() if l_p > 0 else None,
        scores_out.data_ptr() if scores_out is not None else None,
        workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    if st != 0:
        raise ApbvError(st, "apbv_compress_kv")
    if not batched:
        idx_out, k_c_out, v_c_out = idx_out[0], k_c_out[0], v_c_out[0]
        scores_out = scores_out[0] if scores_out is not None else None
    if return_scores:
        return idx_out, k_c_out, v_c_out, scores_out
    return idx_out, k_c_out, v_c_out


NOALLOC_MAX_WORKSPACE_BYTES = 4194304      # APBV_NOALLOC_MAX_WORKSPACE_BYTES of include/apbv.h


def apbv_compress_kv_noalloc(q_probe: torch.Tensor, k_local: torch.Tensor, v_local: torch.Tensor, l_p: int, *,
                             idx_out: torch.Tensor, k_c_out: torch.Tensor, v_c_out: torch.Tensor,
                             scores_out: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None):
    """apbv_compress_kv without a workspace (the library's static scratch array) and without any allocation here
    either: the caller passes every output.  See apbv_compress_kv_noalloc in include/apbv.h."""
    lib = load_library()
    qv, bq = tensor_view(q_probe)
    kv, b = tensor_view(k_local)
    vv, bv = tensor_view(v_local)
    if not (bq == b == bv):
        raise ValueError("batch sizes differ")
    hq, d = q_probe.shape[-2], q_probe.shape[-1]
    hkv, L = k_local.shape[-2], k_local.shape[-3]
    dev = k_local.device
    _check_buffer(idx_out, "idx_out", torch.int32, (b, hkv, l_p), dev)
    _check_buffer(k_c_out, "k_c_out", torch.bfloat16, (b, l_p, hkv, d), dev)
    _check_buffer(v_c_out, "v_c_out", torch.bfloat16, (b, l_p, hkv, d), dev)
    _check_buffer(scores_out, "scores_out", torch.float64, (b, hkv, L), dev)
    st = lib.apbv_compress_kv_noalloc(
        b, hq, hkv, d, qv, kv, vv, int(l_p),
        idx_out.data_ptr() if l_p > 0 else None, k_c_out.data_ptr() if l_p > 0 else None,
        v_c_out.data_ptr() if l_p > 0 else None,
        scores_out.data_ptr() if scores_out is not None else None, _stream_ptr(stream))
    if st != 0:
        raise ApbvError(st, "apbv_compress_kv_noalloc")
    return idx_out, k_c_out, v_c_out


def apbv_host_attention(q_local: torch.Tensor, k_anchor: torch.Tensor, v_anchor: torch.Tensor,
                        k_pass: torch.Tensor, v_pass: torch.Tensor, k_local: torch.Tensor, v_local: torch.Tensor,
                        softmax_scale: float, *, return_lse: bool = False, out: Optional[torch.Tensor] = None,
                        lse_out: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None):
    """Fused host attention over [anchor | passing | local(causal)]; see apbv_host_attention in
    include/apbv.h.  Returns ``out [.., L, Hq, d]`` bf16 (and ``lse [.., Hq, L]`` fp32)."""
    lib = load_library()
    batched = q_local.dim() == 4
    views = []
    b = None
    for t in (q_local, k_anchor, v_anchor, k_pass, v_pass, k_local, v_local):
        view, bt = tensor_view(t)
        if b is None:
            b = bt
        elif bt != b:
            raise ValueError("batch sizes differ")
        views.append(view)
    L, hq, d = q_local.shape[-3], q_local.shape[-2], q_local.shape[-1]
    hkv = k_anchor.shape[-2]
    dev = q_local.device
    _check_buffer(out, "out", torch.bfloat16, (b, L, hq, d), dev)
    _check_buffer(lse_out, "lse_out", torch.float32, (b, hq, L), dev)
    if out is None:
        out = torch.empty((b, L, hq, d), dtype=torch.bfloat16, device=dev)
    if return_lse and lse_out is None:
        lse_out = torch.empty((b, hq, L), dtype=torch.float32, device=dev)
    st = lib.apbv_host_attention(b, hq, hkv, d, *views, float(softmax_scale), out.data_ptr(),
                                 lse_out.data_ptr() if lse_out is not None else None, _stream_ptr(stream))
    if st != 0:
        raise ApbvError(st, "apbv_host_attention")
    if not batched:
        out = out[0] if out.dim() == 4 else out
        lse_out = lse_out[0] if (lse_out is not None and lse_out.dim() == 3) else lse_out
    return (out, lse_out) if return_lse else out


def apbv_host_attention_group(problems, softmax_scale: float, *, return_lse: bool = False,
                              stream: Optional[torch.cuda.Stream] = None):
    """Several unbatched attention problems in one launch; see apbv_host_attention_group in include/apbv.h.
    ``problems`` is a sequence of ``(q_local, k_anchor, v_anchor, k_pass, v_pass, k_local, v_local)`` tuples of
    ``[tokens, heads, d]`` tensors (optionally followed by preallocated ``out`` and ``lse_out``).  Returns the list of
    outputs (of ``(out, lse)`` pairs with ``return_lse``)."""
    lib = load_library()
    n = len(problems)
    items = (ApbvAttentionItem * max(n, 1))()
    results = []
    hq = hkv = d = 0
    for m, prob in enumerate(problems):
        tensors = prob[:7]
        out = prob[7] if len(prob) > 7 else None
        lse = prob[8] if len(prob) > 8 else None
        views = []
        for t in tensors:
            if t.dim() != 3:
                raise ValueError("group problems are unbatched [tokens, heads, d] tensors")
            views.append(tensor_view(t)[0])
        q = tensors[0]
        L, hq_m, d_m = q.shape
        hkv_m = tensors[1].shape[-2]
        if m == 0:
            hq, hkv, d = hq_m, hkv_m, d_m
        elif (hq_m, hkv_m, d_m) != (hq, hkv, d):
            raise ValueError("all problems of a group share the head counts and head_dim")
        _check_buffer(out, "out", torch.bfloat16, (L, hq, d), q.device)
        _check_buffer(lse, "lse_out", torch.float32, (hq, L), q.device)
        if out is None:
            out = torch.empty((L, hq, d), dtype=torch.bfloat16, device=q.device)
        if return_lse and lse is None:
            lse = torch.empty((hq, L), dtype=torch.float32, device=q.device)
        it = items[m]
        (it.q_local, it.k_anchor, it.v_anchor, it.k_pass, it.v_pass, it.k_local, it.v_local) = views
        it.out = out.data_ptr()
        it.lse_out = lse.data_ptr() if lse is not None else None
        results.append((out, lse) if return_lse else out)
    st = lib.apbv_host_attention_group(n, items, hq, hkv, d, float(softmax_scale), _stream_ptr(stream))
    if st != 0:
        raise ApbvError(st, "apbv_host_attention_group")
    return results


def apbv_query_attention_workspace_bytes(batch: int, n_q_heads: int, head_dim: int, n_q: int, n_keys: int,
                                         n_splits: int = 0) -> int:
    return int(load_library().apbv_query_attention_workspace_bytes(batch, n_q_heads, head_dim, n_q, n_keys, n_splits))


def apbv_query_attention(q_block: torch.Tensor, k_anchor: torch.Tensor, v_anchor: torch.Tensor,
                         k_pass: torch.Tensor, v_pass: torch.Tensor, k_local: torch.Tensor, v_local: torch.Tensor,
                         softmax_scale: float, *, n_splits: int = 0, return_lse: bool = False,
                         out: Optional[torch.Tensor] = None, lse_out: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None):
    """Attention of a short query block with the key axis split over workgroups; see apbv_query_attention in
    include/apbv.h.  Same tensors and results as :func:`apbv_host_attention`."""
    lib = load_library()
    batched = q_block.dim() == 4
    views = []
    b = None
    for t in (q_block, k_anchor, v_anchor, k_pass, v_pass, k_local, v_local):
        view, bt = tensor_view(t)
        if b is None:
            b = bt
        elif bt != b:
            raise ValueError("batch sizes differ")
        views.append(view)
    n_q, hq, d = q_block.shape[-3], q_block.shape[-2], q_block.shape[-1]
    hkv = k_anchor.shape[-2]
    n_keys = k_anchor.shape[-3] + k_pass.shape[-3] + k_local.shape[-3]
    dev = q_block.device
    _check_buffer(out, "out", torch.bfloat16, (b, n_q, hq, d), dev)
    _check_buffer(lse_out, "lse_out", torch.float32, (b, hq, n_q), dev)
    _check_buffer(workspace, "workspace", torch.uint8, 0, dev)
    if out is None:
        out = torch.empty((b, n_q, hq, d), dtype=torch.bfloat16, device=dev)
    if return_lse and lse_out is None:
        lse_out = torch.empty((b, hq, n_q), dtype=torch.float32, device=dev)
    if workspace is None:
        nbytes = apbv_query_attention_workspace_bytes(b, hq, d, n_q, max(n_keys, 1), n_splits)
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
    st = lib.apbv_query_attention(b, hq, hkv, d, *views, float(softmax_scale), int(n_splits), out.data_ptr(),
                                  lse_out.data_ptr() if lse_out is not None else None,
                                  workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                  _stream_ptr(stream))
    if st != 0:
        raise ApbvError(st, "apbv_query_attention")
    if not batched:
        out = out[0] if out.dim() == 4 else out
        lse_out = lse_out[0] if (lse_out is not None and lse_out.dim() == 3) else lse_out
    return (out, lse_out) if return_lse else out


def apbv_merge_lse(parts_out: torch.Tensor, parts_lse: torch.Tensor, *, return_lse: bool = False,
                   out: Optional[torch.Tensor] = None, lse_out: Optional[torch.Tensor] = None,
                   stream: Optional[torch.cuda.Stream] = None):
    """Merge partial attention results; see apbv_merge_lse in include/apbv.h.
    ``parts_out [n_parts, rows, Hq, d]`` bf16 (parts may be strided along dim 0), ``parts_lse [n_parts, Hq, rows]``
    fp32.  Returns ``out [rows, Hq, d]`` bf16 (and ``lse [Hq, rows]`` fp32)."""
    lib = load_library()
    if parts_out.dtype != torch.bfloat16 or parts_lse.dtype != torch.float32:
        raise TypeError("expected bfloat16 partial outputs and float32 log-sum-exps")
    n, rows, hq, d = parts_out.shape
    if parts_lse.shape != (n, hq, rows):
        raise ValueError("parts_lse must be [n_parts, Hq, rows]")
    if not parts_out[0].is_contiguous() or not parts_lse[0].is_contiguous():
        raise ValueError("each part must be dense")
    _check_buffer(out, "out", torch.bfloat16, (rows, hq, d), parts_out.device)
    _check_buffer(lse_out, "lse_out", torch.float32, (hq, rows), parts_out.device)
    if out is None:
        out = torch.empty((rows, hq, d), dtype=torch.bfloat16, device=parts_out.device)
    if return_lse and lse_out is None:
        lse_out = torch.empty((hq, rows), dtype=torch.float32, device=parts_out.device)
    st = lib.apbv_merge_lse(n, rows, hq, d, parts_out.data_ptr(), parts_out.stride(0), parts_lse.data_ptr(),
                            parts_lse.stride(0), out.data_ptr(), lse_out.data_ptr() if lse_out is not None else None,
                            _stream_ptr(stream))
    if st != 0:
        raise ApbvError(st, "apbv_merge_lse")
    return (out, lse_out) if return_lse else out
