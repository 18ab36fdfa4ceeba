"""ctypes binding of include/hydra_attn.h.  Argument marshalling only: tensors in, raw device
pointers and sizes out; every step of the computation runs in the HIP kernels.  There is no
fallback: if the shared library is missing, loading raises."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libhydra_attn.so")
_lib = None

HYDRA_OK = 0


class HydraError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {hydra_status_string(status)} (status {status})")


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """dlopen the in-tree library.  Raises if it has not been built (python -m paper_2505_12658_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2505_12658_amd.build`; "
                              "there is no CPU or PyTorch fallback for this library")
        lib = ctypes.CDLL(_LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        lib.hydra_attn_varlen_fwd.restype = ctypes.c_int
        lib.hydra_attn_varlen_fwd.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, i32, i32, i32, i32, i32, i32, i32, ctypes.c_float,
                                              vp, sz, vp]
        lib.hydra_attn_varlen_fwd_prebuilt.restype = ctypes.c_int
        lib.hydra_attn_varlen_fwd_prebuilt.argtypes = lib.hydra_attn_varlen_fwd.argtypes
        lib.hydra_attn_varlen_fwd_shared.restype = ctypes.c_int
        lib.hydra_attn_varlen_fwd_shared.argtypes = lib.hydra_attn_varlen_fwd.argtypes[:-1] + [i32, vp]
        lib.hydra_attn_varlen_fwd_static.restype = ctypes.c_int
        lib.hydra_attn_varlen_fwd_static.argtypes = lib.hydra_attn_varlen_fwd.argtypes[:-3] + [vp]
        lib.hydra_attn_build_worklist.restype = ctypes.c_int
        lib.hydra_attn_build_worklist.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, vp, sz, vp]
        lib.hydra_kv_cache_write.restype = ctypes.c_int
        lib.hydra_kv_cache_write.argtypes = [vp, vp, i64, i64, vp, vp, vp, i32, i32, i32, i32, i64, vp]
        lib.hydra_attn_paged_fwd.restype = ctypes.c_int
        lib.hydra_attn_paged_fwd.argtypes = [vp, vp, i64, vp, vp, vp, i32, vp, vp, i32, i32, i32, i32, i32, i32, i32, i64, ctypes.c_float, vp, sz, vp]
        lib.hydra_attn_paged_workspace_bytes.restype = sz
        lib.hydra_attn_paged_workspace_bytes.argtypes = [i32] * 5
        lib.hydra_page_cache_write.restype = ctypes.c_int
        lib.hydra_page_cache_write.argtypes = [vp, i64, vp, vp, i32, i32, i64, vp]
        lib.hydra_page_cache_gather.restype = ctypes.c_int
        lib.hydra_page_cache_gather.argtypes = [vp, vp, vp, i64, i32, i32, i64, vp]
        lib.hydra_attn_workspace_bytes.restype = sz
        lib.hydra_attn_workspace_bytes.argtypes = [i32] * 6
        lib.hydra_status_string.restype = ctypes.c_char_p
        lib.hydra_status_string.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def hydra_status_string(status: int) -> str:
    return load_library().hydra_status_string(int(status)).decode()


def hydra_attn_workspace_bytes(batch: int, total_tokens: int, max_seqlen: int, n_q_heads: int, n_kv_heads: int, head_dim: int) -> int:
    return int(load_library().hydra_attn_workspace_bytes(batch, total_tokens, max_seqlen, n_q_heads, n_kv_heads, head_dim))


def hydra_attn_paged_workspace_bytes(batch: int, n_kv_heads: int, head_dim: int, max_blocks_per_seq: int, block_size: int) -> int:
    return int(load_library().hydra_attn_paged_workspace_bytes(batch, n_kv_heads, head_dim, max_blocks_per_seq, block_size))


def _stream_handle(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _check_token_major(t: torch.Tensor, name: str):
    if t.dtype != torch.bfloat16 or t.dim() != 3 or not t.is_cuda:
        raise TypeError(f"{name} must be a CUDA bf16 tensor [tokens, heads, head_dim]")
    if t.stride(2) != 1 or t.stride(1) != t.shape[2]:
        raise ValueError(f"{name}: head_dim must be contiguous and the head stride must equal head_dim")


def hydra_attn_varlen_fwd(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cu_seqlens: torch.Tensor, max_seqlen: int, causal: bool,
                          softmax_scale: float, out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                          stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """q [N, Hq, d], k/v [N, Hkv, d] bf16 (token-strided views allowed), cu_seqlens int32 [B+1] on the device."""
    lib = load_library()
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _check_token_major(t, n)
    if cu_seqlens.dtype != torch.int32 or not cu_seqlens.is_cuda or not cu_seqlens.is_contiguous():
        raise TypeError("cu_seqlens must be a contiguous CUDA int32 tensor")
    N, Hq, d = q.shape
    Hkv = k.shape[1]
    batch = cu_seqlens.numel() - 1
    if out is None:
        out = torch.empty((N, Hq, d), dtype=torch.bfloat16, device=q.device)
    elif not out.is_contiguous() or out.shape != (N, Hq, d) or out.dtype != torch.bfloat16:
        raise ValueError("out must be a contiguous bf16 tensor shaped like q")
    need = hydra_attn_workspace_bytes(batch, N, max_seqlen, Hq, Hkv, d)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    rc = lib.hydra_attn_varlen_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), q.stride(0), k.stride(0), v.stride(0),
                                   cu_seqlens.data_ptr(), batch, N, int(max_seqlen), Hq, Hkv, d, int(bool(causal)), float(softmax_scale),
                                   workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if rc != HYDRA_OK:
        raise HydraError(rc, "hydra_attn_varlen_fwd")
    return out


def hydra_attn_varlen_fwd_static(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cu_seqlens: torch.Tensor, max_seqlen: int, causal: bool,
                                 softmax_scale: float, out: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """hydra_attn_varlen_fwd with the work list in the library's own static device array: nothing is allocated,
    here or in the library, so `out` is the caller's."""
    lib = load_library()
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _check_token_major(t, n)
    if cu_seqlens.dtype != torch.int32 or not cu_seqlens.is_cuda or not cu_seqlens.is_contiguous():
        raise TypeError("cu_seqlens must be a contiguous CUDA int32 tensor")
    N, Hq, d = q.shape
    if not out.is_contiguous() or out.shape != (N, Hq, d) or out.dtype != torch.bfloat16:
        raise ValueError("out must be a contiguous bf16 tensor shaped like q")
    rc = lib.hydra_attn_varlen_fwd_static(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), q.stride(0), k.stride(0), v.stride(0),
                                          cu_seqlens.data_ptr(), cu_seqlens.numel() - 1, N, int(max_seqlen), Hq, k.shape[1], d,
                                          int(bool(causal)), float(softmax_scale), _stream_handle(stream))
    if rc != HYDRA_OK:
        raise HydraError(rc, "hydra_attn_varlen_fwd_static")
    return out


def hydra_attn_build_worklist(cu_seqlens: torch.Tensor, total_tokens: int, max_seqlen: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
                              causal: bool, workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Builds the tile work list for one packed batch into `workspace` (allocated if None) and returns it."""
    lib = load_library()
    if cu_seqlens.dtype != torch.int32 or not cu_seqlens.is_cuda or not cu_seqlens.is_contiguous():
        raise TypeError("cu_seqlens must be a contiguous CUDA int32 tensor")
    batch = cu_seqlens.numel() - 1
    if workspace is None:
        need = hydra_attn_workspace_bytes(batch, total_tokens, max_seqlen, n_q_heads, n_kv_heads, head_dim)
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=cu_seqlens.device)
    rc = lib.hydra_attn_build_worklist(cu_seqlens.data_ptr(), batch, int(total_tokens), int(max_seqlen), n_q_heads, n_kv_heads, head_dim,
                                       int(bool(causal)), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                       _stream_handle(stream))
    if rc != HYDRA_OK:
        raise HydraError(rc, "hydra_attn_build_worklist")
    return workspace


def hydra_attn_varlen_fwd_prebuilt(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cu_seqlens: torch.Tensor, max_seqlen: int,
                                   causal: bool, softmax_scale: float, out: torch.Tensor, workspace: torch.Tensor,
                                   stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Attention against a work list built earlier by hydra_attn_build_worklist for the same batch."""
    lib = load_library()
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _check_token_major(t, n)
    N, Hq, d = q.shape
    if not out.is_contiguous() or out.shape != (N, Hq, d) or out.dtype != torch.bfloat16:
        raise ValueError("out must be a contiguous bf16 tensor shaped like q")
    rc = lib.hydra_attn_varlen_fwd_prebuilt(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), q.stride(0), k.stride(0),
                                            v.stride(0), cu_seqlens.data_ptr(), cu_seqlens.numel() - 1, N, int(max_seqlen), Hq,
                                            k.shape[1], d, int(bool(causal)), float(softmax_scale), workspace.data_ptr(),
                                            workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if rc != HYDRA_OK:
        raise HydraError(rc, "hydra_attn_varlen_fwd_prebuilt")
    return out


def hydra_attn_varlen_fwd_shared(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cu_seqlens: torch.Tensor, max_seqlen: int,
                                 causal: bool, softmax_scale: float, out: torch.Tensor, workspace: torch.Tensor, workgroups_per_cu: int,
                                 stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """hydra_attn_varlen_fwd_prebuilt with at most `workgroups_per_cu` persistent workgroups per compute unit, for a caller
    that runs another kernel beside it on a second stream."""
    lib = load_library()
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _check_token_major(t, n)
    N, Hq, d = q.shape
    if not out.is_contiguous() or out.shape != (N, Hq, d) or out.dtype != torch.bfloat16:
        raise ValueError("out must be a contiguous bf16 tensor shaped like q")
    rc = lib.hydra_attn_varlen_fwd_shared(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), q.stride(0), k.stride(0),
                                          v.stride(0), cu_seqlens.data_ptr(), cu_seqlens.numel() - 1, N, int(max_seqlen), Hq,
                                          k.shape[1], d, int(bool(causal)), float(softmax_scale), workspace.data_ptr(),
                                          workspace.numel() * workspace.element_size(), int(workgroups_per_cu), _stream_handle(stream))
    if rc != HYDRA_OK:
        raise HydraError(rc, "hydra_attn_varlen_fwd_shared")
    return out


def hydra_kv_cache_write(k: torch.Tensor, v: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor, slot_mapping: torch.Tensor,
                         stream: Optional[torch.cuda.Stream] = None) -> None:
    """k/v [N, Hkv, d] bf16; caches [num_blocks, block_size, Hkv, d] bf16 contiguous; slot_mapping int64 [N]."""
    lib = load_library()
    for t, n in ((k, "k"), (v, "v")):
        _check_token_major(t, n)
    if k_cache.dim() != 4 or not k_cache.is_contiguous() or not v_cache.is_contiguous() or k_cache.shape != v_cache.shape:
        raise ValueError("caches must be contiguous [num_blocks, block_size, n_kv_heads, head_dim] of equal shape")
    if k_cache.dtype != torch.bfloat16 or v_cache.dtype != torch.bfloat16 or not k_cache.is_cuda:
        raise TypeError("caches must be CUDA bf16 tensors")
    if slot_mapping.dtype != torch.int64 or not slot_mapping.is_cuda or not slot_mapping.is_contiguous():
        raise TypeError("slot_mapping must be a contiguous CUDA int64 tensor")
    N, Hkv, d = k.shape
    if slot_mapping.numel() != N or tuple(k_cache.shape[2:]) != (Hkv, d) or v.shape != k.shape:
        raise ValueError("shape mismatch between k/v, caches and slot_mapping")
    rc = lib.hydra_kv_cache_write(k.data_ptr(), v.data_ptr(), k.stride(0), v.stride(0), k_cache.data_ptr(), v_cache.data_ptr(),
                                  slot_mapping.data_ptr(), N, Hkv, d, k_cache.shape[1], k_cache.shape[0], _stream_handle(stream))
    if rc != HYDRA_OK:
        raise HydraError(rc, "hydra_kv_cache_write")


def hydra_attn_paged_fwd(q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor, block_tables: torch.Tensor,
                         cu_seqlens_q: torch.Tensor, kv_lens: torch.Tensor, max_q_len: int, softmax_scale: float,
                         out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, use_workspace: bool = True,
                         stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """q [Nq, Hq, d] bf16 (new tokens of all requests, packed); caches [num_blocks, block_size, Hkv, d] bf16 contiguous;
    block_tables int32 [B, max_blocks_per_seq]; cu_seqlens_q int32 [B+1]; kv_lens int32 [B] (context lengths, new tokens included).
    workspace: uint8 tensor for the split of decode contexts over workgroups (allocated at the size the library asks for when
    None and use_workspace; use_workspace=False runs without splitting)."""
    lib = load_library()
    _check_token_major(q, "q")
    if k_cache.dim() != 4 or not k_cache.is_contiguous() or not v_cache.is_contiguous() or k_cache.shape != v_cache.shape:
        raise ValueError("caches must be contiguous [num_blocks, block_size, n_kv_heads, head_dim] of equal shape")
    if k_cache.dtype != torch.bfloat16 or v_cache.dtype != torch.bfloat16 or not k_cache.is_cuda:
        raise TypeError("caches must be CUDA bf16 tensors")
    for t, n in ((block_tables, "block_tables"), (cu_seqlens_q, "cu_seqlens_q"), (kv_lens, "kv_lens")):
        if t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous():
            raise TypeError(f"{n} must be a contiguous CUDA int32 tensor")
    Nq, Hq, d = q.shape
    batch = cu_seqlens_q.numel() - 1
    if block_tables.dim() != 2 or block_tables.shape[0] != batch or kv_lens.numel() != batch or k_cache.shape[3] != d:
        raise ValueError("shape mismatch between q, caches, block_tables, cu_seqlens_q and kv_lens")
    if out is None:
        out = torch.empty((Nq, Hq, d), dtype=torch.bfloat16, device=q.device)
    elif not out.is_contiguous() or out.shape != (Nq, Hq, d) or out.dtype != torch.bfloat16:
        raise ValueError("out must be a contiguous bf16 tensor shaped like q")
    if workspace is None and use_workspace:
        need = hydra_attn_paged_workspace_bytes(batch, k_cache.shape[2], d, block_tables.shape[1], k_cache.shape[1])
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device) if need else None
    ws_ptr, ws_bytes = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) if workspace is not None else (None, 0)
    rc = lib.hydra_attn_paged_fwd(q.data_ptr(), out.data_ptr(), q.stride(0), k_cache.data_ptr(), v_cache.data_ptr(), block_tables.data_ptr(),
                                  block_tables.shape[1], cu_seqlens_q.data_ptr(), kv_lens.data_ptr(), batch, Nq, int(max_q_len), Hq,
                                  k_cache.shape[2], d, k_cache.shape[1], k_cache.shape[0], float(softmax_scale), ws_ptr, ws_bytes,
                                  _stream_handle(stream))
    if rc != HYDRA_OK:
        raise HydraError(rc, "hydra_attn_paged_fwd")
    return out


def _check_page_cache(rows: torch.Tensor, cache: torch.Tensor, slot_mapping: torch.Tensor):
    if rows.dtype != torch.bfloat16 or rows.dim() != 2 or not rows.is_cuda or rows.stride(1) != 1:
        raise TypeError("rows must be a CUDA bf16 matrix with contiguous rows")
    if cache.dtype != torch.bfloat16 or not cache.is_cuda or not cache.is_contiguous() or cache.shape[-1] != rows.shape[1]:
        raise TypeError("cache must be a contiguous CUDA bf16 tensor [..., row_elems]")
    if slot_mapping.dtype != torch.int64 or not slot_mapping.is_cuda or not slot_mapping.is_contiguous() or slot_mapping.numel() != rows.shape[0]:
        raise TypeError("slot_mapping must be a contiguous CUDA int64 tensor with one entry per row")


def hydra_page_cache_write(rows: torch.Tensor, cache: torch.Tensor, slot_mapping: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
    """rows [n, row_elems] bf16 (row-strided view allowed) -> cache [pages, page_rows, row_elems] at slot_mapping (int64 [n], < 0 skips)."""
    _check_page_cache(rows, cache, slot_mapping)
    rc = load_library().hydra_page_cache_write(rows.data_ptr(), rows.stride(0), cache.data_ptr(), slot_mapping.data_ptr(), rows.shape[0],
                                               rows.shape[1], cache.numel() // rows.shape[1], _stream_handle(stream))
    if rc != HYDRA_OK:
        raise HydraError(rc, "hydra_page_cache_write")


def hydra_page_cache_gather(cache: torch.Tensor, slot_mapping: torch.Tensor, rows: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
    """cache rows at slot_mapping -> rows [n, row_elems] bf16 (row-strided view allowed); rows with a negative slot keep their contents."""
    _check_page_cache(rows, cache, slot_mapping)
    rc = load_library().hydra_page_cache_gather(cache.data_ptr(), slot_mapping.data_ptr(), rows.data_ptr(), rows.stride(0), rows.shape[0],
                                                rows.shape[1], cache.numel() // rows.shape[1], _stream_handle(stream))
    if rc != HYDRA_OK:
        raise HydraError(rc, "hydra_page_cache_gather")
