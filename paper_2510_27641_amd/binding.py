"""Thin ctypes binding of libspecattn.so: argument marshalling only.

Tensors are torch tensors on the GPU (torch is used for device memory and
streams, nothing else); every step of the path runs inside the library's
kernels.  There is no CPU fallback: a missing library is an error.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspecattn.so")

OK, EINVAL, ESHAPE, EALIGN, EWORKSPACE, EUNSUPPORTED, EHIP = 0, -1, -2, -3, -4, -5, -6
ROW_INVALID, ROW_NEAR_BOUNDARY, ROW_OVERFLOW = 1, 2, 4
SEL_BLOCK = 1024
F32, BF16, F16 = 0, 1, 2

EXPORTS = ("specattn_topp_select", "specattn_topp_select_union", "specattn_union_workspace_size", "specattn_sparse_decode_attn", "specattn_sparse_decode_attn_static", "specattn_fused",
           "specattn_workspace_size", "specattn_layer_similarity", "specattn_layer_similarity_workspace_size",
           "specattn_layer_map", "specattn_layer_map_workspace_size", "specattn_check_lists", "specattn_lists_to_csr", "specattn_stream_read", "specattn_init", "specattn_last_error", "specattn_version")


class SelectArgs(C.Structure):
    _fields_ = [
        ("probs", C.c_void_p), ("probs_stride_b", C.c_int64), ("probs_stride_h", C.c_int64),
        ("B", C.c_int32), ("H_kv", C.c_int32), ("n_max", C.c_int32),
        ("seq_lens", C.c_void_p), ("top_p", C.c_float),
        ("indices", C.c_void_p), ("idx_stride_row", C.c_int64), ("idx_capacity", C.c_int32),
        ("counts", C.c_void_p), ("thresholds", C.c_void_p), ("row_flags", C.c_void_p),
        ("page_table", C.c_void_p), ("page_size", C.c_int32), ("max_pages_per_seq", C.c_int32),
        ("emit_physical", C.c_int32),
        ("block_counts", C.c_void_p), ("reuse_selection", C.c_int32),
        ("chunk_size", C.c_int32), ("bisect_iters", C.c_int32),
        ("kept_mask", C.c_void_p),
    ]


class AttnArgs(C.Structure):
    _fields_ = [
        ("q", C.c_void_p), ("k", C.c_void_p), ("v", C.c_void_p), ("dtype", C.c_int),
        ("B", C.c_int32), ("H_q", C.c_int32), ("H_kv", C.c_int32), ("T", C.c_int32),
        ("d", C.c_int32), ("n_max", C.c_int32), ("sm_scale", C.c_float),
        ("q_stride_b", C.c_int64), ("q_stride_h", C.c_int64), ("q_stride_t", C.c_int64),
        ("kv_stride_b", C.c_int64), ("kv_stride_h", C.c_int64), ("kv_stride_n", C.c_int64),
        ("page_table", C.c_void_p), ("page_size", C.c_int32), ("max_pages_per_seq", C.c_int32),
        ("kv_stride_page", C.c_int64),
        ("seq_lens", C.c_void_p),
        ("indices", C.c_void_p), ("idx_stride_row", C.c_int64), ("counts", C.c_void_p),
        ("idx_capacity", C.c_int32), ("indices_are_physical", C.c_int32),
        ("out", C.c_void_p), ("lse", C.c_void_p),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
        ("k_new", C.c_void_p), ("v_new", C.c_void_p),
        ("chunk_size", C.c_int32),
        ("out_lowp", C.c_void_p),
    ]


class UnionArgs(C.Structure):
    _fields_ = [
        ("probs", C.c_void_p), ("probs_stride_b", C.c_int64), ("probs_stride_row", C.c_int64),
        ("B", C.c_int32), ("H_draft", C.c_int32), ("S", C.c_int32), ("H_kv", C.c_int32), ("n_max", C.c_int32),
        ("seq_lens", C.c_void_p), ("top_p", C.c_float),
        ("indices", C.c_void_p), ("idx_stride_row", C.c_int64), ("idx_capacity", C.c_int32),
        ("counts", C.c_void_p), ("row_flags", C.c_void_p),
        ("member_thresholds", C.c_void_p), ("member_counts", C.c_void_p),
        ("page_table", C.c_void_p), ("page_size", C.c_int32), ("max_pages_per_seq", C.c_int32),
        ("emit_physical", C.c_int32),
    ]


class SpecAttnError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"specattn status {status}: {text}")
        self.status = status


_lib = None


def load() -> C.CDLL:
    """Load libspecattn.so (built by `python -m paper_2510_27641_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2510_27641_amd.build`")
        lib = C.CDLL(LIB_PATH)
        lib.specattn_topp_select.restype = C.c_int
        lib.specattn_topp_select.argtypes = [C.POINTER(SelectArgs), C.c_void_p, C.c_size_t, C.c_void_p]
        lib.specattn_topp_select_union.restype = C.c_int
        lib.specattn_topp_select_union.argtypes = [C.POINTER(UnionArgs), C.c_void_p, C.c_size_t, C.c_void_p]
        lib.specattn_union_workspace_size.restype = C.c_size_t
        lib.specattn_union_workspace_size.argtypes = [C.POINTER(UnionArgs)]
        lib.specattn_sparse_decode_attn.restype = C.c_int
        lib.specattn_sparse_decode_attn.argtypes = [C.POINTER(AttnArgs), C.c_void_p]
        lib.specattn_sparse_decode_attn_static.restype = C.c_int
        lib.specattn_sparse_decode_attn_static.argtypes = [C.POINTER(AttnArgs), C.c_void_p]
        lib.specattn_fused.restype = C.c_int
        lib.specattn_fused.argtypes = [C.POINTER(SelectArgs), C.POINTER(AttnArgs), C.c_void_p]
        lib.specattn_workspace_size.restype = C.c_size_t
        lib.specattn_workspace_size.argtypes = [C.POINTER(SelectArgs), C.POINTER(AttnArgs)]
        lib.specattn_layer_similarity_workspace_size.restype = C.c_size_t
        lib.specattn_layer_similarity_workspace_size.argtypes = [C.c_int32] * 4
        lib.specattn_layer_similarity.restype = C.c_int
        lib.specattn_layer_similarity.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                                  C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        lib.specattn_layer_map_workspace_size.restype = C.c_size_t
        lib.specattn_layer_map_workspace_size.argtypes = [C.c_int32] * 2
        lib.specattn_layer_map.restype = C.c_int
        lib.specattn_layer_map.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_size_t, C.c_void_p]
        lib.specattn_check_lists.restype = C.c_int
        lib.specattn_check_lists.argtypes = [C.POINTER(AttnArgs), C.c_int64, C.c_void_p, C.c_void_p]
        lib.specattn_stream_read.restype = C.c_int
        lib.specattn_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        lib.specattn_lists_to_csr.restype = C.c_int
        lib.specattn_lists_to_csr.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.specattn_init.restype = C.c_int
        lib.specattn_init.argtypes = []
        lib.specattn_last_error.restype = C.c_char_p
        lib.specattn_last_error.argtypes = []
        lib.specattn_version.restype = C.c_int
        lib.specattn_version.argtypes = []
        _lib = lib
    return _lib


def last_error() -> str:
    return load().specattn_last_error().decode()


def _check(status: int):
    if status != OK:
        raise SpecAttnError(status, last_error())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


# ------------------------------------------------------------------------------------------
# argument structs from tensors
# ------------------------------------------------------------------------------------------
def select_args(probs: torch.Tensor, top_p: float, *, indices: Optional[torch.Tensor],
                counts: torch.Tensor, thresholds: Optional[torch.Tensor] = None,
                row_flags: Optional[torch.Tensor] = None, seq_lens: Optional[torch.Tensor] = None,
                page_table: Optional[torch.Tensor] = None, page_size: int = 0,
                emit_physical: bool = False, block_counts: Optional[torch.Tensor] = None,
                reuse_selection: bool = False, chunk_size: int = 0,
                bisect_iters: int = 0, kept_mask: Optional[torch.Tensor] = None) -> SelectArgs:
    """probs [B,H_kv,n] fp32 (last dim contiguous); indices [B*H_kv, cap] int32."""
    assert probs.dtype == torch.float32 and probs.dim() == 3 and probs.stride(2) == 1
    B, H, n = probs.shape
    a = SelectArgs()
    a.probs = probs.data_ptr()
    a.probs_stride_b, a.probs_stride_h = probs.stride(0), probs.stride(1)
    a.B, a.H_kv, a.n_max = B, H, n
    a.seq_lens = None if seq_lens is None else seq_lens.data_ptr()
    a.top_p = top_p
    if indices is not None:
        assert indices.dtype == torch.int32 and indices.dim() == 2 and indices.stride(1) == 1
        a.indices = indices.data_ptr()
        a.idx_stride_row, a.idx_capacity = indices.stride(0), indices.shape[1]
    a.counts = counts.data_ptr()
    a.thresholds = None if thresholds is None else thresholds.data_ptr()
    a.row_flags = None if row_flags is None else row_flags.data_ptr()
    if page_table is not None:
        assert page_table.dtype == torch.int32 and page_table.is_contiguous()
        a.page_table = page_table.data_ptr()
        a.page_size, a.max_pages_per_seq = page_size, page_table.shape[1]
    a.emit_physical = int(emit_physical)
    if block_counts is not None:
        assert block_counts.dtype == torch.int32 and block_counts.is_contiguous()
        a.block_counts = block_counts.data_ptr()
    a.reuse_selection = int(reuse_selection)
    a.chunk_size = chunk_size
    a.bisect_iters = bisect_iters
    if kept_mask is not None:
        assert kept_mask.dtype == torch.int32 and kept_mask.is_contiguous()
        assert kept_mask.numel() == B * H * ((n + SEL_BLOCK - 1) // SEL_BLOCK) * (SEL_BLOCK // 32)
        a.kept_mask = kept_mask.data_ptr()
    return a


def union_args(probs: torch.Tensor, top_p: float, H_kv: int, *, indices: torch.Tensor, counts: torch.Tensor,
               row_flags: Optional[torch.Tensor] = None, seq_lens: Optional[torch.Tensor] = None,
               member_thresholds: Optional[torch.Tensor] = None, member_counts: Optional[torch.Tensor] = None,
               page_table: Optional[torch.Tensor] = None, page_size: int = 0,
               emit_physical: bool = False) -> UnionArgs:
    """probs [B,H_draft,S,n] fp32 with the (head, step) rows evenly spaced; indices [B*H_kv, cap] int32."""
    assert probs.dtype == torch.float32 and probs.dim() == 4 and probs.stride(3) == 1
    B, H_d, S, n = probs.shape
    assert probs.stride(1) == S * probs.stride(2), "rows (head, step) must be evenly spaced"
    a = UnionArgs()
    a.probs = probs.data_ptr()
    a.probs_stride_b, a.probs_stride_row = probs.stride(0), probs.stride(2)
    a.B, a.H_draft, a.S, a.H_kv, a.n_max = B, H_d, S, H_kv, n
    a.seq_lens = None if seq_lens is None else seq_lens.data_ptr()
    a.top_p = top_p
    assert indices.dtype == torch.int32 and indices.dim() == 2 and indices.stride(1) == 1
    a.indices = indices.data_ptr()
    a.idx_stride_row, a.idx_capacity = indices.stride(0), indices.shape[1]
    a.counts = counts.data_ptr()
    a.row_flags = None if row_flags is None else row_flags.data_ptr()
    a.member_thresholds = None if member_thresholds is None else member_thresholds.data_ptr()
    a.member_counts = None if member_counts is None else member_counts.data_ptr()
    if page_table is not None:
        assert page_table.dtype == torch.int32 and page_table.is_contiguous()
        a.page_table = page_table.data_ptr()
        a.page_size, a.max_pages_per_seq = page_size, page_table.shape[1]
    a.emit_physical = int(emit_physical)
    return a


def attn_args(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, *, out: torch.Tensor,
              indices: Optional[torch.Tensor] = None, counts: Optional[torch.Tensor] = None,
              lse: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
              n_max: Optional[int] = None, sm_scale: float = 0.0,
              page_table: Optional[torch.Tensor] = None, page_size: int = 0,
              indices_are_physical: bool = False, seq_lens: Optional[torch.Tensor] = None,
              k_new: Optional[torch.Tensor] = None, v_new: Optional[torch.Tensor] = None,
              chunk_size: int = 0, out_lowp: Optional[torch.Tensor] = None) -> AttnArgs:
    """q [B,H_q,T,d]; contiguous k/v [B,H_kv,n,d]; paged k/v pool [pages,H_kv,page_size,d];
    k_new/v_new [B,H_kv,T,d] contiguous (the new tokens behind the cache), optional."""
    assert q.dim() == 4 and k.dim() == 4 and k.shape == v.shape and k.stride() == v.stride()
    assert q.dtype == k.dtype == v.dtype and q.dtype in (torch.float32, torch.bfloat16, torch.float16)
    assert q.stride(3) == 1 and k.stride(3) == 1
    B, H_q, T, d = q.shape
    paged = page_table is not None or indices_are_physical
    a = AttnArgs()
    a.q, a.k, a.v = q.data_ptr(), k.data_ptr(), v.data_ptr()
    a.dtype = {torch.bfloat16: BF16, torch.float16: F16, torch.float32: F32}[q.dtype]
    a.B, a.H_q, a.H_kv, a.T, a.d = B, H_q, k.shape[1], T, d
    a.sm_scale = sm_scale
    a.q_stride_b, a.q_stride_h, a.q_stride_t = q.stride(0), q.stride(1), q.stride(2)
    if paged:
        a.n_max = int(n_max if n_max is not None else
                      (page_table.shape[1] * page_size if page_table is not None else 0))
        a.kv_stride_page, a.kv_stride_h, a.kv_stride_n = k.stride(0), k.stride(1), k.stride(2)
        a.kv_stride_b = 0
        a.page_size = page_size
        if page_table is not None:
            assert page_table.dtype == torch.int32 and page_table.is_contiguous()
            a.page_table = page_table.data_ptr()
            a.max_pages_per_seq = page_table.shape[1]
    else:
        a.n_max = k.shape[2] if n_max is None else n_max
        a.kv_stride_b, a.kv_stride_h, a.kv_stride_n = k.stride(0), k.stride(1), k.stride(2)
    a.seq_lens = None if seq_lens is None else seq_lens.data_ptr()
    if indices is not None:
        assert indices.dtype == torch.int32 and indices.dim() == 2 and indices.stride(1) == 1
        a.indices = indices.data_ptr()
        a.idx_stride_row, a.idx_capacity = indices.stride(0), indices.shape[1]
    a.counts = None if counts is None else counts.data_ptr()
    a.indices_are_physical = int(indices_are_physical)
    assert out.dtype == torch.float32 and out.is_contiguous() and tuple(out.shape) == (B, H_q, T, d)
    a.out = out.data_ptr()
    a.lse = None if lse is None else lse.data_ptr()
    a.chunk_size = chunk_size
    if out_lowp is not None:
        assert out_lowp.dtype == q.dtype and out_lowp.is_contiguous() and tuple(out_lowp.shape) == (B, H_q, T, d)
        a.out_lowp = out_lowp.data_ptr()
    if k_new is not None:
        assert v_new is not None and k_new.dtype == v_new.dtype == q.dtype
        assert k_new.is_contiguous() and v_new.is_contiguous()
        assert tuple(k_new.shape) == tuple(v_new.shape) == (B, a.H_kv, T, d)
        a.k_new, a.v_new = k_new.data_ptr(), v_new.data_ptr()
    if workspace is not None:
        a.workspace, a.workspace_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    return a


# ------------------------------------------------------------------------------------------
# the three entry points (same names as the C ABI)
# ------------------------------------------------------------------------------------------
def specattn_workspace_size(sel: Optional[SelectArgs], attn: Optional[AttnArgs]) -> int:
    return int(load().specattn_workspace_size(None if sel is None else C.byref(sel),
                                              None if attn is None else C.byref(attn)))


def specattn_topp_select(sel: SelectArgs, workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().specattn_topp_select(C.byref(sel), _ptr(workspace), nbytes, _stream(stream)))


def specattn_union_workspace_size(args: UnionArgs) -> int:
    return int(load().specattn_union_workspace_size(C.byref(args)))


def specattn_topp_select_union(args: UnionArgs, workspace: torch.Tensor, stream=None) -> None:
    nbytes = workspace.numel() * workspace.element_size()
    _check(load().specattn_topp_select_union(C.byref(args), _ptr(workspace), nbytes, _stream(stream)))


def specattn_sparse_decode_attn(attn: AttnArgs, stream=None) -> None:
    _check(load().specattn_sparse_decode_attn(C.byref(attn), _stream(stream)))


def specattn_sparse_decode_attn_static(attn: AttnArgs, stream=None) -> None:
    """The same call on the library's built-in scratch buffer: allocates nothing, ignores attn.workspace."""
    _check(load().specattn_sparse_decode_attn_static(C.byref(attn), _stream(stream)))


def specattn_layer_similarity(attn_draft: torch.Tensor, attn_verifier: torch.Tensor, S: torch.Tensor,
                              workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """attn_draft [m, rows, L], attn_verifier [n, rows, L] fp32 contiguous; S [m, n] fp64 (out)."""
    assert attn_draft.dtype == attn_verifier.dtype == torch.float32 and S.dtype == torch.float64
    assert attn_draft.is_contiguous() and attn_verifier.is_contiguous() and S.is_contiguous()
    m, rows, L = attn_draft.shape
    n = attn_verifier.shape[0]
    assert tuple(attn_verifier.shape[1:]) == (rows, L) and tuple(S.shape) == (m, n)
    ws = workspace if workspace is not None else alloc_workspace(int(load().specattn_layer_similarity_workspace_size(m, n, rows, L)))
    _check(load().specattn_layer_similarity(_ptr(attn_draft), _ptr(attn_verifier), m, n, rows, L, _ptr(S), _ptr(ws),
                                            ws.numel(), _stream(stream)))


def specattn_layer_map(S: torch.Tensor, f: torch.Tensor, total: torch.Tensor, workspace: Optional[torch.Tensor] = None,
                       stream=None) -> None:
    """S [m, n] fp64 contiguous; f [n] int32 (out); total [1] fp64 (out)."""
    assert S.dtype == torch.float64 and S.is_contiguous() and S.dim() == 2
    m, n = S.shape
    assert f.dtype == torch.int32 and f.numel() == n and total.dtype == torch.float64 and total.numel() == 1
    ws = workspace if workspace is not None else alloc_workspace(int(load().specattn_layer_map_workspace_size(m, n)))
    _check(load().specattn_layer_map(_ptr(S), m, n, _ptr(f), _ptr(total), _ptr(ws), ws.numel(), _stream(stream)))


def specattn_fused(sel: SelectArgs, attn: AttnArgs, stream=None) -> None:
    _check(load().specattn_fused(C.byref(sel), C.byref(attn), _stream(stream)))


def specattn_lists_to_csr(indices: Optional[torch.Tensor], counts: torch.Tensor, indptr: torch.Tensor,
                          packed: Optional[torch.Tensor] = None, capacity: Optional[int] = None, stream=None) -> None:
    """indptr [rows + 1] int64 <- exclusive prefix of the list lengths; packed (optional) <- the lists back to back."""
    assert counts.dtype == torch.int32 and indptr.dtype == torch.int64 and indptr.numel() == counts.numel() + 1
    stride = 0 if indices is None else indices.stride(0)
    cap = capacity if capacity is not None else (indices.shape[1] if indices is not None else 2 ** 31 - 1)
    _check(load().specattn_lists_to_csr(_ptr(indices), stride, cap, _ptr(counts), counts.numel(), _ptr(indptr), _ptr(packed),
                                        _stream(stream)))


def specattn_init() -> None:
    """One-time set-up of the current device (kernel attributes); needed only before capturing a first call."""
    _check(load().specattn_init())


def specattn_check_lists(attn: AttnArgs, n_bad: torch.Tensor, pool_slots: int = 0, stream=None) -> None:
    """Counts the index-list violations of an attention call into n_bad (int32 device tensor of one element)."""
    assert n_bad.dtype == torch.int32 and n_bad.numel() == 1
    _check(load().specattn_check_lists(C.byref(attn), pool_slots, _ptr(n_bad), _stream(stream)))


def specattn_stream_read(src: torch.Tensor, sink: Optional[torch.Tensor] = None, stream=None) -> None:
    """Plain read of every byte of `src` (contiguous); the caller times it."""
    assert src.is_contiguous()
    _check(load().specattn_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream(stream)))


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    """A 256-byte aligned device buffer of at least nbytes (torch's allocator aligns to 512)."""
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
