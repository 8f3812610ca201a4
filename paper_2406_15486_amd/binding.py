"""ctypes binding of the C ABI declared in include/sa.h.

Same names as the C entry points.  Tensors are torch CUDA tensors (device
memory only); the current torch stream is passed to the library.  There is no
fallback: if the shared library is missing the import of any entry point
raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libsampleattn.so"

SA_OUT_BF16, SA_OUT_F32 = 0, 1
SA_OP_SAMPLE_SCORES, SA_OP_SELECT_STRIPS, SA_OP_SPARSE_ATTN, SA_OP_DENSE_ATTN = 0, 1, 2, 3
SA_OP_BLOCK_SPARSE_ATTN = 4
SA_OP_SAMPLE_SCORES_MIN = 5


class SaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = load_library().sa_status_string(status).decode()
        super().__init__(f"{where}: {msg} (status {status})")


class _CShape(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("seq_len", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("causal", ctypes.c_int32),
                ("softmax_scale", ctypes.c_float)]


class _CPartition(ctypes.Structure):
    _fields_ = [("heads_per_pass", ctypes.c_int32), ("n_query_segments", ctypes.c_int32)]


class _CSampling(ctypes.Structure):
    _fields_ = [("n_sample_rows", ctypes.c_int32), ("n_chunks", ctypes.c_int32),
                ("granularity", ctypes.c_int32)]


@dataclass(frozen=True)
class Shape:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    seq_len: int
    head_dim: int = 128
    causal: int = 1
    softmax_scale: float = 0.0

    def c(self) -> _CShape:
        return _CShape(self.batch, self.n_q_heads, self.n_kv_heads, self.seq_len,
                       self.head_dim, self.causal, self.softmax_scale)

    @property
    def n_bh(self) -> int:
        return self.batch * self.n_q_heads


_lib = None


def lib_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


def load_library() -> ctypes.CDLL:
    """Load the in-tree shared library; raise loudly if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is missing: build it first (python -m paper_2406_15486_amd.build "
            "or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(path)
    vp, i32p, f32p = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
    lib.sa_workspace_bytes.restype = ctypes.c_size_t
    lib.sa_workspace_bytes.argtypes = [ctypes.c_int, ctypes.POINTER(_CShape), ctypes.POINTER(_CSampling)]
    lib.sa_rows_from_ratio.restype = ctypes.c_int32
    lib.sa_rows_from_ratio.argtypes = [ctypes.c_int32, ctypes.c_float]
    lib.sa_sample_scores.restype = ctypes.c_int
    lib.sa_sample_scores.argtypes = [ctypes.POINTER(_CShape), ctypes.POINTER(_CSampling), vp, vp,
                                     f32p, f32p, f32p, vp, ctypes.c_size_t, vp]
    lib.sa_select_strips.restype = ctypes.c_int
    lib.sa_select_strips.argtypes = [ctypes.POINTER(_CShape), f32p, f32p, ctypes.c_float, ctypes.c_float,
                                     i32p, i32p, i32p, i32p, vp, ctypes.c_size_t, vp]
    lib.sa_sparse_attn.restype = ctypes.c_int
    lib.sa_sparse_attn.argtypes = [ctypes.POINTER(_CShape), vp, vp, vp, i32p, i32p, i32p, i32p,
                                   ctypes.c_int32, vp, ctypes.c_int, f32p, vp, vp, ctypes.c_size_t, vp]
    lib.sa_block_scores.restype = ctypes.c_int
    lib.sa_block_scores.argtypes = [ctypes.POINTER(_CShape), ctypes.c_int32, f32p, f32p, f32p, f32p, vp]
    lib.sa_select_blocks.restype = ctypes.c_int
    lib.sa_select_blocks.argtypes = [ctypes.POINTER(_CShape), ctypes.c_int32, f32p, f32p, ctypes.c_float,
                                     ctypes.c_float, i32p, i32p, i32p, i32p, vp, ctypes.c_size_t, vp]
    lib.sa_block_sparse_attn.restype = ctypes.c_int
    lib.sa_block_sparse_attn.argtypes = [ctypes.POINTER(_CShape), ctypes.c_int32, vp, vp, vp, i32p, i32p, i32p, i32p,
                                         ctypes.c_int32, vp, ctypes.c_int, f32p, vp, vp, ctypes.c_size_t, vp]
    lib.sa_select_chunked.restype = ctypes.c_int
    lib.sa_select_chunked.argtypes = [ctypes.POINTER(_CShape), ctypes.POINTER(_CSampling), f32p, f32p,
                                      ctypes.c_float, ctypes.c_float, i32p, i32p, i32p, i32p, vp,
                                      ctypes.c_size_t, vp]
    lib.sa_sparse_attn_chunked.restype = ctypes.c_int
    lib.sa_sparse_attn_chunked.argtypes = [ctypes.POINTER(_CShape), ctypes.POINTER(_CSampling), vp, vp, vp,
                                           i32p, i32p, i32p, i32p, ctypes.c_int32, vp, ctypes.c_int, f32p, vp,
                                           vp, ctypes.c_size_t, vp]
    lib.sa_dense_attn.restype = ctypes.c_int
    lib.sa_dense_attn.argtypes = [ctypes.POINTER(_CShape), vp, vp, vp, vp, ctypes.c_int, f32p,
                                  vp, ctypes.c_size_t, vp]
    lib.sa_partitioned_workspace_bytes.restype = ctypes.c_size_t
    lib.sa_partitioned_workspace_bytes.argtypes = [ctypes.POINTER(_CShape), ctypes.POINTER(_CPartition)]
    lib.sa_sparse_attn_partitioned.restype = ctypes.c_int
    lib.sa_sparse_attn_partitioned.argtypes = [ctypes.POINTER(_CShape), ctypes.POINTER(_CPartition), vp, vp, vp,
                                               i32p, i32p, i32p, i32p, ctypes.c_int32, vp, ctypes.c_int, f32p, vp,
                                               vp, ctypes.c_size_t, vp]
    lib.sa_dense_attn_static.restype = ctypes.c_int
    lib.sa_dense_attn_static.argtypes = [ctypes.POINTER(_CShape), vp, vp, vp, vp, ctypes.c_int, f32p, vp]
    lib.sa_probe_mfma.restype = ctypes.c_int
    lib.sa_probe_mfma.argtypes = [ctypes.c_int32, ctypes.c_int32, f32p, vp]
    lib.sa_probe_copy.restype = ctypes.c_int
    lib.sa_probe_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    lib.sa_profile_enable.restype = ctypes.c_int
    lib.sa_profile_enable.argtypes = [ctypes.c_int]
    lib.sa_profile_read.restype = ctypes.c_int
    lib.sa_profile_read.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_float), ctypes.c_int]
    lib.sa_status_string.restype = ctypes.c_char_p
    lib.sa_status_string.argtypes = [ctypes.c_int]
    lib.sa_version.restype = ctypes.c_int
    _lib = lib
    return lib


# ------------------------------------------------------------------ helpers --
def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(t: torch.Tensor, dtype, shape: Tuple[int, ...], name: str) -> None:
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype or tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected contiguous CUDA {dtype} tensor of shape {tuple(shape)}, "
                         f"got {t.dtype} {tuple(t.shape)} on {t.device}")


def _shape_of(q: torch.Tensor, k: torch.Tensor, scale: float) -> Shape:
    if q.dim() != 4 or k.dim() != 4:
        raise ValueError("q and k must be [batch, heads, seq, head_dim]")
    return Shape(q.shape[0], q.shape[1], k.shape[1], q.shape[2], q.shape[3], 1, float(scale))


def _workspace(nbytes: int, device) -> Optional[torch.Tensor]:
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def n_blocks(seq_len: int, granularity: int) -> int:
    return (seq_len + granularity - 1) // granularity


def sa_workspace_bytes(op: int, shape: Shape, n_sample_rows: int = 0, granularity: int = 1,
                       n_chunks: int = 1) -> int:
    lib = load_library()
    cs = shape.c()
    sm = _CSampling(n_sample_rows, n_chunks, granularity)
    return int(lib.sa_workspace_bytes(op, ctypes.byref(cs), ctypes.byref(sm)))


def sa_rows_from_ratio(seq_len: int, ratio: float) -> int:
    return int(load_library().sa_rows_from_ratio(seq_len, ratio))


# -------------------------------------------------------------- entry points --
def sa_sample_scores(q, k, n_sample_rows: int, scale: float = 0.0, workspace=None, want_lse=False,
                     granularity: int = 1, n_chunks: int = 1):
    """Stage 1: column and slash scores of the last ``n_sample_rows`` queries.
    Returns (col [B*Hq, S] f32, slash [B*Hq, S] f32[, row_lse [B*Hq, n] f32]);
    with granularity > 1 the two score tensors are [B*Hq, ceil(S / granularity)];
    with n_chunks > 1 they carry a leading chunk dimension."""
    lib = load_library()
    sh = _shape_of(q, k, scale)
    _check(q, torch.bfloat16, (sh.batch, sh.n_q_heads, sh.seq_len, sh.head_dim), "q")
    _check(k, torch.bfloat16, (sh.batch, sh.n_kv_heads, sh.seq_len, sh.head_dim), "k")
    cs, sm = sh.c(), _CSampling(n_sample_rows, n_chunks, granularity)
    need = int(lib.sa_workspace_bytes(SA_OP_SAMPLE_SCORES, ctypes.byref(cs), ctypes.byref(sm)))
    ws = workspace if workspace is not None else _workspace(need, q.device)
    dims = (sh.n_bh, n_blocks(sh.seq_len, max(granularity, 1)))
    if n_chunks != 1:
        dims = (max(n_chunks, 1),) + dims
    col = torch.empty(*dims, dtype=torch.float32, device=q.device)
    slash = torch.empty_like(col)
    lse = torch.empty(sh.n_bh, max(n_sample_rows, 1), dtype=torch.float32, device=q.device) if want_lse else None
    st = lib.sa_sample_scores(ctypes.byref(cs), ctypes.byref(sm), _ptr(q), _ptr(k), _ptr(col), _ptr(slash),
                              _ptr(lse), _ptr(ws), ws.numel() if ws is not None else 0, _stream())
    if st != 0:
        raise SaError(st, "sa_sample_scores")
    return (col, slash, lse) if want_lse else (col, slash)


def sa_select_strips(col_scores, slash_scores, alpha_c: float, alpha_s: float, shape: Shape):
    """Stage 2: returns (col_idx, col_cnt, slash_idx, slash_cnt) int32 device tensors."""
    lib = load_library()
    _check(col_scores, torch.float32, (shape.n_bh, shape.seq_len), "col_scores")
    _check(slash_scores, torch.float32, (shape.n_bh, shape.seq_len), "slash_scores")
    dev = col_scores.device
    col_idx = torch.empty(shape.n_bh, shape.seq_len, dtype=torch.int32, device=dev)
    slash_idx = torch.empty_like(col_idx)
    col_cnt = torch.empty(shape.n_bh, dtype=torch.int32, device=dev)
    slash_cnt = torch.empty_like(col_cnt)
    cs = shape.c()
    st = lib.sa_select_strips(ctypes.byref(cs), _ptr(col_scores), _ptr(slash_scores),
                              ctypes.c_float(alpha_c), ctypes.c_float(alpha_s),
                              _ptr(col_idx), _ptr(col_cnt), _ptr(slash_idx), _ptr(slash_cnt),
                              None, 0, _stream())
    if st != 0:
        raise SaError(st, "sa_select_strips")
    return col_idx, col_cnt, slash_idx, slash_cnt


def sa_block_scores(col_scores, slash_scores, granularity: int, shape: Shape):
    """Per-token scores -> block scores (Algorithm 1 block_reduction)."""
    lib = load_library()
    _check(col_scores, torch.float32, (shape.n_bh, shape.seq_len), "col_scores")
    _check(slash_scores, torch.float32, (shape.n_bh, shape.seq_len), "slash_scores")
    nb = n_blocks(shape.seq_len, max(granularity, 1))
    cb = torch.empty(shape.n_bh, nb, dtype=torch.float32, device=col_scores.device)
    sb = torch.empty_like(cb)
    cs = shape.c()
    st = lib.sa_block_scores(ctypes.byref(cs), int(granularity), _ptr(col_scores), _ptr(slash_scores),
                             _ptr(cb), _ptr(sb), _stream())
    if st != 0:
        raise SaError(st, "sa_block_scores")
    return cb, sb


def sa_select_blocks(col_block_scores, slash_block_scores, alpha_c: float, alpha_s: float, granularity: int,
                     shape: Shape):
    """Stage 2 over blocks: (col_blocks, col_cnt, slash_blocks, slash_cnt) int32 device tensors."""
    lib = load_library()
    nb = n_blocks(shape.seq_len, max(granularity, 1))
    _check(col_block_scores, torch.float32, (shape.n_bh, nb), "col_block_scores")
    _check(slash_block_scores, torch.float32, (shape.n_bh, nb), "slash_block_scores")
    dev = col_block_scores.device
    col_blk = torch.empty(shape.n_bh, nb, dtype=torch.int32, device=dev)
    slash_blk = torch.empty_like(col_blk)
    col_cnt = torch.empty(shape.n_bh, dtype=torch.int32, device=dev)
    slash_cnt = torch.empty_like(col_cnt)
    cs = shape.c()
    st = lib.sa_select_blocks(ctypes.byref(cs), int(granularity), _ptr(col_block_scores), _ptr(slash_block_scores),
                              ctypes.c_float(alpha_c), ctypes.c_float(alpha_s),
                              _ptr(col_blk), _ptr(col_cnt), _ptr(slash_blk), _ptr(slash_cnt), None, 0, _stream())
    if st != 0:
        raise SaError(st, "sa_select_blocks")
    return col_blk, col_cnt, slash_blk, slash_cnt


def sa_block_sparse_attn(q, k, v, col_blocks, col_cnt, slash_blocks, slash_cnt, local_window: int,
                         granularity: int, scale: float = 0.0, out_dtype: int = SA_OUT_BF16, workspace=None,
                         want_lse: bool = False, want_tiles: bool = False):
    """Attention under the block mask.  Returns (out, lse or None, tiles or None)."""
    lib = load_library()
    sh = _shape_of(q, k, scale)
    _check(q, torch.bfloat16, (sh.batch, sh.n_q_heads, sh.seq_len, sh.head_dim), "q")
    _check(k, torch.bfloat16, (sh.batch, sh.n_kv_heads, sh.seq_len, sh.head_dim), "k")
    _check(v, torch.bfloat16, (sh.batch, sh.n_kv_heads, sh.seq_len, sh.head_dim), "v")
    nb = n_blocks(sh.seq_len, max(granularity, 1))
    for t, nm in ((col_blocks, "col_blocks"), (slash_blocks, "slash_blocks")):
        _check(t, torch.int32, (sh.n_bh, nb), nm)
    for t, nm in ((col_cnt, "col_cnt"), (slash_cnt, "slash_cnt")):
        _check(t, torch.int32, (sh.n_bh,), nm)
    cs, sm = sh.c(), _CSampling(0, 1, granularity)
    need = int(lib.sa_workspace_bytes(SA_OP_BLOCK_SPARSE_ATTN, ctypes.byref(cs), ctypes.byref(sm)))
    ws = workspace if workspace is not None else _workspace(need, q.device)
    out = torch.empty(q.shape, dtype=torch.float32 if out_dtype == SA_OUT_F32 else torch.bfloat16, device=q.device)
    lse = torch.empty(sh.n_bh, sh.seq_len, dtype=torch.float32, device=q.device) if want_lse else None
    tiles = torch.empty(sh.n_bh, dtype=torch.int64, device=q.device) if want_tiles else None
    st = lib.sa_block_sparse_attn(ctypes.byref(cs), int(granularity), _ptr(q), _ptr(k), _ptr(v),
                                  _ptr(col_blocks), _ptr(col_cnt), _ptr(slash_blocks), _ptr(slash_cnt),
                                  int(local_window), _ptr(out), out_dtype, _ptr(lse), _ptr(tiles), _ptr(ws),
                                  ws.numel() if ws is not None else 0, _stream())
    if st != 0:
        raise SaError(st, "sa_block_sparse_attn")
    return out, lse, tiles


def sa_select_chunked(col_scores, slash_scores, alpha_c: float, alpha_s: float, shape: Shape,
                      n_chunks: int, granularity: int = 1):
    """Stage 2 for every (chunk, head): inputs [C, B*Hq, n]; returns
    (col_idx [C, B*Hq, n], col_cnt [C, B*Hq], slash_idx, slash_cnt)."""
    lib = load_library()
    n = n_blocks(shape.seq_len, max(granularity, 1))
    _check(col_scores, torch.float32, (n_chunks, shape.n_bh, n), "col_scores")
    _check(slash_scores, torch.float32, (n_chunks, shape.n_bh, n), "slash_scores")
    dev = col_scores.device
    col_idx = torch.empty(n_chunks, shape.n_bh, n, dtype=torch.int32, device=dev)
    slash_idx = torch.empty_like(col_idx)
    col_cnt = torch.empty(n_chunks, shape.n_bh, dtype=torch.int32, device=dev)
    slash_cnt = torch.empty_like(col_cnt)
    cs, sm = shape.c(), _CSampling(0, n_chunks, granularity)
    st = lib.sa_select_chunked(ctypes.byref(cs), ctypes.byref(sm), _ptr(col_scores), _ptr(slash_scores),
                               ctypes.c_float(alpha_c), ctypes.c_float(alpha_s),
                               _ptr(col_idx), _ptr(col_cnt), _ptr(slash_idx), _ptr(slash_cnt), None, 0, _stream())
    if st != 0:
        raise SaError(st, "sa_select_chunked")
    return col_idx, col_cnt, slash_idx, slash_cnt


def sa_sparse_attn_chunked(q, k, v, col_idx, col_cnt, slash_idx, slash_cnt, local_window: int, n_chunks: int,
                           granularity: int = 1, scale: float = 0.0, out_dtype: int = SA_OUT_BF16,
                           workspace=None, want_lse: bool = False, want_tiles: bool = False):
    """Attention where segment m of the queries is masked by chunk m's lists.
    Returns (out, lse or None, tiles or None)."""
    lib = load_library()
    sh = _shape_of(q, k, scale)
    _check(q, torch.bfloat16, (sh.batch, sh.n_q_heads, sh.seq_len, sh.head_dim), "q")
    _check(k, torch.bfloat16, (sh.batch, sh.n_kv_heads, sh.seq_len, sh.head_dim), "k")
    _check(v, torch.bfloat16, (sh.batch, sh.n_kv_heads, sh.seq_len, sh.head_dim), "v")
    n = n_blocks(sh.seq_len, max(granularity, 1))
    for t, nm in ((col_idx, "col_idx"), (slash_idx, "slash_idx")):
        _check(t, torch.int32, (n_chunks, sh.n_bh, n), nm)
    for t, nm in ((col_cnt, "col_cnt"), (slash_cnt, "slash_cnt")):
        _check(t, torch.int32, (n_chunks, sh.n_bh), nm)
    cs, sm = sh.c(), _CSampling(0, n_chunks, granularity)
    op = SA_OP_SPARSE_ATTN if granularity == 1 else SA_OP_BLOCK_SPARSE_ATTN
    need = int(lib.sa_workspace_bytes(op, ctypes.byref(cs), ctypes.byref(sm)))
    ws = workspace if workspace is not None else _workspace(need, q.device)
    out = torch.empty(q.shape, dtype=torch.float32 if out_dtype == SA_OUT_F32 else torch.bfloat16, device=q.device)
    lse = torch.empty(sh.n_bh, sh.seq_len, dtype=torch.float32, device=q.device) if want_lse else None
    tiles = torch.empty(sh.n_bh, dtype=torch.int64, device=q.device) if want_tiles else None
    st = lib.sa_sparse_attn_chunked(ctypes.byref(cs), ctypes.byref(sm), _ptr(q), _ptr(k), _ptr(v),
                                    _ptr(col_idx), _ptr(col_cnt), _ptr(slash_idx), _ptr(slash_cnt),
                                    int(local_window), _ptr(out), out_dtype, _ptr(lse), _ptr(tiles), _ptr(ws),
                                    ws.numel() if ws is not None else 0, _stream())
    if st != 0:
        raise SaError(st, "sa_sparse_attn_chunked")
    return out, lse, tiles


def sa_sparse_attn(q, k, v, col_idx, col_cnt, slash_idx, slash_cnt, local_window: int,
                   scale: float = 0.0, out_dtype: int = SA_OUT_BF16, workspace=None,
                   want_lse: bool = False, want_tiles: bool = False):
    """Attention under the strip mask.  Returns (out, lse or None, tiles or None)."""
    lib = load_library()
    sh = _shape_of(q, k, scale)
    _check(q, torch.bfloat16, (sh.batch, sh.n_q_heads, sh.seq_len, sh.head_dim), "q")
    _check(k, torch.bfloat16, (sh.batch, sh.n_kv_heads, sh.seq_len, sh.head_dim), "k")
    _check(v, torch.bfloat16, (sh.batch, sh.n_kv_heads, sh.seq_len, sh.head_dim), "v")
    for t, nm in ((col_idx, "col_idx"), (slash_idx, "slash_idx")):
        _check(t, torch.int32, (sh.n_bh, sh.seq_len), nm)
    for t, nm in ((col_cnt, "col_cnt"), (slash_cnt, "slash_cnt")):
        _check(t, torch.int32, (sh.n_bh,), nm)
    cs = sh.c()
    need = int(lib.sa_workspace_bytes(SA_OP_SPARSE_ATTN, ctypes.byref(cs), None))
    ws = workspace if workspace is not None else _workspace(need, q.device)
    out = torch.empty(q.shape, dtype=torch.float32 if out_dtype == SA_OUT_F32 else torch.bfloat16, device=q.device)
    lse = torch.empty(sh.n_bh, sh.seq_len, dtype=torch.float32, device=q.device) if want_lse else None
    tiles = torch.empty(sh.n_bh, dtype=torch.int64, device=q.device) if want_tiles else None
    st = lib.sa_sparse_attn(ctypes.byref(cs), _ptr(q), _ptr(k), _ptr(v), _ptr(col_idx), _ptr(col_cnt),
                            _ptr(slash_idx), _ptr(slash_cnt), int(local_window), _ptr(out), out_dtype,
                            _ptr(lse), _ptr(tiles), _ptr(ws), ws.numel() if ws is not None else 0, _stream())
    if st != 0:
        raise SaError(st, "sa_sparse_attn")
    return out, lse, tiles


def sa_partitioned_workspace_bytes(shape: Shape, heads_per_pass: int, n_query_segments: int = 1) -> int:
    cs, part = shape.c(), _CPartition(heads_per_pass, n_query_segments)
    return int(load_library().sa_partitioned_workspace_bytes(ctypes.byref(cs), ctypes.byref(part)))


def sa_sparse_attn_partitioned(q, k, v, col_idx, col_cnt, slash_idx, slash_cnt, local_window: int,
                               heads_per_pass: int, n_query_segments: int = 1, scale: float = 0.0,
                               out_dtype: int = SA_OUT_BF16, workspace=None, want_lse: bool = False,
                               want_tiles: bool = False, out=None):
    """sa_sparse_attn with the heads taken ``heads_per_pass`` at a time and the queries
    in ``n_query_segments`` launches: same result, workspace for one pass only.
    Returns (out, lse or None, tiles or None)."""
    lib = load_library()
    sh = _shape_of(q, k, scale)
    _check(q, torch.bfloat16, (sh.batch, sh.n_q_heads, sh.seq_len, sh.head_dim), "q")
    _check(k, torch.bfloat16, (sh.batch, sh.n_kv_heads, sh.seq_len, sh.head_dim), "k")
    _check(v, torch.bfloat16, (sh.batch, sh.n_kv_heads, sh.seq_len, sh.head_dim), "v")
    for t, nm in ((col_idx, "col_idx"), (slash_idx, "slash_idx")):
        _check(t, torch.int32, (sh.n_bh, sh.seq_len), nm)
    for t, nm in ((col_cnt, "col_cnt"), (slash_cnt, "slash_cnt")):
        _check(t, torch.int32, (sh.n_bh,), nm)
    cs, part = sh.c(), _CPartition(heads_per_pass, n_query_segments)
    need = int(lib.sa_partitioned_workspace_bytes(ctypes.byref(cs), ctypes.byref(part)))
    ws = workspace if workspace is not None else _workspace(need, q.device)
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32 if out_dtype == SA_OUT_F32 else torch.bfloat16,
                          device=q.device)
    lse = torch.empty(sh.n_bh, sh.seq_len, dtype=torch.float32, device=q.device) if want_lse else None
    tiles = torch.empty(sh.n_bh, dtype=torch.int64, device=q.device) if want_tiles else None
    st = lib.sa_sparse_attn_partitioned(ctypes.byref(cs), ctypes.byref(part), _ptr(q), _ptr(k), _ptr(v),
                                        _ptr(col_idx), _ptr(col_cnt), _ptr(slash_idx), _ptr(slash_cnt),
                                        int(local_window), _ptr(out), out_dtype, _ptr(lse), _ptr(tiles), _ptr(ws),
                                        ws.numel() if ws is not None else 0, _stream())
    if st != 0:
        raise SaError(st, "sa_sparse_attn_partitioned")
    return out, lse, tiles


def sa_dense_attn(q, k, v, scale: float = 0.0, out_dtype: int = SA_OUT_BF16, workspace=None,
                  want_lse: bool = False):
    """Dense causal attention.  Returns (out, lse or None)."""
    lib = load_library()
    sh = _shape_of(q, k, scale)
    _check(q, torch.bfloat16, (sh.batch, sh.n_q_heads, sh.seq_len, sh.head_dim), "q")
    _check(k, torch.bfloat16, (sh.batch, sh.n_kv_heads, sh.seq_len, sh.head_dim), "k")
    _check(v, torch.bfloat16, (sh.batch, sh.n_kv_heads, sh.seq_len, sh.head_dim), "v")
    cs = sh.c()
    need = int(lib.sa_workspace_bytes(SA_OP_DENSE_ATTN, ctypes.byref(cs), None))
    ws = workspace if workspace is not None else _workspace(need, q.device)
    out = torch.empty(q.shape, dtype=torch.float32 if out_dtype == SA_OUT_F32 else torch.bfloat16, device=q.device)
    lse = torch.empty(sh.n_bh, sh.seq_len, dtype=torch.float32, device=q.device) if want_lse else None
    st = lib.sa_dense_attn(ctypes.byref(cs), _ptr(q), _ptr(k), _ptr(v), _ptr(out), out_dtype, _ptr(lse),
                           _ptr(ws), ws.numel() if ws is not None else 0, _stream())
    if st != 0:
        raise SaError(st, "sa_dense_attn")
    return out, lse


SA_STATIC_SCRATCH_BYTES = 16 << 20


def sa_dense_attn_static(q, k, v, out, scale: float = 0.0, lse=None):
    """sa_dense_attn for callers that cannot allocate: the caller passes the output
    (bf16 or fp32, q's shape) and, optionally, the log-sum-exp buffer; the library
    keeps its scratch in a static device array.  Nothing is allocated here either."""
    lib = load_library()
    sh = _shape_of(q, k, scale)
    _check(q, torch.bfloat16, (sh.batch, sh.n_q_heads, sh.seq_len, sh.head_dim), "q")
    _check(k, torch.bfloat16, (sh.batch, sh.n_kv_heads, sh.seq_len, sh.head_dim), "k")
    _check(v, torch.bfloat16, (sh.batch, sh.n_kv_heads, sh.seq_len, sh.head_dim), "v")
    if out.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("out must be bf16 or fp32")
    _check(out, out.dtype, tuple(q.shape), "out")
    if lse is not None:
        _check(lse, torch.float32, (sh.n_bh, sh.seq_len), "lse")
    cs = sh.c()
    st = lib.sa_dense_attn_static(ctypes.byref(cs), _ptr(q), _ptr(k), _ptr(v), _ptr(out),
                                  SA_OUT_F32 if out.dtype == torch.float32 else SA_OUT_BF16, _ptr(lse), _stream())
    if st != 0:
        raise SaError(st, "sa_dense_attn_static")
    return out


def sa_probe_mfma(iters: int, waves_per_simd: int, sink) -> float:
    """Enqueue the back-to-back MFMA probe; returns the flop it performs."""
    st = load_library().sa_probe_mfma(int(iters), int(waves_per_simd), _ptr(sink), _stream())
    if st != 0:
        raise SaError(st, "sa_probe_mfma")
    return 1024.0 * waves_per_simd * iters * 16 * 32768


def sa_probe_copy(src, dst) -> int:
    """Enqueue a plain copy src -> dst (uint8 CUDA tensors of equal size); returns bytes read + written."""
    n = src.numel() * src.element_size()
    st = load_library().sa_probe_copy(_ptr(src), _ptr(dst), n, _stream())
    if st != 0:
        raise SaError(st, "sa_probe_copy")
    return 2 * n


SA_KERNELS = {"row_lse": 0, "score_accum": 1, "score_final": 2, "select": 3, "mask_prep": 4,
              "sparse_flash": 5, "dense_flash": 6, "transpose_v": 7}


def sa_profile_enable(enable: bool) -> None:
    st = load_library().sa_profile_enable(1 if enable else 0)
    if st != 0:
        raise SaError(st, "sa_profile_enable")


def sa_profile_read(kernel: str):
    """Durations (ms, oldest first) of the recorded launches of one kernel."""
    buf = (ctypes.c_float * 64)()
    n = load_library().sa_profile_read(SA_KERNELS[kernel], buf, 64)
    if n < 0:
        raise RuntimeError("sa_profile_read failed (profiling never enabled?)")
    return [float(buf[i]) for i in range(n)]


class SampleAttentionPlan:
    """Buffers for repeated calls on one shape: workspaces, score vectors, index
    lists and the output are allocated once, so a step is three library calls
    and nothing else (no allocation, no host synchronisation)."""

    def __init__(self, shape: Shape, n_sample_rows: int, device="cuda", out_dtype: int = SA_OUT_BF16,
                 granularity: int = 1, n_chunks: int = 1, with_lse: bool = False,
                 heads_per_pass: Optional[int] = None, n_query_segments: int = 1):
        """``heads_per_pass``: bound the workspace (long sequences): the attention call is
        sa_sparse_attn_partitioned with that many heads per pass, and stage 1 gets room for
        as many heads per pass (per-key strips, one chunk only)."""
        lib = load_library()
        self.lib, self.shape, self.n_s, self.out_dtype = lib, shape, n_sample_rows, out_dtype
        self.granularity, self.n_chunks = granularity, n_chunks
        self.cs = shape.c()
        self.sm = _CSampling(n_sample_rows, n_chunks, granularity)
        self.part = None
        if heads_per_pass is not None:
            if granularity != 1 or n_chunks != 1:
                raise ValueError("the head partition is offered for per-key strips with one chunk")
            self.part = _CPartition(heads_per_pass, n_query_segments)
            one_head = int(lib.sa_workspace_bytes(SA_OP_SAMPLE_SCORES_MIN, ctypes.byref(self.cs), ctypes.byref(self.sm)))
            sizes = [one_head * heads_per_pass + 4096,
                     int(lib.sa_partitioned_workspace_bytes(ctypes.byref(self.cs), ctypes.byref(self.part))),
                     int(lib.sa_workspace_bytes(SA_OP_DENSE_ATTN, ctypes.byref(self.cs), ctypes.byref(self.sm)))]
        else:
            ops = (SA_OP_SAMPLE_SCORES, SA_OP_SPARSE_ATTN if granularity == 1 else SA_OP_BLOCK_SPARSE_ATTN,
                   SA_OP_DENSE_ATTN)
            sizes = [int(lib.sa_workspace_bytes(op, ctypes.byref(self.cs), ctypes.byref(self.sm))) for op in ops]
        if min(sizes) == 0:
            raise ValueError("invalid shape or sampling for this library")
        need = max(sizes)
        n, S = shape.n_bh, n_blocks(shape.seq_len, granularity)   # candidates per head and direction
        lead = (n_chunks,) if n_chunks != 1 else ()               # chunked arrays: [chunk_n, heads, ...]
        self.ws = torch.empty(need, dtype=torch.uint8, device=device)
        self.col = torch.empty(*lead, n, S, dtype=torch.float32, device=device)
        self.slash = torch.empty_like(self.col)
        self.col_idx = torch.empty(*lead, n, S, dtype=torch.int32, device=device)
        self.slash_idx = torch.empty_like(self.col_idx)
        self.col_cnt = torch.empty(*lead, n, dtype=torch.int32, device=device)
        self.slash_cnt = torch.empty_like(self.col_cnt)
        self.tiles = torch.zeros(n, dtype=torch.int64, device=device)
        # optional log-sum-exp of every row, as the attention calls write it (masked or dense)
        self.lse = torch.empty(n, shape.seq_len, dtype=torch.float32, device=device) if with_lse else None
        odt = torch.float32 if out_dtype == SA_OUT_F32 else torch.bfloat16
        self.out = torch.empty(shape.batch, shape.n_q_heads, shape.seq_len, shape.head_dim, dtype=odt, device=device)

    def _ok(self, st, where):
        if st != 0:
            raise SaError(st, where)

    def sample(self, q, k):
        self._ok(self.lib.sa_sample_scores(ctypes.byref(self.cs), ctypes.byref(self.sm), _ptr(q), _ptr(k),
                                           _ptr(self.col), _ptr(self.slash), None, _ptr(self.ws),
                                           self.ws.numel(), _stream()), "sa_sample_scores")

    def select(self, alpha_c, alpha_s):
        if self.n_chunks != 1:
            self._ok(self.lib.sa_select_chunked(ctypes.byref(self.cs), ctypes.byref(self.sm), _ptr(self.col),
                                                _ptr(self.slash), ctypes.c_float(alpha_c), ctypes.c_float(alpha_s),
                                                _ptr(self.col_idx), _ptr(self.col_cnt), _ptr(self.slash_idx),
                                                _ptr(self.slash_cnt), None, 0, _stream()), "sa_select_chunked")
            return
        if self.granularity != 1:
            self._ok(self.lib.sa_select_blocks(ctypes.byref(self.cs), self.granularity, _ptr(self.col),
                                               _ptr(self.slash), ctypes.c_float(alpha_c), ctypes.c_float(alpha_s),
                                               _ptr(self.col_idx), _ptr(self.col_cnt), _ptr(self.slash_idx),
                                               _ptr(self.slash_cnt), None, 0, _stream()), "sa_select_blocks")
            return
        self._ok(self.lib.sa_select_strips(ctypes.byref(self.cs), _ptr(self.col), _ptr(self.slash),
                                           ctypes.c_float(alpha_c), ctypes.c_float(alpha_s),
                                           _ptr(self.col_idx), _ptr(self.col_cnt), _ptr(self.slash_idx),
                                           _ptr(self.slash_cnt), None, 0, _stream()), "sa_select_strips")

    def attend(self, q, k, v, window):
        if self.part is not None:
            self._ok(self.lib.sa_sparse_attn_partitioned(ctypes.byref(self.cs), ctypes.byref(self.part), _ptr(q),
                                                         _ptr(k), _ptr(v), _ptr(self.col_idx), _ptr(self.col_cnt),
                                                         _ptr(self.slash_idx), _ptr(self.slash_cnt), int(window),
                                                         _ptr(self.out), self.out_dtype, _ptr(self.lse),
                                                         _ptr(self.tiles), _ptr(self.ws), self.ws.numel(), _stream()),
                     "sa_sparse_attn_partitioned")
            return
        if self.n_chunks != 1:
            self._ok(self.lib.sa_sparse_attn_chunked(ctypes.byref(self.cs), ctypes.byref(self.sm), _ptr(q), _ptr(k),
                                                     _ptr(v), _ptr(self.col_idx), _ptr(self.col_cnt),
                                                     _ptr(self.slash_idx), _ptr(self.slash_cnt), int(window),
                                                     _ptr(self.out), self.out_dtype, _ptr(self.lse), _ptr(self.tiles),
                                                     _ptr(self.ws), self.ws.numel(), _stream()),
                     "sa_sparse_attn_chunked")
            return
        if self.granularity != 1:
            self._ok(self.lib.sa_block_sparse_attn(ctypes.byref(self.cs), self.granularity, _ptr(q), _ptr(k), _ptr(v),
                                                   _ptr(self.col_idx), _ptr(self.col_cnt), _ptr(self.slash_idx),
                                                   _ptr(self.slash_cnt), int(window), _ptr(self.out),
                                                   self.out_dtype, _ptr(self.lse), _ptr(self.tiles), _ptr(self.ws),
                                                   self.ws.numel(), _stream()), "sa_block_sparse_attn")
            return
        self._ok(self.lib.sa_sparse_attn(ctypes.byref(self.cs), _ptr(q), _ptr(k), _ptr(v), _ptr(self.col_idx),
                                         _ptr(self.col_cnt), _ptr(self.slash_idx), _ptr(self.slash_cnt),
                                         int(window), _ptr(self.out), self.out_dtype, _ptr(self.lse), _ptr(self.tiles),
                                         _ptr(self.ws), self.ws.numel(), _stream()), "sa_sparse_attn")

    def dense(self, q, k, v):
        self._ok(self.lib.sa_dense_attn(ctypes.byref(self.cs), _ptr(q), _ptr(k), _ptr(v), _ptr(self.out),
                                        self.out_dtype, _ptr(self.lse), _ptr(self.ws), self.ws.numel(), _stream()),
                 "sa_dense_attn")

    def run(self, q, k, v, alpha_c, alpha_s, window):
        self.sample(q, k)
        self.select(alpha_c, alpha_s)
        self.attend(q, k, v, window)
        return self.out


def sample_attention(q, k, v, n_sample_rows: int, alpha_c: float, alpha_s: float, local_window: int,
                     scale: float = 0.0, out_dtype: int = SA_OUT_BF16):
    """The whole path (Algorithm 1, chunk_n = 1): three library calls chained on
    the current stream with no host synchronisation in between."""
    sh = _shape_of(q, k, scale)
    col, slash = sa_sample_scores(q, k, n_sample_rows, scale)
    ci, cc, si, sc = sa_select_strips(col, slash, alpha_c, alpha_s, sh)
    out, _, _ = sa_sparse_attn(q, k, v, ci, cc, si, sc, local_window, scale, out_dtype)
    return out


def block_sample_attention(q, k, v, n_sample_rows: int, alpha_c: float, alpha_s: float, local_window: int,
                           granularity: int = 128, scale: float = 0.0, out_dtype: int = SA_OUT_BF16):
    """The whole path at block granularity (Algorithm 1 with blk = granularity)."""
    sh = _shape_of(q, k, scale)
    cb, sb = sa_sample_scores(q, k, n_sample_rows, scale, granularity=granularity)
    ci, cc, si, sc = sa_select_blocks(cb, sb, alpha_c, alpha_s, granularity, sh)
    out, _, _ = sa_block_sparse_attn(q, k, v, ci, cc, si, sc, local_window, granularity, scale, out_dtype)
    return out


def chunked_sample_attention(q, k, v, n_sample_rows: int, n_chunks: int, alpha_c: float, alpha_s: float,
                             local_window: int, granularity: int = 1, scale: float = 0.0,
                             out_dtype: int = SA_OUT_BF16):
    """The whole path with chunk_n = n_chunks (Algorithm 1 as printed: the bottom
    rows of every query segment are sampled, each segment gets its own mask)."""
    sh = _shape_of(q, k, scale)
    col, slash = sa_sample_scores(q, k, n_sample_rows, scale, granularity=granularity, n_chunks=n_chunks)
    if n_chunks == 1:
        col, slash = col[None], slash[None]
    ci, cc, si, sc = sa_select_chunked(col, slash, alpha_c, alpha_s, sh, n_chunks, granularity)
    out, _, _ = sa_sparse_attn_chunked(q, k, v, ci, cc, si, sc, local_window, n_chunks, granularity, scale, out_dtype)
    return out
