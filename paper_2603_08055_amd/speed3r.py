"""Thin ctypes binding of libspeed3r.so: same names as the C ABI (include/speed3r.h), argument
marshalling only.  Tensors are torch tensors on the GPU (torch is used for device memory and
streams, nothing else); every step of the path runs in the library's HIP kernels.  There is no
fallback: if the library is missing or a call fails, an exception is raised."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspeed3r.so")

S3R_OK, S3R_ERR_INVALID_ARG, S3R_ERR_UNSUPPORTED, S3R_ERR_WORKSPACE, S3R_ERR_HIP = range(5)
S3R_F32, S3R_BF16 = 0, 1
S3R_DIAG_FORCED_RANGE, S3R_DIAG_FORCED_ORDER = 1, 2
STAGES = ("pool", "split", "compress", "topk", "select", "dense")
HEAD_DIM = 64

_vp = ctypes.c_void_p
_i64 = ctypes.c_int64
_int = ctypes.c_int
_flt = ctypes.c_float


class s3r_params(ctypes.Structure):
    _fields_ = [("q", _vp), ("k", _vp), ("v", _vp), ("out", _vp), ("gate_logits", _vp),
                ("forced_blocks", _vp), ("n_forced", _int), ("status", _vp),
                ("tokens_per_view", _int), ("special_per_view", _int),
                ("grid_h", _int), ("grid_w", _int), ("window", _int), ("compress_queries", _int),
                ("n_tok", _i64), ("stride_tok", _i64), ("stride_head", _i64), ("heads", _int), ("head_dim", _int), ("block", _int),
                ("topk", _int), ("dtype", _int), ("softmax_scale", _flt), ("topk_idx", _vp),
                ("lse_sel", _vp), ("o_comp", _vp), ("o_sel", _vp), ("workspace", _vp),
                ("workspace_bytes", ctypes.c_size_t), ("stream", _vp)]


EXPORTS = {
    "speed3r_workspace_bytes": (ctypes.c_size_t, [_i64, _int, _int, _int, _int, _int, _int]),
    "speed3r_workspace_bytes_ex": (ctypes.c_size_t, [ctypes.POINTER(s3r_params)]),
    "speed3r_num_blocks": (_i64, [ctypes.POINTER(s3r_params)]),
    "speed3r_selected_per_row": (_int, [_i64, _int, _int, _int]),
    "speed3r_sparse_global_attn_ex": (_int, [ctypes.POINTER(s3r_params)]),
    "speed3r_sparse_global_attn": (_int, [_vp, _vp, _vp, _vp, _i64, _int, _int, _int, _int, _vp]),
    "speed3r_sparse_global_attn_noalloc": (_int, [_vp, _vp, _vp, _vp, _i64, _int, _int, _int, _int, _vp]),
    "speed3r_dense_attn": (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _int, _int, _int, _flt, _vp]),
    "speed3r_pool_blocks": (_int, [_vp, _vp, _vp, _vp, _vp, _vp, _i64, _int, _int, _int, _int, _vp]),
    "speed3r_compress_attn_scores": (_int, [_vp, _vp, _vp, _vp, _i64, _vp, _i64, _int, _int, _flt,
                                            _int, _vp]),
    "speed3r_compress_attn_topk": (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _int, _int, _int, _flt, _int, _vp]),
    "speed3r_topk_blocks": (_int, [_vp, _i64, _vp, _i64, _int, _int, _vp]),
    "speed3r_select_attn": (_int, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _int, _int,
                                   _int, _int, _int, _flt, _vp]),
    "speed3r_probe_select_loads": (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _int, _int, _int, _int, _int, _int, _vp]),
    "speed3r_set_profiling": (_int, [_int]),
    "speed3r_get_stage_ms": (_int, [ctypes.POINTER(_flt), ctypes.POINTER(_int)]),
    "speed3r_set_kernel_choice": (_int, [_int]),
    "speed3r_release_scratch": (_int, []),
    "speed3r_last_error": (ctypes.c_char_p, []),
}

_lib = None


class Speed3rError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"speed3r status {status}: {message}")
        self.status = status


def load():
    """Load libspeed3r.so (built by paper_2603_08055_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it first (python -m paper_2603_08055_amd.build)")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _check(status: int):
    if status != S3R_OK:
        raise Speed3rError(status, speed3r_last_error())


def speed3r_last_error() -> str:
    return load().speed3r_last_error().decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return S3R_F32
    if t.dtype == torch.bfloat16:
        return S3R_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _dev(t, name, dtype=None):
    """data_ptr of a contiguous CUDA tensor (None -> NULL)."""
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous tensor on the GPU")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def _strided_qkv(q, k, v):
    """data_ptrs and the common (stride_tok, stride_head) of q, k, v: CUDA tensors [n_tok, heads, head_dim]
    whose channels are contiguous (views of a packed projection output are fine)."""
    for name, t in (("q", q), ("k", k), ("v", v)):
        if not (isinstance(t, torch.Tensor) and t.is_cuda):
            raise TypeError(f"{name} must be a tensor on the GPU")
        if t.stride(2) != 1 and t.shape[2] > 1:
            raise TypeError(f"the channels of {name} must be contiguous")
    st = (q.stride(0), q.stride(1))
    if (k.stride(0), k.stride(1)) != st or (v.stride(0), v.stride(1)) != st:
        raise TypeError("q, k and v must share their row and head strides")
    if q.is_contiguous():
        st = (0, 0)
    return q.data_ptr(), k.data_ptr(), v.data_ptr(), st


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if isinstance(stream, torch.cuda.Stream) else int(stream)


def _qkv(q, k, v):
    if q.dim() != 3 or k.shape != q.shape or v.shape != q.shape or k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v must share shape [n_tok, heads, head_dim] and dtype")
    return q.shape[0], q.shape[1], q.shape[2], _dtype_code(q)


def speed3r_workspace_bytes(n_tok, heads, head_dim, block, topk, dtype, n_forced=0) -> int:
    return int(load().speed3r_workspace_bytes(n_tok, heads, head_dim, block, topk, n_forced, dtype))


def _shape_params(n_tok, heads, head_dim, block, topk, dtype, n_forced, tokens_per_view, special_per_view, grid,
                  compress_queries=0):
    p = s3r_params()
    p.compress_queries = int(compress_queries)
    p.n_tok, p.heads, p.head_dim, p.block, p.topk, p.dtype = n_tok, heads, head_dim, block, topk, dtype
    p.n_forced, p.tokens_per_view, p.special_per_view = n_forced, tokens_per_view, special_per_view
    p.grid_h, p.grid_w, p.window = grid if grid else (0, 0, 0)
    return p


def speed3r_workspace_bytes_ex(n_tok, heads, head_dim, block, topk, dtype, n_forced=0, tokens_per_view=0,
                               special_per_view=0, grid=None, compress_queries=0) -> int:
    """grid = (grid_h, grid_w, window) for spatial pooling windows."""
    p = _shape_params(n_tok, heads, head_dim, block, topk, dtype, n_forced, tokens_per_view, special_per_view, grid,
                      compress_queries)
    return int(load().speed3r_workspace_bytes_ex(ctypes.byref(p)))


def speed3r_num_blocks(n_tok, heads, head_dim, block, topk, dtype, tokens_per_view=0, special_per_view=0,
                       grid=None) -> int:
    p = _shape_params(n_tok, heads, head_dim, block, topk, dtype, 0, tokens_per_view, special_per_view, grid)
    n = int(load().speed3r_num_blocks(ctypes.byref(p)))
    if n < 0:
        raise Speed3rError(S3R_ERR_INVALID_ARG, speed3r_last_error())
    return n


def speed3r_selected_per_row(n_tok, block, topk, n_forced=0) -> int:
    w = int(load().speed3r_selected_per_row(n_tok, block, topk, n_forced))
    if w < 0:
        raise ValueError("invalid arguments to speed3r_selected_per_row")
    return w


def speed3r_sparse_global_attn_ex(q, k, v, out, block, topk, *, gate_logits=None, softmax_scale=0.0,
                                  topk_idx=None, lse_sel=None, o_comp=None, o_sel=None,
                                  forced_blocks=None, tokens_per_view=0, special_per_view=0, grid=None,
                                  compress_queries=0, workspace=None, status=None, stream=None):
    """The whole path on caller-provided buffers.  `workspace` is a uint8 CUDA tensor of at least
    speed3r_workspace_bytes(...) bytes (allocated here when None).  `forced_blocks` is an int32
    CUDA tensor of ascending distinct block indices attended by every query block.  With
    special_per_view > 0 the first rows of every view of tokens_per_view rows are special tokens
    (dense attention over all rows); the other rows form the sequence of the sparse path.
    grid = (grid_h, grid_w, window) makes the blocks spatial windows of each view's patch grid.
    compress_queries = 1: every row's own query (instead of its block's pooled query) attends the
    pooled keys in the compression branch.  `status`: an int32 CUDA tensor of one element that receives
    0 or the S3R_DIAG_* bits for a forced_blocks list that is out of range or not strictly ascending.  q, k, v may be strided views with contiguous channels
    and common strides (slices of one packed tensor).  Returns the workspace used."""
    n_tok, heads, head_dim, dt = _qkv(q, k, v)
    n_forced = 0 if forced_blocks is None else int(forced_blocks.numel())
    if workspace is None:
        need = speed3r_workspace_bytes_ex(n_tok, heads, head_dim, block, topk, dt, n_forced, tokens_per_view,
                                          special_per_view, grid, compress_queries)
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=q.device)   # 0: the call below says why
    p = s3r_params()
    p.q, p.k, p.v, (p.stride_tok, p.stride_head) = _strided_qkv(q, k, v)
    p.out = _dev(out, "out", q.dtype)
    p.gate_logits = _dev(gate_logits, "gate_logits", q.dtype)
    p.forced_blocks = _dev(forced_blocks, "forced_blocks", torch.int32) if n_forced else None
    p.n_forced = n_forced
    p.status = _dev(status, "status", torch.int32)
    p.tokens_per_view, p.special_per_view = int(tokens_per_view), int(special_per_view)
    p.grid_h, p.grid_w, p.window = grid if grid else (0, 0, 0)
    p.compress_queries = int(compress_queries)
    p.n_tok, p.heads, p.head_dim, p.block, p.topk, p.dtype = n_tok, heads, head_dim, block, topk, dt
    p.softmax_scale = float(softmax_scale)
    p.topk_idx = _dev(topk_idx, "topk_idx", torch.int32)
    p.lse_sel = _dev(lse_sel, "lse_sel", torch.float32)
    p.o_comp = _dev(o_comp, "o_comp", torch.float32)
    p.o_sel = _dev(o_sel, "o_sel", q.dtype)
    p.workspace = _dev(workspace, "workspace", torch.uint8)
    p.workspace_bytes = workspace.numel()
    p.stream = _stream(stream)
    _check(load().speed3r_sparse_global_attn_ex(ctypes.byref(p)))
    return workspace


def speed3r_sparse_global_attn(q, k, v, out, block, topk, stream=None):
    n_tok, heads, head_dim, dt = _qkv(q, k, v)
    if dt != S3R_BF16:
        raise TypeError("the short form is bf16 only; use speed3r_sparse_global_attn_ex")
    _check(load().speed3r_sparse_global_attn(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"),
                                             _dev(out, "out", q.dtype), n_tok, heads, head_dim,
                                             block, topk, _stream(stream)))


STATIC_SCRATCH_BYTES = 64 << 20


def speed3r_sparse_global_attn_noalloc(q, k, v, out, block, topk, stream=None):
    """The short form on the library's fixed device scratch: the call allocates nothing."""
    n_tok, heads, head_dim, dt = _qkv(q, k, v)
    if dt != S3R_BF16:
        raise TypeError("the short forms are bf16 only; use speed3r_sparse_global_attn_ex")
    _check(load().speed3r_sparse_global_attn_noalloc(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"),
                                                     _dev(out, "out", q.dtype), n_tok, heads, head_dim,
                                                     block, topk, _stream(stream)))


def speed3r_dense_attn(q, k, v, out, lse=None, softmax_scale=0.0, stream=None):
    n_tok, heads, head_dim, dt = _qkv(q, k, v)
    _check(load().speed3r_dense_attn(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"),
                                     _dev(out, "out", q.dtype), _dev(lse, "lse", torch.float32),
                                     n_tok, heads, head_dim, dt, float(softmax_scale), _stream(stream)))


def speed3r_pool_blocks(q, k, v, qc, kc, vc, block, stream=None):
    n_tok, heads, head_dim, dt = _qkv(q, k, v)
    f32 = torch.float32
    _check(load().speed3r_pool_blocks(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(qc, "qc", f32),
                                      _dev(kc, "kc", f32), _dev(vc, "vc", f32), n_tok, heads,
                                      head_dim, block, dt, _stream(stream)))


def speed3r_compress_attn_scores(qc, kc, vc, s_guide, o_comp, softmax_scale=0.0, accurate_pv=False,
                                 stream=None):
    heads, n_blk, head_dim = qc.shape
    if s_guide.dim() != 3 or s_guide.shape[0] != heads or s_guide.shape[1] != n_blk:
        raise ValueError("s_guide must be [heads, n_blk, ld_s]")
    f32 = torch.float32
    _check(load().speed3r_compress_attn_scores(_dev(qc, "qc", f32), _dev(kc, "kc", f32),
                                               _dev(vc, "vc", f32), _dev(s_guide, "s_guide", f32),
                                               s_guide.shape[2], _dev(o_comp, "o_comp", f32), n_blk,
                                               heads, head_dim, float(softmax_scale),
                                               int(bool(accurate_pv)), _stream(stream)))


def speed3r_compress_attn_topk(qc, kc, vc, o_comp, idx, topk, softmax_scale=0.0, accurate_pv=False, stream=None):
    heads, n_blk, head_dim = qc.shape
    f32 = torch.float32
    _check(load().speed3r_compress_attn_topk(_dev(qc, "qc", f32), _dev(kc, "kc", f32), _dev(vc, "vc", f32),
                                             _dev(o_comp, "o_comp", f32), _dev(idx, "idx", torch.int32), n_blk,
                                             heads, head_dim, int(topk), float(softmax_scale),
                                             int(bool(accurate_pv)), _stream(stream)))


def speed3r_topk_blocks(s_guide, idx, n_blk, topk, stream=None):
    heads, rows, ld_s = s_guide.shape
    if rows != n_blk:
        raise ValueError("s_guide must be [heads, n_blk, ld_s]")
    _check(load().speed3r_topk_blocks(_dev(s_guide, "s_guide", torch.float32), ld_s,
                                      _dev(idx, "idx", torch.int32), n_blk, heads, topk,
                                      _stream(stream)))


def speed3r_select_attn(q, k, v, idx, out, block, *, o_comp=None, gate_logits=None, o_sel=None,
                        lse=None, softmax_scale=0.0, stream=None):
    n_tok, heads, head_dim, dt = _qkv(q, k, v)
    if idx.dim() != 3 or idx.shape[0] != heads:
        raise ValueError("idx must be [heads, n_blk, kk]")
    _check(load().speed3r_select_attn(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"),
                                      _dev(idx, "idx", torch.int32),
                                      _dev(o_comp, "o_comp", torch.float32),
                                      _dev(gate_logits, "gate_logits", q.dtype),
                                      _dev(out, "out", q.dtype), _dev(o_sel, "o_sel", q.dtype),
                                      _dev(lse, "lse", torch.float32), n_tok, heads, head_dim, block,
                                      idx.shape[2], dt, float(softmax_scale), _stream(stream)))


def speed3r_probe_select_loads(q, k, v, idx, out, block, ring_stages=0, wg_per_cu=0, stream=None):
    """The selection kernel's data movement without its arithmetic (measurement utility); out receives q.
    ring_stages 0/2..4 and wg_per_cu 0/1..5 vary the LDS ring depth and the workgroups per CU."""
    n_tok, heads, head_dim, dt = _qkv(q, k, v)
    if dt != S3R_BF16 or idx.dim() != 3 or idx.shape[0] != heads:
        raise ValueError("bf16 q, k, v and idx [heads, n_blk, kk] expected")
    _check(load().speed3r_probe_select_loads(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(idx, "idx", torch.int32),
                                             _dev(out, "out", q.dtype), n_tok, heads, head_dim, block, idx.shape[2],
                                             int(ring_stages), int(wg_per_cu), _stream(stream)))


def speed3r_set_profiling(enable: bool):
    _check(load().speed3r_set_profiling(int(bool(enable))))


def speed3r_get_stage_ms():
    """(ms, launches) dictionaries keyed by stage name, summed over the profiled calls since the
    previous read."""
    ms = (_flt * len(STAGES))()
    n = (_int * len(STAGES))()
    _check(load().speed3r_get_stage_ms(ms, n))
    return ({s: float(ms[i]) for i, s in enumerate(STAGES)},
            {s: int(n[i]) for i, s in enumerate(STAGES)})


def speed3r_set_kernel_choice(choice: int):
    _check(load().speed3r_set_kernel_choice(int(choice)))


def speed3r_release_scratch():
    _check(load().speed3r_release_scratch())
