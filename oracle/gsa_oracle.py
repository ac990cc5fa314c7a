"""ctypes front end of the fp64 CPU oracle (``gsa_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by ``bench.py``'s ``cpu_baseline`` leg.  The product package never imports
this module, and this module never imports the product package.

Every function takes numpy arrays; q, k, v and gate logits are float32 arrays of
shape [n_tok, heads, d] holding the exact values the device path receives (bf16
inputs widened exactly).  All arithmetic happens in double inside the C file.
The steps follow Sec. 3.2 of the paper (eqs. 2-8) in its own order; see the
header of ``gsa_oracle.c`` for the conventions and for what pins each step.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gsa_oracle.c")
_LIB = os.path.join(_HERE, "libgsa_oracle.so")

_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_i64p = ctypes.POINTER(ctypes.c_int64)
_i32p = ctypes.POINTER(ctypes.c_int32)
_i64 = ctypes.c_int64
_int = ctypes.c_int
_dbl = ctypes.c_double


def build(force: bool = False) -> str:
    """Compile gsa_oracle.c with gcc into libgsa_oracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-fno-fast-math",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.gsa_oracle_threads.restype = _int
        lib.gsa_oracle_pool.argtypes = [_f32p, _i64, _int, _int, _int, _f64p]
        lib.gsa_oracle_scores.argtypes = [_f64p, _f64p, _i64, _int, _int, _i64p, _i64, _f64p]
        lib.gsa_oracle_compressed_attn.argtypes = [_f64p, _f64p, _i64, _int, _int, _i64, _dbl, _f64p]
        lib.gsa_oracle_topk.argtypes = [_f64p, _i64, _int, _i64, _int, _i32p]
        lib.gsa_oracle_topk_excluding.argtypes = [_f64p, _i64, _int, _i64, _int,
                                                  ctypes.POINTER(ctypes.c_uint8), _i32p]
        lib.gsa_oracle_select_attn.argtypes = [_f32p, _f32p, _f32p, _i64, _int, _int, _int, _i64p,
                                               _i64, _i32p, _int, _dbl, _f64p, _f64p]
        lib.gsa_oracle_merge.argtypes = [_f64p, _f64p, _f32p, _i64, _int, _int, _int, _i64p, _i64,
                                         _f64p]
        lib.gsa_oracle_dense_attn.argtypes = [_f32p, _f32p, _f32p, _i64, _int, _int, _i64p, _i64,
                                              _dbl, _f64p, _f64p]
        for name in ("gsa_oracle_pool", "gsa_oracle_scores", "gsa_oracle_compressed_attn",
                     "gsa_oracle_topk", "gsa_oracle_topk_excluding", "gsa_oracle_select_attn", "gsa_oracle_merge",
                     "gsa_oracle_dense_attn"):
            getattr(lib, name).restype = None
        _lib = lib
    return _lib


def threads() -> int:
    """Number of OpenMP threads the oracle will use."""
    return int(_load().gsa_oracle_threads())


def _f32(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None:
        assert a.shape == tuple(shape), (a.shape, shape)
    return a


def _ptr(a, typ):
    return a.ctypes.data_as(typ)


def n_blocks(n_tok: int, block: int) -> int:
    return (n_tok + block - 1) // block


def _rows(rows, n_blk):
    if rows is None:
        rows = np.arange(n_blk, dtype=np.int64)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    assert rows.ndim == 1 and (rows.size == 0 or (rows.min() >= 0 and rows.max() < n_blk))
    return rows


def pool(x, block: int) -> np.ndarray:
    """Block means of x [n_tok, heads, d] -> float64 [heads, n_blk, d]."""
    x = _f32(x)
    n_tok, heads, d = x.shape
    out = np.empty((heads, n_blocks(n_tok, block), d), dtype=np.float64)
    _load().gsa_oracle_pool(_ptr(x, _f32p), n_tok, heads, d, block, _ptr(out, _f64p))
    return out


def scores(qc, kc, rows=None) -> np.ndarray:
    """Eq. 4, S_guide rows for the query blocks `rows` -> [heads, n_rows, n_blk]."""
    qc = np.ascontiguousarray(qc, dtype=np.float64)
    kc = np.ascontiguousarray(kc, dtype=np.float64)
    heads, n_blk, d = qc.shape
    assert kc.shape == qc.shape
    rows = _rows(rows, n_blk)
    out = np.empty((heads, rows.size, n_blk), dtype=np.float64)
    _load().gsa_oracle_scores(_ptr(qc, _f64p), _ptr(kc, _f64p), n_blk, heads, d,
                              _ptr(rows, _i64p), rows.size, _ptr(out, _f64p))
    return out


def compressed_attn(s, vc, scale: float) -> np.ndarray:
    """Eq. 3 on precomputed score rows s [heads, n_rows, n_blk] -> [heads, n_rows, d]."""
    s = np.ascontiguousarray(s, dtype=np.float64)
    vc = np.ascontiguousarray(vc, dtype=np.float64)
    heads, n_rows, n_blk = s.shape
    assert vc.shape[:2] == (heads, n_blk)
    d = vc.shape[2]
    out = np.empty((heads, n_rows, d), dtype=np.float64)
    _load().gsa_oracle_compressed_attn(_ptr(s, _f64p), _ptr(vc, _f64p), n_blk, heads, d, n_rows,
                                       float(scale), _ptr(out, _f64p))
    return out


def topk(s, k: int) -> np.ndarray:
    """TopKSelect per row of s [heads, n_rows, n_blk] -> int32 [heads, n_rows, k], ascending."""
    s = np.ascontiguousarray(s, dtype=np.float64)
    heads, n_rows, n_blk = s.shape
    assert 1 <= k <= n_blk
    out = np.empty((heads, n_rows, k), dtype=np.int32)
    _load().gsa_oracle_topk(_ptr(s, _f64p), n_blk, heads, n_rows, k, _ptr(out, _i32p))
    return out


def forced_mask(forced, n_blk: int) -> np.ndarray:
    """uint8 [n_blk] mask of the always-attended blocks; `forced` = ascending distinct indices."""
    forced = np.asarray(forced, dtype=np.int64).reshape(-1)
    assert forced.size == 0 or (forced.min() >= 0 and forced.max() < n_blk)
    assert np.all(np.diff(forced) > 0), "forced blocks must be ascending and distinct"
    m = np.zeros(n_blk, dtype=np.uint8)
    m[forced] = 1
    return m


def topk_with_forced(s, k: int, forced) -> np.ndarray:
    """Sec. 3.3 hybrid selection set per row of s [heads, n_rows, n_blk]: the fixed blocks `forced`
    plus the k_dyn = min(k, n_blk - len(forced)) best of the remaining blocks, merged ascending.
    Returns int32 [heads, n_rows, len(forced) + k_dyn]."""
    s = np.ascontiguousarray(s, dtype=np.float64)
    heads, n_rows, n_blk = s.shape
    forced = np.asarray(forced, dtype=np.int32).reshape(-1)
    mask = forced_mask(forced, n_blk)
    k_dyn = min(int(k), n_blk - forced.size)
    assert k_dyn >= 0
    fixed = np.broadcast_to(forced, (heads, n_rows, forced.size))
    if k_dyn == 0:
        return np.ascontiguousarray(fixed)
    dyn = np.empty((heads, n_rows, k_dyn), dtype=np.int32)
    _load().gsa_oracle_topk_excluding(_ptr(s, _f64p), n_blk, heads, n_rows, k_dyn,
                                      _ptr(mask, ctypes.POINTER(ctypes.c_uint8)), _ptr(dyn, _i32p))
    return np.sort(np.concatenate([fixed, dyn], axis=2), axis=2).astype(np.int32)


def select_attn(q, k, v, block: int, idx, scale: float, rows=None):
    """Eq. 6 with a given index set idx [heads, n_rows, kk].

    Returns (o_sel [n_rows, block, heads, d], lse [heads, n_rows, block])."""
    q = _f32(q)
    k = _f32(k, q.shape)
    v = _f32(v, q.shape)
    n_tok, heads, d = q.shape
    n_blk = n_blocks(n_tok, block)
    rows = _rows(rows, n_blk)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    assert idx.shape[:2] == (heads, rows.size)
    kk = idx.shape[2]
    assert idx.size == 0 or (idx.min() >= 0 and idx.max() < n_blk)
    o = np.empty((rows.size, block, heads, d), dtype=np.float64)
    lse = np.empty((heads, rows.size, block), dtype=np.float64)
    _load().gsa_oracle_select_attn(_ptr(q, _f32p), _ptr(k, _f32p), _ptr(v, _f32p), n_tok, heads, d,
                                   block, _ptr(rows, _i64p), rows.size, _ptr(idx, _i32p), kk,
                                   float(scale), _ptr(o, _f64p), _ptr(lse, _f64p))
    return o, lse


def merge(oc, o_sel, gate, n_tok: int, block: int, rows=None) -> np.ndarray:
    """Eqs. 5, 7, 8 -> out [n_rows, block, heads, d]; gate None means g = 1/2."""
    oc = np.ascontiguousarray(oc, dtype=np.float64)
    o_sel = np.ascontiguousarray(o_sel, dtype=np.float64)
    heads, n_rows, d = oc.shape
    assert o_sel.shape == (n_rows, block, heads, d)
    rows = _rows(rows, n_blocks(n_tok, block))
    assert rows.size == n_rows
    gp = None
    if gate is not None:
        gate = _f32(gate, (n_tok, heads, d))
        gp = _ptr(gate, _f32p)
    out = np.empty_like(o_sel)
    _load().gsa_oracle_merge(_ptr(oc, _f64p), _ptr(o_sel, _f64p), gp, n_tok, heads, d, block,
                             _ptr(rows, _i64p), n_rows, _ptr(out, _f64p))
    return out


def dense_attn(q, k, v, scale: float, q_tok=None, want_lse: bool = False):
    """Plain softmax attention (eq. 2 form) of the query tokens q_tok over all keys.

    Returns out [n_q, heads, d] (and lse [heads, n_q] if want_lse)."""
    q = _f32(q)
    k = _f32(k, q.shape)
    v = _f32(v, q.shape)
    n_tok, heads, d = q.shape
    if q_tok is None:
        q_tok = np.arange(n_tok, dtype=np.int64)
    q_tok = np.ascontiguousarray(q_tok, dtype=np.int64)
    out = np.empty((q_tok.size, heads, d), dtype=np.float64)
    lse = np.empty((heads, q_tok.size), dtype=np.float64) if want_lse else None
    _load().gsa_oracle_dense_attn(_ptr(q, _f32p), _ptr(k, _f32p), _ptr(v, _f32p), n_tok, heads, d,
                                  _ptr(q_tok, _i64p), q_tok.size, float(scale), _ptr(out, _f64p),
                                  _ptr(lse, _f64p) if want_lse else None)
    return (out, lse) if want_lse else out


def compressed_attn_tokens(q, kc, vc, scale: float, q_tok=None) -> np.ndarray:
    """Variant of eq. 3 in which the queries are NOT pooled: every token's own query attends the
    pooled keys ("coarse attention of queries against the pooled keys"),
        O_comp[t, h] = sum_j softmax_j(scale * q[t, h] . Kc[h, j]) Vc[h, j].
    The block scores S_guide and TopK stay those of the pooled queries (eq. 4).
    Plain numpy in float64.  Returns [n_q, heads, d] for the tokens q_tok (all if None)."""
    q = np.asarray(_f32(q), dtype=np.float64)
    kc = np.asarray(kc, dtype=np.float64)
    vc = np.asarray(vc, dtype=np.float64)
    if q_tok is None:
        q_tok = np.arange(q.shape[0], dtype=np.int64)
    q_tok = np.asarray(q_tok, dtype=np.int64)
    heads = q.shape[1]
    out = np.empty((q_tok.size, heads, q.shape[2]), dtype=np.float64)
    for h in range(heads):
        logits = scale * (q[q_tok, h, :] @ kc[h].T)                 # [n_q, n_blk]
        logits -= logits.max(axis=1, keepdims=True)
        p = np.exp(logits)
        p /= p.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ vc[h]
    return out


def merge_tokens(oc_tok, o_sel_tok, gate_tok) -> np.ndarray:
    """Eqs. 7, 8 on per-token compressed outputs (no upsampling needed): g * O_comp + (1 - g) * O_sel,
    g = sigmoid(gate logits) or 1/2 when gate_tok is None.  All arrays [m, heads, d]."""
    oc_tok = np.asarray(oc_tok, dtype=np.float64)
    o_sel_tok = np.asarray(o_sel_tok, dtype=np.float64)
    g = 0.5 if gate_tok is None else 1.0 / (1.0 + np.exp(-np.asarray(gate_tok, dtype=np.float64)))
    return g * oc_tok + (1.0 - g) * o_sel_tok


def gsa_forward(q, k, v, block: int, topk_blocks: int, gate=None, scale=None, rows=None,
                idx_override=None, forced=None, token_queries: bool = False) -> dict:
    """The whole GSA path of Sec. 3.2 for the query blocks `rows` (all if None).

    Steps, in the paper's order: pool (compression branch), S_guide (eq. 4),
    compressed attention (eq. 3), TopKSelect, selection attention (eq. 6),
    upsample + gated merge (eqs. 5, 7, 8).  `forced` (ascending block indices) switches
    the selection set to the hybrid of Sec. 3.3: those blocks always, TopK over the
    rest.  `idx_override` replaces the TopK
    result for the selection step (used to score a valid alternative resolution
    of a near-tie).  `token_queries` switches the compression branch's output to the unpooled-query
    variant (compressed_attn_tokens): "out" then has the tokens' own compressed outputs merged in,
    "o_comp_tok" holds them ([n_rows, block, heads, d], zero beyond n_tok) and "o_comp" remains the
    pooled-query result.  Returns every intermediate."""
    q = _f32(q)
    n_tok, heads, d = q.shape
    n_blk = n_blocks(n_tok, block)
    kk = min(int(topk_blocks), n_blk)
    if scale is None or scale <= 0:
        scale = 1.0 / math.sqrt(d)
    rows = _rows(rows, n_blk)
    qc, kc, vc = pool(q, block), pool(k, block), pool(v, block)
    s = scores(qc, kc, rows)
    oc = compressed_attn(s, vc, scale)
    idx = topk(s, kk) if forced is None else topk_with_forced(s, int(topk_blocks), forced)
    use_idx = idx if idx_override is None else np.ascontiguousarray(idx_override, dtype=np.int32)
    o_sel, lse = select_attn(q, k, v, block, use_idx, scale, rows)
    res = {"qc": qc, "kc": kc, "vc": vc, "s": s, "o_comp": oc, "idx": idx, "o_sel": o_sel,
           "lse": lse, "rows": rows, "k": kk, "scale": scale}
    if not token_queries:
        res["out"] = merge(oc, o_sel, gate, n_tok, block, rows)
        return res
    tok = (rows[:, None] * block + np.arange(block)[None, :]).reshape(-1)
    keep = tok < n_tok
    oc_tok = np.zeros((tok.size, heads, d), dtype=np.float64)
    oc_tok[keep] = compressed_attn_tokens(q, kc, vc, scale, tok[keep])
    out = np.zeros_like(oc_tok)
    g_tok = None if gate is None else _f32(gate, q.shape)[tok[keep]]
    out[keep] = merge_tokens(oc_tok[keep], o_sel.reshape(tok.size, heads, d)[keep], g_tok)
    res["o_comp_tok"] = oc_tok.reshape(rows.size, block, heads, d)
    res["out"] = out.reshape(rows.size, block, heads, d)
    return res


def rows_to_tokens(x_rows, rows, n_tok: int, block: int):
    """Flatten a [n_rows, block, ...] result to its valid tokens.

    Returns (token_ids int64 [m], values [m, ...]) in the order of `rows`."""
    rows = np.asarray(rows, dtype=np.int64)
    tok = (rows[:, None] * block + np.arange(block)[None, :]).reshape(-1)
    vals = np.asarray(x_rows).reshape((tok.size,) + tuple(np.asarray(x_rows).shape[2:]))
    keep = tok < n_tok
    return tok[keep], vals[keep]


def token_partition(n_tok: int, tokens_per_view: int, special_per_view: int):
    """Row indices (spec_rows, img_rows) of the special and image tokens of a sequence made of
    views of `tokens_per_view` rows whose first `special_per_view` rows are special tokens
    (camera / register tokens, Sec. 3.2 eq. 1; one view holding everything is the paper's own
    [X_spec; X_img] arrangement)."""
    assert tokens_per_view > 0 and n_tok % tokens_per_view == 0
    assert 0 <= special_per_view < tokens_per_view
    pos = np.arange(n_tok, dtype=np.int64) % tokens_per_view
    return np.nonzero(pos < special_per_view)[0], np.nonzero(pos >= special_per_view)[0]


def gsa_layer(q, k, v, block: int, topk_blocks: int, tokens_per_view: int, special_per_view: int,
              gate=None, scale=None, rows=None, forced=None, idx_override=None) -> dict:
    """The whole layer of Sec. 3.2 on a sequence holding special and image tokens.

    Special tokens: plain softmax attention over ALL tokens (eq. 2).  Image tokens: the sparse
    two-branch path (eqs. 3-8) among the image tokens only, taken in their original order
    (`rows`, `forced`, `idx_override` refer to blocks of that image-only sequence).  The
    results go back to the rows they came from ("concatenating ... in their original order").

    Returns {"spec_rows", "o_spec" [n_spec, heads, d], "img_rows", "img": gsa_forward's
    dictionary on the image tokens, "out" [n_tok, heads, d] (only when rows is None)}."""
    q = _f32(q)
    k = _f32(k, q.shape)
    v = _f32(v, q.shape)
    n_tok, heads, d = q.shape
    if scale is None or scale <= 0:
        scale = 1.0 / math.sqrt(d)
    spec_rows, img_rows = token_partition(n_tok, tokens_per_view, special_per_view)
    o_spec = dense_attn(q, k, v, scale, q_tok=spec_rows) if spec_rows.size else np.zeros((0, heads, d))
    g_img = None if gate is None else _f32(gate, q.shape)[img_rows]
    img = gsa_forward(q[img_rows], k[img_rows], v[img_rows], block, topk_blocks, gate=g_img, scale=scale,
                      rows=rows, forced=forced, idx_override=idx_override)
    res = {"spec_rows": spec_rows, "o_spec": o_spec, "img_rows": img_rows, "img": img}
    if rows is None:
        out = np.empty((n_tok, heads, d), dtype=np.float64)
        out[spec_rows] = o_spec
        tok, vals = rows_to_tokens(img["out"], img["rows"], img_rows.size, block)
        out[img_rows[tok]] = vals
        res["out"] = out
    return res


def window_blocks(views: int, tokens_per_view: int, special_per_view: int, grid_h: int, grid_w: int,
                  window: int):
    """Rows of each spatial pooling window (Sec. 3.2: non-overlapping s x s average pooling on
    every image's patch grid).  A view is `special_per_view` special rows followed by the
    grid_h x grid_w patch tokens in row-major order.  Windows tile the grid from the top left;
    those on the right and bottom edges are cut where the grid ends (the paper leaves this
    case open).  Returns a list over (view, window row, window column) of int64 arrays of
    row numbers, each window's cells in row-major order."""
    assert tokens_per_view == special_per_view + grid_h * grid_w
    blocks = []
    for view in range(views):
        base = view * tokens_per_view + special_per_view
        for y0 in range(0, grid_h, window):
            for x0 in range(0, grid_w, window):
                rows = [base + y * grid_w + x
                        for y in range(y0, min(y0 + window, grid_h))
                        for x in range(x0, min(x0 + window, grid_w))]
                blocks.append(np.asarray(rows, dtype=np.int64))
    return blocks


def gsa_forward_blocks(q, k, v, blocks, topk_blocks: int, gate=None, scale=None, forced=None,
                       idx_override=None) -> dict:
    """The sparse two-branch path (eqs. 3-8) for pooling blocks given as explicit lists of rows
    (any lengths >= 1), written out in numpy without any blocking: block means, S_guide,
    softmax over the pooled keys, TopK (ties to the smaller index; `forced` blocks always taken
    and out of the competition), per-row softmax over the tokens of the selected blocks, gated
    merge.  Returns {"idx" [heads, n_blk, w], "o_comp" [heads, n_blk, d], "out", "o_sel"
    [n_tok, heads, d], "lse" [heads, n_tok] (rows outside every block are NaN),
    "s" [heads, n_blk, n_blk]}."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    n_tok, heads, d = q.shape
    n_blk = len(blocks)
    if scale is None or scale <= 0:
        scale = 1.0 / math.sqrt(d)
    qc = np.stack([q[b].mean(axis=0) for b in blocks], axis=1)          # [heads, n_blk, d]
    kc = np.stack([k[b].mean(axis=0) for b in blocks], axis=1)
    vc = np.stack([v[b].mean(axis=0) for b in blocks], axis=1)
    s = np.einsum("hid,hjd->hij", qc, kc)                               # eq. 4
    z = scale * s
    p = np.exp(z - z.max(axis=2, keepdims=True))
    o_comp = np.einsum("hij,hjd->hid", p / p.sum(axis=2, keepdims=True), vc)   # eq. 3
    forced = np.asarray([] if forced is None else forced, dtype=np.int64)
    k_dyn = min(int(topk_blocks), n_blk - forced.size)
    idx = np.empty((heads, n_blk, forced.size + k_dyn), dtype=np.int32)
    free = np.setdiff1d(np.arange(n_blk), forced)
    for h in range(heads):
        for i in range(n_blk):
            order = sorted(free, key=lambda j: (-s[h, i, j], j))[:k_dyn]
            idx[h, i] = np.sort(np.concatenate([forced, np.asarray(order, dtype=np.int64)]))
    use = idx if idx_override is None else np.asarray(idx_override)
    out = np.full((n_tok, heads, d), np.nan)
    o_sel = np.full((n_tok, heads, d), np.nan)
    lse = np.full((heads, n_tok), np.nan)
    for h in range(heads):
        for i, rows in enumerate(blocks):
            keys = np.concatenate([blocks[j] for j in use[h, i]])
            logit = scale * (q[rows, h] @ k[keys, h].T)                  # eq. 6
            mx = logit.max(axis=1, keepdims=True)
            w = np.exp(logit - mx)
            o = (w / w.sum(axis=1, keepdims=True)) @ v[keys, h]
            o_sel[rows, h] = o
            lse[h, rows] = mx[:, 0] + np.log(w.sum(axis=1))              # Alg. 2's L
            g = 0.5 if gate is None else 1.0 / (1.0 + np.exp(-np.asarray(gate, dtype=np.float64)[rows, h]))
            out[rows, h] = g * o_comp[h, i][None, :] + (1.0 - g) * o      # eqs. 5, 7, 8
    return {"idx": idx, "o_comp": o_comp, "out": out, "o_sel": o_sel, "lse": lse, "s": s}
