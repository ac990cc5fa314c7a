"""Helpers of the GPU parity tests: tolerances, the TopK acceptance rule, and a driver that runs
the device path through the C ABI binding and the fp64 oracle on the same inputs."""
from __future__ import annotations

import math
import sys
import time

import numpy as np
import torch

# Output tolerance: max relative error, bf16 I/O 2e-2, fp32 I/O 1e-4.  The error of an element is
# |gpu - ref| / max(|ref|, rms(ref)).  Every output here is a softmax-weighted average
# o_c = sum_u p_u v_uc; rounding p (and v) perturbs it by at most eps * sum_u p_u |v_uc|, a quantity
# of the order of the tensor's RMS whatever the size of o_c itself, so an element that happens to
# lie near zero is judged against the RMS, a large one against itself.  (Plain element-wise
# relative error is unbounded at the zero crossings of the reference.)  The global form
# max|gpu - ref| / max|ref| is reported too and must pass as well.
TOL = {"bf16": 2e-2, "f32": 1e-4}
# Near-tie rule for TopK: with tau the oracle's k-th largest score and s_next the (k+1)-th,
# delta = 1e-3 * max(|tau|, |s_next|, 1e-30).  A device index set is valid iff it has k distinct
# in-range indices, holds every j with S > tau + delta and none with S < tau - delta.  When
# tau - s_next > delta this forces the oracle's exact set.
TIE_REL = 1e-3


def log(msg):
    print(f"[parity {time.strftime('%H:%M:%S')}] {msg}", flush=True)
    sys.stdout.flush()


def rel_errors(gpu, ref):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape, (gpu.shape, ref.shape)
    if ref.size == 0:
        return 0.0, 0.0
    assert np.isfinite(gpu).all(), "non-finite values in the device result"
    diff = np.abs(gpu - ref)
    rms = math.sqrt(float(np.mean(ref * ref)))
    floor = max(rms, 1e-30)
    elem = float(np.max(diff / np.maximum(np.abs(ref), floor)))
    glob = float(np.max(diff) / max(float(np.max(np.abs(ref))), 1e-30))
    return elem, glob


def strict_errors(gpu, ref):
    """The element-wise relative error with the denominator floored at 1e-2 * rms(ref) instead of rms(ref):
    (max, 99.9th percentile).  Reported beside the gated figure, never gated on: an element a hundred
    times smaller than the tensor's RMS carries the same absolute rounding error as any other (the error
    of a softmax average scales with the RMS of the values averaged), so its ratio is up to 100 times
    the gated one by construction."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0, 0.0
    rms = math.sqrt(float(np.mean(ref * ref)))
    r = np.abs(gpu - ref) / np.maximum(np.abs(ref), max(1e-2 * rms, 1e-30))
    return float(np.max(r)), float(np.quantile(r, 0.999))


def assert_close(gpu, ref, tol, what):
    elem, glob = rel_errors(gpu, ref)
    assert elem <= tol and glob <= tol, f"{what}: rel err elem {elem:.3e} glob {glob:.3e} > {tol:.1e}"
    return elem


def check_topk_sets_fast(s_rows, gpu_idx, k):
    """check_topk_sets for many rows: rows whose device set equals the oracle's own choice (stable sort:
    equal scores go to the smaller index) are counted at once, the others go through the near-tie rule
    one by one.  Returns (n_exact, n_tie_resolved)."""
    H, R, n_blk = s_rows.shape
    assert gpu_idx.shape == (H, R, k), (gpu_idx.shape, (H, R, k))
    want = np.sort(np.argsort(-s_rows, axis=-1, kind="stable")[..., :k], axis=-1)
    same = (want == gpu_idx).all(axis=-1)
    n_tie = 0
    for h, r in zip(*np.nonzero(~same)):
        e, t = check_topk_sets(s_rows[h:h + 1, r:r + 1], gpu_idx[h:h + 1, r:r + 1], k)
        assert e == 0 and t == 1
        n_tie += 1
    return int(same.sum()), n_tie


def check_topk_sets(s_rows, gpu_idx, k):
    """s_rows [H, R, n_blk] oracle scores, gpu_idx [H, R, k].  Asserts validity of every set under
    the near-tie rule; returns (n_exact, n_tie_resolved) against the oracle's own choice."""
    H, R, n_blk = s_rows.shape
    assert gpu_idx.shape == (H, R, k), (gpu_idx.shape, (H, R, k))
    n_exact = n_tie = 0
    for h in range(H):
        for r in range(R):
            s = s_rows[h, r]
            got = gpu_idx[h, r]
            assert np.all(np.diff(got) > 0), f"indices not strictly ascending at h={h} r={r}: {got}"
            assert got[0] >= 0 and got[-1] < n_blk, f"index out of range at h={h} r={r}"
            order = np.lexsort((np.arange(n_blk), -s))          # score desc, then index asc
            want = np.sort(order[:k])
            if np.array_equal(want, got):
                n_exact += 1
                continue
            tau = s[order[k - 1]]
            s_next = s[order[k]] if k < n_blk and np.isfinite(s[order[k]]) else tau
            delta = TIE_REL * max(abs(tau), abs(s_next), 1e-30)
            chosen = np.zeros(n_blk, dtype=bool)
            chosen[got] = True
            must = s > tau + delta
            never = s < tau - delta
            assert not np.any(must & ~chosen), (
                f"h={h} r={r}: device set misses a block above the tie band "
                f"(tau={tau:.6g}, delta={delta:.3g}, missing={np.where(must & ~chosen)[0][:5]})")
            assert not np.any(never & chosen), (
                f"h={h} r={r}: device set holds a block below the tie band "
                f"(tau={tau:.6g}, delta={delta:.3g}, bad={np.where(never & chosen)[0][:5]})")
            n_tie += 1
    return n_exact, n_tie


def to_host_f32(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a (bf16 / fp32) tensor to a float32 numpy array on the host."""
    return t.detach().to("cpu").to(torch.float32).numpy()


def run_device(s3r, q, k, v, block, topk, gate=None, scale=0.0, want=("idx", "lse", "o_comp", "o_sel"),
               forced=None, tokens_per_view=0, special_per_view=0, grid=None, compress_queries=0):
    """One call of the whole path through the C ABI; returns device tensors.  `forced`: ascending
    block indices (host array) every query block attends besides its TopK.  With special tokens
    the block-level outputs are sized for the image-only sequence."""
    n_tok, heads, d = q.shape
    n_forced = 0 if forced is None else len(forced)
    dt_code = s3r.S3R_BF16 if q.dtype == torch.bfloat16 else s3r.S3R_F32
    n_blk = s3r.speed3r_num_blocks(n_tok, heads, d, block, topk, dt_code, tokens_per_view, special_per_view, grid)
    kk = s3r.speed3r_selected_per_row(n_blk * block, block, topk, n_forced)
    dev = q.device
    out = torch.full(q.shape, float("nan"), dtype=q.dtype, device=dev)     # packed whatever the strides of q
    bufs = {}
    if "idx" in want:
        bufs["topk_idx"] = torch.full((heads, n_blk, kk), -1, dtype=torch.int32, device=dev)
    if "lse" in want:
        bufs["lse_sel"] = torch.full((heads, n_tok), float("nan"), dtype=torch.float32, device=dev)
    if "o_comp" in want:
        bufs["o_comp"] = torch.full((heads, n_blk, d), float("nan"), dtype=torch.float32, device=dev)
    if "o_sel" in want:
        bufs["o_sel"] = torch.full(q.shape, float("nan"), dtype=q.dtype, device=dev)
    forced_t = None if n_forced == 0 else torch.from_numpy(np.asarray(forced, dtype=np.int32)).to(dev)
    s3r.speed3r_sparse_global_attn_ex(q, k, v, out, block, topk, gate_logits=gate,
                                      softmax_scale=scale, forced_blocks=forced_t,
                                      tokens_per_view=tokens_per_view, special_per_view=special_per_view,
                                      grid=grid, compress_queries=compress_queries, **bufs)
    torch.cuda.synchronize()
    res = {"out": out}
    res.update({"idx": bufs.get("topk_idx"), "lse": bufs.get("lse_sel"),
                "o_comp": bufs.get("o_comp"), "o_sel": bufs.get("o_sel")})
    return res


def compare_with_oracle(oracle, dev_res, qf, kf, vf, gate_f, block, topk, dtype, rows=None, scale=None,
                        label="", forced=None, token_queries=False):
    """Element-by-element comparison of a device result (tensors from run_device) with the oracle
    on the query blocks `rows` (all when None).  qf, kf, vf, gate_f: host float32 arrays holding
    exactly the device inputs.  TopK sets are checked with the near-tie rule; selection outputs are
    compared against the oracle evaluated on the device's (validated) index sets.  With `forced`
    blocks every device set must hold them all, and what remains is checked as the TopK of the
    scores with the forced columns removed from the competition.  `token_queries`: the merged output
    is checked against the variant whose compression branch keeps every token's own query."""
    n_tok, heads, d = qf.shape
    n_blk = (n_tok + block - 1) // block
    kk = min(topk, n_blk)
    tol = TOL[dtype]
    if scale is None or scale <= 0:
        scale = 1.0 / math.sqrt(d)
    rows = np.arange(n_blk, dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    qc, kc, vc = oracle.pool(qf, block), oracle.pool(kf, block), oracle.pool(vf, block)
    s = oracle.scores(qc, kc, rows)
    o_comp = oracle.compressed_attn(s, vc, scale)
    stats = {}

    def tok_sel(x):          # device tensor [n_tok, ...] -> valid tokens of `rows` (rows order), host f32
        tok = (rows[:, None] * block + np.arange(block)[None, :]).reshape(-1)
        tok_t = torch.from_numpy(tok[tok < n_tok]).to(x.device)
        return to_host_f32(x.index_select(0, tok_t))

    if dev_res.get("o_comp") is not None:
        g = dev_res["o_comp"][:, torch.from_numpy(rows).to(dev_res["o_comp"].device)].cpu().numpy()
        stats["o_comp"] = assert_close(g, o_comp, tol, f"{label} o_comp")
    assert dev_res.get("idx") is not None
    gidx = dev_res["idx"][:, torch.from_numpy(rows).to(dev_res["idx"].device)].cpu().numpy()
    if forced is None or len(forced) == 0:
        n_exact, n_tie = check_topk_sets(s, gidx, kk)
    else:
        forced = np.asarray(forced, dtype=np.int64)
        k_dyn = min(topk, n_blk - forced.size)
        assert gidx.shape[2] == forced.size + k_dyn, (gidx.shape, forced.size, k_dyn)
        assert np.all(np.diff(gidx, axis=2) > 0), "united index sets not strictly ascending"
        assert gidx.min() >= 0 and gidx.max() < n_blk
        is_forced = np.isin(gidx, forced)
        assert np.all(is_forced.sum(axis=2) == forced.size), "a forced block is missing from a device set"
        n_exact = n_tie = 0
        if k_dyn > 0:
            dyn = gidx[~is_forced].reshape(gidx.shape[0], gidx.shape[1], k_dyn)
            s_free = s.copy()
            s_free[:, :, forced] = -np.inf
            n_exact, n_tie = check_topk_sets(s_free, dyn, k_dyn)
            want = oracle.topk_with_forced(s, topk, forced)
            if n_tie == 0:
                assert np.array_equal(want, gidx)
    stats["topk_exact"], stats["topk_tie_resolved"] = n_exact, n_tie
    o_sel, lse = oracle.select_attn(qf, kf, vf, block, gidx, scale, rows)
    out = oracle.merge(o_comp, o_sel, gate_f, n_tok, block, rows)
    _, o_sel_v = oracle.rows_to_tokens(o_sel, rows, n_tok, block)
    _, out_v = oracle.rows_to_tokens(out, rows, n_tok, block)
    _, lse_v = oracle.rows_to_tokens(lse.transpose(1, 2, 0), rows, n_tok, block)      # [m, H]
    if dev_res.get("o_sel") is not None:
        stats["o_sel"] = assert_close(tok_sel(dev_res["o_sel"]), o_sel_v, tol, f"{label} o_sel")
    if dev_res.get("lse") is not None:
        g = tok_sel(dev_res["lse"].T)
        # L is a logarithm: compare absolutely (an absolute error in L is a relative error in exp L)
        err = float(np.max(np.abs(g - lse_v)))
        assert err <= tol, f"{label} lse abs err {err:.3e} > {tol:.1e}"
        stats["lse_abs"] = err
    if token_queries:
        tok = (rows[:, None] * block + np.arange(block)[None, :]).reshape(-1)
        tok = tok[tok < n_tok]
        oc_tok = oracle.compressed_attn_tokens(qf, kc, vc, scale, tok)
        out_v = oracle.merge_tokens(oc_tok, o_sel_v, None if gate_f is None else gate_f[tok])
    got_out = tok_sel(dev_res["out"])
    stats["out"] = assert_close(got_out, out_v, tol, f"{label} out")
    stats["out_strict_max"], stats["out_strict_p999"] = strict_errors(got_out, out_v)
    return stats


def compare_layer_with_oracle(oracle, dev_res, qf, kf, vf, gate_f, block, topk, dtype, tokens_per_view,
                              special_per_view, rows=None, spec_sample=None, forced=None, label="",
                              token_queries=False):
    """Layer with special tokens: the image rows go through compare_with_oracle on the image-only
    sequence (device outputs gathered from their original rows), the special rows (all, or the
    sample `spec_sample` of them) against the oracle's dense attention over every row."""
    n_tok = qf.shape[0]
    spec_rows, img_rows = oracle.token_partition(n_tok, tokens_per_view, special_per_view)
    img_t = torch.from_numpy(img_rows).to(dev_res["out"].device)
    sub = dict(dev_res)
    sub["out"] = dev_res["out"].index_select(0, img_t)
    if dev_res.get("o_sel") is not None:
        sub["o_sel"] = dev_res["o_sel"].index_select(0, img_t)
    if dev_res.get("lse") is not None:
        sub["lse"] = dev_res["lse"].index_select(1, img_t).contiguous()
    stats = compare_with_oracle(oracle, sub, qf[img_rows], kf[img_rows], vf[img_rows],
                                None if gate_f is None else gate_f[img_rows], block, topk, dtype, rows=rows,
                                label=label, forced=forced, token_queries=token_queries)
    pick = spec_rows if spec_sample is None else spec_rows[np.asarray(spec_sample, dtype=np.int64)]
    if pick.size:
        ref = oracle.dense_attn(qf, kf, vf, 1.0 / math.sqrt(qf.shape[2]), q_tok=pick)
        got = to_host_f32(dev_res["out"].index_select(0, torch.from_numpy(pick).to(dev_res["out"].device)))
        stats["o_spec"] = assert_close(got, ref, TOL[dtype], f"{label} special rows")
    return stats


def compare_windows_with_oracle(oracle, dev_res, qf, kf, vf, gate_f, topk, dtype, views, tokens_per_view,
                                special_per_view, grid, forced=None, label="", token_queries=False):
    """Blocks = spatial windows: everything against the oracle's explicit-rows route (all rows; sizes
    are kept small), special rows against its dense attention."""
    grid_h, grid_w, window = grid
    tol = TOL[dtype]
    blocks = oracle.window_blocks(views, tokens_per_view, special_per_view, grid_h, grid_w, window)
    ref = oracle.gsa_forward_blocks(qf, kf, vf, blocks, topk, gate=gate_f, forced=forced)
    gidx = dev_res["idx"].cpu().numpy()
    n_blk = len(blocks)
    stats = {}
    if forced is None or len(forced) == 0:
        stats["topk_exact"], stats["topk_tie_resolved"] = check_topk_sets(ref["s"], gidx, min(topk, n_blk))
    else:
        forced = np.asarray(forced, dtype=np.int64)
        is_forced = np.isin(gidx, forced)
        assert np.all(is_forced.sum(axis=2) == forced.size)
        k_dyn = min(topk, n_blk - forced.size)
        s_free = ref["s"].copy()
        s_free[:, :, forced] = -np.inf
        dyn = gidx[~is_forced].reshape(gidx.shape[0], gidx.shape[1], k_dyn)
        stats["topk_exact"], stats["topk_tie_resolved"] = (check_topk_sets(s_free, dyn, k_dyn) if k_dyn > 0
                                                           else (0, 0))     # every block forced
    if stats["topk_tie_resolved"]:
        ref = oracle.gsa_forward_blocks(qf, kf, vf, blocks, topk, gate=gate_f, forced=forced, idx_override=gidx)
    img_rows = np.concatenate(blocks)
    if token_queries:
        kc = np.stack([kf[b].astype(np.float64).mean(axis=0) for b in blocks], axis=1)
        vc = np.stack([vf[b].astype(np.float64).mean(axis=0) for b in blocks], axis=1)
        oc_tok = oracle.compressed_attn_tokens(qf, kc, vc, 1.0 / math.sqrt(qf.shape[2]), img_rows)
        ref["out"][img_rows] = oracle.merge_tokens(oc_tok, ref["o_sel"][img_rows],
                                                   None if gate_f is None else gate_f[img_rows])
    stats["o_comp"] = assert_close(dev_res["o_comp"].cpu().numpy(), ref["o_comp"], tol, f"{label} o_comp")
    take = torch.from_numpy(img_rows).to(dev_res["out"].device)
    stats["o_sel"] = assert_close(to_host_f32(dev_res["o_sel"].index_select(0, take)), ref["o_sel"][img_rows], tol,
                                  f"{label} o_sel")
    stats["out"] = assert_close(to_host_f32(dev_res["out"].index_select(0, take)), ref["out"][img_rows], tol,
                                f"{label} out")
    err = float(np.max(np.abs(dev_res["lse"].index_select(1, take).cpu().numpy() - ref["lse"][:, img_rows])))
    assert err <= tol, f"{label} lse abs err {err:.3e}"
    stats["lse_abs"] = err
    spec_rows, _ = oracle.token_partition(qf.shape[0], tokens_per_view, special_per_view)
    if spec_rows.size:
        dense = oracle.dense_attn(qf, kf, vf, 1.0 / math.sqrt(qf.shape[2]), q_tok=spec_rows)
        got = to_host_f32(dev_res["out"].index_select(0, torch.from_numpy(spec_rows).to(dev_res["out"].device)))
        stats["o_spec"] = assert_close(got, dense, tol, f"{label} special rows")
    return stats
