"""GPU parity: the HIP path, called through the C ABI binding, against the fp64 CPU oracle on the
same seeded inputs -- stage by stage and end to end.  Run with `-m gpu` on an MI355X."""
import math

import numpy as np
import pytest
import torch

from paper_2603_08055_amd import workloads
from tests.parity_util import (TOL, assert_close, check_topk_sets, compare_layer_with_oracle, compare_windows_with_oracle,
                               compare_with_oracle, log,
                               rel_errors, run_device, to_host_f32)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def s3r():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2603_08055_amd import speed3r
    speed3r.load()          # raises if libspeed3r.so is missing: there is no fallback
    return speed3r


def draw(n_tok, heads, dtype, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    x = torch.randn((n_tok, heads, 64), generator=g) * scale
    return x.to(torch.bfloat16 if dtype == "bf16" else torch.float32)


# ------------------------------------------------------------------------------- stage: pool --

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n_tok,block", [(1024, 64), (1000, 64), (333, 16), (333, 32), (700, 128),
                                         (1, 64), (129, 128)])
def test_pool_blocks(s3r, oracle, dtype, n_tok, block):
    heads = 3
    q, k, v = (draw(n_tok, heads, dtype, 100 + i) for i in range(3))
    n_blk = (n_tok + block - 1) // block
    outs = [torch.full((heads, n_blk, 64), float("nan"), device="cuda") for _ in range(3)]
    s3r.speed3r_pool_blocks(q.cuda(), k.cuda(), v.cuda(), *outs, block)
    torch.cuda.synchronize()
    for x, got in zip((q, k, v), outs):
        ref = oracle.pool(to_host_f32(x), block)
        # fp32 accumulation of <= 128 terms: ~1e-7 of mean|x| absolute, far inside the fp32 output bound
        assert_close(got.cpu().numpy(), ref, TOL["f32"], f"pool {dtype} n={n_tok} B={block}")
        assert rel_errors(got.cpu().numpy(), ref)[1] <= 2e-6


# --------------------------------------------------------------------- stage: compress/score --

@pytest.mark.parametrize("n_blk,heads,accurate", [(16, 2, True), (172, 4, False), (172, 4, True),
                                                  (300, 2, True), (1, 1, True), (33, 3, False),
                                                  (2147, 2, False)])
def test_compress_attn_scores(s3r, oracle, n_blk, heads, accurate):
    rng = np.random.default_rng(7 + n_blk)
    qc = (rng.standard_normal((heads, n_blk, 64)) * 0.5).astype(np.float32)
    kc = (rng.standard_normal((heads, n_blk, 64)) * 0.5).astype(np.float32)
    vc = rng.standard_normal((heads, n_blk, 64)).astype(np.float32)
    ld_s = (n_blk + 3) // 4 * 4
    s_dev = torch.full((heads, n_blk, ld_s), float("nan"), device="cuda")
    oc_dev = torch.full((heads, n_blk, 64), float("nan"), device="cuda")
    scale = 0.125
    s3r.speed3r_compress_attn_scores(torch.from_numpy(qc).cuda(), torch.from_numpy(kc).cuda(),
                                     torch.from_numpy(vc).cuda(), s_dev, oc_dev, scale, accurate)
    torch.cuda.synchronize()
    s_ref = oracle.scores(qc, kc)
    oc_ref = oracle.compressed_attn(s_ref, vc, scale)
    s_got = s_dev.cpu().numpy()[:, :, :n_blk]
    # scores: hi/lo bf16 operand pairs -> error ~2^-16 of |q||k| per row/column pair
    bound = 4e-5 * np.linalg.norm(qc, axis=2)[:, :, None] * np.linalg.norm(kc, axis=2)[:, None, :]
    assert np.all(np.abs(s_got - s_ref) <= bound + 1e-7), float(np.max(np.abs(s_got - s_ref) / (bound + 1e-7)))
    assert_close(oc_dev.cpu().numpy(), oc_ref, 1e-4 if accurate else 2e-2, f"o_comp n_blk={n_blk}")


# ------------------------------------------------------------------------------- stage: topk --

def topk_case(s3r, oracle, s_np, k):
    heads, n_blk, _ = s_np.shape
    ld_s = (n_blk + 3) // 4 * 4
    s_dev = torch.zeros((heads, n_blk, ld_s), device="cuda")
    s_dev[:, :, :n_blk] = torch.from_numpy(s_np).cuda()
    s_dev[:, :, n_blk:] = 1e30          # the padding columns must never be selected
    kk = min(k, n_blk)
    idx = torch.full((heads, n_blk, kk), -1, dtype=torch.int32, device="cuda")
    s3r.speed3r_topk_blocks(s_dev, idx, n_blk, k)
    torch.cuda.synchronize()
    ref = oracle.topk(s_np.astype(np.float64), kk)
    assert np.array_equal(idx.cpu().numpy(), ref)       # integer work: bit-exact, ties included


@pytest.mark.parametrize("n_blk,k", [(16, 4), (172, 16), (300, 1), (300, 300), (300, 1000), (257, 256),
                                     (700, 300), (5, 3), (1, 1), (2147, 32), (4100, 64)])
def test_topk_random_rows(s3r, oracle, n_blk, k):
    rng = np.random.default_rng(n_blk * 31 + k)
    heads = 2
    rows = min(n_blk, 64)
    s = rng.standard_normal((heads, n_blk, n_blk)).astype(np.float32)
    s[:, rows:] = s[:, :1]              # keep the oracle's sort work small: repeat one row
    topk_case(s3r, oracle, s, k)


@pytest.mark.parametrize("n_blk,k", [(300, 16), (2000, 64), (2000, 300), (64, 64)])
def test_topk_ties_and_degenerate_rows(s3r, oracle, n_blk, k):
    rng = np.random.default_rng(n_blk + k)
    s = np.zeros((1, n_blk, n_blk), dtype=np.float32)
    s[0, 0] = 0.0                                               # all equal -> first k indices
    s[0, 1] = rng.integers(0, 3, n_blk)                          # three distinct values, many ties
    s[0, 2] = -np.arange(n_blk)                                  # descending: first k
    s[0, 3] = np.arange(n_blk)                                   # ascending: last k
    s[0, 4] = np.where(np.arange(n_blk) % 2 == 0, -0.0, 0.0)     # signed zeros compare equal
    s[0, 5] = rng.integers(0, 2, n_blk) * 1e-30                  # tiny values
    s[0, 6] = np.where(np.arange(n_blk) % 256 < 3, 5.0, rng.standard_normal(n_blk))  # stride-256 pattern
    s[0, 7] = -np.abs(rng.standard_normal(n_blk)) * 1e20         # all negative, large
    for r in range(8, n_blk):
        s[0, r] = s[0, r % 8]
    topk_case(s3r, oracle, s, k)


# ----------------------------------------------------------------------------- stage: select --

def select_case(s3r, oracle, dtype, n_tok, heads, block, kk, choice, with_gate, seed):
    s3r.speed3r_set_kernel_choice(choice)
    try:
        q, k, v = (draw(n_tok, heads, dtype, seed + i, 1.0 if i else 0.7) for i in range(3))
        n_blk = (n_tok + block - 1) // block
        rng = np.random.default_rng(seed)
        idx = np.stack([[np.sort(rng.choice(n_blk, kk, replace=False)) for _ in range(n_blk)]
                        for _ in range(heads)]).astype(np.int32)
        idx[:, 0, -1] = n_blk - 1                                    # make sure the tail block is used
        idx[:, 0] = np.sort(idx[:, 0], axis=-1)
        for h in range(heads):                                       # keep rows duplicate-free
            if len(set(idx[h, 0])) < kk:
                idx[h, 0] = np.arange(n_blk - kk, n_blk)
        gate = draw(n_tok, heads, dtype, seed + 9) if with_gate else None
        oc = torch.randn((heads, n_blk, 64), generator=torch.Generator().manual_seed(seed + 5))
        out = torch.full_like(q, float("nan")).cuda()
        o_sel = torch.full_like(q, float("nan")).cuda()
        lse = torch.full((heads, n_tok), float("nan"), device="cuda")
        s3r.speed3r_select_attn(q.cuda(), k.cuda(), v.cuda(), torch.from_numpy(idx).cuda(), out, block,
                                o_comp=oc.cuda(), gate_logits=None if gate is None else gate.cuda(),
                                o_sel=o_sel, lse=lse)
        torch.cuda.synchronize()
        qf, kf, vf = (to_host_f32(x) for x in (q, k, v))
        scale = 1 / math.sqrt(64)
        ref_sel, ref_lse = oracle.select_attn(qf, kf, vf, block, idx, scale)
        ref_out = oracle.merge(oc.numpy().astype(np.float64), ref_sel,
                               None if gate is None else to_host_f32(gate), n_tok, block)
        rows = np.arange(n_blk)
        _, sel_v = oracle.rows_to_tokens(ref_sel, rows, n_tok, block)
        _, out_v = oracle.rows_to_tokens(ref_out, rows, n_tok, block)
        _, lse_v = oracle.rows_to_tokens(ref_lse.transpose(1, 2, 0), rows, n_tok, block)
        tol = TOL[dtype]
        label = f"select {dtype} n={n_tok} B={block} k={kk} choice={choice}"
        assert_close(to_host_f32(o_sel), sel_v, tol, label + " o_sel")
        assert_close(to_host_f32(out), out_v, tol, label + " out")
        assert float(np.max(np.abs(lse.cpu().numpy().T - lse_v))) <= tol, label + " lse"
    finally:
        s3r.speed3r_set_kernel_choice(0)


@pytest.mark.parametrize("block,n_tok,kk", [(64, 1024, 4), (64, 1000, 5), (128, 1100, 3), (64, 64, 1),
                                            (128, 2000, 16), (64, 2500, 40),
                                            # blocks of 16 / 32 tokens: units put together from 4 / 2 blocks
                                            (16, 1024, 8), (16, 1000, 7), (16, 200, 5), (16, 16, 1), (16, 37, 3),
                                            (32, 1024, 6), (32, 333, 4), (32, 1000, 3), (32, 40, 2), (16, 3000, 32)])
@pytest.mark.parametrize("with_gate", [False, True])
def test_select_attn_mfma_bf16(s3r, oracle, block, n_tok, kk, with_gate):
    select_case(s3r, oracle, "bf16", n_tok, 3, block, kk, 0, with_gate, 1000 + n_tok)


@pytest.mark.parametrize("block,n_tok,kk", [(64, 1024, 4), (64, 1000, 5), (128, 1100, 3), (64, 64, 1),
                                            (128, 2000, 16), (64, 2500, 40),
                                            (16, 1000, 7), (16, 37, 3), (32, 333, 4), (32, 1024, 6)])
@pytest.mark.parametrize("with_gate", [False, True])
def test_select_attn_mfma_f32(s3r, oracle, block, n_tok, kk, with_gate):
    """fp32 problems run on the matrix cores with K, V, Q and P in bf16 operand parts and must stay within the
    fp32 tolerance."""
    select_case(s3r, oracle, "f32", n_tok, 3, block, kk, 0, with_gate, 1000 + n_tok)


@pytest.mark.parametrize("kk,rising", [(41, False), (64, False), (40, True), (97, False), (128, True)])
def test_select_attn_long_rows_on_long_sequences(s3r, oracle, kk, rising):
    """Rows of 40 or more blocks on sequences of 3000 or more blocks of 64 tokens run with two pairs of waves
    per query block, each pair on every second unit of the list, their two partial softmaxes combined at
    the end (eq. 6 over all selected keys): odd and even row lengths, a ragged last block, gate and merge,
    and (rising) logits that grow along the list so that both pairs keep raising their running maxima.
    Sampled query blocks against the oracle."""
    block, heads = 64, 2
    n_blk = 3001
    n_tok = n_blk * block - 17
    g = torch.Generator().manual_seed(1000 + kk)
    q, k, v = (torch.randn((n_tok, heads, 64), generator=g) for _ in range(3))
    if rising:
        q, k = 0.05 * q, 0.05 * k
        q[:, :, 0] = 4.0
        k[:, :, 0] = torch.arange(n_tok, dtype=torch.float32)[:, None] / 256.0       # logits grow by 8 per 64 x 64 keys
    q, k, v = (x.to(torch.bfloat16) for x in (q, k, v))
    gate = torch.randn((n_tok, heads, 64), generator=g).to(torch.bfloat16)
    oc = torch.randn((heads, n_blk, 64), generator=g)
    rows = np.array([0, 1, 1500, n_blk - 2, n_blk - 1])
    rng = np.random.default_rng(kk)
    idx = np.zeros((heads, n_blk, kk), dtype=np.int32)
    idx[:] = np.sort(rng.choice(n_blk, kk, replace=False))[None, None, :]
    for h in range(heads):
        for r in rows:
            pick = np.sort(rng.choice(n_blk - 1, kk - 1, replace=False))
            idx[h, r] = np.sort(np.concatenate([pick, [n_blk - 1]]))          # the ragged last block in every sampled row
    out = torch.full(q.shape, float("nan"), dtype=q.dtype, device="cuda")
    o_sel = torch.full(q.shape, float("nan"), dtype=q.dtype, device="cuda")
    lse = torch.full((heads, n_tok), float("nan"), device="cuda")
    s3r.speed3r_select_attn(q.cuda(), k.cuda(), v.cuda(), torch.from_numpy(idx).cuda(), out, block, o_comp=oc.cuda(),
                            gate_logits=gate.cuda(), o_sel=o_sel, lse=lse)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()
    qf, kf, vf = (to_host_f32(x) for x in (q, k, v))
    ref_sel, ref_lse = oracle.select_attn(qf, kf, vf, block, idx[:, rows], 0.125, rows)
    ref_out = oracle.merge(oc.numpy().astype(np.float64)[:, rows], ref_sel, to_host_f32(gate), n_tok, block, rows)
    tok, sel_v = oracle.rows_to_tokens(ref_sel, rows, n_tok, block)
    _, out_v = oracle.rows_to_tokens(ref_out, rows, n_tok, block)
    _, lse_v = oracle.rows_to_tokens(ref_lse.transpose(1, 2, 0), rows, n_tok, block)
    take = torch.from_numpy(np.asarray(tok)).cuda()
    assert_close(to_host_f32(o_sel.index_select(0, take)), sel_v, TOL["bf16"], f"o_sel k={kk}")
    assert_close(to_host_f32(out.index_select(0, take)), out_v, TOL["bf16"], f"out k={kk}")
    assert float(np.max(np.abs(lse.index_select(1, take).cpu().numpy().T - lse_v))) <= TOL["bf16"]


@pytest.mark.parametrize("dtype,block", [("bf16", 64), ("bf16", 128), ("bf16", 16), ("bf16", 32), ("f32", 64), ("f32", 16)])
def test_select_attn_holds_out_of_range_indices_in_range(s3r, dtype, block):
    """A caller's index tensor is device memory the library cannot inspect: entries outside [0, n_blk) are held
    into the range by the kernels (the documented behaviour), so the result equals that of the clamped list."""
    n_tok, heads, kk = 21 * block + 5, 2, 6
    n_blk = 22
    q, k, v = (draw(n_tok, heads, dtype, 8800 + i).cuda() for i in range(3))
    rng = np.random.default_rng(block)
    idx = np.stack([[np.sort(rng.choice(n_blk, kk, replace=False)) for _ in range(n_blk)] for _ in range(heads)]).astype(np.int32)
    bad = idx.copy()
    bad[:, ::3, 0] = -7
    bad[:, 1::3, kk - 1] = n_blk + 1000
    bad[0, 5, kk - 1] = 2 ** 30
    good = np.clip(bad, 0, n_blk - 1)
    outs = []
    for lists in (bad, good):
        out = torch.full_like(q, float("nan"))
        s3r.speed3r_select_attn(q, k, v, torch.from_numpy(lists).cuda(), out, block)
        torch.cuda.synchronize()
        outs.append(out)
    assert torch.isfinite(outs[0].float()).all()
    assert torch.equal(outs[0], outs[1])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("block,n_tok,kk", [(16, 200, 5), (32, 333, 4), (64, 1000, 5), (128, 700, 3)])
def test_select_attn_generic(s3r, oracle, dtype, block, n_tok, kk):
    select_case(s3r, oracle, dtype, n_tok, 2, block, kk, 1, True, 2000 + n_tok)


# ------------------------------------------------------------------------------ stage: dense --

@pytest.mark.parametrize("dtype,n_tok,choice", [("bf16", 1024, 0), ("bf16", 1000, 0), ("bf16", 300, 0),
                                                ("bf16", 777, 1), ("f32", 1024, 0), ("f32", 500, 0), ("f32", 777, 1)])   # (dense attention has no block size: 64-key units)
def test_dense_attn(s3r, oracle, dtype, n_tok, choice):
    s3r.speed3r_set_kernel_choice(choice)
    try:
        heads = 2
        q, k, v = (draw(n_tok, heads, dtype, 3000 + i) for i in range(3))
        out = torch.full_like(q, float("nan")).cuda()
        lse = torch.full((heads, n_tok), float("nan"), device="cuda")
        s3r.speed3r_dense_attn(q.cuda(), k.cuda(), v.cuda(), out, lse)
        torch.cuda.synchronize()
        ref, ref_lse = oracle.dense_attn(*(to_host_f32(x) for x in (q, k, v)), 0.125, want_lse=True)
        assert_close(to_host_f32(out), ref, TOL[dtype], f"dense {dtype} n={n_tok}")
        assert float(np.max(np.abs(lse.cpu().numpy() - ref_lse))) <= TOL[dtype]
    finally:
        s3r.speed3r_set_kernel_choice(0)


@pytest.mark.timeout(600)
def test_dense_attn_in_several_bounded_launches(s3r, oracle):
    """Large problems run the dense kernel (the speed-up denominator, eq. 2 form) as several launches of
    about 2e14 FLOP, each starting at a query-group offset.  250 037 tokens x 16 heads take two launches,
    the second starting at query group 1525 (row 195 200): rows at both ends, either side of that
    boundary and at random against the oracle."""
    n_tok, heads = 250_037, 16
    per_launch = int(2e14 / (4.0 * 64.0 * 128 * n_tok * heads))
    groups = (n_tok + 127) // 128
    assert 1 <= per_launch < groups <= 2 * per_launch          # exactly two launches
    edge = per_launch * 128
    g = torch.Generator(device="cuda").manual_seed(4242)
    q, k, v = (torch.randn((n_tok, heads, 64), generator=g, device="cuda").to(torch.bfloat16) for _ in range(3))
    out = torch.full_like(q, float("nan"))
    lse = torch.full((heads, n_tok), float("nan"), device="cuda")
    s3r.speed3r_dense_attn(q, k, v, out, lse)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()      # every row was written
    rng = np.random.default_rng(17)
    rows = np.unique(np.concatenate([[0, 1, 127, 128, edge - 129, edge - 128, edge - 1, edge, edge + 1, edge + 127,
                                      edge + 128, n_tok - 38, n_tok - 37, n_tok - 2, n_tok - 1],
                                     rng.choice(n_tok, 49, replace=False)]))
    ref, ref_lse = oracle.dense_attn(to_host_f32(q), to_host_f32(k), to_host_f32(v), 0.125, q_tok=rows, want_lse=True)
    take = torch.from_numpy(rows).cuda()
    assert_close(to_host_f32(out.index_select(0, take)), ref, TOL["bf16"], "dense, two launches")
    assert float(np.max(np.abs(lse.index_select(1, take).cpu().numpy() - ref_lse))) <= TOL["bf16"]


# ------------------------------------------------------------------------------- end to end --

def end_to_end(s3r, oracle, wl, rows=None, with_gate=False, device_gen="cpu", label=None, forced=None,
               token_queries=False):
    label = label or wl.name
    log(f"{label}: drawing inputs n_tok={wl.n_tok} heads={wl.heads} block={wl.block} topk={wl.topk}")
    q, k, v = workloads.make_inputs(wl, device=device_gen)
    gate = workloads.make_gate_logits(wl, device=device_gen) if with_gate else None
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    gd = None if gate is None else gate.cuda()
    log(f"{label}: device path")
    res = run_device(s3r, qd, kd, vd, wl.block, wl.topk, gate=gd, forced=forced,
                     compress_queries=int(token_queries))
    log(f"{label}: oracle")
    stats = compare_with_oracle(oracle, res, to_host_f32(q), to_host_f32(k), to_host_f32(v),
                                None if gate is None else to_host_f32(gate), wl.block, wl.topk,
                                wl.dtype, rows=rows, label=label, forced=forced, token_queries=token_queries)
    log(f"{label}: {stats}")
    return stats


def test_config1_tiny_f32(s3r, oracle):
    end_to_end(s3r, oracle, workloads.config(1))
    end_to_end(s3r, oracle, workloads.config(1), with_gate=True, label="config1+gate")


def test_config2_vggt_8_views(s3r, oracle):
    end_to_end(s3r, oracle, workloads.config(2), with_gate=True)


@pytest.mark.parametrize("dtype,block,prescale", [
    ("bf16", 64, 16.0), ("bf16", 64, 1e-3), ("bf16", 128, 16.0), ("bf16", 16, 16.0),
    ("f32", 64, 16.0), ("f32", 64, 1e-3), ("f32", 32, 16.0),
])
def test_peaked_and_flat_softmax(s3r, oracle, dtype, block, prescale):
    """Queries 16 times larger (logits of standard deviation 16: nearly all the weight on one or two keys, exponents
    far below the running maximum everywhere else, maxima that rise by tens from unit to unit) and a thousand
    times smaller (all keys weigh the same)."""
    wl = workloads.Workload(f"prescale_{dtype}_{block}_{prescale}", 3, 700, 2, 64, dtype, block, 5, 77, "normal",
                            q_prescale=prescale)
    end_to_end(s3r, oracle, wl, with_gate=True)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("block", [16, 64, 128])
@pytest.mark.parametrize("case", ["q_zero", "k_zero", "v_zero", "all_ones", "one_hot_rows"])
def test_degenerate_inputs(s3r, oracle, dtype, block, case):
    """Inputs on which every score ties (zero queries or keys, constant tensors), on which the result is zero, and
    on which each row has a single non-zero channel: the index sets are then any valid ones under the near-tie
    rule, and the outputs are compared on the device's sets."""
    n_tok, heads = 5 * block + 7, 2
    q, k, v = (draw(n_tok, heads, dtype, 4400 + i) for i in range(3))
    if case == "q_zero":
        q = torch.zeros_like(q)
    elif case == "k_zero":
        k = torch.zeros_like(k)
    elif case == "v_zero":
        v = torch.zeros_like(v)
    elif case == "all_ones":
        q, k, v = torch.ones_like(q), torch.ones_like(k), torch.ones_like(v)
    else:
        hot = torch.arange(n_tok)[:, None] % 64
        mask = (torch.arange(64)[None, None, :] == hot[:, :, None]).to(q.dtype)
        q, k = q * mask, k * mask
    res = run_device(s3r, q.cuda(), k.cuda(), v.cuda(), block, 3)
    assert torch.isfinite(res["out"].float()).all()
    compare_with_oracle(oracle, res, to_host_f32(q), to_host_f32(k), to_host_f32(v), None, block, 3, dtype,
                        label=f"{case} {dtype} B={block}")


def test_config2_generic_kernels(s3r, oracle):
    s3r.speed3r_set_kernel_choice(1)
    try:
        end_to_end(s3r, oracle, workloads.config(2, views=3), label="config2/3views/generic")
    finally:
        s3r.speed3r_set_kernel_choice(0)


def test_config3_100_views_sampled_rows(s3r, oracle):
    wl = workloads.config(3)
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, 1, wl.n_blk - 2, wl.n_blk - 1], rng.choice(wl.n_blk, 44, replace=False)]))
    end_to_end(s3r, oracle, wl, rows=rows, device_gen="cuda")


@pytest.mark.timeout(600)
def test_config4_1000_views_full_size_sampled_rows(s3r, oracle):
    """The benchmark workload at full size, in the launch configuration bench.py times (caller
    workspace, S_guide in head chunks): TopK sets and outputs of sampled query blocks, first and
    last (ragged) blocks included, against the oracle."""
    wl = workloads.config(4)
    rng = np.random.default_rng(8)
    rows = np.unique(np.concatenate([[0, 1, wl.n_blk - 2, wl.n_blk - 1], rng.choice(wl.n_blk, 20, replace=False)]))
    end_to_end(s3r, oracle, wl, rows=rows, device_gen="cuda")


@pytest.mark.timeout(300)
@pytest.mark.parametrize("topk", [32, 64])
def test_config5_pi3_300_views_full_size_sampled_rows(s3r, oracle, topk):
    wl = workloads.config(5, topk=topk)
    rng = np.random.default_rng(9)
    rows = np.unique(np.concatenate([[0, wl.n_blk - 1], rng.choice(wl.n_blk, 14, replace=False)]))
    end_to_end(s3r, oracle, wl, rows=rows, device_gen="cuda")


@pytest.mark.timeout(300)
@pytest.mark.parametrize("topk", [16, 128])
def test_config5_pi3_300_views_full_size_sampled_rows_top16_top128(s3r, oracle, topk):
    """The two ends of config 5's top-k sweep at full size: 16 (TopK inside the sweep) and 128 (TopK from
    scores written to memory, 16 384 selected keys per query)."""
    wl = workloads.config(5, topk=topk)
    rng = np.random.default_rng(19 + topk)
    rows = np.unique(np.concatenate([[0, wl.n_blk - 1], rng.choice(wl.n_blk, 10, replace=False)]))
    end_to_end(s3r, oracle, wl, rows=rows, device_gen="cuda")


@pytest.mark.parametrize("topk", [16, 128])
def test_config5_pi3_block128_small(s3r, oracle, topk):
    wl = workloads.config(5, views=12, topk=topk)
    rng = np.random.default_rng(6)
    rows = np.unique(np.concatenate([[0, wl.n_blk - 1], rng.choice(wl.n_blk, 22, replace=False)]))
    end_to_end(s3r, oracle, wl, rows=rows, with_gate=(topk == 16))


# ---------------------------------------- compressed attention + TopK without S_guide in memory --

def compress_topk_case(s3r, qc, kc, vc, k, accurate, scale=0.0):
    heads, n_blk, _ = qc.shape
    kk = min(k, n_blk)
    o_comp = torch.full((heads, n_blk, 64), float("nan"), device="cuda")
    idx = torch.full((heads, n_blk, kk), -1, dtype=torch.int32, device="cuda")
    s3r.speed3r_compress_attn_topk(torch.from_numpy(qc).cuda(), torch.from_numpy(kc).cuda(), torch.from_numpy(vc).cuda(),
                                   o_comp, idx, k, softmax_scale=scale, accurate_pv=accurate)
    torch.cuda.synchronize()
    return o_comp.cpu().numpy(), idx.cpu().numpy()


@pytest.mark.parametrize("n_blk,k,span", [(5, 3, 2), (63, 7, 2), (64, 64, 3), (65, 1, 2), (200, 16, 8), (1000, 64, 8),
                                          (2100, 32, 8), (2100, 64, 1), (50, 1000, 4)])
def test_compress_attn_topk_exact_on_integer_scores(s3r, oracle, n_blk, k, span):
    """Pooled tensors of small integers: every product and sum is exact in bf16 pairs, fp32 and
    fp64 alike, so the TopK sets must equal the oracle's bit for bit, ties (there are many) going to
    the smaller index; with span 1 the ties are so massive that the candidate lists run over and the
    call takes its fallback, which must give the same sets."""
    rng = np.random.default_rng(n_blk * 7 + k)
    heads = 2
    qc = rng.integers(-span, span + 1, (heads, n_blk, 64)).astype(np.float32)
    kc = rng.integers(-span, span + 1, (heads, n_blk, 64)).astype(np.float32)
    vc = rng.standard_normal((heads, n_blk, 64)).astype(np.float32)
    _, idx = compress_topk_case(s3r, qc, kc, vc, k, False)
    ref = oracle.topk(oracle.scores(qc.astype(np.float64), kc.astype(np.float64)), min(k, n_blk))
    assert np.array_equal(idx, ref)


@pytest.mark.parametrize("n_blk,heads,k,accurate", [(16, 2, 4, True), (172, 4, 16, False), (172, 4, 16, True),
                                                    (1000, 2, 64, False), (2147, 3, 32, False), (33, 1, 5, False)])
def test_compress_attn_topk_random(s3r, oracle, n_blk, heads, k, accurate):
    rng = np.random.default_rng(n_blk + 13 * k)
    qc, kc, vc = (rng.standard_normal((heads, n_blk, 64)).astype(np.float32) for _ in range(3))
    o_comp, idx = compress_topk_case(s3r, qc, kc, vc, k, accurate)
    s64 = oracle.scores(qc.astype(np.float64), kc.astype(np.float64))
    n_exact, n_tie = check_topk_sets(s64, idx, min(k, n_blk))
    assert n_tie <= max(1, (heads * n_blk) // 100)            # fp32-grade scores: near-ties are rare
    ref = oracle.compressed_attn(s64, vc.astype(np.float64), 0.125)
    assert_close(o_comp, ref, TOL["f32"] if accurate else TOL["bf16"], "o_comp")


@pytest.mark.parametrize("accurate", [False, True])
@pytest.mark.parametrize("route", ["in_sweep", "stored"])
@pytest.mark.parametrize("step", [0.25, 0.5, -0.25])
def test_compress_attn_running_maximum_rises_along_the_keys(s3r, oracle, route, accurate, step):
    """Logits that grow steadily with the key index (by `step` per key, i.e. by 8 or 16 per 32 keys): the
    online softmax has to raise its running maximum over and over while earlier partial sums are still
    being accumulated (eq. 3, Alg. 1's rescaling of O and l).  A negative step puts the maximum first.
    The dominant components are multiples of 0.25, exact in every operand format the sweeps use, so that
    what is tested is the rescaling and not the rounding of logits of size 75 to 150."""
    n_blk, heads = 300, 2
    rng = np.random.default_rng(int(abs(step) * 100) + 3)
    qc = np.zeros((heads, n_blk, 64), dtype=np.float32)
    kc = np.zeros((heads, n_blk, 64), dtype=np.float32)
    qc[:, :, 0] = 8.0
    kc[:, :, 0] = step * np.arange(n_blk, dtype=np.float32)          # logit_j = 0.125 * 8 * step * j
    qc[:, :, 1:] = 0.01 * rng.standard_normal((heads, n_blk, 63)).astype(np.float32)
    kc[:, :, 1:] = 0.01 * rng.standard_normal((heads, n_blk, 63)).astype(np.float32)
    vc = rng.standard_normal((heads, n_blk, 64)).astype(np.float32)
    s64 = oracle.scores(qc.astype(np.float64), kc.astype(np.float64))
    ref = oracle.compressed_attn(s64, vc.astype(np.float64), 0.125)
    if route == "in_sweep":
        o_comp, idx = compress_topk_case(s3r, qc, kc, vc, 16, accurate, scale=0.125)
        check_topk_sets(s64, idx, 16)
    else:
        s_dev = torch.full((heads, n_blk, n_blk), float("nan"), device="cuda")
        oc_dev = torch.full((heads, n_blk, 64), float("nan"), device="cuda")
        s3r.speed3r_compress_attn_scores(torch.from_numpy(qc).cuda(), torch.from_numpy(kc).cuda(),
                                         torch.from_numpy(vc).cuda(), s_dev, oc_dev, 0.125, accurate)
        torch.cuda.synchronize()
        o_comp = oc_dev.cpu().numpy()
    # fp32-grade route: scores from bf16 hi/lo operand pairs are good to 4e-5 |qc||kc| (the bound the score
    # test holds them to), which at logits of up to 135 is what limits the output
    tol_f32 = max(TOL["f32"], 4e-5 * 8.0 * abs(step) * n_blk * 0.125)
    assert_close(o_comp, ref, tol_f32 if accurate else TOL["bf16"], f"o_comp, {route}, step {step}")


@pytest.mark.parametrize("block,kk", [(64, 40), (128, 20), (32, 60), (16, 100), (64, 120)])
def test_select_attn_running_maximum_rises_along_the_keys(s3r, oracle, block, kk):
    """The same for the selection branch (eq. 6, Alg. 2's rescaling): keys whose logits grow by 0.25 per
    token along the sequence, every block selected in ascending order."""
    n_tok, heads = kk * block, 2
    g = torch.Generator().manual_seed(block + kk)
    q = 0.05 * torch.randn((n_tok, heads, 64), generator=g)
    k = 0.05 * torch.randn((n_tok, heads, 64), generator=g)
    v = torch.randn((n_tok, heads, 64), generator=g)
    q[:, :, 0] = 4.0
    k[:, :, 0] = 0.5 * torch.arange(n_tok, dtype=torch.float32)[:, None] / (block / 16)   # logit step 0.25 * 16 / block per token
    q, k, v = (x.to(torch.bfloat16) for x in (q, k, v))
    n_blk = n_tok // block
    idx = torch.arange(kk, dtype=torch.int32).expand(heads, n_blk, kk).contiguous()
    out = torch.full(q.shape, float("nan"), dtype=q.dtype, device="cuda")
    lse = torch.full((heads, n_tok), float("nan"), device="cuda")
    s3r.speed3r_select_attn(q.cuda(), k.cuda(), v.cuda(), idx.cuda(), out, block, lse=lse)
    torch.cuda.synchronize()
    rows = np.array([0, n_blk // 2, n_blk - 1])
    o_ref, l_ref = oracle.select_attn(to_host_f32(q), to_host_f32(k), to_host_f32(v), block, idx.numpy()[:, rows], 0.125, rows)
    tok = (rows[:, None] * block + np.arange(block)[None, :]).reshape(-1)
    got = to_host_f32(out.index_select(0, torch.from_numpy(tok).cuda()))
    assert_close(got, o_ref.reshape(-1, heads, 64), TOL["bf16"], f"o_sel rising maximum B={block}")
    got_l = lse.index_select(1, torch.from_numpy(tok).cuda()).cpu().numpy()
    assert float(np.max(np.abs(got_l - l_ref.reshape(heads, -1)))) <= TOL["bf16"]


@pytest.mark.parametrize("n_blk,k,offset,noise", [(1000, 16, 0.5, 0.05), (1500, 64, 0.5, 0.05), (700, 8, 0.25, 0.2)])
def test_compress_attn_topk_large_common_component(s3r, oracle, n_blk, k, offset, noise):
    """Pooled keys that share a large common vector: all scores of a row sit within a narrow band on
    top of |q||k| ~ 16..64, so scores computed from the bf16 hi parts alone (error up to 2^-8 |q||k|)
    would rank them wrongly (typical error 0.03 against a spacing of 0.01 to 0.02 between the scores
    around rank k).  The sweeps may only use such scores to shortlist; the sets must still be the
    TopK of fp32-grade scores: nearly every row must match the oracle's set exactly."""
    rng = np.random.default_rng(n_blk + k)
    heads = 2
    base = np.full((heads, 1, 64), offset) * np.sign(rng.standard_normal((heads, 1, 64)))
    qc = (base * 8 + rng.standard_normal((heads, n_blk, 64))).astype(np.float32)
    kc = (base + noise * rng.standard_normal((heads, n_blk, 64))).astype(np.float32)
    vc = rng.standard_normal((heads, n_blk, 64)).astype(np.float32)
    o_comp, idx = compress_topk_case(s3r, qc, kc, vc, k, False)
    s64 = oracle.scores(qc.astype(np.float64), kc.astype(np.float64))
    n_exact, n_tie = check_topk_sets(s64, idx, k)
    assert n_tie <= (heads * n_blk) // 20, (n_exact, n_tie)
    ref = oracle.compressed_attn(s64, vc.astype(np.float64), 0.125)
    assert_close(o_comp, ref, TOL["bf16"], "o_comp")


@pytest.mark.parametrize("q_mag,k_mag", [(3e4, 1e-5), (1e-7, 1e-6), (2e6, 5e5), (1.0, 1.0)])
def test_compress_attn_topk_input_magnitudes(s3r, oracle, q_mag, k_mag):
    """The sweeps work on fp16 copies of the pooled tensors, scaled per head by a power of two: sets and
    outputs must not depend on the magnitude of the inputs (far outside fp16's range here), heads of
    very different magnitude must not disturb each other, and rows of tiny norm beside rows of large
    norm must still get valid sets."""
    rng = np.random.default_rng(5)
    heads, n_blk, k = 3, 900, 16
    qc, kc, vc = (rng.standard_normal((heads, n_blk, 64)) for _ in range(3))
    head_mag = np.array([1.0, 1e-3, 64.0])[:, None, None]
    qc = qc * q_mag * head_mag
    kc = kc * k_mag / head_mag
    qc[:, 5] *= 1e-6                     # a query row far below the head's scale
    kc[:, 7] *= 1e-5                     # and such a key
    qc, kc, vc = (x.astype(np.float32) for x in (qc, kc, vc))
    scale = 0.125 / (q_mag * k_mag)
    o_comp, idx = compress_topk_case(s3r, qc, kc, vc, k, False, scale=scale)
    s64 = oracle.scores(qc.astype(np.float64), kc.astype(np.float64))
    n_exact, n_tie = check_topk_sets(s64, idx, k)
    assert n_tie <= max(1, (heads * n_blk) // 100)
    ref = oracle.compressed_attn(s64, vc.astype(np.float64), scale)
    assert_close(o_comp, ref, TOL["bf16"], "o_comp")


@pytest.mark.parametrize("kind", ["row_norms_6_decades", "heavy_tails", "sparse_vectors", "nearly_equal_scores"])
def test_compress_attn_topk_hard_distributions(s3r, oracle, kind):
    """Inputs that stress the shortlist margin of the sweeps: rows whose norms span six decades inside
    one head (the small ones sit in fp16's subnormal range after the per-head scaling), heavy-tailed
    components, vectors with few non-zeros, and scores that differ only in the 4th digit (the margin
    then admits nearly every key and the call must fall back without changing the result)."""
    rng = np.random.default_rng({"row_norms_6_decades": 1, "heavy_tails": 2, "sparse_vectors": 3, "nearly_equal_scores": 4}[kind])
    heads, n_blk, k = 2, 1100, 24
    qc, kc = (rng.standard_normal((heads, n_blk, 64)) for _ in range(2))
    if kind == "row_norms_6_decades":
        qc *= 10.0 ** rng.uniform(-6, 0, (heads, n_blk, 1))
        kc *= 10.0 ** rng.uniform(-6, 0, (heads, n_blk, 1))
    elif kind == "heavy_tails":
        qc = rng.standard_t(1.5, (heads, n_blk, 64))
        kc = rng.standard_t(1.5, (heads, n_blk, 64))
    elif kind == "sparse_vectors":
        qc *= rng.random((heads, n_blk, 64)) < 0.08
        kc *= rng.random((heads, n_blk, 64)) < 0.08
    else:
        kc = 1.0 + 1e-4 * kc
        qc = 1.0 + 0.0 * qc
    qc, kc = qc.astype(np.float32), kc.astype(np.float32)
    vc = rng.standard_normal((heads, n_blk, 64)).astype(np.float32)
    s64 = oracle.scores(qc.astype(np.float64), kc.astype(np.float64))
    scale = 1.0 / max(1e-30, float(np.abs(s64).max()))          # logits within [-1, 1]
    o_comp, idx = compress_topk_case(s3r, qc, kc, vc, k, False, scale=scale)
    check_topk_sets(s64, idx, k)
    ref = oracle.compressed_attn(s64, vc.astype(np.float64), scale)
    assert_close(o_comp, ref, TOL["bf16"], f"o_comp {kind}")


def test_compress_attn_topk_rejects_large_k(s3r):
    z = torch.zeros((1, 128, 64), device="cuda")
    idx = torch.zeros((1, 128, 65), dtype=torch.int32, device="cuda")
    with pytest.raises(s3r.Speed3rError) as e:
        s3r.speed3r_compress_attn_topk(z, z, z, torch.empty_like(z), idx, 65)
    assert e.value.status == s3r.S3R_ERR_UNSUPPORTED


# ------------------------------------ TopK inside the compression sweep vs from stored scores --

@pytest.mark.parametrize("cfg,over", [(2, {}), (3, {"views": 20}), (5, {"views": 12, "topk": 64}),
                                      (1, {})])
def test_topk_from_stored_scores_path(s3r, oracle, cfg, over):
    """The default path selects without S_guide in memory whenever k <= 64; this keeps the
    stored-score TopK covered end to end on the same workloads."""
    s3r.speed3r_set_kernel_choice(2)
    try:
        end_to_end(s3r, oracle, workloads.config(cfg, **over), with_gate=True, label=f"config{cfg}/stored scores")
    finally:
        s3r.speed3r_set_kernel_choice(0)


def test_topk_in_sweep_candidate_overflow_falls_back(s3r, oracle):
    """All-zero queries make every score of a row equal: every key passes the filter, the candidate
    lists run over, and the call must redo TopK from stored scores (first k blocks win the tie)."""
    wl = workloads.Workload("ties_2000_blocks", 1, 2000 * 64, 2, 64, "bf16", 64, 8, 93, "normal")
    q, k, v = workloads.make_inputs(wl, device="cuda")
    q.zero_()
    res = run_device(s3r, q, k, v, wl.block, wl.topk)
    want = torch.arange(8, dtype=torch.int32, device="cuda").expand(2, 2000, 8)
    assert torch.equal(res["idx"], want)
    rows = np.array([0, 1, 777, 1999])
    compare_with_oracle(oracle, res, to_host_f32(q), to_host_f32(k), to_host_f32(v), None, wl.block, wl.topk,
                        wl.dtype, rows=rows, label="all-tie rows")
    # half the rows tie, half do not: the fallback redoes the whole call consistently
    q2, _, _ = workloads.make_inputs(wl, device="cuda")
    q2[: wl.n_tok // 2].zero_()
    res2 = run_device(s3r, q2, k, v, wl.block, wl.topk)
    assert torch.equal(res2["idx"][:, :1000], want[:, :1000])
    rows2 = np.array([0, 999, 1000, 1500, 1999])
    compare_with_oracle(oracle, res2, to_host_f32(q2), to_host_f32(k), to_host_f32(v), None, wl.block, wl.topk,
                        wl.dtype, rows=rows2, label="half-tie rows")


def test_topk_in_sweep_is_deterministic_and_agrees_with_stored_scores(s3r):
    """Two runs agree bit for bit; the stored-score route picks the same sets except where the two
    roundings of a score resolve a near-tie differently (rare), and Oc' agrees within the bf16 tolerance."""
    wl = workloads.Workload("two_routes", 1, 700 * 64, 2, 64, "bf16", 64, 12, 95, "normal")
    q, kx, v = workloads.make_inputs(wl, device="cuda")
    a = run_device(s3r, q, kx, v, wl.block, wl.topk)
    b = run_device(s3r, q, kx, v, wl.block, wl.topk)
    assert torch.equal(a["idx"], b["idx"]) and torch.equal(a["out"], b["out"])
    s3r.speed3r_set_kernel_choice(2)
    try:
        c = run_device(s3r, q, kx, v, wl.block, wl.topk)
    finally:
        s3r.speed3r_set_kernel_choice(0)
    same_rows = (a["idx"] == c["idx"]).all(dim=2).float().mean().item()
    assert same_rows > 0.99, same_rows
    # the two routes run the online softmax at different granularity (different running maxima, hence
    # differently rounded bf16 probabilities): same values within the bf16 tolerance
    assert_close(a["o_comp"].cpu().numpy(), c["o_comp"].cpu().numpy(), TOL["bf16"], "o_comp of the two routes")


# ------------------------------------------------- forced global-context blocks (Sec. 3.3) --

def test_forced_blocks_vggt_8_views(s3r, oracle):
    """Reference view always attended: its blocks join every row's set and leave the TopK."""
    wl = workloads.config(2)
    forced = workloads.vggt_forced_blocks(wl)
    assert forced[0] == 0 and len(forced) == (wl.tokens_per_view - 1) // wl.block + 1
    end_to_end(s3r, oracle, wl, with_gate=True, forced=forced, label="config2+reference view")


def test_forced_blocks_view_stride_sampled_rows(s3r, oracle):
    """Views at a stride (here every 10th of 30) forced, on top of TopK over the rest."""
    wl = workloads.config(3, views=30)
    forced = workloads.vggt_forced_blocks(wl, view_stride=10)
    rng = np.random.default_rng(15)
    rows = np.unique(np.concatenate([[0, int(forced[-1]), wl.n_blk - 1], rng.choice(wl.n_blk, 20, replace=False)]))
    end_to_end(s3r, oracle, wl, rows=rows, forced=forced, device_gen="cuda", label="config3/30views+stride10")


@pytest.mark.parametrize("dtype,block,n_tok,topk,forced", [
    ("f32", 16, 333, 4, [0, 1, 20]),                 # generic kernels, ragged tail, last block forced
    ("f32", 64, 1000, 3, [5]),
    ("f32", 128, 1100, 2, [0, 8]),                   # fp32 on the matrix cores, two units per block, ragged tail
    ("bf16", 64, 1000, 5, [0, 3, 4, 15]),            # 16 blocks; last (ragged) one forced
    ("bf16", 64, 1000, 14, [1, 2]),                  # topk + forced = n_blk: every block attended
    ("bf16", 64, 1000, 64, [0, 7, 9]),               # topk > free blocks: k_dyn clamps to 13
    ("bf16", 64, 1024, 2, list(range(16))),          # everything forced: TopK has nothing to pick
    ("bf16", 128, 1100, 2, [0, 8]),
    ("bf16", 64, 70 * 64, 3, list(range(60, 70))),   # forced bits in the second 64-key word only
    ("bf16", 64, 130 * 64 + 7, 6, [0, 63, 64, 127, 128, 130]),   # word boundaries
])
def test_forced_blocks_edge_cases(s3r, oracle, dtype, block, n_tok, topk, forced):
    wl = workloads.Workload(f"forced_{dtype}_{block}_{n_tok}_{topk}", 1, n_tok, 2, 64, dtype, block, topk, 91,
                            "normal")
    end_to_end(s3r, oracle, wl, with_gate=True, forced=np.asarray(forced, dtype=np.int32))


def test_forced_blocks_list_is_diagnosed_through_the_status_word(s3r):
    """A forced-block list that is out of range or not strictly ascending cannot be refused on the host (it is
    device memory and no call synchronises): the device status word says so, and the call stays memory-safe."""
    q, k, v = (draw(40 * 64, 2, "bf16", 7700 + i).cuda() for i in range(3))
    out = torch.empty_like(q)
    cases = [([1, 5, 9], 0), ([1, 5, 40], s3r.S3R_DIAG_FORCED_RANGE), ([-2, 5, 9], s3r.S3R_DIAG_FORCED_RANGE),
             ([5, 1, 9], s3r.S3R_DIAG_FORCED_ORDER), ([1, 5, 5], s3r.S3R_DIAG_FORCED_ORDER),
             ([9, 5, 77], s3r.S3R_DIAG_FORCED_RANGE | s3r.S3R_DIAG_FORCED_ORDER), (None, 0)]
    for forced, want in cases:
        status = torch.full((1,), -1, dtype=torch.int32, device="cuda")
        f = None if forced is None else torch.tensor(forced, dtype=torch.int32, device="cuda")
        s3r.speed3r_sparse_global_attn_ex(q, k, v, out, 64, 4, forced_blocks=f, status=status)
        torch.cuda.synchronize()
        assert int(status.item()) == want, (forced, int(status.item()), want)
        assert torch.isfinite(out.float()).all()


def test_forced_blocks_leave_compressed_branch_unchanged(s3r):
    """The forced list only changes the selection set: Oc' is bit-identical with and without it."""
    wl = workloads.config(2, views=4)
    q, k, v = (t.cuda() for t in workloads.make_inputs(wl))
    plain = run_device(s3r, q, k, v, wl.block, wl.topk)
    forced = run_device(s3r, q, k, v, wl.block, wl.topk, forced=workloads.vggt_forced_blocks(wl))
    assert torch.equal(plain["o_comp"], forced["o_comp"])
    assert forced["idx"].shape[2] == plain["idx"].shape[2] + len(workloads.vggt_forced_blocks(wl))


# ------------------------------------- special tokens: dense rows + concat (Sec. 3.2 eqs. 1-2) --

def layer_case(s3r, oracle, wl, special, rows=None, spec_sample=None, with_gate=False, forced=None,
               device_gen="cpu", label=None, token_queries=False):
    label = label or f"{wl.name}+{special} special"
    log(f"{label}: drawing inputs n_tok={wl.n_tok} views={wl.views} block={wl.block} topk={wl.topk}")
    q, k, v = workloads.make_inputs(wl, device=device_gen)
    gate = workloads.make_gate_logits(wl, device=device_gen) if with_gate else None
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    gd = None if gate is None else gate.cuda()
    res = run_device(s3r, qd, kd, vd, wl.block, wl.topk, gate=gd, forced=forced,
                     tokens_per_view=wl.tokens_per_view, special_per_view=special,
                     compress_queries=int(token_queries))
    log(f"{label}: oracle")
    stats = compare_layer_with_oracle(oracle, res, to_host_f32(q), to_host_f32(k), to_host_f32(v),
                                      None if gate is None else to_host_f32(gate), wl.block, wl.topk, wl.dtype,
                                      wl.tokens_per_view, special, rows=rows, spec_sample=spec_sample,
                                      forced=forced, label=label, token_queries=token_queries)
    log(f"{label}: {stats}")
    return res, stats


def test_special_tokens_vggt_8_views(s3r, oracle):
    """5 special tokens lead each of 8 views of 1374: their rows get dense attention over all rows,
    the 1369 x 8 image rows the sparse path."""
    layer_case(s3r, oracle, workloads.config(2), 5, with_gate=True)


@pytest.mark.parametrize("dtype,block,views,tpv,special,topk", [
    ("f32", 16, 3, 111, 2, 3),           # generic kernels, blocks straddle views, ragged tail
    ("f32", 64, 2, 300, 7, 2),
    ("f32", 64, 1, 1000, 100, 3),        # fp32 operand pairs: special rows over two key segments, two special units
    ("f32", 128, 3, 700, 5, 2),
    ("bf16", 64, 4, 333, 5, 4),          # image sequence 1312 = 20.5 blocks; 20 special rows (< one unit)
    ("bf16", 64, 1, 1000, 100, 3),       # the paper's [spec; img] arrangement, 100 special rows (two units)
    ("bf16", 128, 3, 700, 5, 2),         # block 128: dense rows walk half-block units, odd unit count
    ("bf16", 64, 70, 65, 1, 2),          # one special token per view; image blocks = views
    ("bf16", 64, 2, 200, 136, 1),        # more special than image rows
])
def test_special_tokens_edge_cases(s3r, oracle, dtype, block, views, tpv, special, topk):
    wl = workloads.Workload(f"special_{dtype}_{block}_{views}x{tpv}_{special}", views, tpv, 2, 64, dtype, block,
                            topk, 92, "normal")
    layer_case(s3r, oracle, wl, special, with_gate=True)


def test_special_tokens_with_forced_reference_view(s3r, oracle):
    wl = workloads.config(2, views=6)
    img = workloads.Workload("img_only", wl.views, wl.tokens_per_view - 5, wl.heads, 64, wl.dtype, wl.block,
                             wl.topk, wl.seed, wl.kind)
    forced = workloads.vggt_forced_blocks(img)          # blocks of the image-only sequence
    layer_case(s3r, oracle, wl, 5, forced=forced, label="config2/6views+special+reference view")


def test_special_tokens_sampled_100_views(s3r, oracle):
    wl = workloads.config(3)
    n_blk_img = (wl.views * (wl.tokens_per_view - 5) + wl.block - 1) // wl.block
    rng = np.random.default_rng(16)
    rows = np.unique(np.concatenate([[0, n_blk_img - 1], rng.choice(n_blk_img, 14, replace=False)]))
    spec = np.unique(np.concatenate([[0, 4, 5, 499], rng.choice(500, 12, replace=False)]))
    layer_case(s3r, oracle, wl, 5, rows=rows, spec_sample=spec, device_gen="cuda")


@pytest.mark.timeout(600)
def test_special_tokens_config4_full_size_sampled(s3r, oracle):
    """The 1000-view workload read as the VGGT layout (5 special tokens lead every view): sampled
    image query blocks and sampled special rows (each attends all 1,374,000 keys) against the oracle."""
    wl = workloads.config(4)
    n_blk_img = (wl.views * (wl.tokens_per_view - 5) + wl.block - 1) // wl.block
    rng = np.random.default_rng(17)
    rows = np.unique(np.concatenate([[0, n_blk_img - 1], rng.choice(n_blk_img, 10, replace=False)]))
    spec = np.unique(np.concatenate([[0, 4999], rng.choice(5000, 6, replace=False)]))
    layer_case(s3r, oracle, wl, 5, rows=rows, spec_sample=spec, device_gen="cuda")


def test_special_tokens_untouched_outputs_and_zero_special(s3r):
    """special_per_view = 0 with a period is the plain path bit for bit; with special tokens the
    optional per-token outputs of the special rows are left as they were."""
    wl = workloads.config(2, views=3)
    q, k, v = (t.cuda() for t in workloads.make_inputs(wl))
    plain = run_device(s3r, q, k, v, wl.block, wl.topk)
    same = run_device(s3r, q, k, v, wl.block, wl.topk, tokens_per_view=wl.tokens_per_view, special_per_view=0)
    for key in ("out", "idx", "lse", "o_comp", "o_sel"):
        assert torch.equal(plain[key], same[key]), key
    res = run_device(s3r, q, k, v, wl.block, wl.topk, tokens_per_view=wl.tokens_per_view, special_per_view=5)
    spec = torch.arange(wl.n_tok, device="cuda") % wl.tokens_per_view < 5
    assert torch.isnan(res["o_sel"][spec].float()).all() and torch.isnan(res["lse"][:, spec]).all()
    assert torch.isfinite(res["out"].float()).all()
    assert torch.isfinite(res["o_sel"][~spec].float()).all() and torch.isfinite(res["lse"][:, ~spec]).all()


# ------------------------------------------ spatial pooling windows on the patch grid (Sec. 3.2) --

@pytest.mark.parametrize("dtype,views,special,grid_h,grid_w,window,topk,forced", [
    ("bf16", 3, 5, 37, 37, 8, 6, None),        # the VGGT grid: 5 x 5 windows per view, edge windows of 5 columns / rows
    ("bf16", 2, 0, 37, 37, 8, 4, None),        # the pi3 layout: no special tokens
    ("bf16", 4, 1, 16, 24, 8, 3, None),        # windows divide the grid: every block full
    ("bf16", 2, 5, 37, 37, 8, 5, [0, 4, 24]),  # forced windows incl. the corner one of view 0
    ("f32", 2, 2, 9, 10, 4, 3, None),          # 4 x 4 windows (block 16): generic kernels
    ("f32", 3, 0, 8, 8, 4, 2, [1]),
    ("f32", 2, 5, 37, 37, 8, 5, [0, 4, 24]),   # fp32 on the matrix cores: cut windows, special rows, forced windows
    ("bf16", 2, 3, 11, 13, 4, 4, None),        # block 16 in bf16: generic kernels
    ("bf16", 1, 0, 5, 5, 8, 1, None),          # a single cut window
])
def test_spatial_windows(s3r, oracle, dtype, views, special, grid_h, grid_w, window, topk, forced):
    tpv = special + grid_h * grid_w
    wl = workloads.Workload(f"windows_{dtype}_{views}x{grid_h}x{grid_w}_w{window}", views, tpv, 2, 64, dtype,
                            window * window, topk, 96, "normal")
    q, k, v = workloads.make_inputs(wl)
    gate = workloads.make_gate_logits(wl)
    grid = (grid_h, grid_w, window)
    forced_a = None if forced is None else np.asarray(forced, dtype=np.int32)
    res = run_device(s3r, q.cuda(), k.cuda(), v.cuda(), wl.block, topk, gate=gate.cuda(), forced=forced_a,
                     tokens_per_view=tpv, special_per_view=special, grid=grid)
    stats = compare_windows_with_oracle(oracle, res, to_host_f32(q), to_host_f32(k), to_host_f32(v),
                                        to_host_f32(gate), topk, dtype, views, tpv, special, grid, forced=forced_a,
                                        label=wl.name)
    log(f"{wl.name}: {stats}")


def test_spatial_windows_equal_plain_path_on_permuted_tokens(s3r, oracle):
    """When the windows divide the grid, the windowed call on the original token order and the
    plain blocked call on the tokens gathered into window-major order are the same computation:
    bit-identical results, row for row."""
    views, gh, gw, win = 3, 16, 24, 8
    wl = workloads.Workload("windows_vs_permuted", views, gh * gw, 2, 64, "bf16", 64, 4, 97, "normal")
    q, k, v = (t.cuda() for t in workloads.make_inputs(wl))
    gate = workloads.make_gate_logits(wl).cuda()
    perm = torch.from_numpy(np.concatenate(oracle.window_blocks(views, gh * gw, 0, gh, gw, win))).cuda()
    a = run_device(s3r, q, k, v, 64, 4, gate=gate, tokens_per_view=gh * gw, special_per_view=0, grid=(gh, gw, win))
    b = run_device(s3r, q[perm].contiguous(), k[perm].contiguous(), v[perm].contiguous(), 64, 4,
                   gate=gate[perm].contiguous())
    assert torch.equal(a["idx"], b["idx"]) and torch.equal(a["o_comp"], b["o_comp"])
    assert torch.equal(a["out"][perm], b["out"]) and torch.equal(a["o_sel"][perm], b["o_sel"])
    assert torch.equal(a["lse"][:, perm], b["lse"])


@pytest.mark.parametrize("n_tok,block,topk,dtype", [(1, 64, 4, "bf16"), (63, 64, 1, "bf16"), (65, 64, 2, "bf16"),
                                                    (130, 128, 7, "bf16"), (100, 16, 3, "bf16"),
                                                    (100, 32, 2, "f32"), (64, 64, 1, "f32"),
                                                    (4097, 64, 1000, "bf16")])
def test_edge_shapes(s3r, oracle, n_tok, block, topk, dtype):
    wl = workloads.Workload(f"edge_{n_tok}_{block}_{topk}", 1, n_tok, 2, 64, dtype, block, topk, 77, "normal")
    end_to_end(s3r, oracle, wl, with_gate=True)


@pytest.mark.parametrize("block,views,topk", [(16, 6, 32), (32, 6, 16)])
def test_small_blocks_end_to_end(s3r, oracle, block, views, topk):
    """The paper's default pooling size (4 x 4 = 16 tokens, top-32) and 32-token blocks on the MFMA
    path, on 1374-token views (ragged last block), sampled query blocks."""
    wl = workloads.config(2, views=views, block=block, topk=topk)
    rng = np.random.default_rng(18)
    rows = np.unique(np.concatenate([[0, 1, wl.n_blk - 2, wl.n_blk - 1], rng.choice(wl.n_blk, 40, replace=False)]))
    end_to_end(s3r, oracle, wl, rows=rows, with_gate=True, label=f"config2/{views}views/block{block}")


def test_full_topk_equals_dense_kernel(s3r, oracle):
    """topk >= n_blk makes the selection branch dense attention: the sparse path's O_sel must agree
    with the in-house dense kernel (and both with the oracle's dense attention)."""
    wl = workloads.config(2, views=2, topk=10 ** 6)
    q, k, v = (x.cuda() for x in workloads.make_inputs(wl))
    res = run_device(s3r, q, k, v, wl.block, wl.topk)
    dense = torch.empty_like(q)
    s3r.speed3r_dense_attn(q, k, v, dense)
    torch.cuda.synchronize()
    ref = oracle.dense_attn(to_host_f32(q), to_host_f32(k), to_host_f32(v), 0.125)
    assert_close(to_host_f32(res["o_sel"]), ref, TOL["bf16"], "o_sel with all blocks vs dense oracle")
    assert_close(to_host_f32(dense), ref, TOL["bf16"], "dense kernel vs dense oracle")


@pytest.mark.parametrize("block,stages,wg", [(64, 0, 0), (64, 3, 2), (64, 4, 1), (128, 0, 0), (128, 2, 2), (128, 4, 1)])
def test_load_probe_moves_data_and_leaves_q(s3r, block, stages, wg):
    """The measurement kernel (the selection kernel without its arithmetic) must run its whole index walk with
    every ring depth and occupancy limit, write a copy of q, and refuse what it does not cover."""
    n_tok, heads, kk = 37 * block + 11, 3, 9
    g = torch.Generator().manual_seed(block + stages)
    q, k, v = (torch.randn((n_tok, heads, 64), generator=g).to(torch.bfloat16).cuda() for _ in range(3))
    n_blk = (n_tok + block - 1) // block
    idx = torch.stack([torch.stack([torch.sort(torch.randperm(n_blk, generator=g)[:kk]).values for _ in range(n_blk)])
                       for _ in range(heads)]).to(torch.int32).cuda()
    out = torch.full_like(q, float("nan"))
    s3r.speed3r_probe_select_loads(q, k, v, idx, out, block, stages, wg)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), q.view(torch.int16))
    with pytest.raises(s3r.Speed3rError):
        s3r.speed3r_probe_select_loads(q, k, v, idx, out, block, 5, 0)
    with pytest.raises(s3r.Speed3rError):
        s3r.speed3r_probe_select_loads(q, k, v, idx, out, block, 4, 3)          # three rings of 64 KiB do not fit a CU's 160 KiB


def test_deterministic_and_stream(s3r):
    wl = workloads.config(2, views=2)
    q, k, v = (x.cuda() for x in workloads.make_inputs(wl))
    a = run_device(s3r, q, k, v, wl.block, wl.topk)
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        b = run_device(s3r, q, k, v, wl.block, wl.topk)
    st.synchronize()
    for key in ("out", "idx", "lse", "o_comp", "o_sel"):
        assert torch.equal(a[key], b[key]), key
    out = torch.empty_like(q)
    s3r.speed3r_sparse_global_attn(q, k, v, out, wl.block, wl.topk)      # short form, library scratch
    torch.cuda.synchronize()
    assert torch.equal(out, a["out"])


def test_errors_on_device_arguments(s3r):
    q = torch.zeros((128, 2, 64), dtype=torch.bfloat16, device="cuda")
    out = torch.empty_like(q)
    ws = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(s3r.Speed3rError) as e:
        s3r.speed3r_sparse_global_attn_ex(q, q, q, out, 64, 2, workspace=ws)
    assert e.value.status == s3r.S3R_ERR_WORKSPACE
    with pytest.raises(s3r.Speed3rError) as e:
        s3r.speed3r_sparse_global_attn_ex(q, q, q, out, 48, 2)
    assert e.value.status == s3r.S3R_ERR_UNSUPPORTED
    with pytest.raises(s3r.Speed3rError) as e:
        s3r.speed3r_sparse_global_attn_ex(q, q, q, q, 64, 2)
    assert e.value.status == s3r.S3R_ERR_INVALID_ARG


# -------------------------- compression branch with unpooled queries (every token's own query) --

def test_token_queries_config1_f32(s3r, oracle):
    end_to_end(s3r, oracle, workloads.config(1), with_gate=True, token_queries=True, label="config1 token queries")
    end_to_end(s3r, oracle, workloads.config(1), token_queries=True, label="config1 token queries, no gate")


def test_token_queries_vggt_8_views(s3r, oracle):
    end_to_end(s3r, oracle, workloads.config(2), with_gate=True, token_queries=True, label="config2 token queries")


@pytest.mark.parametrize("dtype,block,n_tok,topk", [
    ("bf16", 64, 1000, 4),       # ragged last block: 15.6 blocks, a quarter of one key unit
    ("bf16", 64, 64 * 65 + 1, 3),  # 66 pooled keys: a second, nearly empty key unit
    ("bf16", 128, 128 * 9 + 5, 2),
    ("bf16", 32, 700, 5),
    ("bf16", 16, 333, 6),
    ("f32", 16, 200, 3),
    ("f32", 128, 900, 2),
    ("bf16", 64, 50, 2),         # a single short block
])
def test_token_queries_edge_cases(s3r, oracle, dtype, block, n_tok, topk):
    wl = workloads.Workload(f"tokq_{dtype}_{block}_{n_tok}", 1, n_tok, 2, 64, dtype, block, topk, 97, "normal")
    end_to_end(s3r, oracle, wl, with_gate=True, token_queries=True)


def test_token_queries_with_forced_and_special_tokens(s3r, oracle):
    wl = workloads.config(2, views=6)
    img = workloads.Workload("img_only", wl.views, wl.tokens_per_view - 5, wl.heads, 64, wl.dtype, wl.block,
                             wl.topk, wl.seed, wl.kind)
    forced = workloads.vggt_forced_blocks(img)
    layer_case(s3r, oracle, wl, 5, forced=forced, with_gate=True, token_queries=True,
               label="config2/6views+special+reference view, token queries")
    wl32 = workloads.Workload("tokq_special_f32", 3, 111, 2, 64, "f32", 16, 3, 98, "normal")
    layer_case(s3r, oracle, wl32, 2, with_gate=True, token_queries=True)


@pytest.mark.parametrize("dtype,views,special,grid_h,grid_w,window,topk", [
    ("bf16", 3, 5, 37, 37, 8, 6),        # cut edge windows: query slots past a window's cells do not exist
    ("bf16", 2, 3, 11, 13, 4, 4),
    ("f32", 2, 2, 9, 10, 4, 3),
])
def test_token_queries_spatial_windows(s3r, oracle, dtype, views, special, grid_h, grid_w, window, topk):
    tpv = special + grid_h * grid_w
    wl = workloads.Workload(f"tokq_windows_{dtype}_{views}x{grid_h}x{grid_w}_w{window}", views, tpv, 2, 64, dtype,
                            window * window, topk, 99, "normal")
    q, k, v = workloads.make_inputs(wl)
    gate = workloads.make_gate_logits(wl)
    grid = (grid_h, grid_w, window)
    res = run_device(s3r, q.cuda(), k.cuda(), v.cuda(), wl.block, topk, gate=gate.cuda(),
                     tokens_per_view=tpv, special_per_view=special, grid=grid, compress_queries=1)
    stats = compare_windows_with_oracle(oracle, res, to_host_f32(q), to_host_f32(k), to_host_f32(v),
                                        to_host_f32(gate), topk, dtype, views, tpv, special, grid,
                                        label=wl.name, token_queries=True)
    log(f"{wl.name}: {stats}")


def test_token_queries_sampled_100_views(s3r, oracle):
    """100 views (2147 pooled keys per head): sampled query blocks against the oracle."""
    wl = workloads.config(3)
    n_blk = (wl.n_tok + wl.block - 1) // wl.block
    rng = np.random.default_rng(19)
    rows = np.unique(np.concatenate([[0, n_blk - 1], rng.choice(n_blk, 10, replace=False)]))
    end_to_end(s3r, oracle, wl, rows=rows, with_gate=True, device_gen="cuda", token_queries=True,
               label="config3 token queries")


def test_token_queries_leave_everything_else_unchanged_and_reject_bad_values(s3r):
    """Only `out` depends on the option: TopK, the selection branch and the per-block compressed
    output are those of the default path bit for bit.  Values other than 0 and 1 are refused, and
    so is the option on bf16 data while the generic kernels are forced."""
    wl = workloads.config(2, views=3)
    q, k, v = (t.cuda() for t in workloads.make_inputs(wl))
    a = run_device(s3r, q, k, v, wl.block, wl.topk)
    b = run_device(s3r, q, k, v, wl.block, wl.topk, compress_queries=1)
    for key in ("idx", "lse", "o_comp", "o_sel"):
        assert torch.equal(a[key], b[key]), key
    assert not torch.equal(a["out"], b["out"])
    out = torch.empty_like(q)
    with pytest.raises(s3r.Speed3rError) as e:
        s3r.speed3r_sparse_global_attn_ex(q, k, v, out, wl.block, wl.topk, compress_queries=2)
    assert e.value.status == s3r.S3R_ERR_INVALID_ARG
    s3r.speed3r_set_kernel_choice(1)
    try:
        with pytest.raises(s3r.Speed3rError) as e:
            s3r.speed3r_sparse_global_attn_ex(q, k, v, out, wl.block, wl.topk, compress_queries=1)
        assert e.value.status == s3r.S3R_ERR_UNSUPPORTED
    finally:
        s3r.speed3r_set_kernel_choice(0)


# ------------------------------------------------- strided q, k, v (views of a packed tensor) --

@pytest.mark.parametrize("dtype,block,views,tpv,special,topk,grid,layout", [
    ("bf16", 64, 4, 333, 0, 4, None, "packed_qkv"),        # [n_tok, 3, heads, 64]: slices of one projection output
    ("bf16", 64, 4, 333, 5, 4, None, "packed_qkv"),        # special tokens: both pooling launches and the dense rows
    ("bf16", 128, 3, 500, 0, 2, None, "head_major"),       # [heads, n_tok, 64] seen as [n_tok, heads, 64]
    ("bf16", 16, 2, 3 + 11 * 13, 3, 4, (11, 13, 4), "padded_heads"),   # windows; heads padded to 96 channels
    ("f32", 64, 2, 300, 7, 2, None, "packed_qkv"),         # generic kernels: k and v follow the same strides
    ("f32", 16, 3, 111, 0, 3, None, "head_major"),
])
def test_strided_inputs_match_packed_inputs(s3r, oracle, dtype, block, views, tpv, special, topk, grid, layout):
    """q, k, v given as strided views: every output equals, bit for bit, that of the same call on packed
    copies (which the other tests hold against the oracle); `out` is checked against the oracle as well
    on the plain layouts."""
    wl = workloads.Workload(f"strided_{dtype}_{block}_{layout}", views, tpv, 2, 64, dtype, block, topk, 101, "normal")
    q, k, v = (t.cuda() for t in workloads.make_inputs(wl))
    gate = workloads.make_gate_logits(wl).cuda()
    n, h = wl.n_tok, wl.heads
    if layout == "packed_qkv":
        big = torch.stack([q, k, v], dim=1).contiguous()               # [n, 3, h, 64]
        qs, ks, vs = big[:, 0], big[:, 1], big[:, 2]
    elif layout == "head_major":
        qs, ks, vs = (t.permute(1, 0, 2).contiguous().permute(1, 0, 2) for t in (q, k, v))
    else:
        pad = [torch.zeros((n, h, 96), dtype=q.dtype, device="cuda") for _ in range(3)]
        for dst, src in zip(pad, (q, k, v)):
            dst[:, :, 16:80] = src
        qs, ks, vs = (t[:, :, 16:80] for t in pad)
    assert not qs.is_contiguous() and torch.equal(qs, q)
    kw = dict(gate=gate, tokens_per_view=tpv if (special or grid) else 0, special_per_view=special, grid=grid)
    ref = run_device(s3r, q, k, v, block, topk, **kw)
    for cq in (0, 1):
        want = ref if cq == 0 else run_device(s3r, q, k, v, block, topk, compress_queries=1, **kw)
        got = run_device(s3r, qs, ks, vs, block, topk, compress_queries=cq, **kw)
        for key in ("idx", "o_comp", "out"):
            assert torch.equal(got[key], want[key]), (key, cq)
        for key in ("o_sel", "lse"):                                      # special rows stay NaN in both
            assert torch.equal(torch.nan_to_num(got[key].float(), nan=-7.0),
                               torch.nan_to_num(want[key].float(), nan=-7.0)), (key, cq)
    if grid is None:
        res = run_device(s3r, qs, ks, vs, block, topk, **kw)
        host = [to_host_f32(t) for t in (q, k, v, gate)]
        if special:
            stats = compare_layer_with_oracle(oracle, res, *host, block, topk, dtype, tpv, special, label=wl.name)
        else:
            stats = compare_with_oracle(oracle, res, *host, block, topk, dtype, label=wl.name)
        log(f"{wl.name}: {stats}")


def test_strides_are_validated(s3r):
    q = torch.zeros((128, 2, 64), dtype=torch.bfloat16, device="cuda")
    out = torch.empty_like(q)
    big = torch.zeros((128, 2, 68), dtype=torch.bfloat16, device="cuda")     # rows of 68 elements: not 16-byte steps
    with pytest.raises(s3r.Speed3rError) as e:
        s3r.speed3r_sparse_global_attn_ex(big[:, :, :64], big[:, :, :64], big[:, :, :64], out, 64, 2)
    assert e.value.status == s3r.S3R_ERR_INVALID_ARG and "stride" in str(e.value)
    with pytest.raises(TypeError):                                             # channels not contiguous
        t = torch.zeros((128, 64, 2), dtype=torch.bfloat16, device="cuda").permute(0, 2, 1)
        s3r.speed3r_sparse_global_attn_ex(t, t, t, out, 64, 2)
    with pytest.raises(TypeError):                                             # q and k laid out differently
        kt = q.permute(1, 0, 2).contiguous().permute(1, 0, 2)
        s3r.speed3r_sparse_global_attn_ex(q, kt, q, out, 64, 2)


# --------------------- long index rows: two query blocks per workgroup on the merged list --

@pytest.mark.parametrize("n_tok,topk,n_forced,with_gate", [
    (64 * 202 + 17, 30, 100, True),      # 203 blocks (odd: the last workgroup holds one query block), ragged tail
    (64 * 150, 16, 100, False),          # mostly forced blocks, common to every query block
    (64 * 140 + 40, 50, 55, True),       # forced and selected interleaved, about half and half
    (64 * 130, 1, 129, False),           # all blocks but one forced
    (64 * 202 + 17, 120, 0, True),       # long rows without forced blocks: one query block per workgroup
    (64 * 129 + 1, 200, 0, False),       # topk > n_blk: every block selected by every query block
    (64 * 140 + 40, 60, 45, True),       # forced blocks the smaller part of a long row
])
def test_long_index_rows_pair_kernel(s3r, oracle, n_tok, topk, n_forced, with_gate):
    """Rows of more than 96 blocks of 64 tokens, at least half of them forced, run two query blocks
    per workgroup on the union of their lists; other long rows one; every output against the oracle."""
    wl = workloads.Workload(f"longrows_{n_tok}_{topk}_{n_forced}", 1, n_tok, 2, 64, "bf16", 64, topk, 111, "clustered")
    forced = None
    if n_forced:
        forced = np.sort(np.random.default_rng(112).choice(wl.n_blk, n_forced, replace=False)).astype(np.int32)
    end_to_end(s3r, oracle, wl, with_gate=with_gate, forced=forced)


def test_long_index_rows_spatial_windows(s3r, oracle):
    """The same kernel with 8 x 8 windows (per-block lengths, cut edge windows): 9 views of 37 x 37
    patches = 225 blocks (odd), 60 of them forced (the corner windows among them), 50 selected."""
    views, special, grid = 9, 5, (37, 37, 8)
    tpv = special + 37 * 37
    wl = workloads.Workload("longrows_windows", views, tpv, 2, 64, "bf16", 64, 50, 113, "normal")
    q, k, v = workloads.make_inputs(wl)
    gate = workloads.make_gate_logits(wl)
    forced = np.unique(np.concatenate([[4, 20, 24, 224], np.random.default_rng(114).choice(225, 56, replace=False)]))
    forced = forced.astype(np.int32)
    res = run_device(s3r, q.cuda(), k.cuda(), v.cuda(), 64, 50, gate=gate.cuda(), forced=forced, tokens_per_view=tpv,
                     special_per_view=special, grid=grid)
    stats = compare_windows_with_oracle(oracle, res, to_host_f32(q), to_host_f32(k), to_host_f32(v),
                                        to_host_f32(gate), 50, "bf16", views, tpv, special, grid, forced=forced,
                                        label=wl.name)
    log(f"{wl.name}: {stats}")


# ------------------------------------- the options at the benchmark's full size, sampled rows --

@pytest.mark.timeout(600)
def test_config4_full_size_forced_reference_views_sampled_rows(s3r, oracle):
    """1000 views with the VGGT variant's fixed context (reference view + every 100th view: 224
    forced blocks, 288 blocks per query block): the long-row selection kernel at full size."""
    wl = workloads.config(4)
    forced = workloads.vggt_forced_blocks(wl)
    rng = np.random.default_rng(21)
    rows = np.unique(np.concatenate([[0, int(forced[-1]), wl.n_blk - 1], rng.choice(wl.n_blk, 9, replace=False)]))
    end_to_end(s3r, oracle, wl, rows=rows, forced=forced, device_gen="cuda", label="config4+reference views")


@pytest.mark.timeout(600)
def test_config4_full_size_token_queries_sampled_rows(s3r, oracle):
    """1000 views with the unpooled-query compression branch: every one of the 1,374,000 rows
    against 21,469 pooled keys; sampled query blocks against the oracle."""
    wl = workloads.config(4)
    rng = np.random.default_rng(22)
    rows = np.unique(np.concatenate([[0, wl.n_blk - 1], rng.choice(wl.n_blk, 8, replace=False)]))
    end_to_end(s3r, oracle, wl, rows=rows, with_gate=True, device_gen="cuda", token_queries=True,
               label="config4 token queries")


# --------------------------------------------------- seeded sweep over randomly drawn shapes --

def _random_case(seed):
    """One small problem with every option drawn at random (seeded): shape, data type, block size,
    special tokens, forced blocks, gate, query kind of the compression branch, input strides."""
    rng = np.random.default_rng(1000 + seed)
    dtype = "bf16" if rng.random() < 0.7 else "f32"
    block = int(rng.choice([16, 32, 64, 128]))
    heads = int(rng.integers(1, 4))
    views = int(rng.integers(1, 5))
    special = int(rng.choice([0, 0, 1, 3, 7]))
    img = int(rng.integers(max(block // 2, 2), 5 * block))       # image rows per view
    tpv = special + img
    n_blk = (views * img + block - 1) // block
    grid = None
    if rng.random() < 0.25:                                      # blocks = spatial windows of a patch grid
        window = int(rng.choice([4, 8]))
        grid = (int(rng.integers(3, 21)), int(rng.integers(3, 21)), window)
        block, img = window * window, grid[0] * grid[1]
        tpv = special + img
        n_blk = views * (-(-grid[0] // window)) * (-(-grid[1] // window))
    topk = int(rng.integers(1, 7))
    n_forced = int(rng.integers(0, min(3, n_blk) + 1)) if rng.random() < 0.4 else 0
    forced = np.sort(rng.choice(n_blk, n_forced, replace=False)).astype(np.int32) if n_forced else None
    return dict(dtype=dtype, block=block, heads=heads, views=views, special=special, tpv=tpv, topk=topk, grid=grid,
                forced=forced, with_gate=bool(rng.random() < 0.6), token_queries=bool(rng.random() < 0.3),
                strided=bool(rng.random() < 0.3), kind=str(rng.choice(["normal", "clustered", "outliers"])),
                seed=200 + seed)


@pytest.mark.parametrize("seed", range(160))
def test_random_shapes(s3r, oracle, seed):
    c = _random_case(seed)
    wl = workloads.Workload(f"random{seed}", c["views"], c["tpv"], c["heads"], 64, c["dtype"], c["block"], c["topk"],
                            c["seed"], c["kind"])
    log(f"random case {seed}: { {k: (v.tolist() if isinstance(v, np.ndarray) else v) for k, v in c.items()} }")
    q, k, v = workloads.make_inputs(wl)
    gate = workloads.make_gate_logits(wl) if c["with_gate"] else None
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    if c["strided"]:                                   # slices of one packed [n_tok, 3, heads, 64] tensor
        big = torch.stack([qd, kd, vd], dim=1).contiguous()
        qd, kd, vd = big[:, 0], big[:, 1], big[:, 2]
    res = run_device(s3r, qd, kd, vd, c["block"], c["topk"], gate=None if gate is None else gate.cuda(),
                     forced=c["forced"], tokens_per_view=c["tpv"] if (c["special"] or c["grid"]) else 0,
                     special_per_view=c["special"], grid=c["grid"], compress_queries=int(c["token_queries"]))
    host = [to_host_f32(q), to_host_f32(k), to_host_f32(v), None if gate is None else to_host_f32(gate)]
    if c["grid"]:
        stats = compare_windows_with_oracle(oracle, res, *host, c["topk"], c["dtype"], c["views"], c["tpv"],
                                            c["special"], c["grid"], forced=c["forced"], label=wl.name,
                                            token_queries=c["token_queries"])
    elif c["special"]:
        stats = compare_layer_with_oracle(oracle, res, *host, c["block"], c["topk"], c["dtype"], c["tpv"], c["special"],
                                          forced=c["forced"], label=wl.name, token_queries=c["token_queries"])
    else:
        stats = compare_with_oracle(oracle, res, *host, c["block"], c["topk"], c["dtype"], forced=c["forced"],
                                    label=wl.name, token_queries=c["token_queries"])
    log(f"random case {seed}: {stats}")


@pytest.mark.parametrize("seed", range(24))
def test_random_medium_shapes_sampled_rows(s3r, oracle, seed):
    """Hundreds to thousands of blocks (the TopK-in-the-sweep route with real candidate lists, several
    key units per split, long index rows), 14 sampled query blocks each against the oracle."""
    rng = np.random.default_rng(5000 + seed)
    dtype = "bf16" if rng.random() < 0.8 else "f32"
    block = int(rng.choice([16, 32, 64, 64, 128]))
    heads = int(rng.integers(1, 5))
    special = int(rng.choice([0, 0, 5]))
    img = int(rng.integers(300, 1400))
    views = int(rng.integers(6, 40)) * (2 if block >= 64 else 1)
    if dtype == "f32":
        views = max(views // 4, 2)                                  # the generic kernels are slow
    tpv = special + img
    n_blk = (views * img + block - 1) // block
    topk = int(rng.choice([4, 16, 32, 64, 100]))
    forced = None
    if rng.random() < 0.35:
        forced = np.sort(rng.choice(n_blk, int(rng.integers(1, 24)), replace=False)).astype(np.int32)
    kind = str(rng.choice(["normal", "clustered", "outliers"]))
    wl = workloads.Workload(f"medium{seed}", views, tpv, heads, 64, dtype, block, topk, 700 + seed, kind)
    rows = np.unique(np.concatenate([[0, n_blk - 1], rng.choice(n_blk, 12, replace=False)]))
    token_queries = bool(rng.random() < 0.25)
    log(f"medium case {seed}: {dtype} block {block} heads {heads} views {views} x {tpv} ({special} special) "
        f"n_blk {n_blk} topk {topk} forced {None if forced is None else forced.size} {kind} token_queries {token_queries}")
    q, k, v = workloads.make_inputs(wl)
    gate = workloads.make_gate_logits(wl)
    res = run_device(s3r, q.cuda(), k.cuda(), v.cuda(), block, topk, gate=gate.cuda(), forced=forced,
                     tokens_per_view=tpv if special else 0, special_per_view=special,
                     compress_queries=int(token_queries))
    host = [to_host_f32(q), to_host_f32(k), to_host_f32(v), to_host_f32(gate)]
    if special:
        spec = rng.choice(views * special, 8, replace=False)
        stats = compare_layer_with_oracle(oracle, res, *host, block, topk, dtype, tpv, special, rows=rows,
                                          spec_sample=spec, forced=forced, label=wl.name, token_queries=token_queries)
    else:
        stats = compare_with_oracle(oracle, res, *host, block, topk, dtype, rows=rows, forced=forced, label=wl.name,
                                    token_queries=token_queries)
    log(f"medium case {seed}: {stats}")


# ------------------------------------------------------------------- HIP graph capture --

def test_full_path_replays_from_a_hip_graph(s3r):
    """With a caller workspace the whole path is kernel launches on the caller's stream and nothing
    else (no allocation, no host synchronisation, no memset nodes), so it can be captured into a HIP
    graph.  Every replay, on new inputs written into the captured buffers and with eager work in
    between, must reproduce the eager result bit for bit."""
    wl = workloads.config(2)
    q, k, v = workloads.make_inputs(wl, device="cuda")
    forced = torch.tensor(workloads.vggt_forced_blocks(wl), dtype=torch.int32, device="cuda")
    n_forced = forced.numel()
    ws = torch.empty(s3r.speed3r_workspace_bytes(wl.n_tok, wl.heads, 64, wl.block, wl.topk, s3r.S3R_BF16, n_forced),
                     dtype=torch.uint8, device="cuda")
    out = torch.empty_like(q)

    def run(o):
        s3r.speed3r_sparse_global_attn_ex(q, k, v, o, wl.block, wl.topk, workspace=ws, forced_blocks=forced)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(out)                                     # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run(out)
    for seed in (11, 12, 13):
        g = torch.Generator(device="cuda").manual_seed(seed)
        for t in (q, k, v):
            t.copy_(torch.randn(t.shape, generator=g, device="cuda").to(t.dtype))
        eager = torch.empty_like(q)
        run(eager)                                   # eager work between the replays
        torch.cuda.synchronize()
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay with seed {seed} differs from the eager call"
