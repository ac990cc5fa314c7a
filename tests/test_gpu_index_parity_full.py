"""GPU parity of the selected block indices over whole problems (Sec. 3.2 "Selection Branch"): every
query block of config 3 against the oracle's scores; at configs 4 and 5 (full size, the launch
configuration bench.py times) 1024 query blocks x all heads against the oracle, and ALL rows of the two
device TopK routes (inside the compression sweep / from scores written to memory) against each other,
every row on which they differ being validated against the oracle's scores as well."""
import numpy as np
import pytest
import torch

from paper_2603_08055_amd import workloads
from tests.parity_util import check_topk_sets_fast, log, to_host_f32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def s3r():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2603_08055_amd import speed3r
    speed3r.load()
    return speed3r


def device_indices(s3r, q, k, v, wl, choice=0):
    """TopK index tensor [heads, n_blk, k] of the whole path under kernel choice `choice`."""
    kk = min(wl.topk, wl.n_blk)
    idx = torch.full((wl.heads, wl.n_blk, kk), -1, dtype=torch.int32, device="cuda")
    out = torch.empty_like(q)
    s3r.speed3r_set_kernel_choice(choice)
    try:
        s3r.speed3r_sparse_global_attn_ex(q, k, v, out, wl.block, wl.topk, topk_idx=idx)
        torch.cuda.synchronize()
    finally:
        s3r.speed3r_set_kernel_choice(0)
    return idx


def check_rows(oracle, qc, kc, gidx, rows, k, chunk):
    """Near-tie rule on the query blocks `rows` (all heads), scores from the oracle in chunks of rows."""
    n_exact = n_tie = 0
    for c0 in range(0, len(rows), chunk):
        r = np.asarray(rows[c0:c0 + chunk], dtype=np.int64)
        s = oracle.scores(qc, kc, r)
        e, t = check_topk_sets_fast(s, gidx[:, r], k)
        n_exact += e
        n_tie += t
    return n_exact, n_tie


def check_pairs(oracle, qc, kc, gidx_list, pairs, k, chunk):
    """Near-tie rule on single (head, query block) pairs for each index tensor of gidx_list."""
    counts = [[0, 0] for _ in gidx_list]
    for c0 in range(0, len(pairs), chunk):
        part = pairs[c0:c0 + chunk]
        rows = np.unique(part[:, 1])
        s = oracle.scores(qc, kc, rows)
        pos = {int(r): i for i, r in enumerate(rows)}
        for h, r in part:
            i = pos[int(r)]
            for n, g in enumerate(gidx_list):
                e, t = check_topk_sets_fast(s[h:h + 1, i:i + 1], g[h:h + 1, r:r + 1], k)
                counts[n][0] += e
                counts[n][1] += t
    return counts


def pooled_on_host(oracle, q, k, block):
    return oracle.pool(to_host_f32(q), block), oracle.pool(to_host_f32(k), block)


@pytest.mark.timeout(600)
def test_config3_index_parity_every_row(s3r, oracle):
    wl = workloads.config(3)
    q, k, v = workloads.make_inputs(wl, device="cuda")
    gidx = device_indices(s3r, q, k, v, wl).cpu().numpy()
    qc, kc = pooled_on_host(oracle, q, k, wl.block)
    n_exact, n_tie = check_rows(oracle, qc, kc, gidx, np.arange(wl.n_blk), wl.topk, 256)
    log(f"config 3, all {wl.heads * wl.n_blk} rows: {n_exact} exact, {n_tie} tie-resolved")
    assert n_exact + n_tie == wl.heads * wl.n_blk


def full_size_case(s3r, oracle, wl, n_sample, seed):
    log(f"{wl.name} top-{wl.topk}: inputs")
    q, k, v = workloads.make_inputs(wl, device="cuda")
    k_eff = min(wl.topk, wl.n_blk)
    a = device_indices(s3r, q, k, v, wl, choice=0)
    b = device_indices(s3r, q, k, v, wl, choice=2)
    differ = (a != b).any(dim=2)
    pairs = differ.nonzero().cpu().numpy()              # [n, 2] = (head, query block)
    n_rows = wl.heads * wl.n_blk
    log(f"{wl.name} top-{wl.topk}: the two TopK routes differ on {len(pairs)} of {n_rows} rows")
    assert len(pairs) <= 0.01 * n_rows
    a_h, b_h = a.cpu().numpy(), b.cpu().numpy()
    del a, b, v
    qc, kc = pooled_on_host(oracle, q, k, wl.block)
    del q, k
    rng = np.random.default_rng(seed)
    rows = np.unique(np.concatenate([[0, 1, wl.n_blk - 2, wl.n_blk - 1],
                                     rng.choice(wl.n_blk, n_sample - 4, replace=False)]))
    n_exact, n_tie = check_rows(oracle, qc, kc, a_h, rows, k_eff, 64)
    log(f"{wl.name} top-{wl.topk}: {len(rows)} query blocks x {wl.heads} heads vs oracle: "
        f"{n_exact} exact, {n_tie} tie-resolved")
    assert n_exact + n_tie == len(rows) * wl.heads
    if len(pairs):
        take = pairs if len(pairs) <= 4096 else pairs[rng.choice(len(pairs), 4096, replace=False)]
        take = take[np.argsort(take[:, 1], kind="stable")]
        (ea, ta), (eb, tb) = check_pairs(oracle, qc, kc, [a_h, b_h], take, k_eff, 64)
        log(f"{wl.name} top-{wl.topk}: {len(take)} differing rows vs oracle: in-sweep route {ea} exact / {ta} "
            f"tie-resolved, stored-score route {eb} exact / {tb} tie-resolved")
        assert ea + ta == len(take) and eb + tb == len(take)


@pytest.mark.timeout(900)
def test_config4_index_parity_sampled_and_route_agreement(s3r, oracle):
    full_size_case(s3r, oracle, workloads.config(4), 1024, 41)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("topk", [16, 64])
def test_config5_index_parity_sampled_and_route_agreement(s3r, oracle, topk):
    full_size_case(s3r, oracle, workloads.config(5, topk=topk), 1024, 51 + topk)
