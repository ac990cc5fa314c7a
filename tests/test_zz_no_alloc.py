"""GPU test of speed3r_sparse_global_attn_noalloc: the entry point for callers that cannot allocate
(its scratch is a fixed device array inside the library).  Its output must equal that of
speed3r_sparse_global_attn (library-held hipMalloc scratch, same kernels) bit for bit, on two calls in a
row that share the static array, the second on a smaller problem; and both are held to the oracle's bar."""
import numpy as np
import pytest
import torch

from paper_2603_08055_amd import workloads
from tests.parity_util import compare_with_oracle, log, run_device, to_host_f32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def s3r():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2603_08055_amd import speed3r
    speed3r.load()
    return speed3r


def draw(n_tok, heads, seed):
    g = torch.Generator().manual_seed(seed)
    return tuple(torch.randn((n_tok, heads, 64), generator=g).to(torch.bfloat16).cuda() for _ in range(3))


def test_noalloc_entry_matches_short_form_twice(s3r, oracle):
    # call 1: config 2 (8 views x 1374 tokens, 16 heads, block 64, top-16: 57 MiB of the 64 MiB array);
    # call 2: a smaller, ragged problem with another block size, which reuses the front of the same array
    wl = workloads.config(2)
    q, k, v = (t.cuda() for t in workloads.make_inputs(wl))
    cases = [(q, k, v, wl.block, wl.topk), (*draw(3 * 700 + 13, 5, 77), 32, 8)]
    for n, (q, k, v, block, topk) in enumerate(cases):
        log(f"noalloc call {n}: n_tok={q.shape[0]} heads={q.shape[1]} block={block} topk={topk}")
        need = s3r.speed3r_workspace_bytes(q.shape[0], q.shape[1], 64, block, topk, s3r.S3R_BF16)
        assert need <= s3r.STATIC_SCRATCH_BYTES
        got = torch.full(q.shape, float("nan"), dtype=q.dtype, device="cuda")
        s3r.speed3r_sparse_global_attn_noalloc(q, k, v, got, block, topk)
        torch.cuda.synchronize()
        want = torch.full(q.shape, float("nan"), dtype=q.dtype, device="cuda")
        s3r.speed3r_sparse_global_attn(q, k, v, want, block, topk)
        torch.cuda.synchronize()
        assert torch.isfinite(got.float()).all()
        assert torch.equal(got.view(torch.int16), want.view(torch.int16)), \
            f"call {n}: {(got.float() - want.float()).abs().max().item()}"
        # and against the oracle, through the index sets of the full path on the same inputs
        res = run_device(s3r, q, k, v, block, topk)
        assert torch.equal(res["out"].view(torch.int16), got.view(torch.int16))
        rows = None if n == 1 else np.arange(0, 172, 7)
        res["out"] = got
        compare_with_oracle(oracle, res, to_host_f32(q), to_host_f32(k), to_host_f32(v), None, block, topk, "bf16",
                            rows=rows, label=f"noalloc call {n}")


def test_noalloc_entry_refuses_what_does_not_fit(s3r):
    q, k, v = draw(64 * 1374, 16, 5)      # needs several hundred MiB
    out = torch.zeros_like(q)
    with pytest.raises(s3r.Speed3rError) as e:
        s3r.speed3r_sparse_global_attn_noalloc(q, k, v, out, 64, 32)
    assert e.value.status == s3r.S3R_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert float(out.float().abs().max()) == 0.0          # nothing was enqueued
