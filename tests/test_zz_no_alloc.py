"""as_step_static, the entry point that allocates nothing, against as_step on the same inputs: the two share
their kernels, so tokens and codes must be identical bit for bit.  Two calls in a row on one GPU share the
static workspace; the second is smaller, and what the first left behind must not leak into it."""
import numpy as np
import pytest
import torch

from paper_2210_15458_amd import binding as B
from paper_2210_15458_amd import synth

pytestmark = pytest.mark.gpu


def _inputs(rows, V, ld, dtype, seed):
    rng = np.random.Generator(np.random.Philox(key=[seed, 77]))
    x = (3.0 * rng.standard_normal((rows, ld))).astype(np.float32)
    logits = torch.from_numpy(x).cuda().to(dtype).contiguous()
    codes = torch.from_numpy(rng.random(rows).astype(np.float32)).cuda()
    return logits, codes


def _both(rows, V, ld, dtype, seed, temp, top_k, top_p):
    logits, codes = _inputs(rows, V, ld, dtype, seed)
    ctx = B.Ctx(rows, V, dtype)
    tok_a = torch.full((rows,), -1, dtype=torch.int32, device="cuda")
    c_a = torch.full((rows,), -1.0, dtype=torch.float32, device="cuda")
    B.as_step(ctx, logits, codes, temp, top_k, top_p, tok_a, c_a)
    tok_b = torch.full((rows,), -2, dtype=torch.int32, device="cuda")
    c_b = torch.full((rows,), -2.0, dtype=torch.float32, device="cuda")
    B.as_step_static(logits, V, codes, temp, top_k, top_p, tok_b, c_b)
    torch.cuda.synchronize()
    ctx.close()
    return tok_a.cpu().numpy(), c_a.cpu().numpy(), tok_b.cpu().numpy(), c_b.cpu().numpy()


# (dtype, V, ld, top_k, top_p): the first three go through the threshold kernel and the static workspace
CASES = [
    (torch.float32, 5000, 5000, 0, 0.9),          # fp32 nucleus: threshold kernel, then the sampling kernel
    (torch.bfloat16, 40000, 40000, 50, 1.0),      # rows beyond 32768 logits: streamed threshold kernel
    (torch.float32, 3001, 3003, 300, 0.8),        # k above 128, ragged rows
    (torch.bfloat16, 4096, 4096, 40, 1.0),        # finished inside the top-k kernel: workspace unused
    (torch.bfloat16, 4096, 4096, 0, 1.0),         # no truncation
]


@pytest.mark.parametrize("dtype,V,ld,top_k,top_p", CASES)
def test_static_entry_point_equals_as_step_twice_in_a_row(dtype, V, ld, top_k, top_p):
    for rows, seed in ((700, 1), (130, 2)):       # the second call is smaller
        tok_a, c_a, tok_b, c_b = _both(rows, V, ld, dtype, seed, 0.9, top_k, top_p)
        assert np.array_equal(tok_a, tok_b), f"rows={rows}: tokens differ"
        assert np.array_equal(c_a.view(np.uint32), c_b.view(np.uint32)), f"rows={rows}: codes differ"
        assert np.all((tok_a >= 0) & (tok_a < V))


def test_static_entry_point_refuses_what_does_not_fit():
    logits, codes = _inputs(4, 64, 64, torch.float32, 3)
    tok = torch.zeros(4, dtype=torch.int32, device="cuda")
    L = B.lib()
    rc = L.as_step_static(logits.data_ptr(), 0, 65537, 64, 64, codes.data_ptr(), 1.0, 0, 1.0, tok.data_ptr(),
                          codes.data_ptr(), None)
    assert rc == 1 and b"AS_STATIC_MAX_ROWS" in L.as_last_error(None)
    rc = L.as_step_static(logits.data_ptr(), 0, 4, 32, 64, codes.data_ptr(), 1.0, 0, 1.0, tok.data_ptr(),
                          codes.data_ptr(), None)
    assert rc == 1 and b"ld" in L.as_last_error(None)
    rc = L.as_step_static(logits.data_ptr(), 0, 0, 64, 64, None, 1.0, 0, 1.0, None, None, None)
    assert rc == 0                                # nothing to do
