"""Helpers for the GPU parity tests: upload seeded arrays, run the HIP path
through the C ABI, run the CPU oracle on the same arrays, compare.

Acceptance (one step, identical inputs on both sides):
  tokens   identical on every row whose code is farther than BAND = 1e-5 from
           every interior end of the emitted token's interval (the oracle's
           `delta`); a row inside the band may emit the neighbouring token and
           is counted.  Nucleus rows whose cumulative mass is within BAND of
           top_p at the closing group are a second, separately counted class.
  prob     |p_gpu - p| <= 1e-5 * p on rows with matching tokens.
  code     |c'_gpu - c'| <= max(1e-5 * c', CDF_EPS / p): the rescale divides an
           absolute error of the fp32 cumulative sums (CDF_EPS = 1e-6, in units
           of the whole distribution) by the token's probability, so a relative
           bound alone cannot hold for rare tokens in fp32.
"""
import numpy as np
import torch

import oracle
from paper_2210_15458_amd import binding as B

BAND = 1e-5
CDF_EPS = 1e-6


def to_dev_logits(stored):
    """uint16 bf16 bits -> torch.bfloat16 on the GPU; float32 -> float32."""
    if stored.dtype == np.uint16:
        return torch.from_numpy(stored.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(stored).cuda()


def from_dev_logits(t):
    """GPU logits -> stored NumPy form (uint16 bits for bf16)."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def run_gpu_step(stored, codes, V, temp=1.0, top_k=0, top_p=1.0, finished=None, eos_id=-1, row_ids=None,
                 max_rows=None):
    logits = to_dev_logits(stored)
    rows = codes.shape[0]
    ctx = B.Ctx(max_rows or max(rows, 1), V, logits.dtype)
    c = torch.from_numpy(np.ascontiguousarray(codes, dtype=np.float32)).cuda()
    tok = torch.full((rows,), -7, dtype=torch.int32, device="cuda")
    cout = torch.full((rows,), -1.0, dtype=torch.float32, device="cuda")
    prob = torch.full((rows,), -1.0, dtype=torch.float32, device="cuda")
    flo = torch.full((rows,), -1.0, dtype=torch.float32, device="cuda")
    fout = torch.full((rows,), 9, dtype=torch.uint8, device="cuda")
    fin = None if finished is None else torch.from_numpy(np.ascontiguousarray(finished, np.uint8)).cuda()
    rid = None if row_ids is None else torch.from_numpy(np.ascontiguousarray(row_ids, np.int32)).cuda()
    B.as_step_ex(ctx, logits, c, temp, top_k, top_p, tok, cout, finished_in=fin, eos_id=eos_id,
                 finished_out=fout, prob_out=prob, flo_out=flo, row_ids=rid)
    torch.cuda.synchronize()
    out = dict(token=tok.cpu().numpy(), c_next=cout.cpu().numpy(), p=prob.cpu().numpy(),
               f_lo=flo.cpu().numpy(), finished=fout.cpu().numpy())
    ctx.close()
    return out


def compare_step(gpu, ref, V, label="", trunc=False):
    """Assert the acceptance rules above; return a dict of counts."""
    tok_g, tok_o = gpu["token"], ref["token"]
    assert np.all((tok_g >= 0) & (tok_g < V)), f"{label}: token outside the vocabulary"
    assert np.all((gpu["c_next"] >= 0) & (gpu["c_next"] < 1.0)), f"{label}: code outside [0,1)"
    mism = tok_g != tok_o
    near = ref["delta"] <= BAND
    nuc = ref["nuc_margin"] <= BAND if trunc else np.zeros_like(mism)
    bad = mism & ~near & ~nuc
    assert not bad.any(), (f"{label}: {bad.sum()} token mismatches away from any boundary; first rows "
                           f"{np.nonzero(bad)[0][:5]}, gpu {tok_g[bad][:5]}, oracle {tok_o[bad][:5]}, "
                           f"delta {ref['delta'][bad][:5]}")
    # rows whose nucleus closes within the band of top_p may keep one group more or less than the oracle: their
    # tokens are excused above, and their probabilities and codes are not comparable either (another kept set
    # is another normalisation); they are counted below
    ok = ~mism & ~nuc
    p = ref["p"][ok]
    rel_p = np.abs(gpu["p"][ok] - p) / p
    assert np.all(rel_p <= 1e-5), f"{label}: probability off by {rel_p.max():.3g} relative"
    dc = np.abs(gpu["c_next"][ok].astype(np.float64) - ref["c_next"][ok])
    tol = np.maximum(1e-5 * ref["c_next"][ok], CDF_EPS / p) + 2.0 ** -24
    assert np.all(dc <= tol), (f"{label}: code off: worst |dc|*p = {(dc * p).max():.3g}, "
                               f"rows {np.nonzero(dc > tol)[0][:5]}")
    if "f_lo" in gpu:
        assert np.all(np.abs(gpu["f_lo"][ok] - ref["f_lo"][ok]) <= 2e-6)
    if "finished" in gpu and "finished" in ref:
        assert np.array_equal(gpu["finished"][ok], ref["finished"][ok])
    strict = dc <= 1e-5 * np.maximum(ref["c_next"][ok], 1e-30) + 2.0 ** -24
    return dict(rows=len(tok_o), mismatches=int(mism.sum()), boundary=int((mism & near).sum()),
                nucleus=int((mism & nuc & ~near).sum()), nucleus_rows=int(np.sum(nuc)), in_band=int(near.sum()),
                code_within_1e5_rel=float(strict.mean()) if strict.size else 1.0, worst_dc_times_p=float((dc * p).max(initial=0.0)),
                worst_rel_p=float(rel_p.max(initial=0.0)))


def oracle_step(stored, codes_f32, V, nthreads=8, **kw):
    return oracle.step(stored, np.asarray(codes_f32, dtype=np.float32).astype(np.float64), V=V,
                       nthreads=nthreads, **kw)
