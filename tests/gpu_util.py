"""Helpers for the GPU parity tests: upload seeded arrays, run the HIP path
through the C ABI, run the CPU oracle on the same arrays, compare.

Acceptance (one step, identical inputs on both sides).  Every row is checked; a
row passes if, against the oracle's result under the rule or, for a nucleus row
whose running mass passes within BAND = 1e-5 of top_p at a group end, under one
of the other admissible closings of the nucleus (the oracle hands those out),
either
  (A) the token is the oracle's, |p_gpu - p| <= 1e-5 * p, and
      |c'_gpu - c'| <= max(1e-5 * c', CDF_EPS / p): the rescale divides an
      absolute error of the fp32 cumulative sums (CDF_EPS = 1e-6, in units of
      the whole distribution) by the token's probability, so a relative bound
      alone cannot hold for rare tokens in fp32;  or
  (B) the token is another one whose interval, as the oracle has it, lies
      within BAND of the code (the neighbour across an interval end the code is
      next to; a few tokens on, where the ones in between are narrower than the
      band), its probability matches the oracle's for THAT token, and its new
      code matches, to the same tolerance, the code the oracle's sums give on
      that token's interval (which lies just outside [0,1); since the GPU's
      code is inside [0,1), this in effect admits a token across an interval end
      only when the code is within CDF_EPS of that end).
Rows passing by (B) or by an alternative closing are counted and reported.
"""
import numpy as np
import torch

import oracle
from paper_2210_15458_amd import binding as B

BAND = 1e-5
CDF_EPS = 1e-6
MAX_ALT_SHIFTS = 256     # closings of the nucleus tried on either side of the oracle's for a row that needs one


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
                 max_rows=None, tuning=None):
    logits = to_dev_logits(stored)
    rows = codes.shape[0]
    ctx = B.Ctx(max_rows or max(rows, 1), V, logits.dtype)
    for knob, value in (tuning or {}).items():
        ctx.set_tuning(knob, value)
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


def _check_against(gpu, cand, rows_idx, codes, eos_id, cdf_eps=CDF_EPS):
    """Rows (indices into the GPU arrays) that pass against one oracle result `cand` (arrays aligned with rows_idx).

    Returns (pass by (A), pass by (B), |dc|*p of the (A) rows else nan, strict 1e-5-relative flag of the (A) rows).
    """
    tg = gpu["token"][rows_idx]
    have_p = "p" in gpu                                  # (an entry point without a probability record: not compared)
    pg = gpu["p"][rows_idx].astype(np.float64) if have_p else None
    cg = gpu["c_next"][rows_idx].astype(np.float64)
    fin_ok = np.ones(len(rows_idx), dtype=bool)
    flo_ok = np.ones(len(rows_idx), dtype=bool)

    def code_ok(c_ref, p_ref):
        with np.errstate(divide="ignore", invalid="ignore"):
            tol = np.maximum(1e-5 * np.abs(c_ref), cdf_eps / p_ref) + 2.0 ** -24
        return np.abs(cg - c_ref) <= tol

    # (A) same token
    p = cand["p"]
    with np.errstate(divide="ignore", invalid="ignore"):
        same = (tg == cand["token"]) & code_ok(cand["c_next"], p)
        if have_p:
            same &= np.abs(pg - p) <= 1e-5 * p
    if "f_lo" in gpu:
        flo_ok = np.abs(gpu["f_lo"][rows_idx] - cand["f_lo"]) <= 2e-6
    if "finished" in gpu:
        fin_ok = gpu["finished"][rows_idx] == cand["finished"]
    a_ok = same & flo_ok & fin_ok

    # (B) another token whose interval, as the oracle has it, lies within BAND of the code
    c = codes[rows_idx]
    b_ok = np.zeros(len(rows_idx), dtype=bool)
    other = np.nonzero(~a_ok & (tg != cand["token"]) & (cand["token"] >= 0))[0]
    if other.size:
        flo_g, p_g = oracle.interval_in(cand, other, tg[other])
        co, cgo = c[other], cg[other]
        with np.errstate(divide="ignore", invalid="ignore"):
            c_virtual = (co - flo_g) / p_g               # where the oracle's sums put the code on that interval
            tol = np.maximum(1e-5 * np.abs(c_virtual), cdf_eps / p_g) + 2.0 ** -24
            ok = (p_g > 0) & (co >= flo_g - BAND) & (co <= flo_g + p_g + BAND) & (np.abs(cgo - c_virtual) <= tol)
            if have_p:
                ok &= np.abs(pg[other] - p_g) <= 1e-5 * p_g
        if "f_lo" in gpu:
            ok &= np.abs(gpu["f_lo"][rows_idx][other] - flo_g) <= 2e-6
        if "finished" in gpu:
            ok &= gpu["finished"][rows_idx][other] == ((eos_id >= 0) & (tg[other] == eos_id)).astype(np.uint8)
        b_ok[other] = ok
    with np.errstate(invalid="ignore"):
        dcp = np.where(a_ok, np.abs(cg - cand["c_next"]) * p, np.nan)
        strict = np.abs(cg - cand["c_next"]) <= 1e-5 * np.maximum(cand["c_next"], 1e-30) + 2.0 ** -24
    return a_ok, b_ok & ~a_ok, dcp, strict


def compare_step(gpu, ref, V, label="", trunc=False, codes=None, eos_id=-1, max_alt_frac=None, cdf_eps=CDF_EPS):
    """Assert the acceptance rules above on every row; return a dict of counts.

    `ref` is oracle.step's result (with band=BAND when the nucleus is on, so that it carries the alternatives);
    `codes` the step's input codes (needed for (B); rows that would need it fail without).
    """
    tok_g, tok_o = gpu["token"], ref["token"]
    R = len(tok_o)
    assert np.all((tok_g >= 0) & (tok_g < V)), f"{label}: token outside the vocabulary"
    assert np.all((gpu["c_next"] >= 0) & (gpu["c_next"] < 1.0)), f"{label}: code outside [0,1)"
    assert np.all(tok_o >= 0), f"{label}: the oracle found a row without weight"
    codes = np.full(R, np.nan) if codes is None else np.asarray(codes, dtype=np.float32).astype(np.float64)
    allrows = np.arange(R)
    a_ok, b_ok, dcp, strict = _check_against(gpu, ref, allrows, codes, eos_id, cdf_eps)
    via_alt = np.zeros(R, dtype=bool)
    alt_rows = (np.asarray(ref["nuc_alt"]) != 0).any(axis=1) if "nuc_alt" in ref else np.zeros(R, dtype=bool)
    alts = ref.get("alt")
    if alts is not None and not (a_ok | b_ok).all():
        # only the rows that still need an answer, nearest closings first, and not without end
        for shift, idx, sub in alts.among(~(a_ok | b_ok), limit=MAX_ALT_SHIFTS):
            todo = ~(a_ok[idx] | b_ok[idx])
            if not todo.any():
                continue
            a2, b2, dcp2, strict2 = _check_against(gpu, sub, idx, codes, eos_id, cdf_eps)
            take_a, take_b = todo & a2, todo & b2 & ~a2
            via_alt[idx[take_a | take_b]] = True
            a_ok[idx[take_a]] = True
            b_ok[idx[take_b]] = True
            dcp[idx[take_a]] = dcp2[take_a]
            strict[idx[take_a]] = strict2[take_a]
            if (a_ok | b_ok).all():
                break
    bad = ~(a_ok | b_ok)
    if bad.any():
        i = int(np.nonzero(bad)[0][0])
        raise AssertionError(
            f"{label}: {bad.sum()} of {R} rows match neither the oracle nor an admissible alternative; first row {i}: "
            f"gpu token {tok_g[i]} p {gpu['p'][i] if 'p' in gpu else float('nan'):.9g} c' {gpu['c_next'][i]:.9g} "
            f"code {codes[i]:.9g} | oracle token {tok_o[i]} "
            f"p {ref['p'][i]:.9g} c' {ref['c_next'][i]:.9g} delta {ref['delta'][i]:.3g} "
            f"nuc_margin {ref['nuc_margin'][i]:.3g} alternatives {ref['nuc_alt'][i].tolist()} "
            f"tokens with weight next to the oracle's {ref['tok_nb'][i].tolist()}")
    if max_alt_frac is not None:
        assert alt_rows.mean() <= max_alt_frac, (f"{label}: {alt_rows.sum()} of {R} rows have a nucleus that closes "
                                                 f"within the band of top_p (more than {max_alt_frac:.3g})")
    # rows that miss a pure 1e-5 relative bound on the new code, by the distance c'*p of the code from the
    # start of its token's interval: the fp32 sums carry an absolute error, so these must all be close to it
    am = a_ok
    dist = np.where(am, np.asarray(ref["c_next"]) * np.asarray(ref["p"]), np.nan)
    edges = [0.0, 1e-6, 1e-5, 1e-4, 1e-3, 1e-2, 1e-1, 1.01]
    table = {}
    for lo, hi in zip(edges, edges[1:]):
        sel = am & (dist >= lo) & (dist < hi) & ~via_alt
        if sel.any():
            table[f"[{lo:g},{hi:g})"] = (int((~strict[sel]).sum()), int(sel.sum()))
    far = am & ~via_alt & (dist >= 1e5 * cdf_eps)
    assert strict[far].all(), f"{label}: a code far from its interval start misses 1e-5 relative"
    n_strict = am & ~via_alt
    return dict(rows=R, mismatches=int((tok_g != tok_o).sum()), boundary=int(b_ok.sum()),
                nucleus=int(via_alt.sum()), nucleus_rows=int(alt_rows.sum()),
                in_band=int((ref["delta"] <= BAND).sum()),
                code_within_1e5_rel=float(strict[n_strict].mean()) if n_strict.any() else 1.0,
                worst_dc_times_p=float(np.nanmax(dcp)) if np.isfinite(dcp).any() else 0.0,
                code_misses_by_distance=table)


def oracle_step(stored, codes_f32, V, nthreads=8, **kw):
    kw.setdefault("band", BAND)
    return oracle.step(stored, np.asarray(codes_f32, dtype=np.float32).astype(np.float64), V=V,
                       nthreads=nthreads, **kw)
