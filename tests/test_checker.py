"""The parity checker itself (tests/gpu_util.py: compare_step), on the CPU: it accepts what it must accept (the
oracle's own answers rounded to fp32, the token across an interval end for a code next to that end, another
admissible closing of the nucleus) and rejects planted mistakes.  The mistakes are planted in copies of the
oracle's results; no GPU is involved."""
import numpy as np
import pytest

import oracle
from gpu_util import BAND, compare_step, oracle_step
from paper_2210_15458_amd import synth

V, R = 3000, 400
TOP = np.float32(1 - 2.0 ** -24)


def _as_gpu(ref):
    return dict(token=ref["token"].copy(), c_next=np.minimum(ref["c_next"].astype(np.float32), TOP),
                p=ref["p"].astype(np.float32), f_lo=ref["f_lo"].astype(np.float32), finished=ref["finished"].copy())


def _case(**kw):
    stored = synth.gaussian_logits(R, V, seed=5, dtype="bf16")
    codes = synth.uniform_codes(R, seed=6)
    return stored, codes, oracle_step(stored, codes, V, temp=0.8, **kw)


@pytest.mark.parametrize("kw", [dict(), dict(top_k=40), dict(top_p=0.9), dict(top_k=50, top_p=0.8)])
def test_checker_accepts_the_oracle_and_rejects_planted_mistakes(kw):
    stored, codes, ref = _case(**kw)
    good = _as_gpu(ref)
    st = compare_step(good, ref, V, "self", codes=codes)
    assert st["mismatches"] == 0 and st["boundary"] == 0 and st["nucleus"] == 0
    r = int(np.argmax(np.where(np.isfinite(ref["delta"]) & (ref["tok_nb"][:, 1] >= 0), ref["delta"], 0.0)))       # a row far from every interval end
    for name, plant in [
        ("neighbouring token far from the end", lambda g: g["token"].__setitem__(r, ref["tok_nb"][r, 1])),
        ("probability off by 1e-4", lambda g: g["p"].__setitem__(r, g["p"][r] * np.float32(1.0001))),
        ("code off", lambda g: g["c_next"].__setitem__(r, np.float32(min(0.99, g["c_next"][r] + 2e-3 / ref["p"][r] + 1e-3)))),
        ("interval start off", lambda g: g["f_lo"].__setitem__(r, g["f_lo"][r] + np.float32(1e-4))),
        ("finished flag wrong", lambda g: g["finished"].__setitem__(r, 1 - g["finished"][r])),
    ]:
        bad = {k: v.copy() for k, v in good.items()}
        plant(bad)
        with pytest.raises(AssertionError):
            compare_step(bad, ref, V, name, codes=codes)


def test_checker_takes_the_token_across_a_nearby_interval_end_and_nothing_else():
    stored, codes, ref = _case()
    # move the codes of a few rows to just below the end of their token's interval: the token after it is then
    # admissible, with a code at the start of its interval; the token two further on is not
    rows = [r for r in range(R) if ref["tok_nb"][r, 1] >= 0 and ref["p_nb"][r, 1] > 1e-3][:6]
    codes = codes.copy()
    for r in rows:
        codes[r] = np.float32(ref["f_hi"][r] - 4e-7)
    ref = oracle_step(stored, codes, V, temp=0.8)
    rows = [r for r in rows if ref["delta"][r] <= BAND and ref["tok_nb"][r, 1] >= 0]
    assert len(rows) >= 3
    gpu = _as_gpu(ref)
    for r in rows:
        nxt = ref["tok_nb"][r, 1]
        gpu["token"][r] = nxt
        gpu["p"][r] = np.float32(ref["p_nb"][r, 1])
        gpu["c_next"][r] = 0.0
        gpu["f_lo"][r] = np.float32(ref["f_hi"][r])
    st = compare_step(gpu, ref, V, "across the end", codes=codes)
    assert st["boundary"] == len(rows) and st["mismatches"] == len(rows)
    # (the new code has to fit as well, which in effect narrows the band to the tolerance of the sums: a code
    # 5e-6 below the end cannot come out at the start of the next interval without an error of 5e-6 in the sums)
    c2 = codes.copy()
    c2[rows[0]] = np.float32(ref["f_hi"][rows[0]] - 5e-6)
    ref2 = oracle_step(stored, c2, V, temp=0.8)
    with pytest.raises(AssertionError):
        compare_step(gpu, ref2, V, "too far below the end", codes=c2)
    # the same token with a code in the middle of its interval is a wrong answer
    bad = {k: v.copy() for k, v in gpu.items()}
    bad["c_next"][rows[0]] = 0.5
    with pytest.raises(AssertionError):
        compare_step(bad, ref, V, "middle of the neighbour", codes=codes)
    # a token whose interval is not next to the code is a wrong answer however small the distance to the end
    bad = {k: v.copy() for k, v in gpu.items()}
    far = int(np.argmax(ref["p"]))
    r0 = rows[0] if gpu["token"][rows[0]] != ref["token"][far] else rows[1]
    bad["token"][r0] = (gpu["token"][r0] + 7) % V
    with pytest.raises(AssertionError):
        compare_step(bad, ref, V, "some other token", codes=codes)


def test_checker_takes_another_admissible_nucleus_and_nothing_else():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal((40, 500)) * 2).astype(np.float32)
    stored = synth.f32_to_bf16_bits(x)
    codes = synth.uniform_codes(40, seed=9)
    # put top_p a hair above the mass of the first few groups of row 7: the rule keeps one group more than the
    # alternative one closing earlier
    wide = synth.bf16_bits_to_f32(stored[7]).astype(np.float64)
    p = np.exp(wide - wide.max()); p /= p.sum()
    vals = np.unique(wide)[::-1]
    cum = np.cumsum([p[wide == v].sum() for v in vals])
    top_p = float(cum[5] + 3e-6)
    ref = oracle_step(stored, codes, 500, top_p=top_p)
    assert ref["nuc_alt"][7].tolist() == [1, 0]
    (shift, idx, sub), = [a for a in ref["alt"] if a[0] == -1]
    j = int(np.nonzero(idx == 7)[0][0])
    gpu = _as_gpu(ref)
    for k in ("token", "p", "f_lo"):
        gpu[k][7] = sub[k][j]
    gpu["c_next"][7] = min(np.float32(sub["c_next"][j]), TOP)
    st = compare_step(gpu, ref, 500, "other closing", codes=codes, max_alt_frac=0.5)
    assert st["nucleus_rows"] >= 1 and st["nucleus"] == (1 if sub["p"][j] != ref["p"][7] else 0)
    with pytest.raises(AssertionError):                 # too many such rows for a peaked distribution
        compare_step(gpu, ref, 500, "bounded", codes=codes, max_alt_frac=0.0)
    # the same change on a row whose nucleus closes nowhere near top_p is a wrong answer
    for clear in np.argsort(-ref["nuc_margin"]):
        other = oracle.step(stored[clear:clear + 1], codes[clear:clear + 1].astype(np.float64), V=500, top_p=top_p,
                            nuc_shift=-1)
        if other["n_kept"][0] != ref["n_kept"][clear]:      # (a nucleus of one group cannot close any earlier)
            break
    assert ref["nuc_margin"][clear] > 1e-3
    bad = _as_gpu(ref)
    for k in ("token", "p", "f_lo"):
        bad[k][clear] = other[k][0]
    bad["c_next"][clear] = min(np.float32(other["c_next"][0]), TOP)
    with pytest.raises(AssertionError):
        compare_step(bad, ref, 500, "closing moved on a clear row", codes=codes)
