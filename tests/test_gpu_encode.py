"""GPU parity of the encode direction (sequence -> code interval, Sec. 4.1) against the CPU oracle."""
import math

import numpy as np
import pytest

from paper_2210_15458_amd import synth

pytestmark = pytest.mark.gpu

REL = 1e-5          # relative tolerance on a token's probability (fp32 weights, fp64 sums)
ABS_F = 2e-6        # absolute tolerance on a cumulative probability in [0, 1]


def _interval_step(stored, tokens, V, temp=1.0, top_k=0, top_p=1.0, finished=None, eos_id=-1, lo0=None, w0=None,
                   tuning=None):
    import torch
    from paper_2210_15458_amd import binding as B
    from gpu_util import to_dev_logits
    logits = to_dev_logits(stored)
    R = tokens.shape[0]
    ctx = B.Ctx(R, V, logits.dtype)
    for knob, value in (tuning or {}).items():
        ctx.set_tuning(knob, value)
    lo = torch.from_numpy(np.zeros(R) if lo0 is None else lo0.copy()).cuda()
    w = torch.from_numpy(np.ones(R) if w0 is None else w0.copy()).cuda()
    fin_in = None if finished is None else torch.from_numpy(finished.astype(np.uint8)).cuda()
    fin_out = torch.full((R,), 7, dtype=torch.uint8, device="cuda") if eos_id >= 0 else None
    B.as_interval_step(ctx, logits, torch.from_numpy(tokens.astype(np.int32)).cuda(), temp, top_k, top_p, lo, w,
                       finished_in=fin_in, eos_id=eos_id, finished_out=fin_out)
    torch.cuda.synchronize()
    ctx.close()
    return lo.cpu().numpy(), w.cpu().numpy(), None if fin_out is None else fin_out.cpu().numpy()


_MODS = [(1.0, 0, 1.0), (0.7, 0, 1.0), (1.0, 40, 1.0), (1.0, 0, 0.9)]
# rows that start on and off 16 bytes (odd strides), rows shorter than a
# block's one sweep and rows of many sweeps, every logit modifier on the general shapes, the untruncated ones
# on three more lengths, one plain case on the large vocabulary
_INTERVAL_CASES = (
    [(dt, V, ld, *m) for dt in ("bf16", "f32") for (V, ld) in [(32128, None), (1001, None), (1001, 1008), (5, None)]
     for m in _MODS]
    + [(dt, V, None, *m) for dt in ("bf16", "f32") for V in (12000, 16384, 16392) for m in _MODS[:2]]
    + [("bf16", 256000, None, 1.0, 0, 1.0), ("bf16", 1 << 21, None, 1.0, 0, 1.0), ("f32", (1 << 21) - 5, None, 0.8, 40, 1.0)])


@pytest.mark.parametrize("dtype,V,ld,temp,top_k,top_p", _INTERVAL_CASES)
def test_interval_step_matches_oracle(dtype, V, ld, temp, top_k, top_p):
    import oracle
    R = 8 if V > 1000000 else (24 if V > 100000 else 48)
    stored = synth.gaussian_logits(R, V, sigma=3.0, seed=V + 5, dtype=dtype, ld=ld)
    rng = np.random.default_rng(V)
    # half the tokens where the mass is (decoded from uniform codes), half anywhere
    codes = rng.random(R)
    likely = oracle.step(stored, codes, temp=temp, top_k=top_k, top_p=top_p, V=V)["token"]
    tokens = np.where(np.arange(R) % 2 == 0, likely, rng.integers(0, V, R)).astype(np.int32)
    f_lo, p = oracle.token_interval(stored, tokens, temp=temp, top_k=top_k, top_p=top_p, V=V, nthreads=8)
    # a row whose nucleus closes within 1e-5 of top_p may close a group earlier or later: every admissible
    # closing the oracle counts for it is tried, and the row must match one of them
    nuc_alt = oracle.step(stored, codes, temp=temp, top_k=top_k, top_p=top_p, V=V, band=1e-5)["nuc_alt"]
    lo0 = rng.random(R) * 0.5
    w0 = rng.random(R) * 0.5
    lo, w, _ = _interval_step(stored, tokens, V, temp=temp, top_k=top_k, top_p=top_p, lo0=lo0, w0=w0)

    def matches(r, f_lo_r, p_r):
        return (abs(w[r] - w0[r] * p_r) <= REL * w0[r] * p_r + 1e-300 and
                abs(lo[r] - (lo0[r] + w0[r] * f_lo_r)) <= w0[r] * ABS_F + 1e-15)

    for r in range(R):
        if matches(r, f_lo[r], p[r]):
            continue
        shifts = [s for s in range(-int(nuc_alt[r, 0]), int(nuc_alt[r, 1]) + 1) if s != 0]
        alts = [oracle.token_interval(stored[r:r + 1], tokens[r:r + 1], temp=temp, top_k=top_k, top_p=top_p, V=V,
                                      nuc_shift=s) for s in shifts]
        assert any(matches(r, a[0][0], a[1][0]) for a in alts), (r, w[r], w0[r] * p[r], lo[r], f_lo[r], shifts)


def test_interval_step_finished_rows_and_bad_tokens():
    import oracle
    V, R, eos = 1000, 40, 3
    stored = synth.gaussian_logits(R, V, sigma=3.0, seed=9, dtype="bf16")
    rng = np.random.default_rng(9)
    tokens = rng.integers(0, V, R).astype(np.int32)
    tokens[5] = eos
    tokens[6] = -1          # outside the vocabulary: probability zero
    tokens[7] = V + 3
    fin = (rng.random(R) < 0.3)
    fin[5] = fin[6] = fin[7] = False
    lo, w, fout = _interval_step(stored, tokens, V, finished=fin, eos_id=eos)
    f_lo, p = oracle.token_interval(stored, np.clip(tokens, 0, V - 1), V=V, finished=fin.astype(np.uint8))
    for r in range(R):
        if fin[r]:
            assert lo[r] == 0.0 and w[r] == 1.0 and fout[r] == 1
        elif r in (6, 7):
            assert w[r] == 0.0 and fout[r] == 0
        else:
            assert abs(w[r] - p[r]) <= REL * p[r] and abs(lo[r] - f_lo[r]) <= ABS_F
            assert fout[r] == (1 if tokens[r] == eos else 0)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_interval_single_tile_kernel_edges(dtype):
    """Rows of whole vectors that fit one tile take a kernel of their own (the single-tile sampling kernel with a
    look-up in place of the search): tokens at the ends of elements, lanes, chunks, shares and of the row, tokens
    outside the vocabulary, rows whose first chunk is tiny against what follows (sums beyond fp32: the block
    falls back to the one-pass routine), masked rows, truncation, short and ragged rows; the one-pass kernel on
    the same rows (the step-shape knob) must agree."""
    import oracle
    V = 32128 if dtype == "bf16" else 16000
    epv = 8 if dtype == "bf16" else 4
    rng = np.random.default_rng(491)
    places = [0, 1, epv - 1, epv, 64 * epv - 1, 64 * epv, 1024 * epv - 1, 1024 * epv, 2048 * epv + 3, V - epv - 1, V - epv,
              V - 1]
    R = len(places) + 6
    x = rng.normal(0.0, 3.0, (R, V)).astype(np.float32)
    tokens = np.array(places + [5, 700, V // 2, -1, V, V + 100], dtype=np.int32)
    x[len(places), :600] = -80.0; x[len(places), 700] = 80.0             # a first chunk that says little
    x[len(places) + 1, :] = -60.0; x[len(places) + 1, 700] = 70.0         # the token is the far outlier itself
    x[len(places) + 2, 1::2] = -np.inf
    stored = synth.f32_to_bf16_bits(x) if dtype == "bf16" else x
    for temp, top_k, top_p in [(1.0, 0, 1.0), (0.5, 0, 1.0), (1.0, 40, 1.0), (1.0, 0, 0.9), (0.05, 0, 1.0)]:
        ok_tok = np.clip(tokens, 0, V - 1)
        f_lo, p = oracle.token_interval(stored, ok_tok, temp=temp, top_k=top_k, top_p=top_p, V=V, nthreads=8)
        res = {}
        for shape in (0, 6):
            lo, w, _ = _interval_step(stored, tokens, V, temp=temp, top_k=top_k, top_p=top_p, tuning={"step_shape": shape})
            res[shape] = (lo, w)
            for r in range(R):
                if tokens[r] < 0 or tokens[r] >= V:
                    assert w[r] == 0.0 and lo[r] == (0.0 if tokens[r] < 0 else 1.0), (temp, top_k, top_p, shape, r, lo[r], w[r])
                else:
                    # (weights are fp32 against the row's reference: probabilities below 2^-126 come out as 0)
                    assert abs(w[r] - p[r]) <= REL * p[r] + 1e-36, (temp, top_k, top_p, shape, r, w[r], p[r])
                    assert abs(lo[r] - f_lo[r]) <= ABS_F, (temp, top_k, top_p, shape, r, lo[r], f_lo[r])
        # (the one-pass kernel, with a reference per thread, keeps probabilities below 2^-126 that the other loses)
        assert np.allclose(res[0][1], res[6][1], rtol=2e-5, atol=1e-36) and np.allclose(res[0][0], res[6][0], rtol=0, atol=2e-6)
    for Vs in (epv, 64 * epv, 65 * epv, 1024 * epv, 1025 * epv, 4096 * epv - epv, 4096 * epv):
        st = synth.gaussian_logits(7, Vs, sigma=3.0, seed=Vs, dtype=dtype)
        tk = rng.integers(0, Vs, 7).astype(np.int32)
        tk[0], tk[1] = 0, Vs - 1
        f_lo, p = oracle.token_interval(st, tk, temp=0.8, V=Vs, nthreads=8)
        lo, w, _ = _interval_step(st, tk, Vs, temp=0.8)
        assert np.all(np.abs(w - p) <= REL * p) and np.all(np.abs(lo - f_lo) <= ABS_F), Vs


def _model(V, d, dtype, seed=0):
    import torch
    from paper_2210_15458_amd import binding as B
    from gpu_util import to_dev_logits
    E, U = synth.bigram_weights(V, d, seed=seed, dtype=dtype)
    Ed, Ud = to_dev_logits(E), to_dev_logits(U)
    model = B.Model(Ed, Ud, scale=3.0)
    torch.cuda.synchronize()
    return E, U, Ed, model


@pytest.mark.parametrize("cfg_id,T,top_k,top_p", [(0, 8, 0, 1.0), (1, 3, 0, 1.0), (1, 3, 40, 1.0), (1, 3, 0, 0.9),
                                                  (1, 3, 300, 0.8), (0, 8, 5, 0.7)])
def test_encode_inverts_decode(cfg_id, T, top_k, top_p):
    """The interval of a decoded sequence contains the code it was decoded from (Sec. 4.1), for as long as
    the interval is wide against the rounding of an fp32 code.  With truncation both directions have to keep
    the same tokens of every row (the decode's fused kernels and the encode's threshold kernel agree)."""
    import torch
    from paper_2210_15458_amd import binding as B
    cfg = synth.CONFIGS[cfg_id]
    V, d, Bn, N = cfg["V"], cfg["d"], cfg["B"], cfg["N"]
    tdt = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    E, U, Ed, model = _model(V, d, cfg["dtype"])
    R = Bn * N
    ctx = B.Ctx(R, V, tdt)
    prompts = torch.from_numpy(synth.prompts(Bn, V, seed=1)).cuda()
    u = torch.from_numpy(synth.shifts(Bn, seed=2)).cuda()
    codes0 = torch.empty(R, dtype=torch.float32, device="cuda")
    B.as_lattice(ctx, u, N, codes0)
    inside = total = 0
    for t_len in range(1, T + 1):
        tokens = torch.empty((Bn, N, t_len), dtype=torch.int32, device="cuda")
        B.as_decode(ctx, model, prompts, N, t_len, u, cfg["temp"], top_k, top_p, cfg["eos_id"], tokens)
        lo = torch.empty(R, dtype=torch.float64, device="cuda")
        w = torch.empty(R, dtype=torch.float64, device="cuda")
        B.as_encode(ctx, model, prompts, N, t_len, tokens, cfg["temp"], top_k, top_p, cfg["eos_id"], lo, w)
        torch.cuda.synchronize()
        c = codes0.cpu().numpy().astype(np.float64)
        lo_h, w_h = lo.cpu().numpy(), w.cpu().numpy()
        assert np.all(w_h > 0) and np.all(lo_h >= 0) and np.all(lo_h + w_h <= 1 + 1e-9)
        wide = w_h > 1e-4                                   # the fp32 decode has resolved this interval cleanly
        slack = 2e-6                                        # cumulative rounding of the fp32 path, code units
        ok = (c >= lo_h - slack) & (c < lo_h + w_h + slack)
        assert np.all(ok[wide]), (t_len, int((~ok & wide).sum()))
        inside += int(ok[wide].sum()); total += int(wide.sum())
    print("codes inside their sequence's interval:", inside, "of", total, flush=True)
    assert total > R
    ctx.close(); model.close()


def test_encode_matches_oracle_on_tiny_config():
    import torch
    import oracle
    from paper_2210_15458_amd import binding as B
    cfg = synth.CONFIGS[0]
    V, d, Bn, N, T = cfg["V"], cfg["d"], cfg["B"], cfg["N"], cfg["T"]
    E, U, Ed, model = _model(V, d, cfg["dtype"])
    R = Bn * N
    ctx = B.Ctx(R, V, torch.float32)
    prompts_h = synth.prompts(Bn, V, seed=1)
    rng = np.random.default_rng(3)
    tokens_h = rng.integers(0, V, (Bn, N, T)).astype(np.int32)
    for eos in (-1, 1):
        lo = torch.empty(R, dtype=torch.float64, device="cuda")
        w = torch.empty(R, dtype=torch.float64, device="cuda")
        B.as_encode(ctx, model, torch.from_numpy(prompts_h).cuda(), N, T, torch.from_numpy(tokens_h).cuda(), 1.0, 0,
                    1.0, eos, lo, w)
        torch.cuda.synchronize()
        lo_h, w_h = lo.cpu().numpy(), w.cpu().numpy()
        for r in range(R):
            w_ref, P_ref = oracle.encode(E, U, int(prompts_h[r // N]), tokens_h.reshape(R, T)[r], eos_id=eos)
            # fp32 logits from an fp32 dot product against fp64: relative 1e-5 per step
            assert abs(w_h[r] - P_ref) <= 1e-5 * T * P_ref, (eos, r)
            assert abs(lo_h[r] - w_ref) <= 1e-6 * T, (eos, r)
    ctx.close(); model.close()


def test_interval_argument_errors():
    import torch
    from paper_2210_15458_amd import binding as B
    ctx = B.Ctx(8, 100, torch.float32)
    logits = torch.zeros((4, 104), dtype=torch.float32, device="cuda")
    tok = torch.zeros(4, dtype=torch.int32, device="cuda")
    lo = torch.zeros(4, dtype=torch.float64, device="cuda")
    w = torch.ones(4, dtype=torch.float64, device="cuda")
    with pytest.raises(B.ArithSamplingError):
        B.as_interval_step(ctx, logits, tok, 0.0, 0, 1.0, lo, w)
    with pytest.raises(B.ArithSamplingError):
        B.as_interval_step(ctx, logits, tok, 1.0, 0, 1.0, lo, w, finished_in=torch.zeros(4, dtype=torch.uint8, device="cuda"))
    B.as_interval_step(ctx, logits, tok, 1.0, 0, 1.0, lo, w)
    torch.cuda.synchronize()
    assert np.allclose(w.cpu().numpy(), 0.01) and np.all(lo.cpu().numpy() == 0.0)
    ctx.close()
