"""Ancestral mode (fresh uniforms per step, Sec. 3.3) and the estimator of Sec. 4.2 on the GPU."""
import math

import numpy as np
import pytest

from paper_2210_15458_amd import synth

pytestmark = pytest.mark.gpu


def _setup(V, d, dtype, Bn, N, same_prompt=False, seed=0):
    import torch
    from paper_2210_15458_amd import binding as B
    from gpu_util import to_dev_logits
    E, U = synth.bigram_weights(V, d, seed=seed, dtype=dtype)
    Ed, Ud = to_dev_logits(E), to_dev_logits(U)
    model = B.Model(Ed, Ud, scale=3.0)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    ctx = B.Ctx(Bn * N, V, tdt)
    p = synth.prompts(Bn, V, seed=seed + 1)
    if same_prompt:
        p[:] = p[0]
    return E, U, Ed, model, ctx, torch.from_numpy(p).cuda(), tdt


@pytest.mark.parametrize("V,d,dtype,Bn,N,T,top_k,top_p", [(16, 8, "f32", 2, 32, 6, 0, 1.0),
                                                            (32128, 512, "bf16", 3, 40, 4, 0, 1.0),
                                                            (32128, 512, "bf16", 2, 24, 3, 40, 0.9)])
def test_ancestral_decode_is_the_loop_of_exported_calls(V, d, dtype, Bn, N, T, top_k, top_p):
    import torch
    from paper_2210_15458_amd import binding as B
    E, U, Ed, model, ctx, prompts, tdt = _setup(V, d, dtype, Bn, N)
    R, eos, temp = Bn * N, 1, 0.9
    uni = torch.from_numpy(np.random.default_rng(5).random((T, R), dtype=np.float32)).cuda()
    tokens = torch.empty((Bn, N, T), dtype=torch.int32, device="cuda")
    B.as_decode_ancestral(ctx, model, prompts, N, T, uni, temp, top_k, top_p, eos, tokens)
    # the same thing step by step
    ld = (V + 7) // 8 * 8
    logits = torch.empty((R, ld), dtype=tdt, device="cuda")
    prev = prompts.repeat_interleave(N).contiguous()
    fin = torch.zeros(R, dtype=torch.uint8, device="cuda")
    want = torch.empty((R, T), dtype=torch.int32, device="cuda")
    for t in range(T):
        B.as_bigram_logits(ctx, model, prev, logits)
        tok = torch.empty(R, dtype=torch.int32, device="cuda")
        cout = torch.empty(R, dtype=torch.float32, device="cuda")
        B.as_step_ex(ctx, logits, uni[t].contiguous(), temp, top_k, top_p, tok, cout, finished_in=fin, eos_id=eos,
                     finished_out=fin)
        want[:, t] = tok
        prev = tok.clone()
    torch.cuda.synchronize()
    assert torch.equal(tokens.reshape(R, T), want)
    ctx.close(); model.close()


def test_ancestral_first_step_is_categorical_sampling():
    """With fresh uniforms the bucket search is inverse-CDF sampling (Sec. 3.1): token counts follow the row's
    probabilities, and every draw is the oracle's token for that uniform."""
    import torch
    import oracle
    from paper_2210_15458_amd import binding as B
    from gpu_util import BAND, from_dev_logits
    V, d, N = 32128, 512, 32768
    E, U, Ed, model, ctx, prompts, tdt = _setup(V, d, "bf16", 1, N)
    uni_h = np.random.default_rng(6).random((1, N), dtype=np.float32)
    tokens = torch.empty((1, N, 1), dtype=torch.int32, device="cuda")
    B.as_decode_ancestral(ctx, model, prompts, N, 1, torch.from_numpy(uni_h).cuda(), 0.7, 0, 1.0, -1, tokens)
    logits = torch.empty((1, V), dtype=tdt, device="cuda")
    B.as_bigram_logits(ctx, model, prompts, logits)
    torch.cuda.synchronize()
    stored = from_dev_logits(logits)
    ref = oracle.step(stored, uni_h[0].astype(np.float64), temp=0.7, row_ids=np.zeros(N, np.int64), V=V, nthreads=8)
    got = tokens.cpu().numpy().reshape(N)
    # a draw next to an interval end may come out as another token, but only one whose own interval (as the
    # oracle has it) lies within BAND of the draw
    c = uni_h[0].astype(np.float64)
    mism = np.nonzero(got != ref["token"])[0]
    f_lo_g, p_g = oracle.interval_in(ref, mism, got[mism])
    assert np.all((p_g > 0) & (c[mism] >= f_lo_g - BAND) & (c[mism] <= f_lo_g + p_g + BAND)), (mism, got[mism])
    print(f"  {mism.size} of {N} draws come out as a token next to the oracle's", flush=True)
    # counts against N*p for the tokens that carry mass
    x = synth.bf16_bits_to_f32(stored[0]).astype(np.float64) / 0.7
    p = np.exp(x - x.max()); p /= p.sum()
    top = np.argsort(p)[::-1][:20]
    counts = np.bincount(got, minlength=V)
    for v in top:
        sd = math.sqrt(N * p[v] * (1 - p[v]))
        assert abs(counts[v] - N * p[v]) <= 5 * sd + 1, (int(v), int(counts[v]), N * p[v])
    ctx.close(); model.close()


def test_estimator_matches_oracle_and_lattice_beats_iid_draws():
    """(1/N) sum s(x_i) on the GPU equals the plain sums; over many shifts its mean agrees with the mean over
    i.i.d. draws and its variance is smaller (the shape of the paper's variance experiment, Sec. 5, on a
    synthetic additive score)."""
    import torch
    import oracle
    from paper_2210_15458_amd import binding as B
    V, d, K, N, T, eos = 1000, 64, 512, 16, 4, 1
    E, U, Ed, model, ctx, prompts, tdt = _setup(V, d, "bf16", K, N, same_prompt=True, seed=3)
    rng = np.random.default_rng(8)
    score_h = rng.standard_normal(V).astype(np.float32)
    score = torch.from_numpy(score_h).cuda()
    u = torch.from_numpy(rng.random(K, dtype=np.float32)).cuda()
    tok_a = torch.empty((K, N, T), dtype=torch.int32, device="cuda")
    B.as_decode(ctx, model, prompts, N, T, u, 1.0, 0, 1.0, eos, tok_a)
    uni = torch.from_numpy(rng.random((T, K * N), dtype=np.float32)).cuda()
    tok_i = torch.empty((K, N, T), dtype=torch.int32, device="cuda")
    B.as_decode_ancestral(ctx, model, prompts, N, T, uni, 1.0, 0, 1.0, eos, tok_i)
    est_a = torch.empty(K, dtype=torch.float64, device="cuda")
    est_i = torch.empty(K, dtype=torch.float64, device="cuda")
    B.as_estimate_mean(ctx, tok_a, score, eos, est_a)
    B.as_estimate_mean(ctx, tok_i, score, eos, est_i)
    torch.cuda.synchronize()
    ea, ei = est_a.cpu().numpy(), est_i.cpu().numpy()
    for est, tok in ((ea, tok_a), (ei, tok_i)):
        want = oracle.estimate_mean(tok.cpu().numpy(), score_h.astype(np.float64), eos_id=eos)
        assert np.allclose(est, want, rtol=1e-13, atol=1e-13)
    se = math.sqrt(ea.var(ddof=1) / K + ei.var(ddof=1) / K)
    print("mean lattice %.5f iid %.5f (se %.5f); variance lattice %.5f iid %.5f ratio %.3f" % (
        ea.mean(), ei.mean(), se, ea.var(ddof=1), ei.var(ddof=1), ea.var(ddof=1) / ei.var(ddof=1)), flush=True)
    assert abs(ea.mean() - ei.mean()) <= 5 * se
    assert ea.var(ddof=1) < 0.9 * ei.var(ddof=1)
    ctx.close(); model.close()


def test_ancestral_and_estimator_argument_errors():
    import torch
    from paper_2210_15458_amd import binding as B
    E, U, Ed, model, ctx, prompts, tdt = _setup(16, 8, "f32", 2, 4)
    tokens = torch.zeros((2, 4, 3), dtype=torch.int32, device="cuda")
    with pytest.raises(ValueError):
        B.as_decode_ancestral(ctx, model, prompts, 4, 3, torch.zeros(5, dtype=torch.float32, device="cuda"), 1.0, 0,
                              1.0, -1, tokens)
    with pytest.raises(B.ArithSamplingError):
        B.as_estimate_mean(ctx, tokens, torch.zeros(16, dtype=torch.float32, device="cuda"), 99,
                           torch.zeros(2, dtype=torch.float64, device="cuda"))
    ctx.close(); model.close()
