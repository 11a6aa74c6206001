"""Fused decode (logits kept on chip, Sec. 4.1 Algorithm 1 unchanged) against the CPU oracle."""
import math

import numpy as np
import pytest

from paper_2210_15458_amd import synth

pytestmark = pytest.mark.gpu

BAND = 1e-5            # a code this close to a bucket boundary may fall on either side
CODE_TOL = 4e-6        # |c' error| * p, code units of the step: fp32-accumulated logits against fp64 ones


def _setup(V, d, Bn, N, seed=0):
    import torch
    from paper_2210_15458_amd import binding as B
    from gpu_util import to_dev_logits
    E, U = synth.bigram_weights(V, d, seed=seed, dtype="bf16")
    Ed, Ud = to_dev_logits(E), to_dev_logits(U)
    model = B.Model(Ed, Ud, scale=3.0)
    ctx = B.Ctx(Bn * N, V, torch.bfloat16)
    prompts_h = synth.prompts(Bn, V, seed=seed + 1)
    u_h = synth.shifts(Bn, seed=seed + 2)
    return E, U, Ed, model, ctx, prompts_h, u_h


def _oracle_step_rows(E, U, prev, codes, temp, fin, eos):
    """oracle.step on fp64 logits computed by the oracle from the stored weights (one logits row per distinct
    conditioning token, shared through row_ids)."""
    import oracle
    uniq, inv = np.unique(prev, return_inverse=True)
    rows = np.stack([oracle.bigram_logits(E, U, int(k), scale=3.0) for k in uniq])
    return oracle.step(rows, codes, temp=temp, row_ids=inv.astype(np.int64), finished=fin.astype(np.uint8),
                       eos_id=eos, nthreads=8)


@pytest.mark.parametrize("V,d,Bn,N,T,temp,eos", [(32128, 512, 3, 16, 4, 0.7, 1), (32128, 512, 2, 24, 3, 1.0, -1),
                                                  (5000, 128, 2, 150, 3, 1.0, 1), (1003, 256, 1, 300, 2, 1.3, 1),
                                                  # rows of more than one tile of 1024 groups: one group into
                                                  # the second tile, two tiles, eight tiles
                                                  (32800, 128, 2, 40, 2, 0.9, -1), (50257, 256, 2, 32, 3, 1.0, 1),
                                                  (256000, 256, 1, 24, 2, 1.0, 1)])
def test_fused_decode_lockstep_against_oracle(V, d, Bn, N, T, temp, eos):
    """Follow the GPU's trajectory: at every step the oracle gets the GPU's conditioning tokens and codes and
    must emit the same token unless the code sits within BAND of a bucket boundary."""
    import torch
    from paper_2210_15458_amd import binding as B
    E, U, Ed, model, ctx, prompts_h, u_h = _setup(V, d, Bn, N)
    R = Bn * N
    prompts = torch.from_numpy(prompts_h).cuda()
    u = torch.from_numpy(u_h).cuda()
    codes0 = torch.empty(R, dtype=torch.float32, device="cuda")
    B.as_lattice(ctx, u, N, codes0)
    toks, codes = [], [codes0.cpu().numpy()]
    for t_len in range(1, T + 1):            # the fused decode has no per-step hook: decode prefixes
        tok = torch.empty((Bn, N, t_len), dtype=torch.int32, device="cuda")
        cf = torch.empty(R, dtype=torch.float32, device="cuda")
        B.as_decode_fused(ctx, model, prompts, N, t_len, u, temp, eos, tok, cf)
        torch.cuda.synchronize()
        toks.append(tok.cpu().numpy().reshape(R, t_len))
        codes.append(cf.cpu().numpy())
    for t_len in range(2, T + 1):            # prefixes agree with each other (deterministic)
        assert np.array_equal(toks[t_len - 1][:, :t_len - 1], toks[t_len - 2])
    full = toks[-1]
    from gpu_util import compare_step
    mism = band = 0
    fin = np.zeros(R, dtype=bool)
    for t in range(T):
        prev = np.repeat(prompts_h, N) if t == 0 else full[:, t - 1]
        ref = _oracle_step_rows(E, U, prev, codes[t].astype(np.float64), temp, fin, eos)
        # every row: the oracle's token and code, or inside the band the neighbouring token at the matching end
        # of its interval; the tolerance of the code is CODE_TOL (fp32-accumulated logits against fp64 ones)
        st = compare_step(dict(token=full[:, t], c_next=codes[t + 1]), ref, V, f"fused step {t}", codes=codes[t],
                          eos_id=eos, cdf_eps=CODE_TOL)
        mism += st["mismatches"]
        band += st["in_band"]
        if eos >= 0:
            fin |= full[:, t] == eos
    print(f"fused lock-step V={V} R={R} T={T}: mismatches (all in the band, neighbouring token) {mism}, rows in the band {band}", flush=True)
    ctx.close(); model.close()


def test_fused_decode_agrees_with_unfused_on_fp32_logits():
    """Same model, logits kept in fp32: the two paths differ only by accumulation order, so tokens agree except
    at codes next to a bucket boundary (counted)."""
    import torch
    from paper_2210_15458_amd import binding as B
    V, d, Bn, N, T = 32128, 512, 4, 64, 2
    E, U, Ed, model, ctx, prompts_h, u_h = _setup(V, d, Bn, N)
    R = Bn * N
    prompts = torch.from_numpy(prompts_h).cuda()
    u = torch.from_numpy(u_h).cuda()
    tok_f = torch.empty((Bn, N, T), dtype=torch.int32, device="cuda")
    B.as_decode_fused(ctx, model, prompts, N, T, u, 0.8, 1, tok_f)
    ctx32 = B.Ctx(R, V, torch.float32)
    tok_u = torch.empty((Bn, N, T), dtype=torch.int32, device="cuda")
    B.as_decode(ctx32, model, prompts, N, T, u, 0.8, 0, 1.0, 1, tok_u)
    torch.cuda.synchronize()
    a, b = tok_f.cpu().numpy().reshape(R, T), tok_u.cpu().numpy().reshape(R, T)
    first = a[:, 0] != b[:, 0]
    print("rows whose first token differs between fused and unfused fp32:", int(first.sum()), "of", R, flush=True)
    assert first.sum() <= max(2, R // 50)
    ctx.close(); ctx32.close(); model.close()


def test_fused_decode_unsupported_shapes_say_so():
    import torch
    from paper_2210_15458_amd import binding as B
    from gpu_util import to_dev_logits
    E, U = synth.bigram_weights(64, 8, seed=0, dtype="f32")
    model = B.Model(to_dev_logits(E), to_dev_logits(U), scale=3.0)
    ctx = B.Ctx(4, 64, torch.float32)
    tok = torch.empty((1, 4, 2), dtype=torch.int32, device="cuda")
    with pytest.raises(B.ArithSamplingError) as ei:
        B.as_decode_fused(ctx, model, torch.zeros(1, dtype=torch.int32, device="cuda"), 4, 2,
                          torch.zeros(1, dtype=torch.float32, device="cuda"), 1.0, -1, tok)
    assert ei.value.code == 2
    ctx.close(); model.close()
