"""GPU parity of the lattice, the logits GEMM and the whole decode (as_decode)
against the CPU oracle, through the C ABI.

Decode parity is lock-step: the loop of exported calls (as_lattice,
as_bigram_logits, as_step_ex) is driven from the test, every step's inputs as
the GPU saw them (stored logits, fp32 codes, finished flags) are handed to the
oracle's step, and as_decode must then reproduce that loop bit for bit.  A
float code carries 24 bits while a T-step sequence consumes sum(-log2 p) bits,
so free-running trajectories of two different precisions must part after a few
steps whatever the kernel does; free-running agreement is therefore only
required while the consumed bits leave the code exact enough (Tiny config).
"""
import math

import numpy as np
import pytest

from paper_2210_15458_amd import synth

pytestmark = pytest.mark.gpu


def _upload_model(V, d, dtype, seed=0, scale=3.0):
    import torch
    from paper_2210_15458_amd import binding as B
    from gpu_util import to_dev_logits
    E, U = synth.bigram_weights(V, d, seed=seed, dtype=dtype)
    Ed, Ud = to_dev_logits(E), to_dev_logits(U)
    model = B.Model(Ed, Ud, scale=scale)
    del Ud
    torch.cuda.synchronize()
    return E, U, model


def test_lattice_matches_oracle_bit_for_bit():
    import torch
    import oracle
    from paper_2210_15458_amd import binding as B
    for Bn, N in [(1, 64), (16, 64), (3, 7), (1, 65536), (5, 1)]:
        u = synth.shifts(Bn, seed=Bn + N)
        ctx = B.Ctx(Bn * N, 16, torch.float32)
        out = torch.empty(Bn * N, dtype=torch.float32, device="cuda")
        B.as_lattice(ctx, torch.from_numpy(u).cuda(), N, out)
        torch.cuda.synchronize()
        want = np.concatenate([oracle.lattice(N, float(x)) for x in u]).astype(np.float32)
        want = np.minimum(want, np.float32(1 - 2.0 ** -24))
        assert np.array_equal(out.cpu().numpy(), want), (Bn, N)
        ctx.close()


# (V, d, weights, logits, R, extra leading-dimension padding, logits kernel knob)
_GEMM_CASES = [
    (32128, 512, "bf16", "bf16", 130, 0, 0), (32128, 512, "bf16", "f32", 40, 0, 0), (16, 8, "f32", "f32", 64, 0, 0),
    (1000, 64, "bf16", "bf16", 257, 0, 0), (333, 24, "bf16", "bf16", 50, 0, 0), (4100, 128, "f32", "bf16", 20, 0, 0),
    # persistent kernel: three row tiles (two workers of every XCD idle), two tiles per worker
    (32128, 512, "bf16", "bf16", 700, 0, 0),
    # ... the shortest rank it takes, a ragged last tile in both directions, rows that cannot take 16-byte stores
    (5000, 128, "bf16", "bf16", 300, 0, 0), (1003, 128, "bf16", "bf16", 300, 5, 0), (1003, 128, "bf16", "f32", 260, 1, 0),
    # ... more row tiles than workers per XCD: every worker changes its row tile between tiles
    (2500, 128, "bf16", "bf16", 8200, 0, 0),
    # ... sixteen row tiles: the workers of an XCD stand 8 x 4 over row and column tiles, two row tiles each
    (9000, 128, "bf16", "bf16", 4096, 0, 0),
    # the tile kernel on the headline shape
    (32128, 512, "bf16", "bf16", 130, 0, 1), (32128, 512, "bf16", "f32", 40, 0, 1),
    # the largest vocabulary the library takes: 8192 column tiles
    (1 << 21, 128, "bf16", "bf16", 260, 0, 0)]


@pytest.mark.parametrize("gm", [32, 4, 1])
def test_bigram_logits_worker_placement(gm):
    """How the persistent kernel's workers are spread over the tiles changes which block computes a tile, not
    what the tile holds: every placement gives the default one's logits bit for bit."""
    import torch
    from paper_2210_15458_amd import binding as B
    V, d, R = 2500, 128, 8200 + 256 * 3
    _, _, model = _upload_model(V, d, "bf16")
    prev = torch.from_numpy(np.random.default_rng(2).integers(0, V, R).astype(np.int32)).cuda()
    outs = []
    for knob in (None, gm):
        ctx = B.Ctx(R, V, torch.bfloat16)
        if knob is not None:
            ctx.set_tuning("gemm_gm", knob)
        out = torch.full((R, (V + 7) // 8 * 8), 7.0, dtype=torch.bfloat16, device="cuda")
        B.as_bigram_logits(ctx, model, prev, out)
        torch.cuda.synchronize()
        outs.append(out.view(torch.int16).cpu())
        ctx.close()
    assert torch.equal(outs[0], outs[1])


@pytest.mark.parametrize("V,d,wdtype,ldtype,R,ldpad,knob", _GEMM_CASES)
def test_bigram_logits_against_fp64(V, d, wdtype, ldtype, R, ldpad, knob):
    import torch
    import oracle
    from paper_2210_15458_amd import binding as B
    from gpu_util import from_dev_logits
    E, U, model = _upload_model(V, d, wdtype)
    tdt = torch.bfloat16 if ldtype == "bf16" else torch.float32
    ctx = B.Ctx(R, V, tdt)
    ctx.set_tuning("gemm_shape", knob)
    prev = np.random.default_rng(1).integers(0, V, R).astype(np.int32)
    ld = (V + 7) // 8 * 8 + ldpad
    out = torch.full((R, ld), 7.0, dtype=tdt, device="cuda")
    B.as_bigram_logits(ctx, model, torch.from_numpy(prev).cuda(), out)
    torch.cuda.synchronize()
    got = from_dev_logits(out)
    gotf = synth.bf16_bits_to_f32(got) if ldtype == "bf16" else got
    assert np.all(gotf[:, V:] == 7.0)                       # padding columns untouched
    Ew = (synth.bf16_bits_to_f32(E) if wdtype == "bf16" else E).astype(np.float64)
    Uw = (synth.bf16_bits_to_f32(U) if wdtype == "bf16" else U).astype(np.float64)
    step = max(1, R // 9) if V > 8000 else max(1, R // 90)
    rows = list(range(0, R, step)) + [R - 1]
    for r in rows:
        ref = oracle.bigram_logits(E, U, int(prev[r]), scale=3.0)
        mag = 3.0 / math.sqrt(d) * (np.abs(Ew[prev[r]]) @ np.abs(Uw))     # sum of |terms|
        tol = 4 * d * 2.0 ** -24 * mag + 1e-30                            # fp32 accumulation
        if ldtype == "bf16":
            tol = tol + np.abs(ref) * 2.0 ** -8                           # one rounding to bf16
        err = np.abs(gotf[r, :V].astype(np.float64) - ref)
        assert np.all(err <= tol), (r, float((err / tol).max()))
    ctx.close()
    model.close()


def _lockstep(cfg, B_, N, T, seed=0, check_steps=None, nthreads=8):
    """Drive the exported calls step by step, check each step against the oracle,
    then require as_decode to reproduce the loop exactly."""
    import torch
    import oracle
    from paper_2210_15458_amd import binding as B
    from gpu_util import BAND, compare_step, from_dev_logits
    V, d, temp, top_k, top_p, eos = cfg["V"], cfg["d"], cfg["temp"], cfg["top_k"], cfg["top_p"], cfg["eos_id"]
    tdt = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    E, U, model = _upload_model(V, d, cfg["dtype"], seed=seed)
    R = B_ * N
    ctx = B.Ctx(R, V, tdt)
    prompts = synth.prompts(B_, V, seed=seed + 1)
    u = synth.shifts(B_, seed=seed + 2)
    pd, ud = torch.from_numpy(prompts).cuda(), torch.from_numpy(u).cuda()

    codes = torch.empty(R, dtype=torch.float32, device="cuda")
    B.as_lattice(ctx, ud, N, codes)
    prev = pd.repeat_interleave(N).contiguous()
    fin = torch.zeros(R, dtype=torch.uint8, device="cuda")
    ld = (V + 7) // 8 * 8
    logits = torch.empty((R, ld), dtype=tdt, device="cuda")
    toks = torch.empty((R, T), dtype=torch.int32, device="cuda")
    tok_t = torch.empty(R, dtype=torch.int32, device="cuda")
    prob = torch.empty(R, dtype=torch.float32, device="cuda")
    totals = dict(rows=0, mismatches=0, boundary=0, nucleus=0, nucleus_rows=0, in_band=0)
    for t in range(T):
        B.as_bigram_logits(ctx, model, prev, logits)
        torch.cuda.synchronize()
        codes_in = codes.cpu().numpy().copy()
        fin_in = fin.cpu().numpy().copy()
        B.as_step_ex(ctx, logits, codes, temp, top_k, top_p, tok_t, codes, finished_in=fin, eos_id=eos,
                     finished_out=fin, prob_out=prob)
        torch.cuda.synchronize()
        toks[:, t] = tok_t
        prev = tok_t.clone()
        if check_steps is None or t in check_steps:
            stored = from_dev_logits(logits)
            ref = oracle.step(stored, codes_in.astype(np.float64), temp=temp, top_k=top_k, top_p=top_p,
                              finished=fin_in, eos_id=eos, V=V, nthreads=nthreads, band=BAND)
            gpu = dict(token=tok_t.cpu().numpy(), c_next=codes.cpu().numpy(), p=prob.cpu().numpy(),
                       finished=fin.cpu().numpy())
            # (the model's rows are peaked: a nucleus that closes within the band of top_p is rare)
            st = compare_step(gpu, ref, V, f"{cfg['name']} step {t}", trunc=(top_k > 0 or top_p < 1.0),
                              codes=codes_in, eos_id=eos, max_alt_frac=0.02)
            for k in totals:
                totals[k] += st[k]
            print(f"  step {t}: {st}", flush=True)
    manual_tokens = toks.cpu().numpy().reshape(B_, N, T)
    manual_codes = codes.cpu().numpy().reshape(B_, N)

    out = torch.full((B_, N, T), -3, dtype=torch.int32, device="cuda")
    cf = torch.empty((B_, N), dtype=torch.float32, device="cuda")
    B.as_decode(ctx, model, pd, N, T, ud, temp, top_k, top_p, eos, out, cf)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), manual_tokens), "as_decode differs from the loop of exported calls"
    assert np.array_equal(cf.cpu().numpy(), manual_codes)
    # EOS is sticky
    tk = out.cpu().numpy().reshape(R, T)
    for row in tk:
        hit = np.nonzero(row == eos)[0]
        if len(hit):
            assert np.all(row[hit[0]:] == eos)
    print("  totals", totals, flush=True)
    ctx.close()
    model.close()
    return E, U, prompts, u, manual_tokens, totals


def test_decode_tiny_lockstep_and_free_running():
    import oracle
    cfg = synth.CONFIGS[0]
    E, U, prompts, u, toks, _ = _lockstep(cfg, cfg["B"], cfg["N"], cfg["T"])
    # free-running oracle (fp64 code, logits rounded to fp32 as the device stores them)
    N, T = cfg["N"], cfg["T"]
    codes0 = np.concatenate([oracle.lattice(N, float(x)) for x in u]).astype(np.float32).astype(np.float64)
    ref = oracle.decode(E, U, prompts, N, T, codes0, temp=cfg["temp"], eos_id=cfg["eos_id"],
                        round_mode=1, records=True)
    agree_required, agree_all, total = 0, 0, 0
    for b in range(cfg["B"]):
        for i in range(N):
            bits, safe = 0.0, True
            for t in range(T):
                # the fp32 code has lost `bits` of its 24 bits by step t
                safe = safe and ref["delta"][b, i, t] > 1e-5 + 2.0 ** (bits - 20)
                same = toks[b, i, t] == ref["tokens"][b, i, t]
                total += 1
                agree_all += int(same)
                if safe:
                    assert same, (b, i, t, toks[b, i], ref["tokens"][b, i])
                    agree_required += 1
                else:
                    break
                bits += -math.log2(ref["p"][b, i, t])
    print(f"  tiny free-running: {agree_required} (code, step) pairs required and equal, "
          f"{agree_all}/{total} equal over the compared prefix", flush=True)
    assert agree_required >= N        # at least the first step of every code is decided


def test_decode_headline_shape_lockstep():
    cfg = dict(synth.CONFIGS[1])
    _lockstep(cfg, 4, 16, 6)


def test_decode_truncated_lockstep():
    cfg = dict(synth.CONFIGS[2])
    cfg["top_p"] = 1.0
    _lockstep(cfg, 4, 8, 4)
    cfg = dict(synth.CONFIGS[2])
    cfg["top_k"] = 0
    _lockstep(cfg, 4, 8, 4)


def test_decode_large_vocab_lockstep():
    cfg = dict(synth.CONFIGS[3])
    cfg["V"], cfg["d"] = 256000, 128      # full row width (multi-tile scan); smaller rank keeps the weights quick to draw
    _lockstep(cfg, 2, 8, 3)


@pytest.mark.parametrize("cfg_id,trunc", [(1, "as given"), (2, "as given"), (2, "top-k only"), (2, "nucleus only"),
                                          (3, "as given")])
def test_decode_full_size_sampled_steps(cfg_id, trunc):
    """The benchmark's own shapes (all rows, all steps, the launch configurations bench.py times): the whole
    decode must equal the loop of exported calls, and a sample of steps is checked row by row against the
    oracle (every row of those steps).  The truncated configuration also in the two separate runs the
    benchmark describes (top-k alone, nucleus alone)."""
    cfg = dict(synth.CONFIGS[cfg_id])
    if trunc == "top-k only":
        cfg["top_p"] = 1.0
    elif trunc == "nucleus only":
        cfg["top_k"] = 0
    T = cfg["T"]
    _, _, _, _, _, totals = _lockstep(cfg, cfg["B"], cfg["N"], T, check_steps={0, 1, T // 2, T - 1}, nthreads=16)
    assert totals["rows"] >= 3 * cfg["B"] * cfg["N"] // 2


def _free_running_oracle(ctx, model, prompts_h, N, T, codes0, V, tdt, temp, top_k, top_p, eos, nthreads=16):
    """The oracle decoding on its own, with an fp64 code state, from the same start codes.  Its logits are the
    rows the DEVICE stores for the conditioning tokens the oracle reaches (one row per distinct token, through
    as_bigram_logits), so what parts the two trajectories is the code state and the per-element arithmetic, not
    a differently rounded logit.  Returns tokens [R, T], p [R, T], delta [R, T]."""
    import torch
    import oracle
    from paper_2210_15458_amd import binding as B
    from gpu_util import from_dev_logits
    R = codes0.shape[0]
    codes = codes0.astype(np.float64)
    prev = np.repeat(prompts_h.astype(np.int64), N)
    fin = np.zeros(R, dtype=np.uint8)
    toks = np.empty((R, T), dtype=np.int32)
    ps = np.empty((R, T))
    deltas = np.empty((R, T))
    margins = np.empty((R, T))
    ld = (V + 7) // 8 * 8
    for t in range(T):
        uniq, inv = np.unique(prev, return_inverse=True)
        logits = torch.empty((len(uniq), ld), dtype=tdt, device="cuda")
        B.as_bigram_logits(ctx, model, torch.from_numpy(uniq.astype(np.int32)).cuda(), logits)
        torch.cuda.synchronize()
        stored = from_dev_logits(logits)
        del logits
        ref = oracle.step(stored, codes, temp=temp, top_k=top_k, top_p=top_p, finished=fin, eos_id=eos,
                          row_ids=inv.astype(np.int64), V=V, nthreads=nthreads)
        toks[:, t], ps[:, t], deltas[:, t], margins[:, t] = ref["token"], ref["p"], ref["delta"], ref["nuc_margin"]
        codes, fin, prev = ref["c_next"], ref["finished"], ref["token"].astype(np.int64)
    return toks, ps, deltas, margins


def _first_divergence_histogram(gpu_tokens, ref_tokens):
    """How many codes first part from the reference at step t (index T: never within T steps)."""
    T = gpu_tokens.shape[1]
    diff = gpu_tokens != ref_tokens
    first = np.where(diff.any(axis=1), diff.argmax(axis=1), T)
    return np.bincount(first, minlength=T + 1)


def _distinct_prefixes(tok):
    """Number of distinct prefixes of every length 1..T among the rows of tok."""
    out = []
    for t in range(1, tok.shape[1] + 1):
        out.append(len(np.unique(np.ascontiguousarray(tok[:, :t]), axis=0)))
    return out


def test_wide_lattice_full_shape():
    """configs[4] at its own shape: one prompt, N = 65536 codes, T = 16 steps (Sec. 4.2 lattice, Sec. 4.3
    duplicate bounds).
      * every step, every row, lock-step against the oracle on the GPU's own inputs (the oracle is handed one
        logits row per distinct conditioning token, after the device's rows for equal tokens have been shown
        to be the same bits);
      * as_decode equals that loop of exported calls;
      * step 1, where all codes share one row: per-token counts are floor or ceil of N*p_v up to the fp32
        rounding of the codes and the counted boundary rows, and equal the oracle's counts up to those rows;
      * sequences are lexicographically non-decreasing in the lattice index (codes ascending, Sec. 4.3), so
        the number of distinct prefixes is one more than the number of adjacent changes;
      * the number of distinct prefixes of every length 1..T equals that of the oracle's tokens up to the rows
        that differ (each boundary row moves a count by at most one);
      * reported: the same counts and the first-divergence histogram against the oracle decoding on its own
        with an fp64 code."""
    import torch
    import oracle
    from paper_2210_15458_amd import binding as B
    from gpu_util import BAND, compare_step, from_dev_logits
    cfg = synth.CONFIGS[4]
    V, d, N, T, temp, eos = cfg["V"], cfg["d"], cfg["N"], cfg["T"], cfg["temp"], cfg["eos_id"]
    E, U, model = _upload_model(V, d, cfg["dtype"])
    tdt = torch.bfloat16
    ctx = B.Ctx(N, V, tdt)
    prompts_h = synth.prompts(1, V, seed=1)
    u_h = synth.shifts(1, seed=2)
    pd, ud = torch.from_numpy(prompts_h).cuda(), torch.from_numpy(u_h).cuda()

    codes = torch.empty(N, dtype=torch.float32, device="cuda")
    B.as_lattice(ctx, ud, N, codes)
    torch.cuda.synchronize()
    codes0 = codes.cpu().numpy().copy()
    assert np.all(np.diff(codes0) > 0)
    prev = pd.repeat_interleave(N).contiguous()
    fin = torch.zeros(N, dtype=torch.uint8, device="cuda")
    ld = (V + 7) // 8 * 8
    logits = torch.empty((N, ld), dtype=tdt, device="cuda")
    tok_t = torch.empty(N, dtype=torch.int32, device="cuda")
    prob = torch.empty(N, dtype=torch.float32, device="cuda")
    G = np.empty((N, T), dtype=np.int32)            # the GPU's tokens
    O = np.empty((N, T), dtype=np.int32)            # the oracle's, step by step on the GPU's inputs
    differs = np.zeros(N, dtype=bool)
    first_ref = None
    for t in range(T):
        B.as_bigram_logits(ctx, model, prev, logits)
        prev_h = prev.cpu().numpy()
        uniq, first_of, inv = np.unique(prev_h, return_index=True, return_inverse=True)
        # rows of equal conditioning tokens hold the same bits: hand the oracle one row per distinct token
        rows_u = logits[torch.from_numpy(first_of.astype(np.int64)).cuda()]
        same = True
        for lo in range(0, N, 8192):                 # (in slices: the gathered copy of all rows would be 4 GB)
            idx = torch.from_numpy(inv[lo:lo + 8192].astype(np.int64)).cuda()
            same = same and bool(torch.equal(logits[lo:lo + 8192].view(torch.int16), rows_u[idx].view(torch.int16)))
        assert same, f"step {t}: rows with the same conditioning token differ"
        stored = from_dev_logits(rows_u)
        del rows_u
        codes_in = codes.cpu().numpy().copy()
        fin_in = fin.cpu().numpy().copy()
        B.as_step_ex(ctx, logits, codes, temp, 0, 1.0, tok_t, codes, finished_in=fin, eos_id=eos, finished_out=fin,
                     prob_out=prob)
        torch.cuda.synchronize()
        ref = oracle.step(stored, codes_in.astype(np.float64), temp=temp, finished=fin_in, eos_id=eos, V=V,
                          row_ids=inv.astype(np.int64), nthreads=16)
        gpu = dict(token=tok_t.cpu().numpy(), c_next=codes.cpu().numpy(), p=prob.cpu().numpy(),
                   finished=fin.cpu().numpy())
        st = compare_step(gpu, ref, V, f"wide lattice step {t}", codes=codes_in, eos_id=eos)
        print(f"  step {t}: distinct conditioning tokens {len(uniq)}; {st}", flush=True)
        G[:, t], O[:, t] = gpu["token"], ref["token"]
        differs |= gpu["token"] != ref["token"]
        if t == 0:
            first_ref = ref
        prev = tok_t.clone()

    out = torch.full((1, N, T), -3, dtype=torch.int32, device="cuda")
    B.as_decode(ctx, model, pd, N, T, ud, temp, 0, 1.0, eos, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy()[0], G), "as_decode differs from the loop of exported calls"

    # ---- step 1: counts
    first = G[:, 0]
    mism = int((first != first_ref["token"]).sum())
    cnt_g = np.bincount(first, minlength=V)
    cnt_o = np.bincount(first_ref["token"], minlength=V)
    assert np.abs(cnt_g - cnt_o).sum() <= 2 * mism
    p = np.zeros(V)
    p[first_ref["token"]] = first_ref["p"]
    eps = 2 * N * 2.0 ** -24 + 1e-9                  # fp32 rounding of the codes moves a count by at most this
    seen = cnt_g > 0
    assert np.all(cnt_g[seen] >= np.floor(N * p[seen] - eps) - mism)
    assert np.all(cnt_g[seen] <= np.ceil(N * p[seen] + eps) + mism)
    print(f"  step 1: {mism} boundary rows of {N}; {int(seen.sum())} distinct tokens", flush=True)

    # ---- monotone sequences, distinct prefixes
    for t in range(1, T + 1):
        a, b = G[:-1, :t], G[1:, :t]
        neq = a != b
        has = neq.any(axis=1)
        k = neq.argmax(axis=1)
        rows = np.nonzero(has)[0]
        assert np.all(a[rows, k[rows]] < b[rows, k[rows]]), f"prefixes of length {t} are not non-decreasing"
    dg, do = _distinct_prefixes(G), _distinct_prefixes(O)
    changes = [1 + int(np.any(G[1:, :t] != G[:-1, :t], axis=1).sum()) for t in range(1, T + 1)]
    nd = int(differs.sum())
    print(f"  distinct prefixes, GPU:    {dg}\n  distinct prefixes, oracle: {do}\n  rows with a boundary "
          f"mismatch at some step: {nd}", flush=True)
    assert dg == changes
    for t in range(T):
        moved = int((G[:, :t + 1] != O[:, :t + 1]).any(axis=1).sum())
        assert abs(dg[t] - do[t]) <= moved, (t + 1, dg[t], do[t], moved)

    # ---- reported: the oracle on its own, fp64 code
    F, Fp, Fd, _ = _free_running_oracle(ctx, model, prompts_h, N, T, codes0, V, tdt, temp, 0, 1.0, eos)
    hist = _first_divergence_histogram(G, F)
    df = _distinct_prefixes(F)
    print(f"  free-running fp64 oracle: first divergence by step {hist.tolist()} (last entry: never)\n"
          f"  distinct prefixes, free-running oracle: {df}", flush=True)
    # the first step has the same inputs on both sides
    assert hist[0] <= mism
    assert abs(dg[0] - df[0]) <= mism
    ctx.close()
    model.close()


@pytest.mark.parametrize("cfg_id,top_k,top_p", [(1, 0, 1.0), (2, 40, 1.0), (2, 0, 0.9)])
def test_free_running_divergence_is_reported(cfg_id, top_k, top_p):
    """How long the GPU's decode (fp32 code state, fp32 weights) stays on the trajectory of the oracle decoding
    on its own with an fp64 code from the same start codes and the same stored logits: the histogram of the
    first step at which they part, and how much of it the bits consumed so far explain (a code that has used
    b bits of its 24 sits within 2^(b-24) of where the fp64 code sits, so it parts once an interval end comes
    that close).  Required: every code whose path keeps farther than that (with a factor of 8) from every
    interval end stays on the oracle's trajectory."""
    import torch
    import oracle
    from paper_2210_15458_amd import binding as B
    cfg = dict(synth.CONFIGS[cfg_id])
    V, d, Bn, N, temp, eos = cfg["V"], cfg["d"], cfg["B"], cfg["N"], cfg["temp"], cfg["eos_id"]
    T = min(cfg["T"], 24)
    E, U, model = _upload_model(V, d, cfg["dtype"])
    R = Bn * N
    ctx = B.Ctx(R, V, torch.bfloat16)
    prompts_h = synth.prompts(Bn, V, seed=1)
    u_h = synth.shifts(Bn, seed=2)
    codes = torch.empty(R, dtype=torch.float32, device="cuda")
    B.as_lattice(ctx, torch.from_numpy(u_h).cuda(), N, codes)
    out = torch.empty((Bn, N, T), dtype=torch.int32, device="cuda")
    B.as_decode(ctx, model, torch.from_numpy(prompts_h).cuda(), N, T, torch.from_numpy(u_h).cuda(), temp, top_k, top_p,
                eos, out)
    torch.cuda.synchronize()
    G = out.cpu().numpy().reshape(R, T)
    F, Fp, Fd, Fm = _free_running_oracle(ctx, model, prompts_h, N, T, codes.cpu().numpy(), V, torch.bfloat16, temp,
                                         top_k, top_p, eos)
    hist = _first_divergence_histogram(G, F)
    bits = np.concatenate([np.zeros((R, 1)), np.cumsum(-np.log2(Fp), axis=1)[:, :-1]], axis=1)   # used before step t
    # (a nucleus that closes within 1e-5 of top_p may legitimately close elsewhere: such a step is not required)
    safe = np.logical_and.accumulate((Fd > 1e-5 + 64.0 * 2.0 ** (bits - 24)) & (Fm > 1e-5), axis=1)
    agree = G == F
    assert np.all(agree[safe]), "a code far from every interval end left the oracle's trajectory"
    med_bits = float(np.median(-np.log2(Fp[:, 0])))
    print(f"  {cfg['name']} k={top_k} p={top_p}: first divergence from the free-running fp64 oracle by step "
          f"{hist.tolist()} (last: none in {T} steps); median bits per step {med_bits:.2f}; "
          f"{int(safe.sum())} (code, step) pairs required and equal", flush=True)
    ctx.close()
    model.close()


def test_decode_hostile_data_stays_in_bounds():
    """Errors in device data are not detected, but nothing leaves its range: weights with NaN and infinities,
    shifts and uniforms outside [0, 1), prompts outside the vocabulary (clamped) -- through the plain, the fused
    and the ancestral decode, bf16 and fp32 logits, with and without truncation."""
    import torch
    from paper_2210_15458_amd import binding as B
    from gpu_util import to_dev_logits
    V, d, Bn, N, T = 5003, 128, 6, 40, 5
    E, U = synth.bigram_weights(V, d, seed=3, dtype="bf16")
    Ef, Uf = synth.bf16_bits_to_f32(E), synth.bf16_bits_to_f32(U)
    rng = np.random.default_rng(5)
    Ef[rng.integers(0, V, 40), rng.integers(0, d, 40)] = np.nan
    Ef[rng.integers(0, V, 40), rng.integers(0, d, 40)] = np.inf
    Uf[rng.integers(0, d, 40), rng.integers(0, V, 40)] = -np.inf
    Uf[:, 77] = np.nan
    Ed, Ud = to_dev_logits(synth.f32_to_bf16_bits(Ef)), to_dev_logits(synth.f32_to_bf16_bits(Uf))
    model = B.Model(Ed, Ud, scale=3.0)
    prompts = torch.tensor([0, V - 1, V, -1, 2 ** 31 - 1, 17], dtype=torch.int32, device="cuda")
    u = torch.tensor([0.5, 1.0, 2.5, -0.5, float("nan"), float("inf")], dtype=torch.float32, device="cuda")
    unif = torch.from_numpy(rng.random((T, Bn * N)).astype(np.float32)).cuda()
    unif[0, ::7] = float("nan")
    unif[1, ::5] = 3.0
    unif[2, ::3] = -1.0
    for ldtype in (torch.bfloat16, torch.float32):
        ctx = B.Ctx(Bn * N, V, ldtype)
        for top_k, top_p in [(0, 1.0), (40, 1.0), (0, 0.9), (7, 0.6)]:
            print("case hostile decode", ldtype, top_k, top_p, flush=True)
            tok = torch.full((Bn, N, T), -7, dtype=torch.int32, device="cuda")
            cf = torch.full((Bn * N,), -1.0, dtype=torch.float32, device="cuda")
            B.as_decode(ctx, model, prompts, N, T, u, 1.0, top_k, top_p, 1, tok, cf)
            torch.cuda.synchronize()
            t, c = tok.cpu().numpy(), cf.cpu().numpy()
            assert ((t >= 0) & (t < V)).all()
            assert np.isfinite(c).all() and (c >= 0).all() and (c <= np.float32(1.0) - np.float32(2.0 ** -24)).all()
            tok.fill_(-7)
            B.as_decode_ancestral(ctx, model, prompts, N, T, unif, 1.0, top_k, top_p, 1, tok)
            torch.cuda.synchronize()
            t = tok.cpu().numpy()
            assert ((t >= 0) & (t < V)).all()
        if ldtype == torch.bfloat16:
            print("case hostile fused decode", flush=True)
            tok = torch.full((Bn, N, T), -7, dtype=torch.int32, device="cuda")
            cf = torch.full((Bn * N,), -1.0, dtype=torch.float32, device="cuda")
            B.as_decode_fused(ctx, model, prompts, N, T, u, 0.8, 1, tok, cf)
            torch.cuda.synchronize()
            t, c = tok.cpu().numpy(), cf.cpu().numpy()
            assert ((t >= 0) & (t < V)).all()
            assert np.isfinite(c).all() and (c >= 0).all() and (c <= np.float32(1.0) - np.float32(2.0 ** -24)).all()
        ctx.close()


@pytest.mark.parametrize("top_k,top_p", [(0, 1.0), (40, 0.9)])
def test_decode_on_side_streams_matches_default_stream(top_k, top_p):
    """A context works on the stream it was made with and on nothing else: two contexts on two streams (default
    priority), half of the prompts each and in flight together, give token for token what one context on the
    default stream gives for all of them (rows are independent and every kernel is deterministic)."""
    import torch
    from paper_2210_15458_amd import binding as B
    V, d, Bn, N, T = 32128, 512, 4, 64, 6
    _, _, model = _upload_model(V, d, "bf16")
    prompts = torch.from_numpy(synth.prompts(Bn, V, seed=1)).cuda()
    u = torch.from_numpy(synth.shifts(Bn, seed=2)).cuda()
    ctx = B.Ctx(Bn * N, V, torch.bfloat16)
    ref = torch.empty((Bn, N, T), dtype=torch.int32, device="cuda")
    ref_c = torch.empty(Bn * N, dtype=torch.float32, device="cuda")
    B.as_decode(ctx, model, prompts, N, T, u, 0.9, top_k, top_p, 1, ref, ref_c)
    torch.cuda.synchronize()
    ctx.close()
    h = Bn // 2
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    ctxs = [B.Ctx(h * N, V, torch.bfloat16, stream=st) for st in streams]
    ps = [prompts[:h].contiguous(), prompts[h:].contiguous()]
    us = [u[:h].contiguous(), u[h:].contiguous()]
    toks = [torch.full((h, N, T), -7, dtype=torch.int32, device="cuda") for _ in range(2)]
    cfs = [torch.full((h * N,), -1.0, dtype=torch.float32, device="cuda") for _ in range(2)]
    torch.cuda.synchronize()
    for rep in range(3):                                 # several rounds, both streams busy at once
        for i in range(2):
            B.as_decode(ctxs[i], model, ps[i], N, T, us[i], 0.9, top_k, top_p, 1, toks[i], cfs[i])
    for st in streams:
        st.synchronize()
    got = torch.cat(toks, dim=0).cpu().numpy()
    got_c = torch.cat(cfs, dim=0).cpu().numpy()
    for c in ctxs:
        c.close()
    assert (got == ref.cpu().numpy()).all()
    assert (got_c == ref_c.cpu().numpy()).all()


@pytest.mark.parametrize("top_k,top_p", [(0, 1.0), (40, 0.9)])
def test_decode_captured_in_a_graph_replays_like_eager(top_k, top_p):
    """Once its workspace exists (first call), as_decode allocates nothing, waits for nothing and reads nothing
    back, so a stream capture takes it whole.  Every replay, with fresh shifts written into the same buffer and
    eager work of the same context in between, gives what the eager call gives for those shifts."""
    import torch
    from paper_2210_15458_amd import binding as B
    V, d, Bn, N, T = 32128, 512, 4, 32, 5
    _, _, model = _upload_model(V, d, "bf16")
    prompts = torch.from_numpy(synth.prompts(Bn, V, seed=1)).cuda()
    u = torch.from_numpy(synth.shifts(Bn, seed=2)).cuda()
    side = torch.cuda.Stream()
    ctx = B.Ctx(Bn * N, V, torch.bfloat16, stream=side)
    tok = torch.full((Bn, N, T), -7, dtype=torch.int32, device="cuda")
    cf = torch.full((Bn * N,), -1.0, dtype=torch.float32, device="cuda")
    etok, ecf = torch.empty_like(tok), torch.empty_like(cf)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        B.as_decode(ctx, model, prompts, N, T, u, 0.9, top_k, top_p, 1, tok, cf)      # makes the workspace
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        B.as_decode(ctx, model, prompts, N, T, u, 0.9, top_k, top_p, 1, tok, cf)
    side.synchronize()
    for rep in range(4):
        new_u = torch.from_numpy(synth.shifts(Bn, seed=10 + rep)).cuda()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            u.copy_(new_u)
            tok.fill_(-7)
            graph.replay()
        side.synchronize()
        got, got_c = tok.cpu().numpy().copy(), cf.cpu().numpy().copy()
        with torch.cuda.stream(side):
            B.as_decode(ctx, model, prompts, N, T, new_u, 0.9, top_k, top_p, 1, etok, ecf)     # eager, same context
        side.synchronize()
        assert (got == etok.cpu().numpy()).all(), rep
        assert (got_c == ecf.cpu().numpy()).all(), rep
    ctx.close()
