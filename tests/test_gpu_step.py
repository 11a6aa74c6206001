"""GPU parity of the fused sampling step (as_step / as_step_ex) against the CPU
oracle, element by element on the same seeded inputs, through the C ABI."""
import numpy as np
import pytest

from paper_2210_15458_amd import synth

pytestmark = pytest.mark.gpu


def _check(V, R, dtype, temp=1.0, top_k=0, top_p=1.0, ld=None, sigma=3.0, seed=3, label=None, tuning=None,
           max_alt_frac=None, **kw):
    from gpu_util import compare_step, oracle_step, run_gpu_step
    stored = synth.gaussian_logits(R, V, sigma=sigma, seed=seed, dtype=dtype, ld=ld)
    codes = synth.uniform_codes(R, seed=seed + 1)
    label = label or f"V={V} R={R} {dtype} temp={temp} k={top_k} p={top_p} ld={ld}"
    print("case", label, flush=True)
    gpu = run_gpu_step(stored, codes, V, temp=temp, top_k=top_k, top_p=top_p, tuning=tuning, **kw)
    ref = oracle_step(stored, codes, V, temp=temp, top_k=top_k, top_p=top_p, **kw)
    stats = compare_step(gpu, ref, V, label, trunc=(top_k > 0 or top_p < 1.0), codes=codes,
                         eos_id=kw.get("eos_id", -1), max_alt_frac=max_alt_frac)
    print("   ", stats, flush=True)
    return gpu, ref, stats


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("temp", [0.7, 1.0])
def test_step_headline_vocab(dtype, temp):
    _check(32128, 96, dtype, temp=temp)


@pytest.mark.parametrize("V,ld", [(1, None), (5, None), (16, None), (511, None), (1000, None), (1001, None),
                                  (1001, 1008), (4097, 4104), (32771, 32776), (32768, None), (40000, 40003)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_step_ragged_vocab_and_padding(V, ld, dtype):
    # odd V without padding gives rows that do not start on 16 bytes: element path
    _check(V, 33, dtype, ld=ld, seed=V)


@pytest.mark.parametrize("V,dtype", [(256000, "bf16"), (70001, "f32"), (131072, "bf16"), (300000, "f32")])
def test_step_multi_tile_rows(V, dtype):
    _check(V, 12, dtype, seed=11)


@pytest.mark.parametrize("sigma,temp", [(0.01, 1.0), (10.0, 0.3), (3.0, 50.0), (30.0, 1.0)])
def test_step_flat_and_peaked_rows(sigma, temp):
    _check(32128, 48, "bf16", temp=temp, sigma=sigma, seed=5)
    _check(5000, 48, "f32", temp=temp, sigma=sigma, seed=6)


def test_step_special_rows_and_codes():
    from gpu_util import compare_step, oracle_step, run_gpu_step
    V, R = 3000, 8
    x = synth.bf16_bits_to_f32(synth.gaussian_logits(R, V, seed=9, dtype="bf16")).copy()
    x[0, :] = -np.inf; x[0, 1234] = 0.5              # one-hot
    x[1, :] = 0.0                                      # uniform
    x[2, ::2] = -np.inf                                # every other token impossible
    x[3, : V - 1] = -np.inf                            # only the last token
    x[4, 1:] = -np.inf                                 # only the first token
    x[5, :] = -80.0; x[5, 7] = 80.0                    # huge dynamic range
    codes = np.array([0.37, 0.5, 0.999, 0.0, 1 - 2.0 ** -24, 0.25, 0.0, 1 - 2.0 ** -24], np.float32)
    for dtype in ("bf16", "f32"):
        stored = synth.f32_to_bf16_bits(x) if dtype == "bf16" else x
        gpu = run_gpu_step(stored, codes, V)
        ref = oracle_step(stored, codes, V)
        print(dtype, compare_step(gpu, ref, V, f"special {dtype}", codes=codes), flush=True)
        assert gpu["token"][0] == 1234 and gpu["token"][3] == V - 1 and gpu["token"][4] == 0
        assert gpu["token"][6] == ref["token"][6] and gpu["token"][7] == ref["token"][7]


def test_step_finished_rows_eos_and_row_ids():
    from gpu_util import compare_step, oracle_step, run_gpu_step
    V, LR, R = 2048, 5, 40
    rng = np.random.default_rng(12)
    stored = synth.gaussian_logits(LR, V, seed=13, dtype="bf16")
    wide = synth.bf16_bits_to_f32(stored).copy()
    wide[:, 1] += 14.0                                  # make EOS (id 1) likely
    stored = synth.f32_to_bf16_bits(wide)
    codes = synth.uniform_codes(R, seed=14)
    rid = rng.integers(0, LR, R).astype(np.int32)
    fin = (rng.random(R) < 0.3).astype(np.uint8)
    gpu = run_gpu_step(stored, codes, V, finished=fin, eos_id=1, row_ids=rid)
    ref = oracle_step(stored, codes, V, finished=fin, eos_id=1, row_ids=rid.astype(np.int64))
    print(compare_step(gpu, ref, V, "finished/row_ids", codes=codes, eos_id=1), flush=True)
    assert np.all(gpu["token"][fin == 1] == 1)
    assert np.array_equal(gpu["c_next"][fin == 1], codes[fin == 1])       # code untouched
    assert np.all(gpu["finished"][fin == 1] == 1)
    assert np.array_equal(gpu["finished"], ref["finished"])
    assert (gpu["finished"][fin == 0] == 1).any()                          # some row emitted EOS now


@pytest.mark.parametrize("top_k,top_p", [(0, 1.0), (40, 1.0), (0, 0.9)])
def test_step_row_ids_out_of_range_read_the_nearest_row(top_k, top_p):
    """A row index outside the logits is a caller's error that no call can report; it is brought into range
    rather than followed: the result is the oracle's for the clamped indices."""
    from gpu_util import compare_step, oracle_step, run_gpu_step
    V, LR = 32128, 6
    stored = synth.gaussian_logits(LR, V, seed=31, dtype="bf16")
    rid = np.array([0, LR - 1, LR, -1, 2 ** 31 - 1, -2 ** 31, 3, 10 ** 6], dtype=np.int32)
    codes = synth.uniform_codes(rid.size, seed=32)
    gpu = run_gpu_step(stored, codes, V, top_k=top_k, top_p=top_p, row_ids=rid)
    ref = oracle_step(stored, codes, V, top_k=top_k, top_p=top_p, row_ids=np.clip(rid.astype(np.int64), 0, LR - 1))
    print(compare_step(gpu, ref, V, "row_ids out of range", trunc=(top_k > 0 or top_p < 1.0), codes=codes), flush=True)


@pytest.mark.parametrize("V,dtype,temp,top_k,top_p", [(32128, "bf16", 1.0, 40, 1.0), (32128, "bf16", 1.0, 0, 0.9),
                                                      (32128, "bf16", 0.7, 200, 0.95), (50257, "f32", 1.0, 40, 1.0),
                                                      (50257, "f32", 1.0, 0, 0.9), (50257, "bf16", 1.3, 1000, 0.8)])
def test_lattice_on_a_truncated_row_counts_and_monotonicity(V, dtype, temp, top_k, top_p):
    """N evenly spaced codes on one row (shared through row_ids), with truncation: every code decodes as the
    oracle says, tokens are non-decreasing in the code, only kept tokens come out, and each token gets floor or
    ceil of N times its probability under the truncated distribution (Sec. 4.3; up to the fp32 rounding of the
    codes and the counted boundary cases)."""
    import oracle
    from gpu_util import compare_step, oracle_step, run_gpu_step
    N = 4096
    stored = synth.gaussian_logits(3, V, seed=V % 1000 + top_k, dtype=dtype)
    rid = np.full(N, 1, dtype=np.int32)
    codes = np.minimum(oracle.lattice(N, 0.37).astype(np.float32), np.float32(1 - 2.0 ** -24))
    gpu = run_gpu_step(stored, codes, V, temp=temp, top_k=top_k, top_p=top_p, row_ids=rid)
    ref = oracle_step(stored, codes, V, temp=temp, top_k=top_k, top_p=top_p, row_ids=rid.astype(np.int64))
    stats = compare_step(gpu, ref, V, "lattice on a truncated row", trunc=True, codes=codes)
    print("   ", stats, flush=True)
    tok = gpu["token"]
    assert np.all(np.diff(tok) >= 0)
    if stats["nucleus_rows"] == 0:                      # (a row whose nucleus closes within the band may keep one group more)
        p = np.zeros(V)
        p[ref["token"]] = ref["p"]
        assert np.all(p[tok] > 0)
        cnt = np.bincount(tok, minlength=V)
        seen = cnt > 0
        eps = 2 * N * 2.0 ** -24 + 1e-9
        slack = stats["mismatches"]
        assert np.all(cnt[seen] >= np.floor(N * p[seen] - eps) - slack)
        assert np.all(cnt[seen] <= np.ceil(N * p[seen] + eps) + slack)


def test_step_is_deterministic_and_in_place():
    import torch
    from paper_2210_15458_amd import binding as B
    from gpu_util import to_dev_logits
    V, R = 32128, 64
    logits = to_dev_logits(synth.gaussian_logits(R, V, seed=21, dtype="bf16"))
    codes = torch.from_numpy(synth.uniform_codes(R, seed=22)).cuda()
    ctx = B.Ctx(R, V, logits.dtype)
    outs = []
    for _ in range(3):
        tok = torch.empty(R, dtype=torch.int32, device="cuda")
        c = codes.clone()
        B.as_step(ctx, logits, c, 0.9, 0, 1.0, tok, c)                      # codes_out aliases codes
        torch.cuda.synchronize()
        outs.append((tok.cpu().numpy(), c.cpu().numpy()))
    for t, c in outs[1:]:
        assert np.array_equal(t, outs[0][0]) and np.array_equal(c, outs[0][1])


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("top_k,top_p,temp", [(40, 1.0, 1.0), (0, 0.9, 1.0), (1, 1.0, 1.0), (5, 0.5, 0.7),
                                              (1000, 0.95, 1.3), (0, 0.3, 0.8),
                                              # k beyond what the thread maxima can bound: by counts per bin
                                              (129, 0.9, 1.0), (200, 1.0, 1.0), (5000, 1.0, 0.7)])
def test_step_truncation(dtype, top_k, top_p, temp):
    _check(32128, 64, dtype, temp=temp, top_k=top_k, top_p=top_p, seed=31)
    _check(1001, 40, dtype, temp=temp, top_k=min(top_k, 900), top_p=top_p, seed=32)
    # rows that take the register-resident kernels and end inside a 16-byte piece (the padding holds +1e30)
    _check(1001, 40, dtype, temp=temp, top_k=min(top_k, 900), top_p=top_p, ld=1008, seed=37)
    _check(4099, 24, dtype, temp=temp, top_k=min(top_k, 4000), top_p=top_p, ld=4104, seed=38)
    _check(50257, 8, dtype, temp=temp, top_k=top_k, top_p=top_p, seed=39)


@pytest.mark.parametrize("top_k,top_p", [(40, 1.0), (0, 0.9), (5, 0.5)])
def test_step_truncation_radix_path(top_k, top_p):
    # the general keep-threshold kernel on rows that would otherwise take the resident one
    _check(32128, 48, "bf16", top_k=top_k, top_p=top_p, seed=35, tuning={"thr_path": 1})
    _check(32128, 24, "f32", top_k=top_k, top_p=top_p, seed=36, tuning={"thr_path": 1})


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_step_truncation_hard_rows(dtype):
    """Rows on which the resident keep-threshold kernel has to hand over to the radix select, and the edges of
    what it takes."""
    from gpu_util import compare_step, oracle_step, run_gpu_step
    V, R = 32128, 12
    rng = np.random.default_rng(77)
    x = rng.normal(0.0, 3.0, (R, V)).astype(np.float32)
    x[0, :] = 1.25                                   # every logit equal: all tie at the k-th place
    x[1, :] = np.round(x[1, :])                      # heavy ties (a few dozen distinct values)
    x[2, :] *= 0.001                                 # flat: the nucleus is 90 % of the vocabulary
    x[3, 100:] = -np.inf                             # only 100 live tokens
    x[4, ::2] = -np.inf                              # every other token masked out
    x[5, :] = -30.0; x[5, 17] = 5.0                  # one-hot
    x[6, :5000] += 40.0                              # 5000 tokens far above the rest
    x[7, :] = np.where(rng.random(V) < 0.5, 2.0, -2.0)   # two values
    stored = synth.f32_to_bf16_bits(x) if dtype == "bf16" else x
    codes = synth.uniform_codes(R, seed=78)
    for top_k, top_p, temp in [(40, 1.0, 1.0), (256, 1.0, 1.0), (257, 1.0, 1.0), (0, 0.9, 1.0), (0, 0.5, 0.7),
                               (100, 0.9, 1.0), (0, 0.999, 2.0)]:
        label = f"hard rows {dtype} k={top_k} p={top_p} temp={temp}"
        print("case", label, flush=True)
        gpu = run_gpu_step(stored, codes, V, temp=temp, top_k=top_k, top_p=top_p)
        ref = oracle_step(stored, codes, V, temp=temp, top_k=top_k, top_p=top_p)
        print("   ", compare_step(gpu, ref, V, label, trunc=True, codes=codes), flush=True)


@pytest.mark.parametrize("V,dtype", [(V, dt) for V in (7, 64, 255, 4097, 50257, 100003) for dt in ("bf16", "f32")
                                     if not (V > 60000 and dt == "f32")])
def test_step_shape_sweep(V, dtype):
    """Vocabulary sizes around the kernels' internal limits (one vector, one chunk, one share, one tile, several
    tiles, beyond what the register-resident kernels take), with and without row padding, flat and peaked rows,
    every kind of logit modifier."""
    rng = np.random.default_rng(V * 2 + (dtype == "f32"))
    for temp, k, p in [(1.0, 0, 1.0), (0.3, 0, 1.0), (2.5, 0, 1.0), (1.0, 40, 1.0), (0.8, 0, 0.92), (1.2, 100, 0.5),
                       (0.7, 128, 0.99)]:
        for pad in (0, 8):
            ld = None if pad == 0 else (V + 7) // 8 * 8 + pad
            _check(V, 12 if V > 20000 else 24, dtype, temp=temp, top_k=min(k, V - 1), top_p=p, ld=ld,
                   sigma=float(rng.choice([0.5, 3.0, 8.0])), seed=int(rng.integers(1, 1 << 30)))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_step_single_tile_kernel_edges(dtype):
    """Rows of whole vectors that fit one tile take a kernel of their own, with one reference per wave taken
    from the share's first chunk: rows on which that reference is far off (a first chunk that is all -inf or
    tiny against what follows, so that the weights overflow fp32 and the block falls back to the plain routine),
    shares that start past the row's end, a ragged last share, keep thresholds from the two-kernel path; and the
    general kernel on the same rows (its knob), which the single-tile one replaces by default."""
    from gpu_util import compare_step, oracle_step, run_gpu_step
    V = 32128 if dtype == "bf16" else 16000
    R = 10
    rng = np.random.default_rng(91)
    x = rng.normal(0.0, 3.0, (R, V)).astype(np.float32)
    x[0, :600] = -80.0; x[0, 700] = 80.0              # first chunk of wave 0 tiny, a huge logit later in the share
    x[1, :9000] = -np.inf                             # wave 0's first chunks all -inf, its share not
    x[2, :] = -np.inf; x[2, V - 1] = 1.0              # only the last token
    x[3, 8192:8192 + 512] = -np.inf                   # wave 1's first chunk all -inf
    x[4, :] = -60.0; x[4, 5000] = 70.0; x[4, 20000 % V] = 69.5
    x[5, 1::2] = -np.inf
    x[6, :] = 0.25                                    # flat
    stored = synth.f32_to_bf16_bits(x) if dtype == "bf16" else x
    codes = synth.uniform_codes(R, seed=92)
    for temp, top_k, top_p in [(1.0, 0, 1.0), (0.5, 0, 1.0), (0.05, 0, 1.0), (1.0, 300, 1.0), (1.0, 0, 0.9)]:
        for shape in (0, 6):
            label = f"single tile {dtype} temp={temp} k={top_k} p={top_p} shape={shape}"
            print("case", label, flush=True)
            gpu = run_gpu_step(stored, codes, V, temp=temp, top_k=top_k, top_p=top_p, tuning={"step_shape": shape})
            ref = oracle_step(stored, codes, V, temp=temp, top_k=top_k, top_p=top_p)
            print("   ", compare_step(gpu, ref, V, label, trunc=True, codes=codes), flush=True)
    # short rows: shares wholly past the row's end, and a ragged last share
    for Vs in (8, 512, 520, 8192, 8200, 16384 if dtype == "f32" else 32768):
        for shape in (0, 6):
            _check(Vs, 9, dtype, temp=0.8, seed=Vs, tuning={"step_shape": shape})


def test_step_topk_single_tile_kernel_edges():
    """bf16 rows of whole vectors that fit one tile, top-k up to 48 (with or without the nucleus), take a kernel
    of their own that bounds the k-th largest logit by the k-th largest of its 256 lane maxima and finishes on at
    most 64 candidates: the smallest and largest k it takes and the first it does not, rows that fill whole
    tiles, one piece, ragged last shares and shares past the row's end; rows whose candidates overflow its
    tables (ties at the bound, flat rows, two-valued rows) and hand over to the general selection; rows with
    fewer live tokens than k; all-negative rows; rows picked through row ids with finished rows among them.
    The register-resident kernel it replaces by default runs on the same rows (its knob) and must give the same
    tokens."""
    from gpu_util import compare_step, oracle_step, run_gpu_step
    V, R = 32128, 14
    rng = np.random.default_rng(191)
    x = rng.normal(0.0, 3.0, (R, V)).astype(np.float32)
    x[0, :] = 1.25                                   # every logit equal
    x[1, :] = np.round(x[1, :])                      # heavy ties at the bound
    x[2, :] *= 0.001                                 # flat
    x[3, 30:] = -np.inf                              # fewer live tokens than k
    x[4, :] = -np.abs(x[4, :]) - 0.5                 # all negative
    x[5, :] = -30.0; x[5, 17] = 5.0                  # one-hot
    x[6, :] = np.where(rng.random(V) < 0.5, 2.0, -2.0)
    x[7, :64] = 25.0 + np.arange(64) * 0.125         # the whole top in one chunk of one wave
    x[8, ::512] = 20.0                               # the top spread one logit per chunk, all equal
    own = ((np.arange(16)[:, None] * 64 + 5) * 8 + np.arange(8)[None, :]).ravel()   # what one lane of the first wave holds
    x[9, own[:60]] = 30.0 + rng.random(60).astype(np.float32)       # the whole top in that lane: its maximum says little
    x[10, V - 8:] = 40.0                             # the top in the row's last piece
    x[11, :] = -np.inf; x[11, 777] = 0.0             # a single live token
    stored = synth.f32_to_bf16_bits(x)
    codes = synth.uniform_codes(R, seed=192)
    for temp, top_k, top_p in [(1.0, 1, 1.0), (1.0, 2, 1.0), (1.0, 40, 1.0), (0.7, 48, 1.0), (1.0, 49, 1.0),
                               (1.0, 40, 0.9), (1.3, 48, 0.5), (1.0, 7, 0.999), (1.0, 3, 1e-6)]:
        toks = {}
        for path in (0, 2):
            label = f"top-k tile k={top_k} p={top_p} temp={temp} thr_path={path}"
            print("case", label, flush=True)
            gpu = run_gpu_step(stored, codes, V, temp=temp, top_k=top_k, top_p=top_p, tuning={"thr_path": path})
            ref = oracle_step(stored, codes, V, temp=temp, top_k=top_k, top_p=top_p)
            print("   ", compare_step(gpu, ref, V, label, trunc=True, codes=codes), flush=True)
            toks[path] = gpu["token"]
        assert (toks[0] == toks[2]).mean() >= (R - 1) / R, (toks[0], toks[2])
    # other widths of one tile: a single piece, a share and a bit, whole tiles, rows that end inside the last share
    for Vs in (8, 64, 520, 8192, 8200, 16392, 32760, 32768):
        for top_k, top_p in ((5, 1.0), (40, 0.95), (48, 1.0)):
            _check(Vs, 9, "bf16", temp=0.9, top_k=min(top_k, Vs - 1), top_p=top_p, seed=Vs + top_k)
    # gathered rows, finished rows and the end-of-sequence flag
    LR, R2 = 6, 50
    st = synth.gaussian_logits(LR, V, seed=193, dtype="bf16")
    wide = synth.bf16_bits_to_f32(st).copy()
    wide[:, 1] += 13.0
    st = synth.f32_to_bf16_bits(wide)
    rid = rng.integers(0, LR, R2).astype(np.int32)
    fin = (rng.random(R2) < 0.3).astype(np.uint8)
    c2 = synth.uniform_codes(R2, seed=194)
    for top_k, top_p in ((40, 1.0), (12, 0.8)):
        gpu = run_gpu_step(st, c2, V, top_k=top_k, top_p=top_p, finished=fin, eos_id=1, row_ids=rid)
        ref = oracle_step(st, c2, V, top_k=top_k, top_p=top_p, finished=fin, eos_id=1, row_ids=rid)
        print("   ", compare_step(gpu, ref, V, f"top-k tile gathered k={top_k} p={top_p}", trunc=True, codes=c2, eos_id=1),
              flush=True)
        assert (gpu["finished"][fin != 0] == 1).all()


def test_step_nucleus_single_tile_kernel_edges():
    """bf16 rows of whole vectors that fit one tile, the nucleus alone, take a kernel that counts logits by stored
    value in a window of 2048 values placed from the row's first chunks: rows whose largest logit lies far above
    what the first chunks show (above the window: the block hands over to the general selection), rows of
    negative logits only (the window runs the other way), negative first chunks with positive logits later,
    rows whose nucleus reaches across zero or below the window (flat rows, two-valued rows), tiny logits (a window
    that would cross zero), one live token, heavy ties; widths that leave shares empty or ragged; gathered and
    finished rows.  The register-resident kernel it replaces by default runs on the same rows (its knob)."""
    from gpu_util import compare_step, oracle_step, run_gpu_step
    V, R = 32128, 16
    rng = np.random.default_rng(291)
    x = rng.normal(0.0, 3.0, (R, V)).astype(np.float32)
    x[0, 20000] = 3.0e4                              # far above the window's top
    x[14, 9000] = 150.0                              # a confident row: one logit far above the rest, inside the window
    x[1, :] = -np.abs(x[1, :]) - 0.25                # negative logits only
    x[2, :512] = -np.abs(x[2, :512]) - 1.0           # the first chunk of the first wave negative, the rest mixed
    for w in range(4):                                # every wave's first chunk negative, positive logits later
        x[3, w * 8192: w * 8192 + 512] = -np.abs(x[3, w * 8192: w * 8192 + 512]) - 1.0
    x[4, :] *= 0.001                                 # flat: the nucleus is most of the row, on both sides of zero
    x[5, :] = np.where(rng.random(V) < 0.5, 2.0, -2.0)
    x[6, :] *= 1e-30                                 # tiny logits
    x[7, :] = -np.inf; x[7, 4321] = 0.5              # one live token
    x[8, :] = np.round(x[8, :])                      # heavy ties
    x[9, :] = np.abs(x[9, :]) + 0.5                  # positive logits only
    x[10, :] = 1.25                                  # every logit equal
    x[11, :] = -7.0; x[11, ::97] = -6.5              # negative, two values
    x[12, :] += 60.0                                 # a large common offset: a few values per factor of two
    x[13, :] = x[13, :] * 0.05 - 3.0                 # negative and narrow
    stored = synth.f32_to_bf16_bits(x)
    codes = synth.uniform_codes(R, seed=292)
    for temp, top_p in [(1.0, 0.9), (0.7, 0.5), (1.5, 0.99), (1.0, 0.05), (1.0, 1e-6), (0.3, 0.999)]:
        for path in (0, 2):
            label = f"nucleus tile p={top_p} temp={temp} thr_path={path}"
            print("case", label, flush=True)
            gpu = run_gpu_step(stored, codes, V, temp=temp, top_p=top_p, tuning={"thr_path": path})
            ref = oracle_step(stored, codes, V, temp=temp, top_p=top_p)
            print("   ", compare_step(gpu, ref, V, label, trunc=True, codes=codes), flush=True)
    for Vs in (8, 64, 520, 8192, 8200, 16392, 32760, 32768):
        for top_p in (0.9, 0.3):
            _check(Vs, 9, "bf16", temp=0.9, top_p=top_p, seed=Vs + 1)
    LR, R2 = 6, 50
    st = synth.gaussian_logits(LR, V, seed=293, dtype="bf16")
    wide = synth.bf16_bits_to_f32(st).copy()
    wide[:, 1] += 13.0
    st = synth.f32_to_bf16_bits(wide)
    rid = rng.integers(0, LR, R2).astype(np.int32)
    fin = (rng.random(R2) < 0.3).astype(np.uint8)
    c2 = synth.uniform_codes(R2, seed=294)
    gpu = run_gpu_step(st, c2, V, top_p=0.9, finished=fin, eos_id=1, row_ids=rid)
    ref = oracle_step(st, c2, V, top_p=0.9, finished=fin, eos_id=1, row_ids=rid)
    print("   ", compare_step(gpu, ref, V, "nucleus tile gathered", trunc=True, codes=c2, eos_id=1), flush=True)
    assert (gpu["finished"][fin != 0] == 1).all()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_step_signed_zero_ties(dtype):
    """-0 and +0 are one value: tied at the k-th place or in the group that closes the nucleus they stay or go
    together (the kernels select by integer keys of the stored bits, in which the two differ)."""
    from gpu_util import compare_step, oracle_step, run_gpu_step
    rng = np.random.default_rng(391)
    for V in (8, 1000, 32128):
        R = 24
        x = np.round(rng.normal(0.0, 0.3, (R, V)) * 2).astype(np.float32) / 2         # -0.5, -0, +0, 0.5 and a few more
        x[R // 2:, :] = np.minimum(x[R // 2:, :], 0.0)                                  # rows whose largest value is zero
        assert np.signbit(x[x == 0]).any() and not np.signbit(x[x == 0]).all()
        stored = synth.f32_to_bf16_bits(x) if dtype == "bf16" else x
        codes = synth.uniform_codes(R, seed=392 + V)
        for temp, top_k, top_p in [(1.0, 1, 1.0), (0.7, 1, 0.5), (1.0, 5, 1.0), (1.0, 40, 0.9), (1.0, 100, 1.0),
                                   (1.0, 0, 0.5), (1.0, 0, 0.05), (1.0, 300, 0.3)]:
            kk = min(top_k, V - 1)
            for tuning in (None, {"thr_path": 1}, {"thr_path": 2}):
                label = f"signed zeros {dtype} V={V} temp={temp} k={kk} p={top_p} tuning={tuning}"
                print("case", label, flush=True)
                gpu = run_gpu_step(stored, codes, V, temp=temp, top_k=kk, top_p=top_p, tuning=tuning)
                ref = oracle_step(stored, codes, V, temp=temp, top_k=kk, top_p=top_p)
                print("   ", compare_step(gpu, ref, V, label, trunc=True, codes=codes), flush=True)


def test_step_three_pass_kernel():
    # the plain three-pass kernel, which no shape needs any more, forced by its knob
    _check(1001, 24, "bf16", seed=41, tuning={"step_shape": 9})
    _check(4097, 12, "f32", temp=0.7, top_k=40, seed=42, tuning={"step_shape": 9})
    _check(32128, 8, "bf16", top_p=0.9, seed=43, tuning={"step_shape": 9})


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("V", [1 << 21, (1 << 21) - 5])
def test_step_maximum_vocab(V, dtype):
    """The largest vocabulary the library takes (AS_MAX_VOCAB): 64 tiles per bf16 row and 128 per fp32 row, so
    a lane of the deciding wave walks several shares; the ragged size has rows that start off 16 bytes."""
    _check(V, 3, dtype, seed=21)
    _check(V, 3, dtype, temp=0.8, top_k=40, seed=22)
    # (a peaked row: with two million near-equal fp32 probabilities every nucleus closes within the band of
    # top_p and the comparison would excuse all of it)
    _, _, stats = _check(V, 3, dtype, top_p=0.9, sigma=8.0, seed=23)
    assert stats["nucleus_rows"] < 3


def test_step_truncation_multi_tile():
    _check(256000, 6, "bf16", top_k=40, seed=33)
    _check(256000, 6, "bf16", top_p=0.9, seed=34)


def _hostile_rows(V, dtype, seed):
    """Rows and codes that break the contract on purpose (NaN, +inf, nothing finite, values near the largest
    float; codes outside [0, 1)): what comes back is undefined, but it must stay inside its bounds."""
    rng = np.random.default_rng(seed)
    R = 16
    x = (rng.standard_normal((R, V)) * 3.0).astype(np.float32)
    nan, inf = np.float32(np.nan), np.float32(np.inf)
    x[0, :] = nan
    x[1, rng.integers(0, V, max(1, V // 50))] = nan
    x[2, rng.integers(0, V, min(3, V))] = inf
    x[3, :] = -inf
    x[4, :] = np.where(rng.random(V) < 0.5, np.float32(3.0e38), np.float32(-3.0e38))
    x[5, :] = inf
    x[6, ::2] = nan
    x[6, 1::2] = inf
    x[7, :] = -inf
    x[7, V // 2] = nan
    x[8, 0] = inf
    x[8, V - 1] = -inf
    codes = rng.random(R).astype(np.float32)
    codes[9], codes[10], codes[11], codes[12], codes[13] = 1.0, 2.5, -0.5, nan, inf
    stored = synth.f32_to_bf16_bits(x) if dtype == "bf16" else x
    return stored, codes


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("V", [7, 1001, 32128, 50257])
def test_step_hostile_inputs_stay_in_bounds(V, dtype):
    """Data errors are not detected, but every path keeps its outputs in range: tokens in [0, V), the next code
    in [0, 1 - 2^-24], flags 0 or 1 (resident, fused and streamed truncation kernels, whole-vector and
    partial-vector rows, extreme temperatures)."""
    from gpu_util import run_gpu_step
    stored, codes = _hostile_rows(V, dtype, seed=V)
    for temp, top_k, top_p in [(1.0, 0, 1.0), (0.7, 40, 1.0), (1.0, 0, 0.9), (1.0, 5, 0.5), (1.0, 300, 0.95),
                               (1e-38, 0, 1.0), (1e38, 0, 0.9), (1e-30, 3, 0.7)]:
        print("case hostile", V, dtype, temp, top_k, top_p, flush=True)
        out = run_gpu_step(stored, codes, V, temp=temp, top_k=top_k, top_p=top_p, eos_id=1)
        tok, c = out["token"], out["c_next"]
        assert ((tok >= 0) & (tok < V)).all(), (temp, top_k, top_p, tok)
        assert np.isfinite(c).all() and (c >= 0.0).all() and (c <= np.float32(1.0) - np.float32(2.0 ** -24)).all(), c
        assert np.isin(out["finished"], (0, 1)).all()


def test_step_argument_errors():
    import torch
    from paper_2210_15458_amd import binding as B
    ctx = B.Ctx(8, 100, torch.float32)
    logits = torch.zeros(8, 100, device="cuda")
    codes = torch.zeros(8, device="cuda")
    tok = torch.zeros(8, dtype=torch.int32, device="cuda")
    with pytest.raises(B.ArithSamplingError) as e:
        B.as_step(ctx, logits, codes, 0.0, 0, 1.0, tok, codes)
    assert e.value.code == 1 and "temp" in str(e.value)
    with pytest.raises(B.ArithSamplingError):
        B.as_step(ctx, torch.zeros(8, 64, device="cuda"), codes, 1.0, 0, 1.0, tok, codes)   # ld < V
    with pytest.raises(B.ArithSamplingError):
        B.as_step(ctx, torch.zeros(9, 100, device="cuda"), torch.zeros(9, device="cuda"), 1.0, 0, 1.0,
                  torch.zeros(9, dtype=torch.int32, device="cuda"), torch.zeros(9, device="cuda"))  # rows > max
    B.as_step(ctx, logits[:0], codes[:0], 1.0, 0, 1.0, tok[:0], codes[:0])                  # empty batch is fine
    ctx.close()
