"""ctypes view of the fp64 CPU oracle (oracle/arith_oracle.c).

TEST INFRASTRUCTURE: only tests/, the smoke check and the benchmark's
cpu_baseline leg may import this package.  It knows nothing about the HIP
library and the HIP library knows nothing about it; both are fed the same
arrays by the caller.

Each wrapper below only marshals NumPy arrays; the arithmetic is in the C file,
which cites the passages of the paper it follows.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

F32, BF16, F64 = 0, 1, 2

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.ao_lattice.argtypes = [C.c_int32, C.c_double, C.c_void_p]
        L.ao_lattice.restype = None
        L.ao_lattice_paper.argtypes = [C.c_int32, C.c_double, C.c_void_p]
        L.ao_lattice_paper.restype = None
        L.ao_step_rows.argtypes = [
            C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int32, C.c_void_p,
            C.c_void_p, C.c_double, C.c_int32, C.c_double, C.c_void_p,
            C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
            C.c_int32, C.c_double, C.c_void_p, C.c_void_p, C.c_void_p]
        L.ao_step_rows.restype = C.c_int
        L.ao_bigram_logits.argtypes = [
            C.c_void_p, C.c_void_p, C.c_int, C.c_int32, C.c_int32, C.c_double,
            C.c_int32, C.c_int, C.c_void_p]
        L.ao_bigram_logits.restype = None
        L.ao_decode.argtypes = [
            C.c_void_p, C.c_void_p, C.c_int, C.c_int32, C.c_int32, C.c_double,
            C.c_int, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
            C.c_double, C.c_int32, C.c_double, C.c_int32, C.c_void_p,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_int]
        L.ao_decode.restype = C.c_int
        L.ao_encode.argtypes = [
            C.c_void_p, C.c_void_p, C.c_int, C.c_int32, C.c_int32, C.c_double,
            C.c_int, C.c_int32, C.c_void_p, C.c_int32, C.c_double, C.c_int32,
            C.c_double, C.c_int32, C.c_void_p, C.c_void_p]
        L.ao_encode.restype = C.c_int
        L.ao_token_interval_rows.argtypes = [
            C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int32, C.c_void_p,
            C.c_void_p, C.c_double, C.c_int32, C.c_double, C.c_void_p,
            C.c_void_p, C.c_void_p, C.c_int]
        L.ao_token_interval_rows.restype = C.c_int
        L.ao_estimate_mean.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int32,
                                       C.c_void_p]
        L.ao_estimate_mean.restype = None
        L.ao_max_threads.argtypes = []
        L.ao_max_threads.restype = C.c_int
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _stored(a):
    """(contiguous array, dtype code) for a stored tensor.

    float32 -> F32, float64 -> F64, uint16 -> BF16 (raw bfloat16 bit patterns).
    """
    a = np.ascontiguousarray(a)
    if a.dtype == np.float32:
        return a, F32
    if a.dtype == np.float64:
        return a, F64
    if a.dtype == np.uint16:
        return a, BF16
    raise TypeError("stored tensors must be float32, float64 or uint16 (bf16 bits)")


def max_threads():
    return int(lib().ao_max_threads())


def lattice(N, u):
    out = np.empty(N, dtype=np.float64)
    lib().ao_lattice(N, float(u), _ptr(out))
    return out


def lattice_paper(N, b):
    out = np.empty(N, dtype=np.float64)
    lib().ao_lattice_paper(N, float(b), _ptr(out))
    return out


def _step_call(logits, dt, ld, V, codes, temp, top_k, top_p, fin, eos_id, rid, nthreads, nuc_shift, band):
    rows = codes.shape[0]
    out = dict(
        token=np.empty(rows, np.int32), c_next=np.empty(rows, np.float64),
        p=np.empty(rows, np.float64), f_lo=np.empty(rows, np.float64),
        f_hi=np.empty(rows, np.float64), delta=np.empty(rows, np.float64),
        nuc_margin=np.empty(rows, np.float64), n_kept=np.empty(rows, np.int32),
        finished=np.empty(rows, np.uint8), nuc_alt=np.empty((rows, 2), np.int32),
        tok_nb=np.empty((rows, 2), np.int32), p_nb=np.empty((rows, 2), np.float64))
    rc = lib().ao_step_rows(
        _ptr(logits), dt, rows, ld, V, _ptr(rid), _ptr(codes), float(temp),
        int(top_k), float(top_p), _ptr(fin), int(eos_id), _ptr(out["token"]),
        _ptr(out["c_next"]), _ptr(out["p"]), _ptr(out["f_lo"]),
        _ptr(out["f_hi"]), _ptr(out["delta"]), _ptr(out["nuc_margin"]),
        _ptr(out["n_kept"]), _ptr(out["finished"]), int(nthreads),
        int(nuc_shift), float(band), _ptr(out["nuc_alt"]), _ptr(out["tok_nb"]), _ptr(out["p_nb"]))
    if rc != 0:
        raise MemoryError("oracle step failed")
    return out


def step(logits, codes, temp=1.0, top_k=0, top_p=1.0, finished=None,
         eos_id=-1, row_ids=None, V=None, nthreads=1, band=0.0, nuc_shift=0):
    """One decode step for every row.  Returns a dict of per-row arrays.

    With band > 0 and the nucleus on, rows whose running mass passes within `band` of top_p at a group end
    also get the step under every other admissible closing of the nucleus: out["alt"] yields
    (shift, row indices, dict of arrays for those rows), one entry per shift != 0 that some row admits
    (the C routine is simply called again for those rows with that shift, when the entry is asked for).
    """
    logits, dt = _stored(logits)
    if logits.ndim == 1:
        logits = logits[None, :]
    ld = logits.shape[1]
    V = ld if V is None else int(V)
    codes = np.ascontiguousarray(codes, dtype=np.float64)
    rows = codes.shape[0]
    rid = None if row_ids is None else np.ascontiguousarray(row_ids, dtype=np.int64)
    fin = None if finished is None else np.ascontiguousarray(finished, dtype=np.uint8)
    out = _step_call(logits, dt, ld, V, codes, temp, top_k, top_p, fin, eos_id, rid, nthreads, nuc_shift, band)
    call = dict(logits=logits, V=V, temp=temp, top_k=top_k, top_p=top_p, nthreads=nthreads)
    out["_call"] = dict(call, row_ids=rid, finished=fin, nuc_shift=nuc_shift)
    out["alt"] = _Alternatives(None, None, None)
    if band > 0.0 and 0.0 < top_p < 1.0 and nuc_shift == 0:
        src = np.arange(rows, dtype=np.int64) if rid is None else rid

        def under(shift, idx):
            sub = _step_call(logits, dt, ld, V, np.ascontiguousarray(codes[idx]), temp, top_k, top_p,
                             None if fin is None else np.ascontiguousarray(fin[idx]), eos_id,
                             np.ascontiguousarray(src[idx]), nthreads, shift, band)
            sub["_call"] = dict(call, row_ids=np.ascontiguousarray(src[idx]),
                                finished=None if fin is None else np.ascontiguousarray(fin[idx]), nuc_shift=shift)
            return sub
        out["alt"] = _Alternatives(under, out["nuc_alt"][:, 0].copy(), out["nuc_alt"][:, 1].copy())
    return out


class _Alternatives:
    """The step under the other admissible closings of the nucleus, computed when asked for: iterating gives
    (shift, row indices, dict of arrays for those rows), nearest closings first (-1, +1, -2, +2, ...), one entry
    per shift != 0 that some row admits.  among(rows) does the same for a subset of the rows (a boolean mask);
    at most `limit` shifts a side (a nucleus whose top_p lies within the band of 1 admits thousands)."""

    def __init__(self, under, lo, hi):
        self.under, self.lo, self.hi = under, lo, hi

    def among(self, mask=None, limit=None):
        if self.under is None:
            return
        lo = self.lo if mask is None else np.where(mask, self.lo, 0)
        hi = self.hi if mask is None else np.where(mask, self.hi, 0)
        nlo, nhi = int(lo.max(initial=0)), int(hi.max(initial=0))
        if limit is not None:
            nlo, nhi = min(nlo, limit), min(nhi, limit)
        for m in range(1, max(nlo, nhi) + 1):
            for shift in (-m, m):
                if (shift < 0 and m > nlo) or (shift > 0 and m > nhi):
                    continue
                idx = np.nonzero((lo >= m) if shift < 0 else (hi >= m))[0]
                if idx.size:
                    yield shift, idx, self.under(shift, idx)

    def __iter__(self):
        return self.among()


def interval_in(step_result, rows, tokens):
    """(f_lo, p) of tokens[i] on row rows[i] of an earlier step() call (or of one of its alternatives), under the
    same logits, modifiers and nucleus closing: where another token than the emitted one sits in that row's
    cumulative distribution."""
    c = step_result["_call"]
    rows = np.asarray(rows, dtype=np.int64)
    src = rows if c["row_ids"] is None else c["row_ids"][rows]
    fin = None if c["finished"] is None else c["finished"][rows]
    return token_interval(c["logits"], np.asarray(tokens, dtype=np.int32), temp=c["temp"], top_k=c["top_k"],
                          top_p=c["top_p"], V=c["V"], finished=fin, row_ids=src, nthreads=c["nthreads"],
                          nuc_shift=c["nuc_shift"])


def bigram_logits(E, U, prev, scale=3.0, round_mode=0):
    E, dt = _stored(E)
    U, dt2 = _stored(U)
    assert dt == dt2
    V, d = E.shape
    assert U.shape == (d, V)
    x = np.empty(V, dtype=np.float64)
    lib().ao_bigram_logits(_ptr(E), _ptr(U), dt, V, d, float(scale), int(prev),
                           int(round_mode), _ptr(x))
    return x


def decode(E, U, prompts, N, T, codes0, temp=1.0, top_k=0, top_p=1.0,
           eos_id=-1, scale=3.0, round_mode=0, nthreads=1, records=False):
    E, dt = _stored(E)
    U, dt2 = _stored(U)
    assert dt == dt2
    V, d = E.shape
    prompts = np.ascontiguousarray(prompts, dtype=np.int32)
    B = prompts.shape[0]
    codes0 = np.ascontiguousarray(codes0, dtype=np.float64).reshape(-1)
    assert codes0.shape[0] == B * N
    tokens = np.empty((B * N, T), dtype=np.int32)
    cf = np.empty(B * N, dtype=np.float64)
    p = np.empty((B * N, T), dtype=np.float64) if records else None
    dl = np.empty((B * N, T), dtype=np.float64) if records else None
    rc = lib().ao_decode(_ptr(E), _ptr(U), dt, V, d, float(scale),
                         int(round_mode), _ptr(prompts), B, int(N), int(T),
                         _ptr(codes0), float(temp), int(top_k), float(top_p),
                         int(eos_id), _ptr(tokens), _ptr(cf), _ptr(p), _ptr(dl),
                         int(nthreads))
    if rc != 0:
        raise MemoryError("oracle decode failed")
    out = dict(tokens=tokens.reshape(B, N, T), codes_final=cf.reshape(B, N))
    if records:
        out["p"] = p.reshape(B, N, T)
        out["delta"] = dl.reshape(B, N, T)
    return out


def estimate_mean(tokens, score, eos_id=-1):
    """(1/N) sum_i s(x_i) per prompt for tokens [B, N, T] and additive per-token scores score[V]."""
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    B, N, T = tokens.shape
    score = np.ascontiguousarray(score, dtype=np.float64)
    est = np.empty(B, dtype=np.float64)
    lib().ao_estimate_mean(_ptr(tokens), B, N, T, _ptr(score), int(eos_id), _ptr(est))
    return est


def token_interval(stored, tokens, temp=1.0, top_k=0, top_p=1.0, V=None,
                   finished=None, row_ids=None, nthreads=1, nuc_shift=0):
    """Per row: (f_lo, p) of tokens[r] in the row's kept, tempered softmax.

    `stored` as in `step`.  One step of the codebook recursion for a known
    next token; finished rows give (0, 1).
    """
    stored, dt = _stored(stored)
    rows_avail, ld = stored.shape
    V = ld if V is None else int(V)
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    rows = tokens.shape[0]
    rid = None if row_ids is None else np.ascontiguousarray(row_ids, dtype=np.int64)
    fin = None if finished is None else np.ascontiguousarray(finished, dtype=np.uint8)
    f_lo = np.empty(rows, dtype=np.float64)
    p = np.empty(rows, dtype=np.float64)
    rc = lib().ao_token_interval_rows(_ptr(stored), dt, rows, ld, V,
                                      _ptr(rid), _ptr(tokens),
                                      float(temp), int(top_k), float(top_p),
                                      _ptr(fin),
                                      _ptr(f_lo), _ptr(p), int(nthreads), int(nuc_shift))
    if rc != 0:
        raise MemoryError("oracle token_interval failed")
    return f_lo, p


def encode(E, U, prompt, seq, temp=1.0, top_k=0, top_p=1.0, eos_id=-1,
           scale=3.0, round_mode=0):
    """Interval (w, P) of a sequence or prefix: codes in [w, w+P) decode to it."""
    E, dt = _stored(E)
    U, dt2 = _stored(U)
    assert dt == dt2
    V, d = E.shape
    seq = np.ascontiguousarray(seq, dtype=np.int32)
    w = C.c_double()
    P = C.c_double()
    rc = lib().ao_encode(_ptr(E), _ptr(U), dt, V, d, float(scale),
                         int(round_mode), int(prompt), _ptr(seq), seq.shape[0],
                         float(temp), int(top_k), float(top_p), int(eos_id),
                         C.byref(w), C.byref(P))
    if rc != 0:
        raise MemoryError("oracle encode failed")
    return w.value, P.value
