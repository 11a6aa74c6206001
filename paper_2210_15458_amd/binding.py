"""Thin ctypes binding of libarith_sampling.so (see include/arith_sampling.h).

Argument marshalling only: every function takes torch tensors that already live
on the GPU, checks device / dtype / contiguity, and passes raw pointers to the
C entry point of the same name.  Nothing is computed here and there is no
fallback: if the library is missing, loading it raises.
"""
import ctypes as C
import os

import torch

AS_F32, AS_BF16 = 0, 1
_STATUS = {0: "AS_OK", 1: "AS_ERR_INVALID_ARG", 2: "AS_ERR_UNSUPPORTED", 3: "AS_ERR_ALLOC", 4: "AS_ERR_DEVICE"}

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libarith_sampling.so")
_lib = None


class ArithSamplingError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"{_STATUS.get(code, code)}: {msg}")
        self.code = code


def lib():
    """Load the HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2210_15458_amd.build` "
            "(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    L.as_ctx_create.argtypes = [C.POINTER(vp), i64, i32, C.c_int, vp]
    L.as_ctx_destroy.argtypes = [vp]
    L.as_last_error.argtypes = [vp]
    L.as_last_error.restype = C.c_char_p
    L.as_step.argtypes = [vp, vp, i64, i64, vp, f32, i32, f32, vp, vp]
    L.as_step_ex.argtypes = [vp, vp, i64, i64, vp, f32, i32, f32, vp, vp, vp, i32, vp, vp, vp, vp, i64]
    L.as_step_static.argtypes = [vp, C.c_int, i64, i64, i32, vp, f32, i32, f32, vp, vp, vp]
    L.as_lattice.argtypes = [vp, vp, i32, i32, vp]
    L.as_model_create_bigram.argtypes = [C.POINTER(vp), vp, vp, i32, i32, f32, C.c_int]
    L.as_model_destroy.argtypes = [vp]
    L.as_bigram_logits.argtypes = [vp, vp, vp, i64, vp, i64]
    L.as_decode.argtypes = [vp, vp, vp, i32, i32, i32, vp, f32, i32, f32, i32, vp, vp]
    L.as_interval_step.argtypes = [vp, vp, i64, i64, vp, f32, i32, f32, vp, vp, vp, i32, vp, vp, i64]
    L.as_encode.argtypes = [vp, vp, vp, i32, i32, i32, vp, f32, i32, f32, i32, vp, vp]
    L.as_decode_ancestral.argtypes = [vp, vp, vp, i32, i32, i32, vp, f32, i32, f32, i32, vp]
    L.as_estimate_mean.argtypes = [vp, vp, i32, i32, i32, vp, i32, vp]
    L.as_decode_fused.argtypes = [vp, vp, vp, i32, i32, i32, vp, f32, i32, vp, vp]
    L.as_bigram_group_mass.argtypes = [vp, vp, vp, i64, f32, vp, i64]
    L.as_step_fused.argtypes = [vp, vp, vp, i64, vp, i64, vp, f32, vp, vp, vp, i32, vp]
    L.as_ctx_set_tuning.argtypes = [vp, C.c_int, i32]
    L.as_ctx_set_tuning.restype = C.c_int
    L.as_ctx_profile.argtypes = [vp, C.c_int]
    L.as_ctx_profile_read.argtypes = [vp, C.c_int, C.POINTER(C.c_double), C.POINTER(i64), C.POINTER(i64)]
    L.as_ctx_profile_samples.argtypes = [vp, C.c_int, C.POINTER(C.c_float), i64, C.POINTER(i64)]
    L.as_ctx_profile_samples.restype = C.c_int
    L.as_ctx_profile.restype = C.c_int
    L.as_ctx_profile_read.restype = C.c_int
    for name in ("as_ctx_create", "as_ctx_destroy", "as_step", "as_step_ex", "as_step_static", "as_lattice",
                 "as_model_create_bigram", "as_model_destroy", "as_bigram_logits", "as_decode",
                 "as_interval_step", "as_encode", "as_decode_ancestral", "as_estimate_mean", "as_decode_fused",
                 "as_bigram_group_mass", "as_step_fused"):
        getattr(L, name).restype = C.c_int
    _lib = L
    return L


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return AS_BF16
    if t.dtype == torch.float32:
        return AS_F32
    raise TypeError(f"unsupported storage dtype {t.dtype}")


def _dev(t, dtype, name, numel=None):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a GPU tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if numel is not None and t.numel() < numel:
        raise ValueError(f"{name} holds {t.numel()} elements, needs {numel}")
    return t.data_ptr()


class Ctx:
    """as_ctx: stream, vocabulary size, logits storage type and workspace."""

    def __init__(self, max_rows, V, logits_dtype=torch.bfloat16, stream=None):
        self._h = C.c_void_p()
        self.V = int(V)
        self.max_rows = int(max_rows)
        self.torch_dtype = logits_dtype
        self.dtype = AS_BF16 if logits_dtype == torch.bfloat16 else AS_F32
        if logits_dtype not in (torch.bfloat16, torch.float32):
            raise TypeError("logits dtype must be bfloat16 or float32")
        self.stream = torch.cuda.current_stream() if stream is None else stream
        rc = lib().as_ctx_create(C.byref(self._h), self.max_rows, self.V, self.dtype,
                                 C.c_void_p(self.stream.cuda_stream))
        if rc != 0:
            raise ArithSamplingError(rc, (lib().as_last_error(None) or b"").decode())

    def _check(self, rc):
        if rc != 0:
            raise ArithSamplingError(rc, (lib().as_last_error(self._h) or b"").decode())

    TUNING = {"step_shape": 0, "gemm_shape": 1, "thr_path": 2, "gemm_gm": 3}

    def set_tuning(self, knob, value):
        """Pick a kernel variant (tests and measurements): knob is one of Ctx.TUNING."""
        self._check(lib().as_ctx_set_tuning(self._h, self.TUNING[knob], int(value)))

    def profile(self, enable):
        self._check(lib().as_ctx_profile(self._h, 1 if enable else 0))

    def profile_read(self, kernel):
        """(total kernel ms, timed launches, untimed launches) since the last read."""
        ms, n, dropped = C.c_double(), C.c_int64(), C.c_int64()
        self._check(lib().as_ctx_profile_read(self._h, int(kernel), C.byref(ms), C.byref(n), C.byref(dropped)))
        return ms.value, n.value, dropped.value

    def profile_samples(self, kernel, capacity=16384):
        """Milliseconds of each timed launch since the last read, in launch order (call before profile_read)."""
        import numpy as np
        buf = np.empty(capacity, dtype=np.float32)
        n = C.c_int64()
        self._check(lib().as_ctx_profile_samples(self._h, int(kernel), buf.ctypes.data_as(C.POINTER(C.c_float)),
                                                 capacity, C.byref(n)))
        return buf[:min(n.value, capacity)].copy()

    def close(self):
        if self._h:
            lib().as_ctx_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Model:
    """as_model: the synthetic low-rank bigram model (borrows E, re-lays U out)."""

    def __init__(self, E, U, scale=3.0):
        V, d = E.shape
        if tuple(U.shape) != (d, V):
            raise ValueError("U must be [d, V] for E [V, d]")
        if E.dtype != U.dtype:
            raise TypeError("E and U must share a dtype")
        self.V, self.d = int(V), int(d)
        self._E = E                       # keep the borrowed tensor alive
        self._h = C.c_void_p()
        rc = lib().as_model_create_bigram(C.byref(self._h), _dev(E, E.dtype, "E"), _dev(U, U.dtype, "U"),
                                          self.V, self.d, float(scale), _dtype_code(E))
        if rc != 0:
            raise ArithSamplingError(rc, (lib().as_last_error(None) or b"").decode())

    def close(self):
        if self._h:
            lib().as_model_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _logits_args(ctx, logits, rows_needed=None):
    if logits.dim() != 2:
        raise ValueError("logits must be [rows, ld]")
    ptr = _dev(logits, ctx.torch_dtype, "logits")
    return ptr, logits.shape[0], logits.shape[1]


def as_step(ctx, logits, codes, temp, top_k, top_p, tokens_out, codes_out):
    ptr, rows, ld = _logits_args(ctx, logits)
    ctx._check(lib().as_step(ctx._h, ptr, rows, ld, _dev(codes, torch.float32, "codes", rows), float(temp),
                             int(top_k), float(top_p), _dev(tokens_out, torch.int32, "tokens_out", rows),
                             _dev(codes_out, torch.float32, "codes_out", rows)))


def as_step_static(logits, V, codes, temp, top_k, top_p, tokens_out, codes_out, stream=None):
    """as_step without a context (the entry point that allocates nothing); V columns of logits [rows, ld]."""
    if logits.dim() != 2:
        raise ValueError("logits must be [rows, ld]")
    rows, ld = logits.shape
    stream = torch.cuda.current_stream() if stream is None else stream
    rc = lib().as_step_static(_dev(logits, logits.dtype, "logits"), _dtype_code(logits), rows, ld, int(V),
                              _dev(codes, torch.float32, "codes", rows), float(temp), int(top_k), float(top_p),
                              _dev(tokens_out, torch.int32, "tokens_out", rows),
                              _dev(codes_out, torch.float32, "codes_out", rows), C.c_void_p(stream.cuda_stream))
    if rc != 0:
        raise ArithSamplingError(rc, (lib().as_last_error(None) or b"").decode())


def as_step_ex(ctx, logits, codes, temp, top_k, top_p, tokens_out, codes_out, finished_in=None, eos_id=-1,
               finished_out=None, prob_out=None, flo_out=None, row_ids=None):
    ptr, lrows, ld = _logits_args(ctx, logits)
    rows = codes.numel() if row_ids is not None else lrows
    ctx._check(lib().as_step_ex(
        ctx._h, ptr, rows, ld, _dev(codes, torch.float32, "codes", rows), float(temp), int(top_k), float(top_p),
        _dev(tokens_out, torch.int32, "tokens_out", rows), _dev(codes_out, torch.float32, "codes_out", rows),
        _dev(finished_in, torch.uint8, "finished_in", rows), int(eos_id),
        _dev(finished_out, torch.uint8, "finished_out", rows), _dev(prob_out, torch.float32, "prob_out", rows),
        _dev(flo_out, torch.float32, "flo_out", rows), _dev(row_ids, torch.int32, "row_ids", rows), lrows))


def as_lattice(ctx, u, N, codes_out):
    B = u.numel()
    ctx._check(lib().as_lattice(ctx._h, _dev(u, torch.float32, "u"), B, int(N),
                                _dev(codes_out, torch.float32, "codes_out", B * int(N))))


def as_bigram_logits(ctx, model, prev, logits_out):
    ptr, rows, ld = _logits_args(ctx, logits_out)
    ctx._check(lib().as_bigram_logits(ctx._h, model._h, _dev(prev, torch.int32, "prev", rows), rows, ptr, ld))


def as_decode(ctx, model, prompts, N, T, u, temp, top_k, top_p, eos_id, tokens_out, codes_out=None):
    B = prompts.numel()
    ctx._check(lib().as_decode(
        ctx._h, model._h, _dev(prompts, torch.int32, "prompts"), B, int(N), int(T),
        _dev(u, torch.float32, "u", B), float(temp), int(top_k), float(top_p), int(eos_id),
        _dev(tokens_out, torch.int32, "tokens_out", B * int(N) * int(T)),
        _dev(codes_out, torch.float32, "codes_out", B * int(N))))


def as_interval_step(ctx, logits, tokens, temp, top_k, top_p, lo, width, finished_in=None, eos_id=-1,
                     finished_out=None, row_ids=None):
    ptr, lrows, ld = _logits_args(ctx, logits)
    rows = tokens.numel() if row_ids is not None else lrows
    ctx._check(lib().as_interval_step(
        ctx._h, ptr, rows, ld, _dev(tokens, torch.int32, "tokens", rows), float(temp), int(top_k), float(top_p),
        _dev(lo, torch.float64, "lo", rows), _dev(width, torch.float64, "width", rows),
        _dev(finished_in, torch.uint8, "finished_in", rows), int(eos_id),
        _dev(finished_out, torch.uint8, "finished_out", rows), _dev(row_ids, torch.int32, "row_ids", rows), lrows))


def as_encode(ctx, model, prompts, N, T, tokens, temp, top_k, top_p, eos_id, lo_out, width_out):
    B = prompts.numel()
    ctx._check(lib().as_encode(
        ctx._h, model._h, _dev(prompts, torch.int32, "prompts"), B, int(N), int(T),
        _dev(tokens, torch.int32, "tokens", B * int(N) * int(T)), float(temp), int(top_k), float(top_p),
        int(eos_id), _dev(lo_out, torch.float64, "lo_out", B * int(N)),
        _dev(width_out, torch.float64, "width_out", B * int(N))))


def as_decode_ancestral(ctx, model, prompts, N, T, uniforms, temp, top_k, top_p, eos_id, tokens_out):
    B = prompts.numel()
    ctx._check(lib().as_decode_ancestral(
        ctx._h, model._h, _dev(prompts, torch.int32, "prompts"), B, int(N), int(T),
        _dev(uniforms, torch.float32, "uniforms", B * int(N) * int(T)), float(temp), int(top_k), float(top_p),
        int(eos_id), _dev(tokens_out, torch.int32, "tokens_out", B * int(N) * int(T))))


def as_estimate_mean(ctx, tokens, score, eos_id, est_out):
    if tokens.dim() != 3:
        raise ValueError("tokens must be [B, N, T]")
    B, N, T = tokens.shape
    ctx._check(lib().as_estimate_mean(
        ctx._h, _dev(tokens, torch.int32, "tokens"), B, N, T, _dev(score, torch.float32, "score", ctx.V),
        int(eos_id), _dev(est_out, torch.float64, "est_out", B)))


def as_decode_fused(ctx, model, prompts, N, T, u, temp, eos_id, tokens_out, codes_out=None):
    B = prompts.numel()
    ctx._check(lib().as_decode_fused(
        ctx._h, model._h, _dev(prompts, torch.int32, "prompts"), B, int(N), int(T),
        _dev(u, torch.float32, "u", B), float(temp), int(eos_id),
        _dev(tokens_out, torch.int32, "tokens_out", B * int(N) * int(T)),
        _dev(codes_out, torch.float32, "codes_out", B * int(N))))


def as_bigram_group_mass(ctx, model, prev, temp, mass_out):
    if mass_out.dim() != 3 or mass_out.shape[2] != 2:
        raise ValueError("mass_out must be [rows, ldp, 2]")
    rows, ldp = mass_out.shape[0], mass_out.shape[1]
    ctx._check(lib().as_bigram_group_mass(ctx._h, model._h, _dev(prev, torch.int32, "prev", rows), rows, float(temp),
                                          _dev(mass_out, torch.float32, "mass_out"), ldp))


def as_step_fused(ctx, model, mass, prev, codes, temp, tokens_out, codes_out, finished_in=None, eos_id=-1,
                  finished_out=None):
    if mass.dim() != 3 or mass.shape[2] != 2:
        raise ValueError("mass must be [rows, ldp, 2]")
    rows, ldp = mass.shape[0], mass.shape[1]
    ctx._check(lib().as_step_fused(
        ctx._h, model._h, _dev(mass, torch.float32, "mass"), ldp, _dev(prev, torch.int32, "prev", rows), rows,
        _dev(codes, torch.float32, "codes", rows), float(temp), _dev(tokens_out, torch.int32, "tokens_out", rows),
        _dev(codes_out, torch.float32, "codes_out", rows), _dev(finished_in, torch.uint8, "finished_in", rows),
        int(eos_id), _dev(finished_out, torch.uint8, "finished_out", rows)))
