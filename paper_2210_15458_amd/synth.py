"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds no part of the sampling method: it only draws the arrays
(model weights, start tokens, lattice shifts, stand-alone logits, uniform codes)
that are then handed, unchanged, both to the HIP library and to the CPU oracle.

Generator: NumPy's Philox (a counter-based generator), keyed by
(seed, stream), so every tensor has its own reproducible stream whatever order
tensors are drawn in.  Narrow storage types are produced by ONE
round-to-nearest-even step from the float32 draw; bfloat16 tensors are carried
as uint16 bit patterns (NumPy has no bfloat16).
"""
import numpy as np

# stream ids (second half of the Philox key)
_STREAM_E, _STREAM_U, _STREAM_PROMPT, _STREAM_SHIFT, _STREAM_LOGITS, _STREAM_CODES = range(6)


def _rng(seed, stream):
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def f32_to_bf16_bits(a):
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = bits + np.uint32(0x7FFF) + lsb
    out = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = (bits & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    if nan.any():
        out[nan] = ((bits[nan] >> np.uint32(16)) | np.uint32(0x40)).astype(np.uint16)
    return out


def bf16_bits_to_f32(b):
    """bfloat16 bit patterns (uint16) -> float32, exact."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_f32(rng, shape, chunk=1 << 24):
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        out[s:e] = rng.standard_normal(e - s, dtype=np.float32)
    return out.reshape(shape)


def bigram_weights(V, d, seed=0, dtype="bf16"):
    """E[V,d], U[d,V] i.i.d. N(0,1).  dtype 'bf16' -> uint16 bits, 'f32' -> float32."""
    E = _normal_f32(_rng(seed, _STREAM_E), (V, d))
    U = _normal_f32(_rng(seed, _STREAM_U), (d, V))
    if dtype == "bf16":
        return f32_to_bf16_bits(E), f32_to_bf16_bits(U)
    if dtype == "f32":
        return E, U
    raise ValueError(dtype)


def prompts(B, V, seed=1):
    """B start tokens, uniform on [0, V)."""
    return _rng(seed, _STREAM_PROMPT).integers(0, V, size=B, dtype=np.int32)


def shifts(B, seed=2):
    """One lattice shift per prompt, uniform on [0,1), float32."""
    u = _rng(seed, _STREAM_SHIFT).random(B, dtype=np.float32)
    return np.minimum(u, np.float32(1.0 - 2.0 ** -24))


def gaussian_logits(R, V, sigma=3.0, seed=3, dtype="bf16", ld=None):
    """Stand-alone logits [R, ld] with N(0, sigma^2) entries in the first V columns.

    Same marginal law as the bigram model's logits (scale 3).  Columns V..ld-1
    (row padding) are filled with +1e30 so that a kernel reading past V shows up
    as a wrong answer rather than passing by luck.
    """
    ld = V if ld is None else int(ld)
    x = np.full((R, ld), 1e30, dtype=np.float32)
    x[:, :V] = _normal_f32(_rng(seed, _STREAM_LOGITS), (R, V)) * np.float32(sigma)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    if dtype == "f32":
        return x
    raise ValueError(dtype)


def uniform_codes(R, seed=4):
    """R codes uniform on [0,1), float32."""
    c = _rng(seed, _STREAM_CODES).random(R, dtype=np.float32)
    return np.minimum(c, np.float32(1.0 - 2.0 ** -24))


# The five benchmark configurations (vocabulary, rank, prompts, codes per
# prompt, steps, temperature, truncation, storage type).
CONFIGS = {
    0: dict(name="tiny", V=16, d=8, B=1, N=64, T=8, temp=1.0, top_k=0, top_p=1.0,
            dtype="f32", eos_id=1, scale=3.0),
    1: dict(name="v32k_b16_n64", V=32128, d=512, B=16, N=64, T=64, temp=0.7,
            top_k=0, top_p=1.0, dtype="bf16", eos_id=1, scale=3.0),
    2: dict(name="v32k_b64_n16_trunc", V=32128, d=512, B=64, N=16, T=128, temp=1.0,
            top_k=40, top_p=0.9, dtype="bf16", eos_id=1, scale=3.0),
    3: dict(name="v256k_b8_n128", V=256000, d=1024, B=8, N=128, T=32, temp=1.0,
            top_k=0, top_p=1.0, dtype="bf16", eos_id=1, scale=3.0),
    4: dict(name="wide_n65536", V=32128, d=512, B=1, N=65536, T=16, temp=1.0,
            top_k=0, top_p=1.0, dtype="bf16", eos_id=1, scale=3.0),
}
