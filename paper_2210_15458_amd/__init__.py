"""MI355X-native arithmetic sampling (arXiv 2210.15458): Python names of the C ABI.

`binding` needs torch and the built HIP library and is imported on first use, so
that the seeded input generators (`synth`) stay importable on their own.
"""

_BINDING_NAMES = ("Ctx", "Model", "as_step", "as_step_ex", "as_lattice", "as_bigram_logits", "as_decode",
                  "as_interval_step", "as_encode", "as_decode_ancestral", "as_estimate_mean", "as_decode_fused", "as_bigram_group_mass", "as_step_fused",
                  "ArithSamplingError", "lib", "LIB_PATH", "AS_F32", "AS_BF16")


def __getattr__(name):
    if name in _BINDING_NAMES:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
