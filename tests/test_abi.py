"""CPU-side checks of the boundary: the shared library builds, loads and exports
every symbol the header declares (no compute call is made without a GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "arith_sampling.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(as_[a-z_]+)\s*\(", text)))


def test_header_declares_the_two_calls_of_the_problem_statement():
    names = _declared_symbols()
    assert "as_step" in names and "as_decode" in names
    assert len(names) >= 10


def test_library_loads_and_exports_every_declared_symbol():
    from paper_2210_15458_amd import build as hip_build
    path = hip_build.build(force=False)
    lib = ctypes.CDLL(path)
    for name in _declared_symbols():
        assert hasattr(lib, name), name


def test_binding_prototypes_cover_the_header():
    from paper_2210_15458_amd import binding
    lib = binding.lib()
    for name in _declared_symbols():
        fn = getattr(lib, name)
        assert fn.argtypes is not None, f"binding has no prototype for {name}"


def test_host_side_argument_checks_need_no_gpu():
    from paper_2210_15458_amd import binding
    lib = binding.lib()
    # every call with a NULL context is refused on the host with a message
    rc = lib.as_step(None, None, 1, 1, None, 1.0, 0, 1.0, None, None)
    assert rc == 1 and b"ctx" in lib.as_last_error(None)
    rc = lib.as_decode(None, None, None, 1, 1, 1, None, 1.0, 0, 1.0, -1, None, None)
    assert rc == 1
    out = ctypes.c_void_p()
    rc = lib.as_ctx_create(ctypes.byref(out), 0, 16, 0, None)
    assert rc == 1 and b"max_rows" in lib.as_last_error(None)
    rc = lib.as_ctx_create(ctypes.byref(out), 4, (1 << 21) + 1, 0, None)
    assert rc == 1 and b"V" in lib.as_last_error(None)
    rc = lib.as_ctx_create(ctypes.byref(out), 4, 16, 7, None)
    assert rc == 1 and b"dtype" in lib.as_last_error(None)
    rc = lib.as_model_create_bigram(ctypes.byref(out), None, None, 16, 8, 3.0, 0)
    assert rc == 1
    # the context-free step refuses more rows than its fixed workspace holds before it looks at a device
    rc = lib.as_step_static(None, 0, 65537, 16, 16, None, 1.0, 0, 1.0, None, None, None)
    assert rc == 1 and b"AS_STATIC_MAX_ROWS" in lib.as_last_error(None)


def test_product_package_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2210_15458_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in src and "from oracle" not in src and "liboracle" not in src, f
                assert "arith_oracle" not in src, f


def test_bench_refuses_more_than_one_gpu():
    """This build is one GPU: `bench.py --gpus N` with N > 1 says so and exits before it touches a device."""
    import subprocess
    import sys
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert out.returncode != 0
    assert "one GPU" in (out.stdout + out.stderr)
    assert "{" not in out.stdout                     # no benchmark line
