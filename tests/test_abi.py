"""The C-ABI library builds, loads and exports every function that
include/pso_ps.h declares; argument checks that need no GPU."""
import ctypes
import os
import re

import paper_2009_03816_amd as pso
from paper_2009_03816_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "pso_ps.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pso_ps_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    names = declared_functions()
    assert {"pso_ps_create", "pso_ps_sync", "pso_ps_destroy"} <= set(names)
    lib = ctypes.CDLL(binding.library_path()) if os.path.exists(binding.library_path()) \
        else binding.load()
    for name in names:
        assert hasattr(lib, name), name
        assert hasattr(pso, name), f"binding lacks {name}"


def test_binding_constants_are_the_headers():
    text = open(os.path.join(ROOT, "include", "pso_ps.h")).read()
    defines = dict(re.findall(r"^#define\s+(PSO_PS_[A-Z_]+)\s+\(?(-?\d+)\)?", text, flags=re.M))
    assert {"PSO_PS_OK", "PSO_PS_ELIMIT", "PSO_PS_STATIC_MAX_K", "PSO_PS_SINGLE_LAUNCH_MAX_K",
            "PSO_PS_SINGLE_LAUNCH_MAX_PARAMS"} <= set(defines)
    for name, value in defines.items():
        assert getattr(pso, name) == int(value), name


def test_status_texts_and_argument_checks_without_a_gpu():
    assert pso.pso_ps_strerror(pso.PSO_PS_OK) == "ok"
    for code in (pso.PSO_PS_EINVAL, pso.PSO_PS_EALIGN, pso.PSO_PS_EHIP, pso.PSO_PS_ENOMEM, -99):
        assert pso.pso_ps_strerror(code)
    lib = binding.load()
    h = ctypes.c_void_p()
    # rejected before any HIP call is made
    assert lib.pso_ps_create(None, 4, 10, 10, 0, None, 0) == pso.PSO_PS_EINVAL
    assert lib.pso_ps_create(ctypes.byref(h), 0, 10, 10, 0, None, 0) == pso.PSO_PS_EINVAL
    assert lib.pso_ps_create(ctypes.byref(h), 4, 10, 9, 0, None, 0) == pso.PSO_PS_EINVAL
    sizes = (ctypes.c_int64 * 2)(4, 5)
    assert lib.pso_ps_create(ctypes.byref(h), 4, 10, 10, 2, sizes, 0) == pso.PSO_PS_EINVAL
    assert lib.pso_ps_sync(None, 0, 0, 0, 0, 0, 0, 0.5, 1.0, 1.0, 0, 0, None) == pso.PSO_PS_EINVAL
    # a flat index must fit the generator's 32-bit pair counter: D <= 2^33
    assert lib.pso_ps_create(ctypes.byref(h), 4, (1 << 33) + 1, (1 << 33) + 1, 0, None, 0) \
        == pso.PSO_PS_EINVAL
    assert lib.pso_ps_destroy(None) == pso.PSO_PS_OK
    assert h.value is None


def test_probe_library_exports_what_its_header_declares():
    from paper_2009_03816_amd import build
    text = open(os.path.join(ROOT, "include", "pso_ps_probes.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(pso_ps_[a-z_]+)\s*\(", text)))
    assert names == ["pso_ps_probe_policy", "pso_ps_probe_stream"]
    if not os.path.exists(build.PROBES_LIBRARY):
        build.build_probes()
    lib = ctypes.CDLL(build.PROBES_LIBRARY)
    for name in names:
        assert hasattr(lib, name), name
    # rejected before any HIP call is made
    assert lib.pso_ps_probe_stream(2, None, None, None, None, 4, 16, 16, 128, 1, 1, 1, 1024, 128,
                                   10, 1, 1, 0, None) == -1
    assert lib.pso_ps_probe_policy(None, None, None, None, 4, 16, 16, 2048, 256, 20, 2, 2, None) == -1
