"""The binding never runs a library that was built from other sources than
the ones next to it: the build stamps a hash of the sources into the library,
and load() rebuilds (or refuses) on a mismatch."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_loaded_library_carries_the_hash_of_the_sources_on_disk():
    import paper_2009_03816_amd as pso
    from paper_2009_03816_amd import binding, build
    assert pso.pso_ps_source_hash() == build.source_hash()
    assert binding._built_from(build.LIBRARY) == build.source_hash()


def run_in_copy(tmp_path, code, path_override=None):
    env = dict(os.environ, PYTHONPATH=str(tmp_path))
    if path_override is not None:
        env["PATH"] = path_override
    return subprocess.run([sys.executable, "-c", code], cwd=str(tmp_path), env=env,
                          capture_output=True, text=True)


def test_a_changed_source_means_a_rebuild_or_a_clear_error(tmp_path):
    if shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"):
        pytest.skip("hipcc not available")
    # a private copy of the package and the header, with a built library
    shutil.copytree(os.path.join(ROOT, "paper_2009_03816_amd"), tmp_path / "paper_2009_03816_amd",
                    ignore=shutil.ignore_patterns("__pycache__", "*.tmp.*"))
    shutil.copytree(os.path.join(ROOT, "include"), tmp_path / "include")
    probe = ("import paper_2009_03816_amd as p; from paper_2009_03816_amd import build; "
             "print(p.pso_ps_source_hash() == build.source_hash(), p.pso_ps_source_hash())")
    first = run_in_copy(tmp_path, probe)
    assert first.returncode == 0 and first.stdout.split()[0] == "True", first.stderr
    lib = tmp_path / "paper_2009_03816_amd" / "libpso_ps.so"
    built_at = os.path.getmtime(lib)

    # the source changes (a comment is enough): the old library must not be used
    src = tmp_path / "paper_2009_03816_amd" / "csrc" / "pso_ps.hip"
    src.write_text(src.read_text() + "\n// touched\n")

    # ... where the compiler cannot be found: a clear error, no silent use
    import paper_2009_03816_amd.build as real_build
    hidden = run_in_copy(tmp_path, "import paper_2009_03816_amd.build as b; b.hipcc = lambda: "
                                   "(_ for _ in ()).throw(RuntimeError('hipcc not found')); "
                                   "import paper_2009_03816_amd as p; p.pso_ps_source_hash()")
    assert hidden.returncode != 0
    assert "built from other sources" in hidden.stderr and "could not be rebuilt" in hidden.stderr
    assert os.path.getmtime(lib) == built_at

    # ... with the compiler: rebuilt, and the new stamp is the new hash
    second = run_in_copy(tmp_path, probe)
    assert second.returncode == 0 and second.stdout.split()[0] == "True", second.stderr
    assert second.stdout.split()[1] != first.stdout.split()[1]
    assert os.path.getmtime(lib) > built_at
    assert real_build.source_hash() == first.stdout.split()[1]     # the real tree is untouched
