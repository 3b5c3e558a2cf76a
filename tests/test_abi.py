"""The C-ABI library loads, exports every function include/ddef.h declares, and its host-side
scalar pieces (k from delta, DeCo of Algorithm 3, argument checks) behave; no GPU needed."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2507_17346_amd import binding, workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


STATED_K = {("C1", 0.01): 10_000, ("C2", 0.01): 117_000, ("C3", 0.001): 124_000,
            ("C4", 0.1): 130_000_000, ("C4", 0.01): 13_000_000, ("C4", 0.001): 1_300_000}   # as the workloads state them


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ddef.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ddef_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.load()
    names = declared_functions()
    assert "ddef_init" in names and "ddef_ef_compress" in names and len(names) >= 25
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(binding.SIGNATURES) == names          # the binding covers the whole header


def test_error_strings():
    assert binding.strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -5):
        assert binding.strerror(code) not in ("ok", "unknown error")
    assert binding.strerror(-99) == "unknown error"


def test_init_rejects_bad_arguments_before_touching_the_device():
    lib = binding.load()
    h = C.c_void_p(1)
    assert lib.ddef_init(0, 1, 0, C.byref(h)) == binding.EINVAL and not h.value
    assert lib.ddef_init(8, 0, 0, C.byref(h)) == binding.EINVAL
    assert lib.ddef_init(1 << 32, 1, 0, C.byref(h)) == binding.EINVAL
    assert lib.ddef_init(8, 1, 1 << 20, C.byref(h)) == binding.EINVAL
    assert lib.ddef_init(8, 1, 0, None) == binding.EINVAL
    assert lib.ddef_destroy(None) == binding.EINVAL
    assert lib.ddef_grad(None) == binding.EINVAL


def test_k_from_delta_matches_oracle(oracle_mod):
    rng = np.random.default_rng(1)
    for _ in range(2000):
        d = int(10 ** rng.uniform(0, 9.5))
        delta = float(10 ** rng.uniform(-9, 0))
        assert binding.k_from_delta(delta, d) == oracle_mod.k_from_delta(delta, d)
    for name in ("C1", "C2", "C3", "C4"):
        w = workloads.get(name)
        for dl in w.deltas:
            assert binding.k_from_delta(dl, w.d) == STATED_K[(name, dl)]
    assert binding.k_from_delta(0.0, 10) == 0 and binding.k_from_delta(1.5, 10) == 0
    assert binding.k_from_delta(float("nan"), 10) == 0


def test_deco_matches_oracle(oracle_mod):
    rng = np.random.default_rng(2)
    for _ in range(500):
        v_g = 32 * 10 ** rng.uniform(6, 9.2)
        a = 10 ** rng.uniform(8, 10)
        b = rng.uniform(0.01, 0.3)
        t_comp = 10 ** rng.uniform(-2, 0)
        got = binding.deco(v_g, a, b, t_comp)
        want = oracle_mod.deco(v_g, a, b, t_comp)
        assert (got is None) == (want is None)
        if got:
            assert got[0] == want[0] and got[1] == pytest.approx(want[1], rel=1e-12)
    tau, delta = C.c_uint32(), C.c_double()
    lib = binding.load()
    assert lib.ddef_deco(-1.0, 1e9, 0.1, 0.1, C.byref(tau), C.byref(delta)) == binding.EINVAL
    assert lib.ddef_deco(1e9, 1e9, 0.1, 0.0, C.byref(tau), C.byref(delta)) == binding.EINVAL
    assert lib.ddef_deco(1e9, 1e9, 0.1, 0.1, None, C.byref(delta)) == binding.EINVAL


def test_adaptive_schedule_exercises_ring_and_k(oracle_mod):
    # the seeded trace of the adaptive workload yields several distinct (tau, delta) pairs
    w = workloads.get("C5")
    tr = workloads.network_trace(w)
    pairs = []
    for a, b in zip(tr.bandwidth_bps, tr.latency_s):
        tau, delta = binding.deco(tr.v_g_bits, a, b, tr.t_comp_s)
        pairs.append((int(np.clip(tau, *tr.tau_bounds)), float(np.clip(delta, *tr.delta_bounds))))
    assert len(pairs) == 10
    assert len({p[0] for p in pairs}) >= 4
    assert max(p[1] for p in pairs) / min(p[1] for p in pairs) > 5


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 (no C++ in it), and a C program
    that names every declared function must link against the built library."""
    import shutil
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    header = os.path.join(root, "include", "ddef.h")
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    subprocess.check_call([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", header])
    names = declared_functions()
    src = tmp_path / "use_all.c"
    src.write_text('#include "ddef.h"\n#include <stdio.h>\nint main(void) {\n  const void* p[] = {\n'
                   + "".join(f"    (const void*){n},\n" for n in names)
                   + "  };\n  printf(\"%d\\n\", (int)(sizeof p / sizeof p[0]));\n  return 0;\n}\n")
    lib = os.path.join(root, "paper_2507_17346_amd", "libddef.so")
    if not os.path.exists(lib):
        pytest.skip("library not built")
    exe = tmp_path / "use_all"
    subprocess.check_call([gcc, "-std=gnu99", "-I", os.path.join(root, "include"), str(src), lib, "-o", str(exe),
                           "-Wl,-rpath," + os.path.dirname(lib), "-Wl,--allow-shlib-undefined"])


def test_product_path_never_reaches_for_the_oracle():
    """Nothing in the package, nor the bench's timed path, imports the CPU oracle: a missing or
    unloadable library must surface as an error, not as a silent CPU result."""
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg = os.path.join(root, "paper_2507_17346_amd")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            text = open(os.path.join(pkg, name)).read()
            assert not re.search(r"^\s*(import|from)\s+oracle\b", text, re.M), name
    # bench.py touches the oracle in one place only: the cpu_baseline leg
    bench = open(os.path.join(root, "bench.py")).read()
    uses = [m.start() for m in re.finditer(r"^\s*(import|from)\s+oracle\b", bench, re.M)]
    assert len(uses) == 1
    assert bench.rfind("def cpu_baseline", 0, uses[0]) > bench.rfind("\ndef main", 0, uses[0])


def test_a_missing_library_is_an_error(tmp_path, monkeypatch):
    from paper_2507_17346_amd import binding, build
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(build, "LIB", str(tmp_path / "libddef_missing.so"))
    monkeypatch.setattr(build, "build_library", lambda *a, **k: (_ for _ in ()).throw(RuntimeError("no compiler here")))
    with pytest.raises((RuntimeError, OSError)):
        binding.load()
    with pytest.raises((RuntimeError, OSError)):
        binding.k_from_delta(0.5, 10)
