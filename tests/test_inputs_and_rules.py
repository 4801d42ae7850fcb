"""CPU tests of the seeded input generators, of bench.py's command line guard and of the rule that the product
package stands on its own (it never imports the oracle, and it fails loudly without its shared library)."""
from __future__ import annotations

import ast
import pathlib
import subprocess
import sys

import numpy as np
import pytest

import synth_inputs as si

ROOT = pathlib.Path(__file__).resolve().parent.parent


# ---- input generators -------------------------------------------------------------------------------------------

def test_workload_table_matches_the_benchmark_configurations():
    shapes = {n: (w.M, w.K, w.N, w.density) for n, w in si.WORKLOADS.items()}
    assert shapes["C1"] == (64, 512, 512, 0.5)
    assert shapes["C2"] == (256, 4096, 4096, 0.5)
    assert shapes["C3a"] == (256, 4096, 4096, 0.25) and shapes["C3b"] == (256, 4096, 4096, 0.125)
    assert shapes["C4-1"] == (1, 4096, 11008, 0.5) and shapes["C4-8"] == (8, 4096, 11008, 0.5)
    assert shapes["C5a"] == (4096, 8192, 8192, 0.5) and shapes["C5b"][3] == 0.25 and shapes["C5c"][3] == 0.0625


def test_inputs_are_reproducible_and_typed():
    a = si.make_inputs(5, 300, 70, 0.25, "normal", seed=42)
    b = si.make_inputs(5, 300, 70, 0.25, "normal", seed=42)
    c = si.make_inputs(5, 300, 70, 0.25, "normal", seed=43)
    for x, y in zip(a, b):
        assert x.dtype == y.dtype and np.array_equal(x, y)
    assert not np.array_equal(a[0], c[0])
    W, X, bias = a
    assert W.dtype == np.int8 and W.shape == (300, 70) and W.flags["C_CONTIGUOUS"]
    assert X.dtype == np.float32 and X.shape == (5, 300) and bias.dtype == np.float32 and bias.shape == (70,)
    assert set(np.unique(W)) <= {-1, 0, 1}


@pytest.mark.parametrize("density", [0.5, 0.25, 0.0625])
def test_ternary_draw_has_the_asked_density_and_balanced_signs(density):
    rng = np.random.Generator(np.random.PCG64(7))
    W = si.draw_ternary(rng, 2048, 512, density)
    n = W.size
    pos, neg = np.count_nonzero(W == 1), np.count_nonzero(W == -1)
    # binomial: standard deviation of a count is sqrt(n p (1 - p)); six of them is far outside chance
    for count in (pos, neg):
        p = density / 2
        assert abs(count - n * p) < 6 * np.sqrt(n * p * (1 - p))
    # per-column counts of one sign follow Binomial(K, d/2): compare mean and spread
    col = np.count_nonzero(W == 1, axis=0)
    assert abs(col.mean() - 2048 * density / 2) < 6 * np.sqrt(2048 * density / 2 / 512)


def test_ternary_draw_extremes():
    rng = np.random.Generator(np.random.PCG64(1))
    assert not si.draw_ternary(rng, 33, 17, 0.0).any()
    assert np.all(si.draw_ternary(rng, 33, 17, 1.0) != 0)


def test_dense_draw_families():
    rng = np.random.Generator(np.random.PCG64(3))
    u = si.draw_dense(rng, (4000,), "uniform")
    assert u.dtype == np.float32 and u.min() >= -1.0 and u.max() < 1.0 and abs(u.mean()) < 0.05
    g = si.draw_dense(rng, (4000,), "normal")
    assert g.dtype == np.float32 and abs(g.std() - 1.0) < 0.1
    i = si.draw_dense(rng, (4000,), "int8")
    assert i.dtype == np.float32 and np.array_equal(i, np.round(i)) and i.min() >= -8 and i.max() <= 8
    with pytest.raises(ValueError):
        si.draw_dense(rng, (3,), "cauchy")


def test_ad_hoc_workload_names():
    w = si.workload("M64-K16384-N4096-d0.5")
    assert (w.M, w.K, w.N, w.density, w.dist) == (64, 16384, 4096, 0.5, "uniform")
    assert si.workload("M64-K16384-N4096-d0.5").seed == w.seed                  # the seed is a function of the name
    assert si.workload("M32-K16384-N4096-d0.5").seed != w.seed
    for bad in ("C9", "M0-K4-N4-d0.5", "M4-K4-N4-d1.5", "M4-K4", "Mx-K4-N4-d0.5"):
        with pytest.raises(KeyError):
            si.workload(bad)


def test_make_workload_overrides():
    W, X, b = si.make_workload("C1", dist="int8", M=3)
    assert X.shape == (3, 512) and W.shape == (512, 512) and np.array_equal(X, np.round(X))
    W2, _, _ = si.make_workload("C1")
    assert np.array_equal(W, W2)   # W is drawn first, so it does not depend on the overrides


def test_input_module_holds_no_arithmetic_of_the_method():
    tree = ast.parse((ROOT / "synth_inputs.py").read_text())
    imported = {a.name.split(".")[0] for n in ast.walk(tree) if isinstance(n, ast.Import) for a in n.names}
    imported |= {n.module.split(".")[0] for n in ast.walk(tree) if isinstance(n, ast.ImportFrom) and n.module}
    assert imported <= {"__future__", "dataclasses", "numpy"}


# ---- the product stands on its own -------------------------------------------------------------------------------

def _imports(path: pathlib.Path):
    tree = ast.parse(path.read_text())
    for node in ast.walk(tree):
        if isinstance(node, ast.Import):
            for a in node.names:
                yield a.name
        elif isinstance(node, ast.ImportFrom) and node.module:
            yield node.module


def test_product_package_never_imports_the_oracle():
    for path in (ROOT / "paper_2510_06957_amd").glob("*.py"):
        for name in _imports(path):
            assert name.split(".")[0] != "oracle", f"{path.name} imports {name}"
    for path in (ROOT / "paper_2510_06957_amd" / "csrc").iterdir():
        assert "oracle" not in path.read_text().lower().replace("oracle's", ""), f"{path.name} mentions the oracle"


def test_oracle_never_imports_the_product():
    for path in (ROOT / "oracle").glob("*.py"):
        for name in _imports(path):
            assert name.split(".")[0] != "paper_2510_06957_amd", f"{path.name} imports {name}"
    for path in (ROOT / "oracle").glob("*.c"):
        assert "tstgemm.h" not in path.read_text(), f"{path.name} includes the product's header"


def test_importing_the_product_does_not_load_the_oracle():
    code = "import sys; sys.path.insert(0, %r); import paper_2510_06957_amd; print('oracle' in sys.modules)" % str(ROOT)
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stderr
    assert out.stdout.strip().splitlines()[-1] == "False"


def test_missing_library_is_an_error_not_a_fallback():
    code = (
        "import sys, pathlib; sys.path.insert(0, %r)\n"
        "from paper_2510_06957_amd import binding\n"
        "binding._LIB_PATH = pathlib.Path('/nonexistent/libtstgemm.so'); binding._lib = None\n"
        "try:\n"
        "    binding.tcsc_strerror(0)\n"
        "except RuntimeError as e:\n"
        "    print('raised', 'no fallback' in str(e))\n"
        "else:\n"
        "    print('returned')\n" % str(ROOT))
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stderr
    assert out.stdout.strip().splitlines()[-1] == "raised True"


# ---- bench.py ------------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("argv,env", [(["--gpus", "2"], {}), (["--gpus", "8"], {}), ([], {"WORLD_SIZE": "2"})])
def test_bench_refuses_more_than_one_gpu(argv, env):
    import os
    out = subprocess.run([sys.executable, str(ROOT / "bench.py"), *argv], capture_output=True, text=True, timeout=120,
                         env={**os.environ, **env})
    assert out.returncode != 0
    assert "ONE GPU" in out.stderr and out.stdout.strip() == ""


def test_bench_traffic_table_names_real_workloads():
    """Every entry of bench.py's table of counter-measured HBM traffic names a real workload and a tracked summary."""
    tree = ast.parse((ROOT / "bench.py").read_text())
    consts = {n.targets[0].id: ast.literal_eval(n.value) for n in tree.body
              if isinstance(n, ast.Assign) and isinstance(n.value, ast.Constant) and isinstance(n.value.value, str)}
    table = next(n for n in tree.body if isinstance(n, ast.Assign) and getattr(n.targets[0], "id", "") == "MEASURED_TRAFFIC")
    for key, value in zip(table.value.keys, table.value.values):
        name, variant = ast.literal_eval(key)
        nbytes, source = value.elts
        source = consts[source.id] if isinstance(source, ast.Name) else ast.literal_eval(source)
        si.workload(name)
        assert variant in ("tcsc", "signed", "packed") and ast.literal_eval(nbytes) > 0
        assert (ROOT / source).is_file(), source
