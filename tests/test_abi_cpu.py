"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and rejects bad arguments before any launch."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_1609_08326_amd import binding, build
    if build.is_stale():
        build.build_library(force=True)
    return binding.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "dcasgd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dcasgd_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound(lib):
    from paper_1609_08326_amd import binding
    names = declared_symbols()
    assert "dcasgd_create" in names and "dcasgd_push_batch" in names and len(names) >= 12
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding._PROTOTYPES) == names


def test_create_validates_without_touching_a_gpu(lib):
    from paper_1609_08326_amd import binding as B
    ok = lib.dcasgd_create(100, 4, 0.1, 2.0, B.MODE_A | B.PULL_ON_PUSH, 0.95, 1e-7)
    assert ok
    assert lib.dcasgd_step(ok) == 0
    # not bound yet: every state-changing call is refused
    assert lib.dcasgd_init(ok, None) == B.ESTATE
    assert lib.dcasgd_push(ok, 0, None, None) == B.ESTATE
    assert lib.dcasgd_sync_fold_ordered_static(ok, None, 1, 0.1, None) == B.ESTATE
    assert lib.dcasgd_sync_fold_ordered_static(None, None, 1, 0.1, None) == B.EINVAL
    assert lib.dcasgd_set_launch(ok, 0, 0, 0, 3) == B.OK and lib.dcasgd_set_launch(ok, 0, 0, 0, 4) == B.EINVAL
    assert not lib.dcasgd_pull(ok, 0)
    assert lib.dcasgd_last_error(ok) == B.ESTATE
    assert lib.dcasgd_bind(ok, None, None, 100, None) == B.EINVAL
    assert lib.dcasgd_bind(ok, 16, 4096, 96, 8192) == B.EINVAL        # stride < d
    assert lib.dcasgd_bind(ok, 20, 4096, 100, 8192) == B.EALIGN       # w not 16-byte aligned
    assert lib.dcasgd_bind(ok, 16, 4096, 102, 8192) == B.EALIGN       # stride not a multiple of 4
    assert lib.dcasgd_bind(ok, 4096, 4096, 100, 81920) == B.EINVAL    # w overlaps bak
    assert lib.dcasgd_set_launch(ok, 100, 0, 0, 1) == B.EINVAL
    assert lib.dcasgd_set_launch(ok, 1024, 0, 0, 1) == B.EINVAL
    assert lib.dcasgd_set_launch(ok, 256, 3, 0, 1) == B.EINVAL
    assert lib.dcasgd_set_launch(ok, 256, 4, -1, 1) == B.EINVAL
    assert lib.dcasgd_set_launch(ok, 256, 4, 0, 1) == B.OK
    assert lib.dcasgd_destroy(ok) == B.OK
    for bad in [(0, 4, 0.1, 2.0, B.MODE_A, 0.9, 1e-7), (10, 0, 0.1, 2.0, B.MODE_A, 0.9, 1e-7),
                (10, 4, 0.1, 2.0, 7, 0.9, 1e-7), (10, 4, 0.1, 2.0, B.MODE_A, 1.0, 1e-7),
                (10, 4, 0.1, 2.0, B.MODE_A, -0.1, 1e-7), (10, 4, float("nan"), 2.0, B.MODE_C, 0, 0),
                (10, 4, 0.1, 2.0, B.MODE_A, 0.9, -1.0), (10, 4, 0.1, 2.0, B.MODE_A | (1 << 8), 0.9, 0)]:
        assert not lib.dcasgd_create(*bad), bad
    assert lib.dcasgd_destroy(None) == B.EINVAL
    assert lib.dcasgd_strerror(B.EALIGN).decode().startswith("pointer")


def test_synth_grad_validates_without_touching_a_gpu(lib):
    from paper_1609_08326_amd import binding as B
    assert lib.dcasgd_synth_grad(None, 16, 32, 0.1, 1, 0, 48, 0, 4, None, 0, 0) == B.EINVAL
    assert lib.dcasgd_synth_grad(16, 4096, 8192, 0.1, 1, 0, 12288, 0, 0, None, 0, 0) == B.EINVAL
    assert lib.dcasgd_synth_grad(20, 4096, 8192, 0.1, 1, 0, 12288, 0, 8, None, 0, 0) == B.EALIGN
    assert lib.dcasgd_synth_grad(16, 4096, 8192, 0.1, 1, 0, 16, 0, 8, None, 0, 0) == B.EINVAL
    assert lib.dcasgd_synth_grad(16, 4096, 8192, 0.1, 1, 0, 12288, 0, 8, None, 96, 1) == B.EINVAL


def test_workloads_are_deterministic_and_shaped():
    from paper_1609_08326_amd import workloads as W
    assert [c.d for c in W.CONFIGS] == [272474, 272474, 25557032, 25557032, 138357544]
    assert [c.M for c in W.CONFIGS] == [4, 8, 16, 16, 32]
    assert [c.T for c in W.CONFIGS] == [2000, 4000, 200, 320, 64]
    c0 = W.CONFIGS[0]
    assert list(c0.arrivals()[:6]) == [0, 1, 2, 3, 0, 1]
    c1 = W.CONFIGS[1]
    a, b = c1.arrivals(), c1.arrivals()
    assert (a == b).all() and a.min() == 0 and a.max() == c1.M - 1
    h = c1.hdiag()
    assert h.dtype.name == "float32" and h.min() >= 1e-3 * 0.999 and h.max() <= 1.0
    assert abs(float(c1.wstar().std()) - 1.0) < 0.01
    c3 = W.CONFIGS[3].replace(d=16)
    q = c3.arrivals().reshape(-1, 16)
    assert all(sorted(r) == list(range(16)) for r in q.tolist())
    idx = W.CONFIGS[2].sample_indices(1000, edge=64)
    assert idx[0] == 0 and idx[-1] == W.CONFIGS[2].d - 1 and (idx[1:] > idx[:-1]).all()


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    """There is no fallback path: without the built library the binding raises."""
    from paper_1609_08326_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libdcasgd.so"))
    with pytest.raises(FileNotFoundError):
        binding.load()
    with pytest.raises(FileNotFoundError):
        binding.strerror(0)


def test_product_path_does_not_import_the_oracle():
    """The oracle is test infrastructure; nothing under the package may reach for it."""
    pkg = os.path.join(ROOT, "paper_1609_08326_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "dcasgd_oracle" not in text, f


def test_header_is_plain_c_and_binding_matches_its_arity(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 on its own, and every
    ctypes prototype must take as many arguments as the declaration it mirrors."""
    import subprocess
    from paper_1609_08326_amd import binding
    src = tmp_path / "use_header.c"
    src.write_text('#include "dcasgd.h"\n'
                   "int main(void) { return DCASGD_MAX_K == 16 && DCASGD_FOLD_WS_BYTES > 0 ? 0 : 1; }\n")
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only",
                           "-I", os.path.join(ROOT, "include"), str(src)])
    text = open(os.path.join(ROOT, "include", "dcasgd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    seen = 0
    for name, args in re.findall(r"\b(dcasgd_[a-z_]+)\s*\(([^)]*)\)\s*;", text):
        n = 0 if args.strip() in ("", "void") else args.count(",") + 1
        assert len(binding._PROTOTYPES[name][1]) == n, name
        seen += 1
    assert seen == len(binding._PROTOTYPES)
    assert binding.FOLD_WS_BYTES == int(re.search(r"#define DCASGD_FOLD_WS_BYTES (\d+)", text).group(1))
    assert binding.MAX_K == int(re.search(r"#define DCASGD_MAX_K (\d+)", text).group(1))


def test_without_a_gpu_launching_calls_report_the_runtime_error_and_nothing_becomes_ready(lib):
    """No GPU in the CPU test environment: dcasgd_init must come back with the HIP error
    code (not crash, not pretend), and the handle must then refuse pushes as not ready.
    Skipped where a GPU is present."""
    import ctypes as C
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    from paper_1609_08326_amd import binding as B
    h = lib.dcasgd_create(1000, 2, 0.1, 0.04, B.MODE_C, 0.0, 0.0)
    # host memory stands in for device memory: nothing can be launched here anyway
    buf = (C.c_float * (1024 * 4 + 64))()
    base = (C.addressof(buf) + 255) // 256 * 256
    assert lib.dcasgd_bind(h, base, base + 4096, 1024, None) == B.OK
    assert lib.dcasgd_init(h, None) == B.EHIP
    assert lib.dcasgd_push(h, 0, base + 3 * 4096, None) == B.ESTATE
    assert lib.dcasgd_pull(h, 0) is None
    assert lib.dcasgd_last_error(h) == B.ESTATE
    assert lib.dcasgd_destroy(h) == B.OK
