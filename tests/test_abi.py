"""CPU-only checks of the boundary: the library loads, exports every symbol the header declares,
and the host-side logic that needs no GPU behaves."""
import ctypes as C
import os
import re
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2506_15733_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return binding.load_library()


def header_functions():
    src = open(os.path.join(ROOT, "include", "specs.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(specs_[a-z_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2506_15733_amd import binding
    names = header_functions()
    assert len(names) >= 13
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTED_SYMBOLS) == names


def test_strerror_and_workspace_arithmetic(lib):
    from paper_2506_15733_amd import binding
    assert binding.specs_strerror(0) == "ok"
    assert "workspace" in binding.specs_strerror(7)
    assert binding.specs_strerror(12345) == "unknown status"
    d = binding.make_desc(2, 64, 4, 4, 16, 256, 512, "f32", "lm")
    a = binding.specs_workspace_bytes(d, 64, 1)
    b = binding.specs_workspace_bytes(d, 128, 1)
    assert 0 < a < b and a % 256 == 0
    bad = binding.make_desc(2, 64, 4, 3, 16, 256, 512, "f32", "lm")     # Hq % Hkv != 0
    assert binding.specs_workspace_bytes(bad, 64, 1) == 0
    assert binding.specs_workspace_bytes(d, 0, 1) == 0


def test_null_arguments_are_rejected_without_touching_a_gpu(lib):
    out = C.c_void_p()
    assert lib.specs_ctx_create(0, None, None, 0, C.byref(out)) == 1          # SPECS_EINVAL
    assert lib.specs_score_blocks(None, None, None, None, 1, 1, None, None) == 1
    assert lib.specs_subsample(None, None, None, None, None, 1, 1, None, 1, None, None, None) == 1
    assert lib.specs_prefill(None, None, None, None) == 1
    assert lib.specs_ctx_destroy(None) == 0


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2506_15733_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                txt = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in txt and "from oracle" not in txt, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            txt = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2506_15733_amd" not in txt and "import workload" not in txt


def test_host_side_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The host code of the ABI (argument checks, description checks, workspace carving arithmetic, handle lifetime,
    counters) built with -fsanitize=address,undefined for the host only and driven by tests/host_sanitizer_driver.cpp,
    which needs no GPU: any report of either sanitizer, or a failed check, fails the test. The other objects are the
    ordinary ones of build() (device code is never sanitized)."""
    import glob
    import subprocess
    import __graft_entry__ as G
    objs = [o for o in glob.glob(os.path.join(ROOT, "_build", "*.o")) if not o.endswith("specs_api.o")]
    if len(objs) < 8:
        G.build()
        objs = [o for o in glob.glob(os.path.join(ROOT, "_build", "*.o")) if not o.endswith("specs_api.o")]
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined", "-g"]
    api_o, drv_o, exe = str(tmp_path / "specs_api_san.o"), str(tmp_path / "driver.o"), str(tmp_path / "driver")
    subprocess.run([G.HIPCC, *G.FLAGS, *san, "-c", os.path.join(G.CSRC, "specs_api.hip"), "-o", api_o], check=True,
                   capture_output=True)
    subprocess.run([G.HIPCC, "-x", "hip", *G.FLAGS, *san, "-c", os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"),
                    "-o", drv_o], check=True, capture_output=True)
    subprocess.run([G.HIPCC, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                    "-o", exe, drv_o, api_o, *objs], check=True, capture_output=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:halt_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0 and "host ABI driver: ok" in r.stdout, (r.stdout[-2000:], r.stderr[-4000:])
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-4000:]
