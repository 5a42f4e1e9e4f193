"""Host-only checks of the C ABI: the built library loads, exports every function the header
declares, and the pure-host entry points behave.  No GPU compute is called here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", "rgc.h"), os.path.join(ROOT, "include", "rgc_diag.h")]


@pytest.fixture(scope="module")
def lib():
    from paper_1808_04357_amd import binding, build
    if not os.path.exists(binding.library_path()):
        build.build(force=True)
    return binding.load_library()


def declared_functions():
    text = "".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rgc_[a-z_0-9]+)\s*\(", text)))


def test_header_functions_are_exported(lib):
    names = declared_functions()
    assert {"rgc_create", "rgc_destroy", "rgc_k_for_density", "rgc_compress_layers",
            "rgc_decompress_accumulate", "rgc_strerror"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name + " is declared in include/*.h but not exported"
    from paper_1808_04357_amd import binding
    assert sorted(binding.EXPORTS) == names


def test_k_for_density_matches_oracle_rule(lib, oracle):
    for n in (0, 1, 2, 999, 1000, 1001, 1 << 20, 25088 * 4096, (1 << 31) - 1):
        for ppm in (1, 1000, 4000, 250_000, 1_000_000):
            want = oracle.k_for_density(n, ppm) if n >= 1 else 0
            assert lib.rgc_k_for_density(n, ppm) == want, (n, ppm)
    assert lib.rgc_k_for_density(1 << 20, 1000) == 1049


def test_status_texts(lib):
    assert lib.rgc_strerror(0) == b"ok"
    for s in (-1, -2, -3, -4, -99):
        assert len(lib.rgc_strerror(s)) > 0


def test_null_arguments_are_rejected_before_any_gpu_call(lib):
    assert lib.rgc_create(None, 0, 100, 1) == -1
    h = ctypes.c_void_p(0)
    assert lib.rgc_create(ctypes.byref(h), 0, 0, 1) == -1
    assert lib.rgc_create(ctypes.byref(h), 0, 100, 0) == -1
    assert lib.rgc_create(ctypes.byref(h), -1, 100, 1) == -1
    assert lib.rgc_destroy(None) == -1
    assert lib.rgc_compress_layers(None, None, 1, 0.0, 0, None) == -1
    assert lib.rgc_decompress_accumulate(None, None, 0, 1, None, None, 1.0, 0x10, None) == -1
    assert lib.rgc_reset_hints(None) == -1
    assert lib.rgc_poison_hints(None, 0, None) == -1
    assert lib.rgc_selftest(None, None) == -1
    assert lib.rgc_last_error(None, None) == -1
    assert lib.rgc_message_means_noalloc(None, None, None, 1, None, None) == -1


def test_struct_layout_matches_header():
    from paper_1808_04357_amd import binding
    assert ctypes.sizeof(binding.rgc_layer) == 64
    assert binding.rgc_layer.n.offset == 24 and binding.rgc_layer.k.offset == 32
    assert binding.rgc_layer.out_idx.offset == 40 and binding.rgc_layer.out_count.offset == 56
    assert ctypes.sizeof(binding.rgc_msg) == 24 and binding.rgc_msg.count.offset == 16


def test_product_reads_no_environment_switches():
    """Nothing in the library or its binding is steered by environment variables (the build script's extra-flags
    hook is a build-time matter and lives in build.py alone)."""
    pkg = os.path.join(ROOT, "paper_1808_04357_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".cpp", ".hip", ".h")) or f in ("binding.py", "__init__.py", "synth.py"):
                src = open(os.path.join(dirpath, f)).read()
                assert "getenv" not in src and "os.environ" not in src, f


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_1808_04357_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in src and "from oracle" not in src, f
                assert "rgc_oracle" not in src, f


def test_bench_refuses_more_than_one_gpu():
    """This build has no collectives: the benchmark says so instead of running a second rank."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_hbm_traffic_figures_are_stamped_with_the_current_kernel_sources():
    """roofline.traffic comes from counter runs that cannot share a process with the timed run; the committed
    figures carry the digest of the kernel sources they were taken with, and the benchmark drops them when the
    sources have changed since.  This checks that the committed pair is in step."""
    import json
    import sys
    sys.path.insert(0, ROOT)
    import bench
    with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
        t = json.load(f)
    assert t["kernel_source_sha256"] == bench.kernel_source_digest()
    assert 0 < t["fetch_bytes_per_launch"] < 4e9 and 0 < t["write_bytes_per_launch"] < 4e9
