"""Host-side contract of bench.py and of the binding, checked without a GPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_bench_refuses_more_than_one_gpu():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert p.returncode != 0
    assert "one GPU" in p.stderr
    assert p.stdout.strip() == ""


def test_algorithmic_bytes_follow_the_memory_model():
    import bench
    # appendix memory model at G = 128: 2 bits per trit and plane, one fp16 scale per plane and group
    N, K = 4096, 14336
    planes_and_scales = N * K // 2 + 4 * N * (K // 128)
    assert planes_and_scales * 8 == N * K * 4.25
    assert bench.algorithmic_bytes(N, K) == planes_and_scales + 2 * K + 4 * N
    assert bench.algorithmic_bytes(N, K, 16) == planes_and_scales + 16 * (2 * K + 4 * N)


def test_recorded_traffic_comes_from_the_committed_profile(monkeypatch):
    import bench
    import workloads
    profile = os.path.join(ROOT, "profiles", "gemv_items_batch_8b_stack.txt")
    named = [l.split(":")[1].split()[0] for l in open(profile) if l.startswith("kernel_source_hash:")]
    assert len(named) == 1
    # handed out only while the library's sources hash to what the summary names ...
    monkeypatch.setattr(bench, "kernel_source_hash", lambda: named[0])
    r = bench.recorded_traffic("batch", 32)
    assert isinstance(r["traffic"], int) and "not measured by this run" in r["traffic_source"]
    # ... the counters saw within 2 % of the algorithmic bytes of the default workload
    algo = 32 * sum(bench.algorithmic_bytes(*workloads.SHAPES_8B[n]) for n in workloads.LINEAR_ORDER)
    assert 0.98 < r["traffic"] / algo < 1.02
    # any other launch mode or stack depth has no recorded figure, nor has a library whose sources have changed
    assert bench.recorded_traffic("graph", 32)["traffic"] is None
    assert bench.recorded_traffic("batch", 8)["traffic"] is None
    monkeypatch.setattr(bench, "kernel_source_hash", lambda: "0" * 16)
    assert bench.recorded_traffic("batch", 32) == {"traffic": None, "traffic_source": None}


def test_per_config_entries_name_the_binding_roof():
    import bench
    e = bench.roof_entry(10.0, [(4096, 4096)], 16)
    assert e["bound"] == "hbm" and abs(e["frac"] - bench.algorithmic_bytes(4096, 4096, 16) / 10.0 / 1e3 / 8000.0) < 1e-4
    e = bench.roof_entry(1000.0, [(8192, 28672)], 2048)
    assert e["bound"] == "mfma" and abs(e["frac"] - 4.0 * 2048 * 8192 * 28672 / 1000.0 / 1e6 / 2500.0) < 1e-4


def test_product_fails_loudly_without_its_library(tmp_path, monkeypatch):
    """No CPU fallback: with the shared library missing, the first call raises and names the build step."""
    from paper_2509_16989_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "libptqtp.so"))
    with pytest.raises(ImportError, match="no CPU fallback"):
        binding.ptqtp_version()


def _sources(*dirs, exts=(".py", ".hip", ".hpp", ".h", ".c")):
    for d in dirs:
        base = os.path.join(ROOT, d)
        if os.path.isfile(base):
            yield base
            continue
        for dirpath, _, files in os.walk(base):
            for f in files:
                if f.endswith(exts):
                    yield os.path.join(dirpath, f)


def test_product_and_oracle_do_not_know_each_other():
    """The HIP path and the CPU oracle share no code: neither names the other, and only tests, the smoke check and
    the benchmark's CPU leg import the oracle."""
    for path in _sources("paper_2509_16989_amd", "include"):
        assert "oracle" not in open(path).read().lower(), path
    for path in _sources("oracle"):
        text = open(path).read()
        assert "paper_2509_16989_amd" not in text and "libptqtp.so" not in text, path
    for path in _sources("workloads"):
        text = open(path).read()
        assert "import oracle" not in text and "paper_2509_16989_amd" not in text, path


def test_nothing_committed_reaches_into_the_scratch_folder():
    for path in _sources("paper_2509_16989_amd", "include", "oracle", "workloads", "tests", "bench.py",
                         "__graft_entry__.py"):
        if os.path.abspath(path) == os.path.abspath(__file__):
            continue
        assert "_work/" not in open(path).read(), path
