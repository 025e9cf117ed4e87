"""The C-ABI library loads and exports every function include/vf.h declares
(no compute calls: this runs without a GPU)."""
import os
import re

import pytest


def declared_functions():
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    text = open(os.path.join(root, "include", "vf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vf_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_2011_14486_amd as pkg
    from paper_2011_14486_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2011_14486_amd.build import build_lib
        build_lib()
    b = pkg.load()
    names = declared_functions()
    assert len(names) >= 20 and {"vf_enumerate", "vf_featurize", "vf_score", "vf_argmin_step",
                                 "vf_greedy_schedule"} <= set(names)
    for n in names:
        assert hasattr(b.lib(), n), f"{n} is declared in vf.h but not exported"
        assert hasattr(b, n) or n in ("vf_strerror", "vf_last_hip_error"), f"binding lacks {n}"
    assert sorted(binding.EXPORTS) == names
    assert b.lib().vf_strerror(0) == b"ok" and b.lib().vf_strerror(-1) == b"invalid argument"


def test_missing_library_fails_loudly(monkeypatch):
    from paper_2011_14486_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libvf.so")
    with pytest.raises(ImportError):
        binding.lib()


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits with an error."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)


def test_bench_takes_traffic_only_from_a_summary_of_the_same_sources(tmp_path, monkeypatch):
    """bench.py reports HBM traffic only when the committed counter summary names the hash of the
    kernel sources being timed and the batch; otherwise the field is null."""
    import bench
    sha = bench.kernel_sources_sha256()
    f = tmp_path / "counters.txt"
    monkeypatch.setattr(bench, "HBM_PROFILE", str(f))
    assert bench.measured_traffic("k_whole", 256) is None                     # no summary at all
    f.write_text(f"# csrc_sha256: {sha}\n# batch: 256\n# traffic_bytes_per_launch k_whole: 12345\n")
    assert bench.measured_traffic("k_whole", 256) == 12345
    assert bench.measured_traffic("k_whole", 128) is None                     # another batch
    assert bench.measured_traffic("k_featurize", 256) is None                 # a kernel the summary does not cover
    f.write_text(f"# csrc_sha256: {'0' * 64}\n# batch: 256\n# traffic_bytes_per_launch k_whole: 12345\n")
    assert bench.measured_traffic("k_whole", 256) is None                     # other kernel sources
