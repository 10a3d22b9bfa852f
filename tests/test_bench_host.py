"""Host-side checks of bench.py: the GPU-count guard and the rule for quoting measured HBM traffic."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr


def test_traffic_is_quoted_only_from_a_summary_of_the_same_kernel_source(monkeypatch, tmp_path):
    import bench
    from paper_2312_00839_amd import profile_summary
    sha = profile_summary.kernel_source_sha256()
    pdir = tmp_path / "profiles"
    pdir.mkdir()
    (pdir / "a.txt").write_text(
        "traffic_bytes_per_launch variant=fused-config5-x bytes=123\nkernel_source_sha256: %s\n"
        "traffic_bytes_per_launch variant=fused-config4-x bytes=77\nkernel_source_sha256: %s\n" % (sha, "0" * 64))
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    value, source = bench.measured_traffic("fused-config5-x")
    assert value == 123 and "a.txt" in source
    value, source = bench.measured_traffic("fused-config4-x")            # taken from other kernel code: never quoted
    assert value is None and "other kernel source" in source
    value, source = bench.measured_traffic("predict-config5-x")          # not covered at all
    assert value is None and "no rocprofv3 counter summary" in source


def test_tracked_summaries_cover_the_headline_variants():
    # the summaries under profiles/ name the variants bench.py asks for by default (whether they are still current
    # is decided at run time by the fingerprint)
    text = "".join(open(os.path.join(ROOT, "profiles", f)).read() for f in os.listdir(os.path.join(ROOT, "profiles")))
    for v in ("fused-config5-adamw-local-gf32-hbf16", "fused-config5-adamw-packed-gf32-hbf16",
              "fused-config5-adamw-learnt-gf32-hbf16"):
        assert "traffic_bytes_per_launch variant=%s " % v in text
