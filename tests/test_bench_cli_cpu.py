"""bench.py's command line on a machine without a GPU: the single-GPU contract and the options."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args, env=None):
    e = dict(os.environ)
    e.update(env or {})
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, env=e,
                          capture_output=True, text=True, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run("--gpus", "2")
    assert r.returncode != 0 and "one GPU" in r.stderr
    r = run(env={"WORLD_SIZE": "4"})
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_help_lists_the_workload_and_measurement_options():
    r = run("--help")
    assert r.returncode == 0
    for opt in ("--gpus", "--steps", "--warmup", "--workload", "--tokens", "--ffn-split", "--ep-sim",
                "--predictor-accuracy", "--no-cpu-baseline"):
        assert opt in r.stdout


def test_hbm_traffic_is_reported_only_for_the_kernel_source_it_was_measured_with(tmp_path, monkeypatch):
    """roofline.traffic comes from a profiles/ summary that names the workload, the entry point and
    the SHA-256 of csrc/ffn.hip it was taken with; anything else gives None, never a stale figure."""
    import hashlib
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    src = os.path.join(ROOT, "paper_2603_06350_amd", "csrc", "ffn.hip")
    sha = hashlib.sha256(open(src, "rb").read()).hexdigest()
    prof = tmp_path / "profiles"
    prof.mkdir()
    pkg = tmp_path / "paper_2603_06350_amd" / "csrc"
    pkg.mkdir(parents=True)
    (pkg / "ffn.hip").write_bytes(open(src, "rb").read())
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))

    def write(sha256, entry="moe_grouped_ffn_gather", workload="mixtral"):
        (prof / "mixtral_ffn_up_hbm_traffic.md").write_text(
            f"# text\n\nworkload: {workload}\nentry_point: {entry}\nffn_hip_sha256: {sha256}\n"
            "hbm_read_bytes: 2800000000\nhbm_written_bytes: 235000000\n")

    write(sha)
    got = bench.measured_hbm_traffic("mixtral", "moe_grouped_ffn_gather")
    assert got["read_bytes"] == 2.8e9 and got["written_bytes"] == 2.35e8
    assert bench.measured_hbm_traffic("mixtral", "moe_grouped_ffn") is None          # another entry point
    assert bench.measured_hbm_traffic("phi", "moe_grouped_ffn_gather") is None       # no summary
    write("0" * 64)
    assert bench.measured_hbm_traffic("mixtral", "moe_grouped_ffn_gather") is None   # another kernel source
    write(sha, workload="phi")
    assert bench.measured_hbm_traffic("mixtral", "moe_grouped_ffn_gather") is None


def test_committed_traffic_summary_parses(repo_root=ROOT):
    path = os.path.join(ROOT, "profiles", "mixtral_ffn_up_hbm_traffic.md")
    if not os.path.exists(path):
        return
    import re
    fields = dict(re.findall(r"^([a-z_0-9]+):\s*(\S+)\s*$", open(path).read(), flags=re.M))
    for key in ("workload", "entry_point", "ffn_hip_sha256", "hbm_read_bytes", "hbm_written_bytes"):
        assert key in fields
    assert len(fields["ffn_hip_sha256"]) == 64 and float(fields["hbm_read_bytes"]) > 1e9


def test_achievable_peaks_takes_the_best_matching_line_of_each_micro_benchmark(tmp_path, monkeypatch):
    """roofline.achievable_peak parses the micro-benchmarks' own output lines: the best 16x16x32 MFMA
    rate, the contiguous HBM stream, the buffer_load L2 -> LDS stream; a program that is not built
    gives None, not a made-up figure."""
    import importlib.util
    import types
    spec = importlib.util.spec_from_file_location("bench_under_test_peaks", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    mb = tmp_path / "paper_2603_06350_amd" / "csrc" / "microbench"
    mb.mkdir(parents=True)
    (mb / "mfma_rate.exe").write_text("")
    (mb / "hbm_read_stream.exe").write_text("")
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    outputs = {
        "mfma_rate.exe": "32x32x16 agpr acc, no barrier   waves/SIMD=2: 6.156 ms 2744 TFLOP/s\n"
                         "16x16x32 vgpr acc, no barrier   waves/SIMD=1: 2.913 ms 1843 TFLOP/s\n"
                         "16x16x32 vgpr acc, no barrier   waves/SIMD=2: 5.483 ms 1958 TFLOP/s\n",
        "hbm_read_stream.exe": "contiguous, 4096 blocks x 256 threads        0.684 ms  6.28 TB/s\n"
                               "packed stages, 2 stages in flight            0.685 ms  7.27 TB/s\n",
    }
    import subprocess as sp
    monkeypatch.setattr(sp, "run", lambda cmd, **kw: types.SimpleNamespace(stdout=outputs[os.path.basename(cmd[0])]))
    got = bench.achievable_peaks()
    assert got["mfma_bf16_16x16x32_tflops"] == 1958.0
    assert abs(got["mfma_frac_of_published_peak"] - 1958.0 / 2500.0) < 1e-12
    assert got["hbm_read_stream_gbs"] == 6280.0
    assert got["l2_to_lds_operand_stream_gbs"] is None
