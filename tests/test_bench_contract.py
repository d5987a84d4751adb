"""bench.py's command-line contract that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, timeout=120)
    assert res.returncode != 0
    assert "one GPU" in res.stderr
    assert res.stdout.strip() == ""          # no JSON line for a run that did not happen


def test_help_lists_the_driver_flags():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--help"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode == 0
    for flag in ("--gpus", "--steps", "--warmup", "--workload"):
        assert flag in res.stdout


def test_overlap_fraction_of_copy_spans():
    """The pipeline workload's headline figure: share of copy time during which some GEMM span runs."""
    from bench_pipeline import overlap_fraction
    # (kind, layer, start, end) with kind 0 = copy, 1 = GEMM; GEMM spans may overlap each other
    spans = [(0, 0, 0.0, 10.0), (1, 0, 2.0, 4.0), (1, 0, 3.0, 6.0), (1, 1, 9.0, 20.0), (0, 1, 30.0, 32.0)]
    frac, total = overlap_fraction(spans)
    # copy 0..10 meets the merged GEMM intervals [2,6] for 4 and [9,20] for 1; copy 30..32 meets none
    assert total == 12.0
    assert abs(frac - 5.0 / 12.0) < 1e-12
    assert overlap_fraction([]) == (0.0, 0.0)
    assert overlap_fraction([(0, 0, 1.0, 2.0), (1, 0, 0.0, 5.0)])[0] == 1.0


def test_hidden_fraction_of_the_copy():
    """Exposed copy time = layer time with the prefetch minus layer time without; hidden share
    relative to the copy's stand-alone time (paper Section 3: T = max(T_compute, T_prefetch))."""
    from bench_pipeline import hidden_fraction
    assert hidden_fraction(4.7, 1.4, 3.3) == (4.7 - 1.4, 0.0)               # compute + copy: nothing hidden
    ex, hid = hidden_fraction(3.3, 1.4, 3.3)                                 # max(compute, copy), copy longer
    assert abs(ex - 1.9) < 1e-12 and abs(hid - (1 - 1.9 / 3.3)) < 1e-12
    assert hidden_fraction(5.0, 5.0, 3.0) == (0.0, 1.0)                      # compute longer, copy fully hidden
    assert hidden_fraction(4.9, 5.0, 3.0) == (0.0, 1.0)                      # timing noise does not go negative


def test_profiled_traffic_is_tied_to_the_kernel_source(tmp_path, monkeypatch):
    import hashlib
    import bench
    src = os.path.join(ROOT, "paper_2604_01621_amd", "csrc", "gemm_stream.hip")
    digest = hashlib.sha256(open(src, "rb").read()).hexdigest()
    prof = tmp_path / "profiles"
    prof.mkdir()
    (tmp_path / "paper_2604_01621_amd" / "csrc").mkdir(parents=True)
    (tmp_path / "paper_2604_01621_amd" / "csrc" / "gemm_stream.hip").write_bytes(open(src, "rb").read())
    (prof / "x.md").write_text("text\nbench-traffic: workload=decode seed=1 T=64 source=gemm_stream.hip "
                               f"sha256={digest} bytes_per_launch=123456\n"
                               "bench-traffic: workload=decode seed=2 T=64 source=gemm_stream.hip "
                               "sha256=00ff bytes_per_launch=9\n")
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    assert bench.profiled_traffic("decode", 1, 64, "gemm_stream.hip") == 123456
    assert bench.profiled_traffic("decode", 2, 64, "gemm_stream.hip") is None     # hash of another source
    assert bench.profiled_traffic("prefill", 1, 64, "gemm_stream.hip") is None
    assert bench.profiled_traffic("decode", 1, 64, "missing.hip") is None
