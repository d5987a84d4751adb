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
    from paper_2604_01621_amd.pipeline_bench import overlap_fraction
    # (kind, layer, start, end) with kind 0 = copy, 1 = GEMM; GEMM spans may overlap each other
    spans = [(0, 0, 0.0, 10.0), (1, 0, 2.0, 4.0), (1, 0, 3.0, 6.0), (1, 1, 9.0, 20.0), (0, 1, 30.0, 32.0)]
    frac, total = overlap_fraction(spans)
    # copy 0..10 meets the merged GEMM intervals [2,6] for 4 and [9,20] for 1; copy 30..32 meets none
    assert total == 12.0
    assert abs(frac - 5.0 / 12.0) < 1e-12
    assert overlap_fraction([]) == (0.0, 0.0)
    assert overlap_fraction([(0, 0, 1.0, 2.0), (1, 0, 0.0, 5.0)])[0] == 1.0
