"""Host-side checks of bench.py's contract that need no GPU: more than one GPU is refused with a message, and
without a GPU the script says so instead of falling back to anything."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    env = dict(os.environ, HIP_VISIBLE_DEVICES="", CUDA_VISIBLE_DEVICES="")      # no GPU for this process
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, env=env,
                          timeout=300)


def test_more_than_one_gpu_is_refused():
    res = _run("--gpus", "2")
    assert res.returncode != 0
    assert "one GPU" in res.stderr and res.stdout.strip() == ""


def test_no_gpu_is_an_error_not_a_fallback():
    res = _run("--steps", "1", "--warmup", "0")
    assert res.returncode != 0
    assert "no GPU" in res.stderr and res.stdout.strip() == ""


def test_measured_traffic_table_belongs_to_the_current_kernels():
    """`roofline.traffic` comes from a table of counter readings keyed by a hash of the scoring kernels' sources;
    a table older than the sources would make bench.py report null.  Every workload of the default run, and the
    two with the paper's scorer shape, must have a current entry whose profile file exists."""
    sys.path.insert(0, ROOT)
    import bench
    from paper_2605_06676_amd import workloads as W

    for cid in (1, 2, 3, 4, 5, 6):
        w = W.CONFIGS[cid]
        kernel = "score_linear_kernel" if w.scorer == "linear" else ("score_mlp_kernel" if w.hidden <= 64 else "score_mlp_wide_kernel")
        nbytes, profile = bench.measured_traffic(w.name, kernel)
        assert nbytes is not None, f"{w.name}: the traffic table was measured on other sources of {kernel}"
        assert os.path.exists(os.path.join(ROOT, profile)), profile
        algorithmic = sum(W.seq_lengths(w)) * w.L * w.H * 516
        assert 0.99 * algorithmic <= nbytes <= 1.06 * algorithmic, (w.name, nbytes, algorithmic)
