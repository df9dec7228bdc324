"""bench.py's command line, without a GPU: more than one GPU is refused with a message that says why, and the
traffic summary it reports from is read for the default workload's GEMM kernels."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)


def test_traffic_summary_has_the_default_workloads_kernels():
    sys.path.insert(0, ROOT)
    import bench
    for kernel in ("gemm_bf16_fwd_dma_256", "gemm_bf16_dw_dense_dma_256", "gemm_bf16_dx_dma_256"):
        t = bench.measured_traffic("mlp4096_bf16", "per_example", 0.1, kernel)
        assert t is not None and 5e7 < t < 1e9, (kernel, t)
    assert bench.measured_traffic("mlp4096_bf16", "per_example", 0.1, "no_such_kernel") is None
