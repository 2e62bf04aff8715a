"""bench.py contract checks that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_roofline_kernel_name_mapping_covers_every_profiled_kernel():
    sys.path.insert(0, ROOT)
    import bench

    for name in ("gemm_fwd_256x256", "gemm_bwd_256x256", "gemm_fwd_128x256", "gemm_bwd_128x256", "gemm_fwd_64x128k", "gemm_fwd_128x64s", "gemm_bwd_128x64s", "gemm_bwd_64x128", "stream_fwd",
                 "stream_bwd", "stream_fwd_finish", "stream_bwd_finish", "f16_stream_fwd", "f16_stream_bwd_finish", "lora_down_finish",
                 "lora_down", "lora_grad", "lora_grad_reduce"):
        pat = bench.rocprof_kernel_pattern(name)
        assert "kernel" in pat, (name, pat)


def test_default_workload_is_the_largest_single_gpu_configuration():
    sys.path.insert(0, ROOT)
    import bench
    from paper_2309_16119_amd import synth

    name, M = bench.HEADLINE
    cfg = synth.CONFIGS[name].with_M(M)
    assert (cfg.K, cfg.N, cfg.M) == (8192, 22016, 4096)
    assert all(cfg.flops_fwd_bwd >= c.flops_fwd_bwd for c in synth.CONFIGS.values())
    assert bench.REPEATS >= 5
