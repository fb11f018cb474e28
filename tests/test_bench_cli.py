"""Host-side checks of bench.py's command line (no GPU needed)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    # the path is a single-GPU one: asking for more must end at once, say why, and print no result line
    proc = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                          stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=120)
    assert proc.returncode == 2
    assert "ONE GPU" in proc.stderr
    assert proc.stdout.strip() == ""


def test_kernel_work_table_matches_the_closed_forms():
    # the algorithmic flops / bytes bench.py prices each kernel with, against the formulas of the workload
    sys.path.insert(0, ROOT)
    import bench
    from paper_2603_22276_amd import inputs as I
    cfg = I.C3
    T, do, di, r = cfg.tokens, cfg.d_out, cfg.d_in, cfg.r
    work = bench.kernel_work(cfg)           # kernel -> (flops, bytes)
    assert work["gemm_base_xWt"][0] == 2.0 * T * do * di
    assert work["gemm_dx"][0] == 2.0 * T * di * (do + r)
    assert work["norm_cross_WAt"][0] == 2.0 * do * di * (r + 1)
    assert work["compose_fwd"][1] == 4.0 * 2 * T * do              # reads base, lora; writes y, inner (bf16)
    assert work["compose_bwd"][1] == 3.0 * 2 * T * do              # reads dy, inner; writes dz
    assert {"compose_fwd", "compose_bwd"} <= bench.HBM_BOUND
