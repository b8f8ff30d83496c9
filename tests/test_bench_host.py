"""Host-side checks of bench.py that need no GPU: the one-GPU rule, the traffic table it reads, its work model."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench
import s24_inputs as si


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_table_has_the_headline_rows_and_nothing_is_assumed_elsewhere():
    for wl in ("c4", "c5"):
        for k in ("mask_compress", "spmm_fwd", "spmm_bwd_dx", "dense_dw"):
            t = bench.measured_traffic(wl, k)
            assert t is not None and t > 0, (wl, k)
    assert bench.measured_traffic("c2", "dense_dw") is None
    assert bench.measured_traffic("c5", "no_such_kernel") is None
    # measured bytes can exceed the algorithmic ones (re-reads) but never fall below what must be written
    wl = si.WORKLOADS["c5"]
    assert bench.measured_traffic("c5", "dense_dw") >= 3 * wl.d_model * wl.d_ff * 4


def test_work_model_counts_the_gemms_of_a_step():
    for name, gemms in (("c2", 6), ("c3", 6), ("c4", 9), ("c5", 9)):
        wl = si.WORKLOADS[name]
        m = bench.kernel_model(wl)
        per = 2.0 * wl.p * wl.d_model * wl.d_ff
        assert m["spmm_fwd"][1] + m["spmm_bwd_dx"][1] + m["dense_dw"][1] == gemms * per == wl.gemm_flops
        assert m["spmm_fwd"][2] == 5000.0 and m["dense_dw"][2] == 2500.0 and m["mask_compress"][2] == 8000.0
        # fused search + compress: 70 bytes per 4 x 4 block of a 16-bit weight
        blocks = len(wl.weight_names) * wl.d_model * wl.d_ff / 16
        assert m["mask_compress"][1] == 70 * blocks
