"""Host-side checks of the benchmark script's contract (no GPU needed)."""
import os
import re
import subprocess
import sys

import paper_2206_10620_amd as pp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr


def test_measured_traffic_belongs_to_the_current_kernel_revision():
    """The HBM traffic bench.py reports was measured with counters on one kernel revision; a stale entry
    must read as null, which bench.py does by comparing revisions.  The committed table and the committed
    profile summaries have to name the revision the library reports."""
    sys.path.insert(0, ROOT)
    import bench
    kernel_of = {2: "k1_tiled", 3: "k3_mfma"}
    for (wl, variant), (rev, nbytes) in bench.MEASURED_TRAFFIC.items():
        assert rev == pp.KERNEL_REVISION, f"{wl}: traffic measured on {rev}, library is {pp.KERNEL_REVISION}"
        assert nbytes > 0
        text = open(os.path.join(ROOT, "profiles", f"{kernel_of[variant]}_{wl}.md")).read()
        assert pp.KERNEL_REVISION in text
        m = re.search(r"= ([0-9.]+) MB, against", text)
        assert m and abs(float(m.group(1)) * 1e6 - nbytes) <= 0.02e6 + 1e-3 * nbytes


def test_block_product_traffic_belongs_to_the_current_kernel_revision():
    sys.path.insert(0, ROOT)
    import bench
    from paper_2206_10620_amd import pp_block_gemm as pb
    rev, nbytes = bench.MEASURED_TRAFFIC_BLOCK
    assert rev == pb.BLOCK_KERNEL_REVISION and nbytes > 0
    text = open(os.path.join(ROOT, "profiles", "k4_block_gemm_block_ffn_4096.md")).read()
    assert pb.BLOCK_KERNEL_REVISION in text
    m = re.search(r"= ([0-9.]+) MB, against", text)
    assert m and abs(float(m.group(1)) * 1e6 - nbytes) <= 0.02e6 + 1e-3 * nbytes


def test_workload_table_covers_the_benchmark_configurations():
    sys.path.insert(0, ROOT)
    import bench
    names = set(bench.workloads())
    assert bench.DEFAULT_WORKLOAD == "cfg5_enhance_1080p"      # the largest single-GPU configuration
    assert {"cfg2_vgg_mid", "cfg5_enhance_1080p"} <= names
    assert sum(n.startswith("cfg4_vgg_L") for n in names) == 13
    assert sum(n.startswith("cfg3_resnet_") and not n.endswith("_f16") for n in names) == 8
    assert {"cfg2_vgg_mid_f16", "cfg2_shape_foreign_patterns_f32", "cfg2_shape_foreign_patterns_f16"} <= names
