"""Command-line contract of bench.py that can be checked without a GPU."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                         stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_committed_traffic_summaries_name_the_kernels_bench_reports():
    """roofline.traffic is looked up by workload and kernel name in profiles/hbm_traffic_<workload>.txt."""
    sys.path.insert(0, ROOT)
    import bench
    for workload, kernel, per_param in (("llama2_7b", "am_row_kernel<am_bf16, 4, 256, 4>", 18),
                                        ("llama3_8b", "am_row_kernel<am_bf16, 4, 256, 4>", 18),
                                        ("llama2_13b", "am_row_kernel<float, 4, 512, 3>", 20),
                                        ("llama2_7b_adamw", "am_elementwise<am_bf16, 4, 256, 4>", 26)):
        traffic = bench.traffic_from_profiles(workload, kernel)
        assert traffic is not None and traffic > 1e9, (workload, kernel)
    # the dominant kernel of the headline workload moves its algorithmic bytes and nothing more
    from paper_2406_16793_amd import workloads
    wl = workloads.get("llama2_7b")
    rows = [s for s in wl.specs if s.block_numel == 4096]
    algorithmic = sum(s.numel for s in rows) * 18 + 8 * sum(s.n_blocks for s in rows)
    measured = bench.traffic_from_profiles("llama2_7b", "am_row_kernel<am_bf16, 4, 256, 4>")
    assert abs(measured / algorithmic - 1.0) < 0.01
    assert bench.traffic_from_profiles("llama2_7b", "no_such_kernel") is None
    assert json.dumps({"traffic": measured})
