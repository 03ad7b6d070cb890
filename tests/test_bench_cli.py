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


def _largest_bucket_kernel(workload, adamw=False):
    """Name of the kernel that serves most parameters of a workload, from a host-only layout."""
    from paper_2406_16793_amd import binding as B, partition, workloads
    wl = workloads.get(workload)
    specs = partition.as_adamw(wl.specs) if adamw else wl.specs
    h = B.adam_mini_init_layout([(s.numel, s.block_numel, s.wd_scale) for s in specs],
                                B.GRAD_BF16 if wl.grad_dtype == "bf16" else B.GRAD_F32, -1)
    buckets = B.adam_mini_profile_read(h)
    B.adam_mini_destroy_layout(h)
    top = max(buckets, key=lambda b: b["numel"])
    return top["kernel"], top["numel"], top["n_blocks"]


def test_committed_traffic_summaries_name_the_kernels_bench_reports():
    """roofline.traffic is looked up by workload and kernel name in profiles/hbm_traffic_<workload>.txt:
    the committed summaries must hold the kernel that the CURRENT layout builder makes the dominant one."""
    sys.path.insert(0, ROOT)
    import bench
    for workload, adamw, per_param in (("llama2_7b", False, 18), ("llama3_8b", False, 18), ("llama2_13b", False, 20),
                                       ("llama2_7b", True, 26), ("gpt2_small", False, 20), ("tiny", False, 20)):
        kernel, numel, n_blocks = _largest_bucket_kernel(workload, adamw)
        tag = workload + ("_adamw" if adamw else "")
        traffic, source = bench.traffic_from_profiles(tag, kernel, with_source=True)
        assert traffic is not None and traffic > 1e7, (tag, kernel)
        assert source.startswith("profiles/hbm_traffic_%s.txt@" % tag), source       # names the tree it was taken on
        if workload.startswith("llama"):
            # the big streaming kernels move their algorithmic bytes and nothing more
            algorithmic = numel * per_param + (0 if adamw else 8 * n_blocks)
            assert abs(traffic / algorithmic - 1.0) < 0.01, (tag, kernel, traffic, algorithmic)
    assert bench.traffic_from_profiles("llama2_7b", "no_such_kernel") is None
