"""Host-side checks of bench.py that need no GPU."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_stored_traffic_figures_are_found_for_the_default_workload():
    """The bench line's roofline.traffic comes from the committed profiler summary: the kernel names
    bench.py looks up have to be the ones the summary lists."""
    for mode in ("literal", "coherent"):
        tag = f"c3_qwen3_256k_{mode}"
        for kernel in ("fp::attn_kernel<128, 128, true>", "fp::search_kernel<128, 128, false>"):
            t = bench.profiled_traffic(tag, kernel)
            assert t is not None, (tag, kernel)
            assert t["bytes"] > 0 and t["live"] is False and t["source"].startswith("profiles/")


def test_more_than_one_gpu_is_refused():
    import subprocess
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr
