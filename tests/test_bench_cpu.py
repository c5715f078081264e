"""bench.py's contract where no GPU is needed: more than one GPU is refused with a message,
and the measured-traffic figures are read from the committed profile summaries."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""
    env = dict(os.environ, WORLD_SIZE="4")
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True,
                         timeout=120, env=env)
    assert res.returncode != 0 and "ONE GPU" in res.stderr


def test_measured_traffic_comes_from_the_profile_summaries():
    """The traffic figure in the bench line is quoted from a committed counter profile, and only
    while that profile was taken with the kernel sources as they are now."""
    sys.path.insert(0, ROOT)
    import bench
    digest = bench.csrc_digest()
    assert len(digest) == 16 and digest == bench.csrc_digest()
    for kernel, wl_, P, k, algorithmic in (("fused_unit_kernel", "resnet50", 4, 4, 920053152),
                                           ("fused_unit_kernel", "vgg16", 4, 4, 4980871584)):
        t, src = bench.traffic_from_profile(kernel, wl_, P, k)
        recorded = [l.split(":")[1].strip() for l in open(os.path.join(ROOT, "profiles", f"fused_unit_{wl_}_P{P}_k{k}.txt"))
                    if l.startswith("csrc_digest:")]
        if recorded and recorded[0] == digest:
            assert t is not None and 0.98 * algorithmic < t < 1.05 * algorithmic and src.startswith("profiles/")
        else:
            assert t is None and "other kernel sources" in src
    t, src = bench.traffic_from_profile("fused_unit_kernel", "no_such_workload", 4, 4)
    assert t is None and "no counter profile" in src
