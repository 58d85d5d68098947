"""Host-side behaviour of bench.py that needs no GPU: more than one GPU is refused with a
message (this build plays the ring's devices in sequence on one GPU), and the workload table
matches the configurations the benchmark is defined on."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args, env=None):
    e = dict(os.environ)
    e.update(env or {})
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True,
                          text=True, env=e, timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
    r = _run(env={"WORLD_SIZE": "4"})
    assert r.returncode == 2 and "ONE GPU" in r.stderr


def test_workloads_are_the_named_configurations():
    sys.path.insert(0, ROOT)
    import bench
    w = bench.WORKLOADS
    assert (w["cfg2"]["H"], w["cfg2"]["S"], w["cfg2"]["N"], w["cfg2"]["d"]) == (16, 32768, 8, 128)
    assert (w["cfg3"]["H"], w["cfg3"]["S"], w["cfg3"]["N"], w["cfg3"]["q_dev"]) == (32, 262144, 8, 7)
    assert (w["cfg4"]["H"], w["cfg4"]["S"], w["cfg4"]["N"]) == (16, 131072, 8)
    assert (w["cfg5"]["H"], w["cfg5"]["S"], w["cfg5"]["N"], w["cfg5"]["q_dev"]) == (8, 786432, 16, 15)
    for cfg in w.values():
        assert cfg["S"] % cfg["N"] == 0 and cfg["B"] == 1
    # useful work of the default pass: 8 triangular steps of c (c + 1) / 2 pairs, 14 d flops each
    c = 32768
    assert bench.useful_flops(w["cfg3"], 1, 14) == 8 * (c * (c + 1) // 2) * 32 * 14 * 128


def test_traffic_comes_from_the_committed_profile_or_not_at_all():
    sys.path.insert(0, ROOT)
    import bench
    t = bench.measured_traffic("cfg3")
    # the summary of the default workload names all three matrix-core kernels
    assert set(t) >= {"fwd_mfma_kernel", "bwd_dq_mfma_kernel", "bwd_dkdv_mfma_kernel"}
    assert all(0 < rd < 100 and 0 < wr < 100 for rd, wr in t.values())
    assert bench.measured_traffic("no-such-workload") == {}
    for _, kernels in bench.FAMILIES.values():
        assert all(k in t for k in kernels)
