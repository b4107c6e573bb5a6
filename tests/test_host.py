"""Host-side behaviour that needs no GPU: the benchmark's command line, the synthetic input recipe (shapes, mixes and
distributions of the benchmark workloads, determinism of the seeds) and the product binding failing loudly - never falling
back to the CPU - where the library cannot run."""
import json
import os
import subprocess
import sys

import numpy as np
import pytest

import gen

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_generators_are_deterministic():
    a, b = gen.make_config(1), gen.make_config(1)
    for k, v in a.items():
        if isinstance(v, np.ndarray):
            np.testing.assert_array_equal(v, b[k], err_msg=k)
        else:
            assert v == b[k], k
    t, u = gen.make_trace(S=2, A=100, seed=9), gen.make_trace(S=2, A=100, seed=9)
    for k, v in t.items():
        if isinstance(v, np.ndarray):
            np.testing.assert_array_equal(v, u[k], err_msg=k)
    assert (gen.make_trace(S=2, A=100, seed=10)["arrival_us"] != t["arrival_us"]).any()


def test_workload_1_shape():
    p = gen.make_config(1)
    assert (p["B"], p["N"], p["M"], p["K"]) == (1, 64, 4, 4)
    assert list(p["k_list"]) == [1, 2, 4, 8]
    assert (p["node_type"] == gen.TYPE_CPU).all() and (p["node_cap"] == 32).all()
    assert (p["act_type"] == gen.TYPE_CPU).all() and (p["act_kmask"] == 0b1111).all()
    assert 0 <= p["node_backlog_us"].min() and p["node_backlog_us"].max() <= 5_000_000


def test_workload_2_recipe():
    """256 snapshots x 1024 actions, 80 % CPU (64 nodes x 128 cores, five options, Amdahl, T ~ LN(ln 2 s, 1)) and
    20 % GPU (8 nodes x 8 GPUs, four options, table k^0.8, T ~ LN(ln 0.3 s, 0.7))."""
    p = gen.make_config(2)
    assert (p["B"], p["N"], p["M"], p["K"]) == (256, 1024, 72, 5)
    nt = p["node_type"].reshape(256, 72)
    assert ((nt == gen.TYPE_CPU).sum(axis=1) == 64).all() and ((nt == gen.TYPE_GPU).sum(axis=1) == 8).all()
    assert (p["node_cap"][p["node_type"] == gen.TYPE_CPU] == 128).all() and (p["node_cap"][p["node_type"] == gen.TYPE_GPU] == 8).all()
    cpu, gpu = p["act_type"] == gen.TYPE_CPU, p["act_type"] == gen.TYPE_GPU
    assert abs(cpu.mean() - 0.8) < 0.005 and abs(gpu.mean() - 0.2) < 0.005
    assert abs(np.median(p["act_t_ori_us"][cpu]) / 2e6 - 1) < 0.02
    assert abs(np.median(p["act_t_ori_us"][gpu]) / 3e5 - 1) < 0.02
    assert abs(np.log(p["act_t_ori_us"][cpu]).std() - 1.0) < 0.02
    assert abs(np.log(p["act_t_ori_us"][gpu]).std() - 0.7) < 0.02
    el = p["act_model"] != 0
    assert (p["act_model"][cpu & el] == 1).all() and (p["act_model"][gpu & el] == 2).all()
    # GPU actions follow class 0 (k^0.8) or class 1 (k^0.9) of the table; row c holds round(65536 k^alpha_c)
    assert set(np.unique(p["act_param"][gpu & el]).tolist()) <= {0, 1}
    np.testing.assert_array_equal(p["speedup_q16"][0:4], np.round(65536 * np.array([1, 2, 4, 8]) ** 0.8).astype(np.uint32))
    np.testing.assert_array_equal(p["speedup_q16"][5:9], np.round(65536 * np.array([1, 2, 4, 8]) ** 0.9).astype(np.uint32))
    assert (p["act_kmask"][gpu] < 16).all()                      # GPU actions use the buddy sizes 1, 2, 4, 8 only


def test_workload_5_recipe():
    t = gen.make_trace(S=8, A=10_000, seed=4)
    assert t["tick_us"] == 100_000 and t["M"] == 256 + 32 + 16
    arr = t["arrival_us"].reshape(8, 10_000)
    assert (np.diff(arr, axis=1) >= 0).all() and arr.max() <= 200_000_000
    gaps = np.diff(arr, axis=1)
    assert abs(gaps[arr[:, 1:] < 199_000_000].mean() / 20_000 - 1) < 0.03      # 50 arrivals per second
    mix = np.bincount(t["act_type"], minlength=3) / t["act_type"].size
    assert np.abs(mix - [0.6, 0.2, 0.2]).max() < 0.01
    c = gen.make_trace(S=1, A=10, seed=5, contended=True)
    assert c["M"] == 4 + 2 + 16 and (c["node_cap"][c["node_type"] == gen.TYPE_CPU] == 32).all()


def test_binding_fails_loudly_without_a_gpu():
    """No GPU, no result: building a problem raises (the library has no CPU path and the binding adds none)."""
    torch = pytest.importorskip("torch")
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    from paper_2603_13019_amd import tg
    tg.load()
    with pytest.raises((tg.TgError, RuntimeError)):              # the library's HIP error, or PyTorch's for the missing device
        tg.Problem(gen.make_config(1))
    with pytest.raises((tg.TgError, RuntimeError)):
        tg.Trace(gen.make_trace(S=1, A=10, seed=1, contended=True))


def test_kernels_keep_their_registers_and_occupancy():
    """From the compiler's own resource report of the build in the tree: no kernel spills to scratch memory, and the
    persistent replay kernel keeps two wavefronts per SIMD (with one, a replay takes twice as long)."""
    import json
    from paper_2603_13019_amd import build
    if not os.path.exists(build.RESOURCES):
        build.build_library()
    k = json.load(open(build.RESOURCES))
    assert len(k) >= 20
    for name, r in k.items():
        assert r["ScratchSize"] == 0, name
    replay = [r for name, r in k.items() if "tg_replay_kernel" in name]
    assert len(replay) == 4 and all(r["Occupancy"] >= 2 for r in replay)
