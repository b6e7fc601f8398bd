"""Host-side checks of the measurement harness (no GPU): the committed counter
summary is found for the library that is built, and only for it; a run on more
than one GPU is refused with a message."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


@pytest.fixture(scope="module")
def B():
    from paper_2509_23638_amd.build import LIB, build
    if not os.path.exists(LIB):
        build(verbose=False)
    import paper_2509_23638_amd.binding as B
    return B


def test_traffic_figure_is_keyed_by_kernel_workload_and_library(B):
    import bench
    from workloads import get_config
    cfg = get_config("c2_mixtral")
    sh = B.make_shape(64, cfg.H, cfg.E, cfg.k, cfg.F, cfg.S, cfg.dtype, "tiled")
    kernel = B.moe_ffn_kernel_name(sh, 0, cfg.E)
    lib = B.moe_version()
    hit = bench.traffic_from_profiles(kernel, "c2_mixtral", 64, "tiled", lib)
    assert hit is not None, "profiles/ holds no traffic_bytes line for the headline kernel of this library"
    assert hit["source"].startswith("profiles/")
    # algorithmic bytes of that launch: 8 experts x 2 matrices + X + h
    algorithmic = 8 * 2 * cfg.F * cfg.H * 2 + 64 * cfg.H * 2 + 64 * cfg.k * cfg.F * 2
    assert algorithmic == 1_883_242_496
    assert 1.0 <= hit["bytes"] / algorithmic < 1.02
    # anything else it was not measured on reports nothing
    assert bench.traffic_from_profiles(kernel, "c2_mixtral", 32, "tiled", lib) is None
    assert bench.traffic_from_profiles(kernel, "c2_mixtral", 64, "row_major", lib) is None
    assert bench.traffic_from_profiles(kernel, "c3_finegrained", 64, "tiled", lib) is None
    assert bench.traffic_from_profiles("ffn_tile_kernel<gate/up>", "c2_mixtral", 64, "tiled", lib) is None
    assert bench.traffic_from_profiles(kernel, "c2_mixtral", 64, "tiled", lib + " next") is None


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""
    env = dict(os.environ, WORLD_SIZE="2")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True,
                       timeout=120, env=env)
    assert r.returncode != 0 and "one GPU" in r.stderr
