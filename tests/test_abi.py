"""The C-ABI library loads and exports every entry point include/sd.h declares
(no compute calls: this runs without a GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib_path = os.path.join(ROOT, "paper_2211_17192_amd", "libsd.so")
    if not os.path.exists(lib_path):
        from paper_2211_17192_amd import build
        build.build(verbose=False)
    header = open(os.path.join(ROOT, "include", "sd.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(sd_[a-z_]+)\s*\(", header))
    assert {"sd_load_models", "sd_prefill", "sd_step", "sd_reset", "sd_step_baseline", "sd_spec_sample"} <= names
    lib = ctypes.CDLL(lib_path)
    for n in sorted(names):
        assert hasattr(lib, n), n


def test_workspace_sizing_needs_no_gpu():
    from paper_2211_17192_amd import binding, synth
    cfg_p, _, cfg_q, _ = synth.tiny_pair()
    cp, cq = binding._cfg_struct(cfg_p), binding._cfg_struct(cfg_q)
    rt = binding._RuntimeCfg(batch=1, max_gamma=4, page_size=16)
    n = binding.lib.sd_workspace_bytes(ctypes.byref(cp), ctypes.byref(cq), ctypes.byref(rt))
    assert 100_000 < n < 50_000_000
    rt.batch = 4                                    # four sequences: four times the KV pages and activations,
    n4 = binding.lib.sd_workspace_bytes(ctypes.byref(cp), ctypes.byref(cq), ctypes.byref(rt))   # plus the batched GEMMs' scratch
    assert n < n4 < 6 * n
    rt.batch = 65
    assert binding.lib.sd_workspace_bytes(ctypes.byref(cp), ctypes.byref(cq), ctypes.byref(rt)) == 0
    rt.batch, rt.max_gamma = 1, 16
    assert binding.lib.sd_workspace_bytes(ctypes.byref(cp), ctypes.byref(cq), ctypes.byref(rt)) == 0


def test_choose_gamma_matches_brute_force_and_the_papers_rule():
    """Section 3.5 host logic through the C ABI: the chosen gamma maximises Theorem 3.8
    (checked against the oracle's search and a direct evaluation), gamma never shrinks as
    alpha grows or c falls, and Corollary 3.9's condition alpha > c decides whether any
    gamma gives an improvement."""
    import numpy as np
    from oracle import analysis
    from paper_2211_17192_amd import binding
    for c in (0.0, 0.01, 0.02, 0.05, 0.1, 0.2, 0.4):
        prev = 0
        for alpha in np.linspace(0.05, 0.95, 19):
            g, v = binding.choose_gamma(alpha, c, 15)
            assert g == analysis.optimal_gamma(alpha, c, 15)
            direct = (1 - alpha ** (g + 1)) / ((1 - alpha) * (g * c + 1))
            assert abs(v - direct) < 1e-12 * direct
            for other in range(1, 16):
                assert v >= analysis.walltime_improvement(alpha, other, c) - 1e-12
            assert (v > 1.0) == (alpha > c) or abs(alpha - c) < 1e-9
            assert g >= prev
            prev = g
    # c = 0: more guesses always help, the search stops at the cap
    assert binding.choose_gamma(0.5, 0.0, 7)[0] == 7
    g = ctypes.c_int32(0)
    for bad in ((1.0, 0.1, 5), (-0.1, 0.1, 5), (0.5, -1.0, 5), (0.5, 0.1, 0), (float("nan"), 0.1, 5)):
        assert binding.lib.sd_choose_gamma(bad[0], bad[1], bad[2], ctypes.byref(g), None) == binding.SD_EINVAL


def test_bench_refuses_more_than_one_gpu_and_unknown_workloads():
    """bench.py runs on one GPU only and says so; its command line is checked before anything
    touches a GPU."""
    import subprocess, sys, os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--workload", "nope"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "invalid choice" in r.stderr
