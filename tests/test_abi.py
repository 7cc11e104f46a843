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
    rt.batch = 2
    assert binding.lib.sd_workspace_bytes(ctypes.byref(cp), ctypes.byref(cq), ctypes.byref(rt)) == 0
    rt.batch, rt.max_gamma = 1, 16
    assert binding.lib.sd_workspace_bytes(ctypes.byref(cp), ctypes.byref(cq), ctypes.byref(rt)) == 0
