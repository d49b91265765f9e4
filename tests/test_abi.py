"""The C-ABI library loads without a GPU and exports every function include/bpd.h declares."""
import ctypes
import os
import re

from paper_1811_03115_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "bpd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bpd_[a-z_0-9]+)\s*\(", text)))


def test_header_functions_are_exported_and_bound():
    names = declared_functions()
    assert "bpd_step" in names and "bpd_encode" in names and "bpd_decode" in names and "bpd_load_weights" in names
    lib = binding.lib()
    for n in names:
        assert hasattr(lib, n), f"{n} declared in bpd.h but not exported by libbpd.so"
    assert sorted(binding.EXPORTS) == names
    for n in names:
        if n not in ("bpd_workspace_bytes", "bpd_last_error", "bpd_create", "bpd_destroy"):  # constructor / close()
            assert hasattr(binding.Context, n), f"binding.Context lacks {n}"


def test_workspace_sizing_and_config_validation_on_host():
    import workloads as wl
    lib = binding.lib()
    sizes = {}
    for name, w in wl.CONFIGS.items():
        cfg = binding.config_from_workload(w)
        sizes[name] = lib.bpd_workspace_bytes(ctypes.byref(cfg))
        assert sizes[name] > 0
    # C2 holds 411 MB of decoder-side bf16 weights plus the encoder, caches and staging
    assert 600e6 < sizes["C2"] < 1.2e9
    assert sizes["C3"] > sizes["C2"]
    bad = binding.config_from_workload(wl.C0)
    bad.k_max = 17
    assert lib.bpd_workspace_bytes(ctypes.byref(bad)) == 0
    bad = binding.config_from_workload(wl.C0)
    bad.vocab = 250                      # not a multiple of 16
    assert lib.bpd_workspace_bytes(ctypes.byref(bad)) == 0
    bad = binding.config_from_workload(wl.C0)
    bad.n_heads = 3
    assert lib.bpd_workspace_bytes(ctypes.byref(bad)) == 0
    # null arguments come back as error codes, not crashes
    assert lib.bpd_create(None, None, 0, None, None) == -1
    assert lib.bpd_step(None, 1, None, None) == -1
    assert lib.bpd_destroy(None) == -1
    assert lib.bpd_last_error(None) == b"null context"
