"""The C-ABI library loads and exports every symbol include/sdlm.h declares (no compute calls)."""
import ctypes
import os
import re

from paper_2509_24007_amd import sdlm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exports_match_header():
    header = open(os.path.join(ROOT, "include", "sdlm.h")).read()
    declared = set(re.findall(r"\b(sdlm_[a-z_]+)\s*\(", header))
    assert declared == set(sdlm.EXPORTS), declared ^ set(sdlm.EXPORTS)
    assert os.path.exists(sdlm.LIB_PATH), "build the library first: python paper_2509_24007_amd/build.py"
    lib = ctypes.CDLL(sdlm.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_workspace_size_and_validation_without_gpu():
    L = sdlm.load()
    m = sdlm.ModelCfg(2, 256, 4, 2, 64, 688, 4096, 1e4, 1e-6, 8.0, 0, 4095, 0)
    r = sdlm.RunCfg(1, 256, 4, 0, 16, 0, 0.5, 0, 0, 0)
    need = L.sdlm_workspace_bytes(ctypes.byref(m), ctypes.byref(r))
    weights = 4 * (2 * 4096 * 256 + 2 * (256 * (4 + 2 * 2) * 64 + 256 * 256 + 3 * 688 * 256))
    assert weights < need < weights + (64 << 20)
    bad = sdlm.RunCfg(1, 256, 17, 0, 16, 0, 0.5, 0, 0, 0)
    assert L.sdlm_workspace_bytes(ctypes.byref(m), ctypes.byref(bad)) == 0
    bad_m = sdlm.ModelCfg(2, 256, 4, 3, 64, 688, 4096, 1e4, 1e-6, 8.0, 0, 4095, 0)
    assert L.sdlm_workspace_bytes(ctypes.byref(bad_m), ctypes.byref(r)) == 0
    # struct layouts agree with the header (field counts and sizes)
    assert ctypes.sizeof(sdlm.ModelCfg) == 14 * 4 and ctypes.sizeof(sdlm.RunCfg) == 10 * 4
    assert ctypes.sizeof(sdlm.Weights) == 15 * ctypes.sizeof(ctypes.c_void_p)
