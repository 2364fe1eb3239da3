"""The C-ABI library loads and exports every symbol include/r3.h declares (no compute)."""
import ctypes as C
import os
import re

from paper_2510_11370_amd import build as hip_build
from paper_2510_11370_amd import r3

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for header in ("r3.h", "r3_profile.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names.update(re.findall(r"\b(r3_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    hip_build.build()
    lib = r3.lib()
    names = declared_symbols()
    assert set(names) == set(r3.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    assert b"gfx950" in lib.r3_version()


def test_workspace_sizes_and_descriptor_checks_run_on_the_host():
    hip_build.build()
    D = r3.desc(16384, 2048, 128, 8, 768, "bf16")
    sizes = [r3.workspace_bytes(D, op) for op in (r3.OP_REPLAY_GATE, r3.OP_PERMUTE, r3.OP_GROUPED_FFN,
                                                  r3.OP_BACKWARD)]
    assert sizes[0] == 16384 * 128 * 4 and all(s % 256 == 0 for s in sizes) and sizes[3] > 5e8
    bad = r3.desc(16, 16, 8, 9, 16)  # K > E
    assert r3.workspace_bytes(bad, r3.OP_PERMUTE) == 0
    # host-detectable errors come back before anything touches a device
    assert r3.lib().r3_combine(C.byref(bad), None, None, None, None, None) == 1
    assert r3.lib().r3_combine(C.byref(D), None, None, None, None, None) == 1
