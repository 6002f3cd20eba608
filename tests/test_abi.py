"""Host-only checks of the C-ABI library: it loads, exports every symbol the header
declares, and no compute call is made (no GPU needed)."""
import ctypes
import os
import re

from paper_2103_00686_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "fae.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fae_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    names = _declared()
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/fae.h but not exported"
    assert sorted(B.EXPORTS) == names


def test_version_and_workspace_queries_run_on_the_host():
    assert "gfx950" in B.fae_version()
    t = B.Tables([1000, 5_000_000], 16)
    assert B.fae_choose_cutoff_workspace_bytes(t) > 0
    assert B.fae_build_workspace_bytes(t) >= (5_001_000 // 2048) * 4
    assert B.fae_partition_workspace_bytes(t, 4096) >= 2 * 4096 * 4
    small = B.fae_bwd_workspace_bytes(t, 4096, [4096, 4096])
    big = B.fae_bwd_workspace_bytes(t, 65536, [65536, 1_300_000])
    assert 16 * 8192 <= small < big


def test_header_is_plain_c():
    import subprocess
    src = '#include "fae.h"\nint main(void){return sizeof(fae_tables)+sizeof(fae_batch)>0?0:1;}\n'
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                        "-x", "c", "-", "-o", "/dev/null"], input=src, text=True, capture_output=True)
    assert r.returncode == 0, r.stderr
