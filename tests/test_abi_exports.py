"""The C-ABI library loads without a GPU and exports every entry point the header declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "cfdecode.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cf_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported():
    import paper_2508_18850_amd as pkg
    path = pkg.lib_path()
    if not os.path.exists(path):
        from paper_2508_18850_amd import build
        build.build()
    lib = ctypes.CDLL(path)
    names = declared_symbols()
    assert "cf_decode_block" in names and len(names) >= 8
    for n in names:
        assert hasattr(lib, n), "missing export " + n
    assert sorted(pkg.EXPORTED_SYMBOLS) == names


def test_host_only_entry_points():
    import paper_2508_18850_amd as pkg
    lib = pkg.load_library()
    assert lib.cf_strerror(0) == b"ok" and lib.cf_strerror(-1) == b"invalid argument"
    cfg = pkg.CfConfig(4096, 32, 32, 128, 1, 4224, 10000.0, 0)
    # weights 128 MiB + KV 64 MiB + appended rows 16 KiB + x/out 16 KiB  (Llama-2-7B shape, L = 4096)
    assert pkg.algorithmic_bytes(cfg, 1, 4096) == 201326592 + 32 * 2 * 128 * 2 + 2 * 4096 * 2
    assert lib.cf_create(None, None) == -1
