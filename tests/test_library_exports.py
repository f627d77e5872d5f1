"""CPU-only checks of the C ABI: the library builds/loads and exports every symbol
declared in include/moe_ffn.h; host-only entry points behave (no compute calls)."""
import ctypes
import os
import re

import pytest

import paper_2605_23764_amd as moe

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(moe.library_path()):
        from paper_2605_23764_amd.build import build_library
        build_library()
    return moe.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "moe_ffn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert "moe_ffn_forward" in names and "moe_ffn_backward" in names and len(names) >= 10
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(moe.binding.EXPORTS)


def test_status_strings_and_workspace_query(lib):
    assert moe.moe_status_string(0) == "ok"
    assert "workspace" in moe.moe_status_string(-3)
    s = moe.make_shape(256, 256, 128, 8, 8, 0, 2, moe.MOE_F32)
    fwd, bwd = moe.moe_ffn_workspace_bytes(s)
    assert fwd > 256 * 2 * (256 * 2 + 128) * 4 and bwd >= fwd
    for bad in (moe.make_shape(256, 250, 128, 8, 8, 0, 2, 0), moe.make_shape(256, 256, 128, 8, 8, 0, 9, 0),
                moe.make_shape(256, 256, 128, 8, 4, 6, 2, 0), moe.make_shape(256, 256, 128, 512, 8, 0, 2, 0)):
        with pytest.raises(moe.MoeError) as ei:
            moe.moe_ffn_workspace_bytes(bad)
        assert ei.value.status == -2
    assert lib.moe_ffn_workspace_bytes(None, None, None) == -1


def test_bench_refuses_more_than_one_gpu():
    """One GPU's share is all this build runs: bench.py --gpus 2 must exit with a message."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout) or "ONE GPU" in (r.stderr + r.stdout)
