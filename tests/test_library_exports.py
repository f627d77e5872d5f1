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


def test_single_launch_alignment_is_checked_on_the_host(lib):
    """The single-launch modes need 128-byte aligned hand-over buffers; the check happens on the host before
    anything is enqueued, so made-up addresses are enough to see it (no launch happens on this path)."""
    import ctypes
    from paper_2605_23764_amd.binding import _MoeSaved
    s = moe.make_shape(64, 64, 64, 4, 4, 0, 1, moe.MOE_BF16)
    fwd, bwd = moe.moe_ffn_workspace_bytes(s)
    P = ctypes.c_void_p
    base = 0x7f0000000000

    def saved(a_off=0, xp_off=0):
        addr = {n: base + (i + 1) * 0x1000000 for i, (n, _) in enumerate(_MoeSaved._fields_)}
        addr["A"] += a_off
        addr["Xp"] += xp_off
        return _MoeSaved(*(P(addr[n]) for n, _ in _MoeSaved._fields_))

    def forward(sv, ws):
        return lib.moe_ffn_forward(ctypes.byref(s), P(base + 0x100), P(base + 0x200), P(base + 0x300), P(base + 0x400),
                                   P(base + 0x500), ctypes.byref(sv), P(ws), ctypes.c_size_t(fwd), 1, None)
    assert forward(saved(a_off=16), base) == -1
    assert forward(saved(xp_off=64), base) == -1
    assert forward(saved(), base + 16) == -1
    sv = saved()
    assert lib.moe_ffn_backward(ctypes.byref(s), P(base + 0x100), P(base + 0x200), P(base + 0x300), P(base + 0x400),
                                ctypes.byref(sv), P(base + 0x500), P(base + 0x600), P(base + 0x700), P(base + 0x800),
                                P(base + 0x900 + 16), ctypes.c_size_t(bwd), 1, None) == -1
    # microbenchmark modes 1 and 3: tiles of whole 128-byte lines on a 128-byte aligned intermediate
    lib.moe_microbench_swiglu_add.argtypes = None
    for mode in (1, 3):
        assert lib.moe_microbench_swiglu_add(4096, 8, P(base), P(base + 0x100000), P(base + 0x200000), P(base + 0x300000),
                                             mode, 1, P(base + 0x400000), ctypes.c_size_t(1 << 20), None) == -1
        assert lib.moe_microbench_swiglu_add(4096, 8, P(base), P(base + 0x100000), P(base + 0x200000 + 16),
                                             P(base + 0x300000), mode, 8, P(base + 0x400000), ctypes.c_size_t(1 << 20),
                                             None) == -1
    assert lib.moe_microbench_swiglu_add_static_scratch(32769, 64, P(base), P(base), P(base), P(base), 1, 8, None, None) == -2
    assert "XCD" in moe.moe_status_string(-6)


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
