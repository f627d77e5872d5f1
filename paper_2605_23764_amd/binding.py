"""ctypes binding of libmoe_ffn.so (C ABI in include/moe_ffn.h).

Marshalling only: torch supplies device memory and the stream; every function
here has the name and meaning of the C entry point it calls.
"""
from __future__ import annotations

import ctypes
import dataclasses
import os
from typing import Optional

import torch

MOE_F32, MOE_BF16 = 0, 1
MODE_SERIALIZED, MODE_PERSISTENT = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class MoeError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: {moe_status_string(status)} ({status})")
        self.status = status


class _MoeShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("T", "H", "I", "E", "E_local", "expert_base", "k", "dtype")]


class _MoeSaved(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("topk_idx", "topk_w", "counts", "offsets", "row_of", "token_of", "slot_of", "Xp", "H1", "A", "Yp")]


EXPORTS = (
    "moe_status_string", "moe_ffn_workspace_bytes", "moe_ffn_forward", "moe_ffn_backward", "moe_ffn_backward_two_streams",
    "moe_ffn_last_status", "moe_ffn_debug_set_spin_limit", "moe_route", "moe_permute", "moe_grouped_gemm_swiglu", "moe_grouped_gemm",
    "moe_combine", "moe_microbench_workspace_bytes", "moe_microbench_swiglu_add", "moe_microbench_last_status",
    "moe_probe_mfma_bf16", "moe_probe_copy", "moe_probe_read", "moe_probe_write", "moe_microbench_swiglu_add_static_scratch",
    "moe_ffn_debug_force_device_scope", "moe_ffn_debug_layout", "moe_dispatch_to_combine",
    "moe_grouped_gemm_scatter", "moe_ffn_forward_scatter",
)
LAYOUT_WORDS = 25   # MOE_LAYOUT_WORDS


def library_path() -> str:
    return os.path.join(_HERE, "libmoe_ffn.so")


def load_library() -> ctypes.CDLL:
    """Load the HIP library; raises if it has not been built (no fallback)."""
    global _LIB
    if _LIB is None:
        path = library_path()
        if not os.path.exists(path):
            raise FileNotFoundError(
                f"{path} is missing: build it with `python -m paper_2605_23764_amd.build` "
                "(or __graft_entry__.build()); there is no CPU fallback")
        lib = ctypes.CDLL(path)
        lib.moe_status_string.restype = ctypes.c_char_p
        lib.moe_status_string.argtypes = [ctypes.c_int]
        for name in EXPORTS[1:]:
            getattr(lib, name).restype = ctypes.c_int
        lib.moe_microbench_workspace_bytes.restype = ctypes.c_size_t
        lib.moe_microbench_workspace_bytes.argtypes = [ctypes.c_int]
        _LIB = lib
    return _LIB


def moe_status_string(status: int) -> str:
    return load_library().moe_status_string(int(status)).decode()


def make_shape(T, H, I, E, E_local, expert_base, k, dtype) -> _MoeShape:
    if isinstance(dtype, torch.dtype):
        dtype = {torch.float32: MOE_F32, torch.bfloat16: MOE_BF16}[dtype]
    return _MoeShape(T, H, I, E, E_local, expert_base, k, dtype)


def _torch_dtype(shape: _MoeShape) -> torch.dtype:
    return torch.bfloat16 if shape.dtype == MOE_BF16 else torch.float32


def moe_ffn_workspace_bytes(shape: _MoeShape):
    fwd, bwd = ctypes.c_size_t(0), ctypes.c_size_t(0)
    st = load_library().moe_ffn_workspace_bytes(ctypes.byref(shape), ctypes.byref(fwd), ctypes.byref(bwd))
    if st != 0:
        raise MoeError(st, "moe_ffn_workspace_bytes")
    return fwd.value, bwd.value


def alloc_workspace(shape: _MoeShape, device="cuda", backward: bool = False) -> torch.Tensor:
    fwd, bwd = moe_ffn_workspace_bytes(shape)
    return torch.empty(max(fwd, bwd) if backward else fwd, dtype=torch.uint8, device=device)


@dataclasses.dataclass
class Saved:
    """Device buffers of MoeSaved (torch tensors own the memory)."""
    topk_idx: torch.Tensor
    topk_w: torch.Tensor
    counts: torch.Tensor
    offsets: torch.Tensor
    row_of: torch.Tensor
    token_of: torch.Tensor
    slot_of: torch.Tensor
    Xp: Optional[torch.Tensor]
    H1: Optional[torch.Tensor]
    A: torch.Tensor
    Yp: torch.Tensor

    def c_struct(self) -> _MoeSaved:
        f = lambda t: ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)  # noqa: E731
        return _MoeSaved(*(f(getattr(self, n)) for n, _ in _MoeSaved._fields_))


def alloc_saved(shape: _MoeShape, device="cuda", store_h1: bool = False, keep_xp: bool = True) -> Saved:
    """keep_xp=False: no permuted copy of x is kept (MoeSaved.Xp = NULL); forward and backward then read x through
    the permutation."""
    T, H, I, k, El = shape.T, shape.H, shape.I, shape.k, shape.E_local
    Rm = T * min(k, El)
    dt = _torch_dtype(shape)
    i32 = dict(dtype=torch.int32, device=device)
    # +4 elements keep zero-size problems at non-null, aligned pointers
    return Saved(
        topk_idx=torch.empty(T * k + 4, **i32)[: T * k].view(T, k),
        topk_w=torch.empty(T * k + 4, dtype=torch.float32, device=device)[: T * k].view(T, k),
        counts=torch.empty(El, **i32),
        offsets=torch.empty(El + 1, **i32),
        row_of=torch.empty(T * k + 4, **i32)[: T * k].view(T, k),
        token_of=torch.empty(Rm + 4, **i32)[:Rm],
        slot_of=torch.empty(Rm + 4, **i32)[:Rm],
        Xp=torch.empty(Rm * H + 8, dtype=dt, device=device)[: Rm * H].view(Rm, H) if keep_xp else None,
        H1=torch.empty(Rm * 2 * I + 8, dtype=dt, device=device)[: Rm * 2 * I].view(Rm, 2 * I) if store_h1 else None,
        A=torch.empty(Rm * I + 8, dtype=dt, device=device)[: Rm * I].view(Rm, I),
        Yp=torch.empty(Rm * H + 8, dtype=dt, device=device)[: Rm * H].view(Rm, H),
    )


def _ptr(t: Optional[torch.Tensor]) -> ctypes.c_void_p:
    if t is None:
        return ctypes.c_void_p(0)
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _check(st: int, what: str) -> None:
    if st != 0:
        raise MoeError(st, what)


def _ws(ws: torch.Tensor):
    return _ptr(ws), ctypes.c_size_t(ws.numel() * ws.element_size())


def moe_ffn_forward(shape, x, logits, w_gate_up, w_down, out, saved: Optional[Saved], workspace,
                    mode: int = MODE_SERIALIZED, stream=None) -> None:
    sv = saved.c_struct() if saved is not None else None
    wp, wb = _ws(workspace)
    st = load_library().moe_ffn_forward(
        ctypes.byref(shape), _ptr(x), _ptr(logits), _ptr(w_gate_up), _ptr(w_down), _ptr(out),
        ctypes.byref(sv) if sv is not None else None, wp, wb, ctypes.c_int(mode), _stream(stream))
    _check(st, "moe_ffn_forward")


def moe_ffn_backward(shape, dy, x, w_gate_up, w_down, saved: Saved, dx, dw_gate_up, dw_down, dtopk_w,
                     workspace, mode: int = MODE_SERIALIZED, stream=None) -> None:
    sv = saved.c_struct()
    wp, wb = _ws(workspace)
    st = load_library().moe_ffn_backward(
        ctypes.byref(shape), _ptr(dy), _ptr(x), _ptr(w_gate_up), _ptr(w_down), ctypes.byref(sv),
        _ptr(dx), _ptr(dw_gate_up), _ptr(dw_down), _ptr(dtopk_w), wp, wb, ctypes.c_int(mode), _stream(stream))
    _check(st, "moe_ffn_backward")


def moe_ffn_backward_two_streams(shape, dy, x, w_gate_up, w_down, saved: Saved, dx, dw_gate_up, dw_down, dtopk_w,
                                 workspace, wgrad_stream, mode: int = MODE_SERIALIZED, stream=None) -> None:
    """`wgrad_stream`: a torch.cuda.Stream for the weight-gradient launches, or None (one stream)."""
    sv = saved.c_struct()
    wp, wb = _ws(workspace)
    side = ctypes.c_void_p(wgrad_stream.cuda_stream) if wgrad_stream is not None else ctypes.c_void_p(None)
    st = load_library().moe_ffn_backward_two_streams(
        ctypes.byref(shape), _ptr(dy), _ptr(x), _ptr(w_gate_up), _ptr(w_down), ctypes.byref(sv),
        _ptr(dx), _ptr(dw_gate_up), _ptr(dw_down), _ptr(dtopk_w), wp, wb, ctypes.c_int(mode), _stream(stream), side)
    _check(st, "moe_ffn_backward_two_streams")


def moe_ffn_last_status(shape, workspace) -> int:
    return load_library().moe_ffn_last_status(ctypes.byref(shape), _ptr(workspace))


def moe_ffn_debug_set_spin_limit(polls: int) -> None:
    _check(load_library().moe_ffn_debug_set_spin_limit(ctypes.c_uint32(polls)), "moe_ffn_debug_set_spin_limit")


def moe_route(shape, logits, saved: Saved, workspace, stream=None) -> None:
    sv = saved.c_struct()
    wp, wb = _ws(workspace)
    _check(load_library().moe_route(ctypes.byref(shape), _ptr(logits), ctypes.byref(sv), wp, wb, _stream(stream)),
           "moe_route")


def moe_permute(shape, x, saved: Saved, workspace, stream=None) -> None:
    sv = saved.c_struct()
    wp, wb = _ws(workspace)
    _check(load_library().moe_permute(ctypes.byref(shape), _ptr(x), ctypes.byref(sv), wp, wb, _stream(stream)),
           "moe_permute")


def moe_grouped_gemm_swiglu(shape, w_gate_up, saved: Saved, workspace, stream=None) -> None:
    sv = saved.c_struct()
    wp, wb = _ws(workspace)
    _check(load_library().moe_grouped_gemm_swiglu(ctypes.byref(shape), _ptr(w_gate_up), ctypes.byref(sv), wp, wb,
                                                  _stream(stream)), "moe_grouped_gemm_swiglu")


def moe_grouped_gemm(shape, w_down, saved: Saved, workspace, stream=None) -> None:
    sv = saved.c_struct()
    wp, wb = _ws(workspace)
    _check(load_library().moe_grouped_gemm(ctypes.byref(shape), _ptr(w_down), ctypes.byref(sv), wp, wb,
                                           _stream(stream)), "moe_grouped_gemm")


def moe_grouped_gemm_scatter(shape, w_down, saved: Saved, out, workspace, stream=None) -> None:
    sv = saved.c_struct()
    wp, wb = _ws(workspace)
    _check(load_library().moe_grouped_gemm_scatter(ctypes.byref(shape), _ptr(w_down), ctypes.byref(sv), _ptr(out), wp, wb,
                                                   _stream(stream)), "moe_grouped_gemm_scatter")


def moe_ffn_forward_scatter(shape, x, logits, w_gate_up, w_down, out, saved: Optional[Saved], workspace,
                            mode: int = MODE_SERIALIZED, stream=None) -> None:
    sv = saved.c_struct() if saved is not None else None
    wp, wb = _ws(workspace)
    st = load_library().moe_ffn_forward_scatter(
        ctypes.byref(shape), _ptr(x), _ptr(logits), _ptr(w_gate_up), _ptr(w_down), _ptr(out),
        ctypes.byref(sv) if sv is not None else None, wp, wb, ctypes.c_int(mode), _stream(stream))
    _check(st, "moe_ffn_forward_scatter")


def moe_combine(shape, saved: Saved, out, workspace, stream=None) -> None:
    sv = saved.c_struct()
    wp, wb = _ws(workspace)
    _check(load_library().moe_combine(ctypes.byref(shape), ctypes.byref(sv), _ptr(out), wp, wb, _stream(stream)),
           "moe_combine")


def moe_dispatch_to_combine(shape, x, w_gate_up, w_down, out, saved: Saved, workspace, mode: int = MODE_SERIALIZED,
                            stream=None) -> None:
    sv = saved.c_struct()
    wp, wb = _ws(workspace)
    _check(load_library().moe_dispatch_to_combine(ctypes.byref(shape), _ptr(x), _ptr(w_gate_up), _ptr(w_down), _ptr(out),
                                                  ctypes.byref(sv), wp, wb, ctypes.c_int(mode), _stream(stream)),
           "moe_dispatch_to_combine")


MB_SERIAL, MB_STATIC, MB_DYNAMIC, MB_DYNAMIC_XCD = 0, 1, 2, 3


def moe_microbench_workspace_bytes(M: int) -> int:
    return int(load_library().moe_microbench_workspace_bytes(int(M)))


def moe_microbench_swiglu_add(M, N, x, y, s, out, mode, tile_rows, workspace, stream=None) -> None:
    wp, wb = _ws(workspace)
    _check(load_library().moe_microbench_swiglu_add(ctypes.c_int(M), ctypes.c_int(N), _ptr(x), _ptr(y), _ptr(s),
                                                    _ptr(out), ctypes.c_int(mode), ctypes.c_int(tile_rows), wp, wb,
                                                    _stream(stream)),
           "moe_microbench_swiglu_add")


def moe_microbench_last_status(workspace) -> int:
    return load_library().moe_microbench_last_status(_ptr(workspace))


def moe_probe_mfma_bf16(n_workgroups, mfma_per_wave, random_operands, sink, stream=None) -> None:
    _check(load_library().moe_probe_mfma_bf16(ctypes.c_int(n_workgroups), ctypes.c_int(mfma_per_wave),
                                              ctypes.c_int(1 if random_operands else 0), _ptr(sink), _stream(stream)),
           "moe_probe_mfma_bf16")


def moe_microbench_swiglu_add_static_scratch(M, N, x, y, s, out, mode, tile_rows, status=None, stream=None) -> None:
    _check(load_library().moe_microbench_swiglu_add_static_scratch(
        ctypes.c_int(M), ctypes.c_int(N), _ptr(x), _ptr(y), _ptr(s), _ptr(out), ctypes.c_int(mode),
        ctypes.c_int(tile_rows), _ptr(status), _stream(stream)), "moe_microbench_swiglu_add_static_scratch")


def moe_ffn_debug_force_device_scope(on: bool) -> None:
    _check(load_library().moe_ffn_debug_force_device_scope(ctypes.c_int(1 if on else 0)),
           "moe_ffn_debug_force_device_scope")


def moe_ffn_debug_layout(shape, backward: bool = False):
    """The LAYOUT_WORDS integers of moe_ffn_debug_layout (offsets of the scheduler's tables in the workspace)."""
    out = (ctypes.c_int64 * LAYOUT_WORDS)()
    _check(load_library().moe_ffn_debug_layout(ctypes.byref(shape), ctypes.c_int(1 if backward else 0), out,
                                               ctypes.c_int(LAYOUT_WORDS)), "moe_ffn_debug_layout")
    return list(out)


def moe_probe_read(src, nbytes, sink, stream=None) -> None:
    _check(load_library().moe_probe_read(_ptr(src), ctypes.c_size_t(nbytes), _ptr(sink), _stream(stream)),
           "moe_probe_read")


def moe_probe_write(dst, nbytes, word=0, stream=None) -> None:
    _check(load_library().moe_probe_write(_ptr(dst), ctypes.c_size_t(nbytes), ctypes.c_uint32(word), _stream(stream)),
           "moe_probe_write")


def moe_probe_copy(src, dst, nbytes, stream=None) -> None:
    _check(load_library().moe_probe_copy(_ptr(src), _ptr(dst), ctypes.c_size_t(nbytes), _stream(stream)),
           "moe_probe_copy")
