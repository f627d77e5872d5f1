"""MI355X-native Dispatch-to-Combine MoE-FFN layer (hand-written gfx950 HIP kernels
behind a C ABI).  This package is the thin Python binding: argument marshalling
only; every step of the layer runs in the HIP library.  Importing the package
does not load the library; the first call does, and fails loudly if it is
missing (there is no CPU fallback)."""
from .binding import (  # noqa: F401
    MB_DYNAMIC,
    MB_DYNAMIC_XCD,
    MB_SERIAL,
    MB_STATIC,
    MOE_BF16,
    MOE_F32,
    MODE_PERSISTENT,
    MODE_SERIALIZED,
    MoeError,
    Saved,
    alloc_saved,
    alloc_workspace,
    library_path,
    load_library,
    make_shape,
    moe_combine,
    moe_ffn_backward,
    moe_ffn_debug_set_spin_limit,
    moe_ffn_forward,
    moe_ffn_last_status,
    moe_ffn_workspace_bytes,
    moe_grouped_gemm,
    moe_microbench_last_status,
    moe_microbench_swiglu_add,
    moe_microbench_workspace_bytes,
    moe_grouped_gemm_swiglu,
    moe_permute,
    moe_probe_copy,
    moe_probe_mfma_bf16,
    moe_route,
    moe_status_string,
)
