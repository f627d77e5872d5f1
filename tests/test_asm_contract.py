"""The generated code keeps the contract of the assembly loads with register destinations (register-fed row block
of the wide GEMM tile): nothing touches their destination registers between the request and the wait that retires
them.  CPU only: the device code is compiled to assembly and read; the checker itself is tried on planted text."""
import os

import pytest

from paper_2605_23764_amd.asm_check import check_register_fed_loads, device_assembly

GOOD = """
\t.amdhsa_kernel k
k:
\t;;#ASMSTART
\tglobal_load_dwordx4 v[10:13], v166, s[2:3] offset:32
\t;;#ASMEND
\tv_add_u32_e32 v14, v9, v20
\tds_read_b128 v[20:23], v5
\t;;#ASMSTART
\tv_mfma_f32_32x32x16_bf16 v[30:45], v[20:23], v[24:27], v[30:45]
\t;;#ASMEND
\ts_waitcnt vmcnt(8)
\ts_barrier
\t;;#ASMSTART
\ts_waitcnt vmcnt(8)
\t;;#ASMEND
\tv_mov_b32_e32 v50, v10
"""


def test_checker_accepts_a_clean_window_and_names_planted_mistakes():
    assert check_register_fed_loads(GOOD) == (1, [])
    # a copy of a destination register before the naming wait (what the compiler did to a value carried round a loop)
    n, bad = check_register_fed_loads(GOOD.replace("v_add_u32_e32 v14, v9, v20", "v_mov_b32_e32 v60, v12"))
    assert n == 1 and len(bad) == 1 and bad[0][2] == [12]
    # a destination register reused as scratch inside the window
    n, bad = check_register_fed_loads(GOOD.replace("ds_read_b128 v[20:23], v5", "ds_read_b128 v[12:15], v5"))
    assert len(bad) == 1 and bad[0][2] == [12, 13]
    # an MFMA fed from the block before it has been retired
    n, bad = check_register_fed_loads(GOOD.replace("v[20:23], v[24:27]", "v[20:23], v[10:13]"))
    assert len(bad) == 1 and bad[0][2] == [10, 11, 12, 13]
    # the compiler's own wait does not end the window: only the assembly wait that names the registers does
    n, bad = check_register_fed_loads(GOOD.replace("\ts_barrier\n", "\ts_barrier\n\tv_mov_b32_e32 v61, v11\n"))
    assert len(bad) == 1 and bad[0][2] == [11]


@pytest.mark.skipif(not os.path.exists(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")), reason="needs hipcc")
def test_generated_code_keeps_the_window_closed():
    n, bad = check_register_fed_loads(device_assembly())
    # four fragments per request, two requests (prologue, loop) per instantiation of the register-fed tile
    assert n >= 8 and n % 4 == 0, n
    assert not bad, bad[:5]
