"""The compiled packed-operand kernel never reads the registers of a weight-fragment load before the load's wait
(a compiler-inserted copy between the two would carry what has not arrived): checked on the gfx950 assembly of
gemm.hip, which hipcc produces without a GPU."""
import shutil

import pytest

from paper_2401_15207_amd import isa_check


def test_checker_flags_a_copy_behind_a_load():
    planted = "\n".join([
        "_ZN4hift12_GLOBAL__N_19gemm_pk_kILi4ELb1EfLi0EEEvNS0_5GemmPEPKDv4_jl:",
        "\tbuffer_load_dwordx4 v[4:7], v254, s[4:7], s22 offen",
        "\tv_accvgpr_write_b32 a235, v7",
        "\ts_waitcnt vmcnt(0)",
        "\tv_mfma_f32_32x32x16_bf16 a[0:15], v[4:7], v[8:11], a[0:15]",
        ".Lfunc_end0:",
    ])
    loads, bad = isa_check.early_reads_of_async_loads(planted)["_ZN4hift12_GLOBAL__N_19gemm_pk_kILi4ELb1EfLi0EEEvNS0_5GemmPEPKDv4_jl"]
    assert loads == 1 and len(bad) == 1
    clean = planted.replace("\tv_accvgpr_write_b32 a235, v7\n", "")
    loads, bad = isa_check.early_reads_of_async_loads(clean)["_ZN4hift12_GLOBAL__N_19gemm_pk_kILi4ELb1EfLi0EEEvNS0_5GemmPEPKDv4_jl"]
    assert loads == 1 and not bad


@pytest.mark.skipif(shutil.which("hipcc") is None and not __import__("os").path.exists("/opt/rocm/bin/hipcc"),
                    reason="needs hipcc")
def test_compiled_kernel_reads_no_fragment_before_its_wait():
    res = isa_check.early_reads_of_async_loads(isa_check.device_assembly("gemm.hip"))
    assert len(res) >= 7, sorted(res)            # every instantiation of the kernel was found
    for name, (loads, bad) in res.items():
        assert loads >= 50, (name, loads)        # and its fragment loads were recognised
        assert not bad, (name, bad[:3])
