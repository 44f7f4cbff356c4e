"""The compiled gemm_mid kernels: no instruction touches a register between the asynchronous load that writes it
and the point where the kernel has waited for that load (paper_2603_16590_amd/check_async_loads.py); and the
checker itself finds a planted early read and a planted early overwrite in a copy of the listing."""
import re

import pytest

from paper_2603_16590_amd import check_async_loads as chk


@pytest.fixture(scope="module")
def kernels():
    ks = chk.kernels_of(chk.compile_listing())
    assert ks, "the listing holds no gemm_mid kernel"
    return ks


def test_no_register_is_touched_before_its_load_has_landed(kernels):
    for name, lines in kernels.items():
        loads, bad = chk.check_listing(lines)
        assert loads >= 20, (name, loads)
        assert not bad, (name, bad[:5])


def test_checker_finds_planted_mistakes(kernels):
    name, lines = sorted(kernels.items())[0]
    at = [i for i, ln in enumerate(lines) if re.match(r"\tglobal_load_dwordx4 v\[\d+:\d+\],", ln)]
    i = at[len(at) // 2]
    first = re.match(r"\tglobal_load_dwordx4 v\[(\d+):(\d+)\],", lines[i]).group(1)
    early_read = lines[:i + 1] + ["\tv_mov_b32_e32 v1, v%s" % first] + lines[i + 1:]
    early_write = lines[:i + 1] + ["\tv_add_u32_e32 v%s, v2, v3" % first] + lines[i + 1:]
    assert chk.check_listing(early_read)[1]
    assert chk.check_listing(early_write)[1]
