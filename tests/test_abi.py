"""Host-only checks of the C-ABI library: it loads, exports every function the header
declares, and its host-side argument validation returns the documented codes.  No kernel
is launched here."""
import ctypes
import os
import re

import pytest

from paper_2303_06182_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "moe.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2303_06182_amd import build
        build.build()
    return binding.load_library()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_header_functions_are_all_exported(lib):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_capacity_helper(lib):
    # the paper's example: S = 6, C = 0.5 -> 3 rows per expert (Sec. 5.1)
    assert binding.moe_capacity(6, 3, 1, 0.5, binding.MOE_CAPACITY_PAPER) == 3
    assert binding.moe_capacity(65536, 128, 2, 1.0, binding.MOE_CAPACITY_SHARE) == 1024
    assert binding.moe_capacity(65536, 128, 2, 2.0, binding.MOE_CAPACITY_SHARE) == 2048
    assert binding.moe_capacity(100, 8, 2, 1.0, binding.MOE_CAPACITY_SHARE) == 25
    assert binding.moe_capacity(10, 3, 2, 1.0, binding.MOE_CAPACITY_SHARE) == 7
    # waste factors of Sec. 3.2: E * capacity / (2 S) = 12.8 and 64
    S = 4000
    assert 512 * binding.moe_capacity(S, 512, 2, 0.05, binding.MOE_CAPACITY_PAPER) / (2 * S) == pytest.approx(12.8)
    assert 128 * binding.moe_capacity(S, 128, 2, 1.0, binding.MOE_CAPACITY_PAPER) / (2 * S) == pytest.approx(64.0)
    with pytest.raises(binding.MoeError):
        binding.moe_capacity(10, 0, 2, 1.0)
    with pytest.raises(binding.MoeError):
        binding.moe_capacity(10, 4, 2, 1.0, 7)


@pytest.mark.parametrize("kw,code", [
    (dict(dtype=5), binding.MOE_ERR_UNSUPPORTED),
    (dict(E=0), binding.MOE_ERR_UNSUPPORTED),
    (dict(E=2000), binding.MOE_ERR_UNSUPPORTED),
    (dict(k=0), binding.MOE_ERR_UNSUPPORTED),
    (dict(k=9, E=16), binding.MOE_ERR_UNSUPPORTED),
    (dict(k=3, E=2), binding.MOE_ERR_UNSUPPORTED),
    (dict(D=12), binding.MOE_ERR_UNSUPPORTED),
    (dict(F=0), binding.MOE_ERR_UNSUPPORTED),
    (dict(T_max=-1), binding.MOE_ERR_INVALID_ARG),
    (dict(renormalize=2), binding.MOE_ERR_INVALID_ARG),
])
def test_create_rejects_bad_configs_before_touching_the_device(lib, kw, code):
    base = dict(T_max=64, D=64, F=128, E=8, k=2, dtype=binding.MOE_DTYPE_BF16, renormalize=1)
    base.update(kw)
    cfg = binding.MoeConfig(**base)
    h = ctypes.c_void_p()
    rc = lib.moe_create(ctypes.byref(cfg), ctypes.byref(h))
    assert rc == code
    assert not h.value
    assert lib.moe_last_error() != b""


def test_null_handle_and_null_out(lib):
    assert lib.moe_workspace_bytes(None) == binding.MOE_ERR_INVALID_ARG
    cfg = binding.MoeConfig(64, 64, 128, 8, 2, binding.MOE_DTYPE_BF16, 1)
    assert lib.moe_create(ctypes.byref(cfg), None) == binding.MOE_ERR_INVALID_ARG
    assert lib.moe_combine(None, None, None, None, 0, None, None) == binding.MOE_ERR_INVALID_ARG
    assert lib.moe_destroy(None) == binding.MOE_OK


def test_build_reads_register_spills_from_the_compiler_report():
    """The build refuses GEMM kernels that spill registers; this checks its reading of the report."""
    from paper_2303_06182_amd import build
    line = "x.hip:94:1: remark:     %s [-Rpass-analysis=kernel-resource-usage]\n"
    report = ("x.hip:94:1: remark: Function Name: kernel_a [-Rpass-analysis=kernel-resource-usage]\n"
              + line % "VGPRs: 254" + line % "SGPRs Spill: 0" + line % "VGPRs Spill: 0"
              + "x.hip:94:1: remark: Function Name: kernel_b [-Rpass-analysis=kernel-resource-usage]\n"
              + line % "VGPRs: 256" + line % "VGPRs Spill: 119")
    bad = build.spilled_kernels(report)
    assert len(bad) == 1 and bad[0][0].startswith("kernel_b") and bad[0][1] == 119
    assert build.spilled_kernels("") == []
