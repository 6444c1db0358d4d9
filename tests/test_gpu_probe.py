"""The device ceilings probe behind `bench.py --ceilings` (a library of its own, not part of the MoE
path): runs with small sizes and must report rates that are positive and below the datasheet peaks."""
import ctypes

import pytest

from paper_2605_02960_amd import build as moe_build

pytestmark = pytest.mark.gpu


def test_ceilings_probe_reports_plausible_rates():
    import torch
    torch.cuda.set_device(0)
    torch.cuda.synchronize()
    lib = ctypes.CDLL(moe_build.PROBE_LIB)
    lib.moe_probe_ceilings.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.c_ulonglong, ctypes.c_int, ctypes.c_int]
    lib.moe_probe_ceilings.restype = ctypes.c_int
    r = (ctypes.c_double * 4)()
    print("case ceilings probe: 256 MiB streams, 2000 MFMA iterations", flush=True)
    assert lib.moe_probe_ceilings(r, 256 << 20, 2000, 2) == 0
    bf16, fp8, rd, wr = list(r)
    print(f"  bf16 {bf16:.0f} TFLOP/s, fp8 {fp8:.0f} TFLOP/s, read {rd:.2f} TB/s, write {wr:.2f} TB/s")
    assert 500.0 < bf16 <= 2500.0 * 1.02
    assert 1000.0 < fp8 <= 5000.0 * 1.02
    assert bf16 < fp8
    # 256 MiB fits the memory-side cache, so these may exceed what HBM streams; they must still be finite and sane
    assert 0.5 < rd < 40.0
    assert 0.5 < wr < 40.0


def test_l2_delivery_probe_reports_plausible_rates():
    import torch
    torch.cuda.set_device(0)
    torch.cuda.synchronize()
    lib = ctypes.CDLL(moe_build.PROBE_LIB)
    lib.moe_probe_l2_paths.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.c_int, ctypes.c_int]
    lib.moe_probe_l2_paths.restype = ctypes.c_int
    r = (ctypes.c_double * 2)()
    print("case L2 delivery probe: 500 iterations of 64 KB per CU", flush=True)
    assert lib.moe_probe_l2_paths(r, 500, 2) == 0
    to_lds, to_reg = list(r)
    print(f"  L2 -> LDS {to_lds:.1f} TB/s, L2 -> registers {to_reg:.1f} TB/s (all CUs)")
    # 256 CUs x 64 B per clock x 2.4 GHz = 39 TB/s is what the L2-to-CU path could carry at most
    assert 1.0 < to_lds < 45.0
    assert 1.0 < to_reg < 45.0
