"""CPU-side checks of the C-ABI library: it loads, exports every function the header declares,
and rejects bad arguments on the host before touching a device."""
import ctypes
import os
import re

import pytest

import paper_2605_02960_amd as moe
from paper_2605_02960_amd import build as moe_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    moe_build.ensure_built()
    return moe.lib()


def header_functions():
    src = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("moe_prefill.h", "moe_sched.h"))
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", src)))


def test_exports_match_header(L):
    names = header_functions()
    assert set(names) == set(moe.EXPORTED_SYMBOLS)
    for n in names:
        assert hasattr(L, n), n
    assert moe.moe_abi_version() == 1


def test_status_strings(L):
    seen = {moe.moe_status_string(s) for s in range(0, -9, -1)}
    assert len(seen) == 9 and "ok" in seen
    assert moe.moe_status_string(-99) == "unknown status"


def test_config_validation_and_workspace(L):
    ok = moe.make_config(8192, 4096, 128, 8, 1536, moe.DTYPE_BF16, moe.DTYPE_BF16)
    sizes = [moe.moe_workspace_bytes(ok, c) for c in range(5)]
    assert sizes[moe.CALL_COMBINE] == 0
    assert sizes[moe.CALL_ROUTE] == 8192 * 128 * 4 + 3 * 128 * 4096 * 2      # logits + bf16 split of the router weight
    assert sizes[moe.CALL_PREFILL_LAYER] > sizes[moe.CALL_GROUPED_FFN] >= 65536 * 1536 * 2
    assert all(s % 256 == 0 for s in sizes)
    bad = [
        (dict(K=0), -2), (dict(K=129), -2), (dict(K=33, E=64), -2), (dict(E=1025), -2), (dict(T=-1), -2),
        (dict(H=4032), -2), (dict(I=1472), -2), (dict(x_dtype=2), -3), (dict(w_dtype=7), -3),
        (dict(w_dtype=moe.DTYPE_F32), -3), (dict(out_dtype=2), -3), (dict(flags=2), -6), (dict(flags=5), -6),
        (dict(T=2 ** 28), -2),
    ]
    for change, want in bad:
        f = dict(T=8192, H=4096, E=128, K=8, I=1536, x_dtype=1, w_dtype=1, out_dtype=0, flags=0)
        f.update(change)
        c = moe.MoEConfig(**f)
        n = ctypes.c_size_t(0)
        assert L.moe_workspace_bytes(ctypes.byref(c), 4, ctypes.byref(n)) == want, change
    n = ctypes.c_size_t(0)
    assert L.moe_workspace_bytes(None, 0, ctypes.byref(n)) == -1
    assert L.moe_workspace_bytes(ctypes.byref(ok), 0, None) == -1
    assert L.moe_workspace_bytes(ctypes.byref(ok), 9, ctypes.byref(n)) == -6


def test_argument_errors_leave_before_any_launch(L):
    """Null and misaligned arguments are rejected on the host (no GPU needed to see that)."""
    c = moe.make_config(64, 128, 8, 2, 128, moe.DTYPE_BF16, moe.DTYPE_BF16)
    p = ctypes.c_void_p
    fake = p(0x1000)        # never dereferenced: validation fails first
    assert L.moe_route(ctypes.byref(c), None, fake, None, fake, fake, fake, None, 0, None) == -1
    assert L.moe_route(ctypes.byref(c), fake, fake, None, None, fake, fake, None, 0, None) == -1     # no logits, no ws
    assert L.moe_route(ctypes.byref(c), fake, fake, None, None, fake, fake, p(0x1010), 1 << 30, None) == -4
    assert L.moe_route(ctypes.byref(c), fake, fake, None, None, fake, fake, fake, 16, None) == -5
    assert L.moe_permute(ctypes.byref(c), fake, None, fake, fake, fake, fake, fake, fake, 1 << 20, None) == -1  # x_perm without x
    assert L.moe_permute(ctypes.byref(c), fake, None, fake, fake, fake, fake, None, fake, 0, None) == -5
    assert L.moe_grouped_ffn(ctypes.byref(c), fake, fake, fake, fake, fake, fake, None, None, None, None, None,
                             None, fake, fake, 0, None) == -5
    assert L.moe_grouped_ffn(ctypes.byref(c), p(0x1008), fake, fake, fake, fake, fake, None, None, None, None,
                             None, None, fake, fake, 1 << 30, None) == -4
    assert L.moe_combine(ctypes.byref(c), fake, fake, None, fake, None) == -1
    assert L.moe_prefill_layer(ctypes.byref(c), fake, fake, None, fake, fake, fake, None, None, None, fake, None,
                               fake, 1024, None) == -5
    c8 = moe.make_config(64, 256, 8, 2, 256, moe.DTYPE_BF16, moe.DTYPE_FP8_E4M3)
    assert L.moe_grouped_ffn(ctypes.byref(c8), fake, fake, fake, fake, fake, fake, None, None, None, None, None,
                             None, fake, fake, 1 << 30, None) == -1   # fp8 needs scales
    assert L.moe_quantize_rows_e4m3(fake, 4, 12, fake, fake, None) == -2
    assert L.moe_quantize_rows_e4m3(None, 4, 16, fake, fake, None) == -1


def test_ceilings_probe_library_loads():
    """The probe behind `bench.py --ceilings` is a library of its own: it loads and exports its one call
    (no GPU call is made here)."""
    lib = ctypes.CDLL(moe_build.PROBE_LIB)
    assert hasattr(lib, "moe_probe_ceilings")


@pytest.mark.parametrize("compiler,std,lang", [("gcc", "-std=c99", "c"), ("g++", "-std=c++11", "c++")])
def test_public_headers_are_plain_c(tmp_path, compiler, std, lang):
    """The boundary is a C ABI: both headers compile as strict C99 and as C++11 with nothing else included."""
    import subprocess
    src = tmp_path / "hdr.c"
    src.write_text('#include "moe_prefill.h"\n#include "moe_sched.h"\n'
                   "int main(void) { moe_config_t c; (void)c; return 0; }\n")
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    subprocess.check_call([compiler, std, "-x", lang, "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", inc,
                           "-fsyntax-only", str(src)])
