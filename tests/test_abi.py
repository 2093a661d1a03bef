"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, describes its cascades, and rejects bad
arguments with the documented status codes before any launch."""
import ctypes
import os
import re

import pytest
import torch

from paper_2603_10026_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2603_10026_amd import build
        build.build_library(verbose=False)
    return B.load_library()


def _declared_symbols(header="rf.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    return sorted(set(re.findall(r"RF_API\s+[\w\s\*]+?\b(rf_\w+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    assert _declared_symbols("rf.h") == sorted(B.ENTRY_POINTS)
    assert _declared_symbols("rf_diag.h") == sorted(B.DIAG_ENTRY_POINTS)
    assert not any(n.startswith("rf_diag") for n in _declared_symbols("rf.h"))


def test_library_exports_every_declared_symbol(lib):
    for header in ("rf.h", "rf_diag.h"):
        for name in _declared_symbols(header):
            assert hasattr(lib, name), name


def test_headers_compile_as_c_and_agree_with_the_binding(tmp_path):
    """rf.h and rf_diag.h are C headers: a C compiler accepts them, and the struct layout and
    enum values it sees are the ones the Python binding hard-codes."""
    import shutil
    import subprocess
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "layout.c"
    src.write_text(r"""
#include <stdio.h>
#include <stddef.h>
#include "rf.h"
#include "rf_diag.h"
int main(void) {
  printf("sizeof_rf_tensor %zu\n", sizeof(rf_tensor));
  printf("off_data %zu\noff_dtype %zu\noff_ndim %zu\noff_shape %zu\noff_stride %zu\n",
         offsetof(rf_tensor, data), offsetof(rf_tensor, dtype), offsetof(rf_tensor, ndim),
         offsetof(rf_tensor, shape), offsetof(rf_tensor, stride));
  printf("sizeof_rf_stage %zu\n", sizeof(rf_stage));
  printf("RF_MAX_DIMS %d\n", RF_MAX_DIMS);
  printf("RF_OK %d\nRF_ERR_INVALID_ARG %d\nRF_ERR_UNSUPPORTED %d\nRF_ERR_ALIGNMENT %d\n"
         "RF_ERR_WORKSPACE %d\nRF_ERR_LAUNCH %d\n", RF_OK, RF_ERR_INVALID_ARG, RF_ERR_UNSUPPORTED,
         RF_ERR_ALIGNMENT, RF_ERR_WORKSPACE, RF_ERR_LAUNCH);
  printf("RF_F32 %d\nRF_BF16 %d\nRF_I32 %d\nRF_FP8_E4M3 %d\n", RF_F32, RF_BF16, RF_I32, RF_FP8_E4M3);
  printf("RF_RED_MAX %d\nRF_RED_MIN %d\nRF_RED_SUM %d\nRF_COMB_ADD %d\nRF_COMB_MUL %d\n",
         RF_RED_MAX, RF_RED_MIN, RF_RED_SUM, RF_COMB_ADD, RF_COMB_MUL);
  printf("RF_DIAG_READ_SINK_BYTES %d\n", RF_DIAG_READ_SINK_BYTES);
  printf("RF_MOE_ROUTING_NOALLOC_MAX_BYTES %zu\n", RF_MOE_ROUTING_NOALLOC_MAX_BYTES);
  return 0;
}
""")
    exe = tmp_path / "layout"
    subprocess.run([cc, "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    got = {k: int(v) for k, v in (ln.split() for ln in out.splitlines())}
    T = B.RfTensor
    assert got["sizeof_rf_tensor"] == ctypes.sizeof(T) == 96
    for f in ("data", "dtype", "ndim", "shape", "stride"):
        assert got["off_" + f] == getattr(T, f).offset, f
    assert got["sizeof_rf_stage"] == ctypes.sizeof(B.RfStage)
    assert got["RF_MAX_DIMS"] == B.RF_MAX_DIMS
    for name in ("RF_OK", "RF_ERR_INVALID_ARG", "RF_ERR_UNSUPPORTED", "RF_ERR_ALIGNMENT", "RF_ERR_WORKSPACE",
                 "RF_ERR_LAUNCH", "RF_F32", "RF_BF16", "RF_I32", "RF_FP8_E4M3"):
        assert got[name] == getattr(B, name), name
    assert (got["RF_RED_MAX"], got["RF_RED_MIN"], got["RF_RED_SUM"]) == (0, 1, 2)
    assert (got["RF_COMB_ADD"], got["RF_COMB_MUL"]) == (0, 1)
    assert got["RF_DIAG_READ_SINK_BYTES"] == B.DIAG_READ_SINK_BYTES
    assert got["RF_MOE_ROUTING_NOALLOC_MAX_BYTES"] == B.MOE_ROUTING_NOALLOC_MAX_BYTES


def test_status_strings(lib):
    assert B.status_string(0) == "RF_OK"
    assert B.status_string(B.RF_ERR_ALIGNMENT) == "RF_ERR_ALIGNMENT"
    assert B.status_string(99) == "RF_ERR_UNKNOWN"


def test_describe_cascade(lib):
    MAX, SUM, ADD, MUL = 0, 2, 0, 1
    assert B.describe_cascade("rf_safe_softmax") == [(MAX, ADD), (SUM, MUL)]
    assert B.describe_cascade("rf_cascade_attention") == [(MAX, ADD), (SUM, MUL), (SUM, MUL)]
    assert B.describe_cascade("rf_rmsnorm_gemm") == [(SUM, MUL), (SUM, MUL)]
    with pytest.raises(KeyError):
        B.describe_cascade("nope")


def _desc(shape, dtype=B.RF_BF16, data=0x1000, stride=None):
    d = B.RfTensor()
    d.data = data
    d.dtype = dtype
    d.ndim = len(shape)
    st = 1
    strides = [0] * len(shape)
    for i in range(len(shape) - 1, -1, -1):
        strides[i] = st
        st *= shape[i]
    if stride is not None:
        strides = list(stride)
    for i, s in enumerate(shape):
        d.shape[i] = s
        d.stride[i] = strides[i]
    return d


def _r(x):
    return ctypes.byref(x)


def test_softmax_validation(lib):
    x, y = _desc([4, 64]), _desc([4, 64])
    assert lib.rf_safe_softmax(None, _r(y), -1, None) == B.RF_ERR_INVALID_ARG
    assert lib.rf_safe_softmax(_r(x), _r(_desc([4, 32])), -1, None) == B.RF_ERR_INVALID_ARG
    assert lib.rf_safe_softmax(_r(x), _r(_desc([4, 64], dtype=B.RF_F32)), -1, None) == B.RF_ERR_UNSUPPORTED
    assert lib.rf_safe_softmax(_r(x), _r(y), 0, None) == B.RF_ERR_UNSUPPORTED      # not the last axis
    assert lib.rf_safe_softmax(_r(x), _r(y), 2, None) == B.RF_ERR_INVALID_ARG
    assert lib.rf_safe_softmax(_r(_desc([4, 64], data=None)), _r(y), -1, None) == B.RF_ERR_INVALID_ARG
    assert lib.rf_safe_softmax(_r(_desc([4, 64], stride=[128, 2])), _r(y), -1, None) == B.RF_ERR_UNSUPPORTED
    # zero-sized problem: OK, nothing launched
    assert lib.rf_safe_softmax(_r(_desc([0, 64], data=None)), _r(_desc([0, 64], data=None)), -1, None) == B.RF_OK


def test_attention_validation(lib):
    q, k, v, o = _desc([2, 8, 16, 128]), _desc([2, 2, 32, 128]), _desc([2, 2, 32, 128]), _desc([2, 8, 16, 128])
    f = lib.rf_cascade_attention
    assert f(None, _r(k), _r(v), _r(o), 1.0, 0, None) == B.RF_ERR_INVALID_ARG
    assert f(_r(q), _r(_desc([2, 3, 32, 128])), _r(_desc([2, 3, 32, 128])), _r(o), 1.0, 0, None) == B.RF_ERR_INVALID_ARG
    assert f(_r(q), _r(k), _r(_desc([2, 2, 31, 128])), _r(o), 1.0, 0, None) == B.RF_ERR_INVALID_ARG
    assert f(_r(q), _r(_desc([2, 2, 32, 128], dtype=B.RF_F32)), _r(v), _r(o), 1.0, 0, None) == B.RF_ERR_UNSUPPORTED
    q96 = _desc([2, 8, 16, 96])
    kv96 = _desc([2, 2, 32, 96])
    assert f(_r(q96), _r(kv96), _r(kv96), _r(_desc([2, 8, 16, 96])), 1.0, 0, None) == B.RF_ERR_UNSUPPORTED
    assert f(_r(_desc([2, 8, 16, 128], data=0x1008)), _r(k), _r(v), _r(o), 1.0, 0, None) == B.RF_ERR_ALIGNMENT
    assert f(_r(q), _r(k), _r(v), _r(_desc([2, 8, 16, 64])), 1.0, 0, None) == B.RF_ERR_INVALID_ARG


def test_splitk_and_merge_validation(lib):
    q, k, v = _desc([2, 8, 1, 128]), _desc([2, 2, 64, 128]), _desc([2, 2, 64, 128])
    F32 = B.RF_F32
    pm, pl, pa = _desc([2, 8, 1, 4], F32), _desc([2, 8, 1, 4], F32), _desc([2, 8, 1, 4, 128], F32)
    f = lib.rf_cascade_attention_splitk
    assert f(_r(q), _r(k), _r(v), 0, _r(pm), _r(pl), _r(pa), 1.0, 0, None) == B.RF_ERR_INVALID_ARG
    assert f(_r(q), _r(k), _r(v), 5, _r(pm), _r(pl), _r(pa), 1.0, 0, None) == B.RF_ERR_WORKSPACE
    assert f(_r(q), _r(k), _r(v), 4, _r(_desc([2, 8, 1, 4])), _r(pl), _r(pa), 1.0, 0, None) == B.RF_ERR_WORKSPACE
    qf = _desc([2, 8, 1, 128], F32)
    kf = _desc([2, 2, 64, 128], F32)
    assert f(_r(qf), _r(kf), _r(kf), 4, _r(pm), _r(pl), _r(pa), 1.0, 0, None) == B.RF_ERR_UNSUPPORTED
    q64, k64 = _desc([2, 8, 1, 64]), _desc([2, 2, 64, 64])
    pa64 = _desc([2, 8, 1, 4, 64], F32)
    assert f(_r(q64), _r(k64), _r(k64), 4, _r(pm), _r(pl), _r(pa64), 1.0, 0, None) == B.RF_ERR_UNSUPPORTED
    o = _desc([2, 8, 1, 128])
    g = lib.rf_merge_states
    assert g(_r(pm), _r(pl), _r(pa), None, None) == B.RF_ERR_INVALID_ARG
    assert g(_r(pm), _r(_desc([2, 8, 1, 5], F32)), _r(pa), _r(o), None) == B.RF_ERR_WORKSPACE
    assert g(_r(pm), _r(pl), _r(pa), _r(_desc([2, 8, 1, 64])), None) == B.RF_ERR_INVALID_ARG
    assert g(_r(pm), _r(pl), _r(_desc([2, 8, 1, 4, 128], F32, data=0x1004)), _r(o), None) == B.RF_ERR_ALIGNMENT


def test_rmsnorm_gemm_validation(lib):
    x, g, w, y = _desc([16, 128]), _desc([128]), _desc([128, 64]), _desc([16, 64])
    f = lib.rf_rmsnorm_gemm
    assert f(_r(x), _r(g), _r(w), None, 1e-6, None) == B.RF_ERR_INVALID_ARG
    assert f(_r(x), _r(_desc([64])), _r(w), _r(y), 1e-6, None) == B.RF_ERR_INVALID_ARG
    assert f(_r(x), _r(g), _r(_desc([128, 64], dtype=B.RF_F32)), _r(y), 1e-6, None) == B.RF_ERR_UNSUPPORTED
    assert f(_r(_desc([16, 96])), _r(_desc([96])), _r(_desc([96, 64])), _r(y), 1e-6, None) == B.RF_ERR_UNSUPPORTED
    assert f(_r(x), _r(g), _r(_desc([128, 60])), _r(_desc([16, 60])), 1e-6, None) == B.RF_ERR_UNSUPPORTED
    assert f(_r(x), _r(g), _r(_desc([128, 64], data=0x1002)), _r(y), 1e-6, None) == B.RF_ERR_ALIGNMENT
    assert f(_r(_desc([0, 128], data=None)), _r(g), _r(w), _r(_desc([0, 64], data=None)), 1e-6, None) == B.RF_OK
    # row pitches the kernel's 32-bit tile offsets cannot express are refused, not wrapped
    big = 1 << 24
    assert f(_r(_desc([16, 128], stride=[big, 1])), _r(g), _r(w), _r(y), 1e-6, None) == B.RF_ERR_UNSUPPORTED
    assert f(_r(x), _r(g), _r(_desc([128, 64], stride=[big, 1])), _r(y), 1e-6, None) == B.RF_ERR_UNSUPPORTED


def test_variance_validation(lib):
    F32 = B.RF_F32
    x, m, v = _desc([8, 256], F32), _desc([8], F32), _desc([8], F32)
    f = lib.rf_variance
    assert f(None, _r(m), _r(v), None) == B.RF_ERR_INVALID_ARG
    assert f(_r(x), _r(_desc([7], F32)), _r(_desc([7], F32)), None) == B.RF_ERR_INVALID_ARG
    assert f(_r(x), _r(_desc([8])), _r(v), None) == B.RF_ERR_UNSUPPORTED          # outputs must be f32
    assert f(_r(_desc([8, 0], F32)), _r(m), _r(v), None) == B.RF_ERR_INVALID_ARG  # empty rows
    assert f(_r(_desc([8, 256], F32, stride=[512, 2])), _r(m), _r(v), None) == B.RF_ERR_UNSUPPORTED
    assert f(_r(_desc([8, 256], F32, data=None)), _r(m), _r(v), None) == B.RF_ERR_INVALID_ARG
    assert f(_r(_desc([0, 256], F32, data=None)), _r(_desc([0], F32, data=None)), _r(_desc([0], F32, data=None)), None) == B.RF_OK
    assert B.describe_cascade("rf_variance") == [(2, 1), (2, 1)]                  # (sum, *) twice


def test_moe_routing_validation(lib):
    F32, I32 = B.RF_F32, B.RF_I32
    x, w = _desc([64, 256]), _desc([256, 64])
    p, i = _desc([64, 4], F32), _desc([64, 4], I32)
    f = lib.rf_moe_routing
    need = lib.rf_moe_routing_workspace_bytes(64, 256, 64)
    assert need >= 64 * 64 * 4 and need % (64 * 64 * 4) == 0
    ws = ctypes.c_void_p(0x10000)
    assert f(None, _r(w), 4, _r(p), _r(i), ws, need, None) == B.RF_ERR_INVALID_ARG
    assert f(_r(x), _r(_desc([128, 64])), 4, _r(p), _r(i), ws, need, None) == B.RF_ERR_INVALID_ARG
    assert f(_r(x), _r(w), 0, _r(p), _r(i), ws, need, None) == B.RF_ERR_INVALID_ARG
    assert f(_r(x), _r(w), 5, _r(p), _r(i), ws, need, None) == B.RF_ERR_INVALID_ARG       # outputs are [64, 4]
    assert f(_r(x), _r(w), 4, _r(p), _r(_desc([64, 4], F32)), ws, need, None) == B.RF_ERR_UNSUPPORTED
    assert f(_r(_desc([64, 256], F32)), _r(w), 4, _r(p), _r(i), ws, need, None) == B.RF_ERR_UNSUPPORTED
    assert f(_r(_desc([64, 192])), _r(_desc([192, 64])), 4, _r(p), _r(i), ws, need, None) == B.RF_ERR_UNSUPPORTED
    assert f(_r(x), _r(_desc([256, 48])), 4, _r(p), _r(i), ws, need, None) == B.RF_ERR_UNSUPPORTED
    p17, i17 = _desc([64, 17], F32), _desc([64, 17], I32)
    assert f(_r(x), _r(w), 17, _r(p17), _r(i17), ws, need, None) == B.RF_ERR_UNSUPPORTED
    assert f(_r(_desc([64, 256], data=0x1008)), _r(w), 4, _r(p), _r(i), ws, need, None) == B.RF_ERR_ALIGNMENT
    assert f(_r(x), _r(w), 4, _r(p), _r(i), None, need, None) == B.RF_ERR_WORKSPACE
    assert f(_r(x), _r(w), 4, _r(p), _r(i), ws, need - 1, None) == B.RF_ERR_WORKSPACE
    assert f(_r(x), _r(w), 4, _r(p), _r(i), ctypes.c_void_p(0x10004), need, None) == B.RF_ERR_WORKSPACE
    # an integer tensor where a floating one is expected is refused, not reinterpreted
    assert lib.rf_safe_softmax(_r(_desc([4, 64], I32)), _r(_desc([4, 64], I32)), -1, None) == B.RF_ERR_UNSUPPORTED
    e0, p0, i0 = _desc([0, 256], data=None), _desc([0, 4], F32, data=None), _desc([0, 4], I32, data=None)
    assert f(_r(e0), _r(w), 4, _r(p0), _r(i0), None, 0, None) == B.RF_OK
    # the entry point that allocates nothing: same argument checks, and a problem whose partial
    # scores do not fit the library's fixed array is refused before any launch
    g = lib.rf_moe_routing_noalloc
    assert g(None, _r(w), 4, _r(p), _r(i), None) == B.RF_ERR_INVALID_ARG
    assert g(_r(x), _r(w), 5, _r(p), _r(i), None) == B.RF_ERR_INVALID_ARG
    assert g(_r(_desc([64, 192])), _r(_desc([192, 64])), 4, _r(p), _r(i), None) == B.RF_ERR_UNSUPPORTED
    assert g(_r(e0), _r(w), 4, _r(p0), _r(i0), None) == B.RF_OK
    Sbig = 1 << 16
    assert lib.rf_moe_routing_workspace_bytes(Sbig, 256, 64) > B.MOE_ROUTING_NOALLOC_MAX_BYTES
    assert g(_r(_desc([Sbig, 256])), _r(w), 4, _r(_desc([Sbig, 4], F32)), _r(_desc([Sbig, 4], I32)), None) == B.RF_ERR_WORKSPACE
    assert B.describe_cascade("rf_moe_routing") == [(0, 0), (2, 1), (0, 0)]      # max, sum, top-k (max-type)


def test_fp8_quant_gemm_validation(lib):
    F8 = B.RF_FP8_E4M3
    a, w, c = _desc([64, 256]), _desc([128, 256], F8), _desc([64, 128])
    f = lib.rf_fp8_quant_gemm
    assert f(None, _r(w), _r(c), None) == B.RF_ERR_INVALID_ARG
    assert f(_r(a), _r(_desc([128, 128], F8)), _r(c), None) == B.RF_ERR_INVALID_ARG     # K mismatch
    assert f(_r(a), _r(w), _r(_desc([64, 120])), None) == B.RF_ERR_INVALID_ARG
    assert f(_r(a), _r(_desc([128, 256])), _r(c), None) == B.RF_ERR_UNSUPPORTED         # weights must be FP8
    assert f(_r(_desc([64, 256], F8)), _r(w), _r(c), None) == B.RF_ERR_UNSUPPORTED      # tokens must be bf16
    assert f(_r(_desc([64, 192])), _r(_desc([128, 192], F8)), _r(c), None) == B.RF_ERR_UNSUPPORTED
    assert f(_r(a), _r(_desc([124, 256], F8)), _r(_desc([64, 124])), None) == B.RF_ERR_UNSUPPORTED
    assert f(_r(a), _r(_desc([128, 256], F8, data=0x1004)), _r(c), None) == B.RF_ERR_ALIGNMENT
    assert f(_r(_desc([0, 256], data=None)), _r(w), _r(_desc([0, 128], data=None)), None) == B.RF_OK
    # FP8 is refused where an entry point does not ask for it
    assert lib.rf_safe_softmax(_r(_desc([4, 64], F8)), _r(_desc([4, 64], F8)), -1, None) == B.RF_ERR_UNSUPPORTED
    assert B.describe_cascade("rf_fp8_quant_gemm") == [(0, 0), (2, 1)]                  # max, then sum


def test_binding_descriptor_from_torch_tensor():
    t = torch.zeros((3, 4, 8), dtype=torch.bfloat16)[:, 1:3]
    d = B.tensor_desc(t)
    assert d.ndim == 3 and list(d.shape[:3]) == [3, 2, 8] and list(d.stride[:3]) == [32, 8, 1]
    assert d.dtype == B.RF_BF16 and d.data == t.data_ptr()
    with pytest.raises(TypeError):
        B.tensor_desc(torch.zeros(4, dtype=torch.float16))


def test_tensor_descriptor_fields():
    """The packed descriptor carries pointer, dtype, rank, shape and element strides field by field."""
    import ctypes
    import torch
    from paper_2603_10026_amd import binding as B
    t = torch.empty(2, 3, 4, 5, 6, dtype=torch.bfloat16).permute(0, 2, 1, 3, 4)
    d = B.tensor_desc(t)
    assert ctypes.sizeof(d) == 96
    assert d.data == t.data_ptr() and d.dtype == B.RF_BF16 and d.ndim == 5
    assert list(d.shape) == [2, 4, 3, 5, 6] and list(d.stride) == list(t.stride())
    d = B.tensor_desc(torch.empty(7, dtype=torch.int32))
    assert d.dtype == B.RF_I32 and d.ndim == 1 and list(d.shape) == [7, 0, 0, 0, 0] and list(d.stride) == [1, 0, 0, 0, 0]
    d = B.tensor_desc(torch.empty(0, 4))
    assert d.data is None and d.dtype == B.RF_F32 and list(d.shape)[:2] == [0, 4]
    with pytest.raises(TypeError):
        B.tensor_desc(torch.empty(3, dtype=torch.float64))
    with pytest.raises(ValueError):
        B.tensor_desc(torch.empty(1, 1, 1, 1, 1, 1))
