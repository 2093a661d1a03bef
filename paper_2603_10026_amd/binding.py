"""ctypes binding over the C-ABI library ``librf.so``.

Argument marshalling only: every function builds ``rf_tensor`` descriptors
from torch tensors (PyTorch is used for device memory and streams) and calls
the entry point of the same name; all arithmetic runs in the HIP kernels.
There is no fallback: if the library is missing, or an entry point returns an
error, a Python exception is raised.
"""
from __future__ import annotations

import ctypes
import os
import struct

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librf.so")

RF_OK = 0
RF_ERR_INVALID_ARG, RF_ERR_UNSUPPORTED, RF_ERR_ALIGNMENT, RF_ERR_WORKSPACE, RF_ERR_LAUNCH = 1, 2, 3, 4, 5
RF_F32, RF_BF16, RF_I32, RF_FP8_E4M3 = 0, 1, 2, 3
RF_MAX_DIMS = 5

ENTRY_POINTS = (
    "rf_status_string",
    "rf_describe_cascade",
    "rf_safe_softmax",
    "rf_cascade_attention",
    "rf_cascade_attention_splitk",
    "rf_merge_states",
    "rf_rmsnorm_gemm",
    "rf_variance",
    "rf_moe_routing_workspace_bytes",
    "rf_moe_routing",
    "rf_moe_routing_noalloc",
    "rf_fp8_quant_gemm",
)
# measurement aids and the fusion-level study, declared in include/rf_diag.h
DIAG_ENTRY_POINTS = (
    "rf_diag_softmax_level",
    "rf_diag_attention_wide",
    "rf_diag_copy",
    "rf_diag_read",
    "rf_diag_mfma",
)


class RfTensor(ctypes.Structure):
    _fields_ = [
        ("data", ctypes.c_void_p),
        ("dtype", ctypes.c_int),
        ("ndim", ctypes.c_int32),
        ("shape", ctypes.c_int64 * RF_MAX_DIMS),
        ("stride", ctypes.c_int64 * RF_MAX_DIMS),
    ]


class RfStage(ctypes.Structure):
    _fields_ = [("reduce", ctypes.c_int), ("combine", ctypes.c_int)]


class RfError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} ({code})")


_lib = None


def load_library():
    """Load ``librf.so`` (built by ``python -m paper_2603_10026_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2603_10026_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER(RfTensor)
    lib.rf_status_string.restype = ctypes.c_char_p
    lib.rf_status_string.argtypes = [ctypes.c_int]
    lib.rf_describe_cascade.restype = ctypes.c_int
    lib.rf_describe_cascade.argtypes = [ctypes.c_char_p, ctypes.POINTER(RfStage), ctypes.c_int]
    lib.rf_safe_softmax.restype = ctypes.c_int
    lib.rf_safe_softmax.argtypes = [P, P, ctypes.c_int, ctypes.c_void_p]
    lib.rf_cascade_attention.restype = ctypes.c_int
    lib.rf_cascade_attention.argtypes = [P, P, P, P, ctypes.c_float, ctypes.c_int, ctypes.c_void_p]
    lib.rf_cascade_attention_splitk.restype = ctypes.c_int
    lib.rf_cascade_attention_splitk.argtypes = [P, P, P, ctypes.c_int, P, P, P, ctypes.c_float,
                                                ctypes.c_int, ctypes.c_void_p]
    lib.rf_merge_states.restype = ctypes.c_int
    lib.rf_merge_states.argtypes = [P, P, P, P, ctypes.c_void_p]
    lib.rf_rmsnorm_gemm.restype = ctypes.c_int
    lib.rf_rmsnorm_gemm.argtypes = [P, P, P, P, ctypes.c_float, ctypes.c_void_p]
    lib.rf_variance.restype = ctypes.c_int
    lib.rf_variance.argtypes = [P, P, P, ctypes.c_void_p]
    lib.rf_moe_routing_workspace_bytes.restype = ctypes.c_size_t
    lib.rf_moe_routing_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64]
    lib.rf_moe_routing.restype = ctypes.c_int
    lib.rf_moe_routing.argtypes = [P, P, ctypes.c_int, P, P, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.rf_moe_routing_noalloc.restype = ctypes.c_int
    lib.rf_moe_routing_noalloc.argtypes = [P, P, ctypes.c_int, P, P, ctypes.c_void_p]
    lib.rf_fp8_quant_gemm.restype = ctypes.c_int
    lib.rf_fp8_quant_gemm.argtypes = [P, P, P, ctypes.c_void_p]
    lib.rf_diag_softmax_level.restype = ctypes.c_int
    lib.rf_diag_attention_wide.argtypes = [P, P, P, P, ctypes.c_float, ctypes.c_void_p]
    lib.rf_diag_attention_wide.restype = ctypes.c_int
    lib.rf_diag_softmax_level.argtypes = [P, P, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    lib.rf_diag_copy.restype = ctypes.c_int
    lib.rf_diag_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
    lib.rf_diag_read.restype = ctypes.c_int
    lib.rf_diag_read.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
    lib.rf_diag_mfma.restype = ctypes.c_int
    lib.rf_diag_mfma.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    _lib = lib
    return lib


def status_string(code):
    return load_library().rf_status_string(int(code)).decode()


def describe_cascade(entry):
    """List of (reduce, combine) enum pairs of an entry point's cascade."""
    lib = load_library()
    buf = (RfStage * 8)()
    n = lib.rf_describe_cascade(entry.encode(), buf, 8)
    if n < 0:
        raise KeyError(entry)
    return [(buf[i].reduce, buf[i].combine) for i in range(n)]


_DTYPES = {torch.float32: RF_F32, torch.bfloat16: RF_BF16, torch.int32: RF_I32,
           torch.float8_e4m3fn: RF_FP8_E4M3}


_PACK_DESC = struct.Struct("@Pii5q5q").pack        # the byte layout of rf_tensor
_ZEROS = [(0,) * k for k in range(RF_MAX_DIMS + 1)]
assert struct.calcsize("@Pii5q5q") == ctypes.sizeof(RfTensor)


def tensor_desc(t):
    """rf_tensor descriptor of a torch tensor (no copy; strides in elements).
    Packed in one call: per-field ctypes assignments cost more host time than the smaller
    kernels take on the GPU."""
    dt = _DTYPES.get(t.dtype)
    if dt is None:
        raise TypeError(f"unsupported dtype {t.dtype}")
    shape = t.shape
    n = len(shape)
    if n < 1 or n > RF_MAX_DIMS:
        raise ValueError("tensor rank must be 1..5")
    pad = _ZEROS[RF_MAX_DIMS - n]
    return RfTensor.from_buffer_copy(
        _PACK_DESC(0 if 0 in shape else t.data_ptr(), dt, n, *shape, *pad, *t.stride(), *pad))


def _stream(stream):
    """hipStream_t handle: a torch stream, a raw integer handle, or None for
    torch's current stream."""
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    if stream is None:
        try:  # raw handle of the current stream without building a Stream object
            return ctypes.c_void_p(torch._C._cuda_getCurrentRawStream(torch.cuda.current_device()))
        except AttributeError:
            stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(code, where):
    if code != RF_OK:
        raise RfError(code, where)


def rf_safe_softmax(x, y=None, axis=-1, stream=None):
    """y = softmax(x) over the last axis; returns y (allocated if not given)."""
    lib = load_library()
    if y is None:
        y = torch.empty_like(x)
    dx, dy = tensor_desc(x), tensor_desc(y)
    _check(lib.rf_safe_softmax(ctypes.byref(dx), ctypes.byref(dy), int(axis), _stream(stream)),
           "rf_safe_softmax")
    return y


def rf_cascade_attention(q, k, v, scale, causal=False, o=None, stream=None):
    lib = load_library()
    if o is None:
        o = torch.empty_like(q)
    dq, dk, dv, do = tensor_desc(q), tensor_desc(k), tensor_desc(v), tensor_desc(o)
    _check(lib.rf_cascade_attention(ctypes.byref(dq), ctypes.byref(dk), ctypes.byref(dv),
                                    ctypes.byref(do), float(scale), int(bool(causal)),
                                    _stream(stream)), "rf_cascade_attention")
    return o


def alloc_partial_states(q, num_splits):
    """Caller-owned workspace for the multi-segment path."""
    B, Hq, Lq, d = q.shape
    pm = torch.empty((B, Hq, Lq, num_splits), dtype=torch.float32, device=q.device)
    pl = torch.empty((B, Hq, Lq, num_splits), dtype=torch.float32, device=q.device)
    pacc = torch.empty((B, Hq, Lq, num_splits, d), dtype=torch.float32, device=q.device)
    return pm, pl, pacc


def rf_cascade_attention_splitk(q, k, v, num_splits, part_m, part_l, part_acc, scale, causal=False,
                                stream=None):
    lib = load_library()
    dq, dk, dv = tensor_desc(q), tensor_desc(k), tensor_desc(v)
    dm, dl, da = tensor_desc(part_m), tensor_desc(part_l), tensor_desc(part_acc)
    _check(lib.rf_cascade_attention_splitk(ctypes.byref(dq), ctypes.byref(dk), ctypes.byref(dv),
                                           int(num_splits), ctypes.byref(dm), ctypes.byref(dl),
                                           ctypes.byref(da), float(scale), int(bool(causal)),
                                           _stream(stream)), "rf_cascade_attention_splitk")
    return part_m, part_l, part_acc


def rf_merge_states(part_m, part_l, part_acc, o, stream=None):
    lib = load_library()
    dm, dl, da, do = tensor_desc(part_m), tensor_desc(part_l), tensor_desc(part_acc), tensor_desc(o)
    _check(lib.rf_merge_states(ctypes.byref(dm), ctypes.byref(dl), ctypes.byref(da),
                               ctypes.byref(do), _stream(stream)), "rf_merge_states")
    return o


def rf_rmsnorm_gemm(x, g, w, eps=1e-6, y=None, stream=None):
    lib = load_library()
    if y is None:
        y = torch.empty((x.shape[0], w.shape[1]), dtype=x.dtype, device=x.device)
    dx, dg, dw, dy = tensor_desc(x), tensor_desc(g), tensor_desc(w), tensor_desc(y)
    _check(lib.rf_rmsnorm_gemm(ctypes.byref(dx), ctypes.byref(dg), ctypes.byref(dw),
                               ctypes.byref(dy), float(eps), _stream(stream)), "rf_rmsnorm_gemm")
    return y


def rf_variance(x, mean=None, var=None, stream=None):
    """Mean and population variance over the last axis; returns (mean, var), fp32."""
    lib = load_library()
    oshape = tuple(x.shape[:-1]) if x.dim() > 1 else (1,)
    if mean is None:
        mean = torch.empty(oshape, dtype=torch.float32, device=x.device)
    if var is None:
        var = torch.empty(oshape, dtype=torch.float32, device=x.device)
    dx, dm, dv = tensor_desc(x), tensor_desc(mean), tensor_desc(var)
    _check(lib.rf_variance(ctypes.byref(dx), ctypes.byref(dm), ctypes.byref(dv), _stream(stream)),
           "rf_variance")
    return mean, var


def moe_routing_workspace_bytes(S, hd, E):
    return int(load_library().rf_moe_routing_workspace_bytes(int(S), int(hd), int(E)))


def rf_moe_routing(x, w, topk, prob=None, idx=None, workspace=None, stream=None):
    """Router scores -> softmax -> top-k; returns (prob [S,topk] f32, idx [S,topk] i32).
    ``workspace``: a uint8 device tensor of at least moe_routing_workspace_bytes(...) bytes
    (allocated here when omitted)."""
    lib = load_library()
    S, hd = x.shape
    E = w.shape[1]
    if prob is None:
        prob = torch.empty((S, topk), dtype=torch.float32, device=x.device)
    if idx is None:
        idx = torch.empty((S, topk), dtype=torch.int32, device=x.device)
    if workspace is None:
        workspace = torch.empty(max(moe_routing_workspace_bytes(S, hd, E), 16), dtype=torch.uint8, device=x.device)
    dx, dw, dp, di = tensor_desc(x), tensor_desc(w), tensor_desc(prob), tensor_desc(idx)
    _check(lib.rf_moe_routing(ctypes.byref(dx), ctypes.byref(dw), int(topk), ctypes.byref(dp), ctypes.byref(di),
                              ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                              _stream(stream)), "rf_moe_routing")
    return prob, idx


MOE_ROUTING_NOALLOC_MAX_BYTES = 8 << 20


def rf_moe_routing_noalloc(x, w, topk, prob, idx, stream=None):
    """rf_moe_routing with the partial scores in the library's own fixed device array: the call
    allocates nothing, so ``prob`` [S,topk] f32 and ``idx`` [S,topk] i32 must be given."""
    lib = load_library()
    dx, dw, dp, di = tensor_desc(x), tensor_desc(w), tensor_desc(prob), tensor_desc(idx)
    _check(lib.rf_moe_routing_noalloc(ctypes.byref(dx), ctypes.byref(dw), int(topk), ctypes.byref(dp),
                                      ctypes.byref(di), _stream(stream)), "rf_moe_routing_noalloc")
    return prob, idx


def rf_fp8_quant_gemm(a, w, c=None, stream=None):
    """c = dequant(quant_fp8(a) @ w^T): a [M,K] bf16, w [N,K] torch.float8_e4m3fn, c [M,N] bf16."""
    lib = load_library()
    if c is None:
        c = torch.empty((a.shape[0], w.shape[0]), dtype=torch.bfloat16, device=a.device)
    da, dw, dc = tensor_desc(a), tensor_desc(w), tensor_desc(c)
    _check(lib.rf_fp8_quant_gemm(ctypes.byref(da), ctypes.byref(dw), ctypes.byref(dc), _stream(stream)),
           "rf_fp8_quant_gemm")
    return c


def rf_diag_softmax_level(x, y, level, ml_buf=None, stream=None):
    """Softmax with the cascade fused at a chosen level (0 unfused .. 3 per workgroup); study aid."""
    lib = load_library()
    dx, dy = tensor_desc(x), tensor_desc(y)
    p = ctypes.c_void_p(ml_buf.data_ptr()) if ml_buf is not None else None
    _check(lib.rf_diag_softmax_level(ctypes.byref(dx), ctypes.byref(dy), int(level), p, _stream(stream)),
           "rf_diag_softmax_level")
    return y


def rf_diag_attention_wide(q, k, v, scale, o=None, stream=None):
    """The attention cascade (no mask) with 64 query rows per wavefront; tiling study aid."""
    lib = load_library()
    if o is None:
        o = torch.empty_like(q)
    dq, dk, dv, do = tensor_desc(q), tensor_desc(k), tensor_desc(v), tensor_desc(o)
    _check(lib.rf_diag_attention_wide(ctypes.byref(dq), ctypes.byref(dk), ctypes.byref(dv), ctypes.byref(do),
                                      ctypes.c_float(scale), _stream(stream)), "rf_diag_attention_wide")
    return o


def rf_diag_copy(src, dst, stream=None):
    """Plain copy kernel of known size (measurement aid): dst <- src, same byte size."""
    lib = load_library()
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(lib.rf_diag_copy(ctypes.c_void_p(src.data_ptr()), ctypes.c_void_p(dst.data_ptr()),
                            nbytes, _stream(stream)), "rf_diag_copy")
    return dst


DIAG_READ_SINK_BYTES = 8192 * 4 * 4


def rf_diag_read(src, sink, stream=None):
    """Read-only streaming kernel of known size (measurement aid); ``sink``: a device tensor of at
    least DIAG_READ_SINK_BYTES bytes that receives one word per wavefront."""
    lib = load_library()
    nbytes = src.numel() * src.element_size()
    assert sink.numel() * sink.element_size() >= DIAG_READ_SINK_BYTES
    _check(lib.rf_diag_read(ctypes.c_void_p(src.data_ptr()), nbytes, ctypes.c_void_p(sink.data_ptr()),
                            _stream(stream)), "rf_diag_read")
    return sink


def rf_diag_mfma(sink, workgroups, iters, random_operands, stream=None):
    """MFMA-only loop (measurement aid); returns the flop count of the launch."""
    lib = load_library()
    assert sink.dtype == torch.float32 and sink.numel() >= workgroups * 256
    _check(lib.rf_diag_mfma(ctypes.c_void_p(sink.data_ptr()), int(workgroups), int(iters),
                            int(bool(random_operands)), _stream(stream)), "rf_diag_mfma")
    return workgroups * 4 * iters * 32 * 32768.0
