"""Seeded synthetic inputs for the five workloads.

This module holds no arithmetic of the method itself: it only draws random
tensors of the stated shapes and distributions and rounds them to the storage
type.  Both the CPU oracle's tests and the HIP path's tests are fed from here,
so that they see bit-identical values.

Host generators return float32 numpy arrays whose values are exactly
representable in the storage type (bf16 workloads are rounded to bf16,
round-to-nearest-even, once, here).  Device generators (used at full benchmark
sizes, where drawing 2 GiB on the host would dominate the run) draw with a
seeded ``torch.Generator`` on the GPU and return torch tensors in the storage
type; a slice of such a tensor copied to the host feeds the oracle.

Seeds: ``SEED_BASE + config_index`` (config_index 0..4 in the order of the
workload list below); tensors are drawn in the order Q, K, V / X / X, g, W.
"""
from __future__ import annotations

import math

import numpy as np

SEED_BASE = 20260310

# The five workloads (index = config_index).
WORKLOADS = {
    0: dict(name="attn_fp32_single_head", kind="attention", dtype="f32",
            B=1, Hq=1, Hkv=1, Lq=128, Lk=512, d=64, causal=False),
    1: dict(name="softmax_bf16_32768x4096", kind="softmax", dtype="bf16",
            rows=32768, n=4096, sigma=2.0),
    2: dict(name="attn_prefill_bf16_b4h32l2048d128", kind="attention", dtype="bf16",
            B=4, Hq=32, Hkv=32, Lq=2048, Lk=2048, d=128, causal=False),
    3: dict(name="attn_decode_gqa_bf16_b16h32kv8l32768d128", kind="decode", dtype="bf16",
            B=16, Hq=32, Hkv=8, Lq=1, Lk=32768, d=128, num_splits=64),
    4: dict(name="rmsnorm_gemm_bf16_4096", kind="rmsnorm_gemm", dtype="bf16",
            M=4096, K=4096, N=4096, eps=1e-6, w_sigma=0.02),
}

# Shapes of the paper's appendix tables for the further cascades.
MOE_ROUTING_TABLE = {   # name: (s, hd, en, topk)
    "R1": (2048, 768, 128, 1), "R2": (2048, 1024, 128, 1), "R3": (2048, 4096, 128, 1), "R4": (2048, 2560, 64, 6),
    "R5": (2048, 8192, 64, 8), "R6": (2048, 2048, 64, 6), "R7": (2048, 2048, 128, 8), "R8": (2048, 4096, 128, 8),
}
FP8_QUANT_GEMM_TABLE = {   # name: (M, N, K)
    "Q1": (4096, 1536, 2560), "Q2": (4096, 2560, 1536), "Q3": (4096, 3584, 8192), "Q4": (4096, 8192, 3584),
    "Q5": (4096, 7168, 2048), "Q6": (4096, 2048, 7168), "Q7": (4096, 2048, 768), "Q8": (4096, 768, 2048),
    "Q9": (4096, 4096, 1536), "Q10": (4096, 1536, 4096),
}
VARIANCE_TABLE = {   # name: (bs, l)
    "V1": (1, 8192), "V2": (1, 32768), "V3": (128, 8192), "V4": (128, 32768),
    "V5": (512, 8192), "V6": (512, 32768), "V7": (1024, 8192), "V8": (1024, 32768),
}


def table_workload(key):
    """Workload description (same fields as EXTRA_WORKLOADS) of one row of the tables above."""
    if key in MOE_ROUTING_TABLE:
        s, hd, en, topk = MOE_ROUTING_TABLE[key]
        return dict(name=f"moe_routing_bf16_s{s}_hd{hd}_en{en}_top{topk}", kind="moe_routing", dtype="bf16",
                    S=s, hd=hd, E=en, topk=topk, score_sigma=1.5)
    if key in FP8_QUANT_GEMM_TABLE:
        m, n, k = FP8_QUANT_GEMM_TABLE[key]
        return dict(name=f"fp8_quant_gemm_m{m}_n{n}_k{k}", kind="fp8_quant_gemm", dtype="fp8", M=m, N=n, K=k)
    if key in VARIANCE_TABLE:
        bs, l = VARIANCE_TABLE[key]
        return dict(name=f"variance_f32_{bs}x{l}", kind="variance", dtype="f32", bs=bs, l=l, mu=1.0, sigma=2.0)
    raise KeyError(key)


# Workloads of the paper's further cascades (its appendix tables), largest configurations.
EXTRA_WORKLOADS = {
    "moe_routing_r5": dict(name="moe_routing_bf16_s2048_hd8192_en64_top8", kind="moe_routing", dtype="bf16",
                           S=2048, hd=8192, E=64, topk=8, score_sigma=1.5),
    "moe_routing_r8": dict(name="moe_routing_bf16_s2048_hd4096_en128_top8", kind="moe_routing", dtype="bf16",
                           S=2048, hd=4096, E=128, topk=8, score_sigma=1.5),
    "fp8_quant_gemm_q3": dict(name="fp8_quant_gemm_m4096_n3584_k8192", kind="fp8_quant_gemm", dtype="fp8",
                              M=4096, N=3584, K=8192),
    "fp8_quant_gemm_q4": dict(name="fp8_quant_gemm_m4096_n8192_k3584", kind="fp8_quant_gemm", dtype="fp8",
                              M=4096, N=8192, K=3584),
    "variance_v8": dict(name="variance_f32_1024x32768", kind="variance", dtype="f32",
                        bs=1024, l=32768, mu=1.0, sigma=2.0),
}


# --------------------------------------------------------------------------
# bf16 storage helpers (host)
# --------------------------------------------------------------------------
def bf16_bits(a):
    """float32 array -> uint16 bf16 bit patterns, round-to-nearest-even."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits):
    """uint16 bf16 bit patterns -> float32 array (exact)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(a):
    """float32 array -> float32 array of bf16-representable values (RNE)."""
    return bf16_bits_to_f32(bf16_bits(a))


def e4m3_table():
    """The 256 OCP E4M3 codes decoded to float32 (NaN codes 0x7f / 0xff as nan)."""
    code = np.arange(256, dtype=np.int64)
    sign = np.where(code & 0x80, -1.0, 1.0)
    ex = (code >> 3) & 0xF
    man = code & 0x7
    val = np.where(ex == 0, man / 8.0 * 2.0 ** -6, (1.0 + man / 8.0) * 2.0 ** (ex.astype(np.float64) - 7.0))
    val = np.where((code & 0x7F) == 0x7F, np.nan, sign * val)
    return val.astype(np.float32)


def e4m3_bits(a):
    """float32 array -> uint8 OCP E4M3 codes: nearest code, ties to the even code, |a| > 448 -> 448."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    pos = e4m3_table()[:127].astype(np.float64)          # 0 .. 448, ascending
    x = np.minimum(np.abs(a).astype(np.float64), 448.0)
    hi = np.clip(np.searchsorted(pos, x, side="left"), 1, 126)
    lo = hi - 1
    dlo, dhi = x - pos[lo], pos[hi] - x
    pick_hi = (dhi < dlo) | ((dhi == dlo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    return np.where(np.signbit(a), code | np.uint8(0x80), code).astype(np.uint8)


def e4m3_bits_to_f32(bits):
    return e4m3_table()[np.ascontiguousarray(bits, dtype=np.uint8)]


def _store(a, dtype):
    a = np.asarray(a, dtype=np.float32)
    if dtype == "bf16":
        return bf16_round(a)
    if dtype == "f32":
        return a
    raise ValueError(f"unknown dtype {dtype}")


# --------------------------------------------------------------------------
# host generators
# --------------------------------------------------------------------------
def attention_inputs(seed, B, Hq, Hkv, Lq, Lk, d, dtype):
    """Q[B,Hq,Lq,d], K,V[B,Hkv,Lk,d] i.i.d. N(0,1)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    q = _store(rng.standard_normal((B, Hq, Lq, d), dtype=np.float32), dtype)
    k = _store(rng.standard_normal((B, Hkv, Lk, d), dtype=np.float32), dtype)
    v = _store(rng.standard_normal((B, Hkv, Lk, d), dtype=np.float32), dtype)
    return q, k, v


def softmax_inputs(seed, rows, n, sigma, dtype):
    """X[rows,n] i.i.d. N(0, sigma^2)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal((rows, n), dtype=np.float32) * np.float32(sigma)
    return _store(x, dtype)


def rmsnorm_gemm_inputs(seed, M, K, N, w_sigma=0.02, dtype="bf16"):
    """X[M,K] ~ N(0,1), g[K] ~ U[0.5,1.5), W[K,N] ~ N(0, w_sigma^2)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    x = _store(rng.standard_normal((M, K), dtype=np.float32), dtype)
    g = _store(rng.random(K, dtype=np.float32) + np.float32(0.5), dtype)
    w = _store(rng.standard_normal((K, N), dtype=np.float32) * np.float32(w_sigma), dtype)
    return x, g, w


def variance_inputs(seed, bs, l, dtype="f32", mu=1.0, sigma=2.0):
    """X[bs,l] i.i.d. N(mu, sigma^2); a non-zero mean makes sum(x^2) - (sum x)^2/L cancel."""
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal((bs, l), dtype=np.float32) * np.float32(sigma) + np.float32(mu)
    return _store(x, dtype)


def moe_routing_inputs(seed, S, hd, E, score_sigma=1.5, dtype="bf16"):
    """Tokens X[S,hd] ~ N(0,1), router weights W[hd,E] ~ N(0, score_sigma^2 / hd): scores have
    standard deviation score_sigma, so the softmax over experts is neither flat nor one-hot."""
    rng = np.random.Generator(np.random.PCG64(seed))
    x = _store(rng.standard_normal((S, hd), dtype=np.float32), dtype)
    w = _store(rng.standard_normal((hd, E), dtype=np.float32) * np.float32(score_sigma / math.sqrt(hd)), dtype)
    return x, w


def fp8_quant_gemm_inputs(seed, M, K, N, outlier_rows=8):
    """Activations A[M,K] ~ N(0,1) in bf16, with `outlier_rows` rows carrying a few large entries
    at random positions (what per-token scales exist for; they also make the running maximum
    move late in the row).  Weights W[N,K] ~ N(0,1) rounded to OCP E4M3 (a weight scale is
    taken as folded into the surrounding layer).  Returns (a float32, w float32 of FP8 values,
    w_bits uint8)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    a = rng.standard_normal((M, K), dtype=np.float32)
    rows = rng.choice(M, size=min(outlier_rows, M), replace=False)
    for r in rows:
        cols = rng.choice(K, size=3, replace=False)
        a[r, cols] *= np.float32(30.0)
    a = bf16_round(a)
    w_bits = e4m3_bits(rng.standard_normal((N, K), dtype=np.float32))
    return a, e4m3_bits_to_f32(w_bits), w_bits


def default_scale(d):
    return 1.0 / math.sqrt(d)


# --------------------------------------------------------------------------
# torch plumbing: host array <-> tensor in the storage type
# --------------------------------------------------------------------------
def to_torch(a, dtype, device="cpu"):
    """float32 host array of storage-representable values -> torch tensor."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)          # exact: values are representable
    return t.to(device)


def to_numpy(t):
    """torch tensor (any float dtype, any device) -> float64 host array."""
    import torch
    return t.detach().to("cpu").to(torch.float64).numpy()


# --------------------------------------------------------------------------
# device generators (full benchmark sizes)
# --------------------------------------------------------------------------
def _torch_dtype(dtype):
    import torch
    return {"bf16": torch.bfloat16, "f32": torch.float32}[dtype]


def _randn_device(gen, shape, dtype, device, sigma=1.0, chunk=1 << 27):
    """Draw N(0, sigma^2) on the device in chunks and store in ``dtype``."""
    import torch
    out = torch.empty(shape, dtype=_torch_dtype(dtype), device=device)
    flat = out.view(-1)
    n = flat.numel()
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        t = torch.randn(hi - lo, generator=gen, device=device, dtype=torch.float32)
        if sigma != 1.0:
            t.mul_(sigma)
        flat[lo:hi].copy_(t)
    return out


def attention_inputs_device(seed, B, Hq, Hkv, Lq, Lk, d, dtype, device="cuda:0"):
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    q = _randn_device(gen, (B, Hq, Lq, d), dtype, device)
    k = _randn_device(gen, (B, Hkv, Lk, d), dtype, device)
    v = _randn_device(gen, (B, Hkv, Lk, d), dtype, device)
    return q, k, v


def softmax_inputs_device(seed, rows, n, sigma, dtype, device="cuda:0"):
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    return _randn_device(gen, (rows, n), dtype, device, sigma=sigma)


def variance_inputs_device(seed, bs, l, dtype="f32", mu=1.0, sigma=2.0, device="cuda:0"):
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    x = torch.randn((bs, l), generator=gen, device=device, dtype=torch.float32)
    x.mul_(sigma).add_(mu)
    return x.to(_torch_dtype(dtype))


def moe_routing_inputs_device(seed, S, hd, E, score_sigma=1.5, dtype="bf16", device="cuda:0"):
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    x = _randn_device(gen, (S, hd), dtype, device)
    w = _randn_device(gen, (hd, E), dtype, device, sigma=score_sigma / math.sqrt(hd))
    return x, w


def fp8_quant_gemm_inputs_device(seed, M, K, N, device="cuda:0"):
    """Device-side draw of the same recipe: tokens N(0,1) in bf16 with three entries of eight
    rows blown up by 30, weights N(0,1) rounded to OCP E4M3 (torch.float8_e4m3fn)."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    a = torch.randn((M, K), generator=gen, device=device, dtype=torch.float32)
    rows = torch.randperm(M, generator=gen, device=device)[:min(8, M)]
    cols = torch.randint(0, K, (rows.numel(), 3), generator=gen, device=device)
    a[rows[:, None], cols] *= 30.0
    a = a.to(torch.bfloat16)
    w = torch.randn((N, K), generator=gen, device=device, dtype=torch.float32).clamp_(-448.0, 448.0)
    return a, w.to(torch.float8_e4m3fn)


def rmsnorm_gemm_inputs_device(seed, M, K, N, w_sigma=0.02, dtype="bf16", device="cuda:0"):
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    x = _randn_device(gen, (M, K), dtype, device)
    g = (torch.rand(K, generator=gen, device=device, dtype=torch.float32) + 0.5).to(_torch_dtype(dtype))
    w = _randn_device(gen, (K, N), dtype, device, sigma=w_sigma)
    return x, g, w
