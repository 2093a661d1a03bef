"""GPU parity on seeded random shapes: every entry point against the fp64 oracle on
shapes drawn from ranges that cross tile boundaries in every dimension (one query
tile / several, ragged key tails, K and N that are not multiples of the tile).
The draw is deterministic (PCG64 with a fixed seed), so a failure names its shape.
"""
import sys

import numpy as np
import pytest
import torch

from oracle import rf_oracle as O
from paper_2603_10026_amd import inputs as I

sys.path.insert(0, __file__.rsplit("/", 1)[0])
from test_gpu_parity import _fp8_tensor, check, check_routing  # noqa: E402
import fp8_checks as F  # noqa: E402

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def rf():
    from paper_2603_10026_amd import binding
    binding.load_library()
    return binding


def say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def draws(seed, n):
    return [np.random.Generator(np.random.PCG64(seed * 1000 + i)) for i in range(n)]


def test_attention_random_shapes(rf):
    for i, rng in enumerate(draws(11, 24)):
        dtype = "bf16" if i % 4 else "f32"
        d = int(rng.choice([64, 128]))
        hkv = int(rng.choice([1, 2, 3]))
        hq = hkv * int(rng.choice([1, 2, 4]))
        b = int(rng.integers(1, 3))
        lq = int(rng.integers(1, 420)) if dtype == "bf16" else int(rng.integers(1, 50))
        lk = int(rng.integers(1, 520)) if dtype == "bf16" else int(rng.integers(1, 300))
        causal = bool(rng.integers(0, 2))
        say(f"attention #{i} {dtype} B{b} Hq{hq} Hkv{hkv} Lq{lq} Lk{lk} d{d} causal={causal}")
        q, k, v = I.attention_inputs(5000 + i, b, hq, hkv, lq, lk, d, dtype)
        scale = I.default_scale(d) * float(rng.choice([1.0, 0.5, 2.0]))
        o = rf.rf_cascade_attention(*(I.to_torch(a, dtype, DEV) for a in (q, k, v)), scale, causal)
        torch.cuda.synchronize()
        check(o, O.attention(q, k, v, scale, causal), dtype, f"attention #{i}")


def test_splitk_random_shapes(rf):
    for i, rng in enumerate(draws(12, 12)):
        hkv = int(rng.choice([1, 2]))
        hq = hkv * int(rng.choice([1, 4, 8]))
        b = int(rng.integers(1, 3))
        lq = int(rng.choice([1, 1, 1, 2, 5]))
        lk = int(rng.integers(1, 1400))
        s = int(rng.choice([1, 2, 3, 7, 16]))
        causal = bool(rng.integers(0, 2)) and lq > 1
        say(f"splitk #{i} B{b} Hq{hq} Hkv{hkv} Lq{lq} Lk{lk} S{s} causal={causal}")
        q, k, v = I.attention_inputs(6000 + i, b, hq, hkv, lq, lk, 128, "bf16")
        scale = I.default_scale(128)
        tq, tk, tv = (I.to_torch(a, "bf16", DEV) for a in (q, k, v))
        pm, pl, pacc = rf.alloc_partial_states(tq, s)
        pacc.fill_(float("nan"))
        rf.rf_cascade_attention_splitk(tq, tk, tv, s, pm, pl, pacc, scale, causal)
        o = torch.empty_like(tq)
        rf.rf_merge_states(pm, pl, pacc, o)
        torch.cuda.synchronize()
        check(o, O.attention(q, k, v, scale, causal), "bf16", f"splitk+merge #{i}")


def test_softmax_random_shapes(rf):
    for i, rng in enumerate(draws(13, 20)):
        dtype = "bf16" if i % 2 else "f32"
        rows = int(rng.integers(1, 200))
        n = int(rng.choice([rng.integers(1, 64), rng.integers(64, 2100), rng.integers(2100, 12000)]))
        say(f"softmax #{i} {dtype} rows{rows} n{n}")
        x = I.softmax_inputs(7000 + i, rows, n, 2.0, dtype)
        y = rf.rf_safe_softmax(I.to_torch(x, dtype, DEV))
        torch.cuda.synchronize()
        check(y, O.safe_softmax(x), dtype, f"softmax #{i}")


def test_rmsnorm_gemm_random_shapes(rf):
    for i, rng in enumerate(draws(14, 12)):
        m = int(rng.integers(1, 400))
        k = 64 * int(rng.integers(1, 12))
        n = 8 * int(rng.integers(1, 150))
        say(f"rmsnorm_gemm #{i} M{m} K{k} N{n}")
        x, g, w = I.rmsnorm_gemm_inputs(8000 + i, m, k, n)
        y = rf.rf_rmsnorm_gemm(*(I.to_torch(a, "bf16", DEV) for a in (x, g, w)), eps=1e-6)
        torch.cuda.synchronize()
        check(y, O.rmsnorm_gemm(x, g, w, 1e-6), "bf16", f"rmsnorm_gemm #{i}")


def test_fp8_quant_gemm_random_shapes(rf):
    for i, rng in enumerate(draws(15, 12)):
        m = int(rng.integers(1, 400))
        k = 128 * int(rng.integers(1, 9))
        n = 8 * int(rng.integers(1, 150))
        say(f"fp8_quant_gemm #{i} M{m} K{k} N{n}")
        a, w, w_bits = I.fp8_quant_gemm_inputs(9000 + i, m, k, n)
        out = rf.rf_fp8_quant_gemm(I.to_torch(a, "bf16", DEV), _fp8_tensor(w_bits))
        torch.cuda.synchronize()
        F.check(I.to_numpy(out), a, w, f"fp8_quant_gemm #{i}")


def test_variance_random_shapes(rf):
    for i, rng in enumerate(draws(16, 16)):
        dtype = "f32" if i % 2 else "bf16"
        bs = int(rng.integers(1, 70))
        l = int(rng.choice([rng.integers(1, 40), rng.integers(40, 3000), rng.integers(3000, 40000)]))
        say(f"variance #{i} {dtype} bs{bs} l{l}")
        x = I.variance_inputs(10000 + i, bs, l, dtype)
        mean, var = rf.rf_variance(I.to_torch(x, dtype, DEV))
        torch.cuda.synchronize()
        m_ref, v_ref = O.variance(x)
        check(mean, m_ref, "f32", f"variance mean #{i}")
        check(var, v_ref, "f32", f"variance var #{i}")


def test_moe_routing_random_shapes(rf):
    for i, rng in enumerate(draws(17, 12)):
        s = int(rng.integers(1, 300))
        hd = 128 * int(rng.integers(1, 20))
        e = int(rng.choice([32, 64, 128]))
        topk = int(rng.integers(1, min(16, e) + 1))
        say(f"moe_routing #{i} S{s} hd{hd} E{e} topk{topk}")
        x, w = I.moe_routing_inputs(11000 + i, s, hd, e)
        prob, idx = rf.rf_moe_routing(I.to_torch(x, "bf16", DEV), I.to_torch(w, "bf16", DEV), topk)
        torch.cuda.synchronize()
        check_routing(prob, idx, x, w, topk, f"moe_routing #{i}", min_exact=0.8)
