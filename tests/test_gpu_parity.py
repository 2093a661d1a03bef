"""GPU parity: every entry point of the C-ABI library against the fp64 CPU
oracle, element by element, on seeded inputs that span several tiles and a
ragged tail, plus the degenerate cases.

Tolerances (fixed by the benchmark spec): max|err| <= 1e-5 * max|ref| for
fp32 inputs, <= 2e-2 * max|ref| for bf16 inputs, max|ref| taken over the whole
output tensor.  A relative-RMS bound (much tighter than the max-norm rule) is
asserted as well so that a systematic error cannot hide behind one large
reference value.
"""
import math
import sys

import numpy as np
import pytest
import torch

from oracle import rf_oracle as O
from paper_2603_10026_amd import inputs as I

sys.path.insert(0, __file__.rsplit("/", 1)[0])
import fp8_checks as F  # noqa: E402

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TOL = {"f32": 1e-5, "bf16": 2e-2}
RMS_TOL = {"f32": 2e-6, "bf16": 6e-3}


@pytest.fixture(scope="module")
def rf():
    from paper_2603_10026_amd import binding
    binding.load_library()          # raises if the HIP library is missing
    return binding


def say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def check(out, ref, dtype, what):
    out = I.to_numpy(out)
    ref = np.asarray(ref, dtype=np.float64)
    assert out.shape == ref.shape, (what, out.shape, ref.shape)
    assert np.all(np.isfinite(out)), f"{what}: non-finite output"
    scale = float(np.max(np.abs(ref))) if ref.size else 0.0
    err = float(np.max(np.abs(out - ref))) if ref.size else 0.0
    rms = float(np.sqrt(np.mean((out - ref) ** 2)) / max(np.sqrt(np.mean(ref ** 2)), 1e-300)) if ref.size else 0.0
    print(f"        {what}: max|err|={err:.3e} max|ref|={scale:.3e} ratio={err / max(scale, 1e-300):.2e} relrms={rms:.2e}",
          flush=True)
    assert err <= TOL[dtype] * scale, f"{what}: max|err| {err:.3e} > {TOL[dtype]} * {scale:.3e}"
    assert rms <= RMS_TOL[dtype], f"{what}: rel rms {rms:.3e}"


# ------------------------------------------------------------------ softmax
@pytest.mark.parametrize("dtype,rows,n", [
    ("bf16", 4, 4096), ("bf16", 37, 512), ("bf16", 5, 8), ("bf16", 3, 1000), ("bf16", 130, 2048),
    ("bf16", 7, 1003), ("bf16", 2, 9000), ("bf16", 1, 1), ("bf16", 3, 8192),
    ("f32", 9, 4096), ("f32", 3, 300), ("f32", 2, 5000), ("f32", 6, 1024), ("f32", 5, 7),
    # short rows: several rows per wavefront (2 / 4 / 8 / 16), ragged last wavefront
    ("bf16", 1000, 64), ("bf16", 77, 128), ("bf16", 131, 256), ("bf16", 9, 8), ("bf16", 33, 24), ("bf16", 3, 200),
    ("f32", 50, 128), ("f32", 7, 4), ("f32", 101, 36), ("f32", 1, 64),
    # long rows held in the registers of one workgroup (4 / 8 / 16 wavefronts), then the streaming kernel
    ("bf16", 3, 16384), ("bf16", 2, 40000), ("bf16", 2, 65536), ("f32", 2, 10000), ("f32", 1, 65536), ("f32", 2, 20004),
    ("bf16", 2, 70000), ("f32", 1, 65540),
])
def test_softmax_shapes(rf, dtype, rows, n):
    say(f"softmax {dtype} rows={rows} n={n}")
    x = I.softmax_inputs(I.SEED_BASE + 1, rows, n, 2.0, dtype)
    y = rf.rf_safe_softmax(I.to_torch(x, dtype, DEV))
    torch.cuda.synchronize()
    check(y, O.safe_softmax(x), dtype, "softmax")


def test_softmax_special_rows_and_inplace(rf):
    say("softmax special rows, in place")
    n = 4096
    x = I.softmax_inputs(11, 6, n, 2.0, "bf16")
    x[0, :] = 1.5                      # all equal -> 1/n
    x[1, :] = -3.0
    x[1, 17] = 80.0                    # one dominant logit
    x[2, :] = -80.0
    x[2, 5] = -79.0                    # very negative logits
    x[3, :] = 0.0
    x[3, -1] = 30.0                    # dominant logit in the last lane's tail
    t = I.to_torch(x, "bf16", DEV)
    ref = O.safe_softmax(x)
    y = rf.rf_safe_softmax(t, t)       # in place
    torch.cuda.synchronize()
    assert y.data_ptr() == t.data_ptr()
    check(t, ref, "bf16", "softmax in place")
    out = I.to_numpy(t)
    assert np.all(out[0] == out[0, 0]) and abs(out[0, 0] * n - 1.0) <= 1e-2
    assert out[1, 17] == 1.0


@pytest.mark.parametrize("n", [16384, 70000])
def test_softmax_inplace_long_rows(rf, n):
    """In place (y == x) on the kernels for long rows: one workgroup holding the row in registers
    (n = 16384) and the two-sweep streaming kernel (n = 70000), which reads x twice."""
    say(f"softmax in place, n={n}")
    x = I.softmax_inputs(13, 3, n, 2.0, "bf16")
    t = I.to_torch(x, "bf16", DEV)
    ref = O.safe_softmax(x)
    y = rf.rf_safe_softmax(t, t)
    torch.cuda.synchronize()
    assert y.data_ptr() == t.data_ptr()
    check(t, ref, "bf16", f"softmax in place n={n}")


def test_softmax_strided_rows_and_3d(rf):
    say("softmax pitched 2-D view and contiguous 3-D")
    big = I.softmax_inputs(12, 16, 1024, 2.0, "bf16")
    tb = I.to_torch(big, "bf16", DEV)
    xv = tb[:, :512]                   # row pitch 1024, row length 512
    y = torch.zeros_like(tb)
    rf.rf_safe_softmax(xv, y[:, 512:])
    torch.cuda.synchronize()
    check(y[:, 512:], O.safe_softmax(big[:, :512]), "bf16", "softmax pitched")
    assert float(y[:, :512].abs().max()) == 0.0
    x3 = big.reshape(4, 4, 1024)
    y3 = rf.rf_safe_softmax(I.to_torch(x3, "bf16", DEV))
    torch.cuda.synchronize()
    check(y3, O.safe_softmax(x3), "bf16", "softmax 3-D")
    # odd pitch: rows not 16-byte aligned -> scalar streaming path
    xo = tb[:, 1:1 + 333]
    yo = rf.rf_safe_softmax(xo, torch.empty((16, 333), dtype=torch.bfloat16, device=DEV))
    torch.cuda.synchronize()
    check(yo, O.safe_softmax(big[:, 1:334]), "bf16", "softmax unaligned")


def test_softmax_empty(rf):
    say("softmax empty")
    x = torch.empty((0, 128), dtype=torch.bfloat16, device=DEV)
    assert rf.rf_safe_softmax(x).shape == (0, 128)


# ---------------------------------------------------------------- attention
ATTN_CASES = [
    # dtype, B, Hq, Hkv, Lq, Lk, d, causal
    ("f32", 1, 1, 1, 128, 512, 64, False),      # workload 0
    ("f32", 1, 2, 2, 1, 1, 64, False),
    ("f32", 2, 2, 1, 17, 33, 64, False),
    ("f32", 1, 3, 3, 17, 17, 64, True),
    ("f32", 1, 2, 2, 5, 40, 64, True),
    ("f32", 1, 1, 1, 40, 513, 128, False),
    ("f32", 1, 4, 2, 33, 33, 128, True),
    ("f32", 1, 1, 1, 20, 7, 64, True),          # Lk < Lq: first rows see no key
    ("bf16", 1, 2, 2, 256, 256, 128, False),
    ("bf16", 1, 2, 2, 256, 256, 128, True),
    ("bf16", 2, 4, 2, 130, 193, 128, False),
    ("bf16", 1, 2, 1, 129, 129, 128, True),
    ("bf16", 1, 1, 1, 127, 63, 128, True),      # Lk < Lq
    ("bf16", 1, 2, 2, 1, 300, 128, False),
    ("bf16", 1, 1, 1, 64, 1, 128, False),
    ("bf16", 1, 2, 2, 200, 200, 64, False),
    ("bf16", 1, 2, 1, 200, 260, 64, True),
    ("bf16", 1, 1, 1, 384, 1024, 128, True),
    ("bf16", 1, 2, 1, 300, 450, 128, False),    # 256-query workgroups, ragged second tile
    ("bf16", 2, 2, 2, 513, 129, 64, False),     # 256-query workgroups, one-row tail tile
    ("bf16", 1, 2, 2, 512, 1000, 128, False),   # many key tiles, ragged key tail
    ("bf16", 1, 1, 1, 300, 5, 128, False),      # a single, mostly empty key tile
    ("bf16", 1, 8, 8, 384, 320, 128, False),    # 8 heads: one head per XCD in the tile order
    ("bf16", 1, 8, 8, 384, 320, 128, True),
    # causal launches with enough heads pair a heavy and a light query tile per workgroup
    ("bf16", 1, 128, 16, 1000, 1300, 128, True),   # pairs of 256-query tiles, ragged last tile, Lk > Lq
    ("bf16", 1, 128, 8, 1024, 1100, 64, True),     # the same for head dimension 64
    ("bf16", 1, 176, 8, 700, 700, 128, True),      # pairs of 128-query tiles (odd count of 256-query tiles)
    ("bf16", 1, 176, 8, 768, 768, 64, True),
    ("bf16", 1, 128, 16, 1024, 600, 128, True),    # Lk < Lq: the light tile of each pair sees no key
    # more 256-query workgroups than compute units, with a ragged last query tile
    ("bf16", 1, 160, 8, 500, 300, 128, False),
    ("bf16", 2, 80, 80, 512, 129, 64, False),
    ("bf16", 1, 136, 8, 1000, 1300, 128, True),    # paired causal tiles, more workgroups than compute units
]


@pytest.mark.parametrize("dtype,B,Hq,Hkv,Lq,Lk,d,causal", ATTN_CASES)
def test_attention_shapes(rf, dtype, B, Hq, Hkv, Lq, Lk, d, causal):
    say(f"attention {dtype} B{B} Hq{Hq} Hkv{Hkv} Lq{Lq} Lk{Lk} d{d} causal={causal}")
    q, k, v = I.attention_inputs(I.SEED_BASE, B, Hq, Hkv, Lq, Lk, d, dtype)
    scale = I.default_scale(d)
    o = rf.rf_cascade_attention(I.to_torch(q, dtype, DEV), I.to_torch(k, dtype, DEV),
                                I.to_torch(v, dtype, DEV), scale, causal)
    torch.cuda.synchronize()
    check(o, O.attention(q, k, v, scale, causal), dtype, "attention")


def test_attention_extreme_logits_and_strided_heads(rf):
    say("attention bf16: large logits, [B,L,H,d] memory order")
    B, H, L, d = 1, 2, 160, 128
    q, k, v = I.attention_inputs(77, B, H, H, L, L, d, "bf16")
    q[0, 0, 3] *= 30.0                 # logits of +-100 and more: tests the max subtraction
    k[0, 1, 100] = I.bf16_round(q[0, 1, 50] * 4.0)
    scale = I.default_scale(d)
    # store as [B, L, H, d] and pass permuted views (head stride = d)
    tq, tk, tv = (I.to_torch(np.ascontiguousarray(a.transpose(0, 2, 1, 3)), "bf16", DEV).permute(0, 2, 1, 3)
                  for a in (q, k, v))
    o = torch.empty((B, L, H, d), dtype=torch.bfloat16, device=DEV).permute(0, 2, 1, 3)
    rf.rf_cascade_attention(tq, tk, tv, scale, False, o=o)
    torch.cuda.synchronize()
    check(o, O.attention(q, k, v, scale, False), "bf16", "attention strided")


def test_attention_empty_keys(rf):
    say("attention Lk=0 -> zeros")
    q = torch.ones((1, 1, 5, 64), dtype=torch.float32, device=DEV)
    kv = torch.empty((1, 1, 0, 64), dtype=torch.float32, device=DEV)
    o = rf.rf_cascade_attention(q, kv, kv, 1.0)
    torch.cuda.synchronize()
    assert float(o.abs().max()) == 0.0


WIDE_CASES = [
    # B, Hq, Hkv, Lq, Lk: head dimension 128, no mask, at least 64 keys
    (1, 2, 2, 256, 256),
    (1, 1, 1, 64, 64),          # a single key tile
    (2, 4, 2, 300, 450),        # ragged query tile, ragged last key tile (moved back to end at the last key)
    (1, 8, 8, 384, 320),        # 5 key tiles: three surplus iterations on all-masked tiles
    (1, 2, 1, 512, 1000),
    (1, 3, 3, 1, 65),           # one query row; the second key tile holds one new key
    (1, 160, 8, 500, 300),      # more workgroups than compute units
]


@pytest.mark.parametrize("B,Hq,Hkv,Lq,Lk", WIDE_CASES)
def test_attention_wide_variant(rf, B, Hq, Hkv, Lq, Lk):
    say(f"attention, 64 rows per wavefront: B{B} Hq{Hq} Hkv{Hkv} Lq{Lq} Lk{Lk}")
    q, k, v = I.attention_inputs(I.SEED_BASE + 5, B, Hq, Hkv, Lq, Lk, 128, "bf16")
    scale = I.default_scale(128)
    tq, tk, tv = (I.to_torch(a, "bf16", DEV) for a in (q, k, v))
    o = torch.full_like(tq, float("nan"))
    rf.rf_diag_attention_wide(tq, tk, tv, scale, o=o)
    torch.cuda.synchronize()
    check(o, O.attention(q, k, v, scale, False), "bf16", "attention wide")


def test_attention_wide_variant_scales_and_refusals(rf):
    say("attention, 64 rows per wavefront: negative and zero scale, large logits; unsupported shapes")
    q, k, v = I.attention_inputs(78, 1, 2, 2, 200, 333, 128, "bf16")
    q[0, 0, 3] *= 30.0
    tq, tk, tv = (I.to_torch(a, "bf16", DEV) for a in (q, k, v))
    for scale in (-I.default_scale(128), 0.0):
        o = rf.rf_diag_attention_wide(tq, tk, tv, scale)
        torch.cuda.synchronize()
        check(o, O.attention(q, k, v, scale, False), "bf16", f"attention wide scale={scale}")
    with pytest.raises(rf.RfError):          # fewer than 64 keys
        rf.rf_diag_attention_wide(tq, tk[:, :, :63], tv[:, :, :63], 1.0)
    q64 = torch.zeros((1, 1, 64, 64), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(rf.RfError):          # head dimension 64
        rf.rf_diag_attention_wide(q64, q64, q64, 1.0)


# ------------------------------------------------------------ split + merge
SPLIT_CASES = [
    # B, Hq, Hkv, Lq, Lk, S, causal
    (2, 8, 2, 1, 1000, 4, False),      # chunk 250: not a multiple of the 32-key step
    (1, 4, 1, 1, 100, 64, False),      # chunk 2: most chunks tiny, many empty
    (1, 32, 8, 1, 2048, 4, False),     # workload-3 head layout, chunk 512
    (1, 32, 1, 1, 700, 3, False),      # 32 rows share one KV head: two row tiles
    (1, 4, 2, 3, 300, 5, True),        # Lq > 1, causal, fully masked chunks for early rows
    (1, 2, 2, 1, 1, 1, False),
    # launches of thousands of workgroups, with chunks shorter than one step of the four wavefronts
    # (some wavefronts have no tile in a chunk), chunks past the end of the keys, and two row tiles
    (16, 32, 8, 1, 2560, 64, False),   # chunk 40
    (8, 16, 16, 1, 4229, 128, False),  # chunk 34, the last chunks short or empty
    (8, 24, 8, 7, 2880, 64, True),     # chunk 45, 21 rows per KV head, causal
]


@pytest.mark.parametrize("B,Hq,Hkv,Lq,Lk,S,causal", SPLIT_CASES)
def test_splitk_partial_states_and_merge(rf, B, Hq, Hkv, Lq, Lk, S, causal):
    say(f"splitk B{B} Hq{Hq} Hkv{Hkv} Lq{Lq} Lk{Lk} S{S} causal={causal}")
    d = 128
    q, k, v = I.attention_inputs(I.SEED_BASE + 3, B, Hq, Hkv, Lq, Lk, d, "bf16")
    scale = I.default_scale(d)
    tq, tk, tv = (I.to_torch(a, "bf16", DEV) for a in (q, k, v))
    pm, pl, pacc = rf.alloc_partial_states(tq, S)
    pm.fill_(float("nan")); pl.fill_(float("nan")); pacc.fill_(float("nan"))
    rf.rf_cascade_attention_splitk(tq, tk, tv, S, pm, pl, pacc, scale, causal)
    o = torch.empty_like(tq)
    rf.rf_merge_states(pm, pl, pacc, o)
    torch.cuda.synchronize()
    rm, rl, racc = O.attention_partial_states(q, k, v, scale, causal, S)
    gm, gl, gacc = I.to_numpy(pm), I.to_numpy(pl), I.to_numpy(pacc)
    # identity chunks are exactly (-inf, 0, 0)
    ident = ~np.isfinite(rm)
    assert np.array_equal(ident, ~np.isfinite(gm))
    assert np.all(gm[ident] == -np.inf) and np.all(gl[ident] == 0.0) and np.all(gacc[ident] == 0.0)
    # the state is unique up to the reference point m: compare m, and (l, acc) moved to the oracle's m
    fin = ~ident
    np.testing.assert_allclose(gm[fin], rm[fin], rtol=0, atol=2e-2 * max(1.0, float(np.max(np.abs(rm[fin])))))
    dm = np.zeros_like(rm)
    dm[fin] = gm[fin] - rm[fin]                 # (identity chunks hold -inf on both sides: no difference taken)
    shift = np.where(fin, np.exp(dm), 0.0)
    check(torch.from_numpy(gl * shift), rl, "bf16", "partial l")
    check(torch.from_numpy(gacc * shift[..., None]), racc, "bf16", "partial acc")
    check(o, O.attention(q, k, v, scale, causal), "bf16", "merged == attention over the whole key axis")


@pytest.mark.parametrize("S,d,out_dtype", [(1, 128, "bf16"), (3, 128, "bf16"), (64, 128, "bf16"),
                                           (300, 128, "f32"), (5, 64, "f32"), (7, 4, "f32"), (2, 256, "bf16")])
def test_merge_states_alone(rf, S, d, out_dtype):
    say(f"merge S{S} d{d} -> {out_dtype}")
    rng = np.random.Generator(np.random.PCG64(500 + S))
    B, H, L = 2, 3, 2
    pm = rng.standard_normal((B, H, L, S)).astype(np.float32) * 5.0
    pl = (rng.random((B, H, L, S)).astype(np.float32) + 0.5) * 10.0
    pacc = rng.standard_normal((B, H, L, S, d)).astype(np.float32) * 8.0
    if S >= 3:                          # identity chunks in the middle and at the end
        pm[:, :, :, 1] = -np.inf; pl[:, :, :, 1] = 0.0; pacc[:, :, :, 1] = 0.0
        pm[0, 0, 0, -1] = -np.inf; pl[0, 0, 0, -1] = 0.0; pacc[0, 0, 0, -1] = 0.0
    pm[1, 2, 1, :] = -np.inf; pl[1, 2, 1, :] = 0.0; pacc[1, 2, 1, :] = 0.0     # a row with nothing visible
    o = torch.empty((B, H, L, d), dtype=torch.float32 if out_dtype == "f32" else torch.bfloat16, device=DEV)
    rf.rf_merge_states(*(torch.from_numpy(a).to(DEV) for a in (pm, pl, pacc)), o)
    torch.cuda.synchronize()
    ref = O.merge_states(pm, pl, pacc)
    assert np.all(ref[1, 2, 1] == 0.0)
    check(o, ref, out_dtype, "merge")


# --------------------------------------------------------- RMSNorm + linear
@pytest.mark.parametrize("M,K,N", [(128, 256, 128), (77, 64, 72), (300, 512, 264), (1, 128, 8), (256, 1024, 384)])
def test_rmsnorm_gemm_shapes(rf, M, K, N):
    say(f"rmsnorm_gemm M{M} K{K} N{N}")
    x, g, w = I.rmsnorm_gemm_inputs(I.SEED_BASE + 4, M, K, N)
    y = rf.rf_rmsnorm_gemm(*(I.to_torch(a, "bf16", DEV) for a in (x, g, w)), eps=1e-6)
    torch.cuda.synchronize()
    check(y, O.rmsnorm_gemm(x, g, w, 1e-6), "bf16", "rmsnorm_gemm")


def test_rmsnorm_gemm_row_scales_and_pitched_output(rf):
    say("rmsnorm_gemm rows of very different norm, pitched y")
    M, K, N = 64, 256, 128
    x, g, w = I.rmsnorm_gemm_inputs(91, M, K, N)
    x[0] = I.bf16_round(x[0] * 1e-3)       # tiny row: eps matters
    x[1] = I.bf16_round(x[1] * 300.0)      # huge row
    x[2] = 0.0                             # zero row -> zeros
    x[2, 5] = 0.0
    ybig = torch.zeros((M, 2 * N), dtype=torch.bfloat16, device=DEV)
    rf.rf_rmsnorm_gemm(*(I.to_torch(a, "bf16", DEV) for a in (x, g, w)), eps=1e-6, y=ybig[:, N:])
    torch.cuda.synchronize()
    ref = O.rmsnorm_gemm(x, g, w, 1e-6)
    check(ybig[:, N:], ref, "bf16", "rmsnorm_gemm pitched")
    assert float(ybig[:, :N].abs().max()) == 0.0
    # per-row check so that the small row is not hidden by the large ones
    out = I.to_numpy(ybig[:, N:])
    for i in (0, 1, 3):
        assert np.max(np.abs(out[i] - ref[i])) <= 2e-2 * np.max(np.abs(ref[i]))
    assert np.all(out[2] == 0.0)


# ----------------------------------------------------------------- variance
# Outputs are fp32 and the state arithmetic is fp32 whatever the storage type of x
# (bf16 inputs are exact for both sides), so the fp32 rule applies to both.
@pytest.mark.parametrize("dtype,bs,l", [
    ("f32", 3, 8192), ("f32", 2, 32768), ("f32", 5, 1000), ("f32", 4, 4099), ("f32", 7, 3), ("f32", 2, 1),
    ("f32", 1, 70001), ("bf16", 3, 8192), ("bf16", 4, 1003), ("bf16", 2, 9), ("bf16", 130, 2048),
    # rows that end in one chunk of every size (8, 4, 2, 1 vectors per lane), a partial vector round and
    # a ragged tail: 4-wavefront kernel, then the 16-wavefront kernel (few long rows), fp32 and bf16
    ("f32", 3, 11666), ("f32", 300, 15669), ("f32", 2, 62643), ("bf16", 2, 125285), ("bf16", 3, 31339),
])
def test_variance_shapes(rf, dtype, bs, l):
    say(f"variance {dtype} bs={bs} l={l}")
    x = I.variance_inputs(I.SEED_BASE + 6, bs, l, dtype)
    mean, var = rf.rf_variance(I.to_torch(x, dtype, DEV))
    torch.cuda.synchronize()
    m_ref, v_ref = O.variance(x)
    check(mean, m_ref, "f32", "variance mean")
    check(var, v_ref, "f32", "variance var")


def test_variance_large_offset_unaligned_and_pitched(rf):
    say("variance: mean >> spread, unaligned rows, pitched rows, 1-D, 3-D")
    # mean 1000, sigma 0.5: sum(x^2) - (sum x)^2/L would lose every digit in fp32
    x = I.variance_inputs(77, 4, 5000, "f32", mu=1000.0, sigma=0.5)
    mean, var = rf.rf_variance(I.to_torch(x, "f32", DEV))
    m_ref, v_ref = O.variance(x)
    check(mean, m_ref, "f32", "variance mean (offset)")
    out = I.to_numpy(var)
    assert np.max(np.abs(out - v_ref)) <= 2e-4 * np.max(v_ref), (out, v_ref)   # input rounding at 1000 is 6e-5
    # constant rows: variance exactly 0
    c = torch.full((3, 777), 2.5, device=DEV)
    mean, var = rf.rf_variance(c)
    assert torch.all(mean == 2.5) and torch.all(var == 0.0)
    # rows at an odd element offset (no 128-bit loads) and with a pitch
    x = I.variance_inputs(78, 6, 1001, "f32")
    big = torch.zeros((6, 1030), device=DEV)
    big[:, 3:1004] = I.to_torch(x, "f32", DEV)
    mean, var = rf.rf_variance(big[:, 3:1004])
    m_ref, v_ref = O.variance(x)
    check(mean, m_ref, "f32", "variance mean (unaligned, pitched)")
    check(var, v_ref, "f32", "variance var (unaligned, pitched)")
    # 1-D and 3-D inputs
    mean, var = rf.rf_variance(I.to_torch(x[0], "f32", DEV))
    assert mean.shape == (1,)
    check(var, v_ref[:1], "f32", "variance var (1-D)")
    x3 = I.variance_inputs(79, 6, 512, "bf16").reshape(2, 3, 512)
    mean, var = rf.rf_variance(I.to_torch(x3, "bf16", DEV))
    m_ref, v_ref = O.variance(x3)
    check(mean, m_ref, "f32", "variance mean (3-D)")
    check(var, v_ref, "f32", "variance var (3-D)")
    torch.cuda.synchronize()


# -------------------------------------------------------------- MoE routing
def check_routing(prob, idx, x, w, topk, what, min_exact=0.9):
    """GPU routing against the fp64 oracle.  The scores are accumulated in fp32 on the GPU, so
    two experts whose fp64 scores differ by less than that arithmetic's error may be ordered
    either way: what is unique is compared exactly, the rest is checked to be valid."""
    prob = I.to_numpy(prob)
    idx = idx.detach().cpu().numpy().astype(np.int64)
    p_ref, i_ref, p = O.moe_routing(x, w, topk)
    S, E = p.shape
    assert prob.shape == (S, topk) and idx.shape == (S, topk)
    assert np.all(np.isfinite(prob))
    assert np.all((idx >= 0) & (idx < E)), f"{what}: expert index out of range"
    delta = 4e-6 * max(1.0, float(np.max(np.abs(p))))          # fp32 accumulation error of a score
    m = p.max(axis=1, keepdims=True)
    soft = np.exp(p - m) / np.exp(p - m).sum(axis=1, keepdims=True)
    exact = 0
    for i in range(S):
        sel = idx[i]
        assert len(set(sel.tolist())) == topk, f"{what}: row {i} selects an expert twice"
        ps = p[i, sel]
        assert np.all(ps[:-1] >= ps[1:] - delta), f"{what}: row {i} not in descending order"
        rest = np.delete(p[i], sel)
        if rest.size:
            assert rest.max() <= ps[-1] + delta, f"{what}: row {i} misses a larger score"
        # decisions that the arithmetic cannot flip must match the oracle exactly
        srt = np.sort(p[i])[::-1][:topk + 1]
        if np.all(srt[:-1] - srt[1:] > 2 * delta):
            assert np.array_equal(sel, i_ref[i]), f"{what}: row {i}: {sel} != {i_ref[i]}"
            exact += 1
        # probabilities of the experts it chose
        np.testing.assert_allclose(prob[i], soft[i, sel], rtol=2e-4, atol=1e-7,
                                   err_msg=f"{what}: row {i} probabilities")
    err = float(np.max(np.abs(np.sort(prob, axis=1) - np.sort(p_ref, axis=1))))
    print(f"        {what}: rows with margin-safe decisions {exact}/{S}, max|prob err|={err:.2e}", flush=True)
    assert exact >= min_exact * S
    assert err <= 1e-5 * float(np.max(p_ref)) + 1e-7


@pytest.mark.parametrize("S,hd,E,topk", [
    (128, 256, 64, 6), (100, 128, 32, 1), (300, 768, 128, 1), (64, 1024, 128, 8), (257, 512, 64, 8),
    (1, 128, 128, 16), (70, 2560, 64, 6), (33, 384, 32, 16),
])
def test_moe_routing_shapes(rf, S, hd, E, topk):
    say(f"moe_routing S{S} hd{hd} E{E} top{topk}")
    x, w = I.moe_routing_inputs(I.SEED_BASE + 5, S, hd, E)
    prob, idx = rf.rf_moe_routing(I.to_torch(x, "bf16", DEV), I.to_torch(w, "bf16", DEV), topk)
    torch.cuda.synchronize()
    check_routing(prob, idx, x, w, topk, "moe_routing")


def test_moe_routing_exact_ties_and_pitched_outputs(rf):
    say("moe_routing: exactly representable scores (many exact ties), pitched outputs, reused workspace")
    # x in {-1, 0, 1} and w in multiples of 1/4: every partial sum is exact in fp32 in any
    # order, so the GPU scores equal the fp64 ones bit for bit and ties are exact ties.
    S, hd, E, topk = 96, 256, 64, 8
    rng = np.random.Generator(np.random.PCG64(501))
    x = rng.integers(-1, 2, size=(S, hd)).astype(np.float32)
    w = rng.integers(-2, 3, size=(hd, E)).astype(np.float32) * 0.25
    w[:, 40] = w[:, 3]            # duplicated experts on top of the accidental ties
    w[:, 18] = w[:, 17]
    w[:, 60] = w[:, 17]
    x[5] = 0.0                    # all scores equal: experts 0..k-1, probability 1/E each
    ws = torch.empty(rf.moe_routing_workspace_bytes(S, hd, E), dtype=torch.uint8, device=DEV)
    pbig = torch.zeros((S, 2 * topk), dtype=torch.float32, device=DEV)
    ibig = torch.full((S, 2 * topk), -7, dtype=torch.int32, device=DEV)
    for rep in range(2):          # the second call reuses the workspace as the first left it
        rf.rf_moe_routing(I.to_torch(x, "bf16", DEV), I.to_torch(w, "bf16", DEV), topk,
                          prob=pbig[:, topk:], idx=ibig[:, :topk], workspace=ws)
    torch.cuda.synchronize()
    assert float(pbig[:, :topk].abs().max()) == 0.0 and int((ibig[:, topk:] != -7).sum()) == 0
    prob, idx = I.to_numpy(pbig[:, topk:]), ibig[:, :topk].cpu().numpy().astype(np.int64)
    p_ref, i_ref, p = O.moe_routing(x, w, topk)
    n_ties = sum(len(set(np.sort(p[i])[::-1][:topk + 1].tolist())) < topk + 1 for i in range(S))
    print(f"        rows with a tie among their top {topk + 1} scores: {n_ties}/{S}", flush=True)
    assert n_ties > S // 4
    np.testing.assert_array_equal(idx, i_ref)                 # bit-exact decisions, ties included
    np.testing.assert_allclose(prob, p_ref, rtol=2e-5, atol=1e-8)
    assert list(idx[5]) == list(range(topk)) and np.all(prob[5] == np.float32(1.0 / E))


# ------------------------------------------------- FP8 per-token quant + GEMM
def _fp8_tensor(w_bits):
    return torch.from_numpy(np.ascontiguousarray(w_bits)).to(DEV).view(torch.float8_e4m3fn)


@pytest.mark.parametrize("M,K,N", [(128, 256, 512), (77, 128, 72), (300, 512, 264), (1, 128, 8), (256, 1024, 1032),
                                   (130, 384, 520),
                                   # more than 256 tiles of 256 channels: the 512-channel tiling, with a ragged
                                   # last tile in both directions
                                   (1152, 256, 7424), (1100, 384, 7400)])
def test_fp8_quant_gemm_shapes(rf, M, K, N):
    say(f"fp8_quant_gemm M{M} K{K} N{N}")
    a, w, w_bits = I.fp8_quant_gemm_inputs(I.SEED_BASE + 7, M, K, N)
    first = list(range(0, M, 3))               # these tokens have their maximum in the first element
    a[first, 0] = I.bf16_round(1.5 * np.max(np.abs(a[first]), axis=1))
    c = rf.rf_fp8_quant_gemm(I.to_torch(a, "bf16", DEV), _fp8_tensor(w_bits))
    torch.cuda.synchronize()
    # against the two-pass definition, within quantisation noise (no knowledge of the kernel's segments)
    F.check(I.to_numpy(c), a, w, "fp8_quant_gemm", first_max_rows=first)


def test_fp8_quant_gemm_special_rows_and_pitched_output(rf):
    say("fp8_quant_gemm: zero token, late maximum, maximum first, scaled tokens, exact tokens, pitched c")
    M, K, N = 64, 1024, 128
    a, w, w_bits = I.fp8_quant_gemm_inputs(93, M, K, N, outlier_rows=0)
    a[0] = 0.0                                  # all-zero token -> zeros
    a[1, K - 1] = 200.0                         # maximum arrives last: everything before it is rescaled
    a[2, 0] = 200.0                             # maximum first: the two-pass definition itself
    a[3] = I.bf16_round(a[3] * 1e-3)            # small token: its own scale
    a[4] = I.bf16_round(a[4] * 1e3)
    # tokens made of powers of two whose maximum keeps moving (2^-7 ... 2^0 in rising runs): MAX a / m'
    # is an FP8 value for every prefix maximum m', so any segmentation must return a @ w^T itself
    rng = np.random.Generator(np.random.PCG64(94))
    for r in (5, 6, 7):
        e = np.sort(rng.integers(-7, 1, size=K)) if r != 7 else rng.integers(-7, 1, size=K)
        a[r] = (np.exp2(e) * rng.choice([-1.0, 1.0], size=K)).astype(np.float32)
    cbig = torch.zeros((M, 2 * N), dtype=torch.bfloat16, device=DEV)
    rf.rf_fp8_quant_gemm(I.to_torch(a, "bf16", DEV), _fp8_tensor(w_bits), c=cbig[:, N:])
    torch.cuda.synchronize()
    out = I.to_numpy(cbig[:, N:])
    assert float(cbig[:, :N].abs().max()) == 0.0
    assert np.all(out[0] == 0.0)
    F.check(out, a, w, "fp8_quant_gemm special rows", first_max_rows=[2])
    exact = a.astype(np.float64) @ w.astype(np.float64).T
    for r in (5, 6, 7):                         # exact up to fp32 accumulation and the bf16 rounding of c
        assert np.max(np.abs(out[r] - exact[r])) <= 2.0 ** -7 * np.max(np.abs(exact[r])), r


# ------------------------------------------- softmax fused at different levels
@pytest.mark.parametrize("level", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("rows,n", [(37, 512), (9, 4096), (5, 8192), (130, 1000)])
def test_softmax_fusion_levels(rf, level, rows, n):
    say(f"softmax fusion level {level} rows={rows} n={n}")
    x = I.softmax_inputs(I.SEED_BASE + 1, rows, n, 2.0, "bf16")
    tx = I.to_torch(x, "bf16", DEV)
    ty = torch.empty_like(tx)
    ml = torch.full((8 * rows,), float("nan"), dtype=torch.float32, device=DEV)
    rf.rf_diag_softmax_level(tx, ty, level, ml)
    torch.cuda.synchronize()
    check(ty, O.safe_softmax(x), "bf16", f"softmax level {level}")


# --------------------------------------------------------- measurement aids
def test_diag_copy_and_read(rf):
    say("diag copy / read-only aids")
    g = torch.Generator(device=DEV)
    g.manual_seed(5)
    n = (1 << 20) + 4 * 77                       # 128-bit vectors, not a multiple of the workgroup share
    src = torch.randint(-2**31, 2**31 - 1, (n,), dtype=torch.int32, device=DEV, generator=g)
    dst = torch.zeros_like(src)
    rf.rf_diag_copy(src, dst)
    sink = torch.zeros(rf.DIAG_READ_SINK_BYTES // 4, dtype=torch.int32, device=DEV)
    rf.rf_diag_read(src, sink)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    # every word is read exactly once: the XOR of the per-workgroup words is the XOR of the data
    want = np.bitwise_xor.reduce(src.cpu().numpy().view(np.uint32))
    got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))
    assert int(want) == int(got)
