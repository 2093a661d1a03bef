"""GPU parity at the full benchmark sizes, in the launch configuration that
bench.py times.  The inputs are generated on the device from the benchmark
seeds; the oracle is evaluated on sampled outputs it can compute one by one
(rows of softmax / attention / GEMM, whole (batch, head) pairs of decode), on
host copies of exactly the device values.  Properties that hold at any size
(softmax rows sum to one) are checked on the whole output.

Tolerance as in the small-size tests: max|err| <= tol * max|ref| with
max|ref| over the sampled reference values (a subset of the full tensor, hence
never looser than the full-tensor rule would be by more than sampling noise;
the per-row relative check below is stricter than either).
"""
import sys

import numpy as np
import pytest
import torch

from oracle import rf_oracle as O
from paper_2603_10026_amd import inputs as I

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
W = I.WORKLOADS


@pytest.fixture(scope="module")
def rf():
    from paper_2603_10026_amd import binding
    binding.load_library()
    return binding


def say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def check_rows(out_rows, ref_rows, tol, what, row_tol=None):
    out_rows = np.asarray(out_rows, dtype=np.float64)
    ref_rows = np.asarray(ref_rows, dtype=np.float64)
    assert np.all(np.isfinite(out_rows)), what
    scale = float(np.max(np.abs(ref_rows)))
    err = float(np.max(np.abs(out_rows - ref_rows)))
    print(f"        {what}: {len(ref_rows)} sampled rows, max|err|={err:.3e} max|ref|={scale:.3e} "
          f"ratio={err / scale:.2e}", flush=True)
    assert err <= tol * scale, what
    if row_tol is not None:     # every sampled row against its own scale
        for o, r in zip(out_rows, ref_rows):
            assert np.max(np.abs(o - r)) <= row_tol * np.max(np.abs(r)), what


def test_workload0_attention_f32_full(rf):
    c = W[0]
    say(c["name"])
    q, k, v = I.attention_inputs_device(I.SEED_BASE + 0, c["B"], c["Hq"], c["Hkv"], c["Lq"], c["Lk"], c["d"], "f32", DEV)
    sc = I.default_scale(c["d"])
    o = rf.rf_cascade_attention(q, k, v, sc, False)
    torch.cuda.synchronize()
    ref = O.attention(I.to_numpy(q), I.to_numpy(k), I.to_numpy(v), sc, False)
    out = I.to_numpy(o)
    err, scale = np.max(np.abs(out - ref)), np.max(np.abs(ref))
    print(f"        full output: max|err|={err:.3e} max|ref|={scale:.3e}", flush=True)
    assert err <= 1e-5 * scale


def test_workload1_softmax_full(rf):
    c = W[1]
    say(c["name"])
    x = I.softmax_inputs_device(I.SEED_BASE + 1, c["rows"], c["n"], c["sigma"], "bf16", DEV)
    y = rf.rf_safe_softmax(x)
    torch.cuda.synchronize()
    # property over the whole output: rows sum to 1 (bf16 output rounding: 4096 terms of 2^-9 relative error)
    sums = y.to(torch.float32).sum(dim=1)
    assert float((sums - 1.0).abs().max()) < 5e-3
    assert bool((y >= 0).all())
    rng = np.random.Generator(np.random.PCG64(11))
    rows = np.unique(np.concatenate([[0, 1, c["rows"] - 1, c["rows"] - 2, 3, 4 * 8191 + 3],
                                     rng.integers(0, c["rows"], size=58)]))
    xs = I.to_numpy(x[torch.from_numpy(rows).to(DEV)])
    ys = I.to_numpy(y[torch.from_numpy(rows).to(DEV)])
    check_rows(ys, O.safe_softmax(xs), 2e-2, "softmax rows", row_tol=2e-2)


@pytest.mark.parametrize("causal", [False, True])
def test_workload2_prefill_full(rf, causal):
    c = W[2]
    say(f"{c['name']} causal={causal}")
    q, k, v = I.attention_inputs_device(I.SEED_BASE + 2, c["B"], c["Hq"], c["Hkv"], c["Lq"], c["Lk"], c["d"], "bf16", DEV)
    sc = I.default_scale(c["d"])
    o = rf.rf_cascade_attention(q, k, v, sc, causal)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(o.to(torch.float32)).all())
    rng = np.random.Generator(np.random.PCG64(12))
    # two whole heads (first and last) + scattered rows incl. tile boundaries and the first/last query
    L = c["Lq"]
    picks = [(0, 0, i) for i in (0, 1, 31, 32, 63, 64, 127, 128, 129, 1023, 1024, L - 2, L - 1)]
    picks += [(c["B"] - 1, c["Hq"] - 1, i) for i in (0, 5, 127, 128, 2047)]
    picks += [(int(rng.integers(c["B"])), int(rng.integers(c["Hq"])), int(rng.integers(L))) for _ in range(46)]
    heads = sorted({(b, h) for b, h, _ in picks})
    host = {bh: tuple(I.to_numpy(t[bh[0], bh[1]])[None, None] for t in (q, k, v)) for bh in heads}
    outs, refs = [], []
    for (b, h, i) in picks:
        qh, kh, vh = host[(b, h)]
        refs.append(O.attention_rows(qh, kh, vh, sc, causal, [(0, 0, i)])[0])
        outs.append(I.to_numpy(o[b, h, i]))
    # under the causal mask row 0 equals V[0] (|ref| ~ 4) while late rows are ~0.05: the per-row
    # check (5e-2 of the row's own max) keeps those rows honest
    check_rows(outs, refs, 2e-2, "prefill rows", row_tol=5e-2)


def test_workload3_decode_full(rf):
    c = W[3]
    say(c["name"])
    q, k, v = I.attention_inputs_device(I.SEED_BASE + 3, c["B"], c["Hq"], c["Hkv"], c["Lq"], c["Lk"], c["d"], "bf16", DEV)
    sc = I.default_scale(c["d"])
    S = c["num_splits"]
    pm, pl, pacc = rf.alloc_partial_states(q, S)
    rf.rf_cascade_attention_splitk(q, k, v, S, pm, pl, pacc, sc, False)
    o = rf.rf_merge_states(pm, pl, pacc, torch.empty_like(q))
    torch.cuda.synchronize()
    assert bool(torch.isfinite(o.to(torch.float32)).all())
    grp = c["Hq"] // c["Hkv"]
    outs, refs = [], []
    for (b, hk) in [(0, 0), (c["B"] - 1, c["Hkv"] - 1), (7, 3)]:
        kh, vh = (I.to_numpy(t[b, hk])[None, None] for t in (k, v))
        qh = I.to_numpy(q[b, hk * grp:(hk + 1) * grp])[None]          # the 4 query heads of this KV head
        ref = O.attention(qh, kh, vh, sc, False)[0]                   # [grp, 1, d]
        refs.extend(ref[:, 0, :])
        outs.extend(I.to_numpy(o[b, hk * grp:(hk + 1) * grp, 0]))
        # the partial states of this group against the oracle's, chunk by chunk
        rm, rl, racc = O.attention_partial_states(qh, kh, vh, sc, False, S)
        gm = I.to_numpy(pm[b, hk * grp:(hk + 1) * grp])[None]
        gl = I.to_numpy(pl[b, hk * grp:(hk + 1) * grp])[None]
        ga = I.to_numpy(pacc[b, hk * grp:(hk + 1) * grp])[None]
        shift = np.exp(gm - rm)
        assert np.max(np.abs(gm - rm)) < 1e-3
        assert np.max(np.abs(gl * shift - rl)) <= 2e-2 * np.max(np.abs(rl))
        assert np.max(np.abs(ga * shift[..., None] - racc)) <= 2e-2 * np.max(np.abs(racc))
    check_rows(outs, refs, 2e-2, "decode rows (3 KV heads x 4 query heads)", row_tol=2e-2)


def test_workload4_rmsnorm_gemm_full(rf):
    c = W[4]
    say(c["name"])
    x, g, w = I.rmsnorm_gemm_inputs_device(I.SEED_BASE + 4, c["M"], c["K"], c["N"], c["w_sigma"], "bf16", DEV)
    y = rf.rf_rmsnorm_gemm(x, g, w, eps=c["eps"])
    torch.cuda.synchronize()
    assert bool(torch.isfinite(y.to(torch.float32)).all())
    rng = np.random.Generator(np.random.PCG64(14))
    rows = np.unique(np.concatenate([[0, 1, 127, 128, 255, 256, 257, c["M"] - 1], rng.integers(0, c["M"], size=24)]))
    idx = torch.from_numpy(rows).to(DEV)
    ref = O.rmsnorm_gemm(I.to_numpy(x[idx]), I.to_numpy(g), I.to_numpy(w), c["eps"])
    check_rows(I.to_numpy(y[idx]), ref, 2e-2, "rmsnorm_gemm rows", row_tol=2e-2)


@pytest.mark.parametrize("key", sorted(I.VARIANCE_TABLE, key=lambda k: int(k[1:])))
def test_variance_full(rf, key):
    c = I.table_workload(key)
    say(f"{key} {c['name']}")
    x = I.variance_inputs_device(I.SEED_BASE + 6, c["bs"], c["l"], c["dtype"], c["mu"], c["sigma"], DEV)
    mean, var = rf.rf_variance(x)
    torch.cuda.synchronize()
    m_ref, v_ref = O.variance(I.to_numpy(x))                 # every row: the oracle takes seconds
    check_rows(I.to_numpy(mean)[:, None], m_ref[:, None], 1e-5, "variance mean")
    check_rows(I.to_numpy(var)[:, None], v_ref[:, None], 1e-5, "variance var", row_tol=1e-5)


@pytest.mark.parametrize("key", sorted(I.MOE_ROUTING_TABLE))
def test_moe_routing_full(rf, key):
    c = I.table_workload(key)
    say(f"{key} {c['name']}")
    x, w = I.moe_routing_inputs_device(I.SEED_BASE + 5, c["S"], c["hd"], c["E"], c["score_sigma"], "bf16", DEV)
    prob, idx = rf.rf_moe_routing(x, w, c["topk"])
    torch.cuda.synchronize()
    p_ref, i_ref, p = O.moe_routing(I.to_numpy(x), I.to_numpy(w), c["topk"])   # every token
    prob, idx = I.to_numpy(prob), idx.cpu().numpy().astype(np.int64)
    S, E = p.shape
    delta = 4e-6 * max(1.0, float(np.max(np.abs(p))))
    m = p.max(axis=1, keepdims=True)
    soft = np.exp(p - m) / np.exp(p - m).sum(axis=1, keepdims=True)
    same = int(np.sum(np.all(idx == i_ref, axis=1)))
    print(f"        tokens whose selection equals the oracle's: {same}/{S}", flush=True)
    assert same >= 0.995 * S
    for i in np.nonzero(np.any(idx != i_ref, axis=1))[0]:
        # a different order is legitimate only between scores closer than the fp32 accumulation error
        ps = p[i, idx[i]]
        assert len(set(idx[i].tolist())) == c["topk"]
        assert np.all(ps[:-1] >= ps[1:] - delta)
        assert np.delete(p[i], idx[i]).max() <= ps[-1] + delta
    np.testing.assert_allclose(prob, np.take_along_axis(soft, idx, axis=1), rtol=2e-4, atol=1e-7)
    assert float(np.max(np.abs(np.sort(prob, axis=1) - np.sort(p_ref, axis=1)))) <= 1e-5 * float(np.max(p_ref)) + 1e-7


@pytest.mark.parametrize("key", sorted(I.FP8_QUANT_GEMM_TABLE, key=lambda k: int(k[1:])))
def test_fp8_quant_gemm_full(rf, key):
    c = I.table_workload(key)
    say(f"{key} {c['name']}")
    a, w = I.fp8_quant_gemm_inputs_device(I.SEED_BASE + 7, c["M"], c["K"], c["N"], DEV)
    out = rf.rf_fp8_quant_gemm(a, w)
    torch.cuda.synchronize()
    # sampled token rows (tokens are independent): every 61st row plus the tile edges
    rows = sorted(set(list(range(0, c["M"], 61)) + [127, 128, c["M"] - 1]))
    ah = I.to_numpy(a[rows]).astype(np.float32)
    wh = I.to_numpy(w.to(torch.float32))
    ref = O.fp8_quant_gemm(ah, wh, 128)
    check_rows(I.to_numpy(out[rows]), ref, 2e-2, "fp8_quant_gemm", row_tol=2e-2)
    assert bool(torch.isfinite(out.float()).all())
