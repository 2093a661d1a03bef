"""What the GPU tests assert about rf_fp8_quant_gemm, independent of how the kernel segments
the contraction axis.

The entry point promises the two-pass definition (Section 3.4: m = max|a|, c = sum q(MAX a/m) w)
up to quantisation noise: it quantises every element with the maximum of a PREFIX of its row
that contains the element (the incremental form), so each dequantised element
a_hat = (m'/MAX) q(MAX a / m') with some m' <= m.  For E4M3 (3 mantissa bits, subnormal step
2^-9, no overflow because |MAX a / m'| <= MAX):
    |a_hat - a| <= 2^-4 |a| + 2^-10 m / MAX            (half a unit in the last place)
and the same holds for the two-pass value, hence for every output element
    |c_gpu - c_twopass| <= 2 sum_k (2^-4 |a_k| + 2^-10 m / MAX) |w_nk|  =: bound,
whatever the prefixes were.  Beyond that worst case the tests ask for what quantisation noise
really looks like: the difference to the definition is of the size of the definition's own
error against the exact product a @ w^T (two roundings of the same values: about sqrt(2)
times it), the result approximates a @ w^T at least as well as the definition does, and rows
for which every prefix maximum is the final one (the maximum is the first element) reproduce
the definition up to fp32 accumulation and the bf16 rounding of the output.
"""
import numpy as np

from oracle import rf_oracle as O

BF16_HALF_ULP = 2.0 ** -9


def reference(a, w):
    """(two-pass definition, exact product, elementwise worst-case bound) in fp64."""
    a32 = np.asarray(a, dtype=np.float32)
    a64 = a32.astype(np.float64)
    w64 = np.asarray(w, dtype=np.float64)
    two = O.fp8_quant_gemm_twopass(a32, w64)
    exact = a64 @ w64.T
    m = np.max(np.abs(a64), axis=1)
    bound = 2.0 * (2.0 ** -4 * (np.abs(a64) @ np.abs(w64).T)
                   + (2.0 ** -10 / O.E4M3_MAX) * m[:, None] * np.sum(np.abs(w64), axis=1)[None, :])
    return two, exact, bound


def _rms(x):
    return np.sqrt(np.mean(np.square(x), axis=1))


def check(out, a, w, what, first_max_rows=()):
    """out: GPU result [M,N] as float64; a [M,K] float32 of bf16 values; w [N,K] FP8 values."""
    out = np.asarray(out, dtype=np.float64)
    two, exact, bound = reference(a, w)
    assert out.shape == two.shape, (what, out.shape, two.shape)
    assert np.all(np.isfinite(out)), f"{what}: non-finite output"
    # the output is rounded to bf16 once; fp32 accumulation over K adds far less
    rnd = 2.0 * BF16_HALF_ULP * np.abs(two) + 1e-30
    diff = np.abs(out - two)
    worst = float(np.max(diff / (bound * (1.0 + 1e-4) + rnd)))
    noise = _rms(two - exact)                      # the definition's own quantisation error, per token
    floor = 2.0 * BF16_HALF_ULP * _rms(two) + 1e-30
    d_two = _rms(out - two)
    d_exact = _rms(out - exact)
    print(f"        {what}: max |out-twopass| / bound = {worst:.3f}; rms(out-twopass)/rms(twopass-exact) "
          f"max {float(np.max(d_two / (noise + floor))):.2f}; rms(out-exact)/rms(twopass-exact) "
          f"max {float(np.max(d_exact / (noise + floor))):.2f}", flush=True)
    assert worst <= 1.0, f"{what}: an element leaves the quantisation-error bound"
    assert np.all(d_two <= 2.0 * noise + floor), f"{what}: further from the definition than quantisation noise"
    assert np.all(d_exact <= 1.25 * noise + floor), f"{what}: a worse approximation of a @ w^T than the definition"
    zero = np.max(np.abs(np.asarray(a, dtype=np.float64)), axis=1) == 0
    assert np.all(out[zero] == 0.0), f"{what}: an all-zero token must give zeros"
    for r in first_max_rows:                       # every prefix maximum is the final one: the definition itself
        s = float(np.max(np.abs(two[r])))
        assert float(np.max(np.abs(out[r] - two[r]))) <= 4.0 * BF16_HALF_ULP * s + 1e-30, (what, r)
