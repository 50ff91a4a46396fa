"""Pins for the point-wise block glue of the oracle (LayerNorm + linear map with row gather/scatter and residual):
a scalar loop re-computation on tiny sizes, closed forms, and the row-map semantics."""
import math

import numpy as np

import oracle
from paper_2412_16481_amd import workloads as wl


def bits(a):
    return wl.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def test_scalar_loops_on_a_tiny_case():
    rng = np.random.default_rng(70)
    n, ci, co = 5, 6, 4
    x, w = bits(rng.standard_normal((n, ci))), bits(rng.standard_normal((co, ci)))
    gamma, beta, bias = rng.standard_normal(ci), rng.standard_normal(ci), rng.standard_normal(co)
    res = bits(rng.standard_normal((n, co)))
    row_in, row_out = rng.permutation(n), rng.permutation(n)
    got = oracle.ln_linear(x, w, bias, gamma, beta, 1e-3, row_in, res, row_out)
    xf, wf, rf = (wl.bf16_bits_to_f32(a).astype(float) for a in (x, w, res))
    for p in range(n):
        v = [xf[row_in[p]][c] for c in range(ci)]
        mu = sum(v) / ci
        var = sum((t - mu) ** 2 for t in v) / ci
        ln = [(v[c] - mu) / math.sqrt(var + 1e-3) * gamma[c] + beta[c] for c in range(ci)]
        for o in range(co):
            want = sum(ln[c] * wf[o][c] for c in range(ci)) + bias[o] + rf[row_out[p]][o]
            assert abs(got[row_out[p]][o] - want) < 1e-12


def test_closed_forms():
    rng = np.random.default_rng(71)
    n, c = 7, 16
    x = bits(rng.standard_normal((n, c)) * 3 + 1)
    eye = bits(np.eye(c))
    # no LayerNorm, identity weight: the input comes back; with a bias it is shifted
    assert np.array_equal(oracle.ln_linear(x, eye), wl.bf16_bits_to_f32(x).astype(np.float64))
    np.testing.assert_allclose(oracle.ln_linear(x, eye, bias=np.arange(c)), wl.bf16_bits_to_f32(x) + np.arange(c), atol=1e-12)
    # LayerNorm output has zero mean and unit variance per row (gamma = 1, beta = 0, eps -> 0)
    y = oracle.ln_linear(x, eye, gamma=np.ones(c), beta=np.zeros(c), eps=0.0)
    np.testing.assert_allclose(y.mean(axis=1), 0, atol=1e-12)
    np.testing.assert_allclose(y.var(axis=1), 1, atol=1e-12)
    # a constant row normalises to beta; a zero weight leaves the bias
    const = bits(np.full((2, c), 2.5))
    np.testing.assert_allclose(oracle.ln_linear(const, eye, gamma=np.ones(c), beta=np.arange(c), eps=1e-5), np.tile(np.arange(c), (2, 1)), atol=1e-9)
    np.testing.assert_allclose(oracle.ln_linear(x, bits(np.zeros((3, c))), bias=[1, 2, 3]), np.tile([1.0, 2.0, 3.0], (n, 1)))
    # LayerNorm is invariant to shifting and (for eps = 0) scaling a row
    x2 = bits(wl.bf16_bits_to_f32(x) * 2.0)
    np.testing.assert_allclose(oracle.ln_linear(x2, eye, gamma=np.ones(c), eps=0.0), oracle.ln_linear(x, eye, gamma=np.ones(c), eps=0.0), atol=1e-12)


def test_row_maps_compose_with_unpermute():
    rng = np.random.default_rng(72)
    n, c = 50, 8
    x, w = bits(rng.standard_normal((n, c))), bits(rng.standard_normal((c, c)))
    perm = rng.permutation(n).astype(np.int32)
    plain = oracle.ln_linear(x, w, gamma=np.ones(c), beta=np.zeros(c))
    gathered = oracle.ln_linear(x, w, gamma=np.ones(c), beta=np.zeros(c), row_in=perm)      # bucket-major rows
    assert np.array_equal(gathered, plain[perm])
    back = oracle.ln_linear(x, w, gamma=np.ones(c), beta=np.zeros(c), row_in=perm, row_out=perm)
    assert np.array_equal(back, plain) and np.array_equal(oracle.unpermute(gathered, perm), plain)
