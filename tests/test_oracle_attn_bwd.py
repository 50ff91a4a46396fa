"""Pins for the attention-gradient half of the CPU oracle: central finite differences of an independent numpy
forward (dense attention under a same-scope mask), closed forms, and identities every softmax-attention
gradient satisfies. The formulas of the oracle are retyped nowhere in this file."""
import numpy as np
import pytest

import oracle
from paper_2412_16481_amd import workloads as wl


def layout(sizes_per_scan):
    sizes = [s for scan in sizes_per_scan for s in scan]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    sbs = np.concatenate([[0], np.cumsum([len(s) for s in sizes_per_scan])]).astype(np.int32)
    return off, sbs


def scope_ids(off, sbs, m, mode, s=2, t=2):
    gid = np.zeros(off[-1], dtype=np.int64)
    base = 0
    for b in range(len(sbs) - 1):
        top = 0
        for j in range(sbs[b + 1] - sbs[b]):
            g = oracle.group_of_bucket(j, m, mode, s, t)
            gid[off[sbs[b] + j]:off[sbs[b] + j + 1]] = base + g
            top = max(top, g + 1)
        base += top
    return gid


def forward_f64(q, k, v, same, heads, d, scale):
    """Dense masked attention on binary64 arrays (independent of the oracle)."""
    out = np.zeros_like(q)
    for h in range(heads):
        sl = slice(h * d, (h + 1) * d)
        s = np.where(same, q[:, sl] @ k[:, sl].T * scale, -np.inf)
        p = np.exp(s - s.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        out[:, sl] = p @ v[:, sl]
    return out


def finite_difference(fn, x, g, eps=1e-5):
    """d/dx of sum(fn(x) * g) by central differences, entry by entry."""
    grad = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + eps
        up = (fn(x) * g).sum()
        x[i] = old - eps
        dn = (fn(x) * g).sum()
        x[i] = old
        grad[i] = (up - dn) / (2 * eps)
    return grad


@pytest.mark.parametrize("mode,kw", [("plain", {}), ("shift", {"shift": 1}), ("stride", {"stride": 2})])
@pytest.mark.parametrize("use_perm", [False, True])
def test_gradients_match_finite_differences_of_an_independent_forward(mode, kw, use_perm):
    rng = np.random.default_rng(50)
    off, sbs = layout([[3, 3, 2, 3, 1], [2, 3]])          # ragged buckets, two scans, m = 2
    n, H, d, m = int(off[-1]), 2, 4, 2
    C = H * d
    qb, kb, vb, gb = (wl.f32_to_bf16_bits(rng.standard_normal((n, C)).astype(np.float32)) for _ in range(4))
    perm = rng.permutation(n).astype(np.int32) if use_perm else None
    got = oracle.attn_bwd(qb, kb, vb, gb, perm, off, sbs, m, mode, H, d, scale=0.37, **kw)
    assert got["done"].all()
    gid = scope_ids(off, sbs, m, mode, kw.get("shift", 2), kw.get("stride", 2))
    same = gid[:, None] == gid[None, :]
    q, k, v, g = (wl.bf16_bits_to_f32(a).astype(np.float64) for a in (qb, kb, vb, gb))
    if use_perm:                                              # the oracle reads row p of q,k,v from perm[p]
        q, k, v = q[perm], k[perm], v[perm]
    dq = finite_difference(lambda x: forward_f64(x, k, v, same, H, d, 0.37), q.copy(), g)
    dk = finite_difference(lambda x: forward_f64(q, x, v, same, H, d, 0.37), k.copy(), g)
    dv = finite_difference(lambda x: forward_f64(q, k, x, same, H, d, 0.37), v.copy(), g)
    np.testing.assert_allclose(got["dq"], dq, rtol=0, atol=2e-8)
    np.testing.assert_allclose(got["dk"], dk, rtol=0, atol=2e-8)
    np.testing.assert_allclose(got["dv"], dv, rtol=0, atol=2e-8)
    # log-sum-exp of the scaled scores, from the same independent forward
    for h in range(H):
        s = np.where(same, q[:, h * d:(h + 1) * d] @ k[:, h * d:(h + 1) * d].T * 0.37, -np.inf)
        want = np.log(np.exp(s - s.max(axis=1, keepdims=True)).sum(axis=1)) + s.max(axis=1)
        np.testing.assert_allclose(got["lse"][:, h], want, rtol=0, atol=1e-12)


def test_closed_forms():
    rng = np.random.default_rng(51)
    H, d = 2, 8
    C = H * d
    # a scope of one row: P = 1, so dV = dO and nothing flows into q and k
    off, sbs = layout([[1, 1, 1]])
    qb, kb, vb, gb = (wl.f32_to_bf16_bits(rng.standard_normal((3, C)).astype(np.float32)) for _ in range(4))
    r = oracle.attn_bwd(qb, kb, vb, gb, None, off, sbs, 1, "plain", H, d)
    assert np.array_equal(r["dv"], wl.bf16_bits_to_f32(gb).astype(np.float64))
    assert not r["dq"].any() and not r["dk"].any()
    # identical keys: uniform attention whatever q is; dV_j = mean of dO over the scope; rows of dS sum to zero, so dQ = 0
    n = 12
    off, sbs = layout([[4, 4, 4]])
    kb = np.tile(kb[:1], (n, 1))
    qb, vb, gb = (wl.f32_to_bf16_bits(rng.standard_normal((n, C)).astype(np.float32)) for _ in range(3))
    r = oracle.attn_bwd(qb, kb, vb, gb, None, off, sbs, 4, "plain", H, d)
    g = wl.bf16_bits_to_f32(gb).astype(np.float64)
    np.testing.assert_allclose(r["dv"], np.tile(g.mean(axis=0), (n, 1)), rtol=0, atol=1e-13)
    np.testing.assert_allclose(r["dq"], 0, atol=1e-13)


def test_identities_of_softmax_attention_gradients():
    rng = np.random.default_rng(52)
    off, sbs = layout([[16] * 6 + [5], [16] * 3])
    n, H, d, m = int(off[-1]), 3, 8, 4
    C = H * d
    qb, kb, vb, gb = (wl.f32_to_bf16_bits(rng.standard_normal((n, C)).astype(np.float32)) for _ in range(4))
    for mode in ("plain", "shift", "stride"):
        r = oracle.attn_bwd(qb, kb, vb, gb, None, off, sbs, m, mode, H, d)
        gid = scope_ids(off, sbs, m, mode)
        q, k, g = (wl.bf16_bits_to_f32(a).astype(np.float64) for a in (qb, kb, gb))
        for sc in np.unique(gid):
            rows = gid == sc
            # the scores do not change when one vector is added to every key of a scope: the dK of a scope sum to zero
            np.testing.assert_allclose(r["dk"][rows].sum(axis=0), 0, atol=1e-11)
            # rows of P sum to one: the dV of a scope sum to the dO of the scope
            np.testing.assert_allclose(r["dv"][rows].sum(axis=0), g[rows].sum(axis=0), atol=1e-11)
            # scaling q by a and k by 1/a leaves the output unchanged: <q, dQ> = <k, dK> inside every scope and head
            for h in range(H):
                sl = slice(h * d, (h + 1) * d)
                np.testing.assert_allclose((q[rows, sl] * r["dq"][rows, sl]).sum(), (k[rows, sl] * r["dk"][rows, sl]).sum(),
                                           atol=1e-10)
        # gradient is linear in dO
        r2 = oracle.attn_bwd(qb, kb, vb, wl.f32_to_bf16_bits((2 * wl.bf16_bits_to_f32(gb)).astype(np.float32)), None, off,
                             sbs, m, mode, H, d)
        for name in ("dq", "dk", "dv"):
            np.testing.assert_allclose(r2[name], 2 * r[name], rtol=1e-12, atol=1e-13)


def test_scope_selection_and_forward_consistency():
    rng = np.random.default_rng(53)
    off, sbs = layout([[8] * 9])
    n, H, d, m = int(off[-1]), 2, 16, 4
    qb, kb, vb, gb = (wl.f32_to_bf16_bits(rng.standard_normal((n, H * d)).astype(np.float32)) for _ in range(4))
    full = oracle.attn_bwd(qb, kb, vb, gb, None, off, sbs, m, "shift", H, d)
    sel = np.zeros(n, dtype=np.uint8)
    sel[40] = 1
    part = oracle.attn_bwd(qb, kb, vb, gb, None, off, sbs, m, "shift", H, d, scope_sel=sel)
    rows = part["done"].astype(bool)
    assert rows.sum() == 32 and rows[40]
    for name in ("dq", "dk", "dv"):
        assert np.array_equal(part[name][rows], full[name][rows]) and np.isnan(part[name][~rows]).all()
    # dV with dO = one-hot picks out a column of P: sum over value rows of dV . v reproduces the forward output
    out = oracle.attn(qb, kb, vb, None, off, sbs, m, "shift", H, d)
    v = wl.bf16_bits_to_f32(vb).astype(np.float64)
    g = wl.bf16_bits_to_f32(gb).astype(np.float64)
    np.testing.assert_allclose((full["dv"] * v).sum(), (out * g).sum(), rtol=1e-12)


# ----------------------------------------------------------------------------- the gradient from saved forward results


def test_scope_rows_reproduces_the_worked_example_of_section_4_2():
    # eight buckets of two rows, four buckets per scope: plain {0-3},{4-7}; shifted by two {0,1},{2-5},{6,7};
    # every second bucket {0,2,4,6},{1,3,5,7}
    off = np.arange(0, 18, 2)
    sbs = np.array([0, 8])
    buckets = lambda scopes: [sorted(set((r // 2).tolist())) for r in scopes]
    assert buckets(oracle.scope_rows(off, sbs, 4, "plain")) == [[0, 1, 2, 3], [4, 5, 6, 7]]
    assert buckets(oracle.scope_rows(off, sbs, 4, "shift", shift=2)) == [[0, 1], [2, 3, 4, 5], [6, 7]]
    assert buckets(oracle.scope_rows(off, sbs, 4, "stride", stride=2)) == [[0, 2, 4, 6], [1, 3, 5, 7]]
    # rows of a scope come bucket after bucket, and the scopes of a pass partition the rows
    allrows = np.concatenate(oracle.scope_rows(off, sbs, 4, "stride", stride=2))
    assert sorted(allrows.tolist()) == list(range(16))


@pytest.mark.parametrize("mode,kw", [("plain", {}), ("shift", {"shift": 1}), ("stride", {"stride": 3})])
@pytest.mark.parametrize("use_perm", [False, True])
def test_gradient_from_exact_saved_results_is_the_plain_gradient(mode, kw, use_perm):
    """D = rowsum(dO o O) and P = exp(S - lse) with the exact O and lse give the gradient of the definition: two different
    formulas (the C oracle sums P o dP and normalises its own softmax) must agree to rounding."""
    off, sbs = layout([[16, 16, 9, 16, 1, 16, 16], [5], [16, 16, 16, 16, 16, 16, 16, 16, 3]])
    n, heads, d, m = int(off[-1]), 3, 16, 4
    rng = np.random.default_rng(70)
    q, k, v, g = (wl.f32_to_bf16_bits(rng.standard_normal((n, heads * d)).astype(np.float32)) for _ in range(4))
    perm = rng.permutation(n).astype(np.int32) if use_perm else None
    want = oracle.attn_bwd(q, k, v, g, perm, off, sbs, m, mode, heads, d, **kw)
    out = oracle.attn(q, k, v, perm, off, sbs, m, mode, heads, d, **kw)
    got = oracle.attn_bwd_saved(q, k, v, g, out, want["lse"], perm, off, sbs, m, mode, heads, d, **kw)
    assert got["done"].all()
    for name in ("dq", "dk", "dv"):
        assert np.abs(got[name] - want[name]).max() <= 1e-11 * max(1.0, np.abs(want[name]).max())
    # a scope selection computes exactly the scopes of the flagged rows
    sel = np.zeros(n, dtype=np.uint8)
    sel[[0, n - 1]] = 1
    part = oracle.attn_bwd_saved(q, k, v, g, out, want["lse"], perm, off, sbs, m, mode, heads, d, scope_sel=sel, **kw)
    part_c = oracle.attn_bwd(q, k, v, g, perm, off, sbs, m, mode, heads, d, scope_sel=sel, **kw)
    assert np.array_equal(part["done"], part_c["done"]) and 0 < part["done"].sum() < n
    rows = part["done"].astype(bool)
    assert np.allclose(part["dq"][rows], want["dq"][rows], rtol=0, atol=1e-11)


def test_a_change_of_the_saved_output_moves_dq_and_dk_through_D_only():
    """dq, dk are affine in the saved output: out + E changes D by rowsum(dO o E) and leaves dv alone,
    dq_i -> dq_i - scale * dD_i * sum_j P_ij k_j."""
    off, sbs = layout([[16, 16, 7]])
    n, heads, d, m = int(off[-1]), 2, 16, 4
    rng = np.random.default_rng(71)
    q, k, v, g = (wl.f32_to_bf16_bits(rng.standard_normal((n, heads * d)).astype(np.float32)) for _ in range(4))
    out = oracle.attn(q, k, v, None, off, sbs, m, "plain", heads, d)
    lse = oracle.attn_bwd(q, k, v, g, None, off, sbs, m, "plain", heads, d)["lse"]
    base = oracle.attn_bwd_saved(q, k, v, g, out, lse, None, off, sbs, m, "plain", heads, d)
    E = rng.standard_normal(out.shape) * 1e-2
    moved = oracle.attn_bwd_saved(q, k, v, g, out + E, lse, None, off, sbs, m, "plain", heads, d)
    assert np.array_equal(moved["dv"], base["dv"])
    kf = wl.bf16_bits_to_f32(k).astype(np.float64)
    gf = wl.bf16_bits_to_f32(g).astype(np.float64)
    scale = 1.0 / np.sqrt(d)
    (rows, per_head), = base["scopes"]
    for h in range(heads):
        sl = slice(h * d, (h + 1) * d)
        dD = (gf[:, sl] * E[:, sl]).sum(axis=1)
        expect = base["dq"][:, sl] - scale * dD[:, None] * (per_head[h]["P"] @ kf[:, sl])
        assert np.abs(moved["dq"][:, sl] - expect).max() <= 1e-12
