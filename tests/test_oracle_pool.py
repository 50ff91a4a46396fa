"""Pins for the in-bucket pooling half of the CPU oracle (Section 4.2 "In-bucket Pooling"; Appendix
"In-bucket Pooling"): a hand trace, a literal thread-by-thread simulation with an AtomicInc primitive,
invariants the construction must satisfy on any input, a brute-force check of the nearest-sub-bucket
choice, and the reductions against numpy with an independent bf16 rounding."""
import struct

import numpy as np
import pytest

import oracle
from paper_2412_16481_amd import workloads as wl

HASHES = ["xor_mod", "xor_div", "zorder_mod", "zorder_div"]


def test_hand_trace_of_the_three_steps():
    # seven points on a line, voxel 1: voxels 0,4,8,1,5,2,12; rho = 2 -> M = 4; XOR-mod hash = voxel mod 4
    vx = np.array([0, 4, 8, 1, 5, 2, 12], dtype=np.float32)
    c = np.stack([vx + 0.5, np.full(7, 3.0, np.float32), np.full(7, -1.0, np.float32)], axis=1)
    r = oracle.pool_assign(c, np.array([0, 7]), 1024, 2, 1.0, "xor_mod")
    # initial: rows 0,1 -> sub 0 (hash 0), rows 3,4 -> sub 1 (hash 1), row 5 -> sub 2 (hash 2); rows 2 and 6 overflow hash 0
    # new sub-bucket: row 2 opens sub 3 and the counter reaches M; round 1: row 6 (x=12.5) is nearer to row 2 (8.5) than to row 5 (2.5)
    assert r["n_out"] == 4
    assert r["sub_of"].tolist() == [0, 0, 3, 1, 1, 2, 3]
    assert r["slot_of"].tolist() == [0, 1, 0, 0, 1, 0, 1]
    assert r["step_of"].tolist() == [1, 1, 2, 1, 1, 1, 3]
    assert r["pooled_offsets"].tolist() == [0, 4]


def test_hand_trace_rejected_point_retries_next_round():
    # rho = 2, n = 6 -> M = 3. one voxel for all (voxel size 100), XOR-mod 3: every hash is 0
    # initial: rows 0,1 -> sub 0. new: row 2 -> sub 1 (x 0.3), row 3 -> sub 2 (x 0.4), counter = M. left: rows 4 (x 0.6) and 5 (x 9.5)
    # round 1: row 4 is nearer to 0.4 than to 0.3 -> sub 2; row 5 also (9.1 < 9.2) -> sub 2, which has room for one:
    # row 4 joins, row 5 is turned away; round 2: only sub 1 is open, row 5 joins it
    x = np.array([0.1, 0.2, 0.3, 0.4, 0.6, 9.5], dtype=np.float32)
    c = np.stack([x, np.zeros(6, np.float32), np.zeros(6, np.float32)], axis=1)
    r = oracle.pool_assign(c, np.array([0, 6]), 1024, 2, 100.0, "xor_mod")
    assert r["sub_of"].tolist() == [0, 0, 1, 2, 2, 1]
    assert r["slot_of"].tolist() == [0, 1, 0, 0, 1, 1]
    assert r["step_of"].tolist() == [1, 1, 2, 2, 3, 4]
    # the same with the two left-over points next to sub 1
    x = np.array([0.1, 0.2, 0.3, 5.0, 0.31, 0.32], dtype=np.float32)
    c = np.stack([x, np.zeros(6, np.float32), np.zeros(6, np.float32)], axis=1)
    r = oracle.pool_assign(c, np.array([0, 6]), 1024, 2, 100.0, "xor_mod")
    # initial rows 0,1 -> sub 0; new: row 2 -> sub 1 (x 0.3), row 3 -> sub 2 (x 5.0); rows 4, 5 both pick sub 1; row 4 joins, row 5 retries and takes sub 2
    assert r["sub_of"].tolist() == [0, 0, 1, 2, 1, 2]
    assert r["step_of"].tolist() == [1, 1, 2, 2, 3, 4]


def simulate_tile(c, rho, voxel, hash_name):
    """Literal reading of the Appendix for one tile: threads in row order, a block counter, AtomicInc on the
    sub-bucket fill that returns the old value, a barrier between rounds."""
    n = len(c)
    M = -(-n // rho)
    mn = c.min(axis=0)
    inv = np.float32(1.0) / np.float32(voxel)
    v = np.floor((c - mn).astype(np.float32) * inv).astype(np.int64)
    vmax = v.max(axis=0)
    h = [oracle.hash_bucket(hash_name, M, vmax, v[i])[0] for i in range(n)]
    fill, first, table = {}, {}, {}
    counter = [0]

    def atomic_inc(s):
        old = fill.get(s, 0)
        fill[s] = old + 1
        return old

    sub, step = [-1] * n, [0] * n
    waiting = []
    for i in range(n):                              # initial sub-buckets
        if h[i] not in table:
            table[h[i]] = counter[0]
            first[counter[0]] = i
            counter[0] += 1
        s = table[h[i]]
        if atomic_inc(s) < rho:
            sub[i], step[i] = s, 1
        else:
            fill[s] -= 1                            # roll back, the point moves on
            waiting.append(i)
    still = []
    for i in waiting:                               # new sub-bucket allocation
        if counter[0] < M:
            s = counter[0]
            counter[0] += 1
            first[s] = i
            atomic_inc(s)
            sub[i], step[i] = s, 2
        else:
            still.append(i)
    rnd = 0
    while still:                                    # find new sub-bucket
        rnd += 1
        open_subs = [s for s in range(M) if fill.get(s, 0) < rho]       # identified at the barrier
        choice = {}
        for i in still:
            d = [(np.float32(np.float32(np.float32(c[i, 0] - c[first[s], 0]) ** 2 + np.float32(c[i, 1] - c[first[s], 1]) ** 2)
                             + np.float32(c[i, 2] - c[first[s], 2]) ** 2), s) for s in open_subs]
            choice[i] = min(d)[1]
        nxt = []
        for i in still:
            s = choice[i]
            if atomic_inc(s) < rho:
                sub[i], step[i] = s, 2 + rnd
            else:
                fill[s] -= 1
                nxt.append(i)
        still = nxt
    return sub, step, M


@pytest.mark.parametrize("hash_name", HASHES)
@pytest.mark.parametrize("rho", [2, 3, 4])
def test_literal_simulation_of_the_appendix(hash_name, rho):
    rng = np.random.default_rng(100 + rho)
    for n, voxel in ((1, 0.1), (5, 0.1), (37, 0.3), (150, 0.08), (333, 0.5)):
        c = (rng.random((n, 3)) * np.array([2.0, 1.0, 0.5])).astype(np.float32)
        c[: n // 3] *= 0.2                       # a dense corner: many points overflow their hash value
        got = oracle.pool_assign(c, np.array([0, n]), 1024, rho, voxel, hash_name)
        sub, step, M = simulate_tile(c, rho, voxel, hash_name)
        assert got["n_out"] == M
        assert got["sub_of"].tolist() == sub
        assert got["step_of"].tolist() == step


@pytest.mark.parametrize("hash_name", HASHES)
@pytest.mark.parametrize("rho,tile", [(1, 64), (2, 1024), (4, 1024), (8, 512), (3, 100)])
def test_invariants_on_ragged_multi_scan_input(hash_name, rho, tile):
    rng = np.random.default_rng(7)
    sizes = [2500, 0, 1, tile, tile + 1, 3 * tile - 5]
    ro = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    c = wl.indoor_room(rng, int(ro[-1])) if hasattr(wl, "indoor_room") else rng.random((int(ro[-1]), 3)).astype(np.float32)
    c = np.ascontiguousarray(c[:ro[-1]], dtype=np.float32)
    r = oracle.pool_assign(c, ro, tile, rho, 0.1, hash_name)
    sub, slot, step = r["sub_of"], r["slot_of"], r["step_of"]
    # pooled rows: tiles in order, ceil(n_tile / rho) each; offsets per scan
    expect, po = 0, [0]
    for b in range(len(sizes)):
        for t0 in range(int(ro[b]), int(ro[b + 1]), tile):
            nt = min(t0 + tile, int(ro[b + 1])) - t0
            M = -(-nt // rho)
            s = sub[t0:t0 + nt]
            assert s.min() >= expect and s.max() < expect + M          # a point pools inside its own tile
            cnt = np.bincount(s - expect, minlength=M)
            assert (cnt >= 1).all() and (cnt <= rho).all()             # every sub-bucket exists, none above capacity
            for j in range(M):                                         # slots are 0 .. count-1
                assert sorted(slot[t0:t0 + nt][s == expect + j].tolist()) == list(range(cnt[j]))
            expect += M
        po.append(expect)
    assert r["n_out"] == expect and r["pooled_offsets"].tolist() == po
    assert ((step >= 1)).all()
    # an initial sub-bucket holds points of ONE hash value, in row order, the first rho of them
    first_rows = np.where(slot == 0)[0]
    assert len(first_rows) == expect


def test_round_choices_are_the_nearest_open_sub_bucket():
    # replay the rounds from step_of and check every joining point against a brute-force nearest search
    rng = np.random.default_rng(11)
    n, rho = 700, 2
    c = rng.normal(size=(n, 3)).astype(np.float32)
    r = oracle.pool_assign(c, np.array([0, n]), 1024, rho, 0.4, "zorder_div")
    sub, slot, step = r["sub_of"], r["slot_of"], r["step_of"]
    M = r["n_out"]
    first = np.array([np.where((sub == s) & (slot == 0))[0][0] for s in range(M)])
    fill = np.array([np.sum((sub == s) & (step <= 2)) for s in range(M)])
    for rnd in range(1, int(step.max()) - 1):
        open_subs = np.where(fill < rho)[0]
        joined = np.where(step == 2 + rnd)[0]
        waiting = np.where(step > 2 + rnd)[0]
        for i in joined:
            d = ((c[i] - c[first[open_subs]]).astype(np.float32) ** 2)
            d2 = (d[:, 0] + d[:, 1]).astype(np.float32) + d[:, 2]
            assert open_subs[np.argmin(d2)] == sub[i]
        for i in waiting:                                        # a rejected point had picked a sub-bucket that filled up
            d = ((c[i] - c[first[open_subs]]).astype(np.float32) ** 2)
            d2 = (d[:, 0] + d[:, 1]).astype(np.float32) + d[:, 2]
            s = open_subs[np.argmin(d2)]
            assert fill[s] + np.sum((sub[joined] == s)) == rho
        fill += np.bincount(sub[joined], minlength=M)
    assert (fill == np.bincount(sub, minlength=M)).all()


def rne_bf16(x: float) -> int:
    """binary64 -> bf16 bits, one rounding to nearest even, by integer arithmetic on the exact value."""
    if x == 0.0:
        return 0x8000 if struct.pack(">d", x)[0] & 0x80 else 0
    sign = 0x8000 if x < 0 else 0
    m, e = np.frexp(abs(x))                     # abs(x) = m * 2**e, 0.5 <= m < 1
    scaled = int(m * (1 << 60))                 # exact: binary64 has 53 bits
    shift = 60 - 8                              # keep 8 significant bits
    q, rem = scaled >> shift, scaled & ((1 << shift) - 1)
    half = 1 << (shift - 1)
    if rem > half or (rem == half and (q & 1)):
        q += 1
    if q == 256:
        q, e = 128, e + 1
    exp = e - 1 + 127
    assert 0 < exp < 255
    return sign | (exp << 7) | (q & 0x7F)


@pytest.mark.parametrize("op", ["sum", "mean", "min", "max"])
def test_reduce_matches_numpy_with_an_independent_rounding(op):
    rng = np.random.default_rng(21)
    n, C, rho = 900, 24, 4
    c = rng.random((n, 3)).astype(np.float32)
    a = oracle.pool_assign(c, np.array([0, 500, n]), 256, rho, 0.1)
    f = wl.f32_to_bf16_bits(rng.standard_normal((n, C)).astype(np.float32) * 3)
    got = oracle.pool_reduce(f, a["sub_of"], a["n_out"], op, c)
    x = wl.bf16_bits_to_f32(f).astype(np.float64)
    fn = {"sum": np.sum, "mean": np.mean, "min": np.min, "max": np.max}[op]
    for s in range(0, a["n_out"], 7):
        rows = np.where(a["sub_of"] == s)[0]
        want = fn(x[rows], axis=0)
        assert got["feat"][s].tolist() == [rne_bf16(float(w)) for w in want]
        assert got["counts"][s] == len(rows)
        assert np.allclose(got["coords"][s], c[rows].astype(np.float64).mean(axis=0), rtol=0, atol=1e-6)


def test_special_cases():
    rng = np.random.default_rng(22)
    n, C = 300, 8
    c = rng.random((n, 3)).astype(np.float32)
    f = wl.f32_to_bf16_bits(rng.standard_normal((n, C)).astype(np.float32))
    # rho = 1: every point is its own pooled row; pooling permutes the rows inside a tile
    a = oracle.pool_assign(c, np.array([0, n]), 128, 1, 0.05)
    assert a["n_out"] == n and sorted(a["sub_of"].tolist()) == list(range(n))
    g = oracle.pool_reduce(f, a["sub_of"], n, "mean", c)
    assert np.array_equal(g["feat"][a["sub_of"]], f) and np.array_equal(g["coords"][a["sub_of"]], c)
    # a tile of at most rho points is one sub-bucket
    a = oracle.pool_assign(c[:5], np.array([0, 5]), 128, 8, 0.05)
    assert a["n_out"] == 1 and (a["sub_of"] == 0).all() and (a["step_of"] == 1).all()
    # constant features: every reduction but the sum returns the constant
    const = np.tile(f[:1], (n, 1))
    a = oracle.pool_assign(c, np.array([0, n]), 128, 4, 0.2)
    for op in ("mean", "min", "max"):
        assert np.array_equal(oracle.pool_reduce(const, a["sub_of"], a["n_out"], op)["feat"], np.tile(f[:1], (a["n_out"], 1)))
    # empty input
    a = oracle.pool_assign(np.zeros((0, 3), np.float32), np.array([0, 0]), 128, 2, 0.1)
    assert a["n_out"] == 0
    # bad arguments
    for kw in (dict(tile=0), dict(rho=0), dict(voxel_size=0.0)):
        args = dict(tile=128, rho=2, voxel_size=0.1)
        args.update(kw)
        with pytest.raises(ValueError):
            oracle.pool_assign(c, np.array([0, n]), args["tile"], args["rho"], args["voxel_size"])
