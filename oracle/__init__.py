"""Python face of the CPU oracle (``oracle/flash3d_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the benchmark's
cpu-baseline leg. The product package never imports this module and this module never imports
the product package. Arguments are numpy arrays. The C library holds the bucketing, the attention, its gradient and the
pooling; two definitions are written here in numpy binary64 instead: the block glue (ln_linear) and the attention
gradient as a function of the forward call's saved results (attn_bwd_saved).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, List, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "flash3d_oracle.c")
_LIB = os.path.join(_HERE, "libf3d_oracle.so")

HASHES = {"xor_mod": 0, "xor_div": 1, "zorder_mod": 2, "zorder_div": 3}
MODES = {"plain": 0, "shift": 1, "stride": 2}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction, OpenMP for the attention loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared",
               _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_morton3.restype = ctypes.c_uint64
        _lib.orc_morton3.argtypes = [ctypes.c_uint32] * 3
        _lib.orc_hash.restype = ctypes.c_int64
        _lib.orc_bucketize.restype = ctypes.c_int64
        _lib.orc_bucketize_ex.restype = ctypes.c_int64
        _lib.orc_mix32.restype = ctypes.c_uint32
        _lib.orc_mix32.argtypes = [ctypes.c_uint32]
        _lib.orc_probe_direction.restype = ctypes.c_int32
        _lib.orc_group_of_bucket.restype = ctypes.c_int64
        _lib.orc_group_of_bucket.argtypes = [ctypes.c_int64] + [ctypes.c_int32] * 4
        _lib.orc_attn.restype = ctypes.c_int64
        _lib.orc_attn_fmt.restype = ctypes.c_int64
        _lib.orc_half_to_double.restype = ctypes.c_double
        _lib.orc_half_to_double.argtypes = [ctypes.c_uint16]
        _lib.orc_unpermute.restype = ctypes.c_int
        _lib.orc_max_threads.restype = ctypes.c_int
        _lib.orc_pool_assign.restype = ctypes.c_int64
        _lib.orc_attn_bwd.restype = ctypes.c_int64
        _lib.orc_pool_reduce.restype = ctypes.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def morton3(x: int, y: int, z: int) -> int:
    return int(lib().orc_morton3(x, y, z))


def hash_bucket(hash_name: str, K: int, vmax, v, div: int = 0):
    """Bucket of voxel v for a scan with K buckets and per-axis voxel maximum vmax.
    Returns (bucket, divisor, probe_step)."""
    vm = np.asarray(vmax, dtype=np.int32)
    vv = np.asarray(v, dtype=np.int32)
    d = ctypes.c_int64(0)
    s = ctypes.c_int32(0)
    h = lib().orc_hash(ctypes.c_int32(HASHES[hash_name]), ctypes.c_int64(K), _p(vm), ctypes.c_int32(div), _p(vv),
                       ctypes.byref(d), ctypes.byref(s))
    return int(h), int(d.value), int(s.value)


def group_of_bucket(j: int, m: int, mode: str, shift: int = 2, stride: int = 2) -> int:
    return int(lib().orc_group_of_bucket(j, m, MODES[mode], shift, stride))


ORDERS = {"index": 0, "canonical": 1}
PROBE_MODES = {"axes": 0, "table": 1, "seeded": 2}


def bucketize(coords: np.ndarray, batch_offsets: np.ndarray, voxel_size: float, bucket_size: int,
              hash_name: str = "zorder_div", n_probes: int = 6, div: int = 0, probe_step: int = 0,
              order: str = "index", probe_mode: str = "axes", probe_seed: int = 0,
              probe_table: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """Algorithms 1+2 under the round-synchronous schedule; contenders served by input index (order="index") or
    by (Z-order code of the voxel, coordinates, index) (order="canonical"); probe offsets from the axis table, a
    caller's table [n_probes, 3] of voxel offsets, or a seeded per-voxel draw. Returns a dict with
    bucket_id, bucket_off, round_of, perm, inv_perm, offsets[K+1], scan_bucket_start[n_scans+1]."""
    coords = np.ascontiguousarray(coords, dtype=np.float32).reshape(-1, 3)
    bo = np.ascontiguousarray(batch_offsets, dtype=np.int32)
    n, n_scans = coords.shape[0], bo.shape[0] - 1
    kmax = n // max(bucket_size, 1) + n_scans + 1
    out = {k: np.full(n, -1, dtype=np.int32) for k in ("bucket_id", "bucket_off", "round_of", "perm", "inv_perm")}
    offsets = np.zeros(kmax + 1, dtype=np.int32)
    sbs = np.zeros(n_scans + 1, dtype=np.int32)
    tab = None
    if probe_table is not None:
        tab = np.zeros((6, 3), dtype=np.int32)
        pt = np.asarray(probe_table, dtype=np.int32).reshape(-1, 3)
        tab[: pt.shape[0]] = pt
    K = lib().orc_bucketize_ex(_p(coords), _p(bo), ctypes.c_int64(n), ctypes.c_int32(n_scans),
                               ctypes.c_float(voxel_size), ctypes.c_int32(bucket_size), ctypes.c_int32(HASHES[hash_name]),
                               ctypes.c_int32(n_probes), ctypes.c_int32(div), ctypes.c_int32(probe_step),
                               ctypes.c_int32(ORDERS[order]), ctypes.c_int32(PROBE_MODES[probe_mode]),
                               ctypes.c_uint32(probe_seed & 0xFFFFFFFF), _p(tab),
                               _p(out["bucket_id"]), _p(out["bucket_off"]), _p(out["round_of"]), _p(out["perm"]),
                               _p(out["inv_perm"]), _p(offsets), _p(sbs))
    if K < 0:
        raise ValueError("orc_bucketize_ex: bad arguments")
    out["offsets"] = offsets[: K + 1].copy()
    out["scan_bucket_start"] = sbs
    return out


def mix32(x: int) -> int:
    """The oracle's 32-bit mixer."""
    return int(lib().orc_mix32(ctypes.c_uint32(x & 0xFFFFFFFF)))


def probe_direction(seed: int, r: int, voxel) -> int:
    """Direction 0..5 (+x, -x, +y, -y, +z, -z) of probe r for a point of this voxel under `seed`."""
    v = np.ascontiguousarray(voxel, dtype=np.int32)
    return int(lib().orc_probe_direction(ctypes.c_uint32(seed & 0xFFFFFFFF), ctypes.c_int32(r), _p(v)))


def attn(q: np.ndarray, k: np.ndarray, v: np.ndarray, perm: Optional[np.ndarray], offsets: np.ndarray,
         scan_bucket_start: np.ndarray, scope_buckets: int, mode: str, heads: int, head_dim: int,
         shift: int = 2, stride: int = 2, scale: Optional[float] = None, row_sel: Optional[np.ndarray] = None,
         fmt: str = "bf16") -> np.ndarray:
    """Scope-restricted multi-head self-attention in binary64. q,k,v: uint16 bit patterns [n, heads*head_dim] of
    bfloat16 (fmt="bf16") or binary16 (fmt="f16") numbers. Returns float64 [n, heads*head_dim] in bucket-major row
    order (rows not selected by row_sel are NaN)."""
    q, k, v = (np.ascontiguousarray(a, dtype=np.uint16) for a in (q, k, v))
    n = q.shape[0]
    off = np.ascontiguousarray(offsets, dtype=np.int32)
    sbs = np.ascontiguousarray(scan_bucket_start, dtype=np.int32)
    pm = None if perm is None else np.ascontiguousarray(perm, dtype=np.int32)
    sel = None if row_sel is None else np.ascontiguousarray(row_sel, dtype=np.uint8)
    out = np.full((n, heads * head_dim), np.nan, dtype=np.float64)
    sc = (1.0 / np.sqrt(float(head_dim))) if scale is None else float(scale)
    r = lib().orc_attn_fmt(_p(q), _p(k), _p(v), ctypes.c_int32({"bf16": 0, "f16": 1}[fmt]), _p(pm), _p(off), _p(sbs), ctypes.c_int32(sbs.shape[0] - 1),
                       ctypes.c_int32(scope_buckets), ctypes.c_int32(MODES[mode]), ctypes.c_int32(shift),
                       ctypes.c_int32(stride), ctypes.c_int32(heads), ctypes.c_int32(head_dim), ctypes.c_double(sc),
                       _p(sel), _p(out))
    if r < 0:
        raise ValueError("orc_attn: bad arguments")
    return out


def half_to_double(bits: int) -> float:
    """The oracle's decoder of a binary16 bit pattern."""
    return float(lib().orc_half_to_double(ctypes.c_uint16(bits)))


def attn_bwd(q: np.ndarray, k: np.ndarray, v: np.ndarray, dout: np.ndarray, perm: Optional[np.ndarray], offsets: np.ndarray,
             scan_bucket_start: np.ndarray, scope_buckets: int, mode: str, heads: int, head_dim: int, shift: int = 2,
             stride: int = 2, scale: Optional[float] = None, scope_sel: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """Gradient of the scope-restricted attention in binary64. q,k,v,dout: uint16 bf16 bit patterns
    [n, heads*head_dim]; dout belongs to the bucket-major output rows. Returns dq, dk, dv [n, C] (bucket-major
    rows), lse [n, heads] (natural log) and done [n] (1 where the row's scope was computed)."""
    q, k, v, dout = (np.ascontiguousarray(a, dtype=np.uint16) for a in (q, k, v, dout))
    n, C = q.shape
    off = np.ascontiguousarray(offsets, dtype=np.int32)
    sbs = np.ascontiguousarray(scan_bucket_start, dtype=np.int32)
    pm = None if perm is None else np.ascontiguousarray(perm, dtype=np.int32)
    sel = None if scope_sel is None else np.ascontiguousarray(scope_sel, dtype=np.uint8)
    out = {name: np.full((n, C), np.nan, dtype=np.float64) for name in ("dq", "dk", "dv")}
    out["lse"] = np.full((n, heads), np.nan, dtype=np.float64)
    out["done"] = np.zeros(n, dtype=np.uint8)
    sc = (1.0 / np.sqrt(float(head_dim))) if scale is None else float(scale)
    r = lib().orc_attn_bwd(_p(q), _p(k), _p(v), _p(dout), _p(pm), _p(off), _p(sbs), ctypes.c_int32(sbs.shape[0] - 1),
                           ctypes.c_int32(scope_buckets), ctypes.c_int32(MODES[mode]), ctypes.c_int32(shift),
                           ctypes.c_int32(stride), ctypes.c_int32(heads), ctypes.c_int32(head_dim), ctypes.c_double(sc),
                           _p(sel), _p(out["dq"]), _p(out["dk"]), _p(out["dv"]), _p(out["lse"]), _p(out["done"]))
    if r < 0:
        raise ValueError("orc_attn_bwd: bad arguments")
    return out


def scope_rows(offsets: np.ndarray, scan_bucket_start: np.ndarray, scope_buckets: int, mode: str, shift: int = 2,
               stride: int = 2) -> List[np.ndarray]:
    """Bucket-major rows of every attention scope (Section 4.2), scope after scope, scan after scan: the buckets of a
    scope in increasing order, each bucket's rows in order. The bucket -> scope map is group_of_bucket."""
    off = np.asarray(offsets, dtype=np.int64)
    sbs = np.asarray(scan_bucket_start, dtype=np.int64)
    scopes: List[np.ndarray] = []
    for b in range(sbs.shape[0] - 1):
        members: Dict[int, List[np.ndarray]] = {}
        for j in range(int(sbs[b + 1] - sbs[b])):
            g = group_of_bucket(j, scope_buckets, mode, shift, stride)
            members.setdefault(g, []).append(np.arange(off[sbs[b] + j], off[sbs[b] + j + 1]))
        for g in sorted(members):
            rows = np.concatenate(members[g])
            if rows.size:
                scopes.append(rows)
    return scopes


def attn_bwd_saved(q: np.ndarray, k: np.ndarray, v: np.ndarray, dout: np.ndarray, out: np.ndarray, lse: np.ndarray,
                   perm: Optional[np.ndarray], offsets: np.ndarray, scan_bucket_start: np.ndarray, scope_buckets: int,
                   mode: str, heads: int, head_dim: int, shift: int = 2, stride: int = 2, scale: Optional[float] = None,
                   scope_sel: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """The gradient of the scope-restricted attention (Section 4.2) as a function of the forward call's SAVED results,
    which is how a backward call is defined: with S = scale q k^T inside a scope,
        P = exp(S - lse),  dP = dout v^T,  D = rowsum(dout o out),  dS = P o (dP - D),
        dq = scale dS k,  dk = scale dS^T q,  dv = P^T dout,
    `out` [n, C] and `lse` [n, heads] (natural log) being whatever the caller saved (binary64 arrays here; bucket-major
    rows). With the exact output and log-sum-exp this is the plain gradient (attn_bwd); with a rounded `out` it is that
    gradient's value for the rounded D. Binary64, numpy products per scope and head, nothing blocked or reordered.
    q, k, v, dout: uint16 bf16 bit patterns, q/k/v read through perm as in attn. Returns dq, dk, dv [n, C] (bucket-major
    rows, NaN where not computed), done [n], and the intermediates a tolerance derivation needs, per computed scope:
    `scopes` = list of (rows, [per head: dict(P=, dS=, dP=, D=)])."""
    qf, kf, vf, gf = (_bf16_bits_to_f64(np.ascontiguousarray(a, dtype=np.uint16)) for a in (q, k, v, dout))
    if perm is not None:
        pm = np.asarray(perm, dtype=np.int64)
        qf, kf, vf = qf[pm], kf[pm], vf[pm]
    of = np.asarray(out, dtype=np.float64)
    lf = np.asarray(lse, dtype=np.float64)
    n, C = qf.shape
    sc = (1.0 / np.sqrt(float(head_dim))) if scale is None else float(scale)
    res = {name: np.full((n, C), np.nan, dtype=np.float64) for name in ("dq", "dk", "dv")}
    res["done"] = np.zeros(n, dtype=np.uint8)
    res["scopes"] = []
    for rows in scope_rows(offsets, scan_bucket_start, scope_buckets, mode, shift, stride):
        if scope_sel is not None and not np.asarray(scope_sel)[rows].any():
            continue
        per_head = []
        for h in range(heads):
            sl = slice(h * head_dim, (h + 1) * head_dim)
            Q, K, V, G, O = qf[rows, sl], kf[rows, sl], vf[rows, sl], gf[rows, sl], of[rows, sl]
            P = np.exp(sc * (Q @ K.T) - lf[rows, h][:, None])
            dP = G @ V.T
            D = (G * O).sum(axis=1)
            dS = P * (dP - D[:, None])
            res["dq"][rows, sl] = sc * (dS @ K)
            res["dk"][rows, sl] = sc * (dS.T @ Q)
            res["dv"][rows, sl] = P.T @ G
            per_head.append(dict(P=P, dS=dS, dP=dP, D=D))
        res["done"][rows] = 1
        res["scopes"].append((rows, per_head))
    return res


def unpermute(src: np.ndarray, perm: np.ndarray) -> np.ndarray:
    """dst[perm[p]] = src[p] for 2-D arrays of any dtype."""
    src = np.ascontiguousarray(src)
    pm = np.ascontiguousarray(perm, dtype=np.int32)
    dst = np.zeros_like(src)
    rb = src.strides[0]
    lib().orc_unpermute(_p(src), _p(pm), ctypes.c_int64(src.shape[0]), ctypes.c_int64(rb), _p(dst))
    return dst


POOL_OPS = {"sum": 0, "mean": 1, "min": 2, "max": 3}


def pool_assign(coords_bm: np.ndarray, row_offsets: np.ndarray, tile: int, rho: int, voxel_size: float,
                hash_name: str = "zorder_div") -> Dict[str, np.ndarray]:
    """Sub-bucket construction of the in-bucket pooling (Appendix "In-bucket Pooling") on BUCKET-MAJOR
    coordinates, tile by tile. Returns sub_of, slot_of, step_of (per input row), pooled_offsets
    [n_scans+1] and n_out."""
    c = np.ascontiguousarray(coords_bm, dtype=np.float32).reshape(-1, 3)
    ro = np.ascontiguousarray(row_offsets, dtype=np.int32)
    n = c.shape[0]
    out = {k: np.full(n, -1, dtype=np.int32) for k in ("sub_of", "slot_of", "step_of")}
    po = np.zeros(ro.shape[0], dtype=np.int32)
    r = lib().orc_pool_assign(_p(c), _p(ro), ctypes.c_int32(ro.shape[0] - 1), ctypes.c_int32(tile), ctypes.c_int32(rho),
                              ctypes.c_float(voxel_size), ctypes.c_int32(HASHES[hash_name]), _p(out["sub_of"]),
                              _p(out["slot_of"]), _p(out["step_of"]), _p(po))
    if r < 0:
        raise ValueError("orc_pool_assign: bad arguments")
    out["pooled_offsets"] = po
    out["n_out"] = int(r)
    return out


def pool_reduce(feat_bm: np.ndarray, sub_of: np.ndarray, n_out: int, op: str = "mean",
                coords_bm: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """Reduce the rows of every sub-bucket in binary64, rounded once to bf16. feat_bm: uint16 bf16 bit
    patterns [n, C], bucket-major. Returns feat [n_out, C] (uint16), counts [n_out] and, when coords_bm is
    given, coords [n_out, 3] (mean position, float32)."""
    f = np.ascontiguousarray(feat_bm, dtype=np.uint16)
    so = np.ascontiguousarray(sub_of, dtype=np.int32)
    n, C = f.shape
    out = np.zeros((n_out, C), dtype=np.uint16)
    counts = np.zeros(n_out, dtype=np.int32)
    c = None if coords_bm is None else np.ascontiguousarray(coords_bm, dtype=np.float32).reshape(-1, 3)
    pc = None if c is None else np.zeros((n_out, 3), dtype=np.float32)
    r = lib().orc_pool_reduce(_p(f), ctypes.c_int64(n), ctypes.c_int32(C), _p(so), ctypes.c_int64(n_out),
                              ctypes.c_int32(POOL_OPS[op]), _p(out), _p(counts), _p(c), _p(pc))
    if r < 0:
        raise ValueError("orc_pool_reduce: bad arguments")
    res = {"feat": out, "counts": counts}
    if pc is not None:
        res["coords"] = pc
    return res


def _bf16_bits_to_f64(a: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(a, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def ln_linear(x: np.ndarray, w: np.ndarray, bias: Optional[np.ndarray] = None, gamma: Optional[np.ndarray] = None,
              beta: Optional[np.ndarray] = None, eps: float = 1e-5, row_in: Optional[np.ndarray] = None,
              residual: Optional[np.ndarray] = None, row_out: Optional[np.ndarray] = None) -> np.ndarray:
    """The point-wise part of a transformer block around the attention (Section 4.2, block equations: LayerNorm and
    the linear maps of MHSA / MLP applied to every point), in binary64:
        y[p] = LN(x[row_in[p]]) @ w.T + bias,   LN(v) = (v - mean(v)) / sqrt(var(v) + eps) * gamma + beta  (biased variance)
        out[row_out[p]] = y[p] + residual[row_out[p]]
    x: uint16 bf16 bits [n, c_in]; w: uint16 bf16 bits [c_out, c_in]; gamma/beta/bias: float arrays; gamma=None skips
    the LayerNorm; residual: uint16 bf16 bits [n, c_out] or None. Returns float64 [n, c_out]."""
    xf = _bf16_bits_to_f64(x)
    if row_in is not None:
        xf = xf[np.asarray(row_in, dtype=np.int64)]
    if gamma is not None:
        mu = xf.mean(axis=1, keepdims=True)
        var = ((xf - mu) ** 2).mean(axis=1, keepdims=True)
        xf = (xf - mu) / np.sqrt(var + eps) * np.asarray(gamma, dtype=np.float64)
        if beta is not None:
            xf = xf + np.asarray(beta, dtype=np.float64)
    y = xf @ _bf16_bits_to_f64(w).T
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64)
    out = y
    if row_out is not None:
        out = np.empty_like(y)
        out[np.asarray(row_out, dtype=np.int64)] = y
    if residual is not None:
        out = out + _bf16_bits_to_f64(residual)
    return out


def max_threads() -> int:
    return int(lib().orc_max_threads())
