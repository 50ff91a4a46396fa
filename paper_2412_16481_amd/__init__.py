"""Thin Python binding of libflash3d.so (the C ABI declared in include/flash3d.h).

Argument marshalling only: every step of the path runs in the HIP kernels. torch is used for
device memory and the current stream. There is no fallback: if the shared library is missing the
import of the native handle fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflash3d.so")

F3D_OK = 0
ERR_INVALID_ARG, ERR_BAD_ALIGNMENT, ERR_WORKSPACE_TOO_SMALL, ERR_UNSUPPORTED, ERR_HIP, ERR_SCRATCH_LIMIT = -1, -2, -3, -4, -5, -6
STATIC_SCRATCH_BYTES = 32 << 20
HASHES = {"xor_mod": 0, "xor_div": 1, "zorder_mod": 2, "zorder_div": 3}
MODES = {"plain": 0, "shift": 1, "stride": 2}
SCHEDULES = {"auto": 0, "general": 1, "steps": 2, "scans": 3}
ORDERS = {"index": 0, "canonical": 1}
PROBE_MODES = {"axes": 0, "table": 1, "seeded": 2}

EXPORTS = ("f3d_params_default", "f3d_max_buckets", "f3d_workspace_bytes", "f3d_psh_bucketize", "f3d_psh_bucketize_static",
           "f3d_bucket_swin_attn", "f3d_bucket_swin_attn_f16", "f3d_attn_block_rows", "f3d_attn_bwd_workspace_bytes", "f3d_bucket_swin_attn_bwd", "f3d_ln_linear", "f3d_pool_max_rows", "f3d_pool_workspace_bytes", "f3d_inbucket_pool",
           "f3d_unpermute", "f3d_error_string", "f3d_last_hip_error", "f3d_version")
POOL_OPS = {"sum": 0, "mean": 1, "min": 2, "max": 3}


class f3d_params(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("voxel_size", ctypes.c_float), ("bucket_cap", ctypes.c_int32),
                ("scope_buckets", ctypes.c_int32), ("hash", ctypes.c_int32), ("n_probes", ctypes.c_int32),
                ("div", ctypes.c_int32), ("probe_step", ctypes.c_int32), ("max_scan_points", ctypes.c_int64),
                ("schedule", ctypes.c_int32), ("order", ctypes.c_int32), ("probe_mode", ctypes.c_int32),
                ("probe_seed", ctypes.c_uint32), ("probe_table", ctypes.c_int32 * 18)]


class Flash3DError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        hip = lib().f3d_last_hip_error() if code == ERR_HIP else 0
        super().__init__(f"{where}: {error_string(code)} (code {code}" + (f", hipError {hip})" if hip else ")"))


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded shared library. Raises if it has not been built (python -m paper_2412_16481_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2412_16481_amd.build` "
                              "(there is no CPU fallback)")
        # torch ships its own HIP runtime with the same soname as the system one. Import it first so
        # that the library binds to the runtime that owns torch's device memory and streams; two HIP
        # runtimes in one process do not see each other's devices.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
        L.f3d_params_default.argtypes = [ctypes.POINTER(f3d_params), f32, i32]
        L.f3d_params_default.restype = None
        L.f3d_max_buckets.argtypes = [i64, i32, ctypes.POINTER(f3d_params)]
        L.f3d_max_buckets.restype = i64
        L.f3d_workspace_bytes.argtypes = [i64, i32, ctypes.POINTER(f3d_params), ctypes.POINTER(ctypes.c_size_t)]
        L.f3d_workspace_bytes.restype = ctypes.c_int
        L.f3d_psh_bucketize.argtypes = [vp, vp, i64, i32, ctypes.POINTER(f3d_params), vp, vp, vp, vp, vp, vp,
                                        ctypes.c_size_t, vp]
        L.f3d_psh_bucketize.restype = ctypes.c_int
        L.f3d_psh_bucketize_static.argtypes = [vp, vp, i64, i32, ctypes.POINTER(f3d_params), vp, vp, vp, vp, vp, vp]
        L.f3d_psh_bucketize_static.restype = ctypes.c_int
        L.f3d_bucket_swin_attn.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i64, i32, i32, i32, i32, i32, i32, i32, f32, vp, vp, vp, vp]
        L.f3d_bucket_swin_attn.restype = ctypes.c_int
        L.f3d_bucket_swin_attn_f16.argtypes = L.f3d_bucket_swin_attn.argtypes
        L.f3d_attn_block_rows.argtypes = [i64, i64, i32, i32, i32, i32, i32, i32]
        L.f3d_attn_block_rows.restype = ctypes.c_int
        L.f3d_bucket_swin_attn_f16.restype = ctypes.c_int
        L.f3d_attn_bwd_workspace_bytes.argtypes = [i64, i32, ctypes.POINTER(ctypes.c_size_t)]
        L.f3d_attn_bwd_workspace_bytes.restype = ctypes.c_int
        L.f3d_bucket_swin_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i32, i64, i32, i32, i32, i32, i32, i32, i32, f32,
                                               vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.f3d_bucket_swin_attn_bwd.restype = ctypes.c_int
        L.f3d_ln_linear.argtypes = [vp, vp, vp, vp, f32, vp, vp, vp, i64, i32, i32, ctypes.POINTER(vp), i32, vp, vp]
        L.f3d_ln_linear.restype = ctypes.c_int
        L.f3d_pool_max_rows.argtypes = [i64, i32, i32, i32]
        L.f3d_pool_max_rows.restype = i64
        L.f3d_pool_workspace_bytes.argtypes = [i64, i32, i32, ctypes.POINTER(ctypes.c_size_t)]
        L.f3d_pool_workspace_bytes.restype = ctypes.c_int
        L.f3d_inbucket_pool.argtypes = [vp, vp, vp, vp, i64, i32, i32, i32, i32, f32, i32, i32, vp, vp, vp, vp, vp,
                                        ctypes.c_size_t, vp]
        L.f3d_inbucket_pool.restype = ctypes.c_int
        L.f3d_unpermute.argtypes = [vp, vp, i64, i32, vp, vp]
        L.f3d_unpermute.restype = ctypes.c_int
        L.f3d_error_string.argtypes = [ctypes.c_int]
        L.f3d_error_string.restype = ctypes.c_char_p
        L.f3d_last_hip_error.restype = ctypes.c_int
        L.f3d_version.restype = ctypes.c_int
        _lib = L
    return _lib


def error_string(code: int) -> str:
    return lib().f3d_error_string(code).decode()


def version() -> int:
    return int(lib().f3d_version())


def make_params(voxel_size: float, bucket_cap: int, scope_buckets: int = 4, hash: str = "zorder_div",
                n_probes: int = 6, div: int = 0, probe_step: int = 0, max_scan_points: int = 0,
                schedule: str = "auto", order: str = "index", probe_mode: str = "axes", probe_seed: int = 0,
                probe_table=None) -> f3d_params:
    """f3d_params with the defaults of f3d_params_default. probe_table: up to 6 rows of 3 voxel offsets (ints)."""
    p = f3d_params()
    lib().f3d_params_default(ctypes.byref(p), voxel_size, bucket_cap)
    p.scope_buckets = scope_buckets
    p.hash = HASHES[hash] if isinstance(hash, str) else int(hash)
    p.n_probes = n_probes
    p.div = div
    p.probe_step = probe_step
    p.max_scan_points = max_scan_points
    p.schedule = SCHEDULES[schedule] if isinstance(schedule, str) else int(schedule)
    p.order = ORDERS[order] if isinstance(order, str) else int(order)
    p.probe_mode = PROBE_MODES[probe_mode] if isinstance(probe_mode, str) else int(probe_mode)
    p.probe_seed = int(probe_seed) & 0xFFFFFFFF
    if probe_table is not None:
        flat = [int(x) for row in probe_table for x in row]
        if len(flat) > 18:
            raise ValueError("probe_table holds at most 6 offsets")
        for i, x in enumerate(flat):
            p.probe_table[i] = x
    return p


def max_buckets(n: int, n_scans: int, params: f3d_params) -> int:
    r = int(lib().f3d_max_buckets(n, n_scans, ctypes.byref(params)))
    if r < 0:   # the call itself only says "refused"; the size query on the same arguments names the reason
        out = ctypes.c_size_t(0)
        rc = lib().f3d_workspace_bytes(n, n_scans, ctypes.byref(params), ctypes.byref(out))
        raise Flash3DError(rc if rc != F3D_OK else ERR_INVALID_ARG, "f3d_max_buckets")
    return r


def workspace_bytes(n: int, n_scans: int, params: f3d_params) -> int:
    out = ctypes.c_size_t(0)
    rc = lib().f3d_workspace_bytes(n, n_scans, ctypes.byref(params), ctypes.byref(out))
    if rc != F3D_OK:
        raise Flash3DError(rc, "f3d_workspace_bytes")
    return int(out.value)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _need(t, name: str, dtype, shape=None, optional: bool = False):
    """The C ABI sees only addresses: a tensor of the wrong type, shape or device would be read or written out of
    bounds. Refuse it here, with its name. `shape` entries of None are not checked."""
    if t is None:
        if optional:
            return
        raise ValueError(f"{name} is required")
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous CUDA tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, not {t.dtype}")
    if shape is not None:
        if t.dim() != len(shape) or any(w is not None and int(g) != int(w) for g, w in zip(t.shape, shape)):
            raise ValueError(f"{name} must have shape {tuple(shape)}, not {tuple(t.shape)}")


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


@dataclass
class Buckets:
    """Device tensors written by f3d_psh_bucketize plus the host-side layout parameters."""
    perm: "object"
    inv_perm: "object"
    offsets: "object"
    scan_bucket_start: "object"
    placed_per_round: "object"
    n: int
    n_scans: int
    bucket_cap: int
    scope_buckets: int
    max_buckets: int = 0


def _check_buckets(b: "Buckets", needs_perm: bool) -> None:
    import torch
    _need(b.offsets, "buckets.offsets", torch.int32, (None,))
    if int(b.offsets.shape[0]) < b.max_buckets + 1:
        raise ValueError("buckets.offsets is shorter than max_buckets + 1")
    _need(b.scan_bucket_start, "buckets.scan_bucket_start", torch.int32, (b.n_scans + 1,))
    _need(b.perm, "buckets.perm", torch.int32, (b.n,), optional=not needs_perm)


def psh_bucketize(coords, batch_offsets, params: f3d_params, workspace=None, out: Optional[Buckets] = None,
                  static_scratch: bool = False) -> Buckets:
    """f3d_psh_bucketize on torch CUDA tensors. coords: float32 [n,3]; batch_offsets: int32 [n_scans+1] or None.
    static_scratch: call f3d_psh_bucketize_static instead (no workspace; with `out` given nothing is allocated)."""
    import torch
    _need(coords, "coords", torch.float32, (None, 3))
    n = int(coords.shape[0])
    _need(batch_offsets, "batch_offsets", torch.int32, (None,), optional=True)
    n_scans = 1 if batch_offsets is None else int(batch_offsets.shape[0]) - 1
    dev = coords.device
    if out is None:
        kmax = max_buckets(n, n_scans, params)
        out = Buckets(torch.empty(n, dtype=torch.int32, device=dev), torch.empty(n, dtype=torch.int32, device=dev),
                      torch.empty(kmax + 1, dtype=torch.int32, device=dev),
                      torch.empty(n_scans + 1, dtype=torch.int32, device=dev),
                      torch.empty(8, dtype=torch.int32, device=dev), n, n_scans, params.bucket_cap, params.scope_buckets, kmax)
    else:
        if out.n != n or out.n_scans != n_scans:
            raise ValueError("`out` was made for another input size")
        _need(out.perm, "out.perm", torch.int32, (n,))
        _need(out.inv_perm, "out.inv_perm", torch.int32, (n,), optional=True)
        _need(out.offsets, "out.offsets", torch.int32, (max_buckets(n, n_scans, params) + 1,))
        _need(out.scan_bucket_start, "out.scan_bucket_start", torch.int32, (n_scans + 1,))
        _need(out.placed_per_round, "out.placed_per_round", torch.int32, (8,), optional=True)
    if static_scratch:
        rc = lib().f3d_psh_bucketize_static(_ptr(coords), _ptr(batch_offsets), n, n_scans, ctypes.byref(params), _ptr(out.perm),
                                            _ptr(out.inv_perm), _ptr(out.offsets), _ptr(out.scan_bucket_start),
                                            _ptr(out.placed_per_round), _stream())
        if rc != F3D_OK:
            raise Flash3DError(rc, "f3d_psh_bucketize_static")
        return out
    if workspace is None:
        workspace = torch.empty(workspace_bytes(n, n_scans, params), dtype=torch.uint8, device=dev)
    _need(workspace, "workspace", torch.uint8, (None,))
    rc = lib().f3d_psh_bucketize(_ptr(coords), _ptr(batch_offsets), n, n_scans, ctypes.byref(params), _ptr(out.perm),
                                 _ptr(out.inv_perm), _ptr(out.offsets), _ptr(out.scan_bucket_start),
                                 _ptr(out.placed_per_round), _ptr(workspace), workspace.numel(), _stream())
    if rc != F3D_OK:
        raise Flash3DError(rc, "f3d_psh_bucketize")
    return out


def bucket_swin_attn(q, k, v, buckets: Buckets, heads: int, head_dim: int, mode: str = "plain", shift: int = 2,
                     stride: int = 2, use_perm: bool = True, softmax_scale: float = 0.0, out=None, original_order: bool = False,
                     lse=None):
    """f3d_bucket_swin_attn (bfloat16 tensors) or f3d_bucket_swin_attn_f16 (float16 tensors), by the dtype of q.
    q,k,v: [n, heads*head_dim]; rows in input order when use_perm, else already bucket-major. Returns the same dtype
    [n, heads*head_dim] in bucket-major row order, or, with original_order, in the input order of the points (the
    unpermute folded into the kernel's store). lse: optional float32 [n, heads] tensor that receives the rows'
    log-sum-exp (bucket-major), for the backward pass."""
    import torch
    if q.dtype not in (torch.bfloat16, torch.float16):
        raise TypeError("q, k, v must be bfloat16 or float16")
    shape = (buckets.n, heads * head_dim)
    for name, t in (("q", q), ("k", k), ("v", v)):
        _need(t, name, q.dtype, shape)
    if out is None:
        out = torch.empty_like(q)
    _need(out, "out", q.dtype, shape)
    _need(lse, "lse", torch.float32, (buckets.n, heads), optional=True)
    _check_buckets(buckets, use_perm or original_order)
    entry = lib().f3d_bucket_swin_attn if q.dtype == torch.bfloat16 else lib().f3d_bucket_swin_attn_f16
    rc = entry(_ptr(q), _ptr(k), _ptr(v), _ptr(buckets.perm) if use_perm else None,
                                    _ptr(buckets.offsets), _ptr(buckets.scan_bucket_start), buckets.n, buckets.n_scans,
                                    buckets.max_buckets, buckets.bucket_cap, buckets.scope_buckets, MODES[mode] if isinstance(mode, str) else mode,
                                    shift, stride, heads, head_dim, softmax_scale, _ptr(out),
                                    _ptr(buckets.perm) if original_order else None, _ptr(lse), _stream())
    if rc != F3D_OK:
        raise Flash3DError(rc, "f3d_bucket_swin_attn")
    return out


def attn_block_rows(buckets: "Buckets", heads: int, head_dim: int, mode: str = "plain", stride: int = 2) -> int:
    """f3d_attn_block_rows: query rows per workgroup (128 or 256) the attention kernel uses on this layout."""
    r = int(lib().f3d_attn_block_rows(buckets.n_scans, buckets.max_buckets, buckets.bucket_cap, buckets.scope_buckets,
                                      MODES[mode] if isinstance(mode, str) else mode, stride, heads, head_dim))
    if r < 0:
        raise Flash3DError(r, "f3d_attn_block_rows")
    return r


def bucket_swin_attn_bwd(q, k, v, out, dout, lse, buckets: Buckets, heads: int, head_dim: int, mode: str = "plain",
                         shift: int = 2, stride: int = 2, use_perm: bool = True, softmax_scale: float = 0.0,
                         original_order: bool = False, workspace=None):
    """f3d_bucket_swin_attn_bwd. out, dout: bfloat16 [n, C] bucket-major; lse: float32 [n, heads] from the forward
    call. Returns (dq, dk, dv), bfloat16 [n, C], bucket-major rows or, with original_order, input order."""
    import torch
    n = buckets.n
    for name, t in (("q", q), ("k", k), ("v", v), ("out", out), ("dout", dout)):
        _need(t, name, torch.bfloat16, (n, heads * head_dim))
    _need(lse, "lse", torch.float32, (n, heads))
    _check_buckets(buckets, use_perm or original_order)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
    if workspace is None:
        nb = ctypes.c_size_t(0)
        lib().f3d_attn_bwd_workspace_bytes(n, heads, ctypes.byref(nb))
        workspace = torch.empty(max(int(nb.value), 256), dtype=torch.uint8, device=q.device)
    rc = lib().f3d_bucket_swin_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(dout), _ptr(lse),
                                        _ptr(buckets.perm) if use_perm else None, _ptr(buckets.offsets),
                                        _ptr(buckets.scan_bucket_start), n, buckets.n_scans, buckets.max_buckets,
                                        buckets.bucket_cap, buckets.scope_buckets, MODES[mode] if isinstance(mode, str) else mode,
                                        shift, stride, heads, head_dim, softmax_scale, _ptr(dq), _ptr(dk), _ptr(dv),
                                        _ptr(buckets.perm) if original_order else None, _ptr(workspace), workspace.numel(), _stream())
    if rc != F3D_OK:
        raise Flash3DError(rc, "f3d_bucket_swin_attn_bwd")
    return dq, dk, dv


def ln_linear(x, w, bias=None, gamma=None, beta=None, eps: float = 1e-5, row_in=None, residual=None, row_out=None,
              n_outs: int = 1):
    """f3d_ln_linear on torch CUDA tensors. x bfloat16 [n, c_in]; w bfloat16 [c_out, c_in]; gamma/beta/bias float32.
    Returns a tuple of n_outs bfloat16 tensors [n, c_out / n_outs]."""
    import torch
    n, c_in = int(x.shape[0]), int(x.shape[1])
    c_out = int(w.shape[0])
    _need(x, "x", torch.bfloat16, (n, c_in))
    _need(w, "w", torch.bfloat16, (c_out, c_in))
    if n_outs < 1 or c_out % n_outs:
        raise ValueError("c_out must be a multiple of n_outs")
    _need(gamma, "gamma", torch.float32, (c_in,), optional=True)
    _need(beta, "beta", torch.float32, (c_in,), optional=True)
    _need(bias, "bias", torch.float32, (c_out,), optional=True)
    _need(residual, "residual", torch.bfloat16, (n, c_out), optional=True)
    _need(row_in, "row_in", torch.int32, (n,), optional=True)
    _need(row_out, "row_out", torch.int32, (n,), optional=True)
    outs = tuple(torch.empty(n, c_out // n_outs, dtype=torch.bfloat16, device=x.device) for _ in range(n_outs))
    arr = (ctypes.c_void_p * n_outs)(*[t.data_ptr() for t in outs])
    rc = lib().f3d_ln_linear(_ptr(x), _ptr(row_in), _ptr(gamma), _ptr(beta), eps, _ptr(w), _ptr(bias), _ptr(residual), n, c_in,
                             c_out, arr, n_outs, _ptr(row_out), _stream())
    if rc != F3D_OK:
        raise Flash3DError(rc, "f3d_ln_linear")
    return outs


@dataclass
class Pooled:
    """Outputs of f3d_inbucket_pool (torch tensors on the GPU); rows past pooled_offsets[-1] are unspecified."""
    feat: object            # bfloat16 [max_rows, C]
    coords: object          # float32 [max_rows, 3]
    sub_of: object          # int32 [n]
    pooled_offsets: object  # int32 [n_scans + 1]
    max_rows: int


def pool_max_rows(n: int, n_scans: int, tile: int, rho: int) -> int:
    r = int(lib().f3d_pool_max_rows(n, n_scans, tile, rho))
    if r < 0:
        raise Flash3DError(ERR_INVALID_ARG, "f3d_pool_max_rows")
    return r


def pool_workspace_bytes(n: int, n_scans: int, tile: int) -> int:
    nb = ctypes.c_size_t(0)
    rc = lib().f3d_pool_workspace_bytes(n, n_scans, tile, ctypes.byref(nb))
    if rc != F3D_OK:
        raise Flash3DError(rc, "f3d_pool_workspace_bytes")
    return int(nb.value)


def inbucket_pool(coords, perm, feat, batch_offsets, tile: int, rho: int, voxel_size: float, hash: str = "zorder_div",
                  op: str = "mean", workspace=None, out: Optional[Pooled] = None) -> Pooled:
    """f3d_inbucket_pool on torch CUDA tensors. coords float32 [n,3] (input order with perm, else bucket-major);
    feat bfloat16 [n,C] bucket-major; batch_offsets int32 [n_scans+1] or None."""
    import torch
    n, C = int(feat.shape[0]), int(feat.shape[1])
    _need(coords, "coords", torch.float32, (n, 3))
    _need(feat, "feat", torch.bfloat16, (n, C))
    _need(perm, "perm", torch.int32, (n,), optional=True)
    _need(batch_offsets, "batch_offsets", torch.int32, (None,), optional=True)
    n_scans = 1 if batch_offsets is None else int(batch_offsets.shape[0]) - 1
    dev = feat.device
    if out is None:
        mr = pool_max_rows(n, n_scans, tile, rho)
        out = Pooled(torch.empty(mr, C, dtype=torch.bfloat16, device=dev), torch.empty(mr, 3, dtype=torch.float32, device=dev),
                     torch.empty(n, dtype=torch.int32, device=dev), torch.empty(n_scans + 1, dtype=torch.int32, device=dev), mr)
    else:
        mr = pool_max_rows(n, n_scans, tile, rho)
        _need(out.feat, "out.feat", torch.bfloat16, (mr, C))
        _need(out.coords, "out.coords", torch.float32, (mr, 3))
        _need(out.sub_of, "out.sub_of", torch.int32, (n,))
        _need(out.pooled_offsets, "out.pooled_offsets", torch.int32, (n_scans + 1,))
    _need(workspace, "workspace", torch.uint8, (None,), optional=True)
    if workspace is None:
        nb = ctypes.c_size_t(0)
        rc = lib().f3d_pool_workspace_bytes(n, n_scans, tile, ctypes.byref(nb))
        if rc != F3D_OK:
            raise Flash3DError(rc, "f3d_pool_workspace_bytes")
        workspace = torch.empty(max(int(nb.value), 256), dtype=torch.uint8, device=dev)
    rc = lib().f3d_inbucket_pool(_ptr(coords), _ptr(perm), _ptr(feat), _ptr(batch_offsets), n, n_scans, C, tile, rho,
                                 voxel_size, HASHES[hash] if isinstance(hash, str) else int(hash),
                                 POOL_OPS[op] if isinstance(op, str) else int(op), _ptr(out.feat), _ptr(out.coords),
                                 _ptr(out.sub_of), _ptr(out.pooled_offsets), _ptr(workspace), workspace.numel(), _stream())
    if rc != F3D_OK:
        raise Flash3DError(rc, "f3d_inbucket_pool")
    return out


def unpermute(src, perm, out=None):
    """f3d_unpermute: out[perm[p]] = src[p] for a contiguous 2-D tensor."""
    import torch
    _need(src, "src", src.dtype, (None, None))
    _need(perm, "perm", torch.int32, (int(src.shape[0]),))
    if out is None:
        out = torch.empty_like(src)
    _need(out, "out", src.dtype, tuple(src.shape))
    rc = lib().f3d_unpermute(_ptr(src), _ptr(perm), int(src.shape[0]), int(src.shape[1] * src.element_size()), _ptr(out),
                             _stream())
    if rc != F3D_OK:
        raise Flash3DError(rc, "f3d_unpermute")
    return out
