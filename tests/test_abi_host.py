"""Host-side checks of the C ABI (no GPU): the library loads, exports every declared symbol, and
refuses bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2412_16481_amd as f3d

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "flash3d.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(f3d_[a-z0-9_]+)\s*\(", text))
    names.discard("f3d_psh_bucketize_simple")          # static inline wrapper in the header
    return sorted(names)


def test_library_exports_every_declared_symbol():
    L = f3d.lib()
    names = declared_symbols()
    assert set(names) == set(f3d.EXPORTS)
    for name in names:
        assert getattr(L, name) is not None
    assert f3d.version() >= 1


def test_microbenchmark_library_is_built_and_refuses_bad_arguments_on_the_host():
    # the measurement aid of bench.py --ceilings: built by the same build step, one entry point, checked before any GPU call
    mb = ctypes.CDLL(os.path.join(ROOT, "paper_2412_16481_amd", "libf3d_microbench.so"))
    mb.f3d_mb_run.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)]
    ms, work = ctypes.c_float(0), ctypes.c_double(0)
    assert mb.f3d_mb_run(8, 4, ctypes.byref(ms), ctypes.byref(work)) != 0
    assert mb.f3d_mb_run(0, 0, ctypes.byref(ms), ctypes.byref(work)) != 0
    assert mb.f3d_mb_run(0, 9, ctypes.byref(ms), ctypes.byref(work)) != 0
    assert mb.f3d_mb_run(0, 4, None, ctypes.byref(work)) != 0


def test_params_default_and_sizes():
    p = f3d.make_params(0.02, 1024)
    assert p.struct_size == ctypes.sizeof(f3d.f3d_params)
    assert (p.scope_buckets, p.hash, p.n_probes, p.div, p.probe_step) == (4, 3, 6, 0, 0)
    assert f3d.max_buckets(200_000, 1, p) == 200_000 // 256 + 1
    assert f3d.workspace_bytes(200_000, 1, p) > 200_000 * 8
    assert f3d.workspace_bytes(0, 1, p) > 0


@pytest.mark.parametrize("kw,code", [
    (dict(voxel_size=0.0), f3d.ERR_INVALID_ARG),
    (dict(voxel_size=-1.0), f3d.ERR_INVALID_ARG),
    (dict(voxel_size=float("nan")), f3d.ERR_INVALID_ARG),
    (dict(bucket_cap=1000), f3d.ERR_INVALID_ARG),            # not a multiple of 16 * scope_buckets
    (dict(scope_buckets=0), f3d.ERR_INVALID_ARG),
    (dict(scope_buckets=32, bucket_cap=1024), f3d.ERR_UNSUPPORTED),
    (dict(hash=7), f3d.ERR_INVALID_ARG),
    (dict(n_probes=7), f3d.ERR_INVALID_ARG),
    (dict(n_probes=-1), f3d.ERR_INVALID_ARG),
    (dict(div=-1), f3d.ERR_INVALID_ARG),
    (dict(n=-1), f3d.ERR_INVALID_ARG),
    (dict(n_scans=0), f3d.ERR_INVALID_ARG),
    (dict(n=10_000_000, bucket_cap=64), f3d.ERR_UNSUPPORTED),  # one scan would own > 8192 buckets
    (dict(struct_size=4), f3d.ERR_INVALID_ARG),
    (dict(order=2), f3d.ERR_INVALID_ARG),
    (dict(order=-1), f3d.ERR_INVALID_ARG),
    (dict(probe_mode=3), f3d.ERR_INVALID_ARG),
    (dict(probe_mode=-1), f3d.ERR_INVALID_ARG),
])
def test_workspace_query_refuses_bad_parameters(kw, code):
    kw = dict(kw)
    n = kw.pop("n", 1000)
    n_scans = kw.pop("n_scans", 1)
    struct_size = kw.pop("struct_size", None)
    base = dict(voxel_size=0.02, bucket_cap=1024)
    base.update(kw)
    p = f3d.make_params(**base)
    if struct_size is not None:
        p.struct_size = struct_size
    out = ctypes.c_size_t(0)
    assert f3d.lib().f3d_workspace_bytes(n, n_scans, ctypes.byref(p), ctypes.byref(out)) == code


def test_rebalancing_variants_in_the_parameter_block():
    p = f3d.make_params(0.02, 1024)
    assert (p.order, p.probe_mode, p.probe_seed) == (0, 0, 0) and list(p.probe_table) == [0] * 18
    q = f3d.make_params(0.02, 1024, order="canonical", probe_mode="table", probe_seed=-1, probe_table=[[1, -2, 3], [4, 5, -6]])
    assert (q.order, q.probe_mode, q.probe_seed) == (1, 1, 0xFFFFFFFF)
    assert list(q.probe_table)[:6] == [1, -2, 3, 4, 5, -6]
    with pytest.raises(ValueError):
        f3d.make_params(0.02, 1024, probe_table=[[0, 0, 0]] * 7)
    # the canonical order sorts the points first and needs room for keys, indices and the sorted copy
    assert f3d.workspace_bytes(200_000, 1, q) > f3d.workspace_bytes(200_000, 1, p) + 200_000 * 48


def test_half_precision_attention_refuses_what_the_bfloat16_entry_refuses():
    L = f3d.lib()
    fake = 0x10000
    base = [fake, fake, fake, None, fake, fake, 100, 1, 10, 1024, 4, 0, 2, 2, 4, 16, 0.0, fake, None, None, None]
    def call(entry, changes):
        a = list(base)
        for k, v in changes.items():
            a[k] = v
        return entry(*a)
    for entry in (L.f3d_bucket_swin_attn, L.f3d_bucket_swin_attn_f16):
        assert call(entry, {15: 24}) == f3d.ERR_UNSUPPORTED        # head_dim
        assert call(entry, {0: None}) == f3d.ERR_INVALID_ARG       # q
        assert call(entry, {17: None}) == f3d.ERR_INVALID_ARG      # out
        assert call(entry, {17: fake + 8}) == f3d.ERR_BAD_ALIGNMENT
        assert call(entry, {11: 3}) == f3d.ERR_INVALID_ARG         # mode
        assert call(entry, {6: 0}) == 0                            # an empty input is not an error and launches nothing


def test_max_scan_points_lifts_the_bucket_limit():
    p = f3d.make_params(0.02, 64, max_scan_points=100_000)
    assert f3d.workspace_bytes(10_000_000, 200, p) > 0


def test_bucketize_refuses_null_and_misaligned_pointers_on_the_host():
    L = f3d.lib()
    p = f3d.make_params(0.02, 1024)
    fake = 0x10000  # never dereferenced: the checks fail first
    args = lambda **o: [o.get("coords", fake), None, 100, 1, ctypes.byref(p), o.get("perm", fake), None,
                        o.get("offsets", fake), o.get("sbs", fake), None, o.get("ws", fake), o.get("wsb", 1 << 30), None]
    assert L.f3d_psh_bucketize(*args(coords=None)) == f3d.ERR_INVALID_ARG
    assert L.f3d_psh_bucketize(*args(perm=None)) == f3d.ERR_INVALID_ARG
    assert L.f3d_psh_bucketize(*args(offsets=None)) == f3d.ERR_INVALID_ARG
    assert L.f3d_psh_bucketize(*args(ws=None)) == f3d.ERR_INVALID_ARG
    assert L.f3d_psh_bucketize(*args(coords=fake + 2)) == f3d.ERR_BAD_ALIGNMENT
    assert L.f3d_psh_bucketize(*args(ws=fake + 64)) == f3d.ERR_BAD_ALIGNMENT
    assert L.f3d_psh_bucketize(*args(wsb=16)) == f3d.ERR_WORKSPACE_TOO_SMALL


def test_attention_refuses_bad_arguments_on_the_host():
    L = f3d.lib()
    fake = 0x10000
    def call(**o):
        return L.f3d_bucket_swin_attn(o.get("q", fake), fake, fake, None, o.get("offsets", fake), fake, o.get("n", 100), 1, 10,
                                      o.get("cap", 1024), o.get("m", 4), o.get("mode", 0), o.get("shift", 2),
                                      o.get("stride", 2), o.get("heads", 4), o.get("d", 16), o.get("scale", 0.0), fake, o.get("out_perm"), o.get("lse"), None)
    assert call(d=24) == f3d.ERR_UNSUPPORTED
    assert call(d=64) == f3d.ERR_UNSUPPORTED
    assert call(mode=3) == f3d.ERR_INVALID_ARG
    assert call(mode=1, shift=0) == f3d.ERR_INVALID_ARG
    assert call(mode=1, shift=4) == f3d.ERR_INVALID_ARG
    assert call(mode=2, stride=0) == f3d.ERR_INVALID_ARG
    assert call(cap=1000) == f3d.ERR_INVALID_ARG
    assert call(heads=0) == f3d.ERR_INVALID_ARG
    assert call(scale=-1.0) == f3d.ERR_INVALID_ARG
    assert call(q=None) == f3d.ERR_INVALID_ARG
    assert call(out_perm=fake + 2) == f3d.ERR_BAD_ALIGNMENT
    assert call(lse=fake + 1) == f3d.ERR_BAD_ALIGNMENT
    assert call(q=fake + 2) == f3d.ERR_BAD_ALIGNMENT
    assert call(offsets=None) == f3d.ERR_INVALID_ARG
    assert call(n=-5) == f3d.ERR_INVALID_ARG
    assert call(n=0) == f3d.F3D_OK                      # nothing to do, nothing launched


def test_unpermute_refuses_bad_arguments_on_the_host():
    L = f3d.lib()
    fake = 0x10000
    assert L.f3d_unpermute(fake, fake, 10, 0, fake + 4096, None) == f3d.ERR_INVALID_ARG
    assert L.f3d_unpermute(fake, fake, 10, 6, fake + 4096, None) == f3d.ERR_INVALID_ARG
    assert L.f3d_unpermute(fake, fake, 10, 128, fake, None) == f3d.ERR_INVALID_ARG      # in place
    assert L.f3d_unpermute(None, fake, 10, 128, fake, None) == f3d.ERR_INVALID_ARG
    assert L.f3d_unpermute(fake + 1, fake, 10, 128, fake + 4096, None) == f3d.ERR_BAD_ALIGNMENT
    assert L.f3d_unpermute(fake, fake, 0, 128, fake + 4096, None) == f3d.F3D_OK


def test_error_strings():
    assert f3d.error_string(0) == "ok"
    for c in (-1, -2, -3, -4, -5):
        assert f3d.error_string(c) not in ("ok", "unknown error code")
    assert f3d.error_string(-99) == "unknown error code"


def test_product_package_never_touches_the_oracle():
    pkg = os.path.join(ROOT, "paper_2412_16481_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "import oracle" not in text and "from oracle" not in text and "orc_" not in text, fn


def test_binding_refuses_tensors_the_library_could_not_address():
    """The binding hands raw addresses to the C ABI, so it checks device, layout, dtype and shape first (no GPU needed:
    the checks run before any library call)."""
    import torch
    p = f3d.make_params(0.05, 256)
    with pytest.raises(ValueError, match="coords"):
        f3d.psh_bucketize(torch.zeros(10, 3), None, p)                       # host memory
    bk = f3d.Buckets(None, None, None, None, None, 10, 1, 256, 4, 1)
    with pytest.raises(TypeError):
        f3d.bucket_swin_attn(*(torch.zeros(10, 32) for _ in range(3)), bk, 2, 16)   # float32 features
    with pytest.raises(ValueError, match="q must be a contiguous CUDA tensor"):
        f3d.bucket_swin_attn(*(torch.zeros(10, 32, dtype=torch.bfloat16) for _ in range(3)), bk, 2, 16)
    with pytest.raises(ValueError, match="x must be"):
        f3d.ln_linear(torch.zeros(4, 64, dtype=torch.bfloat16), torch.zeros(64, 64, dtype=torch.bfloat16))
    with pytest.raises(ValueError, match="coords"):
        f3d.inbucket_pool(torch.zeros(4, 3), None, torch.zeros(4, 8, dtype=torch.bfloat16), None, 64, 2, 0.1)
    with pytest.raises(ValueError, match="src"):
        f3d.unpermute(torch.zeros(4, 8), torch.zeros(4, dtype=torch.int32))
