"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function the
header declares, and refuses bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2312_04985_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000      # 16-byte aligned, never dereferenced: validation fails first


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sparq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"^(?:int|const char\*)\s+(\w+)\s*\(", text, flags=re.M)))


def test_library_exports_every_declared_function():
    names = declared_functions()
    assert set(names) == set(B.EXPORTS) and len(names) >= 8
    lib = B.load()
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings():
    assert B.status_string(0) == "ok"
    assert len({B.status_string(s) for s in (0, -1, -2, -3, -4, -99)}) == 6


def shape(**kw):
    d = dict(B=2, H=4, H_kv=2, S_max=128, d_h=128, r=16, k=8, dtype=0, flags=0, local_window=0, S_bound=0)
    d.update(kw)
    return B.SparqShape(*[d[f] for f, _ in B.SparqShape._fields_])


def test_stage_clocks_exist_only_in_a_profiling_build():
    """The default library records no time stamps and says so; a profiling build (if one has been made) describes
    where it leaves them and asks for the room in the workspace."""
    with pytest.raises(B.SparqError) as e:
        B.sparq_stage_clocks(shape())
    assert e.value.status == B.SPARQ_EUNSUPPORTED
    from paper_2312_04985_amd import build
    if os.path.exists(build.LIB_CLOCKS):
        lib = ctypes.CDLL(build.LIB_CLOCKS)
        off, n, m = ctypes.c_size_t(0), ctypes.c_int32(0), ctypes.c_int32(0)
        sh = shape()
        assert lib.sparq_stage_clocks(ctypes.byref(sh), ctypes.byref(off), ctypes.byref(n), ctypes.byref(m)) == 0
        assert (off.value, n.value, m.value) == (65536, 2 * 4, 9)
        need = ctypes.c_size_t(0)
        assert lib.sparq_workspace_bytes(ctypes.byref(sh), ctypes.byref(need)) == 0
        assert need.value >= 65536 + 8 * 9 * 8


def test_a_bound_on_the_lengths_sizes_plan_and_workspace():
    """With S_bound set, the plan and the workspace are those of a cache of S_bound positions."""
    many = dict(B=64, H=32, H_kv=32, r=16, k=256)
    assert "one workgroup per head" in B.sparq_decode_plan(shape(S_max=8192, **many))
    assert "two-level" in B.sparq_decode_plan(shape(S_max=65536, **many))
    assert "one workgroup per head" in B.sparq_decode_plan(shape(S_max=65536, S_bound=8192, **many))
    assert B.sparq_workspace_bytes(shape(S_max=65536, S_bound=8192, **many)) == B.sparq_workspace_bytes(shape(S_max=8192, **many))
    few = dict(B=1, H=32, H_kv=8, r=32, k=2048, dtype=1)
    assert "digit-bucket" in B.sparq_decode_plan(shape(S_max=131072, S_bound=32768, **few))
    assert B.sparq_workspace_bytes(shape(S_max=131072, S_bound=32768, **few)) == B.sparq_workspace_bytes(shape(S_max=32768, **few))
    assert B.sparq_workspace_bytes(shape(S_max=131072, S_bound=131072, **few)) == B.sparq_workspace_bytes(shape(S_max=131072, **few))
    assert "one workgroup per head" in B.sparq_decode_plan(shape(S_max=131072, S_bound=4096, **few))


def test_plan_choice_between_the_bucket_plan_and_one_workgroup_per_unit():
    """Few units with long caches go to the digit-bucket plan only where it was measured faster (or where one
    workgroup cannot hold the keys)."""
    plan = lambda **kw: B.sparq_decode_plan(shape(H=32, H_kv=32, r=32, k=512, **kw))
    one, bucket = "one workgroup per head", "digit-bucket"
    assert one in plan(B=1, S_max=8192) and one in plan(B=4, S_max=8192) and one in plan(B=2, S_max=12224)
    assert bucket in plan(B=1, S_max=12288) and bucket in plan(B=2, S_max=12288) and one in plan(B=3, S_max=12288)
    assert bucket in plan(B=3, S_max=16384) and one in plan(B=4, S_max=16384)
    assert bucket in plan(B=3, S_max=32768) and one in plan(B=4, S_max=32768) and one in plan(B=16, S_max=32768)
    assert bucket in plan(B=4, S_max=65536)                      # beyond one workgroup's LDS: up to 128 units
    assert "two-level" in plan(B=5, S_max=65536)


def test_workspace_bytes_and_shape_validation():
    need = B.sparq_workspace_bytes(shape())
    assert need >= 256 + 2 * 4 * (128 + 2) * 4
    assert B.sparq_workspace_bytes(shape(S_max=32768, B=1, H=32, H_kv=8)) > need
    for bad, code in [(dict(S_max=100), B.SPARQ_EINVAL), (dict(H=5), B.SPARQ_EINVAL), (dict(r=0), B.SPARQ_EINVAL),
                      (dict(r=129), B.SPARQ_EINVAL), (dict(k=0), B.SPARQ_EINVAL), (dict(dtype=2), B.SPARQ_EINVAL),
                      (dict(flags=128), B.SPARQ_EINVAL), (dict(flags=32 | 64), B.SPARQ_EINVAL), (dict(flags=8 | 16), B.SPARQ_EINVAL), (dict(local_window=-1), B.SPARQ_EINVAL),
                      (dict(S_bound=-64), B.SPARQ_EINVAL), (dict(S_bound=100), B.SPARQ_EINVAL), (dict(S_bound=192), B.SPARQ_EINVAL),
                      (dict(B=0), B.SPARQ_EINVAL), (dict(d_h=80, r=16), B.SPARQ_EUNSUPPORTED)]:
        with pytest.raises(B.SparqError) as e:
            B.sparq_workspace_bytes(shape(**bad))
        assert e.value.status == code, bad


def call_decode(sh, cache, q=FAKE, out=FAKE, ws=FAKE, ws_bytes=1 << 30, idx=None, idx_stride=0):
    return B.load().sparq_decode(ctypes.byref(sh), ctypes.byref(cache), q, None, out, None, idx, idx_stride, None, ws, ws_bytes, None)


def test_bad_pointers_and_workspace_are_refused_before_any_launch():
    lib = B.load()
    good = B.SparqCache(FAKE, FAKE, FAKE, FAKE, FAKE)
    sh = shape()
    assert call_decode(sh, B.SparqCache(None, FAKE, FAKE, FAKE, FAKE)) == B.SPARQ_EINVAL
    assert call_decode(sh, B.SparqCache(FAKE, FAKE + 2, FAKE, FAKE, FAKE)) == B.SPARQ_EINVAL
    assert call_decode(sh, good, q=None) == B.SPARQ_EINVAL
    assert call_decode(sh, good, out=FAKE + 8) == B.SPARQ_EINVAL
    assert call_decode(sh, good, ws=None) == B.SPARQ_EWORKSPACE
    assert call_decode(sh, good, ws_bytes=256) == B.SPARQ_EWORKSPACE
    assert call_decode(sh, good, idx=FAKE, idx_stride=0) == B.SPARQ_EINVAL
    assert lib.dense_decode(ctypes.byref(sh), ctypes.byref(good), FAKE, FAKE, FAKE, 64, None) == B.SPARQ_EWORKSPACE
    assert lib.dense_decode(ctypes.byref(sh), ctypes.byref(good), None, FAKE, FAKE, 1 << 30, None) == B.SPARQ_EINVAL
    assert lib.sparq_kv_append(ctypes.byref(sh), ctypes.byref(good), FAKE, FAKE, 0, None, FAKE, 1 << 30, None) == B.SPARQ_EINVAL
    assert lib.sparq_kv_append(ctypes.byref(sh), ctypes.byref(good), FAKE, None, 1, None, FAKE, 1 << 30, None) == B.SPARQ_EINVAL
    assert lib.sparq_kv_append(ctypes.byref(sh), ctypes.byref(good), FAKE, FAKE, 129, None, FAKE, 1 << 30, None) == B.SPARQ_EINVAL
    assert lib.sparq_kv_append(ctypes.byref(sh), ctypes.byref(good), FAKE, FAKE, 1, None, FAKE, 16, None) == B.SPARQ_EWORKSPACE
    assert lib.sparq_copy_probe(FAKE, FAKE, 24, None) == B.SPARQ_EINVAL
    assert lib.sparq_workspace_init(None, 4096, None) == B.SPARQ_EWORKSPACE
    assert lib.sparq_async_error(None, None, None) == B.SPARQ_EINVAL


def test_shapes_without_a_kernel_are_refused_before_any_launch():
    """Sizes no plan can serve, and flag combinations without a kernel, come back as SPARQ_EUNSUPPORTED
    from the host-side planning (which assumes gfx950's 160 KiB of LDS where no device can be asked)."""
    good = B.SparqCache(FAKE, FAKE, FAKE, FAKE, FAKE)
    refused = [
        dict(S_max=1 << 20, k=64),                                   # more than 64 spans of 8192
        dict(S_max=262144, k=2048, B=8, H=32, H_kv=32),               # many heads: 32 spans x 2048 candidates do not fit in LDS
        dict(S_max=262144, k=2048, B=8, H=32, H_kv=8, flags=B.SPARQ_FLAG_GQA_SHARED),   # the same limit under the grouped-query rule
        dict(S_max=65536, flags=B.SPARQ_FLAG_SINGLE_K, H=2, H_kv=2),
        dict(H=8, H_kv=1, flags=B.SPARQ_FLAG_GQA_SHARED),            # groups of 8 query heads
        dict(flags=B.SPARQ_FLAG_GQA_SHARED | B.SPARQ_FLAG_SINGLE_K),
        dict(flags=B.SPARQ_FLAG_GQA_SHARED | B.SPARQ_FLAG_TILED_K),
        dict(S_max=65536, flags=B.SPARQ_FLAG_TILED_K, H=2, H_kv=2),     # the tiled layout is read by the one-workgroup kernel only
    ]
    for kw in refused:
        assert call_decode(shape(**kw), good) == B.SPARQ_EUNSUPPORTED, kw
    # with few heads the digit-bucket plan has no candidate limit: the same length is served
    assert call_decode(shape(S_max=262144, k=2048), good) in (B.SPARQ_OK, B.SPARQ_ELAUNCH)
    assert call_decode(shape(S_max=262144, k=2048, flags=B.SPARQ_FLAG_GQA_SHARED), good) in (B.SPARQ_OK, B.SPARQ_ELAUNCH)
    assert "digit-bucket" in B.sparq_decode_plan(shape(S_max=262144, k=2048, flags=B.SPARQ_FLAG_GQA_SHARED))
    # sizes that the multi-launch plans do serve still get a workspace size (and grow with S_max)
    a = B.sparq_workspace_bytes(shape(S_max=131072, k=2048, H=2, H_kv=2))
    b = B.sparq_workspace_bytes(shape(S_max=65536, k=2048, H=2, H_kv=2))
    assert a > b > B.sparq_workspace_bytes(shape(S_max=8192, k=2048, H=2, H_kv=2))


def test_binding_refuses_host_tensors():
    import torch
    with pytest.raises(ValueError):
        B.make_cache(torch.zeros(4), torch.zeros(4), torch.zeros(4), torch.zeros(4), torch.zeros(4, dtype=torch.int32))
