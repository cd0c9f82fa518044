"""Host-side checks of the C ABI: the library loads, exports every symbol the header declares,
sizes workspaces, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2504_09936_amd", "libkeepkv.so")

pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="libkeepkv.so not built")


def _declared():
    text = open(os.path.join(ROOT, "include", "keepkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(keepkv_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    lib = C.CDLL(LIB)
    names = _declared()
    assert {"keepkv_decode_attn", "keepkv_score", "keepkv_select", "keepkv_match", "keepkv_merge",
            "keepkv_append", "keepkv_workspace_bytes", "keepkv_strerror", "keepkv_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_binding_lists_the_same_entry_points():
    from paper_2504_09936_amd import binding
    assert sorted(binding.EXPORTS) == _declared()
    assert binding.version() >= 100


def test_workspace_and_argument_validation_without_device():
    from paper_2504_09936_amd import binding as kk
    lay = kk.Layout(8, 32, 8, 128, kk.BF16, 128 ** -0.5)
    small = kk.workspace_bytes(lay, 884, 820)
    big = kk.workspace_bytes(lay, 8192, 820)
    assert 0 < small < big
    assert big >= 8 * 8 * 8192 * 8                      # selection keys: one u64 per slot
    assert kk.workspace_bytes(lay, 100, 200) == 0       # budget above capacity
    bad = kk.Layout(8, 30, 8, 128, kk.BF16, 0.1)        # Hq not a multiple of Hkv
    assert kk.workspace_bytes(bad, 884, 820) == 0
    lib = kk._lib
    assert lib.keepkv_strerror(0) == b"ok"
    assert lib.keepkv_strerror(3) == b"workspace missing or too small"
    # null pointers are rejected on the host; nothing is launched
    assert lib.keepkv_score(None, None, None, C.c_float(0.9), None) == kk.ERR_INVALID_ARG
    assert lib.keepkv_decode_attn(C.byref(lay.c()), None, None, None, None, None, None, 0, None) == kk.ERR_INVALID_ARG
    cache = kk._Cache(16, 16, 16, 16, 16, 16, 16, 884, 0)     # non-null dummies; never dereferenced on these paths
    assert lib.keepkv_score(C.byref(lay.c()), C.byref(cache), C.c_void_p(16), C.c_float(1.5), None) == kk.ERR_INVALID_ARG
    lay3 = kk.Layout(8, 24, 8, 128, kk.BF16, 0.1)       # group size 3 is not built
    assert lib.keepkv_decode_attn(C.byref(lay3.c()), C.byref(cache), C.c_void_p(16), C.c_void_p(16), None, None,
                                  None, 0, None) == kk.ERR_UNSUPPORTED
    assert lib.keepkv_decode_attn(C.byref(lay.c()), C.byref(cache), C.c_void_p(16), C.c_void_p(16), None, None,
                                  None, 0, None) == kk.ERR_WORKSPACE
    assert lib.keepkv_select(C.byref(lay.c()), C.byref(cache), 820, 500, 500, C.c_float(0.9), C.c_void_p(16),
                             C.c_void_p(16), C.c_void_p(16), C.c_void_p(16), 1 << 30, None) == kk.ERR_INVALID_ARG
    # the in-place event: a missing slot list, a workspace that is too small, more evictable slots than it handles
    P16 = C.c_void_p(16)
    assert lib.keepkv_select_aged(C.byref(lay.c()), C.byref(cache), None, 820, 4, 652, C.c_float(0.9), P16, P16, P16,
                                  P16, 1 << 30, None) == kk.ERR_INVALID_ARG
    assert lib.keepkv_select_aged(C.byref(lay.c()), C.byref(cache), P16, 820, 4, 652, C.c_float(0.9), P16, P16, P16,
                                  P16, 1024, None) == kk.ERR_WORKSPACE
    assert lib.keepkv_merge_inplace(C.byref(lay.c()), C.byref(cache), None, 820, P16, P16, P16, P16, C.c_float(0.9),
                                    None, None) == kk.ERR_INVALID_ARG
    wide = kk._Cache(16, 16, 16, 16, 16, 16, 16, 820 + 257, 0)
    assert lib.keepkv_merge_inplace(C.byref(lay.c()), C.byref(wide), P16, 820, P16, P16, P16, P16, C.c_float(0.9),
                                    None, None) == kk.ERR_UNSUPPORTED
    assert lib.keepkv_merge_inplace(C.byref(lay.c()), C.byref(cache), P16, 820, P16, P16, P16, P16, C.c_float(1.0),
                                    None, None) == kk.ERR_INVALID_ARG


def test_too_many_heads_is_refused_by_every_call():
    """batch * kv heads above 16384 is outside the built range: refused on the host, nothing launched."""
    from paper_2504_09936_amd import binding as kk
    lib = kk._lib
    lay = kk.Layout(4097, 16, 4, 128, kk.BF16, 0.1)       # 16388 (batch, kv head) pairs
    cache = kk._Cache(16, 16, 16, 16, 16, 16, 16, 884, 0)     # non-null dummies; never dereferenced on these paths
    P = C.c_void_p(16)
    L, K = C.byref(lay.c()), C.byref(cache)
    assert lib.keepkv_score(L, K, P, C.c_float(0.9), None) == kk.ERR_UNSUPPORTED
    assert lib.keepkv_append(L, K, P, P, None, None) == kk.ERR_UNSUPPORTED
    assert lib.keepkv_decode_attn(L, K, P, P, None, None, P, 1 << 40, None) == kk.ERR_UNSUPPORTED
    assert lib.keepkv_decode_step(L, K, P, P, P, P, None, C.c_float(0.9), None, P, 1 << 40, None) == kk.ERR_UNSUPPORTED
    assert lib.keepkv_score_window(L, K, P, 4, C.c_float(0.9), -1, None) == kk.ERR_UNSUPPORTED
    assert lib.keepkv_select(L, K, 820, 4, 652, C.c_float(0.9), P, P, P, P, 1 << 40, None) == kk.ERR_UNSUPPORTED
    assert lib.keepkv_select_by_key(L, K, P, 820, 4, 652, P, P, P, P, 1 << 40, None) == kk.ERR_UNSUPPORTED
    assert lib.keepkv_match(L, K, 820, P, P, P, C.c_float(0.8), P, None, P, 1 << 40, None) == kk.ERR_UNSUPPORTED
    assert lib.keepkv_merge(L, K, K, 820, P, P, P, P, C.c_float(0.9), None, P, 1 << 40, None) == kk.ERR_UNSUPPORTED


def test_decode_plan_is_host_arithmetic():
    """keepkv_decode_plan needs no device: the benchmark shape gets 4 splits of 224 slots on 8-wavefront workgroups
    (256 workgroups, one per compute unit), a batch of 128 one split per head on 4-wavefront workgroups, an f32
    cache the vector-ALU kernel's 4 wavefronts; bad arguments are refused."""
    from paper_2504_09936_amd import binding as kk
    bench = kk.Layout(8, 32, 8, 128, kk.BF16, 128 ** -0.5)
    assert kk.decode_plan(bench, 884) == (4, 224, 8)
    n_split, per, waves = kk.decode_plan(kk.Layout(128, 64, 8, 128, kk.BF16, 128 ** -0.5), 884)
    assert (n_split, waves) == (1, 4) and per >= 884
    for lay, cap in ((bench, 1), (bench, 5000), (kk.Layout(1, 8, 8, 64, kk.BF16, 0.125), 333), (kk.Layout(3, 6, 3, 128, kk.F32, 0.1), 700)):
        n_split, per, waves = kk.decode_plan(lay, cap)
        assert n_split >= 1 and n_split * per >= cap and (n_split - 1) * per < cap and waves in (4, 8)
        assert per % 32 == 0
    assert kk.decode_plan(kk.Layout(3, 6, 3, 128, kk.F32, 0.1), 700)[2] == 4
    with pytest.raises(kk.KeepKVError):
        kk.decode_plan(bench, 0)
    with pytest.raises(kk.KeepKVError):
        kk.decode_plan(kk.Layout(8, 32, 8, 96, kk.BF16, 0.1), 884)        # unsupported head dimension
