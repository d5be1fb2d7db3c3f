"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol include/kvswap_hip.h declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

import paper_2511_11907_amd as kv
from paper_2511_11907_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "kvswap_hip.h")

OK, E_NULL, E_SHAPE, E_DTYPE, E_UNSUP, E_WS, E_DEV, E_ALIGN, E_SCRATCH = range(9)


def _declared():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(kvs_[a-z_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = kv.load_library()
    names = _declared()
    assert set(names) == set(binding.EXPORTS), names
    for n in names:
        assert getattr(lib, n) is not None
    assert "gfx950" in kv.kvs_version()


def test_python_binding_has_the_same_names_as_the_header():
    for n in _declared():
        assert callable(getattr(kv, n)), n


def test_status_strings():
    seen = {kv.kvs_status_str(i) for i in range(9)}
    assert len(seen) == 9 and "ok" in seen
    assert kv.kvs_status_str(99) == "unknown status"


def _p(**kw):
    base = dict(batch=1, n_q_heads=32, n_kv_heads=8, head_dim=128, rank=32, ctx_len=32768,
                group_size=4, n_select=820)
    base.update(kw)
    return kv.Params(**base)


@pytest.mark.parametrize("kw,code", [
    (dict(), OK),
    (dict(batch=0), E_SHAPE),
    (dict(n_q_heads=30), E_SHAPE),            # H_q % H_kv
    (dict(ctx_len=32770), E_SHAPE),           # N % G
    (dict(n_select=0), E_SHAPE),
    (dict(n_select=8193), E_SHAPE),           # M > NG
    (dict(rank=128, head_dim=64), E_SHAPE),   # r > d
    (dict(softmax_scale=-1.0), E_SHAPE),
    (dict(kv_dtype=5), E_DTYPE),
    (dict(meta_dtype=-1), E_DTYPE),
    (dict(reduce=2), E_DTYPE),
    (dict(head_dim=96, rank=32), E_UNSUP),
    (dict(rank=48), E_UNSUP),
    (dict(group_size=3, ctx_len=32769), OK),  # any group size up to 16
    (dict(group_size=12, ctx_len=32760), OK),
    (dict(group_size=12), E_SHAPE),           # 32768 is not a multiple of 12
    (dict(group_size=17, ctx_len=17 * 1900), E_UNSUP),
    (dict(group_size=32), E_UNSUP),
    (dict(n_q_heads=24), OK),                 # 3 heads per kv head (LLaMA3-3B)
    (dict(n_q_heads=40), OK),                 # 5 (Qwen3-14B)
    (dict(n_q_heads=56), OK),                 # 7 (Qwen2.5-VL-7B has 28 / 4)
    (dict(n_q_heads=72), E_UNSUP),            # 9 heads per kv head
    (dict(n_q_heads=128), E_UNSUP),           # 16 heads per kv head
    (dict(group_size=1, ctx_len=65536, n_select=10), E_UNSUP),  # NG > 32768
    (dict(group_size=1, ctx_len=32768, n_select=10), OK),
    # joint-head mode: one adapter over the H_kv*d flattened keys
    (dict(head_mode=1), OK),
    (dict(head_mode=1, rank=128, head_dim=64), OK),          # r may exceed d, not H_kv*d
    (dict(head_mode=1, n_kv_heads=1, n_q_heads=4, rank=128, head_dim=64), E_SHAPE),
    (dict(head_mode=1, n_kv_heads=64, n_q_heads=64), E_UNSUP),  # H_kv*d > 4096
    (dict(head_mode=2), E_DTYPE),
    # 8-bit metadata, metadata scale
    (dict(meta_dtype=2), OK),
    (dict(meta_dtype=2, meta_scale=0.125, rank=16), OK),
    (dict(kv_dtype=2), E_DTYPE),              # keys and values are not stored in 8 bits
    (dict(meta_dtype=3), E_DTYPE),
    (dict(meta_scale=-0.5), E_SHAPE),
    (dict(meta_scale=float("inf")), E_SHAPE),
])
def test_check_params(kw, code):
    assert kv.kvs_check_params(_p(**kw)) == code
    if code != OK:
        assert kv.kvs_workspace_bytes(_p(**kw)) == 0
    else:
        assert kv.kvs_workspace_bytes(_p(**kw)) > 0


def test_workspace_covers_scores_and_partials():
    p = _p()
    ws = kv.kvs_workspace_bytes(p)
    assert ws >= 8 * 8192 * 4 + 8 * 4 * 130 * 4 + 2 * 8 * 4  # scores, one split, counters
    assert ws % 256 == 0
    assert kv.kvs_workspace_bytes(_p(batch=8)) > ws


def test_joint_mode_needs_less_workspace_for_scores_and_a_workspace_for_the_projection():
    sep, jnt = _p(batch=8), _p(batch=8, head_mode=1)
    assert kv.kvs_workspace_bytes(jnt) < kv.kvs_workspace_bytes(sep)   # one score row per sequence
    lib = kv.load_library()
    fake, null = ctypes.c_void_p(0x10000), ctypes.c_void_p(0)
    c = jnt._c()
    # the low-rank queries live in the workspace: scoring without one is refused on the host
    assert lib.kvs_predict_scores(ctypes.byref(c), fake, fake, fake, fake, null, 0, null) == E_WS


def test_entry_points_reject_bad_arguments_before_any_launch():
    """Raw calls with fake (never dereferenced) device addresses: every error below is
    detected on the host, so this is safe without a GPU."""
    lib = kv.load_library()
    c = _p()._c()
    fake = ctypes.c_void_p(0x10000)
    odd = ctypes.c_void_p(0x10004)
    null = ctypes.c_void_p(0)
    big = 1 << 30
    f = lib.kvs_predict_select
    assert f(None, fake, fake, fake, fake, null, fake, big, null) == E_NULL
    assert f(ctypes.byref(c), null, fake, fake, fake, null, fake, big, null) == E_NULL
    assert f(ctypes.byref(c), fake, fake, fake, null, null, fake, big, null) == E_NULL
    assert f(ctypes.byref(c), fake, odd, fake, fake, null, fake, big, null) == E_ALIGN
    assert f(ctypes.byref(c), fake, fake, fake, fake, null, null, big, null) == E_WS
    assert f(ctypes.byref(c), fake, fake, fake, fake, null, fake, 1024, null) == E_WS
    assert f(ctypes.byref(c), fake, fake, fake, fake, null, odd, big, null) == E_WS
    g = lib.kvs_sparse_decode_attn
    assert g(ctypes.byref(c), fake, fake, null, fake, fake, fake, big, null) == E_NULL
    assert g(ctypes.byref(c), fake, fake, fake, fake, odd, fake, big, null) == E_ALIGN
    assert g(ctypes.byref(c), fake, fake, fake, fake, fake, fake, 16, null) == E_WS
    bad = _p(n_select=9000)._c()
    assert g(ctypes.byref(bad), fake, fake, fake, fake, fake, fake, big, null) == E_SHAPE
    assert f(ctypes.byref(bad), fake, fake, fake, fake, null, fake, big, null) == E_SHAPE
    w = lib.kvs_workspace_init
    assert w(ctypes.byref(c), null, big, null) == E_WS
    assert w(ctypes.byref(c), fake, 8, null) == E_WS
    assert w(None, fake, big, null) == E_NULL
    h = lib.kvs_build_metadata
    assert h(ctypes.byref(c), null, fake, fake, null) == E_NULL
    assert h(ctypes.byref(c), fake, odd, fake, null) == E_ALIGN
    unsup = _p(rank=48)._c()
    assert h(ctypes.byref(unsup), fake, fake, fake, null) == E_UNSUP
    s = lib.kvs_decode_step
    assert s(ctypes.byref(c), fake, fake, fake, fake, null, fake, null, fake, fake, big, null) == E_NULL
    assert s(ctypes.byref(c), fake, fake, fake, fake, fake, fake, null, fake, fake, 64, null) == E_WS


def test_rolling_buffer_capacity_and_append_arguments_are_checked_on_the_host():
    lib = kv.load_library()
    fake, odd, null = ctypes.c_void_p(0x10000), ctypes.c_void_p(0x10004), ctypes.c_void_p(0)
    big = 1 << 30
    assert kv.kvs_check_params(_p(ctx_capacity=32768 + 64)) == OK
    assert kv.kvs_check_params(_p(ctx_capacity=32000)) == E_SHAPE           # capacity < ctx_len
    assert kv.kvs_check_params(_p(ctx_capacity=1 << 24)) == E_UNSUP         # capacity * d >= 2^31
    c = _p(ctx_capacity=32768 + 8)._c()
    a = lib.kvs_sparse_decode_attn_rb
    args = lambda rk, rv, n, cap: (ctypes.byref(c), fake, fake, fake, fake, rk, rv, n, cap, fake, fake, big, null)
    assert a(*args(null, null, 3, 4)) == E_NULL                             # tokens but no buffer
    assert a(*args(fake, fake, 5, 4)) == E_SHAPE                            # rb_len > capacity
    assert a(*args(fake, fake, -1, 4)) == E_SHAPE
    assert a(*args(fake, odd, 2, 4)) == E_ALIGN
    assert a(*args(fake, fake, 300, 512)) == E_UNSUP                        # rb_len > 256
    s = lib.kvs_decode_step_rb
    assert s(ctypes.byref(c), fake, fake, fake, fake, fake, null, null, 2, 4, fake, null, fake, fake, big, null) == E_NULL
    assert s(ctypes.byref(c), fake, fake, fake, fake, fake, fake, fake, 9, 4, fake, null, fake, fake, big, null) == E_SHAPE
    g = lib.kvs_append_group
    assert g(ctypes.byref(c), null, fake, 4, fake, fake, fake, fake, null) == E_NULL
    assert g(ctypes.byref(c), fake, fake, 3, fake, fake, fake, fake, null) == E_SHAPE      # buffer < one group
    full = _p()._c()                                                                       # no spare rows
    assert g(ctypes.byref(full), fake, fake, 4, fake, fake, fake, fake, null) == E_SHAPE
    assert g(ctypes.byref(c), fake, odd, 4, fake, fake, fake, fake, null) == E_ALIGN
    r = lib.kvs_build_metadata_rows
    assert r(ctypes.byref(c), fake, fake, fake, 32768, 16, null) == E_SHAPE                # leaves the capacity
    assert r(ctypes.byref(c), fake, fake, fake, -1, 4, null) == E_SHAPE
    assert r(ctypes.byref(c), null, fake, fake, 0, 4, null) == E_NULL


def test_mapping_table_and_overlap_arguments_are_checked_on_the_host():
    lib = kv.load_library()
    fake, odd, null = ctypes.c_void_p(0x10000), ctypes.c_void_p(0x10004), ctypes.c_void_p(0)
    big = 1 << 30
    c = _p()._c()
    a = lib.kvs_sparse_decode_attn_paged
    args = lambda tab, n: (ctypes.byref(c), fake, fake, fake, tab, n, fake, null, null, 0, 0, fake, fake, big, null)
    assert a(*args(null, 100)) == E_NULL
    assert a(*args(fake, 0)) == E_SHAPE
    assert a(*args(odd, 100)) == E_ALIGN
    assert a(ctypes.byref(c), fake, fake, fake, fake, 100, fake, null, null, 0, 0, fake, fake, 64, null) == E_WS
    o = lib.kvs_selection_overlap
    assert o(ctypes.byref(c), fake, null, fake, null) == E_NULL
    assert o(ctypes.byref(c), fake, fake, odd, null) == E_ALIGN
    assert o(ctypes.byref(_p(n_select=0)._c()), fake, fake, fake, null) == E_SHAPE


def test_binding_refuses_host_tensors():
    torch = pytest.importorskip("torch")
    p = _p(ctx_len=64, n_select=2)
    q = torch.zeros(1, 32, 128, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        kv.kvs_predict_select(p, q, q, q, q, None, None)


def test_reciprocal_division_used_by_the_attention_kernels_is_exact():
    """The attention kernels turn a position of the attended-token list into its group with
    one multiply-high by floor(2^32 / G) + 1 when G is not a power of two.  That equals
    position // G for every position below 2^28 / G; the largest position the library can
    see is 32768 groups * 16 tokens + 256 buffer tokens."""
    import numpy as np
    top = 32768 * 16 + 256 + 64
    pos = np.arange(top, dtype=np.uint64)
    edge = np.array([2 ** 28 // 16 - 1], dtype=np.uint64)
    for G in (3, 5, 6, 7, 9, 10, 11, 12, 13, 14, 15):
        recip = np.uint64((1 << 32) // G + 1)
        assert recip < (1 << 32)
        for x in (pos, edge):
            assert np.array_equal((x * recip) >> np.uint64(32), x // np.uint64(G)), G


def test_static_scratch_entry_point_refuses_what_does_not_fit_before_any_launch():
    """kvs_decode_step_static: NULL pointers, bad params and problems whose scratch memory
    exceeds the library's static buffer are refused on the host (fake addresses, no GPU)."""
    lib = kv.load_library()
    fake, null = ctypes.c_void_p(0x10000), ctypes.c_void_p(0)
    call = lambda p, *a: lib.kvs_decode_step_static(ctypes.byref(p._c()), *a)
    ok = _p()
    assert kv.kvs_workspace_bytes(ok) <= kv.KVS_STATIC_SCRATCH_BYTES
    assert call(ok, null, fake, fake, fake, fake, fake, null, fake, null) == E_NULL
    assert call(ok, fake, fake, fake, fake, fake, fake, null, null, null) == E_NULL
    assert call(_p(n_select=0), fake, fake, fake, fake, fake, fake, null, fake, null) == E_SHAPE
    big = _p(batch=64)     # 512 problems: histograms and scores alone exceed the buffer
    assert kv.kvs_workspace_bytes(big) > kv.KVS_STATIC_SCRATCH_BYTES
    assert call(big, fake, fake, fake, fake, fake, fake, null, fake, null) == E_SCRATCH
    # the header's constant and the binding's agree
    text = open(HEADER).read()
    assert re.search(r"#define\s+KVS_STATIC_SCRATCH_BYTES\s+\(8u\s*<<\s*20\)", text)
    assert kv.KVS_STATIC_SCRATCH_BYTES == 8 << 20


def test_pipelined_entry_point_checks_its_arguments_on_the_host():
    """kvs_attend_select_next: NULL pointers, misaligned buffers, a missing or short
    workspace and layouts outside its set are refused before any launch (fake addresses)."""
    lib = kv.load_library()
    fake, odd, null = ctypes.c_void_p(0x10000), ctypes.c_void_p(0x10004), ctypes.c_void_p(0)
    big = 1 << 30
    f = lambda p, *a: lib.kvs_attend_select_next(ctypes.byref(p._c()), *a)
    ok = _p()          # bf16, d = 128, four query heads per KV head
    assert f(ok, fake, fake, fake, fake, fake, null, fake, fake, big, null) == E_NULL      # no scores
    assert f(ok, fake, fake, fake, fake, fake, fake, null, fake, big, null) == E_NULL      # no next_idx
    assert f(ok, fake, fake, fake, null, fake, fake, fake, fake, big, null) == E_NULL      # no idx
    assert f(ok, fake, fake, fake, fake, fake, odd, fake, fake, big, null) == E_ALIGN
    assert f(ok, fake, fake, fake, fake, fake, fake, fake, null, big, null) == E_WS
    assert f(ok, fake, fake, fake, fake, fake, fake, fake, fake, 64, null) == E_WS
    fp32 = _p(kv_dtype=kv.KVS_F32, meta_dtype=kv.KVS_F32, head_dim=64)
    assert f(fp32, fake, fake, fake, fake, fake, fake, fake, fake, big, null) == E_UNSUP
    two_heads = _p(n_q_heads=16, n_kv_heads=8)
    assert f(two_heads, fake, fake, fake, fake, fake, fake, fake, fake, big, null) == E_UNSUP
    g = lambda p, *a: lib.kvs_attend_select_next_rb(ctypes.byref(p._c()), *a)
    assert g(ok, fake, fake, fake, fake, null, null, 3, 8, fake, fake, fake, fake, big, null) == E_NULL   # rb_len without a buffer
    assert g(ok, fake, fake, fake, fake, fake, fake, 9, 8, fake, fake, fake, fake, big, null) == E_SHAPE  # rb_len > capacity
    assert g(ok, fake, fake, fake, fake, fake, fake, 3, 8, fake, fake, fake, null, big, null) == E_WS
    long_ctx = _p(ctx_len=131072, n_select=1638)      # 32768 groups: beyond one 512-lane workgroup's keys
    assert f(long_ctx, fake, fake, fake, fake, fake, fake, fake, fake, big, null) == E_UNSUP
