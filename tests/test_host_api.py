"""Host-side behaviour of the C-ABI library that needs no GPU: exported symbols, size queries,
argument validation (which happens before any launch), and lazy-layer selection."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2410_13846_amd import lt

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_DEV = 0x10000000          # aligned, never dereferenced: no call below reaches a launch


def cfg(**kw):
    base = dict(n_layers=4, batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, w_sink=4, w_recent=60, max_tokens=1000)
    base.update(kw)
    return lt.make_config(**base)


def test_library_exports_every_declared_symbol():
    lib = lt.load()
    declared = set()
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):
        assert name.endswith(".h"), name
        header = open(os.path.join(ROOT, "include", name)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        found = set(re.findall(r"\b(lt_[a-z_]+)\s*\(", header))
        assert found, "no declarations found in " + name
        declared |= found
    assert declared == set(lt.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_kv_and_workspace_sizes():
    c = cfg()
    per_token = 2 * 2 * 128 * 2            # B * Hkv * d * sizeof(bf16)
    full, lazy = per_token * 1000, per_token * 64
    assert lt.kv_bytes(c, [0, 0, 0, 0]) == 4 * 2 * full
    assert lt.kv_bytes(c, [1, 0, 1, 0]) == 2 * 2 * full + 2 * 2 * lazy
    assert lt.kv_bytes(c, [1, 1, 1, 1]) == 4 * 2 * lazy
    assert lt.workspace_bytes(c) > 0
    # the 128K, batch 16 configuration: 16 full layers of 8.59 GB + 16 rings, 64-bit sizes
    big = lt.make_config(32, 16, 32, 8, 128, 4, 4092, 131072 + 32)
    mask = [1] * 16 + [0] * 16
    expect = 16 * 2 * (16 * 8 * (131072 + 32) * 128 * 2) + 16 * 2 * (16 * 8 * 4096 * 128 * 2)
    assert lt.kv_bytes(big, mask) == expect
    assert expect > 2 ** 37


@pytest.mark.parametrize("bad", [dict(head_dim=64), dict(n_q_heads=7), dict(n_q_heads=32, n_kv_heads=2), dict(batch=0),
                                 dict(max_tokens=0), dict(w_sink=-1), dict(max_tokens=2 ** 31)])
def test_invalid_configurations_are_rejected(bad):
    c = cfg(**bad)
    assert lt.kv_bytes(c, [0, 0, 0, 0]) == 0
    assert lt.workspace_bytes(c) == 0
    handle = ctypes.c_void_p()
    st = lt.load().lt_create(ctypes.byref(c), np.zeros(4, np.uint8).ctypes.data, FAKE_DEV, 1 << 40, FAKE_DEV, 1 << 40,
                             ctypes.byref(handle))
    assert st in (lt.ERR_INVALID_ARG, lt.ERR_SHAPE) and not handle.value


def make_ctx(c, mask):
    handle = ctypes.c_void_p()
    m = np.asarray(mask, np.uint8)
    st = lt.load().lt_create(ctypes.byref(c), m.ctypes.data, FAKE_DEV, lt.kv_bytes(c, mask), FAKE_DEV + (1 << 34),
                             lt.workspace_bytes(c), ctypes.byref(handle))
    assert st == lt.OK
    return handle


def test_create_validates_buffers_and_lays_out_layers():
    lib, c, mask = lt.load(), cfg(), [0, 1, 0, 1]
    m = np.asarray(mask, np.uint8)
    handle = ctypes.c_void_p()
    kvb, wsb = lt.kv_bytes(c, mask), lt.workspace_bytes(c)
    assert lib.lt_create(ctypes.byref(c), m.ctypes.data, FAKE_DEV, kvb - 1, FAKE_DEV, wsb, ctypes.byref(handle)) == lt.ERR_CAPACITY
    assert lib.lt_create(ctypes.byref(c), m.ctypes.data, FAKE_DEV, kvb, FAKE_DEV, wsb - 1, ctypes.byref(handle)) == lt.ERR_CAPACITY
    assert lib.lt_create(ctypes.byref(c), m.ctypes.data, FAKE_DEV + 8, kvb, FAKE_DEV, wsb, ctypes.byref(handle)) == lt.ERR_INVALID_ARG
    assert lib.lt_create(ctypes.byref(c), m.ctypes.data, None, kvb, FAKE_DEV, wsb, ctypes.byref(handle)) == lt.ERR_INVALID_ARG
    h = make_ctx(c, mask)
    # blocks are laid out back to back in layer order: K then V, full = 1000 tokens, lazy = 64
    cursor = FAKE_DEV
    for layer in range(4):
        k, v = ctypes.c_void_p(), ctypes.c_void_p()
        sb, sh, cap, lazy = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int32()
        assert lib.lt_layer_view(h, layer, ctypes.byref(k), ctypes.byref(v), ctypes.byref(sb), ctypes.byref(sh),
                                 ctypes.byref(cap), ctypes.byref(lazy)) == lt.OK
        tokens = 64 if mask[layer] else 1000
        block = 2 * 2 * tokens * 128 * 2
        assert (k.value, v.value) == (cursor, cursor + block)
        assert (cap.value, lazy.value, sh.value, sb.value) == (tokens, mask[layer], tokens * 128, tokens * 128 * 2)
        cursor += 2 * block
    assert lib.lt_layer_view(h, 4, None, None, None, None, None, None) == lt.ERR_INVALID_ARG
    lib.lt_destroy(h)
    lib.lt_destroy(None)


def test_calls_out_of_order_or_over_capacity_fail_before_any_launch():
    lib, c = lt.load(), cfg()
    h = make_ctx(c, [0, 1, 0, 1])
    # decode on an empty layer
    assert lib.lt_decode_attn(h, 0, FAKE_DEV, FAKE_DEV, None, None) == lt.ERR_STATE
    assert lib.lt_decode_attn(h, 9, FAKE_DEV, FAKE_DEV, None, None) == lt.ERR_INVALID_ARG
    assert lib.lt_decode_attn(h, 0, None, FAKE_DEV, None, None) == lt.ERR_INVALID_ARG
    # a full layer cannot take more than max_tokens; the failed call leaves the count unchanged
    assert lib.lt_append_kv(h, 0, FAKE_DEV, FAKE_DEV, 1001, None) == lt.ERR_CAPACITY
    assert lib.lt_append_kv(h, 0, FAKE_DEV, FAKE_DEV, 0, None) == lt.ERR_INVALID_ARG
    assert lib.lt_append_kv(h, 0, FAKE_DEV + 2, FAKE_DEV, 1, None) == lt.ERR_INVALID_ARG
    total, stored = ctypes.c_int64(-1), ctypes.c_int64(-1)
    assert lib.lt_layer_len(h, 0, ctypes.byref(total), ctypes.byref(stored)) == lt.OK
    assert (total.value, stored.value) == (0, 0)
    # split sizes: multiples of 64, and never more splits than the workspace holds
    assert lib.lt_set_split(h, 100, 0) == lt.ERR_INVALID_ARG
    assert lib.lt_set_split(h, 64, 0) == lt.ERR_CAPACITY
    assert lib.lt_set_split(h, 512, 64) == lt.OK
    assert lib.lt_profile_read(h, 7, ctypes.byref(total), ctypes.byref(ctypes.c_double())) == lt.ERR_INVALID_ARG
    lib.lt_destroy(h)


def test_lazy_ratio_argument_validation():
    lib, c = lt.load(), cfg()
    need = lt.lazy_ratio_workspace_bytes(c, 500, 16)
    assert need > 0
    assert lt.lazy_ratio_workspace_bytes(c, 500, 65) == 0
    assert lt.lazy_ratio_workspace_bytes(c, 0, 16) == 0

    def call(n=500, w=16, mode=0, ws=need, sb=500 * 128 * 2, sh=500 * 128, st=128, q=FAKE_DEV, mean=FAKE_DEV):
        return lib.lt_lazy_ratio(ctypes.byref(c), q, FAKE_DEV, sb, sh, st, n, w, mode, FAKE_DEV, ws, None, None, mean, None)

    assert call(w=0) == lt.ERR_INVALID_ARG
    assert call(mode=3) == lt.ERR_INVALID_ARG
    assert call(q=None) == lt.ERR_INVALID_ARG
    assert call(mean=None) == lt.ERR_INVALID_ARG
    assert call(n=8, w=16) == lt.ERR_SHAPE              # more scored queries than prompt tokens
    assert call(w=65) == lt.ERR_SHAPE
    assert call(st=64) == lt.ERR_SHAPE                  # rows would overlap
    assert call(sh=500 * 128 + 4) == lt.ERR_SHAPE       # 16-byte alignment of rows
    assert call(ws=need - 1) == lt.ERR_CAPACITY


def test_wrappers_check_tensor_extents_before_the_library_sees_addresses():
    """The C layer gets addresses and strides only, so the binding must refuse tensors whose extents do not cover what
    the kernels will read (a wrong n, a missing head, a short workspace): ERR_SHAPE / ERR_CAPACITY, never a launch.
    Host tensors are enough to reach those checks; well-shaped host tensors are then refused for not being on a GPU."""
    import torch

    c = cfg()                                                       # B 2, Hq 8, Hkv 2, d 128
    bf = torch.bfloat16
    q_last = torch.zeros((2, 8, 16, 128), dtype=bf)
    k = torch.zeros((2, 2, 500, 128), dtype=bf)

    def status_of(fn, *a, **kw):
        with pytest.raises(lt.LtError) as e:
            fn(*a, **kw)
        return e.value.status

    for fn in (lt.lazy_ratio, lambda *a: lt.lazy_ratio_lse(*a, torch.zeros((2, 8, 16))),
               lambda *a: lt.lazy_ratio_static(*a, torch.zeros(1))):
        assert status_of(fn, c, q_last, k, 501, 16) == lt.ERR_SHAPE                  # n beyond the keys that exist
        assert status_of(fn, c, q_last, k, 0, 16) == lt.ERR_SHAPE
        assert status_of(fn, c, q_last, k, 500, 8) == lt.ERR_SHAPE                   # q_last holds 16 queries, not 8
        assert status_of(fn, c, q_last[:, :4].contiguous(), k, 500, 16) == lt.ERR_SHAPE
        assert status_of(fn, c, q_last, k[:, :1], 500, 16) == lt.ERR_SHAPE           # a KV head missing
        assert status_of(fn, c, q_last, k[:1], 500, 16) == lt.ERR_SHAPE              # a sequence missing
        with pytest.raises(TypeError):
            fn(c, q_last, k, 500, 16)                                                # fine shapes, but host memory
    q = torch.zeros((2, 8, 500, 128), dtype=bf)
    v = torch.zeros_like(k)
    assert status_of(lt.prefill_attn, c, q, k, v, 501) == lt.ERR_SHAPE
    assert status_of(lt.prefill_attn, c, q, k, v, 499) == lt.ERR_SHAPE               # fewer positions than queries
    assert status_of(lt.prefill_attn, c, q[:, :4].contiguous(), k, v, 500) == lt.ERR_SHAPE
    assert status_of(lt.prefill_attn, c, q, k[:, :1], v[:, :1], 500) == lt.ERR_SHAPE
    with pytest.raises(TypeError):
        lt.prefill_attn(c, q, k, v, 500)
    if torch.cuda.is_available():                                   # workspace extent and device
        dev = "cuda:0"
        short = torch.empty(lt.lazy_ratio_workspace_bytes(c, 500, 16) - 1, dtype=torch.uint8, device=dev)
        assert status_of(lt.lazy_ratio, c, q_last.to(dev), k.to(dev), 500, 16, workspace=short) == lt.ERR_CAPACITY


def test_lazy_ratio_static_argument_validation():
    """The variant that keeps its partial results in the library's own scratch array: same checks as lt_lazy_ratio,
    and a problem whose partial results exceed the array is refused with ERR_CAPACITY before anything is enqueued."""
    lib, c = lt.load(), cfg()

    def call(conf=c, n=500, w=16, mode=0, q=FAKE_DEV, mean=FAKE_DEV, st=128):
        return lib.lt_lazy_ratio_static(ctypes.byref(conf), q, FAKE_DEV, n * 128 * 2, n * 128, st, n, w, mode, None, None, mean, None)

    assert call(w=0) == lt.ERR_INVALID_ARG
    assert call(mode=3) == lt.ERR_INVALID_ARG
    assert call(q=None) == lt.ERR_INVALID_ARG
    assert call(mean=None) == lt.ERR_INVALID_ARG
    assert call(n=8, w=16) == lt.ERR_SHAPE
    assert call(st=64) == lt.ERR_SHAPE
    big = lt.make_config(1, 512, 64, 8, 128, 4, 2044, 1 << 20)      # 512 sequences x 64 heads x 64 queries: 25 MB of partial sums
    assert lt.lazy_ratio_workspace_bytes(big, 1 << 20, 64) > 8 << 20
    assert call(conf=big, n=1 << 20, w=64) == lt.ERR_CAPACITY
    # the benchmark shapes fit
    for B, n in ((8, 32768), (32, 16384), (1, 131072), (16, 131072)):
        shape = lt.make_config(32, B, 32, 8, 128, 4, 2044, n)
        assert 0 < lt.lazy_ratio_workspace_bytes(shape, n, 64) <= 8 << 20, (B, n)


def test_prefill_and_ratio_from_lse_argument_validation():
    """Error paths of lt_prefill_attn / lt_lazy_ratio_lse that return before anything is enqueued."""
    lib, c = lt.load(), cfg()

    def prefill(q=FAKE_DEV, k=FAKE_DEV, v=FAKE_DEV, out=FAKE_DEV, n=500, nq=None, mask=0, dtype=0, sb=500 * 128 * 2, sh=500 * 128, st=128,
                conf=c):
        return lib.lt_prefill_attn(ctypes.byref(conf), q, k, v, sb, sh, st, n, n if nq is None else nq, mask, dtype, out, None, None)

    assert prefill(q=None) == lt.ERR_INVALID_ARG
    assert prefill(out=None) == lt.ERR_INVALID_ARG
    assert prefill(n=0) == lt.ERR_INVALID_ARG
    assert prefill(nq=0) == lt.ERR_INVALID_ARG
    assert prefill(nq=501) == lt.ERR_SHAPE                   # more queries than positions
    assert prefill(mask=2) == lt.ERR_INVALID_ARG
    assert prefill(dtype=5) == lt.ERR_INVALID_ARG
    assert prefill(k=FAKE_DEV + 2) == lt.ERR_INVALID_ARG
    assert prefill(st=64) == lt.ERR_SHAPE
    assert prefill(st=1 << 24) == lt.ERR_SHAPE
    assert prefill(sh=500 * 128 + 4) == lt.ERR_SHAPE
    empty = lt.make_config(4, 2, 4, 2, 128, 0, 0, 1000)
    assert prefill(mask=1, conf=empty) == lt.ERR_SHAPE          # streaming attention with an empty window

    need = lt.lazy_ratio_lse_workspace_bytes(c, 500, 16)
    assert need > 0
    assert lt.lazy_ratio_lse_workspace_bytes(c, 500, 65) == 0
    assert lt.lazy_ratio_lse_workspace_bytes(c, 8, 16) == 0

    def ratio(n=500, w=16, mode=0, ws=need, lse=FAKE_DEV, lsb=4 * 500, lsh=500):
        return lib.lt_lazy_ratio_lse(ctypes.byref(c), FAKE_DEV, FAKE_DEV, 500 * 128 * 2, 500 * 128, 128, n, w, mode, lse, lsb, lsh,
                                     FAKE_DEV, ws, None, None, FAKE_DEV, None)

    assert ratio(lse=None) == lt.ERR_INVALID_ARG
    assert ratio(lse=FAKE_DEV + 2) == lt.ERR_INVALID_ARG
    assert ratio(lsb=-1) == lt.ERR_INVALID_ARG
    assert ratio(mode=2) == lt.ERR_INVALID_ARG
    assert ratio(n=8, w=16) == lt.ERR_SHAPE
    assert ratio(ws=need - 1) == lt.ERR_CAPACITY
    # the window-only form reads the same number of keys whatever the prompt length, so its workspace does not grow with n
    long_cfg = lt.make_config(1, 8, 32, 8, 128, 4, 2044, 1 << 20)
    assert lt.lazy_ratio_lse_workspace_bytes(long_cfg, 32768, 64) == lt.lazy_ratio_lse_workspace_bytes(long_cfg, 1 << 20, 64)


def test_ragged_and_output_dtype_argument_validation():
    lib, c = lt.load(), cfg()
    h = make_ctx(c, [0, 1, 0, 1])
    counts = (ctypes.c_int64 * 2)(5, 3)
    assert lib.lt_append_kv_ragged(h, 0, FAKE_DEV, FAKE_DEV, 5, None, None) == lt.ERR_INVALID_ARG
    bad = (ctypes.c_int64 * 2)(6, 3)
    assert lib.lt_append_kv_ragged(h, 0, FAKE_DEV, FAKE_DEV, 5, bad, None) == lt.ERR_INVALID_ARG
    over = (ctypes.c_int64 * 2)(1001, 3)
    assert lib.lt_append_kv_ragged(h, 0, FAKE_DEV, FAKE_DEV, 1001, over, None) == lt.ERR_CAPACITY
    total, stored = ctypes.c_int64(-1), ctypes.c_int64(-1)
    assert lib.lt_seq_len(h, 0, 1, ctypes.byref(total), ctypes.byref(stored)) == lt.OK
    assert (total.value, stored.value) == (0, 0)
    assert lib.lt_seq_len(h, 0, 2, ctypes.byref(total), ctypes.byref(stored)) == lt.ERR_INVALID_ARG
    assert lib.lt_set_output_dtype(h, 7) == lt.ERR_INVALID_ARG
    assert lib.lt_set_output_dtype(h, lt.OUT_BF16) == lt.OK
    assert lib.lt_set_output_dtype(None, lt.OUT_BF16) == lt.ERR_INVALID_ARG
    lib.lt_destroy(h)
    wide = lt.make_config(1, 129, 4, 2, 128, 4, 60, 100)             # ragged lengths travel as launch arguments: at most 128 sequences
    hw = make_ctx(wide, [0])
    many = (ctypes.c_int64 * 129)(*([1] * 129))
    assert lib.lt_append_kv_ragged(hw, 0, FAKE_DEV, FAKE_DEV, 1, many, None) == lt.ERR_SHAPE
    lib.lt_destroy(hw)
    del counts


def test_select_lazy_matches_the_oracle_and_the_queue():
    rng = np.random.default_rng(7)
    for L in (1, 2, 32, 64):
        for trial in range(10):
            r = rng.random(L).astype(np.float32)
            if trial % 2:
                r = (np.round(r * 4) / 4).astype(np.float32)        # ties
            for n_lazy in {0, L // 4, L // 2, L}:
                got, order = lt.select_lazy(r, n_lazy)
                ref, ref_order = oracle.select_lazy(r.astype(np.float64), n_lazy)
                queue, _ = oracle.select_lazy_queue(r.astype(np.float64), n_lazy)
                np.testing.assert_array_equal(got, ref)
                np.testing.assert_array_equal(got, queue)
                np.testing.assert_array_equal(order, ref_order)


def test_select_lazy_rejects_bad_input():
    with pytest.raises(lt.LtError) as e:
        lt.select_lazy(np.array([0.5, np.nan], np.float32), 1)
    assert e.value.status == lt.ERR_INVALID_ARG
    with pytest.raises(lt.LtError):
        lt.select_lazy(np.array([0.5, 0.1], np.float32), 3)
    assert lt.status_str(lt.ERR_CAPACITY) == "capacity exceeded"


def test_preselect_lazy_matches_the_oracle():
    """Pre-selection over many samples (host code): frequencies and the most frequent layers, ties to the lower index."""
    rng = np.random.default_rng(13)
    for S, L in ((1, 4), (9, 32), (300, 64)):
        for n_lazy in {0, 1, L // 2, L}:
            sets = (rng.random((S, L)) < rng.random(L)).astype(np.uint8)
            if S > 1:
                sets[:, 1] = sets[:, 0]                                  # two layers with equal frequency
            got, count = lt.preselect_lazy(sets, n_lazy)
            ref, ref_count = oracle.preselect_lazy(sets, n_lazy)
            np.testing.assert_array_equal(got, ref)
            np.testing.assert_array_equal(count, ref_count)
    with pytest.raises(lt.LtError):
        lt.preselect_lazy(np.zeros((2, 4), np.uint8), 5)


# ---- online identification (priority queue + slot pools), host side only -----------------------

def test_select_push_reproduces_the_queue_procedure():
    rng = np.random.default_rng(11)
    for L in (1, 2, 7, 32, 64):
        for trial in range(10):
            r = rng.random(L).astype(np.float32)
            if trial % 2:
                r = (np.round(r * 4) / 4).astype(np.float32)        # ties
            for n_lazy in sorted({0, 1, L // 2, L - 1, L}):
                q = lt.SelectQueue(L - n_lazy)
                popped_at = np.full(L, -1, dtype=np.int32)
                for layer in range(L):
                    out = q.push(r[layer], layer)
                    if out >= 0:
                        assert popped_at[out] < 0
                        popped_at[out] = layer
                q.close()
                ref_lazy, ref_pop = oracle.select_lazy_queue(r.astype(np.float64), n_lazy)
                np.testing.assert_array_equal(popped_at, ref_pop)
                np.testing.assert_array_equal((popped_at >= 0).astype(np.uint8), ref_lazy)
                closed_form, _ = lt.select_lazy(r, n_lazy)
                np.testing.assert_array_equal(closed_form, ref_lazy)


def test_select_push_rejects_bad_input():
    q = lt.SelectQueue(2)
    with pytest.raises(lt.LtError) as e:
        q.push(float("nan"), 0)
    assert e.value.status == lt.ERR_INVALID_ARG
    with pytest.raises(lt.LtError):
        q.push(0.5, -1)
    q.close()
    with pytest.raises(lt.LtError):
        lt.SelectQueue(-1)


def test_online_context_sizes_and_slot_accounting():
    lib, c = lt.load(), cfg()                     # 4 layers, full = 1000 tokens, ring = 64 tokens
    per_token = 2 * 2 * 128 * 2
    full, ring = 2 * per_token * 1000, 2 * per_token * 64
    assert lt.kv_bytes_online(c, 2) == 3 * full + 2 * ring        # P + 1 full slots, L - P rings
    assert lt.kv_bytes_online(c, 4) == 4 * full                   # nothing turns lazy
    assert lt.kv_bytes_online(c, 0) == 1 * full + 4 * ring
    assert lt.kv_bytes_online(c, 5) == 0
    handle = ctypes.c_void_p()
    need = lt.kv_bytes_online(c, 2)
    assert lib.lt_create_online(ctypes.byref(c), 2, FAKE_DEV, need - 1, FAKE_DEV + (1 << 34), lt.workspace_bytes(c),
                                ctypes.byref(handle)) == lt.ERR_CAPACITY
    assert lib.lt_create_online(ctypes.byref(c), 2, FAKE_DEV, need, FAKE_DEV + (1 << 34), lt.workspace_bytes(c),
                                ctypes.byref(handle)) == lt.OK
    # no layer has storage yet; decode is out of order, truncating an empty full layer only flips its kind
    k, v = ctypes.c_void_p(1), ctypes.c_void_p(1)
    cap, lazy = ctypes.c_int64(), ctypes.c_int32()
    assert lib.lt_layer_view(handle, 0, ctypes.byref(k), ctypes.byref(v), None, None, ctypes.byref(cap), ctypes.byref(lazy)) == lt.OK
    assert (k.value, v.value, cap.value, lazy.value) == (None, None, 1000, 0)
    assert lib.lt_decode_attn(handle, 0, FAKE_DEV, FAKE_DEV, None, None) == lt.ERR_STATE
    assert lib.lt_truncate_layer(handle, 0, None) == lt.OK
    assert lib.lt_layer_view(handle, 0, ctypes.byref(k), None, None, None, ctypes.byref(cap), ctypes.byref(lazy)) == lt.OK
    assert (k.value, cap.value, lazy.value) == (FAKE_DEV + 3 * full, 64, 1)
    assert lib.lt_truncate_layer(handle, 0, None) == lt.ERR_STATE          # already lazy
    assert lib.lt_truncate_layer(handle, 1, None) == lt.OK
    assert lib.lt_truncate_layer(handle, 2, None) == lt.ERR_CAPACITY       # only L - P = 2 rings
    assert lib.lt_reset(handle) == lt.OK
    assert lib.lt_layer_view(handle, 0, ctypes.byref(k), None, None, None, ctypes.byref(cap), ctypes.byref(lazy)) == lt.OK
    assert (k.value, cap.value, lazy.value) == (None, 1000, 0)
    lib.lt_destroy(handle)
    # a context with a fixed mask cannot be truncated
    h = make_ctx(c, [0, 1, 0, 1])
    assert lib.lt_truncate_layer(h, 0, None) == lt.ERR_STATE
    lib.lt_destroy(h)


def test_paged_context_sizes_and_argument_validation():
    """Everything checked here happens on the host before any launch or copy."""
    lib, c, mask = lt.load(), cfg(), [0, 1, 0, 1]
    m = np.asarray(mask, np.uint8)
    page, n_pages = 64, 40
    max_pages = -(-1000 // page)
    pool = n_pages * 2 * page * 128 * 2                              # bf16 [n_pages][Hkv][page][128]
    ring = 2 * 2 * 64 * 128 * 2                                      # bf16 [B][Hkv][w_sink + w_recent][128]
    table = -(-(2 * max_pages * 4) // 256) * 256
    assert lt.kv_bytes_paged(c, mask, page, n_pages) == table + 2 * 2 * pool + 2 * 2 * ring
    for bad_page in (0, 32, 96, 1 << 21):
        assert lt.kv_bytes_paged(c, mask, bad_page, n_pages) == 0
    assert lt.kv_bytes_paged(c, mask, page, 0) == 0
    assert lt.kv_bytes_paged(cfg(batch=129), mask, page, n_pages) == 0

    def create(conf, pg, npg, kvb=None):
        handle = ctypes.c_void_p()
        kvb = lt.kv_bytes_paged(conf, mask, pg, npg) if kvb is None else kvb
        st = lib.lt_create_paged(ctypes.byref(conf), m.ctypes.data, pg, npg, FAKE_DEV, kvb, FAKE_DEV + (1 << 34),
                                 lt.workspace_bytes(conf), ctypes.byref(handle))
        return st, handle

    assert create(c, 96, n_pages, 1 << 30)[0] == lt.ERR_SHAPE
    assert create(c, -1, n_pages, 1 << 30)[0] == lt.ERR_INVALID_ARG
    assert create(c, page, n_pages, lt.kv_bytes_paged(c, mask, page, n_pages) - 1)[0] == lt.ERR_CAPACITY
    # 512 ranges of at most 255 pages of 64 tokens: longer contexts need larger pages
    long_c = cfg(max_tokens=512 * 255 * 64 + 1)
    assert create(long_c, 64, n_pages, 1 << 40)[0] == lt.ERR_SHAPE
    assert create(long_c, 128, n_pages)[0] == lt.OK
    st, h = create(c, page, n_pages)
    assert st == lt.OK
    k, v = ctypes.c_void_p(), ctypes.c_void_p()
    sb, sh, cap, lazy = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int32()
    assert lib.lt_layer_view(h, 0, ctypes.byref(k), ctypes.byref(v), ctypes.byref(sb), ctypes.byref(sh), ctypes.byref(cap),
                             ctypes.byref(lazy)) == lt.OK
    assert (sb.value, sh.value, cap.value, lazy.value) == (2 * page * 128, page * 128, max_pages * page, 0)
    assert (k.value, v.value) == (FAKE_DEV + table, FAKE_DEV + table + pool)   # the pools follow the table
    # no page, no append; entries outside the pool are refused; both before anything is enqueued
    assert lib.lt_append_kv(h, 0, FAKE_DEV, FAKE_DEV, 5, None) == lt.ERR_STATE
    assert lib.lt_append_kv(h, 1, FAKE_DEV, FAKE_DEV, 2000, None) != lt.ERR_STATE    # a lazy layer needs no pages
    bad = np.full((2, max_pages), -1, np.int32)
    bad[1, 3] = n_pages
    assert lib.lt_set_block_table(h, bad.ctypes.data, None) == lt.ERR_INVALID_ARG
    bad[1, 3] = -2
    assert lib.lt_set_block_table(h, bad.ctypes.data, None) == lt.ERR_INVALID_ARG
    assert lib.lt_set_block_table(h, None, None) == lt.ERR_INVALID_ARG
    assert lib.lt_truncate_layer(h, 0, None) == lt.ERR_STATE
    assert lib.lt_reset_sequence(h, 2) == lt.ERR_INVALID_ARG
    assert lib.lt_reset_sequence(h, 1) == lt.OK
    lib.lt_destroy(h)
    plain = make_ctx(c, mask)
    ok = np.zeros((2, max_pages), np.int32)
    assert lib.lt_set_block_table(plain, ok.ctypes.data, None) == lt.ERR_STATE
    assert lib.lt_reset_sequence(plain, 0) == lt.OK                  # also works on a contiguous context
    lib.lt_destroy(plain)
    online = ctypes.c_void_p()
    assert lib.lt_create_online(ctypes.byref(c), 2, FAKE_DEV, lt.kv_bytes_online(c, 2), FAKE_DEV + (1 << 34),
                                lt.workspace_bytes(c), ctypes.byref(online)) == lt.OK
    assert lib.lt_reset_sequence(online, 0) == lt.ERR_STATE
    lib.lt_destroy(online)


def test_product_path_has_no_oracle_and_no_fallback(tmp_path, monkeypatch):
    """The package never touches oracle/ (nor does the input generator or the oracle the package), and a missing
    library with no compiler is an error, not a silent CPU path."""
    import subprocess
    import sys

    uses_oracle = re.compile(r"^\s*(import|from)\s+oracle\b|lt_oracle|liblto", re.M)
    pkg = os.path.join(ROOT, "paper_2410_13846_amd")
    for folder, _, files in os.walk(pkg):
        for name in files:
            if name.endswith((".py", ".cpp", ".hip", ".h")):
                assert not uses_oracle.search(open(os.path.join(folder, name)).read()), name
    assert not uses_oracle.search(open(os.path.join(ROOT, "lt_workloads.py")).read())
    for name in os.listdir(os.path.join(ROOT, "oracle")):
        if name.endswith((".py", ".c", ".h")):
            assert "paper_2410_13846_amd" not in open(os.path.join(ROOT, "oracle", name)).read(), name
    probe = ("import sys; sys.path.insert(0, %r)\n"
             "import paper_2410_13846_amd.build as b\n"
             "b.LIB_PATH = %r\n"
             "from paper_2410_13846_amd import lt\n"
             "try:\n    lt.load()\nexcept Exception as e:\n    print('raised', type(e).__name__)\nelse:\n    print('loaded')\n"
             ) % (ROOT, str(tmp_path / "absent" / "liblt_hip.so"))
    env = dict(os.environ, HIPCC=str(tmp_path / "no_such_hipcc"))
    out = subprocess.run([sys.executable, "-c", probe], env=env, capture_output=True, text=True, timeout=120)
    assert out.stdout.strip().startswith("raised"), out.stdout + out.stderr


def test_decode_step_active_argument_validation():
    lib, c = lt.load(), cfg()
    h = make_ctx(c, [0, 1, 0, 1])
    flags = (ctypes.c_uint8 * 2)(1, 0)
    assert lib.lt_decode_step_active(h, 0, FAKE_DEV, FAKE_DEV, FAKE_DEV, None, FAKE_DEV, None, None) == lt.ERR_INVALID_ARG
    assert lib.lt_decode_step_active(h, 0, FAKE_DEV, None, FAKE_DEV, flags, FAKE_DEV, None, None) == lt.ERR_INVALID_ARG
    assert lib.lt_decode_step_active(h, 9, FAKE_DEV, FAKE_DEV, FAKE_DEV, flags, FAKE_DEV, None, None) == lt.ERR_INVALID_ARG
    none = (ctypes.c_uint8 * 2)(0, 0)
    assert lib.lt_decode_step_active(h, 0, FAKE_DEV, FAKE_DEV, FAKE_DEV, none, FAKE_DEV, None, None) == lt.ERR_STATE   # nobody generates
    total = ctypes.c_int64(-1)
    assert lib.lt_seq_len(h, 0, 0, ctypes.byref(total), None) == lt.OK and total.value == 0        # and nothing was counted
    lib.lt_destroy(h)
    online = ctypes.c_void_p()
    assert lib.lt_create_online(ctypes.byref(c), 2, FAKE_DEV, lt.kv_bytes_online(c, 2), FAKE_DEV + (1 << 34),
                                lt.workspace_bytes(c), ctypes.byref(online)) == lt.OK
    assert lib.lt_decode_step_active(online, 0, FAKE_DEV, FAKE_DEV, FAKE_DEV, flags, FAKE_DEV, None, None) == lt.ERR_STATE
    lib.lt_destroy(online)
    wide = lt.make_config(1, 129, 4, 2, 128, 4, 60, 100)
    hw = make_ctx(wide, [0])
    many = (ctypes.c_uint8 * 129)(*([1] * 129))
    assert lib.lt_decode_step_active(hw, 0, FAKE_DEV, FAKE_DEV, FAKE_DEV, many, FAKE_DEV, None, None) == lt.ERR_SHAPE
    lib.lt_destroy(hw)
