"""The host layer of the library (csrc/lt_api.cpp) end to end on the CPU: bookkeeping of token counts, ring slots,
split choice, per-sequence lengths, paged tables, online slots, event timing.

These tests need the CPU build of the host layer against stub launchers (tests/stubs/lt_stub_launchers.cpp), which
records every launch instead of running it.  tests/test_sanitizers.py makes that build with the address and
undefined-behaviour sanitizers and runs this file (and the other host and oracle tests) against it in a child
process; in a process that has loaded the real GPU library the tests here are skipped."""
import ctypes

import numpy as np
import pytest

from paper_2410_13846_amd import lt

FAKE = 0x10000000                        # aligned "device" addresses: the stub launchers never touch them
FAKE2 = 0x7F0000000000


def stub_lib():
    lib = lt.load()
    if not hasattr(lib, "lt_stub_counts"):
        pytest.skip("needs the CPU build of the host layer with stub launchers (run by tests/test_sanitizers.py)")
    lib.lt_stub_reset()
    return lib


def counts(lib):
    out = (ctypes.c_int32 * 8)()
    lib.lt_stub_counts(out)
    return dict(zip(("append", "truncate", "decode", "zero_tickets", "probe", "score", "prefill", "memcpy"), out))


NO_TAIL = 2 ** 31 - 1                                          # DecodeArgs::tail_begin of a launch without a shared tail


def last_decode(lib):
    out = (ctypes.c_int64 * 13)()
    lib.lt_stub_last_decode(out)
    return dict(zip(("stored", "keys_per_block", "n_splits", "new_slot", "spread_tiles", "fused", "lazy_tag", "out_bf16", "stride_b",
                     "stride_h", "mode", "v_minus_k", "tail_begin"), out))


def last_lengths(lib, n):
    a, b = (ctypes.c_int32 * n)(), (ctypes.c_int32 * n)()
    lib.lt_stub_last_lengths(a, b, n)
    return list(a), list(b)


def last_append(lib):
    out = (ctypes.c_int64 * 8)()
    lib.lt_stub_last_append(out)
    return dict(zip(("n_new", "total_before", "is_lazy", "ragged", "stride_b", "stride_h", "paged", "page_shift"), out))


def last_score(lib):
    out = (ctypes.c_int64 * 8)()
    lib.lt_stub_last_score(out)
    return dict(zip(("keys_per_block", "n_chunks", "n_chunks_a", "range_a_end", "range_b_begin", "fixed_mode", "has_lse", "scratch_offset"), out))


class Ctx:
    def __init__(self, lib, cfg, is_lazy=None, online=None, paged=None):
        self.lib, self.cfg = lib, cfg
        h = ctypes.c_void_p()
        ws = lt.workspace_bytes(cfg)
        if online is not None:
            st = lib.lt_create_online(ctypes.byref(cfg), online, FAKE2, lt.kv_bytes_online(cfg, online), FAKE, ws, ctypes.byref(h))
        elif paged is not None:
            m = np.asarray(is_lazy, np.uint8)
            st = lib.lt_create_paged(ctypes.byref(cfg), m.ctypes.data, paged[0], paged[1], FAKE2, lt.kv_bytes_paged(cfg, m, *paged), FAKE, ws,
                                     ctypes.byref(h))
        else:
            m = np.asarray(is_lazy, np.uint8)
            st = lib.lt_create(ctypes.byref(cfg), m.ctypes.data, FAKE2, lt.kv_bytes(cfg, m), FAKE, ws, ctypes.byref(h))
        assert st == lt.OK, st
        self.h = h

    def append(self, layer, n):
        return self.lib.lt_append_kv(self.h, layer, FAKE, FAKE, n, None)

    def append_ragged(self, layer, n_max, per_seq):
        a = np.asarray(per_seq, np.int64)
        return self.lib.lt_append_kv_ragged(self.h, layer, FAKE, FAKE, n_max, a.ctypes.data, None)

    def step(self, layer):
        return self.lib.lt_decode_step(self.h, layer, FAKE, FAKE, FAKE, FAKE, None, None)

    def attn(self, layer):
        return self.lib.lt_decode_attn(self.h, layer, FAKE, FAKE, None, None)

    def step_active(self, layer, active):
        a = np.asarray(active, np.uint8)
        return self.lib.lt_decode_step_active(self.h, layer, FAKE, FAKE, FAKE, a.ctypes.data, FAKE, None, None)

    def len(self, layer):
        t, s = ctypes.c_int64(), ctypes.c_int64()
        assert self.lib.lt_layer_len(self.h, layer, ctypes.byref(t), ctypes.byref(s)) == lt.OK
        return t.value, s.value

    def seq_len(self, layer, b):
        t, s = ctypes.c_int64(), ctypes.c_int64()
        assert self.lib.lt_seq_len(self.h, layer, b, ctypes.byref(t), ctypes.byref(s)) == lt.OK
        return t.value, s.value

    def close(self):
        self.lib.lt_destroy(self.h)


def test_token_counts_ring_slots_and_capacity():
    lib = stub_lib()
    cfg = lt.make_config(2, 2, 8, 2, 128, 4, 12, 40)                 # window 16, full capacity 40
    c = Ctx(lib, cfg, [0, 1])
    assert c.attn(0) == lt.ERR_STATE and counts(lib)["decode"] == 0     # nothing to attend over yet
    assert c.append(0, 30) == lt.OK and c.append(1, 30) == lt.OK
    assert last_append(lib)["is_lazy"] == 1 and last_append(lib)["total_before"] == 0
    assert c.len(0) == (30, 30) and c.len(1) == (30, 16)
    for i in range(10):                                              # positions 30..39
        assert c.step(1) == lt.OK
        d = last_decode(lib)
        p = 30 + i
        assert d["new_slot"] == 4 + (p - 4) % 12 and d["stored"] == 16 and d["fused"] == 1 and d["lazy_tag"] == 1
        assert c.step(0) == lt.OK
        d = last_decode(lib)
        assert d["new_slot"] == p and d["stored"] == p + 1 and d["lazy_tag"] == 0
    assert c.len(0) == (40, 40) and c.len(1) == (40, 16)
    before = counts(lib)
    assert c.step(0) == lt.ERR_CAPACITY and c.append(0, 1) == lt.ERR_CAPACITY     # the full layer is full
    assert c.len(0) == (40, 40) and counts(lib)["decode"] == before["decode"] and counts(lib)["append"] == before["append"]
    assert c.step(1) == lt.OK and c.len(1) == (41, 16)                # a lazy layer never fills up
    assert counts(lib)["zero_tickets"] == 1                           # the split counters are zeroed once ...
    assert lib.lt_reset(c.h) == lt.OK and c.len(0) == (0, 0)
    assert c.append(0, 5) == lt.OK and c.attn(0) == lt.OK
    assert counts(lib)["zero_tickets"] == 2                           # ... and again after a reset
    assert last_decode(lib)["fused"] == 0 and last_decode(lib)["stored"] == 5
    c.close()


def test_window_without_recent_tokens_drops_the_new_token():
    lib = stub_lib()
    cfg = lt.make_config(1, 1, 4, 4, 128, 3, 0, 100)                  # a lazy layer that keeps only three initial tokens
    c = Ctx(lib, cfg, [1])
    assert c.append(0, 2) == lt.OK
    assert c.step(0) == lt.OK and last_decode(lib)["new_slot"] == 2 and last_decode(lib)["fused"] == 1
    assert c.step(0) == lt.OK and last_decode(lib)["fused"] == 0 and last_decode(lib)["stored"] == 3   # position 3 is not stored
    assert c.len(0) == (4, 3)
    c.close()


@pytest.mark.parametrize("B,Hkv,G,n,ws,wr", [(8, 8, 4, 32768, 4, 2044), (32, 8, 4, 16384, 4, 2044), (4, 8, 5, 20000, 4, 2044),
                                              (1, 8, 4, 131072, 4, 4092), (16, 8, 4, 131072, 4, 4092), (1, 1, 1, 1000, 4, 60),
                                              (3, 2, 8, 77, 0, 5)])
def test_split_choice_covers_the_keys_and_fills_the_device(B, Hkv, G, n, ws, wr):
    """Key ranges tile the stored entries, are multiples of 64 keys, fit the workspace, and give about one workgroup
    per compute unit at the benchmark shapes."""
    lib = stub_lib()
    cfg = lt.make_config(2, B, Hkv * G, Hkv, 128, ws, wr, n + 8)
    c = Ctx(lib, cfg, [0, 1])
    assert c.append(0, n) == lt.OK and c.append(1, n) == lt.OK
    for layer, stored in ((0, n + 1), (1, min(n + 1, ws + wr))):
        assert c.step(layer) == lt.OK
        d = last_decode(lib)
        assert d["stored"] == stored and d["keys_per_block"] % 64 == 0
        # the ranges tile the stored entries, or, when the ranges are long, all but a shared tail of about an eighth
        ranged = stored
        if d["tail_begin"] != NO_TAIL:
            ranged = d["tail_begin"]
            assert d["keys_per_block"] >= 3072 and d["n_splits"] > 1 and ranged % 64 == 0
            part = 8 if d["keys_per_block"] >= 7 * 8192 // 8 else 4          # a quarter for shorter ranges of many workgroups
            assert stored // part <= stored - ranged < stored // part + 64
            assert part == 8 or d["n_splits"] >= 16
        else:
            assert d["keys_per_block"] < 8192 + 64 or d["n_splits"] == 1
        assert (d["n_splits"] - 1) * d["keys_per_block"] < ranged <= d["n_splits"] * d["keys_per_block"]
        assert 1 <= d["n_splits"] <= 512
        groups = d["n_splits"] * B * Hkv
        if stored >= 256 * 256:
            assert 200 <= groups <= 512, groups
        if d["spread_tiles"]:
            assert d["spread_tiles"] & (d["spread_tiles"] - 1) == 0 and d["spread_tiles"] * 16 <= d["keys_per_block"]
        assert d["stride_h"] == (n + 8 if layer == 0 else ws + wr) * 128 and d["stride_b"] == d["stride_h"] * Hkv
    # forcing a split: accepted when the workspace holds it, refused otherwise
    # the workspace is sized for ranges of 256 keys in full layers (at most 512 ranges): such a split can be forced,
    # a finer one cannot
    keys = 256 * ((n + 8 + 256 * 512 - 1) // (256 * 512))
    assert lib.lt_set_split(c.h, keys, 64) == lt.OK
    assert c.step(0) == lt.OK and last_decode(lib)["keys_per_block"] == keys and last_decode(lib)["n_splits"] == -(-(n + 2) // keys)
    assert last_decode(lib)["tail_begin"] == NO_TAIL                  # a forced split leaves no shared tail
    assert c.step(1) == lt.OK and last_decode(lib)["keys_per_block"] == 64
    assert lib.lt_set_split(c.h, 64, 0) == lt.ERR_CAPACITY
    assert lib.lt_set_split(c.h, 100, 0) == lt.ERR_INVALID_ARG
    assert c.step(0) == lt.OK and last_decode(lib)["keys_per_block"] == keys       # a refused setting changes nothing
    c.close()


def test_per_sequence_lengths_reach_the_kernel_and_inactive_sequences_look_empty():
    lib = stub_lib()
    cfg = lt.make_config(2, 4, 4, 2, 128, 2, 6, 50)
    c = Ctx(lib, cfg, [0, 1])
    for layer in (0, 1):
        assert c.append_ragged(layer, 20, [20, 0, 7, 11]) == lt.OK
        assert last_append(lib)["ragged"] == 1
    assert c.len(0) == (20, 20) and c.seq_len(0, 2) == (7, 7) and c.seq_len(1, 3) == (11, 8) and c.seq_len(1, 1) == (0, 0)
    assert c.step(0) == lt.OK
    d = last_decode(lib)
    assert d["mode"] == 1 and d["stored"] == 21
    stored_b, slot_b = last_lengths(lib, 4)
    assert stored_b == [21, 1, 8, 12] and slot_b == [20, 0, 7, 11]
    assert c.step(1) == lt.OK
    stored_b, slot_b = last_lengths(lib, 4)
    assert stored_b == [8, 1, 8, 8] and slot_b == [2 + (20 - 2) % 6, 0, 2 + (7 - 2) % 6, 2 + (11 - 2) % 6]
    # sequences 1 and 2 sit a step out: they look empty to the kernel and keep their lengths
    assert c.step_active(0, [1, 0, 0, 1]) == lt.OK
    stored_b, slot_b = last_lengths(lib, 4)
    assert stored_b == [22, 0, 0, 13] and slot_b == [21, -1, -1, 12]
    assert [c.seq_len(0, b)[0] for b in range(4)] == [22, 1, 8, 13]
    # a slot changes hands
    assert lib.lt_reset_sequence(c.h, 0) == lt.OK
    assert c.seq_len(0, 0) == (0, 0) and c.len(0) == (13, 13)
    assert c.append_ragged(0, 5, [5, 0, 0, 0]) == lt.OK and c.seq_len(0, 0) == (5, 5)
    assert c.append_ragged(0, 5, [6, 0, 0, 0]) == lt.ERR_INVALID_ARG       # more tokens than the padded input holds
    assert c.append_ragged(0, 60, [60, 0, 0, 0]) == lt.ERR_CAPACITY
    assert c.seq_len(0, 0) == (5, 5)
    c.close()
    big = lt.make_config(1, 129, 4, 2, 128, 2, 6, 50)                 # the lengths travel as launch arguments: 128 at most
    c = Ctx(lib, big, [0])
    assert c.append_ragged(0, 3, [3] * 129) == lt.ERR_SHAPE and lib.lt_reset_sequence(c.h, 0) == lt.ERR_SHAPE
    c.close()
    most = lt.make_config(1, 128, 4, 2, 128, 2, 6, 50)
    c = Ctx(lib, most, [0])
    assert c.append_ragged(0, 3, [3] * 127 + [1]) == lt.OK and c.step(0) == lt.OK
    stored_b, slot_b = last_lengths(lib, 128)
    assert stored_b == [4] * 127 + [2] and slot_b == [3] * 127 + [1]
    c.close()


def test_paged_context_refuses_tokens_without_a_page_before_any_launch():
    lib = stub_lib()
    cfg = lt.make_config(2, 2, 4, 2, 128, 2, 62, 512)
    c = Ctx(lib, cfg, [0, 1], paged=(64, 10))
    max_pages = 512 // 64
    table = np.full((2, max_pages), -1, np.int32)
    table[0, :2] = [3, 7]
    table[1, :1] = [0]
    assert lib.lt_set_block_table(c.h, table.ctypes.data, None) == lt.OK and counts(lib)["memcpy"] == 1
    assert c.append_ragged(0, 100, [100, 64]) == lt.OK
    assert last_append(lib)["paged"] == 1 and last_append(lib)["page_shift"] == 6
    assert c.append_ragged(0, 30, [30, 0]) == lt.ERR_STATE              # sequence 0 would need a third page
    before = counts(lib)["decode"]
    assert c.step(0) == lt.ERR_STATE and counts(lib)["decode"] == before   # sequence 1's next token has no page
    table[1, 1] = 9
    assert lib.lt_set_block_table(c.h, table.ctypes.data, None) == lt.OK
    assert c.step(0) == lt.OK and last_decode(lib)["mode"] == 2
    assert last_lengths(lib, 2) == ([101, 65], [100, 64])
    bad = table.copy()
    bad[0, 1] = -1                                                      # drops a page that holds tokens
    assert lib.lt_set_block_table(c.h, bad.ctypes.data, None) == lt.ERR_STATE
    bad = table.copy()
    bad[0, 3] = 10                                                      # outside the pool
    assert lib.lt_set_block_table(c.h, bad.ctypes.data, None) == lt.ERR_INVALID_ARG
    # the lazy layer keeps its ring and needs no pages
    assert c.append(1, 200) == lt.OK and c.step(1) == lt.OK and last_decode(lib)["mode"] == 1
    assert lib.lt_truncate_layer(c.h, 0, None) == lt.ERR_STATE
    c.close()


def test_online_slots_are_taken_and_returned():
    lib = stub_lib()
    cfg = lt.make_config(4, 1, 4, 2, 128, 2, 6, 64)
    c = Ctx(lib, cfg, online=2)                                         # three full-size slots, two rings
    assert c.append(0, 10) == lt.OK and c.append(1, 10) == lt.OK and c.append(2, 10) == lt.OK
    assert c.append(3, 10) == lt.ERR_CAPACITY and c.len(3) == (0, 0)     # every full-size slot is taken
    assert lib.lt_truncate_layer(c.h, 1, None) == lt.OK and counts(lib)["truncate"] == 1
    assert c.len(1) == (10, 8)
    assert lib.lt_truncate_layer(c.h, 1, None) == lt.ERR_STATE           # already lazy
    assert c.append(3, 10) == lt.OK                                      # the freed slot
    assert lib.lt_truncate_layer(c.h, 3, None) == lt.OK
    assert lib.lt_truncate_layer(c.h, 0, None) == lt.ERR_CAPACITY        # only two rings exist
    assert c.step(1) == lt.OK and last_decode(lib)["lazy_tag"] == 1 and last_decode(lib)["stored"] == 8
    assert c.append_ragged(0, 1, [1]) == lt.ERR_STATE
    assert lib.lt_reset(c.h) == lt.OK
    assert all(c.append(l, 1) == lt.OK for l in (3, 2, 1))               # all three slots are free again
    c.close()


def test_events_are_made_on_demand_and_reused():
    lib = stub_lib()
    cfg = lt.make_config(2, 1, 4, 2, 128, 2, 6, 64)
    c = Ctx(lib, cfg, [0, 1])
    assert c.append(0, 4) == lt.OK and c.append(1, 4) == lt.OK
    n, ms = ctypes.c_int64(), ctypes.c_double()
    for rounds in range(2):                                             # the second round reuses the first round's events
        assert lib.lt_profile_enable(c.h, 1) == lt.OK
        for _ in range(3):
            assert c.step(0) == lt.OK and c.step(1) == lt.OK
        assert c.append(0, 1) == lt.OK
        assert lib.lt_profile_enable(c.h, 0) == lt.OK
        assert c.step(0) == lt.OK                                       # not measured
        for kind, launches in ((0, 3), (1, 3), (2, 1)):
            assert lib.lt_profile_read(c.h, kind, ctypes.byref(n), ctypes.byref(ms)) == lt.OK
            assert (n.value, ms.value) == (launches, float(launches))   # the stub's events are 1 ms apart
    assert lib.lt_profile_read(c.h, 3, ctypes.byref(n), ctypes.byref(ms)) == lt.ERR_INVALID_ARG
    c.close()                                                           # destroys the seven events made (checked by the leak detector)


def test_scoring_plans_cover_the_prompt():
    lib = stub_lib()
    for B, Hkv, G, n, w in ((8, 8, 4, 32768, 64), (1, 8, 4, 131072, 64), (2, 2, 4, 500, 16), (1, 1, 8, 70, 64), (32, 8, 4, 16384, 8)):
        cfg = lt.make_config(1, B, Hkv * G, Hkv, 128, 4, 60, n)
        need = lt.lazy_ratio_workspace_bytes(cfg, n, w)
        call = lambda fn, *extra: fn(ctypes.byref(cfg), FAKE, FAKE, Hkv * n * 128, n * 128, 128, n, w, 0, *extra, None, None, FAKE, None)
        assert call(lib.lt_lazy_ratio, FAKE2, need) == lt.OK
        s = last_score(lib)
        assert (s["n_chunks"] - 1) * s["keys_per_block"] < n <= s["n_chunks"] * s["keys_per_block"]
        assert s["n_chunks_a"] == s["n_chunks"] and s["range_a_end"] == n and not s["has_lse"]
        assert s["keys_per_block"] % 128 == 0 and s["n_chunks"] * B * Hkv <= 512 + B * Hkv   # at most two ranges per compute unit
        part = B * Hkv * G * w * s["n_chunks"] * 3 * 4
        assert part <= s["scratch_offset"] < part + 256 and s["scratch_offset"] + B * Hkv * G * 4 + (B * Hkv + 1) * 4 <= need
        assert call(lib.lt_lazy_ratio_static) == lt.OK and last_score(lib) == s      # the same plan in the built-in array
        # Table 1's form reads two key ranges only
        need_lse = lt.lazy_ratio_lse_workspace_bytes(cfg, n, w)
        st = lib.lt_lazy_ratio_lse(ctypes.byref(cfg), FAKE, FAKE, Hkv * n * 128, n * 128, 128, n, w, 0, FAKE, Hkv * G * w, w, FAKE2, need_lse,
                                   None, None, FAKE, None)
        assert st == lt.OK
        t = last_score(lib)
        assert t["has_lse"] and t["range_a_end"] <= t["range_b_begin"] <= n and (t["range_a_end"] % 128 == 0 or t["range_a_end"] == n)
        assert t["range_a_end"] >= min(4, n) and t["range_b_begin"] <= max(n - w - 60 + 1, t["range_a_end"])
        covered = t["n_chunks_a"] * t["keys_per_block"] >= t["range_a_end"] and \
            (t["n_chunks"] - t["n_chunks_a"]) * t["keys_per_block"] >= n - t["range_b_begin"]
        assert covered
    assert counts(lib)["score"] == 15


def test_shared_tail_only_for_long_ranges_and_can_be_switched_off():
    lib = stub_lib()
    lib.lt_set_shared_tail.argtypes = [ctypes.c_void_p, ctypes.c_int32]
    lib.lt_set_shared_tail.restype = ctypes.c_int
    cfg = lt.make_config(2, 8, 32, 8, 128, 4, 2044, 40000)
    c = Ctx(lib, cfg, [0, 1])
    assert c.append(0, 32768) == lt.OK and c.append(1, 32768) == lt.OK
    assert c.step(0) == lt.OK
    d = last_decode(lib)
    assert d["tail_begin"] == (32769 - 32769 // 8) // 64 * 64 and d["n_splits"] == 4
    assert c.step(1) == lt.OK and last_decode(lib)["tail_begin"] == NO_TAIL       # a window of 2048 entries: ranges too short
    assert lib.lt_set_shared_tail(c.h, 0) == lt.OK
    assert c.step(0) == lt.OK
    d = last_decode(lib)
    assert d["tail_begin"] == NO_TAIL and d["n_splits"] * d["keys_per_block"] >= 32770
    assert lib.lt_set_shared_tail(c.h, 1) == lt.OK
    assert c.step(0) == lt.OK and last_decode(lib)["tail_begin"] != NO_TAIL
    assert lib.lt_set_shared_tail(None, 1) == lt.ERR_INVALID_ARG
    c.close()
    # eight ranges of 4096 keys per (sequence, KV head): an eighth is shared when a piece is cheap to work through
    # (four heads per group, or the matrix-core kernel that takes eight heads per group), not with five heads per group
    for q_heads, shares in ((32, True), (64, True), (40, False)):
        cfg = lt.make_config(1, 4, q_heads, 8, 128, 4, 2044, 40000)
        c = Ctx(lib, cfg, [0])
        assert c.append(0, 32768) == lt.OK and c.step(0) == lt.OK
        d = last_decode(lib)
        assert d["tail_begin"] == ((32769 - 32769 // 8) // 64 * 64 if shares else NO_TAIL), (q_heads, d)
        assert d["n_splits"] == 8 and d["n_splits"] * d["keys_per_block"] >= (d["tail_begin"] if shares else 32769)
        assert (d["n_splits"] - 1) * d["keys_per_block"] < (d["tail_begin"] if shares else 32769)
        plan = (ctypes.c_int32 * 4)()
        assert lib.lt_decode_plan_read(c.h, 0, plan) == lt.OK
        assert list(plan) == [d["keys_per_block"], 8, d["tail_begin"] if shares else -1, 1 if q_heads == 64 else 0]
        assert lib.lt_decode_plan_read(c.h, 1, plan) == lt.ERR_INVALID_ARG and lib.lt_decode_plan_read(c.h, 0, None) == lt.ERR_INVALID_ARG
        c.close()
    cfg = lt.make_config(2, 1, 8, 2, 128, 4, 60, 500)
    c = Ctx(lib, cfg, [0, 1])
    assert c.append(1, 100) == lt.OK and c.step(1) == lt.OK
    plan = (ctypes.c_int32 * 4)(7, 7, 7, 7)
    assert lib.lt_decode_plan_read(c.h, 0, plan) == lt.ERR_INVALID_ARG and list(plan) == [7, 7, 7, 7]     # layer 0 has not run
    assert lib.lt_decode_plan_read(c.h, 1, plan) == lt.OK and plan[1] >= 1 and plan[2] == -1
    c.close()
    # short ranges (at most 2048 keys per workgroup) go to the matrix-core kernel from four heads per group on
    for group in (1, 2, 3, 4, 5, 8):
        cfg = lt.make_config(1, 8, 8 * group, 8, 128, 4, 2044, 5000)
        c = Ctx(lib, cfg, [0])
        assert c.append(0, 4000) == lt.OK and c.step(0) == lt.OK
        plan = (ctypes.c_int32 * 4)()
        assert lib.lt_decode_plan_read(c.h, 0, plan) == lt.OK
        assert 128 < plan[0] <= 2048 and plan[3] == (1 if group >= 4 else 0), (group, list(plan))
        c.close()
    # a lazy layer at batch 1 (eight streams, a window of 2048 entries): 32 ranges of 64 keys on the vector kernel with up
    # to five heads per group, 16 ranges of 128 keys on the matrix-core kernel with six or more
    for group, keys, matrix in ((1, 64, 0), (4, 64, 0), (5, 64, 0), (6, 128, 1), (8, 128, 1)):
        cfg = lt.make_config(1, 1, 8 * group, 8, 128, 4, 2044, 5000)
        c = Ctx(lib, cfg, [1])
        assert c.append(0, 4000) == lt.OK and c.step(0) == lt.OK
        plan = (ctypes.c_int32 * 4)()
        assert lib.lt_decode_plan_read(c.h, 0, plan) == lt.OK
        assert list(plan) == [keys, 2048 // keys, -1, matrix], (group, list(plan))
        c.close()
    # one workgroup per (sequence, KV head): nothing to share a tail between
    cfg = lt.make_config(1, 32, 32, 8, 128, 4, 2044, 17000)
    c = Ctx(lib, cfg, [0])
    assert c.append(0, 16384) == lt.OK and c.step(0) == lt.OK
    assert last_decode(lib)["n_splits"] == 1 and last_decode(lib)["tail_begin"] == NO_TAIL
    c.close()
