"""GPU parity for ragged batches (every sequence of the batch with its own length) and for the bf16
output variant of the decode calls, through the C ABI.  The oracle has no notion of a ragged batch and needs
none: every sequence is checked on its own against the oracle's plain definition over that sequence's history."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL_LSE, TOL_OUT, bits, f64, randn_bf16, say
from paper_2410_13846_amd import lt

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def ring_slot(p, ws, wr):
    return p if p < ws else ws + (p - ws) % wr


def run_ragged(lengths, Hq, Hkv, ws, wr, steps, seed, second_chunk=None, uniform_chunk=0, forced_split=None):
    B = len(lengths)
    say("ragged case", dict(lengths=lengths, Hq=Hq, Hkv=Hkv, ws=ws, wr=wr, steps=steps, seed=seed, second=second_chunk,
                            uniform=uniform_chunk, split=forced_split))
    extra = (max(second_chunk) if second_chunk else 0) + uniform_chunk
    cfg = lt.make_config(2, B, Hq, Hkv, 128, ws, wr, max(lengths) + extra + steps + 1)
    is_lazy = [0, 1]
    ctx = lt.Context(cfg, is_lazy, DEV)
    if forced_split:
        ctx.set_split(*forced_split)
    hists = [oracle.History(2, is_lazy, ws, wr) for _ in range(B)]
    kept = [[[], []] for _ in range(B)]                        # per sequence and layer: every K row appended, in order

    def append_ragged(counts, seed):
        n_max = max(max(counts), 1)
        for layer in range(2):
            k = randn_bf16((B, Hkv, n_max, 128), seed + 10 * layer)
            v = randn_bf16((B, Hkv, n_max, 128), seed + 10 * layer + 1)
            ctx.append_kv_ragged(layer, k, v, counts)
            for b in range(B):
                if counts[b] > 0:
                    hists[b].append(layer, bits(k[b:b + 1, :, :counts[b]]), bits(v[b:b + 1, :, :counts[b]]))
                    kept[b][layer].append(bits(k[b, :, :counts[b]]))

    append_ragged(lengths, seed)
    if second_chunk:
        append_ragged(second_chunk, seed + 100)
    if uniform_chunk:
        for layer in range(2):
            k = randn_bf16((B, Hkv, uniform_chunk, 128), seed + 200 + layer)
            v = randn_bf16((B, Hkv, uniform_chunk, 128), seed + 210 + layer)
            ctx.append_kv(layer, k, v)
            for b in range(B):
                hists[b].append(layer, bits(k[b:b + 1]), bits(v[b:b + 1]))
                kept[b][layer].append(bits(k[b]))
    worst = 0.0
    for step in range(steps):
        for layer in range(2):
            q = randn_bf16((B, Hq, 128), seed + 1000 + 7 * step + layer)
            kn = randn_bf16((B, Hkv, 1, 128), seed + 2000 + 7 * step + layer)
            vn = randn_bf16((B, Hkv, 1, 128), seed + 3000 + 7 * step + layer)
            if step % 2 == 0:
                out, lse = ctx.decode_step(layer, q, kn, vn, want_lse=True)
            else:                                              # the unfused pair must behave the same
                ctx.append_kv(layer, kn, vn)
                out, lse = ctx.decode_attn(layer, q, want_lse=True)
            for b in range(B):
                hists[b].append(layer, bits(kn[b:b + 1]), bits(vn[b:b + 1]))
                kept[b][layer].append(bits(kn[b]))
                ref, ref_lse = hists[b].decode(layer, bits(q[b:b + 1]))
                worst = max(worst, np.abs(f64(out[b:b + 1]) - ref).max())
                assert np.abs(f64(lse[b:b + 1]) - ref_lse).max() <= TOL_LSE
    assert worst <= TOL_OUT
    totals = [lengths[b] + (second_chunk[b] if second_chunk else 0) + uniform_chunk + steps for b in range(B)]
    kc_full, _ = ctx.layer_tensors(0)
    kc_ring, _ = ctx.layer_tensors(1)
    for b in range(B):
        assert ctx.seq_len(0, b) == (totals[b], totals[b])
        assert ctx.seq_len(1, b) == (totals[b], min(totals[b], ws + wr))
        rows = np.concatenate(kept[b][0], axis=1)              # [Hkv, total_b, 128] bits in position order
        np.testing.assert_array_equal(bits(kc_full[b, :, :totals[b]].contiguous()), rows)
        rows = np.concatenate(kept[b][1], axis=1)
        ring = bits(kc_ring[b].contiguous())
        for p in list(range(min(ws, totals[b]))) + list(range(max(ws, totals[b] - wr), totals[b])):
            np.testing.assert_array_equal(ring[:, ring_slot(p, ws, wr)], rows[:, p])
    assert ctx.layer_len(0)[0] == max(totals)
    ctx.close()


def test_ragged_prompts_short_and_long():
    run_ragged([5, 300, 1, 1500], Hq=8, Hkv=2, ws=4, wr=60, steps=4, seed=8000)


def test_ragged_with_empty_sequences_then_fused_steps():
    run_ragged([0, 77, 0, 2], Hq=4, Hkv=1, ws=4, wr=28, steps=3, seed=8100)


def test_ragged_chunked_prefill_and_uniform_chunk():
    run_ragged([100, 7, 650], Hq=10, Hkv=2, ws=2, wr=126, steps=2, seed=8200, second_chunk=[30, 200, 0], uniform_chunk=17)


def test_ragged_many_splits_and_empty_ranges():
    """Forced small key ranges: the short sequences' workgroups beyond their end contribute empty partial results."""
    run_ragged([2100, 3, 640, 65], Hq=8, Hkv=2, ws=4, wr=252, steps=3, seed=8300, forced_split=(256, 128))


def test_ragged_batch_of_sixteen_groups_of_five():
    lengths = [1 + (37 * i * i) % 900 for i in range(16)]
    run_ragged(lengths, Hq=5, Hkv=1, ws=4, wr=124, steps=2, seed=8400)


def test_ragged_batch_of_128_sequences():
    """The most sequences a ragged launch can carry lengths for."""
    lengths = [(53 * i * i + 7 * i) % 700 for i in range(128)]      # includes empty sequences
    run_ragged(lengths, Hq=4, Hkv=1, ws=4, wr=124, steps=2, seed=8450)


def test_ragged_batch_with_a_shared_tail():
    # two workgroups per (sequence, KV head) with ranges above 8192 keys: the launch leaves keys 14336.. to a shared
    # tail; sequences that end before it, inside it and at its first keys all take part in the same launch
    lengths = [16390, 9000, 14337, 14336, 14400, 16000, 1, 15000, 16390, 12000, 14350, 16389, 8192, 8193, 16200, 14335]
    run_ragged(lengths, Hq=16, Hkv=8, ws=4, wr=1020, steps=3, seed=77)


@pytest.mark.parametrize("Hq", [32, 64])
def test_ragged_batch_with_a_shared_tail_over_eight_ranges(Hq):
    # eight workgroups per (sequence, KV head) with ranges of about 4096 keys leave the last eighth (keys 28672..)
    # to a shared tail, on the vector kernel (four heads per group) and on the matrix-core kernel (eight)
    run_ragged([32780, 20000, 28673, 28672], Hq=Hq, Hkv=8, ws=4, wr=1020, steps=2, seed=78)


def test_sequence_without_tokens_gives_zero():
    cfg = lt.make_config(1, 2, 4, 1, 128, 4, 28, 64)
    ctx = lt.Context(cfg, [0], DEV)
    k, v = randn_bf16((2, 1, 9, 128), 8500), randn_bf16((2, 1, 9, 128), 8501)
    ctx.append_kv_ragged(0, k, v, [0, 9])
    q = randn_bf16((2, 4, 128), 8502)
    out, lse = ctx.decode_attn(0, q, want_lse=True)
    assert (out[0] == 0).all() and torch.isinf(lse[0]).all() and (lse[0] < 0).all()
    ref, ref_lse = oracle.decode_attn(bits(q[1:2]), bits(k[1:2]), bits(v[1:2]), oracle.MODE_FULL)
    assert np.abs(f64(out[1:2]) - ref).max() <= TOL_OUT
    ctx.close()


def test_ragged_errors():
    cfg = lt.make_config(1, 2, 4, 1, 128, 4, 28, 64)
    ctx = lt.Context(cfg, [0], DEV)
    k = randn_bf16((2, 1, 9, 128), 8600)
    with pytest.raises(lt.LtError):
        ctx.append_kv_ragged(0, k, k, [10, 1])                 # more than the padded rows
    with pytest.raises(lt.LtError):
        ctx.append_kv_ragged(0, k, k, [-1, 1])
    ctx.append_kv_ragged(0, k, k, [9, 1])
    big = randn_bf16((2, 1, 60, 128), 8601)
    with pytest.raises(lt.LtError) as e:
        ctx.append_kv_ragged(0, big, big, [56, 1])             # the longest sequence would pass max_tokens
    assert e.value.status == lt.ERR_CAPACITY
    assert ctx.seq_len(0, 0) == (9, 9) and ctx.seq_len(0, 1) == (1, 1)
    ctx.close()


@pytest.mark.parametrize("group,lazy", [(4, 0), (4, 1), (5, 0), (1, 1)])
def test_bf16_output_is_the_rounded_fp32_output(group, lazy):
    B, Hkv, n, ws, wr = 3, 2, 700, 4, 124
    Hq = group * Hkv
    cfg = lt.make_config(1, B, Hq, Hkv, 128, ws, wr, n + 4)
    k, v = randn_bf16((B, Hkv, n, 128), 8700 + group), randn_bf16((B, Hkv, n, 128), 8701 + group)
    outs = {}
    for dtype in (torch.float32, torch.bfloat16):
        ctx = lt.Context(cfg, [lazy], DEV)
        ctx.set_output_dtype(dtype)
        ctx.append_kv(0, k, v)
        for step in range(2):
            q = randn_bf16((B, Hq, 128), 8710 + step)
            kn, vn = randn_bf16((B, Hkv, 1, 128), 8720 + step), randn_bf16((B, Hkv, 1, 128), 8730 + step)
            out = ctx.decode_step(0, q, kn, vn)
            assert out.dtype == dtype
        outs[dtype] = out
        ctx.close()
    assert torch.equal(outs[torch.float32].to(torch.bfloat16), outs[torch.bfloat16])       # same bits: round to nearest even


def test_reset_sequence_frees_a_slot_for_a_new_prompt():
    """A contiguous context: one sequence ends, its slot takes a new prompt (shorter than the ring, then growing
    past it) while the others go on; every sequence is checked against the oracle over its own history."""
    B, Hq, Hkv, ws, wr = 3, 8, 2, 4, 28
    cfg = lt.make_config(2, B, Hq, Hkv, 128, ws, wr, 400)
    is_lazy = [0, 1]
    ctx = lt.Context(cfg, is_lazy, DEV)
    hists = [oracle.History(2, is_lazy, ws, wr) for _ in range(B)]

    def append(counts, seed):
        n_max = max(max(counts), 1)
        for layer in range(2):
            k = randn_bf16((B, Hkv, n_max, 128), seed + 10 * layer)
            v = randn_bf16((B, Hkv, n_max, 128), seed + 10 * layer + 1)
            ctx.append_kv_ragged(layer, k, v, counts)
            for b in range(B):
                if counts[b] > 0:
                    hists[b].append(layer, bits(k[b:b + 1, :, :counts[b]]), bits(v[b:b + 1, :, :counts[b]]))

    def check(seed):
        for layer in range(2):
            q = randn_bf16((B, Hq, 128), seed + layer)
            out, lse = ctx.decode_attn(layer, q, want_lse=True)
            for b in range(B):
                ref, ref_lse = hists[b].decode(layer, bits(q[b:b + 1]))
                assert np.abs(f64(out[b:b + 1]) - ref).max() <= TOL_OUT
                assert np.abs(f64(lse[b:b + 1]) - ref_lse).max() <= TOL_LSE

    append([120, 75, 33], 8700)
    check(8710)
    ctx.reset_sequence(1)
    assert ctx.seq_len(0, 1) == (0, 0) and ctx.seq_len(1, 1) == (0, 0) and ctx.seq_len(0, 0) == (120, 120)
    hists[1] = oracle.History(2, is_lazy, ws, wr)
    append([0, 9, 0], 8720)                                    # shorter than the ring: old ring entries must not show
    check(8730)
    append([1, 40, 1], 8740)                                   # the new sequence wraps its ring; the others step on
    check(8750)
    assert ctx.seq_len(1, 1) == (49, ws + wr) and ctx.layer_len(0)[0] == 121
    ctx.close()


@pytest.mark.parametrize("paged", [False, True])
def test_decode_step_for_the_sequences_still_generating(paged):
    """Some sequences sit steps out: they get no token, keep their length, are not read (rows 0 / -inf), and pick up
    where they left when they are active again; the others are checked against the oracle over their own history."""
    B, Hq, Hkv, ws, wr, page = 4, 8, 2, 4, 28, 64
    cfg = lt.make_config(2, B, Hq, Hkv, 128, ws, wr, 300)
    is_lazy = [0, 1]
    if paged:
        ctx = lt.Context(cfg, is_lazy, DEV, paged=(page, 24))
        ctx.set_block_table(np.random.default_rng(3).permutation(24)[:20].astype(np.int32).reshape(B, 5))
    else:
        ctx = lt.Context(cfg, is_lazy, DEV)
    hists = [oracle.History(2, is_lazy, ws, wr) for _ in range(B)]
    lengths = [70, 63, 5, 130]
    for layer in range(2):
        k = randn_bf16((B, Hkv, max(lengths), 128), 8800 + layer)
        v = randn_bf16((B, Hkv, max(lengths), 128), 8810 + layer)
        if paged:
            ctx.append_kv_ragged(layer, k, v, lengths)
        elif layer == 0:                                       # contiguous: start from a batch of equal lengths
            lengths = [70] * B
        if not paged:
            ctx.append_kv(layer, k[:, :, :70].contiguous(), v[:, :, :70].contiguous())
        for b in range(B):
            hists[b].append(layer, bits(k[b:b + 1, :, :lengths[b]]), bits(v[b:b + 1, :, :lengths[b]]))
    totals = list(lengths)
    patterns = [[1, 0, 1, 1], [1, 0, 0, 1], [0, 1, 1, 0], [1, 1, 1, 1], [0, 0, 0, 1]]
    for step, act in enumerate(patterns):
        for layer in range(2):
            q = randn_bf16((B, Hq, 128), 8820 + 7 * step + layer)
            kn = randn_bf16((B, Hkv, 1, 128), 8830 + 7 * step + layer)
            vn = randn_bf16((B, Hkv, 1, 128), 8840 + 7 * step + layer)
            out, lse = ctx.decode_step(layer, q, kn, vn, want_lse=True, active=act)
            for b in range(B):
                if act[b]:
                    hists[b].append(layer, bits(kn[b:b + 1]), bits(vn[b:b + 1]))
                    ref, ref_lse = hists[b].decode(layer, bits(q[b:b + 1]))
                    assert np.abs(f64(out[b:b + 1]) - ref).max() <= TOL_OUT
                    assert np.abs(f64(lse[b:b + 1]) - ref_lse).max() <= TOL_LSE
                else:
                    assert (out[b] == 0).all() and torch.isinf(lse[b]).all() and (lse[b] < 0).all()
        for b in range(B):
            totals[b] += act[b]
            assert ctx.seq_len(0, b) == (totals[b], totals[b])
            assert ctx.seq_len(1, b) == (totals[b], min(totals[b], ws + wr))
    assert ctx.layer_len(0)[0] == max(totals)
    with pytest.raises(lt.LtError):
        ctx.decode_step(0, q, kn, vn, active=[1, 1])           # one flag per sequence
    ctx.close()
