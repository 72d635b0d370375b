"""GPU parity for the paged storage of the full layers, through the C ABI.  Paging is a matter of where a token
lives, not of what is computed: every sequence is checked against the oracle's plain definition over that
sequence's history, whatever pages the block table scatters it over.  The pools start out filled with a pattern,
so the tests also see that only the pages a table names, and only the rows that hold tokens, are ever written."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL_LSE, TOL_OUT, bits, f64, randn_bf16, say
from paper_2410_13846_amd import lt

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
PATTERN = 0x5A5A                                             # bf16 bit pattern the pools are filled with


class Pager:
    """Hands out pages in a shuffled order, like a server whose pool has been in use for a while."""

    def __init__(self, B, max_pages, n_pages, page, seed):
        self.table = np.full((B, max_pages), -1, dtype=np.int32)
        self.free = list(np.random.default_rng(seed).permutation(n_pages))
        self.page = page

    def cover(self, b, tokens):
        """Make sure sequence b has pages for `tokens` tokens; True if the table changed."""
        changed = False
        for p in range(-(-tokens // self.page)):
            if self.table[b, p] < 0:
                self.table[b, p] = self.free.pop()
                changed = True
        return changed

    def release(self, b):
        self.free.extend(int(x) for x in self.table[b] if x >= 0)
        self.table[b] = -1


def fill_pools(ctx, layers):
    for layer in layers:
        for t in ctx.layer_tensors(layer):
            t.view(torch.int16).fill_(PATTERN)


def check_pools(ctx, layer, pager, totals, kept):
    """Rows that hold tokens carry exactly those tokens; every other row of the pools still holds the pattern."""
    kp, vp = ctx.layer_tensors(layer)
    kbits = bits(kp.contiguous())                            # [n_pages, Hkv, P, 128]
    untouched = np.ones(kbits.shape[:3], dtype=bool)
    P = pager.page
    for b, total in enumerate(totals):
        if total == 0:
            continue
        rows = np.concatenate(kept[b], axis=1)               # [Hkv, total, 128]
        for p in range(-(-total // P)):
            phys = pager.table[b, p]
            n = min(P, total - p * P)
            np.testing.assert_array_equal(kbits[phys, :, :n], rows[:, p * P: p * P + n])
            untouched[phys, :, :n] = False
    assert (kbits[untouched] == PATTERN).all()
    assert (bits(vp.contiguous())[untouched] == PATTERN).all()


def run_paged(lengths, Hq, Hkv, ws, wr, page, steps, seed, second_chunk=None, forced_split=None, spare_pages=3):
    B = len(lengths)
    say("paged case", dict(lengths=lengths, Hq=Hq, Hkv=Hkv, ws=ws, wr=wr, page=page, steps=steps, seed=seed,
                           second=second_chunk, split=forced_split))
    extra = max(second_chunk) if second_chunk else 0
    max_tokens = max(lengths) + extra + steps + 1
    max_pages = -(-max_tokens // page)
    totals_end = [lengths[b] + (second_chunk[b] if second_chunk else 0) + steps for b in range(B)]
    n_pages = sum(-(-t // page) for t in totals_end) + spare_pages
    cfg = lt.make_config(2, B, Hq, Hkv, 128, ws, wr, max_tokens)
    is_lazy = [0, 1]
    ctx = lt.Context(cfg, is_lazy, DEV, paged=(page, n_pages))
    fill_pools(ctx, [0])
    if forced_split:
        ctx.set_split(*forced_split)
    pager = Pager(B, max_pages, n_pages, page, seed)
    hists = [oracle.History(2, is_lazy, ws, wr) for _ in range(B)]
    kept = [[] for _ in range(B)]                            # layer 0: every K row appended, in order
    totals = [0] * B

    def append_ragged(counts, seed):
        for b in range(B):
            pager.cover(b, totals[b] + counts[b])
        ctx.set_block_table(pager.table)
        n_max = max(max(counts), 1)
        for layer in range(2):
            k = randn_bf16((B, Hkv, n_max, 128), seed + 10 * layer)
            v = randn_bf16((B, Hkv, n_max, 128), seed + 10 * layer + 1)
            ctx.append_kv_ragged(layer, k, v, counts)
            for b in range(B):
                if counts[b] > 0:
                    hists[b].append(layer, bits(k[b:b + 1, :, :counts[b]]), bits(v[b:b + 1, :, :counts[b]]))
                    if layer == 0:
                        kept[b].append(bits(k[b, :, :counts[b]]))
        for b in range(B):
            totals[b] += counts[b]

    append_ragged(lengths, seed)
    if second_chunk:
        append_ragged(second_chunk, seed + 100)
    worst = 0.0
    for step in range(steps):
        if any([pager.cover(b, totals[b] + 1) for b in range(B)]):
            ctx.set_block_table(pager.table)                  # some sequence crosses into a new page
        for layer in range(2):
            q = randn_bf16((B, Hq, 128), seed + 1000 + 7 * step + layer)
            kn = randn_bf16((B, Hkv, 1, 128), seed + 2000 + 7 * step + layer)
            vn = randn_bf16((B, Hkv, 1, 128), seed + 3000 + 7 * step + layer)
            if step % 2 == 0:
                out, lse = ctx.decode_step(layer, q, kn, vn, want_lse=True)
            else:                                            # the unfused pair must behave the same
                ctx.append_kv(layer, kn, vn)
                out, lse = ctx.decode_attn(layer, q, want_lse=True)
            for b in range(B):
                hists[b].append(layer, bits(kn[b:b + 1]), bits(vn[b:b + 1]))
                if layer == 0:
                    kept[b].append(bits(kn[b]))
                ref, ref_lse = hists[b].decode(layer, bits(q[b:b + 1]))
                worst = max(worst, np.abs(f64(out[b:b + 1]) - ref).max())
                assert np.abs(f64(lse[b:b + 1]) - ref_lse).max() <= TOL_LSE
        for b in range(B):
            totals[b] += 1
    assert worst <= TOL_OUT
    for b in range(B):
        assert ctx.seq_len(0, b) == (totals[b], totals[b])
        assert ctx.seq_len(1, b) == (totals[b], min(totals[b], ws + wr))
    check_pools(ctx, 0, pager, totals, kept)
    return ctx, pager, hists, totals


def test_paged_short_and_long_prompts_small_pages():
    run_paged([5, 300, 1, 1500], Hq=8, Hkv=2, ws=4, wr=60, page=64, steps=4, seed=9000)[0].close()


def test_paged_steps_cross_page_boundaries():
    """Prompts that end just before a page boundary: the fused and the unfused append both open a new page."""
    run_paged([127, 255, 64, 126], Hq=4, Hkv=1, ws=4, wr=28, page=128, steps=5, seed=9100)[0].close()


def test_paged_chunked_prefill_and_empty_sequence():
    run_paged([100, 0, 650], Hq=10, Hkv=2, ws=2, wr=126, page=256, steps=2, seed=9200, second_chunk=[30, 200, 0])[0].close()


def test_paged_many_splits_ranges_not_page_aligned():
    """Forced key ranges of 320 keys over 128-token pages: ranges start and end inside pages, and the short
    sequences' workgroups beyond their end contribute empty partial results."""
    run_paged([2100, 3, 640, 65], Hq=8, Hkv=2, ws=4, wr=252, page=128, steps=3, seed=9300, forced_split=(320, 128))[0].close()


def test_paged_long_sequence_many_pages_per_range():
    """One workgroup range spans up to 255 pages (all four page registers), and ranges of 100 pages that start inside a
    register; several tiles and a ragged tail."""
    run_paged([17000, 4133], Hq=4, Hkv=1, ws=4, wr=124, page=64, steps=2, seed=9400, forced_split=(16320, 128))[0].close()
    run_paged([9000, 6401], Hq=4, Hkv=1, ws=4, wr=124, page=64, steps=2, seed=9450, forced_split=(6400, 128))[0].close()


def test_paged_groups_of_five_and_eight():
    run_paged([700, 41, 1300], Hq=5, Hkv=1, ws=4, wr=124, page=256, steps=2, seed=9500)[0].close()
    run_paged([333, 1025], Hq=16, Hkv=2, ws=4, wr=60, page=512, steps=2, seed=9600)[0].close()


def test_paged_slot_changes_hands():
    """A sequence ends, its pages go back to the pool, and a new prompt takes the slot with other pages."""
    ctx, pager, hists, totals = run_paged([200, 90, 310], Hq=8, Hkv=2, ws=4, wr=60, page=64, steps=2, seed=9700, spare_pages=8)
    B, Hq, Hkv = 3, 8, 2
    pager.release(1)
    ctx.reset_sequence(1)
    assert ctx.seq_len(0, 1) == (0, 0) and ctx.seq_len(1, 1) == (0, 0)
    hists[1] = oracle.History(2, [0, 1], 4, 60)
    new_len = 150
    pager.cover(1, new_len)
    ctx.set_block_table(pager.table)
    for layer in range(2):
        k = randn_bf16((B, Hkv, new_len, 128), 9750 + layer)
        v = randn_bf16((B, Hkv, new_len, 128), 9760 + layer)
        ctx.append_kv_ragged(layer, k, v, [0, new_len, 0])
        hists[1].append(layer, bits(k[1:2]), bits(v[1:2]))
    for layer in range(2):
        q = randn_bf16((B, Hq, 128), 9770 + layer)
        out, lse = ctx.decode_attn(layer, q, want_lse=True)
        for b in range(B):
            ref, ref_lse = hists[b].decode(layer, bits(q[b:b + 1]))
            assert np.abs(f64(out[b:b + 1]) - ref).max() <= TOL_OUT
            assert np.abs(f64(lse[b:b + 1]) - ref_lse).max() <= TOL_LSE
    ctx.close()


def test_paged_matches_contiguous_context():
    """Same tokens, same queries: the paged and the contiguous context agree to the tolerance both hold against
    the oracle (the key order inside a workgroup differs, so not bit for bit), in fp32 and in bf16 output."""
    B, Hq, Hkv, n = 2, 8, 2, 1111
    cfg = lt.make_config(1, B, Hq, Hkv, 128, 4, 60, n + 8)
    flat = lt.Context(cfg, [0], DEV)
    paged = lt.Context(cfg, [0], DEV, paged=(128, 2 * (-(-(n + 8) // 128))))
    pager = Pager(B, -(-(n + 8) // 128), 2 * (-(-(n + 8) // 128)), 128, 9800)
    for b in range(B):
        pager.cover(b, n + 1)
    paged.set_block_table(pager.table)
    k, v = randn_bf16((B, Hkv, n, 128), 9801), randn_bf16((B, Hkv, n, 128), 9802)
    q = randn_bf16((B, Hq, 128), 9803)
    kn, vn = randn_bf16((B, Hkv, 1, 128), 9804), randn_bf16((B, Hkv, 1, 128), 9805)
    for dtype in (torch.float32, torch.bfloat16):
        outs = []
        for ctx in (flat, paged):
            ctx.reset()
            ctx.set_output_dtype(dtype)
            ctx.append_kv(0, k, v)
            outs.append(ctx.decode_step(0, q, kn, vn, want_lse=True))
        assert outs[1][0].dtype == dtype
        assert (outs[0][0].double() - outs[1][0].double()).abs().max().item() <= (2 * TOL_OUT if dtype == torch.float32 else 0.02)
        assert (outs[0][1] - outs[1][1]).abs().max().item() <= 2 * TOL_LSE
    flat.close()
    paged.close()


def test_paged_errors():
    cfg = lt.make_config(2, 2, 4, 1, 128, 4, 28, 300)
    with pytest.raises(lt.LtError):
        lt.Context(cfg, [0, 1], DEV, paged=(96, 8))          # not a power of two
    with pytest.raises(lt.LtError):
        lt.Context(cfg, [0, 1], DEV, paged=(32, 8))          # below the smallest page
    ctx = lt.Context(cfg, [0, 1], DEV, paged=(64, 6))
    k = randn_bf16((2, 1, 70, 128), 9900)
    with pytest.raises(lt.LtError) as e:
        ctx.append_kv(0, k, k)                               # no table yet: no page for any token
    assert e.value.status == lt.ERR_STATE
    table = np.full((2, 5), -1, dtype=np.int32)
    table[0, 0] = 6
    with pytest.raises(lt.LtError) as e:
        ctx.set_block_table(table)                           # outside the pool
    assert e.value.status == lt.ERR_INVALID_ARG
    table[0, :2] = [3, 1]
    table[1, 0] = 4
    ctx.set_block_table(table)
    with pytest.raises(lt.LtError) as e:
        ctx.append_kv(0, k, k)                               # sequence 1 has one page, 70 tokens need two
    assert e.value.status == lt.ERR_STATE
    assert ctx.seq_len(0, 0) == (0, 0)
    ctx.append_kv_ragged(0, k, k, [70, 64])
    ctx.append_kv_ragged(1, k, k, [70, 64])                  # the lazy layer needs no pages
    q = randn_bf16((2, 4, 128), 9901)
    one = randn_bf16((2, 1, 1, 128), 9902)
    with pytest.raises(lt.LtError) as e:
        ctx.decode_step(0, q, one, one)                      # sequence 1 is at a page boundary without a next page
    assert e.value.status == lt.ERR_STATE
    assert ctx.seq_len(0, 1) == (64, 64)
    shrunk = table.copy()
    shrunk[0, 1] = -1
    with pytest.raises(lt.LtError) as e:
        ctx.set_block_table(shrunk)                          # a page that holds tokens must stay named
    assert e.value.status == lt.ERR_STATE
    with pytest.raises(lt.LtError) as e:
        ctx.truncate_layer(0)
    assert e.value.status == lt.ERR_STATE
    table[1, 1] = 0
    ctx.set_block_table(table)
    ctx.decode_step(0, q, one, one)
    assert ctx.seq_len(0, 1) == (65, 65)
    ctx.close()
    plain = lt.Context(cfg, [0, 1], DEV)
    with pytest.raises(lt.LtError):
        plain.set_block_table(table)
    plain.close()
