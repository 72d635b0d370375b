"""GPU parity: lt_append_kv + lt_decode_attn through the C ABI against the CPU oracle, element by
element on seeded inputs.  The oracle keeps the whole history and applies the streaming set
positionally; the GPU side keeps a ring, so these tests also validate the ring."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL_LSE, TOL_OUT, bits, f64, randn_bf16, say
from paper_2410_13846_amd import lt

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_case(B, Hq, Hkv, n_prefill, steps, w_sink, w_recent, seed, split=None, max_extra=0, fused=False):
    say("decode case", dict(B=B, Hq=Hq, Hkv=Hkv, n=n_prefill, steps=steps, ws=w_sink, wr=w_recent, seed=seed, split=split, fused=fused))
    cfg = lt.make_config(2, B, Hq, Hkv, 128, w_sink, w_recent, n_prefill + steps + max_extra)
    mask = [0, 1]
    ctx = lt.Context(cfg, mask, DEV)
    if split is not None:
        ctx.set_split(*split)
    hist = oracle.History(2, mask, w_sink, w_recent)
    worst = 0.0
    if n_prefill > 0:
        for layer in range(2):
            k = randn_bf16((B, Hkv, n_prefill, 128), seed + 10 + layer)
            v = randn_bf16((B, Hkv, n_prefill, 128), seed + 20 + layer)
            ctx.append_kv(layer, k, v)
            hist.append(layer, bits(k), bits(v))
    for step in range(steps):
        for layer in range(2):
            q = randn_bf16((B, Hq, 128), seed + 1000 * (step + 1) + layer, scale=1.5)
            k = randn_bf16((B, Hkv, 1, 128), seed + 1000 * (step + 1) + 30 + layer)
            v = randn_bf16((B, Hkv, 1, 128), seed + 1000 * (step + 1) + 40 + layer)
            if fused:                                   # one launch: append on the fly + attend
                out, lse = ctx.decode_step(layer, q, k, v, want_lse=True)
            else:
                ctx.append_kv(layer, k, v)
                out, lse = ctx.decode_attn(layer, q, want_lse=True)
            hist.append(layer, bits(k), bits(v))
            ref, ref_lse = hist.decode(layer, bits(q))
            err = np.abs(f64(out) - ref).max()
            err_lse = np.abs(f64(lse) - ref_lse).max()
            assert err <= TOL_OUT, (layer, step, err)
            assert err_lse <= TOL_LSE, (layer, step, err_lse)
            worst = max(worst, err)
            total, stored = ctx.layer_len(layer)
            assert total == hist.length(layer)
            assert stored == (min(total, w_sink + w_recent) if mask[layer] else total)
    ctx.close()
    return worst


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("n_prefill", [0, 1, 15, 16, 17, 63, 64, 65, 300, 1027, 2500])
def test_prefill_lengths_span_tiles_and_ragged_tails(n_prefill, fused):
    run_case(B=2, Hq=8, Hkv=2, n_prefill=n_prefill, steps=3, w_sink=4, w_recent=60, seed=100 + n_prefill, fused=fused)


@pytest.mark.parametrize("group", [1, 2, 3, 4, 5, 6, 7, 8])
def test_every_query_group_size(group):
    run_case(B=1, Hq=2 * group, Hkv=2, n_prefill=333, steps=2, w_sink=4, w_recent=124, seed=200 + group, fused=group % 2 == 0)


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("ws,wr", [(0, 7), (4, 0), (1, 1), (4, 1020), (6, 252), (2, 508), (0, 2044), (300, 5)])
def test_window_shapes_including_the_paper_grid(ws, wr, fused):
    run_case(B=1, Hq=8, Hkv=2, n_prefill=2300, steps=3, w_sink=ws, w_recent=wr, seed=300 + ws + wr, fused=fused)


@pytest.mark.parametrize("fused", [False, True])
def test_ring_wraps_many_times_with_single_token_appends(fused):
    # window of 4 + 12 entries, 70 decode steps from an empty cache: the ring wraps five times
    run_case(B=2, Hq=4, Hkv=1, n_prefill=0, steps=70, w_sink=4, w_recent=12, seed=400, fused=fused)


def test_many_splits_merge_in_one_launch():
    # 20000 keys in 256-key ranges: 79 workgroups per (sequence, KV head) hand their results to the last one
    run_case(B=2, Hq=8, Hkv=2, n_prefill=20000, steps=4, w_sink=4, w_recent=1020, seed=450, split=(256, 64), fused=True)


@pytest.mark.parametrize("fused", [False, True])
def test_long_ranges_share_their_tail(fused):
    # 128 (sequence, KV head) pairs of 16K keys: two workgroups per pair with ranges above 8192 keys, so the last
    # eighth of every pair is handed out piece by piece to whichever wavefront is free, the new token's tile included
    run_case(B=16, Hq=16, Hkv=8, n_prefill=16390, steps=3, w_sink=4, w_recent=1020, seed=470, fused=fused)


def test_shared_tail_switched_off_gives_the_same_bits_every_time():
    B, Hq, Hkv, n = 16, 32, 8, 16500
    cfg = lt.make_config(1, B, Hq, Hkv, 128, 4, 1020, n)
    ctx = lt.Context(cfg, [0], DEV)
    ctx.append_kv(0, randn_bf16((B, Hkv, n, 128), 481), randn_bf16((B, Hkv, n, 128), 482))
    q = randn_bf16((B, Hq, 128), 483, scale=1.5)
    say("shared tail on / off, n", n)
    shared = [ctx.decode_attn(0, q).clone() for _ in range(3)]
    ctx.set_shared_tail(False)
    fixed = [ctx.decode_attn(0, q).clone() for _ in range(3)]
    assert torch.equal(fixed[0], fixed[1]) and torch.equal(fixed[0], fixed[2])
    for out in shared:                                        # the same keys in another order: rounding only
        assert (out - fixed[0]).abs().max().item() <= 2e-6
    ctx.set_shared_tail(True)
    assert (ctx.decode_attn(0, q) - fixed[0]).abs().max().item() <= 2e-6
    ctx.close()


@pytest.mark.parametrize("shape", [(16, 32, 16500), (4, 64, 32768), (4, 32, 32768), (1, 32, 131072)])
def test_shared_tail_gives_the_fixed_order_result_on_every_one_of_many_launches(shape):
    """Which wavefront takes which piece of the shared tail differs from launch to launch: a piece dropped or taken
    twice now and then would show here as one launch in a hundred that is off by more than rounding."""
    B, Hq, n = shape
    Hkv = 8
    cfg = lt.make_config(1, B, Hq, Hkv, 128, 4, 1020, n + 200)
    ctx = lt.Context(cfg, [0], DEV)
    ctx.append_kv(0, randn_bf16((B, Hkv, n, 128), 471), randn_bf16((B, Hkv, n, 128), 472))
    q = randn_bf16((B, Hq, 128), 473, scale=1.5)
    say("shared tail, 100 launches", shape)
    ctx.set_shared_tail(False)
    fixed, fixed_lse = ctx.decode_attn(0, q, want_lse=True)
    fixed, fixed_lse = fixed.clone(), fixed_lse.clone()
    assert ctx.decode_plan(0)["tail_begin"] == -1
    ctx.set_shared_tail(True)
    worst = torch.zeros((), device=DEV)
    for _ in range(100):
        out, lse = ctx.decode_attn(0, q, want_lse=True)
        worst = torch.maximum(worst, torch.maximum((out - fixed).abs().max(), (lse - fixed_lse).abs().max() * 0.1))
    import os
    vector_forced_on_large_group = Hq == 64 and os.environ.get("LT_DECODE_PATH") == "vector"     # then: no tail for 4096-key ranges
    assert ctx.decode_plan(0)["tail_begin"] > 0 or vector_forced_on_large_group
    assert worst.item() <= 2e-6, worst.item()
    # the fused step as well: the appended token is part of the tail's last piece
    k_new, v_new = randn_bf16((B, Hkv, 128), 474), randn_bf16((B, Hkv, 128), 475)
    ctx.set_shared_tail(False)
    outs = []
    for step in range(60):
        if step == 30:
            ctx.set_shared_tail(True)
        outs.append(ctx.decode_step(0, q, k_new, v_new).clone())
    # identical new tokens every step: step s with the tail on has s more copies than step 29 had; compare like with like
    ctx2 = lt.Context(cfg, [0], DEV)
    ctx2.set_shared_tail(False)
    ctx2.append_kv(0, randn_bf16((B, Hkv, n, 128), 471), randn_bf16((B, Hkv, n, 128), 472))
    for step in range(60):
        ref = ctx2.decode_step(0, q, k_new, v_new)
        assert (ref - outs[step]).abs().max().item() <= 2e-6, step
    ctx.close()
    ctx2.close()


def test_decode_plan_names_the_kernel_and_the_ranges_of_the_last_launch():
    import os
    forced = os.environ.get("LT_DECODE_PATH", "auto")        # the forced-kernel runs of this file set it
    # (batch, query heads, keys) -> matrix-core kernel by the library's own rule, shared tail
    cases = [((4, 64, 32768), True, True),                    # eight heads per group: long ranges too, an eighth shared
             ((4, 32, 32768), False, True),                   # four heads per group, ranges of 4096 keys: vector kernel
             ((8, 32, 4000), True, False),                    # ranges of at most 2048 keys, four heads per group
             ((8, 4, 4000), False, False),                    # the same with two heads per group: vector kernel
             ((1, 8, 100), True, False)]                      # the smallest range the library chooses has 256 keys
    for (B, Hq, n), matrix, tail in cases:
        Hkv = 8 if Hq >= 32 else 2
        cfg = lt.make_config(1, B, Hq, Hkv, 128, 4, 1020, n + 8)
        ctx = lt.Context(cfg, [0], DEV)
        with pytest.raises(lt.LtError):
            ctx.decode_plan(0)                                # nothing launched yet
        ctx.append_kv(0, randn_bf16((B, Hkv, n, 128), 491), randn_bf16((B, Hkv, n, 128), 492))
        say("decode plan", (B, Hq, n), forced)
        ctx.decode_attn(0, randn_bf16((B, Hq, 128), 493))
        plan = ctx.decode_plan(0)
        assert plan["matrix_cores"] == {"auto": matrix, "matrix": True, "vector": False}[forced], plan
        if Hq == 64 and forced == "vector":
            tail = False                                      # ranges of 4096 keys share a tail only where a piece is cheap
        assert (plan["tail_begin"] >= 0) == tail, plan
        covered = plan["tail_begin"] if tail else n
        assert (plan["n_splits"] - 1) * plan["keys_per_block"] < covered <= plan["n_splits"] * plan["keys_per_block"], plan
        ctx.set_split(512, 512)
        ctx.decode_attn(0, randn_bf16((B, Hq, 128), 494))
        plan = ctx.decode_plan(0)
        assert plan["keys_per_block"] == 512 and plan["n_splits"] == -(-n // 512) and plan["tail_begin"] == -1, plan
        if n <= 128:                                          # a single tile per wavefront: the vector kernel
            ctx.set_split(128, 128)
            ctx.decode_attn(0, randn_bf16((B, Hq, 128), 495))
            assert ctx.decode_plan(0)["matrix_cores"] == (forced == "matrix")
        ctx.close()


@pytest.mark.parametrize("split", [(256, 64), (512, 128), (2048, 2048)])
def test_result_does_not_depend_on_the_split(split):
    run_case(B=1, Hq=8, Hkv=2, n_prefill=3000, steps=2, w_sink=4, w_recent=1020, seed=500, split=split)


def test_streaming_equals_full_when_window_covers_history():
    B, Hq, Hkv, n = 1, 8, 2, 200
    cfg = lt.make_config(2, B, Hq, Hkv, 128, 4, 1020, n + 1)
    ctx = lt.Context(cfg, [0, 1], DEV)
    k, v = randn_bf16((B, Hkv, n, 128), 601), randn_bf16((B, Hkv, n, 128), 602)
    q = randn_bf16((B, Hq, 128), 603)
    say("streaming == full, n", n)
    outs = []
    for layer in range(2):
        ctx.append_kv(layer, k, v)
        outs.append(ctx.decode_attn(layer, q))
    assert (outs[0] - outs[1]).abs().max().item() <= 1e-6     # same entries, possibly split differently
    ctx.set_split(256, 256)
    outs = [ctx.decode_attn(layer, q) for layer in range(2)]
    assert torch.equal(outs[0], outs[1])                      # same kernel, same entries, same split: same bits
    ctx.close()


def test_uniform_keys_give_mean_of_values():
    B, Hq, Hkv, n = 1, 8, 2, 777
    cfg = lt.make_config(1, B, Hq, Hkv, 128, 4, 60, n)
    ctx = lt.Context(cfg, [0], DEV)
    k = randn_bf16((B, Hkv, 1, 128), 611).expand(B, Hkv, n, 128).contiguous()
    v = randn_bf16((B, Hkv, n, 128), 612)
    say("uniform keys, n", n)
    ctx.append_kv(0, k, v)
    out = ctx.decode_attn(0, randn_bf16((B, Hq, 128), 613))
    mean = v.double().mean(dim=2).repeat_interleave(Hq // Hkv, dim=1)
    assert (out.double() - mean).abs().max().item() <= 1e-5
    ctx.close()


def test_ring_slots_hold_exactly_the_kept_tokens():
    """Byte-exact: after a bulk prefill and some single appends, slot s of the ring holds the token
    the slot rule assigns to it, and a full layer holds every token in order."""
    B, Hkv, ws, wr, n, steps = 2, 2, 4, 28, 100, 45
    cfg = lt.make_config(2, B, 8, Hkv, 128, ws, wr, n + steps)
    ctx = lt.Context(cfg, [0, 1], DEV)
    ks = [randn_bf16((B, Hkv, n, 128), 621)]
    vs = [randn_bf16((B, Hkv, n, 128), 622)]
    say("ring slots")
    for layer in range(2):
        ctx.append_kv(layer, ks[0], vs[0])
    q = randn_bf16((B, 8, 128), 629)
    for s in range(steps):
        ks.append(randn_bf16((B, Hkv, 1, 128), 630 + s))
        vs.append(randn_bf16((B, Hkv, 1, 128), 730 + s))
        for layer in range(2):
            if s % 2:
                ctx.append_kv(layer, ks[-1], vs[-1])
            else:                                       # the fused step must leave the same bytes in the cache
                ctx.decode_step(layer, q, ks[-1], vs[-1])
    K, V = torch.cat(ks, 2), torch.cat(vs, 2)
    T = n + steps
    kf, vf = ctx.layer_tensors(0)
    assert torch.equal(kf[:, :, :T].view(torch.int16), K.view(torch.int16))
    assert torch.equal(vf[:, :, :T].view(torch.int16), V.view(torch.int16))
    kl, vl = ctx.layer_tensors(1)
    assert kl.shape[2] == ws + wr
    for p in list(range(ws)) + list(range(T - wr, T)):
        slot = p if p < ws else ws + (p - ws) % wr
        assert torch.equal(kl[:, :, slot].view(torch.int16), K[:, :, p].view(torch.int16)), p
        assert torch.equal(vl[:, :, slot].view(torch.int16), V[:, :, p].view(torch.int16)), p
    ctx.close()


def test_error_paths_on_the_device():
    cfg = lt.make_config(2, 1, 8, 2, 128, 4, 12, 10)
    ctx = lt.Context(cfg, [0, 1], DEV)
    k = randn_bf16((1, 2, 8, 128), 641)
    q = randn_bf16((1, 8, 128), 642)
    with pytest.raises(lt.LtError) as e:
        ctx.decode_attn(0, q)
    assert e.value.status == lt.ERR_STATE
    ctx.append_kv(0, k, k)
    with pytest.raises(lt.LtError) as e:
        ctx.append_kv(0, k, k)                          # 16 > max_tokens = 10
    assert e.value.status == lt.ERR_CAPACITY
    assert ctx.layer_len(0) == (8, 8)
    for _ in range(5):
        ctx.append_kv(1, k, k)                          # a lazy layer never overflows
    assert ctx.layer_len(1) == (40, 16)
    with pytest.raises(lt.LtError) as e:
        ctx.append_kv(0, k[:, :1], k[:, :1])
    assert e.value.status == lt.ERR_SHAPE
    out = ctx.decode_attn(0, q)
    assert torch.isfinite(out).all()
    ctx.decode_step(0, q, k[:, :, :1].contiguous(), k[:, :, :1].contiguous())
    ctx.decode_step(0, q, k[:, :, :1].contiguous(), k[:, :, :1].contiguous())
    with pytest.raises(lt.LtError) as e:                # 10 tokens stored, max_tokens = 10
        ctx.decode_step(0, q, k[:, :, :1].contiguous(), k[:, :, :1].contiguous())
    assert e.value.status == lt.ERR_CAPACITY
    assert ctx.layer_len(0) == (10, 10)
    ctx.reset()
    assert ctx.layer_len(1) == (0, 0)
    ctx.close()


@pytest.mark.parametrize("slope", [500.0, -500.0, 40.0])
def test_steadily_growing_or_falling_logits_across_splits(slope):
    """Logits that climb (or fall) by hundreds of natural units over the history: whole key ranges carry a weight
    that underflows against the others in the merge, row maxima move in almost every tile of the climbing case."""
    B, Hq, Hkv, T, ws, wr = 2, 8, 2, 3000, 4, 252
    say("decode ramp", slope)
    g = torch.Generator(device=DEV).manual_seed(6500 + int(abs(slope)))
    u = torch.randn(128, generator=g, device=DEV)
    u = u / u.norm()
    coeff = torch.arange(T, device=DEV, dtype=torch.float32) / T * slope            # q.k * scale = coeff
    k = (coeff[None, None, :, None] * u * (128 ** 0.25) + 0.05 * torch.randn(B, Hkv, T, 128, generator=g, device=DEV)).bfloat16()
    v = torch.randn(B, Hkv, T, 128, generator=g, device=DEV).bfloat16()
    q = ((u * (128 ** 0.25)).expand(B, Hq, 128) + 0.05 * torch.randn(B, Hq, 128, generator=g, device=DEV)).bfloat16().contiguous()
    cfg = lt.make_config(2, B, Hq, Hkv, 128, ws, wr, T + 4)
    ctx = lt.Context(cfg, [0, 1], DEV)
    ctx.set_split(256, 128)                                     # a dozen key ranges per sequence and head
    hist = oracle.History(2, [0, 1], ws, wr)
    for layer in range(2):
        ctx.append_kv(layer, k.contiguous(), v.contiguous())
        hist.append(layer, bits(k), bits(v))
        out, lse = ctx.decode_attn(layer, q, want_lse=True)
        ref, ref_lse = hist.decode(layer, bits(q))
        assert torch.isfinite(out).all() and torch.isfinite(lse).all()
        assert np.abs(f64(out) - ref).max() <= TOL_OUT
        assert np.abs(f64(lse) - ref_lse).max() <= TOL_LSE
    ctx.close()
