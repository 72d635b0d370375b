"""GPU parity for the paper's online procedure: layer-by-layer prefill, lazy ratio, priority queue,
immediate reduction of the popped layer's cache, then decoding -- against the oracle, which scores
every layer, runs the queue procedure on the same ratios and keeps whole histories."""
import numpy as np
import pytest
import torch

import lt_workloads as W
import oracle
from gpu_util import TOL_OUT, TOL_RATIO, bits, f64, say
from paper_2410_13846_amd import lt

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def online_prefill(wl, n_full):
    cfg = lt.make_config(wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.w_sink, wl.w_recent,
                         wl.context + wl.decode_steps)
    ctx = lt.Context(cfg, device=DEV, n_full_online=n_full)
    queue = lt.SelectQueue(n_full)
    hist = oracle.History(wl.n_layers, [0] * wl.n_layers, wl.w_sink, wl.w_recent)
    ratios, popped_at = [], np.full(wl.n_layers, -1, dtype=np.int32)
    for layer in range(wl.n_layers):
        say("online prefill layer", layer)
        k, v = W.prefill_kv(wl, layer, DEV)
        q_last = W.last_queries(wl, layer, DEV)
        ctx.append_kv(layer, k, v)                                    # takes a free full-size slot
        k_cache, _ = ctx.layer_tensors(layer)
        mean, _, _ = lt.lazy_ratio(cfg, q_last, k_cache, wl.context, wl.w_last)      # scored in place from the cache
        r = float(mean.cpu()[0])
        ref = oracle.lazy_ratio(bits(q_last), bits(k), wl.w_sink, wl.w_recent)[2]
        assert abs(r - ref) <= TOL_RATIO
        ratios.append(r)
        hist.append(layer, bits(k), bits(v))
        out = queue.push(r, layer)
        if out >= 0:
            ctx.truncate_layer(out)                                   # frees its slot for the next layer
            popped_at[out] = layer
    queue.close()
    return cfg, ctx, hist, np.asarray(ratios, np.float32), popped_at


@pytest.mark.parametrize("n_full", [0, 3, 6])
def test_online_prefill_then_decode(n_full):
    wl = W.WORKLOADS["llama3_8b_32k"].scaled(n_layers=6, batch=2, context=1500, w_recent=252, n_lazy=3, decode_steps=300,
                                             w_last=32)
    cfg, ctx, hist, ratios, popped_at = online_prefill(wl, n_full)
    ref_lazy, ref_pop = oracle.select_lazy_queue(ratios.astype(np.float64), wl.n_layers - n_full)
    np.testing.assert_array_equal(popped_at, ref_pop)
    hist.is_lazy = [bool(x) for x in ref_lazy]
    if n_full == 3:
        assert list(np.nonzero(ref_lazy)[0]) == W.planted_lazy_layers(wl)
    # peak memory: P + 1 full slots were enough for all L layers
    assert ctx.kv_slab.numel() == lt.kv_bytes_online(cfg, n_full)
    for layer in range(wl.n_layers):
        view = ctx.layer_view(layer)
        assert view["is_lazy"] == bool(ref_lazy[layer])
        assert ctx.layer_len(layer) == (wl.context, min(wl.context, wl.w_sink + wl.w_recent) if ref_lazy[layer] else wl.context)
    worst = 0.0
    for step in range(wl.decode_steps):                               # long enough for the rings to wrap
        check = step < 3 or step % 97 == 0 or step == wl.decode_steps - 1
        for layer in range(wl.n_layers):
            q, k, v = W.decode_qkv(wl, layer, step, DEV)
            out = ctx.decode_step(layer, q, k, v)
            hist.append(layer, bits(k), bits(v))
            if check:
                ref, _ = hist.decode(layer, bits(q))
                worst = max(worst, np.abs(f64(out) - ref).max())
    say("online: worst error", worst)
    assert worst <= TOL_OUT
    ctx.close()


def test_truncated_ring_matches_a_ring_filled_by_append():
    """Byte-exact: reducing a full cache leaves the ring exactly as a lazy layer's bulk append does."""
    B, Hkv, ws, wr = 2, 2, 4, 60
    for n in (3, 40, 64, 65, 1000):
        cfg = lt.make_config(2, B, 8, Hkv, 128, ws, wr, 1200)
        online = lt.Context(cfg, device=DEV, n_full_online=1)
        fixed = lt.Context(cfg, [1, 1], DEV)
        g = torch.Generator(device=DEV)
        g.manual_seed(900 + n)
        k = torch.randn(B, Hkv, n, 128, generator=g, device=DEV).to(torch.bfloat16)
        v = torch.randn(B, Hkv, n, 128, generator=g, device=DEV).to(torch.bfloat16)
        say("truncate vs append, n", n)
        online.append_kv(0, k, v)
        online.truncate_layer(0)
        fixed.append_kv(0, k, v)
        stored = min(n, ws + wr)
        for a, b in zip(online.layer_tensors(0), fixed.layer_tensors(0)):
            assert a.shape == b.shape
            assert torch.equal(a[:, :, :stored].view(torch.int16), b[:, :, :stored].view(torch.int16))
        # the freed full-size slot is reusable by the next layer
        online.append_kv(1, k, v)
        assert online.layer_view(1)["k"] == online.kv_slab.data_ptr()
        with pytest.raises(lt.LtError) as e:                          # P + 1 = 2 slots, one free
            pass_ctx = lt.Context(cfg, device=DEV, n_full_online=0)
            pass_ctx.append_kv(0, k, v)
            pass_ctx.append_kv(1, k, v)
        assert e.value.status == lt.ERR_CAPACITY
        online.close()
        fixed.close()
