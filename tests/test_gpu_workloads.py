"""GPU parity at the benchmark configurations' real shapes, in the launch configuration bench.py
times (same batch, heads, context, window, default split choice, fused decode step).

The tiny configuration is compared tensor by tensor.  The large ones keep the real per-layer
shapes but fewer layers (a layer's launch does not depend on how many layers exist).  The
"whole batch" tests compare every output element of a full and a lazy layer over several
consecutive steps; the "sampled" ones cover more layers, scoring and paging on sampled
(layer, sequence) slices plus properties that hold for every output."""
import numpy as np
import pytest
import torch

import lt_workloads as W
import oracle
from gpu_util import TOL_LSE, TOL_OUT, TOL_RATIO, bits, f64, say
from paper_2410_13846_amd import lt

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make_cfg(wl, extra_tokens=0):
    return lt.make_config(wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.w_sink, wl.w_recent,
                          wl.context + wl.decode_steps + extra_tokens)


def test_tiny_hybrid_whole_tensors():
    """2 layers (0 full, 1 streaming), batch 1, 32/8 heads, prompt 4096, 4 + 1020 window, 16 decode steps,
    lazy ratio over the last 64 prompt queries: every output element against the oracle."""
    wl = W.WORKLOADS["tiny"].scaled(bias="planted")
    cfg = make_cfg(wl)
    ratios, kv = [], []
    for layer in range(wl.n_layers):
        say("tiny: scoring layer", layer)
        k, v = W.prefill_kv(wl, layer, DEV)
        q_last = W.last_queries(wl, layer, DEV)
        mean, seq, rho = lt.lazy_ratio(cfg, q_last, k, wl.context, wl.w_last, want_rho=True)
        ref_rho, ref_seq, ref_r = oracle.lazy_ratio(bits(q_last), bits(k), wl.w_sink, wl.w_recent)
        assert np.abs(f64(rho) - ref_rho).max() <= TOL_RATIO
        assert np.abs(f64(seq) - ref_seq).max() <= TOL_RATIO
        assert abs(float(mean.cpu()[0]) - ref_r) <= TOL_RATIO
        ratios.append(float(mean.cpu()[0]))
        kv.append((k, v))
    is_lazy, order = lt.select_lazy(ratios, wl.n_lazy)
    ref_lazy, _ = oracle.select_lazy(np.asarray(ratios, np.float32).astype(np.float64), wl.n_lazy)
    np.testing.assert_array_equal(is_lazy, ref_lazy)
    assert list(np.nonzero(is_lazy)[0]) == W.planted_lazy_layers(wl)

    ctx = lt.Context(cfg, is_lazy, DEV)
    hist = oracle.History(wl.n_layers, is_lazy, wl.w_sink, wl.w_recent)
    for layer, (k, v) in enumerate(kv):
        ctx.append_kv(layer, k, v)
        hist.append(layer, bits(k), bits(v))
    worst = 0.0
    for step in range(wl.decode_steps):
        for layer in range(wl.n_layers):
            q, k, v = W.decode_qkv(wl, layer, step, DEV)
            say("tiny: step", step, "layer", layer)
            out, lse = ctx.decode_step(layer, q, k, v, want_lse=True)
            hist.append(layer, bits(k), bits(v))
            ref, ref_lse = hist.decode(layer, bits(q))
            worst = max(worst, np.abs(f64(out) - ref).max())
            assert np.abs(f64(lse) - ref_lse).max() <= TOL_LSE
    assert worst <= TOL_OUT
    assert ctx.layer_len(0) == (wl.context + wl.decode_steps, wl.context + wl.decode_steps)
    assert ctx.layer_len(1) == (wl.context + wl.decode_steps, wl.w_sink + wl.w_recent)
    ctx.close()


def history_of(wl, layer, b, steps_done):
    """Whole K/V history of one sequence of one layer, regenerated from the seeds: uint16 [1,Hkv,T,d]."""
    k, v = W.prefill_kv(wl, layer, DEV)
    ks, vs = [bits(k[b:b + 1])], [bits(v[b:b + 1])]
    del k, v
    for step in range(steps_done):
        _, kn, vn = W.decode_qkv(wl, layer, step, DEV)
        ks.append(bits(kn[b:b + 1]))
        vs.append(bits(vn[b:b + 1]))
    return np.concatenate(ks, axis=2), np.concatenate(vs, axis=2)


def run_sampled(wl, layers, is_lazy, samples, steps, score_samples=(), page_tokens=0):
    """Fill the stack for `layers` (indices into the workload's recipe), decode `steps` tokens with the
    fused step, and check the sampled (position in `layers`, sequence) pairs at the last step.
    With page_tokens the full layers are paged behind a shuffled block table, as bench.py --paged runs them."""
    sub = wl.scaled(n_layers=len(layers), decode_steps=steps)
    cfg = make_cfg(sub)
    if page_tokens:
        max_pages = -(-int(cfg.max_tokens) // page_tokens)
        ctx = lt.Context(cfg, is_lazy, DEV, paged=(page_tokens, wl.batch * max_pages))
        ctx.set_block_table(np.random.default_rng(7).permutation(wl.batch * max_pages).astype(np.int32).reshape(wl.batch, max_pages))
    else:
        ctx = lt.Context(cfg, is_lazy, DEV)
    for i, layer in enumerate(layers):
        say(wl.name, "prefill layer", layer)
        k, v = W.prefill_kv(wl, layer, DEV)
        if (i, 0) in score_samples or any(s[0] == i for s in score_samples):
            q_last = W.last_queries(wl, layer, DEV)
            mean, seq, rho = lt.lazy_ratio(cfg, q_last, k, wl.context, wl.w_last, want_rho=True)
            rho_h = f64(rho)
            assert np.isfinite(rho_h).all() and rho_h.min() >= 0.0 and rho_h.max() <= 1.0 + 1e-6
            assert abs(float(mean.cpu()[0]) - float(seq.double().mean().cpu())) <= 1e-6
            for (si, b, g) in [s for s in score_samples if s[0] == i]:
                G = wl.group
                qs = bits(q_last[b:b + 1, g * G:(g + 1) * G])
                ksub = bits(k[b:b + 1, g:g + 1])
                ref_rho, _, _ = oracle.lazy_ratio(qs, ksub, wl.w_sink, wl.w_recent)
                err = np.abs(rho_h[b, g * G:(g + 1) * G] - ref_rho[0]).max()
                say(wl.name, "ratio sample layer", layer, "b", b, "kv head", g, "err", err)
                assert err <= TOL_RATIO
            del q_last
        ctx.append_kv(i, k, v)
        del k, v
    outs = {}
    for step in range(steps):
        for i, layer in enumerate(layers):
            q, k, v = W.decode_qkv(wl, layer, step, DEV)
            out, lse = ctx.decode_step(i, q, k, v, want_lse=True)
            if step == steps - 1:
                outs[i] = (q, out, lse)
    torch.cuda.synchronize()
    for i, (q, out, lse) in outs.items():
        assert torch.isfinite(out).all() and torch.isfinite(lse).all()
        assert out.abs().max().item() <= 8.0                  # a convex combination of N(0,1) bf16 values
    for (i, b) in samples:
        layer = layers[i]
        K, V = history_of(wl, layer, b, steps)
        q, out, lse = outs[i]
        mode = oracle.MODE_LAZY if is_lazy[i] else oracle.MODE_FULL
        ref, ref_lse = oracle.decode_attn(bits(q[b:b + 1]), K, V, mode, wl.w_sink, wl.w_recent)
        err = np.abs(f64(out[b:b + 1]) - ref).max()
        err_lse = np.abs(f64(lse[b:b + 1]) - ref_lse).max()
        say(wl.name, "decode sample layer", layer, "lazy" if is_lazy[i] else "full", "b", b, "T", K.shape[2], "err", err)
        assert err <= TOL_OUT and err_lse <= TOL_LSE
    total, stored = ctx.layer_len(0)
    assert total == wl.context + steps
    ctx.close()


def test_llama3_8b_32k_shapes_sampled():
    """Batch 8, 32/8 heads, context 32768, 4 + 2044 window: two planted-lazy and two full layers."""
    wl = W.WORKLOADS["llama3_8b_32k"]
    lazy_layers = W.planted_lazy_layers(wl)
    full_layers = [l for l in range(wl.n_layers) if l not in lazy_layers]
    layers = [full_layers[0], lazy_layers[0], full_layers[-1], lazy_layers[-1]]
    run_sampled(wl, layers, [0, 1, 0, 1], samples=[(0, 0), (1, 3), (2, 7), (3, 5)], steps=3,
                score_samples=[(0, 2, 1), (1, 6, 7)])


def test_llama2_7b_4k_shapes_sampled():
    """Batch 32, 32/32 heads (multi-head attention: 1024 (sequence, KV head) pairs, one workgroup each), context 4096,
    4 + 1020 window."""
    wl = W.WORKLOADS["llama2_7b_4k"]
    lazy_layers = W.planted_lazy_layers(wl)
    full_layers = [l for l in range(wl.n_layers) if l not in lazy_layers]
    layers = [full_layers[0], lazy_layers[0], full_layers[-1], lazy_layers[-1]]
    run_sampled(wl, layers, [0, 1, 0, 1], samples=[(0, 0), (1, 31), (2, 17), (3, 5)], steps=3,
                score_samples=[(0, 2, 1), (1, 30, 31)])


def test_llama3_70b_32k_shapes_sampled():
    """Batch 4, 64/8 heads (eight query heads per KV head: the matrix-core decode kernel on the full layers too, the
    scoring kernel's sixteen-tile form), context 32768, 4 + 2044 window."""
    wl = W.WORKLOADS["llama3_70b_32k"]
    lazy_layers = W.planted_lazy_layers(wl)
    full_layers = [l for l in range(wl.n_layers) if l not in lazy_layers]
    layers = [full_layers[0], lazy_layers[0], full_layers[-1], lazy_layers[-1]]
    run_sampled(wl, layers, [0, 1, 0, 1], samples=[(0, 0), (1, 3), (2, 2), (3, 1)], steps=3,
                score_samples=[(0, 2, 1), (1, 3, 7)])


def test_llama3_8b_32k_paged_shapes_sampled():
    """The same shape with the full layers in pages of 256 tokens handed out in a random order (bench.py --paged 256)."""
    wl = W.WORKLOADS["llama3_8b_32k"]
    lazy_layers = W.planted_lazy_layers(wl)
    full_layers = [l for l in range(wl.n_layers) if l not in lazy_layers]
    run_sampled(wl, [full_layers[1], lazy_layers[1]], [0, 1], samples=[(0, 2), (0, 7), (1, 4)], steps=3, page_tokens=256)


def test_mistral_7b_16k_paged_shapes_sampled():
    """Batch 32, context 16384, pages of 64 tokens: one workgroup's key range spans all four page registers."""
    wl = W.WORKLOADS["mistral_7b_16k"]
    run_sampled(wl, [5], [0], samples=[(0, 0), (0, 29)], steps=2, page_tokens=64)


def test_mistral_7b_16k_shapes_sampled():
    """Batch 32, context 16384: one full and one lazy layer of the sweep."""
    wl = W.WORKLOADS["mistral_7b_16k"]
    run_sampled(wl, [3, 17], [0, 1], samples=[(0, 31), (1, 12)], steps=2, score_samples=[(1, 20, 4)])


def test_qwq_32b_shapes_sampled():
    """40 query heads over 8 KV heads (groups of 5), batch 4, history grown to several thousand tokens."""
    wl = W.WORKLOADS["qwq_32b_gen"].scaled(context=6000)
    run_sampled(wl, [0, 40], [0, 1], samples=[(0, 1), (1, 3)], steps=4, score_samples=[(0, 2, 3)])


def test_llama31_8b_128k_shapes_sampled():
    """Context 131072, 4 + 4092 window, batch 1: decode over 128K keys and scoring at 128K."""
    wl = W.WORKLOADS["llama31_8b_128k_b1"]
    lazy_layers = W.planted_lazy_layers(wl)
    full_layers = [l for l in range(wl.n_layers) if l not in lazy_layers]
    run_sampled(wl, [full_layers[0], lazy_layers[0]], [0, 1], samples=[(0, 0), (1, 0)], steps=2,
                score_samples=[(1, 0, 5)])


def run_whole_batch(wl, layers, is_lazy, steps):
    """Every output element of every sequence and head, at every one of `steps` consecutive fused decode steps of
    the given layers, against the oracle over the whole positional history.  The layers alternate inside a step as
    they do in a stack, so the split workspace and the tickets are reused by launches of different split counts:
    a partial result left over from an earlier launch, or one merged before it was complete, shows up here."""
    sub = wl.scaled(n_layers=len(layers), decode_steps=steps)
    cfg = make_cfg(sub)
    ctx = lt.Context(cfg, is_lazy, DEV)
    n = wl.context
    hist_k, hist_v = [], []
    for i, layer in enumerate(layers):
        say(wl.name, "whole batch: prefill layer", layer)
        k, v = W.prefill_kv(wl, layer, DEV)
        ctx.append_kv(i, k, v)
        K = np.empty((wl.batch, wl.n_kv_heads, n + steps, wl.head_dim), np.uint16)
        V = np.empty_like(K)
        K[:, :, :n] = bits(k)
        V[:, :, :n] = bits(v)
        hist_k.append(K)
        hist_v.append(V)
        del k, v
    worst = {i: 0.0 for i in range(len(layers))}
    for step in range(steps):
        results = []
        for i, layer in enumerate(layers):
            q, k, v = W.decode_qkv(wl, layer, step, DEV)
            out, lse = ctx.decode_step(i, q, k, v, want_lse=True)
            results.append((q, k, v, out, lse))
        torch.cuda.synchronize()
        for i, (q, k, v, out, lse) in enumerate(results):
            T = n + step + 1
            hist_k[i][:, :, T - 1] = bits(k)[:, :, 0]
            hist_v[i][:, :, T - 1] = bits(v)[:, :, 0]
            K = hist_k[i] if T == n + steps else np.ascontiguousarray(hist_k[i][:, :, :T])
            V = hist_v[i] if T == n + steps else np.ascontiguousarray(hist_v[i][:, :, :T])
            mode = oracle.MODE_LAZY if is_lazy[i] else oracle.MODE_FULL
            ref, ref_lse = oracle.decode_attn(bits(q), K, V, mode, wl.w_sink, wl.w_recent)
            err = np.abs(f64(out) - ref)
            err_lse = np.abs(f64(lse) - ref_lse)
            say(wl.name, "whole batch: step", step, "layer", layers[i], "lazy" if is_lazy[i] else "full", "T", T,
                "max err", err.max(), "lse", err_lse.max())
            assert err.max() <= TOL_OUT, np.unravel_index(err.argmax(), err.shape)
            assert err_lse.max() <= TOL_LSE, np.unravel_index(err_lse.argmax(), err_lse.shape)
            worst[i] = max(worst[i], err.max())
    ctx.close()
    return worst


def test_llama3_8b_32k_whole_batch_every_row():
    """Batch 8, context 32768: all 8 x 32 x 128 outputs of one full and one planted-lazy layer, four steps in a row."""
    wl = W.WORKLOADS["llama3_8b_32k"]
    lazy_layers = W.planted_lazy_layers(wl)
    full_layer = [l for l in range(wl.n_layers) if l not in lazy_layers][2]
    run_whole_batch(wl, [full_layer, lazy_layers[2]], [0, 1], steps=4)


def test_mistral_7b_16k_whole_batch_every_row():
    """Batch 32, context 16384: 256 key streams, so one key range per (sequence, KV head) and no merge."""
    wl = W.WORKLOADS["mistral_7b_16k"]
    run_whole_batch(wl, [7, 21], [0, 1], steps=3)


def test_qwq_32b_whole_batch_every_row():
    """Groups of five query heads, batch 4, a history of 20000 tokens: 64 key ranges per (sequence, KV head)."""
    wl = W.WORKLOADS["qwq_32b_gen"].scaled(context=20000)
    run_whole_batch(wl, [1, 33], [0, 1], steps=4)


def test_llama31_8b_128k_b1_whole_batch_every_row():
    """Context 131072, batch 1, 4 + 4092 window: 32 key ranges per KV head merged in one launch."""
    wl = W.WORKLOADS["llama31_8b_128k_b1"]
    lazy_layers = W.planted_lazy_layers(wl)
    full_layer = [l for l in range(wl.n_layers) if l not in lazy_layers][1]
    run_whole_batch(wl, [full_layer, lazy_layers[1]], [0, 1], steps=3)


def test_llama31_8b_128k_batch_16_one_full_layer_every_row():
    """The batch-16 128K shape: one full layer holds 8.6 GB of K and V; offsets exceed 2^31 elements.  Every
    output of the launch against the oracle (the host copy of the layer is 8.6 GB)."""
    wl = W.WORKLOADS["llama31_8b_128k_b16"]
    lazy_layers = W.planted_lazy_layers(wl)
    full_layer = [l for l in range(wl.n_layers) if l not in lazy_layers][0]
    run_whole_batch(wl, [full_layer], [0], steps=1)


def run_whole_batch_ratio(wl, layer, static=False):
    """Every rho of every (sequence, head, query) of one layer's scoring call at the workload's real shape, the
    per-sequence ratios and the layer's ratio, against the oracle's Eq. 1."""
    cfg = make_cfg(wl)
    k, _ = W.prefill_kv(wl, layer, DEV)
    q_last = W.last_queries(wl, layer, DEV)
    say(wl.name, "whole batch: scoring layer", layer, "static scratch" if static else "workspace")
    if static:
        mean = torch.empty(1, dtype=torch.float32, device=DEV)
        seq = torch.empty(wl.batch, dtype=torch.float32, device=DEV)
        rho = torch.empty((wl.batch, wl.n_q_heads, wl.w_last), dtype=torch.float32, device=DEV)
        lt.lazy_ratio_static(cfg, q_last, k, wl.context, wl.w_last, mean, seq, rho)
    else:
        mean, seq, rho = lt.lazy_ratio(cfg, q_last, k, wl.context, wl.w_last, want_rho=True)
    torch.cuda.synchronize()
    ref_rho, ref_seq, ref_r = oracle.lazy_ratio(bits(q_last), bits(k), wl.w_sink, wl.w_recent)
    err = np.abs(f64(rho) - ref_rho)
    say(wl.name, "whole batch: scoring layer", layer, "max |rho - oracle|", err.max(), "r", ref_r, "err", abs(float(mean.cpu()[0]) - ref_r))
    assert err.max() <= TOL_RATIO, np.unravel_index(err.argmax(), err.shape)
    assert np.abs(f64(seq) - ref_seq).max() <= TOL_RATIO
    assert abs(float(mean.cpu()[0]) - ref_r) <= TOL_RATIO


def test_llama3_8b_32k_scoring_every_ratio():
    """Batch 8, n = 32768, w_last = 64: all 8 x 32 x 64 ratios of a planted-lazy and of a plain layer."""
    wl = W.WORKLOADS["llama3_8b_32k"]
    lazy_layers = W.planted_lazy_layers(wl)
    run_whole_batch_ratio(wl, lazy_layers[3])
    run_whole_batch_ratio(wl, [l for l in range(wl.n_layers) if l not in lazy_layers][3], static=True)


def test_llama31_8b_128k_b1_scoring_every_ratio():
    """n = 131072, batch 1: 32 key ranges per KV head merged by the last workgroup."""
    wl = W.WORKLOADS["llama31_8b_128k_b1"]
    run_whole_batch_ratio(wl, W.planted_lazy_layers(wl)[2])


def test_qwq_32b_scoring_every_ratio():
    """Groups of five query heads (ten query tiles dealt to eight wavefronts), batch 4, a prompt of 20000 tokens."""
    wl = W.WORKLOADS["qwq_32b_gen"].scaled(context=20000, bias="planted", n_lazy=32)
    run_whole_batch_ratio(wl, 7)


def test_llama3_8b_32k_prefill_and_ratio_from_lse_sampled():
    """Prefill attention of one planted-lazy layer at batch 8, 32/8 heads, n = 32768 in the launch configuration
    bench.py --prefill times: sampled rows against the oracle's decode of the truncated history (prefill row p ==
    decoding token p over keys 0..p), properties of every row, and the lazy ratio taken from that log-sum-exp."""
    wl = W.WORKLOADS["llama3_8b_32k"]
    layer = W.planted_lazy_layers(wl)[0]
    cfg = make_cfg(wl)
    n, w = wl.context, wl.w_last
    q = W.prefill_queries(wl, layer, DEV)
    k, v = W.prefill_kv(wl, layer, DEV)
    say(wl.name, "prefill layer", layer, "causal")
    out, lse = lt.prefill_attn(cfg, q, k, v, n, out_dtype=torch.float32)
    say(wl.name, "prefill layer", layer, "streaming")
    out_s, lse_s = lt.prefill_attn(cfg, q, k, v, n, lt.MASK_STREAMING, out_dtype=torch.float32)
    torch.cuda.synchronize()
    for o, l in ((out, lse), (out_s, lse_s)):
        assert torch.isfinite(o).all() and torch.isfinite(l).all()
        assert o.abs().max().item() <= 8.0
    assert (lse_s <= lse + 1e-4).all()                                   # a subset of the keys
    window = wl.w_sink + wl.w_recent
    assert torch.equal(out[:, :, :window], out_s[:, :, :window])         # the window still covers the whole history
    eps = 2.0 ** -8
    for b, p in [(0, 0), (1, 31), (2, 32), (3, 63), (4, 64), (5, 2047), (5, 2048), (6, 20000), (7, n - 1)]:
        K, V = bits(k[b:b + 1, :, :p + 1].contiguous()), bits(v[b:b + 1, :, :p + 1].contiguous())
        qp = bits(q[b:b + 1, :, p].contiguous())
        for mode, o, l in ((oracle.MODE_FULL, out, lse), (oracle.MODE_LAZY, out_s, lse_s)):
            ref, ref_lse, probs = oracle.decode_attn(qp, K, V, mode, wl.w_sink, wl.w_recent, return_probs=True)
            absw = np.einsum("bht,bhtd->bhd", probs, np.abs(oracle.bf16_bits_to_f64(np.repeat(V, wl.group, axis=1))))
            err = np.abs(f64(o[b:b + 1, :, p]) - ref)
            say(wl.name, "prefill row b", b, "p", p, "lazy" if mode else "full", "err", err.max())
            assert (err <= eps * absw + 2e-5).all()
            assert np.abs(f64(l[b:b + 1, :, p]) - ref_lse).max() <= 1e-4
    q_last = q[:, :, n - w:].contiguous()
    mean, seq, rho = lt.lazy_ratio_lse(cfg, q_last, k, n, w, lse[:, :, n - w:], want_rho=True)
    mean_d, seq_d, rho_d = lt.lazy_ratio(cfg, q_last, k, n, w, want_rho=True)
    assert (rho - rho_d).abs().max().item() <= TOL_RATIO and abs(float(mean.cpu()[0]) - float(mean_d.cpu()[0])) <= TOL_RATIO
    for b, g in [(2, 1), (6, 7)]:
        G = wl.group
        ref_rho, _, _ = oracle.lazy_ratio(bits(q_last[b:b + 1, g * G:(g + 1) * G]), bits(k[b:b + 1, g:g + 1]), wl.w_sink, wl.w_recent)
        assert np.abs(f64(rho)[b, g * G:(g + 1) * G] - ref_rho[0]).max() <= TOL_RATIO


def test_llama31_8b_128k_prefill_sampled():
    """Prefill attention at n = 131072 (batch 1, 4 + 4092 window): row offsets pass 2^31 bytes; sampled rows of
    both masks against the oracle's decode of the truncated history, and the ratio from the log-sum-exp."""
    wl = W.WORKLOADS["llama31_8b_128k_b1"]
    layer = W.planted_lazy_layers(wl)[0]
    cfg = make_cfg(wl)
    n, w = wl.context, wl.w_last
    q = W.prefill_queries(wl, layer, DEV)
    k, v = W.prefill_kv(wl, layer, DEV)
    say(wl.name, "prefill layer", layer, "causal, n =", n)
    out, lse = lt.prefill_attn(cfg, q, k, v, n, out_dtype=torch.float32)
    say(wl.name, "prefill layer", layer, "streaming")
    out_s, lse_s = lt.prefill_attn(cfg, q, k, v, n, lt.MASK_STREAMING, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all() and torch.isfinite(lse).all() and torch.isfinite(out_s).all() and torch.isfinite(lse_s).all()
    eps = 2.0 ** -8
    for p in (0, 4095, 4096, 65535, 100001, n - 1):
        K, V = bits(k[:, :, :p + 1].contiguous()), bits(v[:, :, :p + 1].contiguous())
        qp = bits(q[:, :, p].contiguous())
        for mode, o, l in ((oracle.MODE_FULL, out, lse), (oracle.MODE_LAZY, out_s, lse_s)):
            ref, ref_lse, probs = oracle.decode_attn(qp, K, V, mode, wl.w_sink, wl.w_recent, return_probs=True)
            absw = np.einsum("bht,bhtd->bhd", probs, np.abs(oracle.bf16_bits_to_f64(np.repeat(V, wl.group, axis=1))))
            err = np.abs(f64(o[:, :, p]) - ref)
            say(wl.name, "prefill row p", p, "lazy" if mode else "full", "err", err.max())
            assert (err <= eps * absw + 2e-5).all()
            assert np.abs(f64(l[:, :, p]) - ref_lse).max() <= 1e-4
    q_last = q[:, :, n - w:].contiguous()
    mean, _, rho = lt.lazy_ratio_lse(cfg, q_last, k, n, w, lse[:, :, n - w:], want_rho=True)
    mean_d, _, rho_d = lt.lazy_ratio(cfg, q_last, k, n, w, want_rho=True)
    assert (rho - rho_d).abs().max().item() <= TOL_RATIO and abs(float(mean.cpu()[0]) - float(mean_d.cpu()[0])) <= TOL_RATIO
