"""Pins for the decode-attention oracle (CPU only).

Each test checks oracle.decode_attn against something other than itself: a closed form,
an invariant of softmax attention, or an explicit N x N masked softmax assembled from
library routines (torch fp64 matmul / softmax) following the appendix's definition of
the causal and sink masks.
"""
import numpy as np
import pytest
import torch
from scipy.special import logsumexp

import oracle

RNG = np.random.default_rng(20241013)


def bf16_randn(*shape, scale=1.0):
    return oracle.f32_to_bf16_bits((RNG.standard_normal(shape) * scale).astype(np.float32))


def small_ints_bf16(*shape, lo=-3, hi=4):
    """Small integers are exact in bf16, so sums and shifts of them are exact too."""
    return oracle.f32_to_bf16_bits(RNG.integers(lo, hi, size=shape).astype(np.float32))


def streaming_positions(T, w_sink, w_recent):
    """Kept positions for the query at T-1: first w_sink and last w_recent (as a set)."""
    keep = set(range(min(w_sink, T))) | set(range(max(0, T - w_recent), T))
    return sorted(keep)


def test_bf16_roundtrip_helpers():
    x = np.array([1.0, -2.5, 3.140625, 0.0, 1e-3, 65280.0], dtype=np.float32)
    bits = oracle.f32_to_bf16_bits(x)
    back = oracle.bf16_bits_to_f64(bits)
    ref = torch.tensor(x).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(back, ref)


@pytest.mark.parametrize("T,ws,wr", [(1, 4, 8), (5, 4, 8), (12, 4, 8), (12, 0, 12), (7, 7, 0)])
def test_streaming_equals_full_when_window_covers_history(T, ws, wr):
    B, Hq, Hkv, d = 2, 4, 2, 16
    q, K, V = bf16_randn(B, Hq, d), bf16_randn(B, Hkv, T, d), bf16_randn(B, Hkv, T, d)
    full, lse_f = oracle.decode_attn(q, K, V, oracle.MODE_FULL)
    lazy, lse_l = oracle.decode_attn(q, K, V, oracle.MODE_LAZY, ws, wr)
    np.testing.assert_array_equal(full, lazy)
    np.testing.assert_array_equal(lse_f, lse_l)


@pytest.mark.parametrize("mode", ["full", "lazy"])
def test_uniform_keys_give_mean_of_values(mode):
    B, Hq, Hkv, d, T, ws, wr = 1, 4, 2, 8, 40, 3, 9
    q = bf16_randn(B, Hq, d)
    K = np.broadcast_to(bf16_randn(B, Hkv, 1, d), (B, Hkv, T, d)).copy()
    V = bf16_randn(B, Hkv, T, d)
    Vf = oracle.bf16_bits_to_f64(V)
    if mode == "full":
        out, lse = oracle.decode_attn(q, K, V, oracle.MODE_FULL)
        keep = list(range(T))
    else:
        out, lse = oracle.decode_attn(q, K, V, oracle.MODE_LAZY, ws, wr)
        keep = streaming_positions(T, ws, wr)
        assert len(keep) == ws + wr
    for h in range(Hq):
        np.testing.assert_allclose(out[0, h], Vf[0, h // 2, keep].mean(axis=0), rtol=0, atol=1e-13)
    # lse = s + log |S| with s the common logit
    qf, Kf = oracle.bf16_bits_to_f64(q), oracle.bf16_bits_to_f64(K)
    for h in range(Hq):
        s = (qf[0, h] * Kf[0, h // 2, 0]).sum() / np.sqrt(d)
        assert abs(lse[0, h] - (s + np.log(len(keep)))) < 1e-12


def test_zero_query_gives_mean_of_values():
    B, Hq, Hkv, d, T = 1, 2, 1, 8, 33
    q = np.zeros((B, Hq, d), dtype=np.uint16)
    K, V = bf16_randn(B, Hkv, T, d), bf16_randn(B, Hkv, T, d)
    out, lse = oracle.decode_attn(q, K, V, oracle.MODE_FULL)
    np.testing.assert_allclose(out[0, 1], oracle.bf16_bits_to_f64(V)[0, 0].mean(axis=0), atol=1e-13)
    np.testing.assert_allclose(lse, np.log(T), atol=1e-13)


@pytest.mark.parametrize("ws,wr", [(4, 8), (0, 5), (2, 0), (6, 30)])
def test_probabilities_sum_to_one_and_vanish_outside_the_set(ws, wr):
    B, Hq, Hkv, d, T = 2, 4, 2, 16, 29
    q, K, V = bf16_randn(B, Hq, d), bf16_randn(B, Hkv, T, d), bf16_randn(B, Hkv, T, d)
    _, _, p_full = oracle.decode_attn(q, K, V, oracle.MODE_FULL, return_probs=True)
    _, _, p_lazy = oracle.decode_attn(q, K, V, oracle.MODE_LAZY, ws, wr, return_probs=True)
    np.testing.assert_allclose(p_full.sum(-1), 1.0, atol=1e-14)
    np.testing.assert_allclose(p_lazy.sum(-1), 1.0, atol=1e-14)
    assert (p_full > 0).all()
    keep = np.zeros(T, dtype=bool)
    keep[streaming_positions(T, ws, wr)] = True
    assert (p_lazy[..., ~keep] == 0).all()
    assert (p_lazy[..., keep] > 0).all()


def test_dominant_key_returns_its_value():
    B, Hq, Hkv, d, T, ws, wr = 1, 2, 1, 16, 50, 4, 10
    q = oracle.f32_to_bf16_bits(np.full((B, Hq, d), 4.0, dtype=np.float32))
    K = np.zeros((B, Hkv, T, d), dtype=np.uint16)
    V = bf16_randn(B, Hkv, T, d)
    j_in, j_out = 45, 20          # 45 is a recent token of the query at 49; 20 is neither sink nor recent
    for j in (j_in, j_out):
        Kj = K.copy()
        Kj[0, 0, j] = oracle.f32_to_bf16_bits(np.full(d, 4.0, dtype=np.float32))   # logit 16*16/4 = 64
        out, _ = oracle.decode_attn(q, Kj, V, oracle.MODE_FULL)
        np.testing.assert_allclose(out[0, 0], oracle.bf16_bits_to_f64(V)[0, 0, j], atol=1e-20 + 50 * np.exp(-64) * 10)
        out_l, _ = oracle.decode_attn(q, Kj, V, oracle.MODE_LAZY, ws, wr)
        if j == j_in:
            np.testing.assert_allclose(out_l[0, 0], oracle.bf16_bits_to_f64(V)[0, 0, j], atol=1e-20 + 50 * np.exp(-64) * 10)
        else:                      # the dominant key is dropped: uniform over the kept set
            keep = streaming_positions(T, ws, wr)
            np.testing.assert_allclose(out_l[0, 0], oracle.bf16_bits_to_f64(V)[0, 0, keep].mean(0), atol=1e-13)


def test_softmax_shift_invariance():
    """Adding one vector to every key shifts all logits of a query equally: output unchanged."""
    B, Hq, Hkv, d, T = 1, 4, 2, 8, 24
    q, V = small_ints_bf16(B, Hq, d), bf16_randn(B, Hkv, T, d)
    Kv = RNG.integers(-3, 4, size=(B, Hkv, T, d)).astype(np.float32)
    delta = RNG.integers(-2, 3, size=(B, Hkv, 1, d)).astype(np.float32)
    K0, K1 = oracle.f32_to_bf16_bits(Kv), oracle.f32_to_bf16_bits(Kv + delta)
    for mode, ws, wr in [(oracle.MODE_FULL, 0, 0), (oracle.MODE_LAZY, 2, 7)]:
        o0, l0 = oracle.decode_attn(q, K0, V, mode, ws, wr)
        o1, l1 = oracle.decode_attn(q, K1, V, mode, ws, wr)
        np.testing.assert_allclose(o0, o1, atol=1e-13)
        qf = oracle.bf16_bits_to_f64(q)
        shift = np.einsum("bhd,bhd->bh", qf, np.repeat(delta[:, :, 0].astype(np.float64), Hq // Hkv, axis=1)) / np.sqrt(d)
        np.testing.assert_allclose(l1 - l0, shift, atol=1e-12)


def paper_masks(N, w_sink, w_recent):
    """Causal mask and sink mask of the appendix as additive N x N matrices (0 keep, -inf drop).

    Row i (0-based) of the sink mask keeps the first w_sink and the last w_recent positions of 0..i.
    """
    i = torch.arange(N).unsqueeze(1)
    j = torch.arange(N).unsqueeze(0)
    causal = j <= i
    kept = causal & ((j < w_sink) | (j > i - w_recent))
    neg = torch.full((N, N), float("-inf"), dtype=torch.float64)
    zero = torch.zeros((N, N), dtype=torch.float64)
    return torch.where(causal, zero, neg), torch.where(kept, zero, neg)


@pytest.mark.parametrize("ws,wr", [(0, 1), (1, 1), (2, 3), (4, 5), (0, 12), (12, 0), (3, 20)])
def test_brute_force_rows_of_the_masked_attention_matrix(ws, wr):
    """Every decode step T reproduces row T-1 of softmax(Q K^T + M) V built with library routines."""
    B, Hq, Hkv, d, N = 2, 4, 2, 8, 12
    G = Hq // Hkv
    Q, K, V = bf16_randn(B, Hq, N, d), bf16_randn(B, Hkv, N, d), bf16_randn(B, Hkv, N, d)
    Qt = torch.from_numpy(oracle.bf16_bits_to_f64(Q))
    Kt = torch.from_numpy(oracle.bf16_bits_to_f64(K)).repeat_interleave(G, dim=1)
    Vt = torch.from_numpy(oracle.bf16_bits_to_f64(V)).repeat_interleave(G, dim=1)
    logits = torch.matmul(Qt, Kt.transpose(-1, -2)) / np.sqrt(d)
    m_causal, m_sink = paper_masks(N, ws, wr)
    ref_full = torch.matmul(torch.softmax(logits + m_causal, dim=-1), Vt).numpy()
    ref_lazy = torch.matmul(torch.softmax(logits + m_sink, dim=-1), Vt).numpy()
    ref_lse_full = torch.logsumexp(logits + m_causal, dim=-1).numpy()
    ref_lse_lazy = torch.logsumexp(logits + m_sink, dim=-1).numpy()
    for T in range(1, N + 1):
        q = np.ascontiguousarray(Q[:, :, T - 1])
        Kc, Vc = np.ascontiguousarray(K[:, :, :T]), np.ascontiguousarray(V[:, :, :T])
        out, lse = oracle.decode_attn(q, Kc, Vc, oracle.MODE_FULL)
        np.testing.assert_allclose(out, ref_full[:, :, T - 1], atol=1e-13)
        np.testing.assert_allclose(lse, ref_lse_full[:, :, T - 1], atol=1e-13)
        out, lse = oracle.decode_attn(q, Kc, Vc, oracle.MODE_LAZY, ws, wr)
        np.testing.assert_allclose(out, ref_lazy[:, :, T - 1], atol=1e-13)
        np.testing.assert_allclose(lse, ref_lse_lazy[:, :, T - 1], atol=1e-13)


def test_grouped_query_heads_read_their_own_kv_head():
    """Head h must use KV head h // G: make each KV head's values a distinct constant."""
    B, Hq, Hkv, d, T = 1, 6, 3, 4, 9
    q, K = bf16_randn(B, Hq, d), bf16_randn(B, Hkv, T, d)
    Vv = np.zeros((B, Hkv, T, d), dtype=np.float32)
    for g in range(Hkv):
        Vv[:, g] = float(g + 1)
    out, _ = oracle.decode_attn(q, K, oracle.f32_to_bf16_bits(Vv), oracle.MODE_FULL)
    for h in range(Hq):
        np.testing.assert_allclose(out[0, h], float(h // 2 + 1), atol=1e-13)


def test_split_invariance_log_sum_exp_merge():
    """Attention over a union of disjoint key sets is the LSE-weighted merge of the parts."""
    B, Hq, Hkv, d, T = 1, 4, 2, 16, 37
    q, K, V = bf16_randn(B, Hq, d), bf16_randn(B, Hkv, T, d), bf16_randn(B, Hkv, T, d)
    whole, lse_whole = oracle.decode_attn(q, K, V, oracle.MODE_FULL)
    cuts = [0, 5, 6, 20, 37]
    outs, lses = [], []
    for a, b in zip(cuts[:-1], cuts[1:]):
        o, l = oracle.decode_attn(q, np.ascontiguousarray(K[:, :, a:b]), np.ascontiguousarray(V[:, :, a:b]), oracle.MODE_FULL)
        outs.append(o)
        lses.append(l)
    lses = np.stack(lses)                                   # [S,B,Hq]
    total = logsumexp(lses, axis=0)
    merged = sum(np.exp(l - total)[..., None] * o for l, o in zip(lses, outs))
    np.testing.assert_allclose(merged, whole, atol=1e-13)
    np.testing.assert_allclose(total, lse_whole, atol=1e-13)


def test_argument_errors():
    q, K, V = bf16_randn(1, 4, 8), bf16_randn(1, 2, 5, 8), bf16_randn(1, 2, 5, 8)
    with pytest.raises(ValueError):
        oracle.decode_attn(q, K, V, oracle.MODE_LAZY, 0, 0)          # empty attended set
    with pytest.raises(ValueError):
        oracle.decode_attn(bf16_randn(1, 3, 8), K, V, oracle.MODE_FULL)  # 3 heads over 2 KV heads
    with pytest.raises(ValueError):
        oracle.decode_attn(q, K, V, 7)
    with pytest.raises(TypeError):
        oracle.decode_attn(q.astype(np.float32), K, V, oracle.MODE_FULL)


def test_history_append_then_decode_matches_direct_call():
    B, Hq, Hkv, d = 1, 4, 2, 8
    hist = oracle.History(2, [False, True], w_sink=2, w_recent=3)
    Ks, Vs = [], []
    for step in range(7):
        k, v = bf16_randn(B, Hkv, 1, d), bf16_randn(B, Hkv, 1, d)
        Ks.append(k)
        Vs.append(v)
        for layer in range(2):
            hist.append(layer, k, v)
        q = bf16_randn(B, Hq, d)
        Kc, Vc = np.concatenate(Ks, 2), np.concatenate(Vs, 2)
        np.testing.assert_array_equal(hist.decode(0, q)[0], oracle.decode_attn(q, Kc, Vc, oracle.MODE_FULL)[0])
        np.testing.assert_array_equal(hist.decode(1, q)[0], oracle.decode_attn(q, Kc, Vc, oracle.MODE_LAZY, 2, 3)[0])
    assert hist.length(0) == hist.length(1) == 7
