"""Pins for the lazy-ratio oracle (CPU only): Eq. 1 against closed forms, against the
log-sum-exp form of Table 1, against the decode oracle, against the streaming-attention
lemma of the appendix, and against rows of an explicit N x N causal softmax."""
import numpy as np
import pytest
import torch

import oracle

RNG = np.random.default_rng(1384620)


def bf16_randn(*shape, scale=1.0):
    return oracle.f32_to_bf16_bits((RNG.standard_normal(shape) * scale).astype(np.float32))


def window_positions(p, w_sink, w_recent):
    return sorted(set(range(min(w_sink, p + 1))) | set(range(max(0, p - w_recent + 1), p + 1)))


def fixed_positions(p, n, w_sink, w_recent):
    return sorted(j for j in (set(range(min(w_sink, n))) | set(range(max(0, n - w_recent), n))) if j <= p)


@pytest.mark.parametrize("mode", [oracle.RECENT_PER_QUERY, oracle.RECENT_FIXED])
@pytest.mark.parametrize("n,w,ws,wr", [(40, 8, 4, 6), (64, 16, 0, 9), (33, 33, 2, 5), (50, 1, 4, 0)])
def test_probability_form_equals_log_sum_exp_form(mode, n, w, ws, wr):
    B, Hq, Hkv, d = 2, 4, 2, 16
    q, K = bf16_randn(B, Hq, w, d, scale=2.0), bf16_randn(B, Hkv, n, d)
    rho, r_seq, r = oracle.lazy_ratio(q, K, ws, wr, recent_mode=mode)
    log_rho, r_seq2, r2 = oracle.lazy_ratio_lse(q, K, ws, wr, recent_mode=mode)
    if ws + wr > 0:
        np.testing.assert_allclose(np.exp(log_rho), rho, rtol=0, atol=1e-12)
    else:
        assert (rho == 0).all() and np.isneginf(log_rho).all()
    np.testing.assert_allclose(r_seq, r_seq2, atol=1e-12)
    assert abs(r - r2) < 1e-12


@pytest.mark.parametrize("n,w,ws,wr", [(100, 16, 4, 12), (64, 64, 4, 12), (30, 8, 0, 5), (30, 8, 6, 0), (90, 32, 4, 70)])
def test_uniform_keys_closed_form(n, w, ws, wr):
    """Equal keys make every causal row uniform: rho = |kept set| / (p + 1)."""
    B, Hq, Hkv, d = 1, 2, 1, 8
    q = bf16_randn(B, Hq, w, d)
    K = np.broadcast_to(bf16_randn(B, Hkv, 1, d), (B, Hkv, n, d)).copy()
    rho, r_seq, r = oracle.lazy_ratio(q, K, ws, wr)
    expect = np.array([min(p + 1, len(window_positions(p, ws, wr))) / (p + 1) for p in range(n - w, n)])
    # independent count of the kept set: sinks + recents - overlap
    count = np.array([min(ws, p + 1) + min(wr, p + 1) - max(0, min(ws, p + 1) - max(0, p - wr + 1)) for p in range(n - w, n)])
    np.testing.assert_array_equal(count, [len(window_positions(p, ws, wr)) for p in range(n - w, n)])
    np.testing.assert_allclose(rho[0, 0], expect, atol=1e-13)
    np.testing.assert_allclose(rho[0, 1], expect, atol=1e-13)
    assert abs(r - expect.mean()) < 1e-13


@pytest.mark.parametrize("n,ws,wr", [(10, 4, 6), (10, 4, 1020), (1024, 4, 1020), (3, 0, 3)])
def test_ratio_is_one_when_window_covers_the_prompt(n, ws, wr):
    B, Hq, Hkv, d = 1, 4, 2, 8
    w = min(n, 8)
    q, K = bf16_randn(B, Hq, w, d), bf16_randn(B, Hkv, n, d)
    rho, _, r = oracle.lazy_ratio(q, K, ws, wr)
    np.testing.assert_allclose(rho, 1.0, atol=1e-14)
    assert abs(r - 1.0) < 1e-14
    # one token more than the window and the ratio drops below 1 for the last query
    if n == ws + wr:
        K2 = bf16_randn(B, Hkv, n + 1, d)
        rho2, _, _ = oracle.lazy_ratio(q, K2, ws, wr)
        assert (rho2[..., -1] < 1.0).all()


def test_ratio_bounds_and_means():
    B, Hq, Hkv, d, n, w, ws, wr = 3, 4, 2, 16, 70, 16, 4, 10
    q, K = bf16_randn(B, Hq, w, d, scale=3.0), bf16_randn(B, Hkv, n, d)
    rho, r_seq, r = oracle.lazy_ratio(q, K, ws, wr)
    assert (rho >= 0).all() and (rho <= 1 + 1e-15).all()
    np.testing.assert_allclose(r_seq, rho.mean(axis=(1, 2)), atol=1e-15)
    assert abs(r - r_seq.mean()) < 1e-15
    # sequences are independent: scoring one sequence alone gives its r_seq
    _, r1, _ = oracle.lazy_ratio(q[1:2], K[1:2], ws, wr)
    np.testing.assert_allclose(r1[0], r_seq[1], atol=1e-15)


def test_dominant_key_inside_or_outside_the_window():
    B, Hq, Hkv, d, n, w, ws, wr = 1, 1, 1, 16, 80, 4, 4, 10
    q = oracle.f32_to_bf16_bits(np.full((B, Hq, w, d), 4.0, dtype=np.float32))
    for j, expect in [(2, 1.0), (75, 1.0), (40, 0.0)]:          # sink, recent for all 4 queries, middle
        K = np.zeros((B, Hkv, n, d), dtype=np.uint16)
        K[0, 0, j] = oracle.f32_to_bf16_bits(np.full(d, 4.0, dtype=np.float32))
        rho, _, r = oracle.lazy_ratio(q, K, ws, wr)
        np.testing.assert_allclose(rho, expect, atol=1e-24)


def test_shift_invariance():
    B, Hq, Hkv, d, n, w = 1, 4, 2, 8, 30, 6
    q = oracle.f32_to_bf16_bits(RNG.integers(-2, 3, size=(B, Hq, w, d)).astype(np.float32))
    Kv = RNG.integers(-3, 4, size=(B, Hkv, n, d)).astype(np.float32)
    delta = RNG.integers(-2, 3, size=(B, Hkv, 1, d)).astype(np.float32)
    a = oracle.lazy_ratio(q, oracle.f32_to_bf16_bits(Kv), 2, 5)[0]
    b = oracle.lazy_ratio(q, oracle.f32_to_bf16_bits(Kv + delta), 2, 5)[0]
    np.testing.assert_allclose(a, b, atol=1e-13)


@pytest.mark.parametrize("ws,wr", [(4, 6), (0, 3), (5, 0), (2, 40)])
def test_ratio_is_the_mass_decode_attention_keeps(ws, wr):
    """rho of the query at p equals exp(lse_streaming - lse_full) of the decode oracle at T = p + 1."""
    B, Hq, Hkv, d, n, w = 2, 4, 2, 16, 30, 5
    q, K = bf16_randn(B, Hq, w, d, scale=2.0), bf16_randn(B, Hkv, n, d)
    V = bf16_randn(B, Hkv, n, d)
    rho, _, _ = oracle.lazy_ratio(q, K, ws, wr)
    for t in range(w):
        T = n - w + t + 1
        qt = np.ascontiguousarray(q[:, :, t])
        Kc, Vc = np.ascontiguousarray(K[:, :, :T]), np.ascontiguousarray(V[:, :, :T])
        _, lse_full = oracle.decode_attn(qt, Kc, Vc, oracle.MODE_FULL)
        _, lse_lazy = oracle.decode_attn(qt, Kc, Vc, oracle.MODE_LAZY, ws, wr)
        np.testing.assert_allclose(rho[:, :, t], np.exp(lse_lazy - lse_full), atol=1e-13)


def test_streaming_attention_lemma_ties_ratio_to_decode_outputs():
    """Appendix lemma on dropping keys: |s1 - s1~|_1 = 1 - rho and |o_stream - o_full|_2 <= 2 (1 - rho) max|V_j|_2."""
    B, Hq, Hkv, d, n, ws, wr = 2, 4, 2, 16, 60, 4, 12
    q1, K, V = bf16_randn(B, Hq, 1, d, scale=2.0), bf16_randn(B, Hkv, n, d), bf16_randn(B, Hkv, n, d)
    rho, _, _ = oracle.lazy_ratio(q1, K, ws, wr)
    qd = np.ascontiguousarray(q1[:, :, 0])
    o_full, _, p_full = oracle.decode_attn(qd, K, V, oracle.MODE_FULL, return_probs=True)
    o_lazy, _, p_lazy = oracle.decode_attn(qd, K, V, oracle.MODE_LAZY, ws, wr, return_probs=True)
    keep = np.zeros(n, dtype=bool)
    keep[window_positions(n - 1, ws, wr)] = True
    dropped_mass = p_full[..., ~keep].sum(-1)
    np.testing.assert_allclose(dropped_mass, 1.0 - rho[:, :, 0], atol=1e-13)
    l1 = np.abs(p_full[..., keep] - p_lazy[..., keep]).sum(-1)
    np.testing.assert_allclose(l1, 1.0 - rho[:, :, 0], atol=1e-13)
    vmax = np.linalg.norm(oracle.bf16_bits_to_f64(V), axis=-1).max(axis=-1)      # [B,Hkv]
    bound = 2.0 * (1.0 - rho[:, :, 0]) * np.repeat(vmax, Hq // Hkv, axis=1)
    assert (np.linalg.norm(o_lazy - o_full, axis=-1) <= bound + 1e-13).all()
    assert (1.0 - rho > 1e-3).all()          # the bound is not vacuous on this input


@pytest.mark.parametrize("mode", [oracle.RECENT_PER_QUERY, oracle.RECENT_FIXED])
@pytest.mark.parametrize("ws,wr", [(0, 1), (1, 2), (2, 5), (4, 3), (0, 12), (3, 20)])
def test_brute_force_rows_of_the_causal_softmax(mode, ws, wr):
    B, Hq, Hkv, d, N, w = 2, 4, 2, 8, 12, 5
    G = Hq // Hkv
    Q, K = bf16_randn(B, Hq, N, d, scale=2.0), bf16_randn(B, Hkv, N, d)
    Qt = torch.from_numpy(oracle.bf16_bits_to_f64(Q))
    Kt = torch.from_numpy(oracle.bf16_bits_to_f64(K)).repeat_interleave(G, dim=1)
    logits = torch.matmul(Qt, Kt.transpose(-1, -2)) / np.sqrt(d)
    causal = torch.tril(torch.ones(N, N, dtype=torch.bool))
    A = torch.softmax(logits.masked_fill(~causal, float("-inf")), dim=-1).numpy()     # [B,Hq,N,N]
    expect = np.zeros((B, Hq, w))
    for t in range(w):
        p = N - w + t
        cols = window_positions(p, ws, wr) if mode == oracle.RECENT_PER_QUERY else fixed_positions(p, N, ws, wr)
        expect[:, :, t] = A[:, :, p, cols].sum(-1)
    q_last = np.ascontiguousarray(Q[:, :, N - w:])
    rho, r_seq, r = oracle.lazy_ratio(q_last, K, ws, wr, recent_mode=mode)
    np.testing.assert_allclose(rho, expect, atol=1e-13)
    assert abs(r - expect.mean()) < 1e-13


def test_fixed_and_per_query_windows_agree_on_the_last_query_only():
    B, Hq, Hkv, d, n, w, ws, wr = 1, 2, 1, 8, 40, 6, 2, 8
    q, K = bf16_randn(B, Hq, w, d, scale=2.0), bf16_randn(B, Hkv, n, d)
    a = oracle.lazy_ratio(q, K, ws, wr, recent_mode=oracle.RECENT_PER_QUERY)[0]
    b = oracle.lazy_ratio(q, K, ws, wr, recent_mode=oracle.RECENT_FIXED)[0]
    np.testing.assert_allclose(a[..., -1], b[..., -1], atol=1e-15)
    assert np.abs(a[..., 0] - b[..., 0]).max() > 1e-6


def test_hyperparameter_grid_of_the_paper(hyperparams):
    """The ablation grid runs through the oracle at a reduced prompt length and keeps its invariants."""
    B, Hq, Hkv, d = 1, 2, 1, 8
    for wr in hyperparams["w_recent_grid"]:
        for ws in hyperparams["w_sink_grid"]:
            n = wr + ws + 40
            w = 8
            q, K = bf16_randn(B, Hq, w, d), bf16_randn(B, Hkv, n, d)
            rho, _, r = oracle.lazy_ratio(q, K, ws, wr)
            assert 0.0 < r < 1.0
            rho_big, _, _ = oracle.lazy_ratio(q, K, ws + 1, wr + 1)
            assert (rho_big >= rho - 1e-15).all()          # a larger kept set never loses mass


def test_argument_errors():
    q, K = bf16_randn(1, 4, 8, 8), bf16_randn(1, 2, 5, 8)
    with pytest.raises(ValueError):
        oracle.lazy_ratio(q, K, 4, 4)                    # w_last larger than the prompt
    with pytest.raises(ValueError):
        oracle.lazy_ratio(bf16_randn(1, 4, 2, 8), K, 4, 4, recent_mode=5)
