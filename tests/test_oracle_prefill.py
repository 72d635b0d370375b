"""Pins for the prefill-attention oracle and for the lazy ratio taken from a supplied log-sum-exp
(CPU only).  Each test checks the oracle against something other than itself: the whole masked
softmax assembled from torch fp64 library routines with the appendix's masks, the decode oracle
on the truncated history (prefill row p == decoding the token at p), closed forms for uniform
keys, the first row, and the two self-contained forms of the lazy ratio."""
import numpy as np
import pytest
import torch

import oracle

RNG = np.random.default_rng(24101384)


def bf16_randn(*shape, scale=1.0):
    return oracle.f32_to_bf16_bits((RNG.standard_normal(shape) * scale).astype(np.float32))


def library_attention(Q, K, V, ws=None, wr=None):
    """softmax(Q K^T / sqrt(d) + M) V with torch fp64 routines; M from the appendix: causal (ws is None) or
    sink mask (kept: j <= i and (j < ws or j > i - wr)).  Also returns the row-wise logsumexp."""
    Qf = torch.from_numpy(oracle.bf16_bits_to_f64(Q))
    Kf = torch.from_numpy(oracle.bf16_bits_to_f64(K))
    Vf = torch.from_numpy(oracle.bf16_bits_to_f64(V))
    G = Q.shape[1] // K.shape[1]
    Kf, Vf = Kf.repeat_interleave(G, dim=1), Vf.repeat_interleave(G, dim=1)
    n, d = Q.shape[2], Q.shape[3]
    i = torch.arange(n)[:, None]
    j = torch.arange(n)[None, :]
    keep = j <= i
    if ws is not None:
        keep = keep & ((j < ws) | (j > i - wr))
    M = torch.where(keep, 0.0, float("-inf")).to(torch.float64)
    S = Qf @ Kf.transpose(-1, -2) / np.sqrt(d) + M
    return (torch.softmax(S, dim=-1) @ Vf).numpy(), torch.logsumexp(S, dim=-1).numpy(), torch.softmax(S, dim=-1).numpy(), Vf.numpy()


@pytest.mark.parametrize("B,Hq,Hkv,n,d", [(2, 4, 2, 37, 16), (1, 6, 2, 70, 8), (1, 2, 2, 5, 4)])
def test_causal_prefill_matches_library_masked_softmax(B, Hq, Hkv, n, d):
    Q, K, V = bf16_randn(B, Hq, n, d), bf16_randn(B, Hkv, n, d), bf16_randn(B, Hkv, n, d)
    out, lse, absw = oracle.prefill_attn(Q, K, V, oracle.MODE_FULL, return_absw=True)
    ref, ref_lse, P, Vf = library_attention(Q, K, V)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, ref_lse, rtol=0, atol=1e-12)
    np.testing.assert_allclose(absw, P @ np.abs(Vf), rtol=0, atol=1e-12)


@pytest.mark.parametrize("ws,wr", [(4, 8), (0, 5), (3, 0), (1, 1), (2, 100)])
def test_streaming_prefill_matches_library_sink_mask(ws, wr):
    B, Hq, Hkv, n, d = 1, 4, 2, 45, 8
    Q, K, V = bf16_randn(B, Hq, n, d), bf16_randn(B, Hkv, n, d), bf16_randn(B, Hkv, n, d)
    out, lse = oracle.prefill_attn(Q, K, V, oracle.MODE_LAZY, ws, wr)
    ref, ref_lse, _, _ = library_attention(Q, K, V, ws, wr)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, ref_lse, rtol=0, atol=1e-12)


@pytest.mark.parametrize("mode,ws,wr", [(oracle.MODE_FULL, 0, 0), (oracle.MODE_LAZY, 4, 6)])
def test_prefill_row_is_decode_of_the_truncated_history(mode, ws, wr):
    """Row p of the prefill == the decode step of token p over keys 0..p (the two stages compute the same
    attention; only the number of rows differs)."""
    B, Hq, Hkv, n, d = 2, 4, 2, 29, 16
    Q, K, V = bf16_randn(B, Hq, n, d), bf16_randn(B, Hkv, n, d), bf16_randn(B, Hkv, n, d)
    out, lse = oracle.prefill_attn(Q, K, V, mode, ws, wr)
    for p in (0, 1, 5, 10, 11, 28):
        o, l = oracle.decode_attn(Q[:, :, p], K[:, :, :p + 1], V[:, :, :p + 1], mode, ws, wr)
        np.testing.assert_allclose(out[:, :, p], o, rtol=0, atol=1e-13)
        np.testing.assert_allclose(lse[:, :, p], l, rtol=0, atol=1e-13)


def test_first_row_is_the_first_value_and_uniform_keys_give_prefix_means():
    B, Hq, Hkv, n, d = 1, 2, 1, 33, 8
    Q = bf16_randn(B, Hq, n, d)
    K = np.broadcast_to(bf16_randn(B, Hkv, 1, d), (B, Hkv, n, d)).copy()
    V = bf16_randn(B, Hkv, n, d)
    Vf = oracle.bf16_bits_to_f64(V)
    out, lse = oracle.prefill_attn(Q, K, V, oracle.MODE_FULL)
    np.testing.assert_array_equal(out[0, :, 0], np.stack([Vf[0, 0, 0]] * Hq))
    prefix = np.cumsum(Vf[0, 0], axis=0) / np.arange(1, n + 1)[:, None]
    np.testing.assert_allclose(out[0, 0], prefix, rtol=0, atol=1e-13)
    s = (oracle.bf16_bits_to_f64(Q)[0, 1] * oracle.bf16_bits_to_f64(K)[0, 0]).sum(-1) / np.sqrt(d)
    np.testing.assert_allclose(lse[0, 1], s + np.log(np.arange(1, n + 1)), rtol=0, atol=1e-12)
    # streaming rows: mean over the kept set only
    ws, wr = 2, 5
    lazy, _ = oracle.prefill_attn(Q, K, V, oracle.MODE_LAZY, ws, wr)
    for p in (0, 3, 7, 20, 32):
        keep = sorted(set(range(min(ws, p + 1))) | set(range(max(0, p - wr + 1), p + 1)))
        np.testing.assert_allclose(lazy[0, 0, p], Vf[0, 0, keep].mean(0), rtol=0, atol=1e-13)


def test_absw_bounds_the_output():
    B, Hq, Hkv, n, d = 1, 2, 2, 20, 8
    Q, K, V = bf16_randn(B, Hq, n, d), bf16_randn(B, Hkv, n, d), bf16_randn(B, Hkv, n, d)
    out, _, absw = oracle.prefill_attn(Q, K, V, oracle.MODE_FULL, return_absw=True)
    assert (np.abs(out) <= absw + 1e-15).all()
    assert (absw <= np.abs(oracle.bf16_bits_to_f64(V)).max() + 1e-15).all()


@pytest.mark.parametrize("recent_mode", [oracle.RECENT_PER_QUERY, oracle.RECENT_FIXED])
@pytest.mark.parametrize("n,w,ws,wr", [(90, 16, 4, 20), (64, 8, 0, 10), (40, 40, 2, 3), (30, 5, 4, 100)])
def test_ratio_from_supplied_lse_equals_both_self_contained_forms(recent_mode, n, w, ws, wr):
    """Feeding the prefill oracle's LSE of the last w rows into the window-only form reproduces Eq. 1 and
    Table 1's self-contained form."""
    B, Hq, Hkv, d = 2, 4, 2, 16
    Q, K, V = bf16_randn(B, Hq, n, d), bf16_randn(B, Hkv, n, d), bf16_randn(B, Hkv, n, d)
    _, lse = oracle.prefill_attn(Q, K, V, oracle.MODE_FULL)
    q_last = np.ascontiguousarray(Q[:, :, n - w:])
    log_rho, r_seq, r = oracle.lazy_ratio_from_lse(q_last, K, lse[:, :, n - w:], ws, wr, recent_mode=recent_mode)
    rho_ref, r_seq_ref, r_ref = oracle.lazy_ratio(q_last, K, ws, wr, recent_mode=recent_mode)
    log_ref, _, r_ref2 = oracle.lazy_ratio_lse(q_last, K, ws, wr, recent_mode=recent_mode)
    np.testing.assert_allclose(np.exp(log_rho), rho_ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(log_rho, log_ref, rtol=0, atol=1e-11)
    np.testing.assert_allclose(r_seq, r_seq_ref, rtol=0, atol=1e-12)
    assert abs(r - r_ref) <= 1e-12 and abs(r - r_ref2) <= 1e-12


def test_ratio_from_lse_brute_force_and_shifted_lse():
    """Brute force over the kept keys with numpy; an LSE shifted by c scales every rho by exp(-c)."""
    B, Hq, Hkv, d, n, w, ws, wr = 1, 2, 1, 8, 50, 6, 3, 7
    Q, K = bf16_randn(B, Hq, n, d), bf16_randn(B, Hkv, n, d)
    Qf, Kf = oracle.bf16_bits_to_f64(Q), oracle.bf16_bits_to_f64(K)
    lse = np.zeros((B, Hq, w))
    expect = np.zeros((B, Hq, w))
    for h in range(Hq):
        for t in range(w):
            p = n - w + t
            s = Kf[0, 0, :p + 1] @ Qf[0, h, p] / np.sqrt(d)
            lse[0, h, t] = np.log(np.exp(s).sum())
            keep = [j for j in range(p + 1) if j < ws or j > p - wr]
            expect[0, h, t] = np.exp(s[keep]).sum() / np.exp(s).sum()
    q_last = np.ascontiguousarray(Q[:, :, n - w:])
    log_rho, _, r = oracle.lazy_ratio_from_lse(q_last, K, lse, ws, wr)
    np.testing.assert_allclose(np.exp(log_rho), expect, rtol=0, atol=1e-13)
    assert abs(r - expect.mean()) <= 1e-13
    log_rho2, _, r2 = oracle.lazy_ratio_from_lse(q_last, K, lse + 0.5, ws, wr)
    np.testing.assert_allclose(log_rho2, log_rho - 0.5, rtol=0, atol=1e-13)
    assert abs(r2 - r * np.exp(-0.5)) <= 1e-13
