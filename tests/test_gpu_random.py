"""Seeded random sweep of shapes through the C ABI against the oracle: decode (uniform and ragged batches, fused
and unfused steps, forced split sizes), prefill attention with both masks, and both forms of the lazy ratio.
The parametrised tests elsewhere pick edge cases by hand; this one draws the combinations nobody thought of."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL_LSE, TOL_OUT, TOL_RATIO, bits, f64, randn_bf16, say
from paper_2410_13846_amd import lt

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
EPS_P = 2.0 ** -8


def draw(rng):
    G = int(rng.integers(1, 9))
    Hkv = int(rng.integers(1, 4))
    ws = int(rng.integers(0, 9))
    wr = int(rng.integers(0 if ws > 0 else 1, 300))
    return dict(B=int(rng.integers(1, 6)), G=G, Hkv=Hkv, Hq=G * Hkv, ws=ws, wr=wr)


@pytest.mark.parametrize("case", range(24))
def test_random_decode(case):
    rng = np.random.default_rng(90000 + case)
    c = draw(rng)
    B, Hq, Hkv, ws, wr = c["B"], c["Hq"], c["Hkv"], c["ws"], c["wr"]
    ragged = bool(rng.integers(0, 2))
    n_max = int(rng.integers(1, 3000))
    lengths = [int(rng.integers(0, n_max + 1)) for _ in range(B)] if ragged else [n_max] * B
    if ragged:
        lengths[int(rng.integers(0, B))] = n_max
    steps = int(rng.integers(1, 4))
    say("random decode", case, c, "lengths", lengths, "steps", steps)
    cfg = lt.make_config(2, B, Hq, Hkv, 128, ws, wr, n_max + steps)
    is_lazy = [0, 1]
    ctx = lt.Context(cfg, is_lazy, DEV)
    if rng.integers(0, 2):
        kf, kl = 256 * int(rng.integers(1, 5)), 128 * int(rng.integers(1, 4))
        try:
            ctx.set_split(kf, kl)
        except lt.LtError:
            pass                                        # more splits than the workspace holds: keep the built-in choice
    hists = [oracle.History(2, is_lazy, ws, wr) for _ in range(B)]
    for layer in range(2):
        k, v = randn_bf16((B, Hkv, n_max, 128), 91000 + 10 * case + layer), randn_bf16((B, Hkv, n_max, 128), 92000 + 10 * case + layer)
        if ragged:
            ctx.append_kv_ragged(layer, k, v, lengths)
        else:
            ctx.append_kv(layer, k, v)
        for b in range(B):
            if lengths[b]:
                hists[b].append(layer, bits(k[b:b + 1, :, :lengths[b]]), bits(v[b:b + 1, :, :lengths[b]]))
    for step in range(steps):
        for layer in range(2):
            q = randn_bf16((B, Hq, 128), 93000 + 100 * case + 7 * step + layer, scale=float(rng.uniform(0.5, 3.0)))
            kn = randn_bf16((B, Hkv, 1, 128), 94000 + 100 * case + 7 * step + layer)
            vn = randn_bf16((B, Hkv, 1, 128), 95000 + 100 * case + 7 * step + layer)
            if rng.integers(0, 2):
                out, lse = ctx.decode_step(layer, q, kn, vn, want_lse=True)
            else:
                ctx.append_kv(layer, kn, vn)
                out, lse = ctx.decode_attn(layer, q, want_lse=True)
            for b in range(B):
                hists[b].append(layer, bits(kn[b:b + 1]), bits(vn[b:b + 1]))
                ref, ref_lse = hists[b].decode(layer, bits(q[b:b + 1]))
                assert np.abs(f64(out[b:b + 1]) - ref).max() <= TOL_OUT
                assert np.abs(f64(lse[b:b + 1]) - ref_lse).max() <= TOL_LSE
    ctx.close()


@pytest.mark.parametrize("case", range(16))
def test_random_prefill_and_ratios(case):
    rng = np.random.default_rng(96000 + case)
    c = draw(rng)
    B, Hq, Hkv, ws, wr = min(c["B"], 2), c["Hq"], c["Hkv"], c["ws"], c["wr"]
    n = int(rng.integers(1, 900))
    w = int(rng.integers(1, min(64, n) + 1))
    mode = int(rng.integers(0, 2))
    say("random prefill", case, dict(B=B, Hq=Hq, Hkv=Hkv, ws=ws, wr=wr, n=n, w=w, mode=mode))
    cfg = lt.make_config(1, B, Hq, Hkv, 128, ws, wr, n)
    q = randn_bf16((B, Hq, n, 128), 97000 + case, scale=float(rng.uniform(0.5, 2.5)))
    k, v = randn_bf16((B, Hkv, n, 128), 98000 + case), randn_bf16((B, Hkv, n, 128), 99000 + case)
    for mask, omode in ((lt.MASK_CAUSAL, oracle.MODE_FULL), (lt.MASK_STREAMING, oracle.MODE_LAZY)):
        out, lse = lt.prefill_attn(cfg, q, k, v, n, mask, out_dtype=torch.float32)
        ref, ref_lse, absw = oracle.prefill_attn(bits(q), bits(k), bits(v), omode, ws, wr, return_absw=True)
        assert (np.abs(f64(out) - ref) <= EPS_P * absw + 2e-5).all()
        assert np.abs(f64(lse) - ref_lse).max() <= 1e-4
        if mask == lt.MASK_CAUSAL:
            causal_lse = lse
    q_last = q[:, :, n - w:].contiguous()
    ref_rho, ref_seq, ref_r = oracle.lazy_ratio(bits(q_last), bits(k), ws, wr, recent_mode=mode)
    for mean, seq, rho in (lt.lazy_ratio(cfg, q_last, k, n, w, mode, want_rho=True),
                           lt.lazy_ratio_lse(cfg, q_last, k, n, w, causal_lse[:, :, n - w:], mode, want_rho=True)):
        assert np.abs(f64(rho) - ref_rho).max() <= TOL_RATIO
        assert np.abs(f64(seq) - ref_seq).max() <= TOL_RATIO
        assert abs(float(mean.cpu()[0]) - ref_r) <= TOL_RATIO
