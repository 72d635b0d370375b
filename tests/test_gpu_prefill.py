"""GPU parity: lt_prefill_attn (MFMA prefill attention with log-sum-exp output) and lt_lazy_ratio_lse (the
lazy ratio from that log-sum-exp, Table 1) against the CPU oracle, through the C ABI.

Tolerance of the attention output.  Logits, the softmax denominator and the accumulation are fp32, but the
probabilities enter the P V product rounded to bf16 (relative error <= 2^-8 each), so the error of an output
element is bounded by 2^-8 * sum_j p_j |V_j| -- a quantity the oracle returns per element (absw) -- plus the
fp32 terms; a bf16 output adds its own rounding, 2^-8 |out|.  The log-sum-exp is fp32 throughout."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL_LSE, TOL_RATIO, bits, f64, randn_bf16, say
from paper_2410_13846_amd import lt

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
EPS_P = 2.0 ** -8
TOL_PREFILL_LSE = 1e-4


def out_tolerance(absw, ref, out_dtype):
    tol = EPS_P * absw + 2e-5
    if out_dtype == torch.bfloat16:
        tol = tol + EPS_P * np.abs(ref)
    return tol


def check(B, Hq, Hkv, n, ws, wr, mask, seed, out_dtype=torch.float32, q_scale=1.0):
    say("prefill case", dict(B=B, Hq=Hq, Hkv=Hkv, n=n, ws=ws, wr=wr, mask=mask, seed=seed, out=str(out_dtype)))
    cfg = lt.make_config(1, B, Hq, Hkv, 128, ws, wr, max(n, 1))
    q = randn_bf16((B, Hq, n, 128), seed, scale=q_scale)
    k = randn_bf16((B, Hkv, n, 128), seed + 1)
    v = randn_bf16((B, Hkv, n, 128), seed + 2)
    out, lse = lt.prefill_attn(cfg, q, k, v, n, mask, out_dtype=out_dtype)
    torch.cuda.synchronize()
    mode = oracle.MODE_LAZY if mask == lt.MASK_STREAMING else oracle.MODE_FULL
    ref, ref_lse, absw = oracle.prefill_attn(bits(q), bits(k), bits(v), mode, ws, wr, return_absw=True)
    err = np.abs(f64(out.float()) - ref)
    tol = out_tolerance(absw, ref, out_dtype)
    worst = (err / tol).max()
    say("  max err", err.max(), "max err/tol", worst, "max lse err", np.abs(f64(lse) - ref_lse).max())
    assert worst <= 1.0
    assert np.abs(f64(lse) - ref_lse).max() <= TOL_PREFILL_LSE
    return out, lse


@pytest.mark.parametrize("n", [1, 2, 31, 32, 33, 64, 65, 127, 128, 200, 333, 1000])
def test_causal_prompt_lengths_span_tiles_and_ragged_tails(n):
    check(B=2, Hq=8, Hkv=2, n=n, ws=4, wr=60, mask=lt.MASK_CAUSAL, seed=5000 + n)


@pytest.mark.parametrize("group", [1, 2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("mask", [lt.MASK_CAUSAL, lt.MASK_STREAMING])
def test_every_query_group_size(group, mask):
    check(B=1, Hq=group, Hkv=1, n=300, ws=4, wr=100, mask=mask, seed=5100 + group)


@pytest.mark.parametrize("ws,wr", [(4, 20), (0, 33), (70, 100), (4, 1020), (3, 0), (0, 1), (64, 64), (4, 5000)])
@pytest.mark.parametrize("n", [700, 1500])
def test_streaming_windows(ws, wr, n):
    check(B=1, Hq=4, Hkv=1, n=n, ws=ws, wr=wr, mask=lt.MASK_STREAMING, seed=5200 + ws + wr + n)


@pytest.mark.parametrize("group", [2, 4, 5])
def test_bf16_output(group):
    check(B=1, Hq=2 * group, Hkv=2, n=450, ws=4, wr=60, mask=lt.MASK_CAUSAL, seed=5300 + group, out_dtype=torch.bfloat16)


def test_large_logits_move_the_softmax_reference():
    """Queries scaled so that row maxima keep growing by more than the rescale step."""
    check(B=1, Hq=4, Hkv=1, n=600, ws=4, wr=60, mask=lt.MASK_CAUSAL, seed=5400, q_scale=6.0)
    check(B=1, Hq=5, Hkv=1, n=600, ws=4, wr=60, mask=lt.MASK_STREAMING, seed=5401, q_scale=6.0)


def test_keys_and_values_read_in_place_from_the_cache():
    B, Hq, Hkv, n, cap = 2, 8, 2, 777, 1000
    cfg = lt.make_config(1, B, Hq, Hkv, 128, 4, 60, cap)
    ctx = lt.Context(cfg, [0], DEV)
    q = randn_bf16((B, Hq, n, 128), 5501)
    k, v = randn_bf16((B, Hkv, n, 128), 5502), randn_bf16((B, Hkv, n, 128), 5503)
    ctx.append_kv(0, k, v)
    kc, vc = ctx.layer_tensors(0)
    say("prefill in place: cache strides", kc.stride())
    out, lse = lt.prefill_attn(cfg, q, kc, vc, n, out_dtype=torch.float32)
    ref, ref_lse, absw = oracle.prefill_attn(bits(q), bits(k), bits(v), oracle.MODE_FULL, return_absw=True)
    assert (np.abs(f64(out) - ref) <= out_tolerance(absw, ref, torch.float32)).all()
    assert np.abs(f64(lse) - ref_lse).max() <= TOL_PREFILL_LSE
    ctx.close()


def test_prefill_errors():
    cfg = lt.make_config(1, 1, 4, 1, 128, 0, 0, 64)
    q, k = randn_bf16((1, 4, 64, 128), 1), randn_bf16((1, 1, 64, 128), 2)
    with pytest.raises(lt.LtError):
        lt.prefill_attn(cfg, q, k, k, 64, lt.MASK_STREAMING)          # empty window
    with pytest.raises(lt.LtError):
        lt.prefill_attn(cfg, q, k, k, 0)
    with pytest.raises(lt.LtError):
        lt.prefill_attn(cfg, q, k, k, 64, mask=7)


# ---- lazy ratio from the prefill's log-sum-exp -------------------------------------------------------------

def check_ratio_lse(B, Hq, Hkv, n, w, ws, wr, seed, mode=lt.RECENT_PER_QUERY, q_scale=2.0):
    say("ratio-from-lse case", dict(B=B, Hq=Hq, Hkv=Hkv, n=n, w=w, ws=ws, wr=wr, mode=mode, seed=seed))
    cfg = lt.make_config(1, B, Hq, Hkv, 128, ws, wr, n)
    q = randn_bf16((B, Hq, n, 128), seed, scale=q_scale)
    k, v = randn_bf16((B, Hkv, n, 128), seed + 1), randn_bf16((B, Hkv, n, 128), seed + 2)
    _, lse = lt.prefill_attn(cfg, q, k, v, n)
    q_last = q[:, :, n - w:].contiguous()
    mean, seq, rho = lt.lazy_ratio_lse(cfg, q_last, k, n, w, lse[:, :, n - w:], mode, want_rho=True)
    # (1) against the oracle fed the same fp32 log-sum-exp values
    log_rho, ref_seq, ref_r = oracle.lazy_ratio_from_lse(bits(q_last), bits(k), f64(lse[:, :, n - w:]), ws, wr, recent_mode=mode)
    assert np.abs(f64(rho) - np.exp(log_rho)).max() <= TOL_RATIO
    assert np.abs(f64(seq) - ref_seq).max() <= TOL_RATIO
    assert abs(float(mean.cpu()[0]) - ref_r) <= TOL_RATIO
    # (2) end to end against Eq. 1 computed by the oracle from scratch, and against the dense GPU form
    ref_rho, _, ref_r1 = oracle.lazy_ratio(bits(q_last), bits(k), ws, wr, recent_mode=mode)
    assert np.abs(f64(rho) - ref_rho).max() <= TOL_RATIO
    assert abs(float(mean.cpu()[0]) - ref_r1) <= TOL_RATIO
    mean_d, _, rho_d = lt.lazy_ratio(cfg, q_last, k, n, w, mode, want_rho=True)
    assert np.abs(f64(rho) - f64(rho_d)).max() <= TOL_RATIO


@pytest.mark.parametrize("n", [64, 65, 100, 257, 1000, 2600, 4133])
def test_ratio_from_lse_prompt_lengths(n):
    check_ratio_lse(B=2, Hq=8, Hkv=2, n=n, w=min(64, n), ws=4, wr=60, seed=6000 + n)


@pytest.mark.parametrize("ws,wr", [(0, 252), (4, 1020), (6, 2044), (4, 0), (0, 1), (40, 70), (130, 300)])
@pytest.mark.parametrize("mode", [lt.RECENT_PER_QUERY, lt.RECENT_FIXED])
def test_ratio_from_lse_windows_and_both_readings(ws, wr, mode):
    check_ratio_lse(B=1, Hq=4, Hkv=1, n=2600, w=64, ws=ws, wr=wr, seed=6100 + ws + wr, mode=mode)


@pytest.mark.parametrize("w", [1, 8, 31, 33, 64])
@pytest.mark.parametrize("group", [1, 5])
def test_ratio_from_lse_scored_queries_and_groups(w, group):
    check_ratio_lse(B=1, Hq=group, Hkv=1, n=900, w=w, ws=4, wr=124, seed=6200 + w + group)


# ---- chunked prefill: the queries are the last n_q of n positions ------------------------------------------

@pytest.mark.parametrize("n,n_q", [(300, 1), (300, 37), (300, 64), (1000, 333), (777, 776), (129, 65), (2000, 96)])
@pytest.mark.parametrize("mask", [lt.MASK_CAUSAL, lt.MASK_STREAMING])
def test_chunk_of_queries_equals_the_rows_of_the_whole_prompt(n, n_q, mask):
    B, Hq, Hkv, ws, wr = 2, 8, 2, 4, 100
    say("chunked prefill", dict(n=n, n_q=n_q, mask=mask))
    cfg = lt.make_config(1, B, Hq, Hkv, 128, ws, wr, n)
    q = randn_bf16((B, Hq, n, 128), 7000 + n + n_q)
    k, v = randn_bf16((B, Hkv, n, 128), 7001 + n), randn_bf16((B, Hkv, n, 128), 7002 + n)
    q_chunk = q[:, :, n - n_q:].contiguous()
    out, lse = lt.prefill_attn(cfg, q_chunk, k, v, n, mask, out_dtype=torch.float32)
    assert out.shape == (B, Hq, n_q, 128) and lse.shape == (B, Hq, n_q)
    mode = oracle.MODE_LAZY if mask == lt.MASK_STREAMING else oracle.MODE_FULL
    ref, ref_lse, absw = oracle.prefill_attn(bits(q), bits(k), bits(v), mode, ws, wr, return_absw=True)
    ref, ref_lse, absw = ref[:, :, n - n_q:], ref_lse[:, :, n - n_q:], absw[:, :, n - n_q:]
    assert (np.abs(f64(out) - ref) <= out_tolerance(absw, ref, torch.float32)).all()
    assert np.abs(f64(lse) - ref_lse).max() <= TOL_PREFILL_LSE


@pytest.mark.parametrize("group", [1, 3, 5, 8])
def test_chunked_prefill_through_the_cache_chunk_by_chunk(group):
    """A prompt prefilled in three chunks, keys and values read in place from the cache after each append: the
    concatenated rows equal the one-shot prefill's; the last chunk's log-sum-exp feeds the lazy ratio."""
    B, Hkv, ws, wr, w = 1, 2, 4, 60, 32
    Hq = group * Hkv
    chunks = [211, 64, 390]
    n = sum(chunks)
    cfg = lt.make_config(1, B, Hq, Hkv, 128, ws, wr, n)
    ctx = lt.Context(cfg, [0], DEV)
    q = randn_bf16((B, Hq, n, 128), 7100 + group, scale=2.0)
    k, v = randn_bf16((B, Hkv, n, 128), 7101 + group), randn_bf16((B, Hkv, n, 128), 7102 + group)
    kc, vc = ctx.layer_tensors(0)
    outs, lses, done = [], [], 0
    for m in chunks:
        ctx.append_kv(0, k[:, :, done:done + m].contiguous(), v[:, :, done:done + m].contiguous())
        done += m
        o, l = lt.prefill_attn(cfg, q[:, :, done - m:done].contiguous(), kc, vc, done, out_dtype=torch.float32)
        outs.append(o)
        lses.append(l)
    out, lse = torch.cat(outs, dim=2), torch.cat(lses, dim=2)
    ref, ref_lse, absw = oracle.prefill_attn(bits(q), bits(k), bits(v), oracle.MODE_FULL, return_absw=True)
    assert (np.abs(f64(out) - ref) <= out_tolerance(absw, ref, torch.float32)).all()
    assert np.abs(f64(lse) - ref_lse).max() <= TOL_PREFILL_LSE
    q_last = q[:, :, n - w:].contiguous()
    mean, _, rho = lt.lazy_ratio_lse(cfg, q_last, kc, n, w, lses[-1][:, :, chunks[-1] - w:], want_rho=True)
    ref_rho, _, ref_r = oracle.lazy_ratio(bits(q_last), bits(k), ws, wr)
    assert np.abs(f64(rho) - ref_rho).max() <= TOL_RATIO and abs(float(mean.cpu()[0]) - ref_r) <= TOL_RATIO
    ctx.close()


# ---- logits that climb or fall steadily: the softmax reference of the fast paths must follow ---------------

def ramp_inputs(B, Hq, Hkv, n, slope, seed):
    """Keys along one direction u with a coefficient that grows linearly with the position (plus noise), queries
    along u: the logit of key j is about slope * j / n natural units, so the row maximum keeps growing (slope > 0:
    the reference has to move again and again, early keys underflow) or the first keys dominate (slope < 0)."""
    g = torch.Generator(device=DEV).manual_seed(seed)
    u = torch.randn(128, generator=g, device=DEV)
    u = u / u.norm()
    coeff = torch.arange(n, device=DEV, dtype=torch.float32) / n * slope            # q.k * scale = coeff
    k = coeff[None, None, :, None] * u * (128 ** 0.25) + 0.05 * torch.randn(B, Hkv, n, 128, generator=g, device=DEV)
    q = (u * (128 ** 0.25)).expand(B, Hq, n, 128) + 0.05 * torch.randn(B, Hq, n, 128, generator=g, device=DEV)
    v = torch.randn(B, Hkv, n, 128, generator=g, device=DEV)
    return q.bfloat16().contiguous(), k.bfloat16().contiguous(), v.bfloat16().contiguous()


@pytest.mark.parametrize("slope", [400.0, 60.0, -60.0, -400.0])
@pytest.mark.parametrize("mask", [lt.MASK_CAUSAL, lt.MASK_STREAMING])
def test_steadily_growing_or_falling_logits(slope, mask):
    B, Hq, Hkv, n, ws, wr, w = 1, 4, 1, 1500, 4, 252, 64
    say("ramp case", dict(slope=slope, mask=mask))
    cfg = lt.make_config(1, B, Hq, Hkv, 128, ws, wr, n)
    q, k, v = ramp_inputs(B, Hq, Hkv, n, slope, 7300 + int(abs(slope)))
    out, lse = lt.prefill_attn(cfg, q, k, v, n, mask, out_dtype=torch.float32)
    mode = oracle.MODE_LAZY if mask == lt.MASK_STREAMING else oracle.MODE_FULL
    ref, ref_lse, absw = oracle.prefill_attn(bits(q), bits(k), bits(v), mode, ws, wr, return_absw=True)
    assert torch.isfinite(out).all() and torch.isfinite(lse).all()
    assert (np.abs(f64(out) - ref) / out_tolerance(absw, ref, torch.float32)).max() <= 1.0
    assert np.abs(f64(lse) - ref_lse).max() <= TOL_PREFILL_LSE * max(1.0, abs(slope) / 60.0)   # lse itself is of the order of slope
    if mask == lt.MASK_CAUSAL:                                   # both forms of the lazy ratio on the same prompt
        q_last = q[:, :, n - w:].contiguous()
        ref_rho, _, ref_r = oracle.lazy_ratio(bits(q_last), bits(k), ws, wr)
        mean_d, _, rho_d = lt.lazy_ratio(cfg, q_last, k, n, w, want_rho=True)
        assert np.abs(f64(rho_d) - ref_rho).max() <= TOL_RATIO and abs(float(mean_d.cpu()[0]) - ref_r) <= TOL_RATIO
        mean_l, _, rho_l = lt.lazy_ratio_lse(cfg, q_last, k, n, w, lse[:, :, n - w:], want_rho=True)
        log_rho, _, _ = oracle.lazy_ratio_from_lse(bits(q_last), bits(k), f64(lse[:, :, n - w:]), ws, wr)
        assert np.abs(f64(rho_l) - np.exp(log_rho)).max() <= TOL_RATIO
