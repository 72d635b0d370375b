"""GPU parity: lt_lazy_ratio (MFMA scoring) and the score -> select chain against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL_RATIO, bits, f64, randn_bf16, say
from paper_2410_13846_amd import lt

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def check(B, Hq, Hkv, n, w, ws, wr, seed, mode=lt.RECENT_PER_QUERY, q_scale=2.0, k=None):
    say("ratio case", dict(B=B, Hq=Hq, Hkv=Hkv, n=n, w=w, ws=ws, wr=wr, mode=mode, seed=seed))
    cfg = lt.make_config(1, B, Hq, Hkv, 128, ws, wr, max(n, 1))
    q_last = randn_bf16((B, Hq, w, 128), seed, scale=q_scale)
    if k is None:
        k = randn_bf16((B, Hkv, n, 128), seed + 1)
    mean, seq, rho = lt.lazy_ratio(cfg, q_last, k, n, w, mode, want_rho=True)
    k_host = bits(k[:, :, :n].contiguous())
    ref_rho, ref_seq, ref_r = oracle.lazy_ratio(bits(q_last), k_host, ws, wr, recent_mode=mode)
    assert np.abs(f64(rho) - ref_rho).max() <= TOL_RATIO
    assert np.abs(f64(seq) - ref_seq).max() <= TOL_RATIO
    assert abs(float(mean.cpu()[0]) - ref_r) <= TOL_RATIO
    return ref_r


@pytest.mark.parametrize("n", [64, 65, 100, 257, 1000, 1024, 1500, 4133])
def test_prompt_lengths_span_tiles_chunks_and_ragged_tails(n):
    check(B=2, Hq=8, Hkv=2, n=n, w=min(64, n), ws=4, wr=60, seed=1000 + n)


@pytest.mark.parametrize("w", [1, 8, 16, 31, 32, 33, 64])
def test_number_of_scored_queries(w):
    check(B=1, Hq=8, Hkv=2, n=900, w=w, ws=4, wr=124, seed=1100 + w)


@pytest.mark.parametrize("group", [1, 2, 3, 4, 5, 6, 7, 8])
def test_every_query_group_size(group):
    check(B=1, Hq=group, Hkv=1, n=700, w=64, ws=4, wr=252, seed=1200 + group)


@pytest.mark.parametrize("group", [5, 6])
@pytest.mark.parametrize("n", [65, 1500, 4133])
@pytest.mark.parametrize("mode", [lt.RECENT_PER_QUERY, lt.RECENT_FIXED])
def test_ten_and_twelve_query_tiles_per_kv_head(group, n, mode):
    """Five and six heads of 64 scored queries: three query tiles per wavefront, two wavefronts sharing the keys."""
    check(B=2, Hq=2 * group, Hkv=2, n=n, w=64, ws=4, wr=252, seed=1250 + 10 * group + n, mode=mode)


@pytest.mark.parametrize("ws,wr", [(0, 252), (2, 508), (4, 1020), (6, 2044), (4, 0), (0, 1), (40, 70)])
@pytest.mark.parametrize("mode", [lt.RECENT_PER_QUERY, lt.RECENT_FIXED])
def test_window_shapes_and_both_readings_of_recent(ws, wr, mode):
    check(B=1, Hq=4, Hkv=1, n=2600, w=64, ws=ws, wr=wr, seed=1300 + ws + wr, mode=mode)


def test_ratio_is_one_when_the_window_covers_the_prompt():
    r = check(B=1, Hq=8, Hkv=2, n=1024, w=64, ws=4, wr=1020, seed=1400)
    assert abs(r - 1.0) < 1e-12


def test_keys_read_in_place_from_the_cache():
    """k may alias a full layer's cache block: strides of the [B][Hkv][capacity][128] layout."""
    B, Hq, Hkv, n, cap = 2, 8, 2, 1111, 1500
    cfg = lt.make_config(1, B, Hq, Hkv, 128, 4, 60, cap)
    ctx = lt.Context(cfg, [0], DEV)
    k, v = randn_bf16((B, Hkv, n, 128), 1501), randn_bf16((B, Hkv, n, 128), 1502)
    ctx.append_kv(0, k, v)
    k_cache, _ = ctx.layer_tensors(0)
    assert k_cache.stride(1) == cap * 128
    check(B, Hq, Hkv, n, 64, 4, 60, seed=1503, k=k_cache)
    ctx.close()


def test_peaked_attention_rows():
    """Large query norms make rows sharply peaked: exercises the running-max rescaling."""
    check(B=1, Hq=4, Hkv=1, n=3000, w=64, ws=4, wr=508, seed=1600, q_scale=8.0)


def test_score_then_select_recovers_planted_layers():
    import lt_workloads as W

    wl = W.WORKLOADS["llama3_8b_32k"].scaled(n_layers=8, batch=2, context=3072, w_recent=252, n_lazy=4)
    cfg = lt.make_config(wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, 128, wl.w_sink, wl.w_recent, wl.context)
    ratios, refs = [], []
    for layer in range(wl.n_layers):
        say("planted layer", layer)
        k, _ = W.prefill_kv(wl, layer, DEV)
        q_last = W.last_queries(wl, layer, DEV)
        mean, _, _ = lt.lazy_ratio(cfg, q_last, k, wl.context, wl.w_last)
        ratios.append(float(mean.cpu()[0]))
        refs.append(oracle.lazy_ratio(bits(q_last), bits(k), wl.w_sink, wl.w_recent)[2])
    assert np.abs(np.array(ratios) - np.array(refs)).max() <= TOL_RATIO
    ref_sorted = np.sort(refs)[::-1]
    assert ref_sorted[wl.n_lazy - 1] - ref_sorted[wl.n_lazy] > 100 * TOL_RATIO      # the planted gap is no tie
    got, _ = lt.select_lazy(ratios, wl.n_lazy)
    ref, _ = oracle.select_lazy(np.array(refs), wl.n_lazy)
    np.testing.assert_array_equal(got, ref)
    assert list(np.nonzero(got)[0]) == W.planted_lazy_layers(wl)
