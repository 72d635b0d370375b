"""lt_lazy_ratio_static -- the lazy ratio for callers that cannot allocate -- against lt_lazy_ratio.

Both run the same kernels; the static variant keeps the partial results in the array that is part
of the library's code object instead of a caller's workspace.  Two calls in a row share that
array, the second with a smaller input, so leftovers of the first call must not leak into it.
Collected last on purpose: a failure here must not hide the tests before it."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL_RATIO, bits, f64, randn_bf16, say
from paper_2410_13846_amd import lt

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def both_ways(B, Hq, Hkv, n, w, ws, wr, seed, mode=lt.RECENT_PER_QUERY):
    cfg = lt.make_config(1, B, Hq, Hkv, 128, ws, wr, n)
    q_last = randn_bf16((B, Hq, w, 128), seed, DEV)
    k = randn_bf16((B, Hkv, n, 128), seed + 1, DEV)
    k[:, :, :ws] = (k[:, :, :ws].float() * 1.5).to(torch.bfloat16)           # some mass on the initial keys
    mean = torch.full((1,), -1.0, dtype=torch.float32, device=DEV)
    seq = torch.full((B,), -1.0, dtype=torch.float32, device=DEV)
    rho = torch.full((B, Hq, w), -1.0, dtype=torch.float32, device=DEV)
    say("static scratch: B", B, "Hq", Hq, "Hkv", Hkv, "n", n, "w", w, "window", ws, wr, "mode", mode)
    lt.lazy_ratio_static(cfg, q_last, k, n, w, mean, seq, rho, mode=mode)
    ref_mean, ref_seq, ref_rho = lt.lazy_ratio(cfg, q_last, k, n, w, mode=mode, want_rho=True)
    torch.cuda.synchronize()
    # same kernels, same order of operations: the two must agree to the last bit
    assert torch.equal(rho, ref_rho) and torch.equal(seq, ref_seq) and torch.equal(mean, ref_mean)
    return cfg, q_last, k, rho, seq, mean


def test_static_scratch_matches_the_workspace_form_on_two_calls_in_a_row():
    # a large problem first (many key ranges, the scratch array well used), then a small one in the same array
    cfg, q_last, k, rho, seq, mean = both_ways(B=4, Hq=32, Hkv=8, n=20000, w=64, ws=4, wr=2044, seed=101)
    cfg2, q2, k2, rho2, seq2, mean2 = both_ways(B=2, Hq=8, Hkv=2, n=777, w=16, ws=4, wr=60, seed=202)
    # and against the oracle, to the bar of the lazy ratio
    ref_rho, ref_seq, ref_r = oracle.lazy_ratio(bits(q2), bits(k2), 4, 60)
    assert np.abs(f64(rho2) - ref_rho).max() <= TOL_RATIO
    assert np.abs(f64(seq2) - ref_seq).max() <= TOL_RATIO
    assert abs(float(mean2.cpu()[0]) - ref_r) <= TOL_RATIO
    ref_rho, ref_seq, ref_r = oracle.lazy_ratio(bits(q_last[:1]), bits(k[:1]), 4, 2044)
    assert np.abs(f64(rho[:1]) - ref_rho).max() <= TOL_RATIO
    # a third call, larger again and in the other reading of the recent keys
    both_ways(B=3, Hq=10, Hkv=2, n=5001, w=33, ws=2, wr=508, seed=303, mode=lt.RECENT_FIXED)


def test_static_scratch_refuses_what_does_not_fit_and_allocates_nothing():
    lib = lt.load()
    big = lt.make_config(1, 512, 64, 8, 128, 4, 2044, 1 << 20)
    dummy = torch.zeros(4096, dtype=torch.bfloat16, device=DEV)
    out = torch.zeros(1, dtype=torch.float32, device=DEV)
    st = lib.lt_lazy_ratio_static(ctypes.byref(big), dummy.data_ptr(), dummy.data_ptr(), (1 << 20) * 128 * 8, (1 << 20) * 128, 128,
                                  1 << 20, 64, 0, None, None, out.data_ptr(), None)
    assert st == lt.ERR_CAPACITY                        # refused on the host; nothing was enqueued
    # device memory in use does not move across calls of the static form (the outputs are the caller's)
    cfg = lt.make_config(1, 2, 8, 2, 128, 4, 60, 3000)
    q_last = randn_bf16((2, 8, 32, 128), 7, DEV)
    k = randn_bf16((2, 2, 3000, 128), 8, DEV)
    mean = torch.empty(1, dtype=torch.float32, device=DEV)
    lt.lazy_ratio_static(cfg, q_last, k, 3000, 32, mean)
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    reserved_before = torch.cuda.memory_reserved()
    for _ in range(5):
        lt.lazy_ratio_static(cfg, q_last, k, 3000, 32, mean)
    torch.cuda.synchronize()
    free_after, _ = torch.cuda.mem_get_info()
    assert torch.cuda.memory_reserved() == reserved_before and free_after == free_before
