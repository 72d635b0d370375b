"""Memory-safety check through the C ABI: every buffer a call may write (KV slab, decode workspace, outputs,
log-sum-exp, scoring workspace) sits between guard bands of a known pattern; after appends, decode steps
(uniform and ragged, fused and unfused, many splits), truncation, scoring and prefill attention at awkward
sizes the bands must be untouched and the results still match the oracle."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL_OUT, TOL_RATIO, bits, f64, randn_bf16, say
from paper_2410_13846_amd import lt

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
GUARD = 4096
PATTERN = 0xA5


def guarded(nbytes):
    """(whole tensor, view of nbytes in the middle), the whole filled with the pattern."""
    nbytes = (int(nbytes) + 255) // 256 * 256
    whole = torch.full((nbytes + 2 * GUARD,), PATTERN, dtype=torch.uint8, device=DEV)
    return whole, whole[GUARD: GUARD + nbytes]


def intact(whole):
    return bool((whole[:GUARD] == PATTERN).all().item()) and bool((whole[-GUARD:] == PATTERN).all().item())


@pytest.mark.parametrize("B,Hq,Hkv,n,ws,wr,split", [(3, 8, 2, 1237, 4, 60, None), (2, 5, 1, 2049, 0, 127, (256, 128)),
                                                   (1, 16, 2, 333, 6, 1020, None), (5, 4, 4, 64, 4, 28, None)])
def test_decode_calls_stay_inside_their_buffers(B, Hq, Hkv, n, ws, wr, split):
    say("guard case", dict(B=B, Hq=Hq, Hkv=Hkv, n=n, ws=ws, wr=wr, split=split))
    cfg = lt.make_config(2, B, Hq, Hkv, 128, ws, wr, n + 8)
    ctx = lt.Context(cfg, [0, 1], DEV, guard_bytes=GUARD)
    if split:
        ctx.set_split(*split)
    lib, stream = lt.load(), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    hist = oracle.History(2, [0, 1], ws, wr)
    for layer in range(2):
        k, v = randn_bf16((B, Hkv, n, 128), 70000 + layer), randn_bf16((B, Hkv, n, 128), 70010 + layer)
        ctx.append_kv(layer, k, v)
        hist.append(layer, bits(k), bits(v))
    out_all, out_mem = guarded(B * Hq * 128 * 4)
    lse_all, lse_mem = guarded(B * Hq * 4)
    out = out_mem[: B * Hq * 128 * 4].view(torch.float32).view(B, Hq, 128)
    lse = lse_mem[: B * Hq * 4].view(torch.float32).view(B, Hq)
    for step in range(4):
        for layer in range(2):
            q = randn_bf16((B, Hq, 128), 70100 + 7 * step + layer)
            kn, vn = randn_bf16((B, Hkv, 1, 128), 70200 + 7 * step + layer), randn_bf16((B, Hkv, 1, 128), 70300 + 7 * step + layer)
            if step % 2:
                ctx.append_kv(layer, kn, vn)
                st = lib.lt_decode_attn(ctx._h, layer, q.data_ptr(), out.data_ptr(), lse.data_ptr(), stream)
            else:
                st = lib.lt_decode_step(ctx._h, layer, q.data_ptr(), kn.data_ptr(), vn.data_ptr(), out.data_ptr(), lse.data_ptr(), stream)
            assert st == lt.OK
            hist.append(layer, bits(kn), bits(vn))
            ref, _ = hist.decode(layer, bits(q))
            assert np.abs(f64(out) - ref).max() <= TOL_OUT
    torch.cuda.synchronize()
    assert ctx.check_guards() and intact(out_all) and intact(lse_all)
    ctx.close()


def test_ragged_and_online_calls_stay_inside_their_buffers():
    B, Hq, Hkv, ws, wr = 4, 8, 2, 4, 60
    cfg = lt.make_config(2, B, Hq, Hkv, 128, ws, wr, 900)
    ctx = lt.Context(cfg, [0, 1], DEV, guard_bytes=GUARD)
    lengths = [0, 800, 33, 65]
    for layer in range(2):
        k, v = randn_bf16((B, Hkv, 800, 128), 71000 + layer), randn_bf16((B, Hkv, 800, 128), 71010 + layer)
        ctx.append_kv_ragged(layer, k, v, lengths)
    for step in range(3):
        for layer in range(2):
            ctx.decode_step(layer, randn_bf16((B, Hq, 128), 71100 + step), randn_bf16((B, Hkv, 1, 128), 71200 + step),
                            randn_bf16((B, Hkv, 1, 128), 71300 + step))
    torch.cuda.synchronize()
    assert ctx.check_guards()
    ctx.close()
    # online identification: slots taken on demand, a full layer reduced to its ring
    cfg = lt.make_config(3, 2, 8, 2, 128, ws, wr, 700)
    ctx = lt.Context(cfg, device=DEV, n_full_online=1, guard_bytes=GUARD)
    for layer in range(3):
        k, v = randn_bf16((2, 2, 650, 128), 72000 + layer), randn_bf16((2, 2, 650, 128), 72010 + layer)
        ctx.append_kv(layer, k, v)
        if layer < 2:
            ctx.truncate_layer(layer)
    for layer in range(3):
        ctx.decode_step(layer, randn_bf16((2, 8, 128), 72100), randn_bf16((2, 2, 1, 128), 72200), randn_bf16((2, 2, 1, 128), 72300))
    torch.cuda.synchronize()
    assert ctx.check_guards()
    ctx.close()


@pytest.mark.parametrize("B,Hq,Hkv,n,w,ws,wr", [(2, 8, 2, 1001, 64, 4, 60), (1, 5, 1, 130, 17, 0, 33), (3, 4, 4, 65, 64, 70, 100)])
def test_scoring_and_prefill_stay_inside_their_buffers(B, Hq, Hkv, n, w, ws, wr):
    say("guard case", dict(B=B, Hq=Hq, Hkv=Hkv, n=n, w=w, ws=ws, wr=wr))
    cfg = lt.make_config(1, B, Hq, Hkv, 128, ws, wr, n)
    lib, stream = lt.load(), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    q = randn_bf16((B, Hq, n, 128), 73000)
    k, v = randn_bf16((B, Hkv, n, 128), 73001), randn_bf16((B, Hkv, n, 128), 73002)
    bands = []
    for dtype_flag, esz in ((lt.OUT_F32, 4), (lt.OUT_BF16, 2)):
        for mask in (lt.MASK_CAUSAL, lt.MASK_STREAMING):
            out_all, out_mem = guarded(B * Hq * n * 128 * esz)
            lse_all, lse_mem = guarded(B * Hq * n * 4)
            st = lib.lt_prefill_attn(ctypes.byref(cfg), q.data_ptr(), k.data_ptr(), v.data_ptr(), k.stride(0), k.stride(1), k.stride(2),
                                     n, n, mask, dtype_flag, out_mem.data_ptr(), lse_mem.data_ptr(), stream)
            assert st == lt.OK
            bands += [out_all, lse_all]
    lse = lse_mem[: B * Hq * n * 4].view(torch.float32).view(B, Hq, n)       # the last one is a streaming-mask LSE: redo causal
    _, lse = lt.prefill_attn(cfg, q, k, v, n)
    q_last = q[:, :, n - w:].contiguous()
    ref_rho, _, ref_r = oracle.lazy_ratio(bits(q_last), bits(k), ws, wr)
    for which in ("dense", "lse"):
        need = lt.lazy_ratio_workspace_bytes(cfg, n, w) if which == "dense" else lt.lazy_ratio_lse_workspace_bytes(cfg, n, w)
        ws_all, ws_mem = guarded(need)
        rho_all, rho_mem = guarded(B * Hq * w * 4)
        seq_all, seq_mem = guarded(B * 4)
        mean_all, mean_mem = guarded(4)
        lse_rows = lse[:, :, n - w:]
        if which == "dense":
            st = lib.lt_lazy_ratio(ctypes.byref(cfg), q_last.data_ptr(), k.data_ptr(), k.stride(0), k.stride(1), k.stride(2), n, w, 0,
                                   ws_mem.data_ptr(), need, rho_mem.data_ptr(), seq_mem.data_ptr(), mean_mem.data_ptr(), stream)
        else:
            st = lib.lt_lazy_ratio_lse(ctypes.byref(cfg), q_last.data_ptr(), k.data_ptr(), k.stride(0), k.stride(1), k.stride(2), n, w, 0,
                                       lse_rows.data_ptr(), lse_rows.stride(0), lse_rows.stride(1), ws_mem.data_ptr(), need,
                                       rho_mem.data_ptr(), seq_mem.data_ptr(), mean_mem.data_ptr(), stream)
        assert st == lt.OK
        rho = rho_mem[: B * Hq * w * 4].view(torch.float32).view(B, Hq, w)
        assert np.abs(f64(rho) - ref_rho).max() <= TOL_RATIO
        assert abs(float(mean_mem[:4].view(torch.float32).cpu()[0]) - ref_r) <= TOL_RATIO
        bands += [ws_all, rho_all, seq_all, mean_all]
    torch.cuda.synchronize()
    assert all(intact(b) for b in bands)
