"""GPU: one decode step of a whole stack (a launch per layer: fused append + attention + merge) recorded into a HIP
graph and replayed.  The library allocates nothing and clears its counters with kernels, so its launches can be
captured; a replay repeats the recorded step (same lengths, same slots) on whatever the input buffers hold, and every
replay is compared with the oracle, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL_LSE, TOL_OUT, bits, f64, randn_bf16, say
from paper_2410_13846_amd import lt

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("B,Hq,Hkv,n,ws,wr", [(2, 8, 2, 3000, 4, 252),        # several key ranges per (sequence, KV head)
                                              (16, 16, 8, 16390, 4, 1020)])   # long ranges: the shared tail and its counters
def test_replays_of_a_captured_decode_step_match_the_oracle(B, Hq, Hkv, n, ws, wr):
    mask = [0, 1, 0]
    L = len(mask)
    cfg = lt.make_config(L, B, Hq, Hkv, 128, ws, wr, n + 8)
    ctx = lt.Context(cfg, mask, DEV)
    prompt = []
    for layer in range(L):
        k, v = randn_bf16((B, Hkv, n, 128), 900 + layer), randn_bf16((B, Hkv, n, 128), 910 + layer)
        ctx.append_kv(layer, k, v)
        prompt.append((bits(k), bits(v)))
    q = torch.zeros((L, B, Hq, 128), dtype=torch.bfloat16, device=DEV)
    kn = torch.zeros((L, B, Hkv, 1, 128), dtype=torch.bfloat16, device=DEV)
    vn = torch.zeros_like(kn)
    out = torch.zeros((L, B, Hq, 128), dtype=torch.float32, device=DEV)
    lse = torch.zeros((L, B, Hq), dtype=torch.float32, device=DEV)

    def fill(seed):
        for layer in range(L):
            q[layer].copy_(randn_bf16((B, Hq, 128), seed + layer, scale=1.5))
            kn[layer].copy_(randn_bf16((B, Hkv, 1, 128), seed + 10 + layer))
            vn[layer].copy_(randn_bf16((B, Hkv, 1, 128), seed + 20 + layer))

    def check(what):
        torch.cuda.synchronize()
        for layer in range(L):
            hist = oracle.History(1, [mask[layer]], ws, wr)
            hist.append(0, *prompt[layer])
            hist.append(0, *first_token[layer])
            hist.append(0, bits(kn[layer]), bits(vn[layer]))
            ref, ref_lse = hist.decode(0, bits(q[layer]))
            assert np.abs(f64(out[layer]) - ref).max() <= TOL_OUT, (what, layer)
            assert np.abs(f64(lse[layer]) - ref_lse).max() <= TOL_LSE, (what, layer)

    # one eager step first: position n of every layer (the graph then records the step that writes position n + 1)
    fill(1000)
    for layer in range(L):
        ctx.decode_step(layer, q[layer], kn[layer], vn[layer], out=out[layer], lse=lse[layer])
    torch.cuda.synchronize()
    first_token = [(bits(kn[layer]), bits(vn[layer])) for layer in range(L)]

    say("capturing a decode step of", L, "layers, B", B, "n", n)
    fill(2000)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for layer in range(L):
            ctx.decode_step(layer, q[layer], kn[layer], vn[layer], out=out[layer], lse=lse[layer])
    assert ctx.layer_len(0)[0] == n + 2                       # the recorded step counts once on the host
    for rep in range(4):
        fill(3000 + 100 * rep)
        out.zero_()
        graph.replay()
        check("replay %d" % rep)
        # eager work of the same library between the replays: it shares the workspace and the counters
        ctx.decode_attn(0, q[0])
        torch.cuda.synchronize()
    ctx.close()
