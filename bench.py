#!/usr/bin/env python3
"""Benchmark of the LightTransfer hot path on one MI355X.

A step is one decode step of the whole hybrid stack: for every layer, lt_decode_step = append of
the new token's K/V + attention over that layer's cache + merge of the key-axis splits, in one
launch (full layers: the whole growing cache; lazy layers: the sink + recent ring).  Before the timed region the stack is set up the way the
method prescribes: lt_lazy_ratio scores every layer on the last w_last prompt queries,
lt_select_lazy picks the lazy layers, and the prompt K/V are appended; those calls are timed
separately and reported under "scoring".  All inputs are seeded synthetic tensors resident in
HBM before timing starts.

Prints one JSON line: tokens/s (value), the roofline of the dominant kernel (split decode over
full layers, HBM-bound) and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HEADLINE_WORKLOAD = "llama31_8b_128k_b16"   # 128K context x batch 16: 141.7 GB of K/V read per decode step
SECOND_WORKLOAD = "llama3_8b_32k"
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=32)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--workload", default=None,
                    help="one configuration; default: the headline run = %s (the largest that fits one GPU), with %s "
                         "and the batch-1 128K speedup measurement as extra keys" % (HEADLINE_WORKLOAD, SECOND_WORKLOAD))
    ap.add_argument("--n-lazy", type=int, default=None, help="override the number of lazy layers")
    ap.add_argument("--keys-full", type=int, default=0, help="keys per workgroup in full layers (0 = built-in)")
    ap.add_argument("--keys-lazy", type=int, default=0)
    ap.add_argument("--q-heads", type=int, default=None,
                    help="override the number of query heads (heads per KV head = this / the workload's KV heads, up to 8)")
    ap.add_argument("--decode-path", choices=("auto", "vector", "matrix"), default="auto",
                    help="force one of the two decode kernels (lt_set_decode_path)")
    ap.add_argument("--no-shared-tail", action="store_true",
                    help="every key in a fixed place (lt_set_shared_tail off): bit-reproducible outputs, for comparison")
    ap.add_argument("--no-speedup", action="store_true", help="skip the all-full comparison run")
    ap.add_argument("--headline-only", action="store_true",
                    help="with the default workload: skip the extra batch-1 and 32K x batch 8 runs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile-pass", action="store_true", help="skip the second pass that times kernels with HIP events")
    ap.add_argument("--prefill", action="store_true",
                    help="time lt_prefill_attn (causal and streaming masks) and lt_lazy_ratio_lse on layers of the workload")
    ap.add_argument("--context", type=int, default=None, help="override the workload's prompt length")
    ap.add_argument("--grid", action="store_true",
                    help="decode and scoring times over the paper's ablation grid of w_recent, w_sink and w_last (Table 7)")
    ap.add_argument("--scoring-only", action="store_true", help="run and report only the lazy-ratio scoring of every layer")
    ap.add_argument("--online", action="store_true",
                    help="(implied when the layers' full caches would not all fit the device) set the stack up the paper's way: prefill layer by layer, score each layer from its cache, push "
                         "it into the priority queue and reduce the popped layer's cache at once (peak P+1 full caches)")
    ap.add_argument("--growth", action="store_true",
                    help="long-generation curve: fixed lazy mask, decode from the prompt length up to the workload's "
                         "final length, timing --steps decode steps at each doubling of the history (the tokens in "
                         "between are bulk-appended); reports tokens/s against generated length")
    ap.add_argument("--whole-run", action="store_true",
                    help="with --growth: decode every step of the generation (prompt to final length) instead of sampling "
                         "the curve; decode inputs cycle through a pool of --steps pre-generated steps")
    ap.add_argument("--paged", type=int, default=0, metavar="PAGE_TOKENS",
                    help="compare the stack with its full layers stored in pages of this many tokens (shuffled block table) "
                         "against the contiguous stack; prints its own JSON line")
    ap.add_argument("--paged-table", choices=("shuffled", "sequential"), default="shuffled",
                    help="with --paged: pages handed out in a random order (a pool in use for a while) or in sequence")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (outside the timed region) so that hardware-counter "
                         "runs have a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    return ap.parse_args()


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Stack:
    """A hybrid stack with its decode inputs pre-generated on the device."""

    shared_tail = True                  # --no-shared-tail clears it for every stack of the run
    decode_path = 0                     # --decode-path: lt.DECODE_VECTOR / lt.DECODE_MATRIX for every stack of the run

    def __init__(self, lt, W, wl, is_lazy, total_steps, dev, keys_full=0, keys_lazy=0, online=False, page_tokens=0,
                 shuffled=True):
        import numpy as np
        import torch

        self.lt, self.wl, self.dev = lt, wl, dev
        self.cfg = lt.make_config(wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.w_sink,
                                  wl.w_recent, wl.context + total_steps)
        if online:
            # prefill -> score in place -> push -> reduce the popped layer, one layer at a time
            self.ctx = lt.Context(self.cfg, device=dev, n_full_online=wl.n_layers - wl.n_lazy)
            queue = lt.SelectQueue(wl.n_layers - wl.n_lazy)
            ws = torch.empty(max(lt.lazy_ratio_workspace_bytes(self.cfg, wl.context, wl.w_last), 256), dtype=torch.uint8, device=dev)
            self.ratios, self.score_ms, mask = [], [], [0] * wl.n_layers
            for layer in range(wl.n_layers):
                k, v = W.prefill_kv(wl, layer, dev)
                q_last = W.last_queries(wl, layer, dev)
                self.ctx.append_kv(layer, k, v)
                del k, v
                k_cache, _ = self.ctx.layer_tensors(layer)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                mean, _, _ = lt.lazy_ratio(self.cfg, q_last, k_cache, wl.context, wl.w_last, workspace=ws)
                e1.record()
                e1.synchronize()
                self.score_ms.append(e0.elapsed_time(e1))
                self.ratios.append(float(mean.cpu()[0]))
                popped = queue.push(self.ratios[-1], layer)
                if popped >= 0:
                    self.ctx.truncate_layer(popped)
                    mask[popped] = 1
            queue.close()
            self.is_lazy = mask
        else:
            self.is_lazy = list(map(int, is_lazy))
            if page_tokens:
                # every sequence gets the pages of its whole run up front, scattered over the pool
                max_pages = -(-(wl.context + total_steps) // page_tokens)
                self.ctx = lt.Context(self.cfg, self.is_lazy, dev, paged=(page_tokens, wl.batch * max_pages))
                order = np.random.default_rng(7).permutation(wl.batch * max_pages) if shuffled else np.arange(wl.batch * max_pages)
                table = order.astype(np.int32).reshape(wl.batch, max_pages)
                self.ctx.set_block_table(table)
            else:
                self.ctx = lt.Context(self.cfg, self.is_lazy, dev)
            for layer in range(wl.n_layers):
                k, v = W.prefill_kv(wl, layer, dev)
                self.ctx.append_kv(layer, k, v)
                del k, v
        if keys_full or keys_lazy:
            self.ctx.set_split(keys_full, keys_lazy)
        if not Stack.shared_tail:
            self.ctx.set_shared_tail(False)
        if Stack.decode_path:
            self.ctx.set_decode_path(Stack.decode_path)
        self.q, self.k, self.v = [], [], []
        for layer in range(wl.n_layers):
            q, k, v = W.decode_qkv_block(wl, layer, 0, total_steps, dev)
            self.q.append(q)
            self.k.append(k)
            self.v.append(v)
        self.out = torch.empty((wl.n_layers, wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.float32, device=dev)
        self.step = 0
        torch.cuda.synchronize()
        # raw pointers so the timed loop is ctypes calls only
        self._lib = lt.load()
        self._h = self.ctx._h
        self._stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        esz_q = wl.batch * wl.n_q_heads * wl.head_dim * 2
        esz_kv = wl.batch * wl.n_kv_heads * wl.head_dim * 2
        self._ptrs = [(self.q[l].data_ptr(), esz_q, self.k[l].data_ptr(), self.v[l].data_ptr(), esz_kv,
                       self.out[l].data_ptr()) for l in range(wl.n_layers)]

    def run(self, n_steps):
        lib, h, stream = self._lib, self._h, self._stream
        for _ in range(n_steps):
            s = self.step
            for layer, (qp, qs, kp, vp, kvs, op) in enumerate(self._ptrs):
                st = lib.lt_decode_step(h, layer, qp + s * qs, kp + s * kvs, vp + s * kvs, op, None, stream)
                if st != 0:
                    raise self.lt.LtError(st, "lt_decode_step")
            self.step += 1

    def tokens_now(self):
        return self.wl.context + self.step

    def close(self):
        self.ctx.close()


def timed(stack, n_steps):
    import torch

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    stack.run(n_steps)
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def score_layers(lt, W, wl, dev):
    """lt_lazy_ratio on every layer (prompt regenerated per layer), timed with events on the launch stream."""
    import torch

    cfg = lt.make_config(wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.w_sink, wl.w_recent, wl.context)
    ws = torch.empty(max(lt.lazy_ratio_workspace_bytes(cfg, wl.context, wl.w_last), 256), dtype=torch.uint8, device=dev)
    ratios, ms = [], []
    for layer in range(wl.n_layers):
        k, _ = W.prefill_kv(wl, layer, dev)
        q_last = W.last_queries(wl, layer, dev)
        if layer == 0:                                     # warm-up launch, not timed
            lt.lazy_ratio(cfg, q_last, k, wl.context, wl.w_last, workspace=ws)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        mean, _, _ = lt.lazy_ratio(cfg, q_last, k, wl.context, wl.w_last, workspace=ws)
        e1.record()
        e1.synchronize()
        ms.append(e0.elapsed_time(e1))
        ratios.append(float(mean.cpu()[0]))
        del k, q_last
    return ratios, ms


def cpu_baseline(W, wl, stack, is_lazy):
    """The oracle, as it stands, on a bounded sample of the workload at its real lengths: one decode step of sequence 0
    of one full and one lazy layer (all host threads, then one thread), and one lazy-ratio scoring call of sequence 0 of
    one layer over the whole prompt (all threads on every head; one thread on the query heads of one KV head)."""
    import numpy as np
    import torch

    import oracle

    def time_call(fn, budget_s, min_reps, max_reps):
        reps, t0 = 0, time.perf_counter()
        while reps < min_reps or (time.perf_counter() - t0 < budget_s and reps < max_reps):
            res = fn()
            reps += 1
        return (time.perf_counter() - t0) / reps, res

    threads = oracle.num_threads()
    T = stack.tokens_now()
    per_kind, per_kind_1 = {}, {}
    score = None
    for kind in (0, 1):
        layers = [l for l in range(wl.n_layers) if is_lazy[l] == kind]
        if not layers:
            continue
        layer = layers[0]
        # rebuild sequence 0's whole history of this layer on the host (the oracle keeps every token)
        k, v = W.prefill_kv(wl, layer, stack.dev)
        K = np.concatenate([W.bf16_bits(k[:1]), W.bf16_bits(stack.k[layer][: stack.step, :1, :, 0].permute(1, 2, 0, 3).contiguous())], axis=2)
        V = np.concatenate([W.bf16_bits(v[:1]), W.bf16_bits(stack.v[layer][: stack.step, :1, :, 0].permute(1, 2, 0, 3).contiguous())], axis=2)
        if score is None:
            q_last = W.bf16_bits(W.last_queries(wl, layer, stack.dev)[:1].contiguous())
            k_prompt = W.bf16_bits(k[:1])
        del k, v
        q = W.bf16_bits(stack.q[layer][stack.step - 1, :1].contiguous())
        mode = oracle.MODE_LAZY if kind else oracle.MODE_FULL
        oracle.decode_attn(q, K, V, mode, wl.w_sink, wl.w_recent)            # touch memory once
        per_kind[kind], (ref, _) = time_call(lambda: oracle.decode_attn(q, K, V, mode, wl.w_sink, wl.w_recent), 4.0, 3, 50)
        oracle.set_num_threads(1)
        try:
            per_kind_1[kind], _ = time_call(lambda: oracle.decode_attn(q, K, V, mode, wl.w_sink, wl.w_recent), 3.0, 1, 20)
        finally:
            oracle.set_num_threads(threads)
        err = float(np.abs(stack.out[layer, 0].cpu().numpy().astype(np.float64) - ref[0]).max())
        log("cpu_baseline: layer %d (%s) T=%d: %.4f s per sequence-step on %d threads, %.4f s on one, max |gpu - oracle| = %.3g"
            % (layer, "lazy" if kind else "full", T, per_kind[kind], threads, per_kind_1[kind], err))
        if err > 2e-3:
            raise RuntimeError("GPU output of the timed run disagrees with the oracle: %g" % err)
        if score is None:
            # Eq. 1 at the real prompt length: every head of sequence 0 on all threads; the heads of KV head 0 on one thread
            t_all, (_, _, r_all) = time_call(lambda: oracle.lazy_ratio(q_last, k_prompt, wl.w_sink, wl.w_recent), 0.0, 1, 1)
            G = wl.group
            q_one, k_one = np.ascontiguousarray(q_last[:, :G]), np.ascontiguousarray(k_prompt[:, :1])
            oracle.set_num_threads(1)
            try:
                t_one, _ = time_call(lambda: oracle.lazy_ratio(q_one, k_one, wl.w_sink, wl.w_recent), 0.0, 1, 1)
            finally:
                oracle.set_num_threads(threads)
            score = {"layer": layer, "ratio": r_all, "s_per_layer_sequence": t_all, "s_single": t_one * wl.n_kv_heads}
            log("cpu_baseline: lazy ratio of layer %d, sequence 0, n=%d: %.2f s on %d threads; one thread %.2f s for one KV head's "
                "query heads (x %d = %.1f s per layer and sequence)" % (layer, wl.context, t_all, threads, t_one, wl.n_kv_heads, score["s_single"]))
            del q_last, k_prompt, q_one, k_one
    n_lazy = sum(is_lazy)
    per_token = (wl.n_layers - n_lazy) * per_kind.get(0, 0.0) + n_lazy * per_kind.get(1, 0.0)
    per_token_1 = (wl.n_layers - n_lazy) * per_kind_1.get(0, 0.0) + n_lazy * per_kind_1.get(1, 0.0)
    step_bytes = W.kv_bytes_per_step(wl, is_lazy, T) / wl.batch
    return {
        "value": 1.0 / per_token, "unit": "tokens/s", "cores": threads, "kind": "oracle",
        "sample": "sequence 0 of one full and one lazy layer, one decode step each at T=%d, repeated >=3 times; "
                  "extrapolated linearly to %d layers x %d sequences" % (T, wl.n_layers, wl.batch),
        "kv_gbs": step_bytes / per_token / 1e9,
        "single_thread": {"value": 1.0 / per_token_1, "unit": "tokens/s", "cores": 1, "kv_gbs": step_bytes / per_token_1 / 1e9,
                          "sample": "the same two calls on one OpenMP thread, extrapolated the same way"},
        "scoring": {"unit": "s per layer (all %d sequences)" % wl.batch, "cores": threads,
                    "value": score["s_per_layer_sequence"] * wl.batch,
                    "single_thread_value": score["s_single"] * wl.batch,
                    "sample": "Eq. 1 on sequence 0 of layer %d over the whole prompt (n=%d, w_last=%d): all %d query heads on %d "
                              "threads, measured once; on one thread the %d query heads of KV head 0, times %d KV heads; both "
                              "extrapolated linearly to %d sequences" % (score["layer"], wl.context, wl.w_last, wl.n_q_heads, threads,
                                                                         wl.group, wl.n_kv_heads, wl.batch)} if score else None,
    }


def growth_curve(args, lt, W, wl, dev):
    """tokens/s against history length for a fixed (pre-selected) lazy mask, LightTransfer-Train style."""
    import numpy as np
    import torch

    final = wl.context + wl.decode_steps
    is_lazy = [1 if l in W.planted_lazy_layers(wl) else 0 for l in range(wl.n_layers)]
    cfg = lt.make_config(wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.w_sink, wl.w_recent, final)
    ctx = lt.Context(cfg, is_lazy, dev)
    if args.keys_full or args.keys_lazy:
        ctx.set_split(args.keys_full, args.keys_lazy)
    lib, h = lt.load(), ctx._h
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    K = args.steps
    q = W.randn_bf16((K, wl.n_layers, wl.batch, wl.n_q_heads, wl.head_dim), W.seed_for(wl, 0, stream=21), dev)
    kn = W.randn_bf16((K, wl.n_layers, wl.batch, wl.n_kv_heads, wl.head_dim), W.seed_for(wl, 0, stream=22), dev)
    vn = W.randn_bf16((K, wl.n_layers, wl.batch, wl.n_kv_heads, wl.head_dim), W.seed_for(wl, 0, stream=23), dev)
    out = torch.empty((wl.n_layers, wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.float32, device=dev)
    qs, ks = q[0, 0].numel() * 2, kn[0, 0].numel() * 2
    filler = W.randn_bf16((wl.batch, wl.n_kv_heads, 4096, wl.head_dim), W.seed_for(wl, 0, stream=24), dev)

    def grow_to(total):
        for layer in range(wl.n_layers):
            have = ctx.layer_len(layer)[0]
            while have < total:
                n = min(4096, total - have)
                ctx.append_kv(layer, filler[:, :, :n].contiguous() if n < 4096 else filler, filler[:, :, :n].contiguous() if n < 4096 else filler)
                have += n

    def decode(n_steps):
        for s in range(n_steps):
            for layer in range(wl.n_layers):
                off_q, off_k = (s * wl.n_layers + layer) * qs, (s * wl.n_layers + layer) * ks
                st = lib.lt_decode_step(h, layer, q.data_ptr() + off_q, kn.data_ptr() + off_k, vn.data_ptr() + off_k,
                                        out[layer].data_ptr(), None, stream)
                if st != 0:
                    raise lt.LtError(st, "lt_decode_step")

    if args.whole_run:
        # the whole generation, step by step: every launch sees the history length it would see in a real run
        grow_to(wl.context)
        decode(min(K, 4))
        torch.cuda.synchronize()
        T_start = ctx.layer_len(0)[0]
        bins, edges = [], []
        T = 2048
        while T < final:
            edges.append(T)
            T *= 2
        edges.append(final)
        t_begin = time.perf_counter()
        done, T_now = 0, T_start
        for edge in edges:
            n_steps = edge - T_now
            if n_steps <= 0:
                continue
            t0 = time.perf_counter()
            left = n_steps
            while left > 0:                            # the input pool is cycled; values do not matter for the timing
                chunk = min(left, K)
                decode(chunk)
                left -= chunk
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            bins.append({"history_from": T_now, "history_to": edge, "steps": n_steps, "seconds": dt,
                         "ms_per_step": dt / n_steps * 1e3, "tokens_per_s": wl.batch * n_steps / dt})
            log("T %6d..%6d: %6d steps in %.2f s, %.3f ms/step, %.0f tokens/s" % (T_now, edge, n_steps, dt, dt / n_steps * 1e3, wl.batch * n_steps / dt))
            done += n_steps
            T_now = edge
        total = time.perf_counter() - t_begin
        ctx.close()
        total_bytes = sum(W.kv_bytes_per_step(wl, is_lazy, t) for t in range(T_start + 1, final + 1, 64)) * 64.0
        return {"metric": "whole generation at a fixed lazy mask: decode tokens/s", "value": wl.batch * done / total, "unit": "tokens/s",
                "n_gpus": 1, "steps": done, "seconds": total, "launches": done * wl.n_layers, "higher_is_better": True, "data": "synthetic",
                "kv_gbs": total_bytes / total / 1e9, "kv_hbm_frac": total_bytes / total / 1e9 / HBM_PEAK_GBS,
                "config": {"workload": wl.name, "layers": wl.n_layers, "lazy_layers": int(sum(is_lazy)), "batch": wl.batch,
                           "q_heads": wl.n_q_heads, "kv_heads": wl.n_kv_heads, "w_sink": wl.w_sink, "w_recent": wl.w_recent,
                           "history_first_step": T_start + 1, "history_last_step": final},
                "bins": bins}

    points, T = [], wl.context
    targets = []
    while T < final:
        targets.append(T)
        T *= 2
    targets.append(final - K)
    for T in targets:
        grow_to(T)
        torch.cuda.synchronize()
        if not points:
            decode(min(K, 4))                          # warm-up launches; they also lengthen the history a little
            torch.cuda.synchronize()
        T0 = ctx.layer_len(0)[0]
        t0 = time.perf_counter()
        decode(K)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        T_mid = T0 + (K + 1) / 2
        nbytes = W.kv_bytes_per_step(wl, is_lazy, int(T_mid))
        points.append({"tokens_in_history": int(T_mid), "ms_per_step": dt / K * 1e3, "tokens_per_s": wl.batch * K / dt,
                       "kv_gbs": nbytes / (dt / K) / 1e9, "ceiling_tokens_per_s_at_8TBs": wl.batch / (nbytes / 8e12)})
        log("T=%6d: %.3f ms/step, %.0f tokens/s, %.0f GB/s" % (T_mid, dt / K * 1e3, wl.batch * K / dt, nbytes / (dt / K) / 1e9))
    ctx.close()
    return {"metric": "decode tokens/s against history length, fixed lazy mask", "unit": "tokens/s", "n_gpus": 1,
            "steps": K, "data": "synthetic", "config": {"workload": wl.name, "layers": wl.n_layers, "lazy_layers": int(sum(is_lazy)),
            "batch": wl.batch, "q_heads": wl.n_q_heads, "kv_heads": wl.n_kv_heads, "w_sink": wl.w_sink, "w_recent": wl.w_recent},
            "curve": points}


def prefill_bench(args, lt, W, wl, dev):
    """Prefill attention of single layers at the workload's prompt shape, the lazy ratio from its log-sum-exp, and the
    dense lazy ratio beside it.  Times are HIP-event times on the launch stream (torch's current stream)."""
    import numpy as np
    import torch
    cfg = lt.make_config(wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.w_sink, wl.w_recent, wl.context)
    n, w = wl.context, min(wl.w_last, wl.context)
    layers = sorted(set(W.planted_lazy_layers(wl)[:1] + [l for l in range(wl.n_layers) if l not in W.planted_lazy_layers(wl)][:1]))
    ws_lse = torch.empty(max(lt.lazy_ratio_lse_workspace_bytes(cfg, n, w), 256), dtype=torch.uint8, device=dev)
    ws_dense = torch.empty(max(lt.lazy_ratio_workspace_bytes(cfg, n, w), 256), dtype=torch.uint8, device=dev)

    def timed_ms(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    rows = []
    for layer in layers:
        q = W.prefill_queries(wl, layer, dev)
        k, v = W.prefill_kv(wl, layer, dev)
        q_last = q[:, :, n - w:].contiguous()
        out, lse = lt.prefill_attn(cfg, q, k, v, n)
        res = {}
        def causal():
            res["o"] = lt.prefill_attn(cfg, q, k, v, n)
        def streaming():
            res["s"] = lt.prefill_attn(cfg, q, k, v, n, lt.MASK_STREAMING)
        def from_lse():
            res["r"] = lt.lazy_ratio_lse(cfg, q_last, k, n, w, lse[:, :, n - w:], workspace=ws_lse)
        def dense():
            res["d"] = lt.lazy_ratio(cfg, q_last, k, n, w, workspace=ws_dense)
        reps = max(1, min(args.steps, 4))
        t_causal, t_stream = timed_ms(causal, reps), timed_ms(streaming, reps)
        t_lse, t_dense = timed_ms(from_lse, 20), timed_ms(dense, 20)
        r_lse, r_dense = float(res["r"][0].cpu()[0]), float(res["d"][0].cpu()[0])
        pairs = n * (n + 1) / 2.0
        window = wl.w_sink + wl.w_recent
        pairs_stream = pairs if n <= window else window * (window + 1) / 2.0 + (n - window) * float(window)
        flops = 4.0 * wl.batch * wl.n_q_heads * wl.head_dim * pairs
        flops_stream = 4.0 * wl.batch * wl.n_q_heads * wl.head_dim * pairs_stream
        row = {"layer": layer, "causal_ms": t_causal, "causal_tflops": flops / t_causal / 1e9,
               "causal_mfma_frac": flops / t_causal / 1e9 / MFMA_BF16_PEAK_TFLOPS,
               "streaming_ms": t_stream, "streaming_tflops": flops_stream / t_stream / 1e9,
               "ratio_from_lse_ms": t_lse, "ratio_dense_ms": t_dense, "ratio_from_lse": r_lse, "ratio_dense": r_dense,
               "ratio_abs_diff": abs(r_lse - r_dense),
               # identification cost relative to the prefill attention it rides on (the paper quotes 0.0058 at 4K to
               # 0.0014 at 32K of whole-model prefill throughput on A100)
               "ratio_from_lse_over_prefill": t_lse / t_causal, "ratio_dense_over_prefill": t_dense / t_causal}
        log("layer %d: causal prefill %.2f ms (%.0f TFLOP/s), streaming %.2f ms (%.0f TFLOP/s), ratio from LSE %.3f ms vs dense %.3f ms, "
            "r %.6f vs %.6f" % (layer, t_causal, row["causal_tflops"], t_stream, row["streaming_tflops"], t_lse, t_dense, r_lse, r_dense))
        if abs(r_lse - r_dense) > 1e-4:
            raise RuntimeError("the two forms of the lazy ratio disagree")
        rows.append(row)
        del q, k, v, out, lse, res
        torch.cuda.empty_cache()
    mean_ms = float(np.mean([r["causal_ms"] for r in rows]))
    flops = 4.0 * wl.batch * wl.n_q_heads * wl.head_dim * n * (n + 1) / 2.0
    achieved = flops / mean_ms / 1e9
    return {"metric": "prefill attention and lazy ratio from its log-sum-exp, per layer", "value": mean_ms, "unit": "ms per layer (causal prefill attention)",
            "higher_is_better": False, "n_gpus": 1, "data": "synthetic",
            "dtype": "bf16 operands, fp32 accumulate", "config": {"workload": wl.name, "batch": wl.batch, "q_heads": wl.n_q_heads,
            "kv_heads": wl.n_kv_heads, "context": n, "w_sink": wl.w_sink, "w_recent": wl.w_recent, "w_last": w},
            "roofline": {"bound": "mfma", "kernel": "lt_prefill_attn_kernel<%d, *> (causal mask)" % wl.group, "achieved": achieved,
                         "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                         "flops_per_launch": flops, "avg_launch_us": mean_ms * 1e3},
            "layers": rows}


def paged_bench(args, lt, W, wl, dev):
    """The same stack and steps with contiguous and with paged full layers: ms per step and per-launch times."""
    import torch

    is_lazy = [0] * wl.n_layers
    for layer in W.planted_lazy_layers(wl)[: wl.n_lazy]:
        is_lazy[layer] = 1
    K, Wm = args.steps, args.warmup
    rows = {}
    # both stacks are allocated before anything is timed: memory taken after a large free has been seen to run the
    # scattered (paged) reads 4 % slower than memory taken by a fresh process, which is what a server's pool is
    stacks = {name: Stack(lt, W, wl, is_lazy, Wm + 2 * K, dev, args.keys_full, args.keys_lazy, page_tokens=page,
                          shuffled=args.paged_table == "shuffled")
              for name, page in (("paged", args.paged), ("contiguous", 0))}
    for name in ("contiguous", "paged"):
        stack = stacks[name]
        stack.run(Wm)
        elapsed = timed(stack, K)
        stack.ctx.profile_enable(True)
        T_first = stack.tokens_now() + 1
        timed(stack, K)
        T_mean = 0.5 * (T_first + stack.tokens_now())
        stack.ctx.profile_enable(False)
        n_full, ms_full = stack.ctx.profile_read(lt.KERNEL_DECODE_FULL)
        n_lazy, ms_lazy = stack.ctx.profile_read(lt.KERNEL_DECODE_LAZY)
        launch_bytes = wl.batch * ((2 * wl.n_kv_heads * wl.head_dim * 2) * T_mean + wl.n_q_heads * wl.head_dim * (2 + 4)
                                   + wl.n_kv_heads * wl.head_dim * 2 * 2)
        full_us = ms_full / max(n_full, 1) * 1e3
        rows[name] = {"ms_per_step": elapsed / K * 1e3, "tokens_per_s": wl.batch * K / elapsed, "full_launch_us": full_us,
                      "full_launch_gbs": launch_bytes / full_us / 1e3, "full_launch_hbm_frac": launch_bytes / full_us / 1e3 / HBM_PEAK_GBS,
                      "lazy_launch_us": (ms_lazy / n_lazy * 1e3) if n_lazy else None, "kv_slab_gb": stack.ctx.kv_slab.numel() / 1e9}
        log("%s: %.3f ms/step, full-layer launch %.1f us (%.0f GB/s)" % (name, rows[name]["ms_per_step"], full_us, rows[name]["full_launch_gbs"]))
    for stack in stacks.values():
        stack.close()
    del stacks
    torch.cuda.empty_cache()
    return {"metric": "decode step, paged against contiguous full layers", "n_gpus": 1, "steps": K, "warmup": Wm, "data": "synthetic",
            "dtype": "bf16 storage, fp32 accumulate",
            "config": {"workload": wl.name, "page_tokens": args.paged, "batch": wl.batch, "context": wl.context, "lazy_layers": wl.n_lazy,
                       "block_table": "a random permutation of the pool" if args.paged_table == "shuffled" else "pages in sequence"},
            "contiguous": rows["contiguous"], "paged": rows["paged"],
            "paged_over_contiguous_ms": rows["paged"]["ms_per_step"] / rows["contiguous"]["ms_per_step"]}


def window_grid(args, lt, W, wl, dev):
    """The ablation grid of Table 7 as a cost sweep: decode time per step of the hybrid stack (planted mask) for every
    w_recent at w_sink = 4 and every w_sink at w_recent = 1020, and scoring time of one layer for every w_last."""
    import numpy as np
    import torch
    K = min(args.steps, 32)
    is_lazy = [1 if l in W.planted_lazy_layers(wl) else 0 for l in range(wl.n_layers)]
    points = [(4, wr) for wr in (252, 508, 1020, 2044)] + [(ws, 1020) for ws in (0, 2, 6)]
    decode = []
    for ws, wr in points:
        w = wl.scaled(w_sink=ws, w_recent=wr, bias="none")
        stack = Stack(lt, W, w, is_lazy, 2 * K + 4, dev)
        stack.run(4)
        elapsed = timed(stack, K)
        stack.ctx.profile_enable(True)
        timed(stack, K)
        stack.ctx.profile_enable(False)
        n_lazy_launches, lazy_ms = stack.ctx.profile_read(lt.KERNEL_DECODE_LAZY)
        nbytes = W.kv_bytes_per_step(w, is_lazy, stack.tokens_now())
        decode.append({"w_sink": ws, "w_recent": wr, "ms_per_step": elapsed / K * 1e3, "tokens_per_s": w.batch * K / elapsed,
                       "kv_gbs": nbytes / (elapsed / K) / 1e9, "lazy_launch_us": lazy_ms / max(n_lazy_launches, 1) * 1e3})
        log("w_sink %d w_recent %4d: %.3f ms/step, %.0f tokens/s, lazy launch %.1f us" % (
            ws, wr, elapsed / K * 1e3, w.batch * K / elapsed, decode[-1]["lazy_launch_us"]))
        stack.close()
        del stack
        torch.cuda.empty_cache()
    scoring = []
    layer = W.planted_lazy_layers(wl)[0]
    k, _ = W.prefill_kv(wl, layer, dev)
    for w_last in (8, 16, 32, 64):
        cfg = lt.make_config(wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.w_sink, wl.w_recent, wl.context)
        q_last = W.last_queries(wl, layer, dev, w_last)
        ws_buf = torch.empty(max(lt.lazy_ratio_workspace_bytes(cfg, wl.context, w_last), 256), dtype=torch.uint8, device=dev)
        lt.lazy_ratio(cfg, q_last, k, wl.context, w_last, workspace=ws_buf)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            mean, _, _ = lt.lazy_ratio(cfg, q_last, k, wl.context, w_last, workspace=ws_buf)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 10
        scoring.append({"w_last": w_last, "ms_per_layer": ms, "ratio": float(mean.cpu()[0])})
        log("w_last %2d: %.3f ms per layer, r = %.4f" % (w_last, ms, scoring[-1]["ratio"]))
    return {"metric": "decode ms/step and scoring ms/layer over the window grid", "n_gpus": 1, "steps": K, "data": "synthetic",
            "config": {"workload": wl.name, "layers": wl.n_layers, "lazy_layers": int(sum(is_lazy)), "batch": wl.batch,
                       "context": wl.context}, "decode": decode, "scoring": scoring}


def needs_online(lt, W, wl, total_steps):
    """True when the caches of all layers at full size (what a caller holds before it knows which layers are lazy) would
    not fit the device: then the stack is set up the paper's way, identifying and reducing layer by layer."""
    import torch

    cfg = lt.make_config(wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.w_sink, wl.w_recent, wl.context + total_steps)
    return not all_full_fits(lt, cfg, wl)


def all_full_fits(lt, cfg, wl):
    """Room for every layer at full size plus the seeded prompt of one layer on its way into the cache (K and V in
    bf16, and the fp32 draws they are rounded from)."""
    import torch

    all_full = lt.kv_bytes(cfg, [0] * wl.n_layers)
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    return all_full + 4 * (all_full // wl.n_layers) < free


def decode_bench(args, lt, W, wl, dev, K, Wm, want_cpu, want_speedup, want_profile, scoring_only=False):
    """One configuration: identification (timed apart), K timed decode steps of the whole stack after Wm warm-up steps,
    the event-timed pass for the dominant kernel's roofline, the oracle on host cores, the all-full comparison.
    Returns the JSON line as a dict."""
    import numpy as np
    import torch

    log("workload %s: L=%d B=%d Hq=%d Hkv=%d n=%d window=%d+%d lazy=%d" % (
        wl.name, wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.context, wl.w_sink, wl.w_recent, wl.n_lazy))
    # ---- identification: score every layer, select ------------------------------------------------
    total_steps = Wm + K + (K if want_profile else 0)
    online = args.online or needs_online(lt, W, wl, total_steps)
    t0 = time.perf_counter()
    stack = None
    if online and not scoring_only:
        stack = Stack(lt, W, wl, None, total_steps, dev, args.keys_full, args.keys_lazy, online=True)
        ratios, score_ms, is_lazy, select_us = stack.ratios, stack.score_ms, np.asarray(stack.is_lazy, np.uint8), 0.0
        closed_form, _ = lt.select_lazy(ratios, wl.n_lazy)
        if list(closed_form) != list(is_lazy):
            raise RuntimeError("the queue procedure and the closed form disagree")
    else:
        ratios, score_ms = score_layers(lt, W, wl, dev)
        t_sel = time.perf_counter()
        is_lazy, _ = lt.select_lazy(ratios, wl.n_lazy)
        select_us = (time.perf_counter() - t_sel) * 1e6
    log("scoring + selection: %.1f s wall, lazy layers %s" % (time.perf_counter() - t0, [int(i) for i in np.nonzero(is_lazy)[0]]))
    if wl.bias == "planted" and list(np.nonzero(is_lazy)[0]) != W.planted_lazy_layers(wl):
        raise RuntimeError("selection did not recover the planted lazy layers")
    score_flops = 2.0 * wl.batch * wl.n_q_heads * wl.w_last * wl.context * wl.head_dim
    score_bytes = wl.batch * wl.n_kv_heads * wl.context * wl.head_dim * 2.0
    med_ms = float(np.median(score_ms))
    scoring = {
        "ms_per_layer": med_ms, "tflops": score_flops / med_ms / 1e9, "mfma_frac": score_flops / med_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS,
        "k_gbs": score_bytes / med_ms / 1e6, "hbm_frac": score_bytes / med_ms / 1e6 / HBM_PEAK_GBS, "select_us": select_us,
        "w_last": wl.w_last, "ratio_min": min(ratios), "ratio_max": max(ratios), "online_queue": bool(online and not scoring_only),
    }
    if scoring_only:
        return {"metric": "lazy-ratio scoring, per layer", "config": {"workload": wl.name}, "scoring": scoring}

    # ---- decode -----------------------------------------------------------------------------------------
    if stack is None:
        stack = Stack(lt, W, wl, is_lazy, total_steps, dev, args.keys_full, args.keys_lazy)
    log("stack ready: KV slab %.2f GB" % (stack.ctx.kv_slab.numel() / 1e9))
    stack.run(Wm)
    T_first = stack.tokens_now() + 1
    elapsed = timed(stack, K)
    T_last = stack.tokens_now()
    ms_per_step = elapsed / K * 1e3
    tokens_per_s = wl.batch * K / elapsed
    T_mean = 0.5 * (T_first + T_last)
    step_bytes = W.kv_bytes_per_step(wl, is_lazy, int(T_mean))
    log("timed %d steps: %.3f ms/step, %.1f tokens/s, %.1f GB/s of KV" % (K, ms_per_step, tokens_per_s, step_bytes / ms_per_step / 1e6))

    # ---- roofline of the dominant kernel: split decode over one full layer -----------------------------------
    roofline = None
    if want_profile:
        stack.ctx.profile_enable(True)
        Tp_first = stack.tokens_now() + 1
        elapsed_p = timed(stack, K)
        Tp_mean = 0.5 * (Tp_first + stack.tokens_now())
        stack.ctx.profile_enable(False)
        kernel = lt.KERNEL_DECODE_FULL if sum(is_lazy) < wl.n_layers else lt.KERNEL_DECODE_LAZY
        launches, total_ms = stack.ctx.profile_read(kernel)
        per_kernel = {}
        for name, kid in (("decode_full", lt.KERNEL_DECODE_FULL), ("decode_lazy", lt.KERNEL_DECODE_LAZY)):
            n, ms = stack.ctx.profile_read(kid)
            per_kernel[name] = {"launches": n, "avg_us": (ms / n * 1e3) if n else None}
        stored = Tp_mean if kernel == lt.KERNEL_DECODE_FULL else min(Tp_mean, wl.w_sink + wl.w_recent)
        # algorithmic bytes of one launch (one layer, all sequences): stored K+V entries once, q in, out, appended K/V
        per_seq = (2 * wl.n_kv_heads * wl.head_dim * 2) * stored + wl.n_q_heads * wl.head_dim * (2 + 4) \
            + wl.n_kv_heads * wl.head_dim * 2 * 2
        launch_bytes = wl.batch * per_seq
        avg_ms = total_ms / max(launches, 1)
        achieved = launch_bytes / avg_ms / 1e6
        # which of the two decode kernels the timed layers ran on (lt_set_decode_path gives the rule), and how
        timed_lazy = 0 if kernel == lt.KERNEL_DECODE_FULL else 1
        plan = stack.ctx.decode_plan(list(stack.is_lazy).index(timed_lazy))
        roofline = {
            "bound": "hbm", "kernel": "%s<%d, %d, *> (%s layers)" % ("lt_decode_mfma_kernel" if plan["matrix_cores"] else "lt_decode_kernel",
                                                                     wl.group, timed_lazy, "lazy" if timed_lazy else "full"),
            "plan": plan,
            "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": read_traffic(wl.name), "launches": launches, "avg_launch_us": avg_ms * 1e3,
            "bytes_per_launch": launch_bytes, "ms_per_step_with_events": elapsed_p / K * 1e3, "kernels": per_kernel,
        }
        log("roofline pass: %d launches, %.1f us each, %.1f GB/s (%.1f%% of 8 TB/s)" % (launches, avg_ms * 1e3, achieved, achieved / 80))
        # what a plain streaming read reaches on this device: 1 GiB inside the layer-0 cache (or all of it)
        try:
            probe_buf = stack.ctx.kv_slab[: min(stack.ctx.kv_slab.numel(), 1 << 30)]
            sink = torch.zeros(256, dtype=torch.uint8, device=dev)
            lt.probe_read(probe_buf, sink)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                lt.probe_read(probe_buf, sink)
            e1.record()
            torch.cuda.synchronize()
            probe_gbs = probe_buf.numel() * 10 / e0.elapsed_time(e1) / 1e6
            roofline["read_probe_gbs"] = probe_gbs
            roofline["frac_of_read_probe"] = achieved / probe_gbs
            log("plain streaming read of %.2f GB: %.0f GB/s; the decode kernel reaches %.1f%% of it" % (
                probe_buf.numel() / 1e9, probe_gbs, 100 * achieved / probe_gbs))
        except lt.LtError as e:                        # measurement aid only
            log("read probe skipped: %s" % e)
        probe_buf = sink = None                        # a view keeps the whole slab alive

    # ---- oracle on host cores --------------------------------------------------------------------------------
    cpu = cpu_baseline(W, wl, stack, [int(x) for x in is_lazy]) if want_cpu else None
    stack.close()
    del stack
    torch.cuda.empty_cache()

    # ---- all-full comparison: attention-time speedup of the hybrid stack -------------------------------------------
    speedup = None
    if want_speedup and wl.n_lazy > 0:
        window = wl.w_sink + wl.w_recent
        f = wl.n_lazy / wl.n_layers
        speedup = {"ms_per_step_all_full": None, "measured": None,
                   "byte_ratio_ideal": 1.0 / (1.0 - f + f * min(window, T_mean) / T_mean), "lazy_fraction": f}
        steps0 = min(K, 16)
        cfg0 = lt.make_config(wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.w_sink, wl.w_recent, wl.context + Wm + steps0)
        if all_full_fits(lt, cfg0, wl):
            full = Stack(lt, W, wl, [0] * wl.n_layers, Wm + steps0, dev, args.keys_full, args.keys_lazy)
            full.run(Wm)
            e0 = timed(full, steps0)
            full.close()
            del full
            torch.cuda.empty_cache()
            ms0 = e0 / steps0 * 1e3
            speedup.update({"ms_per_step_all_full": ms0, "measured": ms0 / ms_per_step})
            log("all-full stack: %.3f ms/step -> speedup %.3fx" % (ms0, ms0 / ms_per_step))
        else:
            speedup["note"] = "a stack of %d full layers does not fit the device at this batch: not measurable" % wl.n_layers
            log("all-full stack does not fit the device: only the byte-ratio ideal %.3fx is reported" % speedup["byte_ratio_ideal"])

    return {
        "metric": "hybrid decode-attn tokens/s + achieved HBM GB/s (% peak), 1 MI355X",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16 storage, fp32 accumulate", "data": "synthetic",
        "config": {"workload": wl.name, "layers": wl.n_layers, "lazy_layers": int(sum(is_lazy)), "batch": wl.batch,
                   "q_heads": wl.n_q_heads, "kv_heads": wl.n_kv_heads, "head_dim": wl.head_dim, "context": wl.context,
                   "w_sink": wl.w_sink, "w_recent": wl.w_recent, "tokens_first_step": T_first, "tokens_last_step": T_last,
                   "identification": "online queue, P+1 full caches" if online else "all layers scored, then the stack is built"},
        "kv_gbs": step_bytes / ms_per_step / 1e6, "kv_hbm_frac": step_bytes / ms_per_step / 1e6 / HBM_PEAK_GBS,
        "roofline": roofline, "cpu_baseline": cpu, "scoring": scoring, "speedup_hybrid_vs_all_full": speedup,
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus %d is not supported (no collectives, no sharding)" % args.gpus,
              file=sys.stderr)
        return 2
    import torch

    import lt_workloads as W
    from paper_2410_13846_amd import lt

    Stack.shared_tail = not args.no_shared_tail
    Stack.decode_path = {"auto": lt.DECODE_AUTO, "vector": lt.DECODE_VECTOR, "matrix": lt.DECODE_MATRIX}[args.decode_path]

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    dev = "cuda:0"
    torch.cuda.set_device(0)
    headline = args.workload is None
    wl = W.WORKLOADS[args.workload or HEADLINE_WORKLOAD]
    if args.n_lazy is not None:
        wl = wl.scaled(n_lazy=args.n_lazy)
    if args.context is not None:
        wl = wl.scaled(context=args.context)
    if args.q_heads is not None:
        wl = wl.scaled(n_q_heads=args.q_heads)
    K, Wm = args.steps, args.warmup

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)                                 # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    if args.growth or args.prefill or args.grid or args.paged:
        if headline:
            wl = W.WORKLOADS["qwq_32b_gen" if args.growth else SECOND_WORKLOAD]
            if args.context is not None:
                wl = wl.scaled(context=args.context)
        log("workload %s: L=%d B=%d Hq=%d Hkv=%d n=%d window=%d+%d lazy=%d" % (
            wl.name, wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.context, wl.w_sink, wl.w_recent, wl.n_lazy))
    if args.growth:
        print(json.dumps(growth_curve(args, lt, W, wl, dev)))
        return 0
    if args.prefill:
        print(json.dumps(prefill_bench(args, lt, W, wl, dev)))
        return 0
    if args.grid:
        print(json.dumps(window_grid(args, lt, W, wl, dev)))
        return 0
    if args.paged:
        print(json.dumps(paged_bench(args, lt, W, wl, dev)))
        return 0

    line = decode_bench(args, lt, W, wl, dev, K, Wm, want_cpu=not args.no_cpu_baseline, want_speedup=not args.no_speedup,
                        want_profile=not args.no_profile_pass, scoring_only=args.scoring_only)
    if headline and not args.scoring_only and not args.headline_only:
        # the all-full stack does not fit at batch 16: the measured 50 %-lazy over 0 %-lazy speedup at this context comes
        # from the same stack at batch 1; and the 32K x batch 8 configuration is kept as a second, complete result
        b1 = decode_bench(args, lt, W, W.WORKLOADS["llama31_8b_128k_b1"], dev, K, Wm, want_cpu=False, want_speedup=True,
                          want_profile=True)
        if line["speedup_hybrid_vs_all_full"] is not None:
            line["speedup_hybrid_vs_all_full"]["measured_at_batch_1"] = {
                "workload": b1["config"]["workload"], "ms_per_step_hybrid": b1["ms_per_step"], "tokens_per_s": b1["value"],
                "kv_hbm_frac": b1["kv_hbm_frac"], **b1["speedup_hybrid_vs_all_full"]}
        second = decode_bench(args, lt, W, W.WORKLOADS[SECOND_WORKLOAD], dev, max(K, 64), Wm, want_cpu=False, want_speedup=True,
                              want_profile=True)
        line["also"] = {b1["config"]["workload"]: {k: b1[k] for k in ("value", "ms_per_step", "kv_gbs", "kv_hbm_frac", "roofline", "scoring")},
                        second["config"]["workload"]: {k: second[k] for k in ("value", "ms_per_step", "steps", "kv_gbs", "kv_hbm_frac", "roofline",
                                                                                "scoring", "speedup_hybrid_vs_all_full")}}
    print(json.dumps(line))
    return 0


def read_traffic(workload):
    """HBM bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc summary (None if absent)."""
    path = os.path.join(ROOT, "profiles", "decode_full_%s_traffic.txt" % workload)
    try:
        with open(path) as f:
            for ln in f:
                if ln.startswith("traffic_bytes_per_launch:"):
                    return float(ln.split(":", 1)[1])
    except OSError:
        pass
    return None


if __name__ == "__main__":
    sys.exit(main())
