"""Sustained rate of the two-stage saving path (one GPU).

The paper sizes this path by the rate at which a forward pass produces hidden states: about
10 MB per layer per 1024 tokens every 3 ms for a 13B model, i.e. ~3 GB/s (Section 6.3.3), and
requires that saving stays off the critical path of generation.  This script pushes batches of
a given shape through hc_saver_save_layer as fast as the library accepts them -- no model
compute in between -- and reports the sustained snapshot + re-chunking rate for a prefill-shaped
batch (many rows of one context) and a decode-shaped batch (one row each of many contexts).
A third part runs a stand-in for the layers' forward compute and shows what saving adds to the
compute stream's time with and without the deferred fence.

    python -m paper_2410_05004_amd.save_rate [--workload 3] [--threads 8]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def run(hc, torch, w, rows_per_step, n_ctx, steps, threads, chunk_tokens):
    L, d = w.n_layers, w.d_model
    tokens_per_ctx = rows_per_step // n_ctx * steps
    cap = n_ctx * L * (-(-tokens_per_ctx // chunk_tokens)) + 8
    store = hc.Store(L, d, chunk_tokens, cap, pinned=True)
    saver = hc.Saver(store, rows_per_step, n_slots=8, n_threads=threads)
    act = torch.randn((rows_per_step, d), device="cuda").to(torch.bfloat16)
    row_seq = np.repeat(np.arange(n_ctx, dtype=np.int64), rows_per_step // n_ctx)
    compute = torch.cuda.current_stream().cuda_stream
    down = torch.cuda.Stream()
    for l in range(L):                                   # warm up: first touch of slots and chunks
        saver.save_layer(l, act, rows_per_step, row_seq, compute, down.cuda_stream)
    saver.flush()
    t0 = time.perf_counter()
    for _ in range(steps - 1):
        for l in range(L):
            saver.save_layer(l, act, rows_per_step, row_seq, compute, down.cuda_stream)
    t_enq = time.perf_counter() - t0
    saver.flush()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    nbytes = (steps - 1) * L * rows_per_step * d * 2
    saver.destroy()
    store.destroy()
    return {"rows_per_step": rows_per_step, "contexts": n_ctx, "steps": steps - 1,
            "GBps": round(nbytes / dt / 1e9, 2), "ms_per_layer": round(dt * 1e3 / ((steps - 1) * L), 4),
            "ms_per_step_all_layers": round(dt * 1e3 / (steps - 1), 3),
            "producer_blocked_fraction": round(t_enq / dt, 3)}


def run_fused(hc, torch, w, prefill_rows, decode_ctx, steps, threads, chunk_tokens):
    """A fused step: a prefill chunk of one context plus one row each of `decode_ctx` others."""
    L, d = w.n_layers, w.d_model
    rows = prefill_rows + decode_ctx
    cap = L * (-(-prefill_rows * steps // chunk_tokens) + decode_ctx * (-(-steps // chunk_tokens)) + 8)
    store = hc.Store(L, d, chunk_tokens, cap, pinned=True)
    saver = hc.Saver(store, rows, n_slots=8, n_threads=threads)
    act = torch.randn((rows, d), device="cuda").to(torch.bfloat16)
    row_seq = np.concatenate([np.zeros(prefill_rows), 1 + np.arange(decode_ctx)]).astype(np.int64)
    compute = torch.cuda.current_stream().cuda_stream
    down = torch.cuda.Stream()
    for l in range(L):
        saver.save_layer(l, act, rows, row_seq, compute, down.cuda_stream)
    saver.flush()
    t0 = time.perf_counter()
    for _ in range(steps - 1):
        for l in range(L):
            saver.save_layer(l, act, rows, row_seq, compute, down.cuda_stream)
    saver.flush()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    nbytes = (steps - 1) * L * rows * d * 2
    saver.destroy()
    store.destroy()
    return {"rows_per_step": rows, "prefill_rows": prefill_rows, "decode_contexts": decode_ctx,
            "steps": steps - 1, "GBps": round(nbytes / dt / 1e9, 2),
            "ms_per_layer": round(dt * 1e3 / ((steps - 1) * L), 4)}


def overlap(hc, torch, w, rows, steps, threads, chunk_tokens):
    """Cost of saving on the compute stream: a stand-in for one layer's forward compute (12
    [rows, d] x [d, d] products = the 24 N D^2 flop of a layer) runs per layer, (a) alone,
    (b) with hc_saver_save_layer, whose wait makes the layer start after its snapshot copy,
    (c) with hc_saver_save_layer_deferred and the fence before the next layer, the paper's
    event discipline.  Returns ms per step (all layers) for each."""
    L, d = w.n_layers, w.d_model
    cap = L * (-(-rows * steps // chunk_tokens)) + 8
    act = torch.randn((rows, d), device="cuda").to(torch.bfloat16)
    wmat = (torch.randn((d, d), device="cuda") * 0.02).to(torch.bfloat16)
    out = torch.empty_like(act)
    row_seq = np.zeros(rows, dtype=np.int64)
    compute = torch.cuda.current_stream().cuda_stream
    down = torch.cuda.Stream()

    def layer_compute():
        for _ in range(12):
            torch.mm(act, wmat, out=out)

    res = {}
    for mode in ("no_saving", "blocking", "deferred"):
        store = hc.Store(L, d, chunk_tokens, cap, pinned=True)
        saver = hc.Saver(store, rows, n_slots=8, n_threads=threads)
        for rep in range(2):                             # first pass warms up, second is timed
            if rep == 1:
                saver.flush()
                store.drop(0) if store.tokens(0, 0) else None
                torch.cuda.synchronize()
                t0 = time.perf_counter()
            for _ in range(steps):
                for l in range(L):
                    if mode == "blocking":
                        saver.save_layer(l, act, rows, row_seq, compute, down.cuda_stream)
                    elif mode == "deferred":
                        saver.save_layer_deferred(l, act, rows, row_seq, compute, down.cuda_stream)
                    layer_compute()
                    if mode == "deferred":
                        saver.fence(compute)
            torch.cuda.synchronize()
        res[mode] = round((time.perf_counter() - t0) * 1e3 / steps, 3)
        saver.flush()
        saver.destroy()
        store.destroy()
    return {"rows_per_step": rows, "steps": steps, "ms_per_step_all_layers": res}


def d2h_rate(torch, nbytes=64 << 20, reps=10):
    """Plain pinned device->host copy rate of the box (one large block), GB/s."""
    src = torch.empty(nbytes // 2, dtype=torch.int16, device="cuda")
    dst = torch.empty(nbytes // 2, dtype=torch.int16).pin_memory()
    for _ in range(2):
        dst.copy_(src, non_blocking=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        dst.copy_(src, non_blocking=True)
    torch.cuda.synchronize()
    return reps * nbytes / (time.perf_counter() - t0) / 1e9


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", type=int, default=3)
    ap.add_argument("--threads", type=int, default=8)
    args = ap.parse_args()
    import torch
    import synthetic as syn
    import paper_2410_05004_amd as hc
    if not torch.cuda.is_available():
        sys.exit("save_rate: no GPU visible")
    w = syn.WORKLOADS[args.workload]
    link = d2h_rate(torch)
    out = {"workload": w.name, "d_model": w.d_model, "layers": w.n_layers, "threads": args.threads,
           "paper_required_GBps": 3.0, "plain_pinned_d2h_GBps": round(link, 2),
           "prefill": run(hc, torch, w, 1024, 1, 9, args.threads, 64),
           "decode": run(hc, torch, w, 64, 64, 65, args.threads, 64),
           "fused": run_fused(hc, torch, w, 960, 64, 9, args.threads, 64),
           "beside_compute": overlap(hc, torch, w, 1024, 4, args.threads, 64)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
