"""Sustained rate of the two-stage saving path (one GPU).

The paper sizes this path by the rate at which a forward pass produces hidden states: about
10 MB per layer per 1024 tokens every 3 ms for a 13B model, i.e. ~3 GB/s (Section 6.3.3), and
requires that saving stays off the critical path of generation.  This script pushes batches of
a given shape through hc_saver_save_layer as fast as the library accepts them -- no model
compute in between -- and reports the sustained snapshot + re-chunking rate for a prefill-shaped
batch (many rows of one context) and a decode-shaped batch (one row each of many contexts).

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
    out = {"workload": w.name, "d_model": w.d_model, "layers": w.n_layers, "threads": args.threads,
           "paper_required_GBps": 3.0,
           "prefill": run(hc, torch, w, 1024, 1, 9, args.threads, 64),
           "decode": run(hc, torch, w, 64, 64, 65, args.threads, 64)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
