"""Restoration-kernel time against the number of restored tokens (one layer).

The paper rejects a token-wise split of the state because the projection's run time is not
proportional to the token count: it moves in steps set by the GEMM library's tile sizes
(Section 4.1.1, "Performance considerations"; Section 6.3.2 shows the measured steps).  This
script measures the same curve for this library's kernel on MI355X: time per launch for
n_tok = step, 2*step, ... at a given model shape, so that a scheduler can pick mini-batch
sizes on the flat part of each step (the kernel's token tile is 256).  Every token count is
timed as the library launches it (hc_set_split mode 1: a partly filled last round of
workgroups is split along d_model where a cost model says it pays), with every tile computed
whole (mode 0), and split whenever the shape allows it (mode 2).

    python -m paper_2410_05004_amd.sweep_tokens [--workload 3] [--max-tokens 4096] [--step 64]

Prints one line per token count and a final JSON object; needs a GPU.
"""
import argparse
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", type=int, default=3, help="model shape (default: Llama-2-13B-shaped)")
    ap.add_argument("--max-tokens", type=int, default=4096)
    ap.add_argument("--step", type=int, default=64)
    ap.add_argument("--reps", type=int, default=20)
    args = ap.parse_args()

    import torch
    import synthetic as syn
    import paper_2410_05004_amd as hc

    if not torch.cuda.is_available():
        sys.exit("sweep_tokens: no GPU visible")
    w = syn.WORKLOADS[args.workload]
    T = args.max_tokens
    layer_norm = w.norm == "layer"
    desc = hc.ModelDesc(1, w.d_model, w.n_q_heads, w.n_kv_heads, w.head_dim, w.block_size, T,
                        w.rope_style, w.rope_theta, w.rms_eps, 1 if layer_norm else 0)
    ctx = hc.Context(desc)
    s = torch.cuda.current_stream().cuda_stream
    wkv, gamma = syn.layer_weights(w, 0)
    x = syn.layer_hidden(w, 0, T)
    d_w = torch.from_numpy(wkv.view(np.int16)).cuda()
    d_g = torch.from_numpy(gamma.view(np.int16)).cuda()
    d_x = torch.from_numpy(x.view(np.int16)).cuda()
    if layer_norm:                                          # OPT-style: shift and biases too
        beta, bias = syn.layer_affine(w, 0)
        d_b = torch.from_numpy(beta.view(np.int16)).cuda()
        d_c = torch.from_numpy(bias.view(np.int16)).cuda()
        ctx.set_layer_weights_affine(0, d_w, d_g, d_b, d_c, s)
    else:
        ctx.set_layer_weights(0, d_w, d_g, s)
    n_blocks = (T + w.block_size - 1) // w.block_size
    pool = torch.zeros((n_blocks, 2, w.block_size, w.n_kv_heads, w.head_dim), dtype=torch.bfloat16, device="cuda")
    ctx.set_kv_pool(0, pool, n_blocks)
    d_bt = torch.arange(n_blocks, dtype=torch.int32, device="cuda")
    d_pos = torch.arange(T, dtype=torch.int32, device="cuda")
    for _ in range(200):                                    # clocks up
        ctx.restore_kv(0, d_x, d_pos, T, d_bt, n_blocks, s)
    torch.cuda.synchronize()
    rows = []
    print(f"# {w.name} shape: d_model {w.d_model}, d_kv {w.d_kv}; one layer; time per launch")
    print("# n_tok   us/launch   TFLOP/s   us per 256 tokens   us unsplit   us split   whole + split tiles x ways (* = the library's choice)")

    def timed(n, split):
        ctx.set_split(split)
        for _ in range(3):
            ctx.restore_kv(0, d_x, d_pos, n, d_bt, n_blocks, s)
        ctx.timing_begin()
        for _ in range(args.reps):
            ctx.restore_kv(0, d_x, d_pos, n, d_bt, n_blocks, s)
        return ctx.timing_end(s)[0] * 1e3

    for n in range(args.step, T + 1, args.step):
        plan = hc.diag_split_plan(w.d_model, w.d_kv, n, 2)
        chosen = hc.diag_split_plan(w.d_model, w.d_kv, n, 1)["split"]
        us0 = timed(n, 0)
        us2 = timed(n, 2) if plan["split"] else None
        us = timed(n, 1)
        tf = 4.0 * n * w.d_model * w.d_kv / (us * 1e-6) / 1e12
        shape = f'{plan["nf"] * plan["nt_main"]} + {plan["n_tail"]} x {plan["n_split"]}' + ("*" if chosen else "")
        rows.append({"n_tok": n, "us": round(us, 2), "tflops": round(tf, 1), "us_unsplit": round(us0, 2),
                     "us_split": None if us2 is None else round(us2, 2), "tiles": shape})
        split_col = "-" if us2 is None else f"{us2:.2f}"
        print(f"{n:7d} {us:10.2f} {tf:9.1f} {us * 256 / n:12.2f} {us0:12.2f} {split_col:>10}   {shape}", flush=True)
    assert ctx.poll_device_error(s) == 0
    print(json.dumps({"workload": w.name, "d_model": w.d_model, "d_kv": w.d_kv, "rows": rows}))
    ctx.destroy()


if __name__ == "__main__":
    main()
