"""Offline profile for the bubble-free layer partition (paper Section 4.1.2) on one GPU.

Measures, for one workload shape, the four per-layer times the partition algorithm takes --
IO_H (host->HBM transfer of one layer's hidden states), IO_KV (transfer of one layer's KV
rows), C_H (the restoration kernel on one layer) -- and derives C_Token from the paper's own
cost model (recomputation costs 6 + N/(4D) times the projection, Section 3.2), which this
library cannot measure because it holds no forward pass.  It then prints the split
hc_partition_layers chooses, and times hc_restore_context_mixed for a sweep of l_h next to the
pipeline model max(compute, transfer) evaluated with the measured per-layer times.

    python -m paper_2410_05004_amd.partition_profile [--workload 1] [--reps 5]
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


def median_ms(fn, torch, reps):
    ts = []
    for _ in range(reps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        ts.append((time.perf_counter() - t0) * 1e3)
    return float(np.median(ts))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", type=int, default=1)
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args()
    import torch
    import synthetic as syn
    import paper_2410_05004_amd as hc
    if not torch.cuda.is_available():
        sys.exit("partition_profile: no GPU visible")
    w = syn.WORKLOADS[args.workload]
    if w.n_seq != 1:
        sys.exit("partition_profile: pick a single-context workload")
    L, d, d_kv, T, B, CT = w.n_layers, w.d_model, w.d_kv, w.tokens, w.block_size, w.chunk_tokens
    desc = hc.ModelDesc(L, d, w.n_q_heads, w.n_kv_heads, w.head_dim, B, w.pos_offset + T + 1, 0,
                        w.rope_theta, w.rms_eps)
    ctx = hc.Context(desc)
    s = torch.cuda.current_stream().cuda_stream
    copy_stream = torch.cuda.Stream()
    n_blocks = (w.pos_offset + T + B - 1) // B
    bt, num_pages = syn.block_table(w, w.pos_offset + T)
    d_bt = torch.from_numpy(bt).cuda()
    g = torch.Generator(device="cuda").manual_seed(syn.BASE_SEED)
    keep, pools = [], []
    for l in range(L):
        wkv = (torch.randn((2 * d_kv, d), device="cuda", generator=g) * 0.02).to(torch.bfloat16)
        gamma = (1 + 0.1 * torch.randn((d,), device="cuda", generator=g)).to(torch.bfloat16)
        keep += [wkv, gamma]
        ctx.set_layer_weights(l, wkv, gamma, s)
        pools.append(torch.zeros((num_pages, 2, B, w.n_kv_heads, w.head_dim), dtype=torch.bfloat16,
                                 device="cuda"))
        ctx.set_kv_pool(l, pools[l], num_pages)
    hidden = torch.randn((T, d), device="cuda", generator=g).to(torch.bfloat16)
    pos = torch.arange(w.pos_offset, w.pos_offset + T, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()

    # C_H: the restoration kernel, hidden states resident
    for l in range(L):
        ctx.restore_kv(l, hidden, pos, T, d_bt, n_blocks, s)
    ctx.timing_begin()
    for _ in range(3):
        for l in range(L):
            ctx.restore_kv(l, hidden, pos, T, d_bt, n_blocks, s)
    c_h, _ = ctx.timing_end(s)                     # milliseconds per launch

    # IO_H, IO_KV: plain pinned copies of one layer's rows
    def copy_ms(nbytes):
        src = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
        dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        dst.copy_(src, non_blocking=True)
        return median_ms(lambda: dst.copy_(src, non_blocking=True), torch, 9)
    io_h, io_kv = copy_ms(T * d * 2), copy_ms(T * 2 * d_kv * 2)
    c_token = c_h * (6.0 + T / (4.0 * d))          # modelled, Section 3.2

    # stores: every layer's hidden states and every layer's KV rows, generation order
    h_rows = hidden.view(torch.int16).cpu().numpy()
    kv_rows = torch.zeros((T, 2 * d_kv), dtype=torch.bfloat16, device="cuda")
    ctx.gather_kv(0, kv_rows, pos, T, d_bt, n_blocks, s)
    k_rows = kv_rows.view(torch.int16).cpu().numpy()

    # the row <-> page copy kernels against the HBM rate (bytes read + bytes written)
    def kernel_us(fn, reps=50):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps
    kv_bytes = 2.0 * T * 2 * d_kv * 2
    us_scatter = kernel_us(lambda: ctx.scatter_kv(0, kv_rows, pos, T, d_bt, n_blocks, s))
    us_gather = kernel_us(lambda: ctx.gather_kv(0, kv_rows, pos, T, d_bt, n_blocks, s))
    n_chunks = -(-T // CT)
    sweep = sorted({L, L - 1, L - 2, L - 4, L * 3 // 4, L // 2, 0})
    out_sweep = []
    hstore = hc.Store(L, d, CT, L * n_chunks + 2)
    for l in range(L):
        hstore.append(1, l, h_rows, T)
    for l_h in sweep:
        kstore = None
        if l_h < L:
            kstore = hc.Store(L - l_h, 2 * d_kv, CT, (L - l_h) * n_chunks + 2)
            for l in range(L - l_h):
                kstore.append(1, l, k_rows, T)

        def go():
            ctx.restore_context_mixed(hstore, kstore, l_h, 1, 0, T, w.pos_offset, d_bt, n_blocks, s,
                                      copy_stream.cuda_stream)
        go()
        ms = median_ms(go, torch, args.reps)
        l_o = L - l_h
        model = max(c_h * l_h, io_h * l_h + io_kv * l_o)
        out_sweep.append({"l_h": l_h, "l_o": l_o, "measured_ms": round(ms, 3), "model_ms": round(model, 3)})
        if kstore is not None:
            kstore.destroy()
    assert ctx.poll_device_error(s) == 0

    out = {"workload": w.name, "tokens": T, "layers": L,
           "io_h_ms": round(io_h, 4), "io_kv_ms": round(io_kv, 4), "c_h_ms": round(c_h, 4),
           "c_token_ms_modelled": round(c_token, 4), "kv_complement_sweep": out_sweep,
           "kv_rows_kernel": {"bytes_moved_per_call": kv_bytes,
                              "scatter_us": round(us_scatter, 2), "gather_us": round(us_gather, 2),
                              "scatter_GBps": round(kv_bytes / us_scatter / 1e3, 1),
                              "gather_GBps": round(kv_bytes / us_gather / 1e3, 1), "hbm_peak_GBps": 8000.0}}
    try:
        l_h, l_o, comp = hc.partition_layers(L, io_h, io_kv, c_h, c_token)
        out["partition"] = {"l_h": l_h, "l_o": l_o,
                            "complement": "kv_offload" if comp == 0 else "token_recompute"}
    except hc.HCacheError as e:
        out["partition"] = {"error": str(e)}
    print(json.dumps(out))
    hstore.destroy()
    ctx.destroy()


if __name__ == "__main__":
    main()
