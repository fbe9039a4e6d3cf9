#!/usr/bin/env python3
"""Benchmark of the HCache restoration hot path on one MI355X.

A step = one restoration of the whole workload: for every layer, the fused kernel
(RMSNorm -> K|V projection -> RoPE -> paged scatter) over all tokens, hidden states
already resident in HBM; the layers of a step go out eight per launch.  `value` is restored tokens per second over all layers.
The same JSON line carries the roofline of the dominant kernel (measured with HIP
events around every launch), the fp64 oracle timed on the host cores on a bounded
sample, and the PCIe-inclusive end-to-end figure (chunk store -> H2D -> kernel,
pipelined) as context.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 2]
"""
import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16, vendor figure without sparsity

# HBM-side traffic of one restore_kernel launch, from two rocprofv3 --pmc runs (FETCH_SIZE, then
# WRITE_SIZE, each scaled by what the counter reads for a plain 256 MiB streaming kernel):
# profiles/restore_kernel_llama3-8b-gqa-T8192.md.  Bytes per layer (a launch over several layers
# moves that many times as much); None where not profiled.
TRAFFIC_BYTES_PER_LAUNCH = {"llama3-8b-gqa-T8192": 2.436e8}
# the same per layer inside a launch over 8 layers (fetched 200.1 MiB + written 32.0 MiB)
TRAFFIC_BYTES_PER_LAYER_FUSED = {"llama3-8b-gqa-T8192": 2.4335e8}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(w, sample_tokens):
    """The oracle as it stands on the host cores: all layers x `sample_tokens` tokens."""
    import synthetic as syn
    import oracle.hcache_oracle as oracle
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    # ragged workload: the first tokens of its first context stand for the batch (rows are
    # independent, the cost per token is the same)
    avail = w.tokens if w.n_seq == 1 else int(syn.ragged_lengths(w)[0])
    T = min(sample_tokens, avail)
    bt, num_pages = syn.block_table(w, w.pos_offset + T)
    pos = w.pos_offset + np.arange(T)
    pool = np.zeros((num_pages, 2, w.block_size, w.n_kv_heads, w.head_dim))
    total = 0.0
    for l in range(w.n_layers):
        wkv, gamma = syn.layer_weights(w, l)
        x = syn.bf16_bits_to_f64(syn.layer_hidden(w, l, T))
        wkv, gamma = syn.bf16_bits_to_f64(wkv), syn.bf16_bits_to_f64(gamma)
        extra = {}
        if w.norm == "layer":
            beta, bias = syn.layer_affine(w, l)
            extra = dict(norm="layer", beta=syn.bf16_bits_to_f64(beta), bias=syn.bf16_bits_to_f64(bias))
        t0 = time.perf_counter()
        oracle.restore_kv(pool, x, gamma, wkv, pos, bt, eps=w.rms_eps, theta=w.rope_theta,
                          n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, block_size=w.block_size,
                          rope_style=w.rope_style, **extra)
        total += time.perf_counter() - t0
    return {"value": T / total, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"all {w.n_layers} layers x first {T} tokens of the workload, fp64 numpy, "
                      f"{total:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=2)
    ap.add_argument("--cpu-sample-tokens", type=int, default=8192,
                    help="tokens of the workload the oracle is timed on (all layers); ~10 s of host work")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-e2e", action="store_true")
    ap.add_argument("--e2e-steps", type=int, default=5)
    ap.add_argument("--streams", type=int, default=1,
                    help="streams the per-layer launches of a step are dealt over (layers are independent)")
    ap.add_argument("--layers-per-launch", type=int, default=32,
                    help="layers restored by one kernel launch (hidden states of all layers are resident "
                         "in HBM here, so they can go out together: hc_restore_kv_layers, which launches "
                         "them eight at a time); 1 = one launch per layer (hc_restore_kv), as the pipelined "
                         "loader issues them")
    ap.add_argument("--rope-style", type=int, default=None,
                    help="override the workload's RoPE convention (0 half-split, 1 interleaved, 2 none)")
    ap.add_argument("--loader", type=int, default=0, help="0 = copy engines, strided runs (default), 1 = gather kernel")
    ap.add_argument("--chunk-tokens", type=int, default=None,
                    help="tokens per chunk of the host store in the end-to-end leg (default: the workload's; "
                         "the paper uses 64)")
    ap.add_argument("--fragmented", action="store_true",
                    help="end-to-end leg on a fragmented arena: eight contexts of the workload's length are "
                         "appended in decode order (a few tokens at a time, taking turns), every other one is "
                         "dropped, four new ones are appended into the holes, and the last of those is the one "
                         "restored (single-context workloads only; needs 8x the pinned memory)")
    ap.add_argument("--zero-inputs", action="store_true",
                    help="diagnostic: all-zero hidden states and weights (same instruction stream, no "
                         "operand toggling) to show how far the matrix pipe's clock is power-limited")
    ap.add_argument("--d-model", type=int, default=None,
                    help="diagnostic: override the workload's d_model (a multiple of 64) to separate the cost "
                         "per channel from the fixed cost per tile; implies a different synthetic shape")
    ap.add_argument("--split", type=int, default=1,
                    help="hc_set_split mode for single-layer launches: 0 never split the d_model loop, "
                         "1 (default) when the library's cost model says it pays, 2 whenever possible")
    ap.add_argument("--tokens", type=int, default=None,
                    help="diagnostic: override the workload's token count (single-context workloads): short "
                         "contexts, where a layer fills only part of the chip")
    ap.add_argument("--one-tile", action="store_true",
                    help="diagnostic: shrink the workload to ONE workgroup tile (256 tokens, one KV head of 128 "
                         "-> 256 fused features), one launch per layer: the kernel alone on an otherwise idle "
                         "chip, at full clock; with two --d-model values it gives the loop's cycles per step")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="context: also time the vendor library's plain bf16 GEMM (torch.mm = hipBLASLt) on the "
                         "same hidden states and unpacked weights, layer after layer, no norm / RoPE / paging")
    ap.add_argument("--power-probe", action="store_true",
                    help="diagnostic: run the matrix-pipe duty-cycle probe (hc_diag_mfma_duty) instead of the "
                         "benchmark and print its table as one JSON line")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB -> 256 MiB streaming kernel three times, so that a "
                         "counter run has a kernel of known traffic to scale FETCH_SIZE/WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding or collectives); "
                 "use --gpus 1")

    import torch
    import synthetic as syn
    import paper_2410_05004_amd as hc

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the restoration path has no CPU fallback")
    if args.power_probe:
        torch.cuda.set_device(0)
        rows = []
        for period_us, duty, half in ((1000, 1.0, False), (200, 0.5, False), (1000, 0.5, False),
                                      (10000, 0.5, False), (1000, 0.25, False), (1000, 0.5, True),
                                      (10000, 0.5, True)):
            rows.append({"period_us": period_us, "duty": duty, "half_of_the_cus_at_a_time": half,
                         "tflops_inside_busy_windows": round(hc.diag_mfma_duty(period_us, duty, half), 1)})
            log(rows[-1])
        zero = round(hc.diag_mfma_duty(1000, 1.0, False, zero_operands=True), 1)
        other = round(hc.diag_mfma_duty(1000, 1.0, False, op_shape=1), 1)
        other_zero = round(hc.diag_mfma_duty(1000, 1.0, False, zero_operands=True, op_shape=1), 1)
        print(json.dumps({"probe": "mfma duty cycle, random bf16 operands in registers, 32x32x16",
                          "rows": rows, "continuous_zero_operands_tflops": zero,
                          "continuous_16x16x32_tflops": other,
                          "continuous_16x16x32_zero_operands_tflops": other_zero,
                          "peak_tflops": MFMA_BF16_PEAK_TFLOPS}), flush=True)
        return
    w = syn.WORKLOADS[args.workload]
    if args.d_model:
        import dataclasses
        w = dataclasses.replace(w, d_model=args.d_model, name=f"{w.name}-d{args.d_model}")
    if args.tokens:
        import dataclasses
        w = dataclasses.replace(w, tokens=args.tokens, name=f"{w.name}-tokens{args.tokens}")
    if args.one_tile:
        import dataclasses
        w = dataclasses.replace(w, n_q_heads=1, n_kv_heads=1, head_dim=128, tokens=256, n_seq=1,
                                name=f"{w.name}-one-tile")
        args.layers_per_launch = 1
    ragged = w.n_seq != 1
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    L, d = w.n_layers, w.d_model
    if ragged:
        lengths = syn.ragged_lengths(w)
        T, max_pos = int(lengths.sum()), int(lengths.max())
    else:
        T, max_pos = w.tokens, w.pos_offset + w.tokens
    log(f"workload {w.name}: L={L} d={d} d_kv={w.d_kv} T={T}")

    desc = hc.ModelDesc(L, d, w.n_q_heads, w.n_kv_heads, w.head_dim, w.block_size,
                        max_pos, w.rope_style if args.rope_style is None else args.rope_style,
                        w.rope_theta, w.rms_eps,
                        hc.HC_NORM_LAYER if w.norm == "layer" else hc.HC_NORM_RMS)
    ctx = hc.Context(desc)
    ctx.set_split(args.split)
    stream = torch.cuda.current_stream().cuda_stream

    def dev_bf16(bits):
        return torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)

    # ---- synthetic inputs (seeded), resident in HBM before anything is timed
    t0 = time.time()
    if ragged:
        tables, num_pages = syn.ragged_block_tables(w, lengths)
        d_bt = torch.from_numpy(tables).to(dev)
        d_cu = torch.from_numpy(np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)).to(dev)
        d_pos = torch.from_numpy(np.concatenate([np.arange(n, dtype=np.int32) for n in lengths])).to(dev)
        bt = tables
    else:
        bt, num_pages = syn.block_table(w, w.pos_offset + T)
        d_bt = torch.from_numpy(bt).to(dev)
        d_pos = torch.arange(w.pos_offset, w.pos_offset + T, dtype=torch.int32, device=dev)
    pools, hidden_dev, hidden_host, raw_weights = [], [], [], []
    def generate(l):
        return syn.layer_weights(w, l), syn.layer_hidden(w, l, T)
    workers = min(8, os.cpu_count() or 8)                  # a few layers at a time: bounded host memory
    pool_ex = ThreadPoolExecutor(workers)
    gen = {}
    for l in range(L):
        if l % workers == 0:
            gen = dict(zip(range(l, min(L, l + workers)), pool_ex.map(generate, range(l, min(L, l + workers)))))
        (wkv, gamma), x = gen.pop(l)
        if args.zero_inputs:
            wkv[:] = 0
            x[:] = 0
        d_w, d_g = dev_bf16(wkv), dev_bf16(gamma)
        if w.norm == "layer":
            beta, bias = syn.layer_affine(w, l)
            d_b, d_c = dev_bf16(beta), dev_bf16(bias)
            ctx.set_layer_weights_affine(l, d_w, d_g, d_b, d_c, stream)
        else:
            ctx.set_layer_weights(l, d_w, d_g, stream)
        torch.cuda.synchronize()
        if args.vendor_gemm:
            raw_weights.append(d_w)
        del d_w, d_g
        pool = torch.zeros((num_pages, 2, w.block_size, w.n_kv_heads, w.head_dim),
                           dtype=torch.bfloat16, device=dev)
        ctx.set_kv_pool(l, pool, num_pages)
        pools.append(pool)
        hidden_dev.append(dev_bf16(x))
        if not args.no_e2e:
            hidden_host.append(x)
    pool_ex.shutdown()
    log(f"inputs generated and uploaded in {time.time() - t0:.1f} s")

    if args.calibrate_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)      # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)                   # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    side = [torch.cuda.Stream() for _ in range(args.streams - 1)]
    lanes = [stream] + [s_.cuda_stream for s_ in side]

    G = max(1, min(args.layers_per_launch, L))
    if ragged:
        G = 1

    def step(use=None):
        use = use or lanes
        if G > 1:
            for i, l0 in enumerate(range(0, L, G)):
                ctx.restore_kv_layers(l0, hidden_dev[l0:l0 + G], d_pos, T, d_bt, len(bt), use[i % len(use)])
            return
        for l in range(L):
            if ragged:
                ctx.restore_kv_ragged(l, hidden_dev[l], d_pos, T, d_cu, w.n_seq, d_bt, bt.shape[1],
                                      use[l % len(use)])
            else:
                ctx.restore_kv(l, hidden_dev[l], d_pos, T, d_bt, len(bt), use[l % len(use)])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    assert ctx.poll_device_error(stream) == 0

    # ---- timed region: exactly K steps, inputs resident in HBM
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    tokens_per_s = T / (ms_per_step * 1e-3)

    # ---- dominant kernel: HIP events around every launch, on the launch stream
    torch.cuda.synchronize()
    ctx.timing_begin()
    for _ in range(max(1, min(args.steps, 4096 // L))):
        step([stream])                                      # one stream: kernels back to back
    avg_ms, min_ms, median_ms, launches = ctx.timing_end_stats(stream)
    layers_per_launch = L / launches * max(1, min(args.steps, 4096 // L))
    flop_per_launch = 4.0 * T * d * w.d_kv * layers_per_launch   # 2 flop per multiply-add, K and V
    achieved = flop_per_launch / (avg_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": "restore_kernel", "achieved": round(achieved, 2),
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
                "traffic": None if args.zero_inputs or w.name not in TRAFFIC_BYTES_PER_LAUNCH
                else (TRAFFIC_BYTES_PER_LAUNCH[w.name] if layers_per_launch == 1
                      else TRAFFIC_BYTES_PER_LAYER_FUSED[w.name] * layers_per_launch),
                "traffic_source": None if args.zero_inputs or w.name not in TRAFFIC_BYTES_PER_LAUNCH
                else "stored: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised in "
                     "profiles/restore_kernel_llama3-8b-gqa-T8192.md (not measured in this run)",
                "avg_launch_us": round(avg_ms * 1e3, 2), "min_launch_us": round(min_ms * 1e3, 2),
                "median_launch_us": round(median_ms * 1e3, 2), "launches_timed": launches,
                "layers_per_launch": round(layers_per_launch, 2),
                "flop_per_launch": flop_per_launch}
    assert ctx.poll_device_error(stream) == 0

    # ---- context: the vendor library's plain GEMM on the same operands
    vendor = None
    if args.vendor_gemm:
        out_buf = torch.empty((T, 2 * w.d_kv), dtype=torch.bfloat16, device=dev)
        for l in range(L):
            torch.mm(hidden_dev[l], raw_weights[l].t(), out=out_buf)
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = max(1, min(args.steps, 50))
        ev0.record()
        for _ in range(reps):
            for l in range(L):
                torch.mm(hidden_dev[l], raw_weights[l].t(), out=out_buf)
        ev1.record()
        torch.cuda.synchronize()
        us = ev0.elapsed_time(ev1) * 1e3 / (reps * L)
        vendor = {"us_per_layer": round(us, 2), "TFLOPs": round(4.0 * T * d * w.d_kv / us / 1e6, 1),
                  "note": "torch.mm (hipBLASLt), bf16, row-major output, no normalisation, RoPE or paging; "
                          "back-to-back launches between one pair of events"}
        del out_buf

    # ---- context: PCIe-inclusive end to end from the pinned chunk store (never `value`)
    e2e = None
    if not args.no_e2e:
        CT = args.chunk_tokens or w.chunk_tokens
        copy_stream = torch.cuda.Stream()
        restored_seq, runs_per_layer = 0, None
        ctx.set_loader(args.loader)
        if ragged:
            # every context arrives as a prefill: chunk by chunk, layer by layer, context after context
            starts = np.concatenate([[0], np.cumsum(lengths)])
            store = hc.Store(L, d, CT, L * int(sum(-(-int(n) // CT) for n in lengths)), pinned=True)
            for i, n in enumerate(lengths):
                for c0 in range(0, int(n), CT):
                    for l in range(L):
                        rows = hidden_host[l][starts[i] + c0:starts[i] + min(c0 + CT, int(n))]
                        store.append(i, l, rows, len(rows))
            ids = np.arange(w.n_seq, dtype=np.int64)

            def restore():
                ctx.restore_contexts(store, ids, lengths, d_bt, bt.shape[1], stream, copy_stream.cuda_stream)
        else:
            n_chunks = (T + CT - 1) // CT

            def feed(ids, piece):                          # decode order: contexts take turns
                for a in range(0, T, piece):
                    for sid in ids:
                        for l in range(L):
                            rows = hidden_host[l][a:a + piece]
                            store.append(sid, l, rows, len(rows))

            if args.fragmented:
                store = hc.Store(L, d, CT, L * (8 * n_chunks + 8), pinned=True)
                feed(range(8), 16)
                for sid in (1, 3, 5, 7):
                    store.drop(sid)
                feed(range(10, 14), 16)
                restored_seq = 13
            else:
                store = hc.Store(L, d, CT, L * n_chunks, pinned=True)
                feed([0], CT)                              # arrival order: chunk by chunk, layer by layer
            # copy-engine transfers per layer = runs of equally spaced chunks (from the index)
            slots = np.array([store.chunk(restored_seq, 0, c)[0] for c in range(n_chunks)], dtype=np.int64)
            runs_per_layer, c = 0, 0
            while c < n_chunks:                            # as the loader groups them
                e = c
                if c + 1 < n_chunks and slots[c + 1] > slots[c]:
                    stride = slots[c + 1] - slots[c]
                    e = c + 1
                    while e + 1 < n_chunks and slots[e + 1] - slots[e] == stride:
                        e += 1
                runs_per_layer += 1
                c = e + 1

            def restore():
                ctx.restore_context(store, restored_seq, 0, T, w.pos_offset, d_bt, len(bt), stream,
                                    copy_stream.cuda_stream)
        for _ in range(2):
            restore()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.e2e_steps):
            restore()
        torch.cuda.synchronize()
        e2e_ms = (time.perf_counter() - t0) * 1e3 / args.e2e_steps
        host_bytes = float(L) * T * d * 2
        # plain pinned H2D rate of the box on one layer-sized block, for comparison
        n_plain = min(T, 8192) * d                        # a layer-sized block, at most 8192 rows
        pin = torch.empty(n_plain, dtype=torch.int16).pin_memory()
        dst = torch.empty(n_plain, dtype=torch.int16, device=dev)
        for _ in range(2):
            dst.copy_(pin, non_blocking=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            dst.copy_(pin, non_blocking=True)
        torch.cuda.synchronize()
        h2d_gbs = 10 * n_plain * 2 / (time.perf_counter() - t0) / 1e9
        e2e = {"ms_per_restore": round(e2e_ms, 3), "tokens_per_s": round(T / (e2e_ms * 1e-3), 1),
               "host_link_GBps": round(host_bytes / (e2e_ms * 1e-3) / 1e9, 2),
               "plain_pinned_h2d_GBps": round(h2d_gbs, 2), "chunk_tokens": CT,
               "arena": "fragmented (8 interleaved contexts, 4 dropped, 4 re-appended)" if args.fragmented
               else "one context, arrival order",
               "copy_transfers_per_layer": runs_per_layer,
               "loader": "copy engines, strided runs" if args.loader == 0 else "gather kernel",
               "note": "pinned chunk store -> loader on a side stream -> kernel, layer pipelined"}
        assert ctx.poll_device_error(stream) == 0
        store.destroy()

    cpu = None if args.no_cpu_baseline else cpu_baseline(w, args.cpu_sample_tokens)

    out = {
        # `value` is the kernel-only figure (inputs already in HBM when the timed region starts);
        # the same workload streamed from the pinned host store is `e2e_tokens_per_s`
        "metric": "restored KV tokens/sec (all layers), hidden states resident in HBM (kernel only)",
        "value": round(tokens_per_s, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic" if not args.zero_inputs else "zeros (diagnostic)",
        "config": {"workload": w.name, "layers": L, "d_model": d, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "tokens": T, "block_size": w.block_size,
                   "hidden_resident_in_hbm": True, "launch_streams": args.streams,
                   "layers_per_launch": round(layers_per_launch, 2),
                   "layers_per_launch_requested": G},
        "e2e_tokens_per_s": None if e2e is None else e2e["tokens_per_s"],
        "e2e_note": "the same workload streamed from the pinned chunk store over the host link, layer "
                    "pipelined (details under e2e_host_link); bounded by the link, never `value`",
        "roofline": roofline,
        "cpu_baseline": cpu,
        "e2e_host_link": e2e,
        "vendor_gemm": vendor,
        "paper_context": "paper reports ratios only: TTFT up to 1.93x vs KV offload and 5.73x vs "
                         "recomputation on A100-40G, fp16 (Section 6); no absolute tokens/s",
    }
    print(json.dumps(out), flush=True)
    ctx.destroy()


if __name__ == "__main__":
    main()
