#!/usr/bin/env python3
"""Benchmark of the shared-KV decode hot path on one MI355X.

A step is one decode step of the whole model: for every layer in order, kvs_append_kv (a no-op
for layers that read a donor's cache) followed by kvs_decode_attention over the slot the
layer's share-map entry resolves to.  Inputs are synthetic (seeded N(0,1), bf16) and resident in
HBM before timing starts.  Prints one JSON line: tokens/s (batch size / step time), the HBM
roofline of the decode-attention launch, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0              # MI355X HBM3E, published peak
MFMA_BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16 matrix peak, published


def algorithmic_bytes_per_launch(w, seq_lens, store_dtype=None):
    """Bytes one decode-attention launch must move: every stored key and value of the layer's
    slot once, q in, fp32 out, and the page-table entries that address the context."""
    store_dtype = store_dtype or w.dtype
    e = {"fp8": 1, "bf16": 2}.get(store_dtype, 4)             # bytes per stored element
    eq = 4 if store_dtype == "f32" else 2                      # queries are bf16 for bf16 and fp8 slots
    kv = int(seq_lens.astype(np.int64).sum()) * w.Hkv * w.d * 2 * e
    qo = w.B * w.Hq * w.d * (eq + 4)
    table = int(((seq_lens.astype(np.int64) + 15) // 16).sum()) * 4
    return kv + qo + table


DECODE_SOURCES = ("kvs_decode.hip", "kvs_attn_tiles.h", "kvs_flat_plan.h", "kvs_device.h")
PREFILL_SOURCES = ("kvs_attention.hip", "kvs_attn_tiles.h", "kvs_device.h")
DISTANCE_SOURCES = ("kvs_distance.hip",)


def recorded_traffic(name, sources):
    """HBM bytes per launch from the committed counter summary profiles/<name>.traffic.txt, or None
    when there is none or the kernel's sources have changed since the counters were taken."""
    import hashlib
    path = os.path.join(ROOT, "profiles", f"{name}.traffic.txt")
    if not os.path.exists(path):
        return None
    rec = {}
    for line in open(path):
        if "=" in line and not line.startswith("#"):
            k, v = line.split("=", 1)
            rec[k.strip()] = v.strip()
    digest = hashlib.sha256()
    for src in sources:                                          # the kernel and the headers it inlines
        digest.update(open(os.path.join(ROOT, "paper_2410_18517_amd", "csrc", src), "rb").read())
    if rec.get("kernel_source_sha256") != digest.hexdigest():
        return None
    return int(rec["traffic_bytes_per_launch"])


def traffic_probe(torch, dev):
    """One plain 1 GiB device copy (torch): a kernel of known traffic in the same counter trace, to
    scale FETCH_SIZE / WRITE_SIZE by."""
    src = torch.ones(1 << 29, dtype=torch.bfloat16, device=dev)      # 1 GiB read, 1 GiB written
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


def _event_time_us(torch, fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    pairs = []
    for _ in range(steps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        pairs.append((e0, e1))
    torch.cuda.synchronize()
    return float(np.mean([a.elapsed_time(b) for a, b in pairs])) * 1e3


def bench_prefill(args, torch, kb, inputs, dev):
    """Causal prefill chunk of the Llama-2-13B shape: 64 new rows per sequence behind a 1984-token
    prefix (--prefill-rows T: the last T rows of the 2048, up to the whole prompt); a step = attention
    of the T rows over the keys they may see, for one layer; the T-row append is timed beside it.
    A short chunk streams the prefix and is priced against HBM; from 512 rows on the score and value
    products dominate and the line is priced against the bf16 MFMA peak."""
    w = inputs.WORKLOADS["llama2-13b"]
    T, n_layers = (args.prefill_rows or w.prefill_rows), 3    # rotate over three layers' slots
    if not 0 < T <= w.context:
        sys.exit(f"--prefill-rows must be in [1, {w.context}]")
    mb = w.max_blocks_per_seq
    table = inputs.make_block_table(w.B, mb, w.B * mb, 1)
    store_dtype = args.store or "bf16"                        # --store fp8: the same rows in 8-bit slots
    store = kb.KVStore(np.arange(n_layers, dtype=np.int32), w.Hq, w.Hkv, w.d, store_dtype, w.B * mb, mb, block_table=table)
    gen = torch.Generator(device=dev)
    gen.manual_seed(inputs.SEED_BASE)
    zeros = torch.zeros(w.B, dtype=torch.int32, device=dev)
    for l in range(n_layers):
        k = torch.randn((w.B, w.context, w.Hkv, w.d), device=dev, generator=gen).bfloat16()
        v = torch.randn((w.B, w.context, w.Hkv, w.d), device=dev, generator=gen).bfloat16()
        kb.kvs_append_kv(store, l, k, v, zeros)
    q = torch.randn((w.B, T, w.Hq, w.d), device=dev, generator=gen).bfloat16()
    k_new = torch.randn((w.B, T, w.Hkv, w.d), device=dev, generator=gen).bfloat16()
    v_new = torch.randn((w.B, T, w.Hkv, w.d), device=dev, generator=gen).bfloat16()
    start = torch.full((w.B,), w.context - T, dtype=torch.int32, device=dev)
    out = torch.empty((w.B, T, w.Hq, w.d), dtype=torch.float32, device=dev)
    ws = store.workspace(w.B, T)
    it = [0]

    def attn():
        kb.kvs_prefill_attention(store, it[0] % n_layers, q, start, out=out, workspace=ws)
        it[0] += 1

    def append():
        kb.kvs_append_kv(store, it[0] % n_layers, k_new, v_new, start)
        it[0] += 1

    if args.traffic_probe:
        traffic_probe(torch, dev)
    attn_us = _event_time_us(torch, attn, args.steps, args.warmup)
    append_us = _event_time_us(torch, append, args.steps, args.warmup)
    kv_bytes = w.B * w.context * w.Hkv * w.d * 2 * (1 if store_dtype == "fp8" else 2) + w.B * T * w.Hq * w.d * (2 + 4)
    # row i of the chunk sees prefix + i + 1 keys; 2 flops per multiply-add, scores and values
    keys_seen = T * (w.context - T) + T * (T + 1) // 2
    flops = 4.0 * w.B * w.Hq * w.d * keys_seen
    # which prefill kernel the library's launch rule picks for this shape
    group = w.Hq // w.Hkv
    ncols = T * group
    fp8 = "true" if store_dtype == "fp8" else "false"
    if ncols > 128:
        kernel = "attn_bf16_wide_kernel<128,2,8,%s,%s>" % ("true" if ncols <= 256 else "false", fp8)   # pages read once?
    elif ncols > 64:
        kernel = "attn_bf16_wide_kernel<128,1,8,true,%s>" % fp8
    elif ncols == 64:
        kernel = "attn_bf16_wide_kernel<128,1,4,true,%s>" % fp8
    else:
        kernel = "attn_bf16_kernel<128,4,2>"
    if T < 512:
        roof = {"bound": "hbm", "kernel": kernel, "achieved": round(kv_bytes / attn_us / 1e3, 1),
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(kv_bytes / attn_us / 1e3 / HBM_PEAK_GBPS, 4)}
    else:
        roof = {"bound": "mfma", "kernel": kernel, "achieved": round(flops / attn_us / 1e6, 1),
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(flops / attn_us / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4)}
    traffic = recorded_traffic("attn_bf16_prefill_llama2-13b", PREFILL_SOURCES) if T == w.prefill_rows and store_dtype == "bf16" else None
    roof.update({"traffic": traffic, "launch_us": round(attn_us, 2), "algorithmic_bytes": kv_bytes, "algorithmic_flops": flops})
    print(json.dumps({
        "metric": "causal prefill chunk attention, rows/s", "value": round(w.B * T / (attn_us * 1e-6), 1),
        "unit": "query rows/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(attn_us * 1e-3, 4), "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "llama2-13b prefill chunk" + (", fp8 slots" if store_dtype == "fp8" else ""), "batch": w.B, "rows": T, "prefix": w.context - T,
                   "q_heads": w.Hq, "kv_heads": w.Hkv, "head_dim": w.d},
        "append_us": round(append_us, 2),
        "append_bytes": w.B * T * w.Hkv * w.d * 2 * (2 + (1 if store_dtype == "fp8" else 2)),   # rows read + pages written
        "roofline": roof}))


def bench_distance(args, torch, kb, inputs, dev):
    """Calibration of the 48-layer workload: 30 samples x 512 tokens x 8 kv heads x 128, bf16, drawn by
    the structured generator (per-layer scale, per-channel offsets, unit noise), so that the ranking
    the matrix feeds is not degenerate.  The fp64 oracle is timed on the same input on the host and
    the GPU's matrix is compared with it."""
    S, L, Hkv, T, d = 30, 48, 8, 512, 128
    N = Hkv * T * d
    print("drawing the calibration caches on the host", file=sys.stderr, flush=True)
    host = inputs.calibration_kv(S, L, Hkv, T, d, 1)
    kv = host.to(dev)
    ws = torch.empty(kb.lib().kvs_distance_workspace_bytes(L), dtype=torch.uint8, device=dev)
    outs = [None]

    def run():
        outs[0] = kb.kvs_layer_distance(kv, workspace=ws)

    if args.traffic_probe:
        traffic_probe(torch, dev)
    us = _event_time_us(torch, run, args.steps, args.warmup)
    torch.cuda.synchronize()
    got = [o.cpu().numpy().astype(np.float64) for o in outs[0]]     # the last timed launch's own output
    nbytes = kv.numel() * 2 + 3 * L * L * 4
    achieved = nbytes / us / 1e3
    line = {
        "metric": "layer-distance matrix, calibration bytes/s", "value": round(achieved, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(us * 1e-3, 4),
        "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "calibration 30 x 48 layers x (8 x 512 x 128), structured", "samples": S, "layers": L, "N": N},
        "roofline": {"bound": "hbm", "kernel": "distance_partial_kernel<bf16, 256-position chunks> + distance_final_kernel",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": recorded_traffic("distance_calibration_48_layers", DISTANCE_SOURCES), "launch_us": round(us, 2),
                     "algorithmic_bytes": nbytes}}
    if not args.no_cpu_baseline:
        print("GPU part done, running the CPU oracle", file=sys.stderr, flush=True)
        from oracle import attention as orc
        arr = inputs.to_oracle_array(host)
        c0 = time.perf_counter()
        want = orc.layer_distance(arr)
        cpu_s = time.perf_counter() - c0
        fro = [float(np.linalg.norm(g - w_) / np.linalg.norm(w_)) for g, w_ in zip(got, want)]
        off = ~np.eye(L, dtype=bool)
        line["cpu_baseline"] = {"value": round(nbytes / cpu_s / 1e9, 3), "unit": "GB/s", "cores": orc.num_threads(),
                                "kind": "oracle", "sample": f"fp64 oracle on the whole calibration input: {cpu_s:.2f} s"}
        line["parity_rel_frobenius"] = {"dK2": fro[0], "dV2": fro[1], "D": fro[2]}
        line["parity_rel_entry_max"] = float((np.abs(got[2] - want[2])[off] / want[2][off]).max())
    print(json.dumps(line))


def bench_similarity(args, torch, kb, inputs, dev):
    """Similarity test of the strategy search: last-layer hidden states of two models on the calibration
    set, 30 sentences x 64 tokens x hidden 5120 (the Llama-2-13B shape), bf16; a step = one
    kvs_avg_cos_sim call (both readings are timed; the line reports the paper text's: mean first).
    A few tens of MB per call: the launch is short against its own start and end, so the line also
    carries a calibration set of 480 sentences of the same shape."""
    hidden, tokens = 5120, 64
    N = tokens * hidden
    line = None
    extra = {}
    for S in (30, 480):
        a = inputs.normal((S, N), 11, S, 0).to(dev)
        b = (a.float() + 0.5 * inputs.normal((S, N), 11, S, 1, dtype="f32").to(dev)).bfloat16()
        ws = torch.zeros(kb.lib().kvs_cos_sim_workspace_bytes(S), dtype=torch.uint8, device=dev)
        res = {}
        for mode in (0, 1):
            out = [None]

            def run():
                out[0] = kb.kvs_avg_cos_sim(a, b, mode, workspace=ws)

            # a call is a few microseconds of GPU time, less than one call through the interpreter:
            # sixteen calls are recorded into a HIP graph (kernel nodes only) and the replays are timed
            run()
            torch.cuda.synchronize()
            eager = float(out[0].item())
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for _ in range(16):
                    run()
            us = _event_time_us(torch, graph.replay, args.steps, args.warmup) / 16
            if float(out[0].item()) != eager:
                raise SystemExit("graph replays gave another similarity than the eager call")
            res[mode] = (us, eager)
        nbytes = 2 * S * N * 2
        if S == 30:
            us, got = res[0]
            achieved = nbytes / us / 1e3
            line = {
                "metric": "calibration similarity test, hidden-state bytes/s", "value": round(achieved, 1), "unit": "GB/s",
                "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(us * 1e-3, 5),
                "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
                "config": {"workload": "calibration similarity, 30 sentences x 64 tokens x hidden 5120", "sentences": S,
                           "N": N, "reading": "cosine of the sentence-averaged vectors"},
                "roofline": {"bound": "hbm", "kernel": "cos_sim_kernel<bf16>", "achieved": round(achieved, 1),
                             "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                             "traffic": None, "launch_us": round(us, 2), "algorithmic_bytes": nbytes},
                "per_sentence_reading_us": round(res[1][0], 2)}
            if not args.no_cpu_baseline:
                from oracle.similarity import avg_cos_sim
                oa, ob = inputs.to_oracle_array(a.cpu()), inputs.to_oracle_array(b.cpu())
                c0 = time.perf_counter()
                want = [avg_cos_sim(oa, ob, m_) for m_ in (0, 1)]
                cpu_s = (time.perf_counter() - c0) / 2
                line["cpu_baseline"] = {"value": round(nbytes / cpu_s / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
                                        "sample": f"fp64 numpy oracle on the same input, mean of the two readings: {cpu_s:.3f} s"}
                line["parity_abs_error"] = {"mean_first": abs(res[0][1] - want[0]), "per_sentence": abs(res[1][1] - want[1])}
        else:
            extra = {"sentences": S, "mean_first_us": round(res[0][0], 2), "per_sentence_us": round(res[1][0], 2),
                     "mean_first_gbps": round(nbytes / res[0][0] / 1e3, 1), "per_sentence_gbps": round(nbytes / res[1][0] / 1e3, 1)}
    line["larger_set"] = extra
    print(json.dumps(line))


def bench_project(args, torch, kb, inputs, dev):
    """Fused K/V projection + rotary embedding + append, Llama-3-8B shape (hidden 4096, 8 kv heads
    x 128): the per-layer work that sharing removes for recipient layers.  One new row per
    sequence (a decode step) streams the weights and is priced against HBM; --project-rows T > 1
    (a prefill chunk of T rows per sequence) is a matrix product priced against the bf16 MFMA peak."""
    w = inputs.WORKLOADS["llama3-8b-32k"]
    hidden, n_layers = 4096, 4                             # rotate over four layers' weights
    mb = w.max_blocks_per_seq
    store = kb.KVStore(np.arange(n_layers, dtype=np.int32), w.Hq, w.Hkv, w.d, "bf16", w.B * mb, mb)
    gen = torch.Generator(device=dev)
    gen.manual_seed(inputs.SEED_BASE)
    n_out = w.Hkv * w.d
    wk = [(torch.randn((n_out, hidden), device=dev, generator=gen) / 64).bfloat16() for _ in range(n_layers)]
    wv = [(torch.randn((n_out, hidden), device=dev, generator=gen) / 64).bfloat16() for _ in range(n_layers)]
    T = args.project_rows
    x = torch.randn((w.B, T, hidden), device=dev, generator=gen).bfloat16()
    ang = torch.outer(torch.arange(w.context, dtype=torch.float64),
                      10000.0 ** (-torch.arange(w.d // 2, dtype=torch.float64) * 2 / w.d))
    cos, sin = torch.cos(ang).float().to(dev), torch.sin(ang).float().to(dev)
    pos = torch.full((w.B,), w.context - T, dtype=torch.int32, device=dev)
    reps = 8 if T == 1 else 1

    def one_round():                                       # all four layers back to back
        for l in range(n_layers):
            kb.kvs_project_append_kv(store, l, x, wk[l], wv[l], pos, cos, sin)

    one_round()                                            # eager: sizes the workspace, gives the expected rows
    torch.cuda.synchronize()
    eager = [t.clone() for t in kb.kvs_gather_kv(store, 0, w.context - 1, 1, w.B)]
    # The kernel is a few microseconds, less than one call through the interpreter, so the launches
    # are recorded once into a HIP graph (kernel nodes only) and the replays are timed.
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for _ in range(reps):
            one_round()
    us = _event_time_us(torch, graph.replay, args.steps, args.warmup) / (reps * n_layers)
    replayed = kb.kvs_gather_kv(store, 0, w.context - 1, 1, w.B)
    if not all(torch.equal(a, b) for a, b in zip(eager, replayed)):
        raise SystemExit("graph replays wrote different rows than the eager launches")
    rows = w.B * T
    nbytes = 2 * n_out * hidden * 2 + rows * hidden * 2 + rows * 2 * n_out * 2
    flops = 2.0 * rows * 2 * n_out * hidden
    if T == 1:
        roof = {"bound": "hbm", "kernel": "project_append_bf16_kernel", "achieved": round(nbytes / us / 1e3, 1),
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4)}
    else:
        # two head blocks per workgroup once those tiles alone fill the chip (the library's rule)
        two_heads = w.d == 128 and w.Hkv * ((rows + 255) // 256) >= 192
        roof = {"bound": "mfma", "kernel": "project_append_pair_kernel" if two_heads else "project_append_tiled_kernel<128>",
                "achieved": round(flops / us / 1e6, 1),
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(flops / us / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4)}
    roof.update({"traffic": None, "launch_us": round(us, 2), "algorithmic_bytes": nbytes, "algorithmic_flops": flops})
    print(json.dumps({
        "metric": "fused K/V projection + rotary + append, layers/s", "value": round(1e6 / us, 1), "unit": "layers/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(us * 1e-3, 5),
        "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "llama3-8b decode projection" if T == 1 else "llama3-8b prefill projection",
                   "batch": w.B, "rows_per_sequence": T, "hidden": hidden, "kv_heads": w.Hkv, "head_dim": w.d},
        "saved_per_recipient_layer": {"weight_bytes": 2 * n_out * hidden * 2, "flops": flops, "us": round(us, 2)},
        "roofline": roof}))


def bench_sparse(args, torch, kb, inputs, dev):
    """Decode attention over intra-layer sparsified slots, Llama-3-8B 32k shape: every (sequence,
    kv head) keeps a random 80 % of its 32768 tokens (the paper's "additional 20 %" on top of layer
    sharing), compacted in place by kvs_compact_kv; a step = one kvs_decode_attention_per_head
    launch per layer.  The compaction is timed separately (a maintenance operation)."""
    w = inputs.WORKLOADS["llama3-8b-32k"]
    n_layers = 4
    mb = w.max_blocks_per_seq
    table = inputs.make_block_table(w.B, mb, w.B * mb, 1)
    store = kb.KVStore(np.arange(n_layers, dtype=np.int32), w.Hq, w.Hkv, w.d, "bf16", w.B * mb, mb, block_table=table)
    gen = torch.Generator(device=dev)
    gen.manual_seed(inputs.SEED_BASE)
    rng = np.random.default_rng(inputs.SEED_BASE)
    zeros = torch.zeros(w.B, dtype=torch.int32, device=dev)
    n_keep = int(0.8 * w.context)
    kv_lens = np.full((n_layers, w.B, w.Hkv), n_keep, np.int32)
    host0 = keep0 = None
    compact_ms = []
    for l in range(n_layers):
        k = torch.randn((w.B, w.context, w.Hkv, w.d), device=dev, generator=gen).bfloat16()
        v = torch.randn((w.B, w.context, w.Hkv, w.d), device=dev, generator=gen).bfloat16()
        assert kb.kvs_append_kv(store, l, k, v, zeros) == kb.KVS_OK
        idx = np.stack([np.stack([np.sort(rng.choice(w.context, size=n_keep, replace=False)) for _ in range(w.Hkv)])
                        for _ in range(w.B)]).astype(np.int32)
        if l == 0:
            host0, keep0 = (k.cpu(), v.cpu()), idx
        idx_d, cnt_d = torch.from_numpy(idx).to(dev), torch.from_numpy(kv_lens[l]).to(dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        assert kb.kvs_compact_kv(store, l, idx_d, cnt_d) == kb.KVS_OK
        e1.record()
        torch.cuda.synchronize()
        compact_ms.append(e0.elapsed_time(e1))
        del k, v
    q = [torch.randn((w.B, w.Hq, w.d), device=dev, generator=gen).bfloat16() for _ in range(n_layers)]
    lens_d = torch.from_numpy(kv_lens).to(dev)
    out = torch.empty((n_layers, w.B, w.Hq, w.d), dtype=torch.float32, device=dev)
    ws = store.workspace(w.B, 1)

    def one_round():
        for l in range(n_layers):
            kb.kvs_decode_attention_per_head(store, l, q[l], lens_d, out=out[l], workspace=ws)

    us = _event_time_us(torch, lambda: [one_round() for _ in range(8)], args.steps, args.warmup) / (8 * n_layers)
    nbytes = int(kv_lens[0].sum()) * w.d * 2 * 2 + w.B * w.Hq * w.d * (2 + 4)
    achieved = nbytes / us / 1e3
    line = {
        "metric": "decode attention over sparsified shared-KV slots, tokens/s per layer",
        "value": round(w.B / (us * 1e-6), 1), "unit": "tokens/s per layer", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(us * 1e-3, 5), "higher_is_better": True, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "llama3-8b-32k, 80 % of the tokens kept per kv head", "batch": w.B, "q_heads": w.Hq,
                   "kv_heads": w.Hkv, "head_dim": w.d, "context": w.context, "kept_per_head": n_keep},
        "compact_ms_per_layer": round(float(np.mean(compact_ms)), 3),
        "roofline": {"bound": "hbm", "kernel": "attn_bf16_kernel<128,1,4,false> (per-head lengths)", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None,
                     "launch_us": round(us, 2), "algorithmic_bytes": nbytes}}
    if not args.no_cpu_baseline:
        from oracle.sparse import sparse_decode_attention
        want = sparse_decode_attention(inputs.to_oracle_array(q[0].cpu()), inputs.to_oracle_array(host0[0]),
                                       inputs.to_oracle_array(host0[1]), keep0)
        got = out[0].cpu().numpy().astype(np.float64)
        err = np.sqrt(((got - want) ** 2).sum(-1)) / np.sqrt((want ** 2).sum(-1))
        line["parity_rel_l2_max"] = float(err.max())
    print(json.dumps(line))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama3-8b-32k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--split-tokens", type=int, default=0)
    ap.add_argument("--two-calls", action="store_true",
                    help="decode mode: kvs_append_kv + kvs_decode_attention per layer instead of kvs_decode_step")
    ap.add_argument("--graph", action="store_true",
                    help="decode mode: record the step's launches once into a HIP graph and time its replays")
    ap.add_argument("--store", choices=["fp8"], default=None,
                    help="decode and prefill modes: keep the slots in fp8 (E4M3) instead of the workload's type")
    ap.add_argument("--seq-lens", default=None,
                    help="decode mode: comma-separated lengths (tokens, counting this step's), one per sequence, in "
                         "place of the workload's: a store below its capacity, or one long sequence among short ones")
    ap.add_argument("--prefill-rows", type=int, default=0,
                    help="--mode prefill: rows per sequence in the chunk (default: the workload's 64)")
    ap.add_argument("--project-rows", type=int, default=1,
                    help="--mode project: new rows per sequence (1 = decode step, more = prefill chunk)")
    ap.add_argument("--mode", choices=["decode", "prefill", "distance", "project", "sparse", "similarity"], default="decode",
                    help="decode (default): the whole decode step, the headline metric.  prefill: the 64-row "
                         "causal chunk of the llama2-13b workload.  distance: the 48-layer calibration matrix. "
                         "project: the fused K/V projection (see --project-rows).  sparse: decode attention over "
                         "sparsified slots.  similarity: the calibration similarity test.  All but decode time the other kernels of the path, one JSON line each.")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="also run one plain 1 GiB device copy (torch) so that a counter trace of this "
                         "command contains a kernel of known traffic to scale FETCH_SIZE/WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this path has no multi-GPU part (run with --gpus 1)")

    import torch
    from paper_2410_18517_amd import binding as kb, inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    if args.split_tokens:
        kb.kvs_testing_force_split_tokens(args.split_tokens)
    if args.mode == "prefill":
        return bench_prefill(args, torch, kb, inputs, dev)
    if args.mode == "distance":
        return bench_distance(args, torch, kb, inputs, dev)
    if args.mode == "project":
        return bench_project(args, torch, kb, inputs, dev)
    if args.mode == "sparse":
        return bench_sparse(args, torch, kb, inputs, dev)
    if args.mode == "similarity":
        return bench_similarity(args, torch, kb, inputs, dev)
    w = inputs.WORKLOADS[args.workload]

    share = inputs.make_share_map(w.L, w.n_shared, 1, fixed=w.fixed_map)
    seq_lens = inputs.make_seq_lens(w, 1)
    if args.seq_lens:
        seq_lens = np.array([int(x) for x in args.seq_lens.split(",")], np.int32)
        if len(seq_lens) != w.B or seq_lens.min() < 1 or seq_lens.max() > w.context:
            sys.exit(f"--seq-lens needs {w.B} lengths in [1, {w.context}]")
    max_blocks = w.max_blocks_per_seq
    num_blocks = w.B * max_blocks
    table = inputs.make_block_table(w.B, max_blocks, num_blocks, 1)
    store_dtype = args.store or w.dtype
    if store_dtype == "fp8" and w.dtype != "bf16":
        sys.exit("--store fp8 needs a bf16 workload")
    store = kb.KVStore(share, w.Hq, w.Hkv, w.d, store_dtype, num_blocks, max_blocks, block_table=table)
    tdt = store.torch_dtype

    # fill every slot through the library's own append path; keep one layer's source rows for the oracle
    gen = torch.Generator(device=dev)
    gen.manual_seed(inputs.SEED_BASE)
    own = [l for l in range(w.L) if share[l] == l]
    zeros = torch.zeros(w.B, dtype=torch.int32, device=dev)
    kept = {}                                       # host copies of the source rows, for the oracle leg
    for l in own:
        k = torch.randn((w.B, w.context, w.Hkv, w.d), device=dev, dtype=torch.float32, generator=gen).to(tdt)
        v = torch.randn((w.B, w.context, w.Hkv, w.d), device=dev, dtype=torch.float32, generator=gen).to(tdt)
        assert kb.kvs_append_kv(store, l, k, v, zeros) == kb.KVS_OK
        if not args.no_cpu_baseline:
            kept[l] = (k.cpu(), v.cpu())
        del k, v
    q = [torch.randn((w.B, w.Hq, w.d), device=dev, dtype=torch.float32, generator=gen).to(tdt) for _ in range(w.L)]
    k_new = torch.randn((w.B, 1, w.Hkv, w.d), device=dev, dtype=torch.float32, generator=gen).to(tdt)
    v_new = torch.randn((w.B, 1, w.Hkv, w.d), device=dev, dtype=torch.float32, generator=gen).to(tdt)
    lens_dev = torch.from_numpy(seq_lens).to(dev)
    pos_dev = lens_dev - 1
    # this step's token, so the oracle sees what the store holds after the appends
    for kc, vc in kept.values():
        for b in range(w.B):
            kc[b, seq_lens[b] - 1] = k_new[b, 0].cpu()
            vc[b, seq_lens[b] - 1] = v_new[b, 0].cpu()
    out = torch.empty((w.L, w.B, w.Hq, w.d), dtype=torch.float32, device=dev)
    ws = store.workspace(w.B, 1)
    torch.cuda.synchronize()

    def step():
        # every layer: store this step's key/value row (layers that read a donor's cache store nothing)
        # and attend; one launch per layer, or the two separate calls with --two-calls
        for l in range(w.L):
            if args.two_calls:
                kb.kvs_append_kv(store, l, k_new, v_new, pos_dev)
                kb.kvs_decode_attention(store, l, q[l], lens_dev, out=out[l], workspace=ws)
            else:
                kb.kvs_decode_step(store, l, q[l], k_new, v_new, lens_dev, out=out[l], workspace=ws)

    if args.traffic_probe:
        traffic_probe(torch, dev)

    print("store filled, timing", file=sys.stderr, flush=True)
    if args.graph:
        # kernel nodes only (the library records no memsets and allocates nothing); the lengths are
        # a device array, so a serving loop would advance them between replays
        step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        step = graph.replay
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = w.B / (ms_per_step * 1e-3)
    out_timed = out.clone()                         # what the last timed step wrote: checked against the oracle below

    # Average duration of one decode-attention launch, by HIP events on the stream the kernels run
    # on.  An event pair around every call inside the step loop costs ~7 % of the step on this
    # runtime (each record stalls the queue), so the same steps x layers launches are issued again,
    # back to back, with one event pair per step's worth of launches.
    launch_ms = []
    for _ in range(args.steps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for l in range(w.L):
            kb.kvs_decode_attention(store, l, q[l], lens_dev, out=out[l], workspace=ws)
        e1.record()
        launch_ms.append((e0, e1))
    torch.cuda.synchronize()
    launch_ms = float(np.mean([a.elapsed_time(b) for a, b in launch_ms])) / w.L
    alg_bytes = algorithmic_bytes_per_launch(w, seq_lens, store_dtype)
    achieved = alg_bytes / (launch_ms * 1e-3) / 1e9
    kernel = ("attn_f32_kernel" if store_dtype == "f32" else
              "attn_decode_flat_kernel<%d,%s> (one kvs_decode_attention launch)" % (w.d, "fp8 pages" if store_dtype == "fp8" else "bf16 pages"))
    roofline = {"bound": "hbm", "kernel": kernel,
                "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                "traffic": None if args.seq_lens else recorded_traffic(
                    f"attn_{'fp8' if store_dtype == 'fp8' else 'bf16'}_decode_{w.name}", DECODE_SOURCES),
                "launch_us": round(launch_ms * 1e3, 2),
                "algorithmic_bytes": alg_bytes}

    result = {
        "metric": "shared-KV decode attention tokens/s", "value": round(tokens_per_s, 2), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name if store_dtype == w.dtype else f"{w.name}, {store_dtype} slots", "layers": w.L, "q_heads": w.Hq, "kv_heads": w.Hkv, "head_dim": w.d,
                   "batch": w.B, "context": [int(n) for n in seq_lens] if args.seq_lens else
                   (w.context if w.min_context is None else [w.min_context, w.context]),
                   "capacity": w.context,
                   "page_tokens": 16, "shared_layers": w.n_shared, "kv_slots": int(store.desc.n_slots),
                   "step": "kvs_append_kv + kvs_decode_attention per layer" if args.two_calls
                           else "kvs_decode_step per layer",
                   "launch": "HIP graph replay" if args.graph else "eager"},
        "hbm_gbps": round(alg_bytes * w.L / (ms_per_step * 1e-3) / 1e9, 1),
        "hbm_frac": round(alg_bytes * w.L / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        print("GPU part done, running the CPU oracle", file=sys.stderr, flush=True)
        from oracle import attention as orc
        K = [inputs.to_oracle_array(kept[l][0]) if l in kept else None for l in range(w.L)]
        V = [inputs.to_oracle_array(kept[l][1]) if l in kept else None for l in range(w.L)]
        if store_dtype == "fp8":                   # the oracle attends to the values as the slots hold them
            from oracle.fp8 import round_e4m3
            # the storage oracle applied to every bf16 bit pattern once, then looked up per element
            with np.errstate(invalid="ignore"):
                every = (np.arange(1 << 16, dtype=np.uint32) << 16).view(np.float32).astype(np.float64)
            lut = (round_e4m3(every).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
            K = [None if a is None else lut[a] for a in K]
            V = [None if a is None else lut[a] for a in V]
            print("fp8: oracle-side copies rounded", file=sys.stderr, flush=True)
        # out_timed: the timed steps' own output; out: that of the launches of the per-launch timing
        got_timed = out_timed.cpu().numpy().astype(np.float64)
        got_launch = out.cpu().numpy().astype(np.float64)
        cpu_s, err, err_launch = 0.0, 0.0, 0.0
        for l in range(w.L):                       # the whole decode step, layer by layer
            qs = inputs.to_oracle_array(q[l])
            c0 = time.perf_counter()
            want = orc.decode_attention(l, share, K, V, qs, seq_lens)
            cpu_s += time.perf_counter() - c0
            norm = np.sqrt((want ** 2).sum(-1))
            err = max(err, float((np.sqrt(((got_timed[l] - want) ** 2).sum(-1)) / norm).max()))
            err_launch = max(err_launch, float((np.sqrt(((got_launch[l] - want) ** 2).sum(-1)) / norm).max()))
        result["cpu_baseline"] = {
            "value": round(w.B / cpu_s, 4), "unit": "tokens/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"fp64 oracle, decode attention of all {w.L} layers of one step (the appends are not "
                      f"timed), all {w.B} sequences x {w.Hq} heads at {'the given lengths' if args.seq_lens else 'full context'}: {cpu_s:.2f} s"}
        result["parity_rel_l2_max"] = err                       # the timed steps (the path `value` is measured on)
        result["parity_rel_l2_max_launch_timing"] = err_launch  # the kvs_decode_attention launches `roofline` is measured on
    print(json.dumps(result))


if __name__ == "__main__":
    main()
