#!/usr/bin/env python3
"""Benchmark of the routed-LoRA hot path on one MI355X.

Workload (default): a LLaMA-2-7B-shaped layer, bf16, batch 32, 32 tenants with rank-32 adapters at all
seven sites.  One "step" is one pass of the whole hot path over that batch: the prompt-aware router
over the 32 prompts of 256 tokens (milora_route, once), then 64 decode steps through the seven routed
linears (milora_layer_decode) that reuse the cached routes.  Inputs are synthetic, seeded and resident
in HBM before the timed region.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, vendor figure
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix cores, vendor figure

def source_digest():
    """Digest of the decode kernels' source: hardware-counter figures are valid for the source they were taken on."""
    import hashlib

    src = os.path.join(ROOT, "paper_2410_18035_amd", "csrc", "decode.hip")
    try:
        return hashlib.sha256(open(src, "rb").read()).hexdigest()[:16]
    except OSError:
        return None


def measured_traffic(workload):
    """HBM bytes per launch of the workload's decode kernel from the FETCH_SIZE and WRITE_SIZE hardware counters,
    each scaled by what the counter reads for a plain 1 GiB device copy.  The figures live in the counter summaries
    under profiles/ (a line `bench-traffic: workload=... source=... fetch_bytes=... write_bytes=...`); None when
    there is none for this workload or the kernel source has changed since the counters were taken."""
    import glob
    import re

    digest = source_digest()
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*hbm_counters*.txt"))):
        for line in open(path):
            m = re.match(r"\s*bench-traffic:\s*workload=(\S+)\s+source=(\S+)\s+fetch_bytes=(\d+)\s+write_bytes=(\d+)", line)
            if m and m.group(1) == workload and m.group(2) == digest:
                return int(m.group(3)) + int(m.group(4))
    return None


STREAM_PHASES = {  # (waves, slot) of milora_layer_decode_trace's stamps, few-row kernel
    "stream_first_input": (range(0, 6), 1), "stream_matrix_work_done": (range(0, 6), 2), "stream_tiles_summed": (range(0, 6), 3),
    "loader_barrier_passed": ([6], 1), "loader_first_chunk": ([6], 2), "loader_all_chunks": ([6], 3),
    "loader_outputs_stored": ([6], 5), "lora_shrink_items_done": ([7], 2), "lora_shrinks_published": ([7], 3),
    "lora_expands_formed": ([7], 4), "loader_partials_swapped": ([6], 8), "lora_outputs_stored": ([7], 6),
    "flag_stored": ([7], 7)}
WIDE_PHASES = {
    "level_entered": (range(0, 8), 0), "stream_first_input": (range(0, 6), 1), "stream_segments_stored": (range(0, 6), 2),
    "loader_barrier_passed": ([6], 1), "loader_copies_landed": ([6], 2), "lora_list_built": ([7], 2),
    "lora_wave_shrink_items_done": ([7], 6), "lora_wave_expand_items_done": ([7], 3),
    "loader_shrink_items_done": ([6], 6), "loader_expand_items_done": ([6], 3),
    "lora_wave_item1_begun": ([7], 8), "lora_wave_item1_flagged": ([7], 9),
    "sums_begun": (range(0, 8), 4), "sums_stored": (range(0, 8), 5)}


def phase_table(np, stamps, wide):
    """Per stage and phase: the time (us after the launch's first stamp) by which half of the workgroups, and the
    last one, have reached it; a workgroup reaches a phase when the last of the waves that have it does."""
    t = stamps.numpy().astype(np.float64)
    t0 = t[t > 0].min()
    out = {}
    for L in range(t.shape[1]):
        row = {}
        for name, (waves, slot) in (WIDE_PHASES if wide else STREAM_PHASES).items():
            v = t[:, L, list(waves), slot]
            v = np.where(v > 0, v - t0, np.nan)
            if np.isnan(v).all():
                continue
            per_wg = np.nanmax(v, axis=1) * 0.01
            per_wg = per_wg[~np.isnan(per_wg)]
            row[name] = [round(float(np.median(per_wg)), 2), round(float(per_wg.max()), 2)]
        out[f"stage{L}"] = row
    return out


def algorithmic_bytes(wl, routes, tenant_ids, ranks):
    """Bytes the method itself must move for one decode layer-step, and for the gate/up launch alone.

    base weights once + A and B of every distinct (tenant, site) some request is routed to + activations.
    """
    from paper_2410_18035_amd import synth

    s = 2 if wl.dtype == "bf16" else 4
    d, F, B = wl.d, wl.F, wl.B
    base = sum(s * d1 * d2 for d1, d2 in (synth.site_dims(m, d, F) for m in range(7)))
    pairs = {(int(t), int(m)) for t, m in zip(tenant_ids, routes) if 0 <= int(m) < 7}
    lora = sum(s * ranks[t] * sum(synth.site_dims(m, d, F)) for t, m in pairs)
    act = s * B * (10 * d + 3 * F) + B + 4 * B
    gate_up = 2 * s * d * F + sum(s * ranks[t] * F for t, m in pairs if m in (4, 5)) + s * B * d + s * B * F
    return {"layer_step": base + lora + act, "base": base, "lora": lora, "act": act, "gate_up_launch": gate_up}


def prefill_leg(torch, mb, synth, dev, reps=5):
    """The many-row side of the path on the prefill configuration (16 prompts padded to 2048 rows, M = 32768):
    router over the valid tokens, then the seven routed linears on all rows.  Returns the rates of both."""
    wl = synth.CONFIGS["llama7b_prefill_b16"]
    W = synth.base_weights(wl, 0, dev)
    ad = synth.adapters(wl, 0, dev)
    tab = mb.AdapterTable.from_tensors(ad.A, ad.B, ad.rank)
    Wr = synth.router_weights(wl, 0, dev)
    tid = synth.tenant_ids(wl).to(dev)
    H, ss_host, sl_host = synth.prompts(wl, 0, dev)
    ss, sl = ss_host.to(dev), sl_host.to(dev)
    M = H.shape[0]
    r2r = (torch.arange(M, device=dev) // wl.pad_to).to(torch.int32)
    route = torch.empty(wl.B, dtype=torch.uint8, device=dev)
    ws_route = torch.empty(mb.route_workspace_bytes(wl.B, wl.d, M), dtype=torch.uint8, device=dev)

    def timed(fn):
        for _ in range(2):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    route_ms = timed(lambda: mb.milora_route(H, ss, sl, tid, Wr, wl.pool, wl.act, route_out=route, want_logits=False,
                                             workspace=ws_route))
    Xm = torch.empty(M, wl.F, dtype=torch.float32, device=dev).normal_(0, 1).to(torch.bfloat16)
    ws = torch.empty(mb.routed_linear_workspace_bytes(M, wl.F, wl.F, tab.r_max), dtype=torch.uint8, device=dev)
    site_ms, flops = [], 0.0
    for site in range(7):
        d1, d2 = synth.site_dims(site, wl.d, wl.F)
        assert mb.milora_routed_linear_kernel(M, d1, d2, torch.bfloat16) == mb.KERNEL_TILES
        X = Xm if site == 6 else H
        Y = torch.empty(M, d2, dtype=torch.bfloat16, device=dev)
        site_ms.append(timed(lambda: mb.milora_routed_linear(X, W[site], tab, site, tid, route, row_to_req=r2r, d2=d2,
                                                             out=Y, workspace=ws)))
        flops += 2.0 * M * d1 * d2
        del Y
    total_ms = sum(site_ms)
    tflops = flops / (total_ms * 1e-3) / 1e12
    valid_bytes = int(sl_host.sum()) * wl.d * 2
    return {"workload": wl.name, "rows": M, "prompts": wl.B, "valid_tokens": int(sl_host.sum()),
            "routed_linear_ms_by_site": [round(v, 3) for v in site_ms], "base_flops": flops,
            "tflops": round(tflops, 1), "frac_of_mfma_peak": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4),
            "route_ms": round(route_ms, 4),
            "route_pool_gbs": round(valid_bytes / (route_ms * 1e-3) / 1e9, 1)}


def bf16_bits(torch, synth, y64):
    """fp64 values -> the bf16 bit patterns a layer's output is stored as (the next layer's input)."""
    import numpy as np

    return synth.as_numpy(torch.from_numpy(np.ascontiguousarray(y64)).to(torch.bfloat16))


def row_rel_err(np, y, ref):
    denom = np.abs(ref).max(axis=1)
    return float((np.abs(y - ref).max(axis=1) / np.where(denom == 0, 1.0, denom)).max())


def copy_calibration(torch, dev):
    """A plain device copy of known size in the same process: what the byte counters read for it scales what they
    read for the kernels."""
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    dst.copy_(src)  # reads 1 GiB, writes 1 GiB
    torch.cuda.synchronize()
    del src, dst


def stack_bench(args, torch, mb, synth, wl, dev):
    """Multi-layer decode stacks (not the headline workload): every layer's packed weights and adapters resident
    in HBM, routes as a given table, one step = one token for all B requests through all L layers.  The oracle
    follows a seeded sample of the requests through the same stack on the host cores while the layers are being
    built (requests are independent rows through the whole chain): its time, scaled by B / sample, is the CPU
    baseline of one step."""
    import random

    import numpy as np

    tid_host = synth.tenant_ids(wl)
    tid = tid_host.to(dev)
    table_host = synth.constructed_routes(wl)
    table = table_host.to(dev)
    x0 = synth.decode_input(wl, 0, dev)
    cpu_on = not args.no_cpu_baseline
    sample = sorted(random.Random(0).sample(range(wl.B), min(wl.B, 32)))
    if cpu_on:
        import oracle

        xr = synth.as_numpy(x0[sample])
        tid_s = np.arange(len(sample), dtype=np.int32)
        t_cpu, y_first_ref, y_last_ref = 0.0, None, None
    layers, nbytes = [], 0
    for layer in range(wl.L):
        W = synth.base_weights(wl, layer, dev)
        Wp = [mb.milora_pack_weight(w) for w in W]
        ad = synth.adapters(wl, layer, dev)
        tab = mb.AdapterTable.from_tensors(ad.A, ad.B, ad.rank)
        layers.append((Wp, ad, tab))
        nbytes += algorithmic_bytes(wl, table_host[layer].numpy(), tid_host.numpy(), ad.rank)["layer_step"]
        if cpu_on:
            Wn = [synth.as_numpy(w) for w in W]
            sub = [int(tid_host[b]) for b in sample]
            adn = oracle.Adapters([[synth.as_numpy(a) for a in ad.A[t]] for t in sub],
                                  [[synth.as_numpy(b) for b in ad.B[t]] for t in sub], [ad.rank[t] for t in sub])
            t0 = time.perf_counter()
            y_ref, _ = oracle.layer_decode(xr, Wn, adn, tid_s, table_host[layer][sample].numpy(), wl.F,
                                           flags=oracle.FLAG_RMSNORM if wl.rmsnorm else 0)
            t_cpu += time.perf_counter() - t0
            xr = bf16_bits(torch, synth, y_ref)
            if layer == 0:
                y_first_ref = y_ref
            y_last_ref = y_ref
            del Wn, adn
        del W
    ws = torch.zeros(mb.layer_decode_workspace_bytes(wl.B, wl.d, wl.F, max(wl.ranks)), dtype=torch.uint8, device=dev)
    bufs = [torch.empty_like(x0), torch.empty_like(x0)]
    qkv = torch.empty(wl.B, 3 * wl.d, dtype=x0.dtype, device=dev)

    def step():
        x = x0
        for layer, (Wp, ad, tab) in enumerate(layers):
            y = bufs[layer & 1]
            mb.milora_layer_decode(x, Wp, tab, tid, table[layer], wl.F, w_layout=mb.W_PACKED, rmsnorm=wl.rmsnorm, y=y,
                                   qkv_out=qkv, workspace=ws)
            x = y

    if args.copy_calibration:
        copy_calibration(torch, dev)
    step()
    torch.cuda.synchronize()
    parity = None
    if cpu_on:
        y_last = bufs[(wl.L - 1) & 1][sample].double().cpu().numpy()
        y_first, _ = mb.milora_layer_decode(x0, layers[0][0], layers[0][2], tid, table[0], wl.F, w_layout=mb.W_PACKED,
                                            rmsnorm=wl.rmsnorm, workspace=ws)
        parity = {"sampled_requests": len(sample),
                  "first_layer_worst_row_rel_err": row_rel_err(np, y_first[sample].double().cpu().numpy(), y_first_ref),
                  "free_running_chains_after_all_layers": row_rel_err(np, y_last, y_last_ref)}
    run = step
    if not args.no_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        run = graph.replay
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    status = mb.milora_packed_workspace_status(ws)
    assert status == 0, "a hand-over inside a decode launch timed out: the figures would be of wrong results"
    # the launches one by one, HIP events on the launch stream around each (the step above is one graph)
    _, _, slot_ms = mb.milora_layer_decode(x0, layers[0][0], layers[0][2], tid, table[0], wl.F, w_layout=mb.W_PACKED,
                                           rmsnorm=wl.rmsnorm, y=bufs[0], qkv_out=qkv, workspace=ws,
                                           profile_reps=args.profile_reps)
    achieved = nbytes / (ms * 1e-3) / 1e9
    cpu = None
    if cpu_on:
        cpu_step_s = t_cpu * wl.B / len(sample)
        cpu = {"value": round(wl.B / cpu_step_s, 2), "unit": "tokens/s", "cores": min(oracle.n_threads(), len(sample)),
               "kind": "oracle",
               "sample": f"one decode step of {len(sample)} of the {wl.B} requests through all {wl.L} layers "
                         f"({t_cpu:.1f} s), scaled by {wl.B}/{len(sample)} (requests are independent rows)"}
    kernel = "decode_wide_kernel" if wl.B > 32 else "decode_stream_kernel"
    traffic = measured_traffic(wl.name)
    print(json.dumps({
        "metric": "routed-LoRA decode tokens/s through the layer stack + % HBM roofline", "value": round(wl.B / (ms * 1e-3), 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "layers": wl.L, "d": wl.d, "ffn": wl.F, "batch": wl.B, "tenants": wl.T,
                   "ranks": list(wl.ranks), "routes": "constructed table", "hip_graph": not args.no_graph},
        "roofline": {"bound": "hbm", "kernel": kernel + " (L launches per step)", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": None if traffic is None else traffic * wl.L,
                     "algorithmic_bytes_per_step": nbytes, "us_per_layer": round(ms * 1e3 / wl.L, 2),
                     "first_layer_launch_us": round(slot_ms[0] * 1e3, 2)},
        "cpu_baseline": cpu, "parity": parity}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama7b_layer_b32")
    ap.add_argument("--batch", type=int, default=0,
                    help="single-layer workloads: run the layer with this many requests (and as many tenants) "
                         "instead of the workload's own batch, e.g. 64 or 128 on llama7b_layer_b32")
    ap.add_argument("--phases", action="store_true",
                    help="single-layer workloads: also run one decode step on the tracing build of the kernel and "
                         "report when the workgroups reach each phase of each stage (median, last; us)")
    ap.add_argument("--no-graph", action="store_true", help="launch every call from Python instead of a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prefill", action="store_true", help="skip the many-row (prefill configuration) leg")
    ap.add_argument("--profile-reps", type=int, default=50)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch one plain 1 GiB device copy, the known-size kernel that hardware byte "
                         "counters are scaled against")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build runs on a single MI355X and has no multi-GPU path "
              "(use --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2410_18035_amd import binding as mb
    from paper_2410_18035_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU: there is no CPU fallback of the HIP path", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    wl = synth.CONFIGS[args.workload]
    assert wl.dtype == "bf16" and wl.decode_steps > 0, "the benchmark runs the bf16 decode configurations"
    if args.batch and wl.L == 1:
        import dataclasses

        wl = dataclasses.replace(wl, name=f"{wl.name.rsplit('_b', 1)[0]}_b{args.batch}", B=args.batch, T=args.batch)
    if wl.L > 1:
        stack_bench(args, torch, mb, synth, wl, dev)
        return
    nsteps = wl.decode_steps

    # ---- inputs, resident in HBM -----------------------------------------------------------------
    W = synth.base_weights(wl, 0, dev)
    Wp = [mb.milora_pack_weight(w) for w in W]
    ad = synth.adapters(wl, 0, dev)
    tab = mb.AdapterTable.from_tensors(ad.A, ad.B, ad.rank)
    Wr = synth.router_weights(wl, 0, dev)
    tid_host = synth.tenant_ids(wl)
    tid = tid_host.to(dev)
    H, ss_host, sl_host = synth.prompts(wl, 0, dev)
    ss, sl = ss_host.to(dev), sl_host.to(dev)
    xs = torch.stack([synth.decode_input(wl, s, dev) for s in range(nsteps)])
    ys = torch.empty_like(xs)
    qkv = torch.empty(wl.B, 3 * wl.d, dtype=xs.dtype, device=dev)
    route = torch.empty(wl.B, dtype=torch.uint8, device=dev)
    ws_route = torch.empty(mb.route_workspace_bytes(wl.B, wl.d, H.shape[0]), dtype=torch.uint8, device=dev)
    ws_layer = torch.zeros(mb.layer_decode_workspace_bytes(wl.B, wl.d, wl.F, tab.r_max), dtype=torch.uint8, device=dev)

    def hot_path_step():
        mb.milora_route(H, ss, sl, tid, Wr, wl.pool, wl.act, route_out=route, want_logits=False, workspace=ws_route)
        for s in range(nsteps):
            mb.milora_layer_decode(xs[s], Wp, tab, tid, route, wl.F, w_layout=mb.W_PACKED, rmsnorm=wl.rmsnorm,
                                   y=ys[s], qkv_out=qkv, workspace=ws_layer)

    hot_path_step()
    torch.cuda.synchronize()
    run = hot_path_step
    graph = None
    if not args.no_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            hot_path_step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            hot_path_step()
        run = graph.replay

    if args.copy_calibration:
        copy_calibration(torch, dev)

    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    tokens_per_step = wl.B * nsteps
    value = tokens_per_step / (ms_per_step * 1e-3)

    # ---- per-launch durations with HIP events on the launch stream -----------------------------
    route_host = route.cpu().numpy()
    nbytes = algorithmic_bytes(wl, route_host, tid_host.numpy(), ad.rank)
    _, _, slot_ms = mb.milora_layer_decode(xs[0], Wp, tab, tid, route, wl.F, w_layout=mb.W_PACKED, rmsnorm=wl.rmsnorm,
                                           y=ys[0], qkv_out=qkv, workspace=ws_layer, profile_reps=args.profile_reps)
    # route launches timed with events around the call
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(20):
        mb.milora_route(H, ss, sl, tid, Wr, wl.pool, wl.act, route_out=route, want_logits=False, workspace=ws_route)
    e1.record()
    torch.cuda.synchronize()
    route_ms = e0.elapsed_time(e1) / 20
    dominant_ms = slot_ms[0]  # the one launch that walks the four stages of the layer
    achieved = nbytes["layer_step"] / (dominant_ms * 1e-3) / 1e9
    layer_ms = sum(slot_ms)
    decode_ms_in_step = (ms_per_step - route_ms) / nsteps
    assert mb.milora_packed_workspace_status(ws_layer) == 0, \
        "a hand-over inside a decode launch timed out: the figures would be of wrong results"
    kernel = "decode_wide_kernel" if wl.B > 32 else "decode_stream_kernel"
    roofline = {"bound": "hbm", "kernel": kernel + " (one decode step of the layer)", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": measured_traffic(wl.name),
                "algorithmic_bytes_per_launch": nbytes["layer_step"], "avg_launch_ms": round(dominant_ms, 5)}

    phases = None
    if args.phases:
        for _ in range(3):
            stamps = mb.milora_layer_decode_trace(xs[0], Wp, tab, tid, route, wl.F, ys[0], qkv, ws_layer, rmsnorm=wl.rmsnorm)
        phases = phase_table(np, stamps, wl.B > 32)

    # ---- the oracle on the host cores, bounded sample ---------------------------------------------
    cpu, parity = None, None
    if not args.no_cpu_baseline:
        import oracle

        Wn = [synth.as_numpy(w) for w in W]
        A, Bm, rank = synth.adapters_as_numpy(ad)
        adn = oracle.Adapters(A, Bm, rank)
        Hn, Wrn = synth.as_numpy(H), synth.as_numpy(Wr)
        t0 = time.perf_counter()
        ref = oracle.route(Hn, ss_host.numpy(), sl_host.numpy(), tid_host.numpy(), Wrn, mb.POOL[wl.pool], mb.ACT[wl.act])
        t_route = time.perf_counter() - t0
        # decode reuses the cached table: the oracle gets the routes the GPU's router wrote
        margin = 1e-3 * float(ref.logits.std())
        keep = ref.gap >= margin
        done, t_dec, worst = 0, 0.0, 0.0
        while done < nsteps and (done < 1 or t_dec + t_dec / done < 20.0):
            t0 = time.perf_counter()
            y_ref, _ = oracle.layer_decode(synth.as_numpy(xs[done]), Wn, adn, tid_host.numpy(), route_host, wl.F,
                                           flags=oracle.FLAG_RMSNORM if wl.rmsnorm else 0)
            t_dec += time.perf_counter() - t0
            worst = max(worst, row_rel_err(np, ys[done].double().cpu().numpy(), y_ref))
            done += 1
        parity = {"routes_differing_outside_margin": int((keep & (route_host != ref.route)).sum()),
                  "routes_excluded_as_near_ties": int((~keep).sum()), "route_margin": margin,
                  "decode_steps_checked": done, "worst_row_rel_err": worst}
        cpu_step_s = t_route + t_dec / done * nsteps
        cpu = {"value": round(tokens_per_step / cpu_step_s, 2), "unit": "tokens/s", "cores": oracle.n_threads(),
               "kind": "oracle",
               "sample": f"router on all {wl.B} prompts ({t_route:.2f} s) + {done} of the {nsteps} decode steps "
                         f"({t_dec / done:.2f} s each), all {wl.B} requests; scaled to {nsteps} steps"}

    # ---- what the GPU sustains on the two bounding resources, and the many-row leg ------------------
    big = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    ceilings = {"hbm_read_gbs": round(mb.milora_measure_read_rate(big, reps=5), 1),
                "mfma_bf16_tflops": round(mb.milora_measure_matrix_rate(
                    4000, dev, shape=mb.MFMA_32X32X16 + mb.MFMA_MIXED_OPERANDS), 1),
                "mfma_bf16_tflops_small_integer_operands": round(mb.milora_measure_matrix_rate(
                    4000, dev, shape=mb.MFMA_32X32X16), 1)}
    del big
    roofline["frac_of_measured_read_rate"] = round(achieved / ceilings["hbm_read_gbs"], 4)
    prefill = None
    if not args.no_prefill:
        del W, Wp, xs, ys
        torch.cuda.empty_cache()
        prefill = prefill_leg(torch, mb, synth, dev)
        prefill["frac_of_measured_mfma_rate"] = round(prefill["tflops"] / ceilings["mfma_bf16_tflops"], 4)

    out = {
        "metric": "routed-LoRA decode tokens/s (batch 32, 32 tenants) + % HBM roofline",
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "shape": "LLaMA-2-7B single layer", "d": wl.d, "ffn": wl.F, "batch": wl.B,
                   "tenants": wl.T, "rank": wl.ranks[0], "prompt_len": wl.prompt_len[0], "decode_steps": nsteps,
                   "tokens_per_step": tokens_per_step, "weights": "bf16 packed", "hip_graph": graph is not None},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "parity": parity,
        "measured_ceilings": ceilings,
        "prefill": prefill,
        "layer_step": {"us_in_timed_region": round(decode_ms_in_step * 1e3, 2),
                       "us_sum_of_launches": round(layer_ms * 1e3, 2),
                       "algorithmic_bytes": nbytes["layer_step"],
                       "hbm_frac_in_timed_region": round(nbytes["layer_step"] / (decode_ms_in_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                       "launch_us": [round(v * 1e3, 2) for v in slot_ms],
                       "route_call_us": round(route_ms * 1e3, 2)},
        "tokens_per_s_32_layer_equivalent_extrapolated": round(value / 32, 1),
    }
    if phases is not None:
        out["phases_us_median_and_last_workgroup"] = phases
    print(json.dumps(out))


if __name__ == "__main__":
    main()
