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

# HBM bytes per launch of the decode kernel from the FETCH_SIZE and WRITE_SIZE hardware counters, each scaled
# by what the counter reads for a plain 1 GiB device copy (profiles/decode_layer_llama7b_b32_hbm_counters.txt).
# Valid only for the kernel source the counters were taken on: keyed by workload and source digest.
MEASURED_TRAFFIC = {
    ("llama7b_layer_b32", "397a6776a1f1db84"): {"fetch_bytes": 504844354, "write_bytes": 3694336},
}


def measured_traffic(workload):
    import hashlib

    src = os.path.join(ROOT, "paper_2410_18035_amd", "csrc", "decode.hip")
    try:
        digest = hashlib.sha256(open(src, "rb").read()).hexdigest()[:16]
    except OSError:
        return None
    m = MEASURED_TRAFFIC.get((workload, digest))
    return None if m is None else m["fetch_bytes"] + m["write_bytes"]


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


def stack_bench(args, torch, mb, synth, wl, dev):
    """Multi-layer decode stacks (not the headline workload): every layer's packed weights and adapters resident
    in HBM, routes as a given table, one step = one token for all B requests through all L layers."""
    tid = synth.tenant_ids(wl).to(dev)
    table = synth.constructed_routes(wl).to(dev)
    layers, nbytes = [], 0
    for layer in range(wl.L):
        W = synth.base_weights(wl, layer, dev)
        Wp = [mb.milora_pack_weight(w) for w in W]
        del W
        ad = synth.adapters(wl, layer, dev)
        tab = mb.AdapterTable.from_tensors(ad.A, ad.B, ad.rank)
        layers.append((Wp, ad, tab))
        nbytes += algorithmic_bytes(wl, table[layer].cpu().numpy(), tid.cpu().numpy(), ad.rank)["layer_step"]
    ws = torch.zeros(mb.layer_decode_workspace_bytes(wl.B, wl.d, wl.F, max(wl.ranks)), dtype=torch.uint8, device=dev)
    x0 = synth.decode_input(wl, 0, dev)
    bufs = [torch.empty_like(x0), torch.empty_like(x0)]
    qkv = torch.empty(wl.B, 3 * wl.d, dtype=x0.dtype, device=dev)

    def step():
        x = x0
        for layer, (Wp, ad, tab) in enumerate(layers):
            y = bufs[layer & 1]
            mb.milora_layer_decode(x, Wp, tab, tid, table[layer], wl.F, w_layout=mb.W_PACKED, rmsnorm=wl.rmsnorm, y=y,
                                   qkv_out=qkv, workspace=ws)
            x = y

    step()
    torch.cuda.synchronize()
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
    achieved = nbytes / (ms * 1e-3) / 1e9
    print(json.dumps({
        "metric": "routed-LoRA decode tokens/s through the layer stack + % HBM roofline", "value": round(wl.B / (ms * 1e-3), 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "layers": wl.L, "d": wl.d, "ffn": wl.F, "batch": wl.B, "tenants": wl.T,
                   "ranks": list(wl.ranks), "routes": "constructed table", "hip_graph": not args.no_graph},
        "roofline": {"bound": "hbm", "kernel": ("decode_wide_kernel" if wl.B > 32 else "decode_stream_kernel") + " (L launches per step)", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes_per_step": nbytes, "us_per_layer": round(ms * 1e3 / wl.L, 2)},
        "cpu_baseline": None}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama7b_layer_b32")
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
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)  # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

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
    roofline = {"bound": "hbm", "kernel": "decode_stream_kernel (one decode step of the layer)", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": measured_traffic(wl.name),
                "algorithmic_bytes_per_launch": nbytes["layer_step"], "avg_launch_ms": round(dominant_ms, 5)}

    # ---- the oracle on the host cores, bounded sample ---------------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        Wn = [synth.as_numpy(w) for w in W]
        A, Bm, rank = synth.adapters_as_numpy(ad)
        adn = oracle.Adapters(A, Bm, rank)
        Hn, Wrn = synth.as_numpy(H), synth.as_numpy(Wr)
        t0 = time.perf_counter()
        ref = oracle.route(Hn, ss_host.numpy(), sl_host.numpy(), tid_host.numpy(), Wrn, mb.POOL[wl.pool], mb.ACT[wl.act])
        t_route = time.perf_counter() - t0
        done, t_dec = 0, 0.0
        while done < nsteps and (done < 1 or t_dec + t_dec / done < 20.0):
            t0 = time.perf_counter()
            oracle.layer_decode(synth.as_numpy(xs[done]), Wn, adn, tid_host.numpy(), ref.route, wl.F,
                                flags=oracle.FLAG_RMSNORM if wl.rmsnorm else 0)
            t_dec += time.perf_counter() - t0
            done += 1
        cpu_step_s = t_route + t_dec / done * nsteps
        cpu = {"value": round(tokens_per_step / cpu_step_s, 2), "unit": "tokens/s", "cores": oracle.n_threads(),
               "kind": "oracle",
               "sample": f"router on all {wl.B} prompts ({t_route:.2f} s) + {done} of the {nsteps} decode steps "
                         f"({t_dec / done:.2f} s each), all {wl.B} requests; scaled to {nsteps} steps"}

    # ---- what the GPU sustains on the two bounding resources, and the many-row leg ------------------
    big = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    ceilings = {"hbm_read_gbs": round(mb.milora_measure_read_rate(big, reps=5), 1),
                "mfma_bf16_tflops": round(mb.milora_measure_matrix_rate(4000, dev), 1)}
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
    print(json.dumps(out))


if __name__ == "__main__":
    main()
