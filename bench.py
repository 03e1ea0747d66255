#!/usr/bin/env python3
"""Throughput of the Expected-Attention compress pass on one MI355X.

A step = the whole hot path (statistics -> scores -> selection -> in-place compaction) over
every layer of a synthetic Llama-3.1-8B-shaped cache (32 layers x 8 KV heads x 131072 tokens x
head_dim 128, bf16, about 16 GiB of K+V), layer by layer through ea_compress_layer, at
compression ratio 0.5.  Inputs are resident in HBM before the timed region; the cache is
restored from a pristine copy between steps, outside the timed region (compaction is in place).
Layers are independent and of one shape, so consecutive layers go to one call as a batch
(--layer-batch, default 4: they are contiguous in memory and share positions and frequencies) and
the calls are issued round-robin on a few HIP streams (--streams, default 3), each with a workspace
of its own; the whole step is bracketed by device synchronisation.

Prints ONE JSON line: metric/value (G KV pairs scored+compacted per second), ms_per_step,
`roofline` for the dominant kernel (score pass A, HBM-bound: it streams every K and V row
once) with its average launch duration measured by HIP events on the launch stream in separate
one-stream instrumented steps (the duration of the kernel running alone), and
`cpu_baseline` (the fp64 oracle timed on this machine's host cores on one layer of the same input).

    python bench.py [--steps K] [--warmup W] [--workload c3|c2|c4|c5] [--ratio R] [--layers L] [--streams S] [--layer-batch LB]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published peak
MFMA_F16_PEAK_TFLOPS = 2500.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c3")
    ap.add_argument("--ratio", type=float, default=0.5)
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (0 = config's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--epsilon", type=float, default=0.02)
    ap.add_argument("--layer-batch", type=int, default=4,
                    help="consecutive layers handed to one ea_compress_layer call as a batch (same shape, "
                         "same positions, contiguous in memory): fewer, larger launches")
    ap.add_argument("--streams", type=int, default=3,
                    help="HIP streams the layers are spread over (each with its own workspace); layers "
                         "are independent, so the short latency-bound kernels of one layer overlap "
                         "with the streaming kernels of another")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step (all calls, one stream) in a HIP graph and time replays of it: "
                         "the launch-latency view for short caches (the library enqueues kernels only, "
                         "so its calls can be captured as they are)")
    return ap.parse_args()


def traffic_from_profile(name, layers_per_launch):
    """HBM bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc summary
    (FETCH_SIZE / WRITE_SIZE runs), if one exists for this workload and launch shape; else None."""
    path = os.path.join(ROOT, "profiles", "k_score_mfma_%s_pmc.txt" % name)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch[%d layers]:" % layers_per_launch):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the compress pass "
              "shards by KV head with no exchange); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import paper_2510_00636_amd as ea
    from ea_inputs import CONFIGS
    from ea_inputs.device import make_layer_device

    if not os.path.exists(ea.lib_path()):
        import __graft_entry__
        __graft_entry__.build()
    ea.load_library()
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    cfg = CONFIGS[a.workload]
    L = a.layers or cfg.layers
    B, Hq, Hkv, d, n, w = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.n, cfg.window
    n_keep = ea.n_keep(n, a.ratio)
    LB = max(1, a.layer_batch)
    while L % LB:
        LB -= 1
    p1 = ea.make_params(B, Hq, Hkv, d, ea.EA_BF16, horizon_T=cfg.horizon_T, epsilon=a.epsilon)
    p = ea.make_params(B * LB, Hq, Hkv, d, ea.EA_BF16, horizon_T=cfg.horizon_T, epsilon=a.epsilon)

    dev = "cuda"
    k0 = torch.empty(L, B, Hkv, n, d, dtype=torch.bfloat16, device=dev)     # pristine copies
    v0 = torch.empty_like(k0)
    q = torch.empty(L, B, Hq, w, d, dtype=torch.bfloat16, device=dev)
    inv = None
    for l in range(L):
        lay = make_layer_device(cfg, l, out_k=k0[l], out_v=v0[l], out_q=q[l])
        inv = lay["inv_freq"]
    k, v = torch.empty_like(k0), torch.empty_like(v0)
    ns = 1 if a.graph else max(1, min(a.streams, L // LB))
    wss = [torch.empty(ea.workspace_bytes(p, n, w), dtype=torch.uint8, device=dev) for _ in range(ns)]
    ws = wss[0]
    streams = [torch.cuda.Stream() for _ in range(ns)] if ns > 1 else [None]      # default priority
    q_pos0, t_next = n - w, n
    torch.cuda.synchronize()

    def restore():
        k.copy_(k0)
        v.copy_(v0)

    def step():
        # layer l runs on stream l % ns with that stream's workspace; the caller synchronises
        # the device before and after a step
        for i, l in enumerate(range(0, L, LB)):
            ea.compress_layer(p, q[l:l + LB], w, q_pos0, inv, t_next, k[l:l + LB], v[l:l + LB], n, n, n_keep,
                              None, None, wss[i % ns], stream=streams[i % ns])

    for _ in range(a.warmup):
        restore()
        torch.cuda.synchronize()
        step()
        torch.cuda.synchronize()
    if a.graph:
        cap = torch.cuda.Stream()
        streams = [cap]
        graph = torch.cuda.CUDAGraph()
        restore()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=cap):
            step()
        torch.cuda.synchronize()
        step = graph.replay
    times = []
    for _ in range(a.steps):
        restore()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        step()
        torch.cuda.synchronize()
        times.append(time.perf_counter() - t0)
    ms_per_step = 1e3 * sum(times) / len(times)
    pairs = L * B * Hkv * n
    value = pairs / (ms_per_step * 1e-3) / 1e9
    f = n_keep / n
    bytes_per_pair = 2 * d * 2 * (1 + 2 * f)                     # K,V read once + kept rows read+written
    path_hbm_frac = pairs * bytes_per_pair / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9)

    # ---- per-stage durations with HIP events on the launch stream (instrumented steps: the same
    #      calls as the timed steps, one after the other on one stream, so each kernel runs alone)
    stage = np.zeros(ea.binding.N_STAGES)
    nst = max(1, min(a.steps, 3))
    ncall = L // LB
    for _ in range(nst):
        restore()
        torch.cuda.synchronize()
        for l in range(0, L, LB):
            stage += np.array(ea.compress_layer_timed(p, q[l:l + LB], w, q_pos0, inv, t_next, k[l:l + LB],
                                                      v[l:l + LB], n, n, n_keep, ws))
    stage /= nst * ncall                                          # ms per launch (= per call of LB layers)
    score_ms = float(stage[2])
    score_bytes = LB * B * Hkv * n * 2 * d * 2                     # algorithmic: every K and V row once
    achieved = score_bytes / (score_ms * 1e-3) / 1e9
    G = Hq // Hkv
    flops = LB * B * Hkv * n * (G * (2 * d * d + 2 * d) + 2 * d)
    roofline = {"kernel": "k_score_mfma", "bound": "hbm", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic_from_profile(cfg.name, LB),
                "avg_launch_ms": round(score_ms, 4), "bytes_per_launch": score_bytes,
                "layers_per_launch": LB,
                "mfma_dense_tflops": round(flops / (score_ms * 1e-3) / 1e12, 1),
                "mfma_frac_of_f16_peak": round(flops / (score_ms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4)}
    stage /= LB                                                    # per layer from here on
    compact_bytes = B * Hkv * n_keep * 2 * d * 2 * 2
    stages = {nm: round(float(ms), 4) for nm, ms in zip(ea.STAGE_NAMES, stage)}
    stages["compact_GBs"] = round(compact_bytes / (float(stage[5]) * 1e-3) / 1e9, 1) if stage[5] > 0 else None

    out = {"metric": "KV pairs scored+compacted/sec", "value": round(value, 4), "unit": "G pairs/s",
           "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(ms_per_step, 4),
           "ms_per_step_p50": round(1e3 * float(np.median(times)), 4), "ms_per_step_max": round(1e3 * max(times), 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
           "data": "synthetic",
           "config": {"workload": "%s: %d layers x %d KV heads x %d tokens x d%d, Hq %d, window %d, "
                                  "ratio %.2f (keep %d), eps %.2f, in place, %d layer(s) per call, calls spread over %d streams%s" %
                                  (cfg.name, L, Hkv * B, n, d, Hq, w, a.ratio, n_keep, a.epsilon, LB, ns,
                                   ", one step replayed from a HIP graph" if a.graph else ""),
                      "pairs_per_step": pairs, "bytes_per_pair": bytes_per_pair},
           "path_hbm_frac": round(path_hbm_frac, 4),
           "stage_ms_per_layer": stages,
           "roofline": roofline}

    # ---- the oracle on this machine's host cores, on one layer of the same input
    if not a.no_cpu_baseline:
        from oracle import ea_oracle as O
        from ea_inputs import widen
        from ea_inputs.torch_io import to_host
        invh = inv.cpu().numpy()
        done, dt = 0, 0.0
        while done < L and dt < 12.0:                      # about 10-30 s of CPU work
            kq = widen(to_host(q[done]))
            kk, vv = to_host(k0[done]), to_host(v0[done])
            t0 = time.perf_counter()
            O.compress_layer(kq, widen(kk), widen(vv), q_pos0, invh, t_next, n_keep, T=cfg.horizon_T,
                             epsilon=a.epsilon, k_store=kk, v_store=vv)
            dt += time.perf_counter() - t0
            done += 1
        out["cpu_baseline"] = {"value": round(done * B * Hkv * n / dt / 1e9, 6), "unit": "G pairs/s",
                               "cores": len(os.sched_getaffinity(0)), "kind": "oracle",
                               "sample": "layers 0..%d of %d (%d pairs), full path incl. widening to "
                                         "fp64, %.1f s" % (done - 1, L, done * B * Hkv * n, dt)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
