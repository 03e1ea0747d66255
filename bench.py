#!/usr/bin/env python3
"""Throughput of the Expected-Attention compress pass on one MI355X.

Default workload (c3): a step = the whole hot path (statistics -> scores -> selection -> in-place
compaction) over every layer of a synthetic Llama-3.1-8B-shaped cache (32 layers x 8 KV heads x
131072 tokens x head_dim 128, bf16, about 16 GiB of K+V) through ea_compress_layer at compression
ratio 0.5.  Inputs are resident in HBM before the timed region; the cache is restored from a
pristine copy between steps, outside the timed region (compaction is in place).  Layers are
independent and of one shape, so consecutive layers go to one call as a batch (--layer-batch,
default 4: contiguous in memory, same positions and frequencies) and the calls are issued
round-robin on a few HIP streams (--streams, default 3), each with a workspace of its own.  The
same pass is also timed strictly layer by layer (one layer per call, one stream) and reported as
`layer_by_layer`.

--workload c5 drives the decode-time schedule instead: 48 layers of a Qwen-14B-shaped cache that
grows from 2048 to 32768 positions; every 512 generated tokens the last 512 queries give the
statistics and the cache (then 4608 pairs per head) is compressed back to 4096.  A step is the
whole schedule (56 real passes; the passes while the cache is still within its budget do nothing);
appending the new tokens is the model's work and outside the timed region.

Prints ONE JSON line: metric/value (G KV pairs scored+compacted per second), ms_per_step,
`roofline` for the dominant kernel (score pass A: it streams every K and V row once) with its
average launch duration measured by HIP events on the launch stream in separate one-stream
instrumented steps, `hbm_copy_ceiling_GBs` (a plain 2 GiB device copy on this machine) and
`cpu_baseline` (the fp64 oracle timed on this machine's host cores on a sample of the same input).

    python bench.py [--steps K] [--warmup W] [--workload c3|c2|c4|c5] [--ratio R] [--layers L]
                    [--streams S] [--layer-batch LB] [--ordered] [--graph] [--skip-layer-by-layer]
                    [--paged BLOCK | --fp8 | --adaptive FLOOR | --scorer knorm|streaming|keydiff | --literal]
The last line's options time variants of the pass (paged or 8-bit caches, head-adaptive budgets, a
comparison scorer in front of the same select + compact, Eq. 5 / Eq. 9 as printed from hidden states,
W_Q and W_o); their JSON line names the variant in config.workload.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published peak
MFMA_F16_PEAK_TFLOPS = 2500.0
SCORE_SOURCES = ("ea_score_hw.hip", "ea_score_mfma.h", "ea_score.hip", "ea_host.cpp")


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
    ap.add_argument("--layer-batch", type=int, default=0,
                    help="consecutive layers handed to one ea_compress_layer call as a batch (0 = 4 for the "
                         "prefill shapes, 24 for the decode schedule)")
    ap.add_argument("--streams", type=int, default=3,
                    help="HIP streams the calls are spread over (each with its own workspace)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step (all calls, one stream) in a HIP graph and time replays of it")
    ap.add_argument("--skip-layer-by-layer", action="store_true",
                    help="leave the layer-by-layer leg out (profiling runs: every launch then has one shape)")
    ap.add_argument("--paged", type=int, default=0, metavar="BLOCK",
                    help="prefill shapes: keep the cache in block pools of BLOCK rows behind a shuffled block "
                         "table and time ea_compress_layer_paged (0 = contiguous tensors)")
    ap.add_argument("--adaptive", type=float, default=-1.0, metavar="FLOOR",
                    help="prefill shapes: time ea_compress_layer_adaptive (one budget per layer shared by its KV "
                         "heads); FLOOR in [0, 1] = the share of n_keep every head keeps whatever its scores")
    ap.add_argument("--scorer", default="", choices=["", "knorm", "streaming", "keydiff"],
                    help="the pass with one of the comparison scorers in front of the same select + compact "
                         "(ea_score_baseline, ea_select, ea_compact per call)")
    ap.add_argument("--literal", action="store_true",
                    help="the pass as Eq. 5 and Eq. 9 are printed: statistics from a hidden-state buffer and W_Q, "
                         "scores weighted by ||W_o v|| (one layer per call: every layer has weights of its own)")
    ap.add_argument("--d-model", type=int, default=4096, help="--literal: width of the hidden states")
    ap.add_argument("--fp8", action="store_true",
                    help="prefill shapes: store K and V as e4m3 bytes with per-head scales and time "
                         "ea_compress_layer_fp8 (half the bytes per pair)")
    ap.add_argument("--ordered", action="store_true",
                    help="decode schedule: use the order-preserving compaction instead of the order-free one")
    return ap.parse_args()


def kernel_source_hash():
    h = hashlib.sha256()
    for f in SCORE_SOURCES:
        h.update(open(os.path.join(ROOT, "paper_2510_00636_amd", "csrc", f), "rb").read())
    return h.hexdigest()[:16]


def traffic_from_profile(name, layers_per_launch):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary of this
    workload, or None: also None when the summary was taken for other kernel sources than the ones
    in the tree now (it names their hash), so a stale figure is never printed."""
    text = None
    for fn in ("score_pass_a_%s_pmc.txt", "score_pass_a_%s_kernel_stats_pmc.txt"):
        try:
            text = open(os.path.join(ROOT, "profiles", fn % name)).read()
            break
        except OSError:
            pass
    if text is None:
        return None
    if "kernel_source_sha256_16: %s" % kernel_source_hash() not in text:
        return None
    for line in text.splitlines():
        if line.startswith("traffic_bytes_per_launch[%d layers]:" % layers_per_launch):
            return float(line.split(":")[1])
    return None


def copy_ceiling(torch):
    """A plain device-to-device copy of 2 GiB: read + written bytes per second, in GB/s."""
    src = torch.empty(1 << 31, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    src.random_(0, 255)
    for _ in range(2):
        dst.copy_(src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    return 5 * 2 * float(1 << 31) / (e0.elapsed_time(e1) * 1e-3) / 1e9


def timed(step, restore, steps, warmup, torch):
    for _ in range(warmup):
        restore()
        torch.cuda.synchronize()
        step()
        torch.cuda.synchronize()
    times = []
    for _ in range(steps):
        restore()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        step()
        torch.cuda.synchronize()
        times.append(time.perf_counter() - t0)
    return times


def score_flops(ea, p_one, n, d, G):
    """(executed, dense) matrix-core flops per key of the score pass: the kernels run nfrag 32x32x16
    steps per tile of 32 keys and pass (triangular Sigma tiling plus the extra tile); the dense count
    is G (2 d^2 + 2 d) of Eq. 7."""
    NF = (d // 32) * (d // 32 + 1)
    gh = {64: min(G, 8), 128: 4 if G % 4 == 0 else min(G, 5), 256: min(G, 2)}[d]
    passes = -(-G // gh)
    nfrag = gh * NF + 2 * (d // 16)
    return passes * nfrag * 1024.0, G * (2.0 * d * d + 2 * d)


def oracle_sample(cfg, q, k0, v0, inv, q_pos0, t_next, n_keep, eps, L, B, Hkv, n, budget_s=12.0):
    from oracle import ea_oracle as O
    from ea_inputs import widen
    from ea_inputs.torch_io import to_host
    invh = inv.cpu().numpy()
    done, dt = 0, 0.0
    while done < L and dt < budget_s:                      # about 10-30 s of CPU work
        kq = widen(to_host(q[done]))
        kk, vv = to_host(k0[done]), to_host(v0[done])
        t0 = time.perf_counter()
        O.compress_layer(kq, widen(kk), widen(vv), q_pos0, invh, t_next, n_keep, T=cfg.horizon_T,
                         epsilon=eps, k_store=kk, v_store=vv)
        dt += time.perf_counter() - t0
        done += 1
    try:
        import threadpoolctl
        blas = max([lib.get("num_threads", 1) for lib in threadpoolctl.threadpool_info()] or [1])
    except Exception:
        blas = None
    # the same sample's first layer once more on one thread
    one = None
    try:
        import threadpoolctl
        with threadpoolctl.threadpool_limits(limits=1):
            kq = widen(to_host(q[0]))
            kk, vv = to_host(k0[0]), to_host(v0[0])
            t0 = time.perf_counter()
            O.compress_layer(kq, widen(kk), widen(vv), q_pos0, invh, t_next, n_keep, T=cfg.horizon_T,
                             epsilon=eps, k_store=kk, v_store=vv)
            one = B * Hkv * n / (time.perf_counter() - t0) / 1e9
    except Exception:
        pass
    return {"value": round(done * B * Hkv * n / dt / 1e9, 6), "unit": "G pairs/s",
            "cores": len(os.sched_getaffinity(0)), "blas_threads": blas, "kind": "oracle",
            "one_thread_value": None if one is None else round(one, 6),
            "sample": "layers 0..%d of %d (%d pairs), full path incl. widening to fp64, %.1f s" %
                      (done - 1, L, done * B * Hkv * n, dt)}


# ------------------------------------------------------------------------------ prefill shapes
def run_prefill(a, torch, ea, cfg):
    import numpy as np
    from ea_inputs.device import make_layer_device
    L = a.layers or cfg.layers
    B, Hq, Hkv, d, n, w = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.n, cfg.window
    n_keep = ea.n_keep(n, a.ratio)
    LB = 1 if a.literal else max(1, a.layer_batch or 4)
    while L % LB:
        LB -= 1
    mk = lambda lb: ea.make_params(B * lb, Hq, Hkv, d, ea.EA_BF16, horizon_T=cfg.horizon_T, epsilon=a.epsilon)
    p, p1 = mk(LB), mk(1)
    dev = "cuda"
    k0 = torch.empty(L, B, Hkv, n, d, dtype=torch.bfloat16, device=dev)     # pristine copies
    v0 = torch.empty_like(k0)
    q = torch.empty(L, B, Hq, w, d, dtype=torch.bfloat16, device=dev)
    inv = None
    for l in range(L):
        inv = make_layer_device(cfg, l, out_k=k0[l], out_v=v0[l], out_q=q[l])["inv_freq"]
    k, v = torch.empty_like(k0), torch.empty_like(v0)
    ns = 1 if a.graph else max(1, min(a.streams, L // LB))
    wss = [torch.empty(ea.workspace_bytes(p, n, w), dtype=torch.uint8, device=dev) for _ in range(ns)]
    streams = [torch.cuda.Stream() for _ in range(ns)] if ns > 1 else [None]      # default priority
    q_pos0, t_next = n - w, n
    torch.cuda.synchronize()

    pg_of = None
    if a.paged:
        # one pool for the whole cache: every (layer, sequence) is a sequence of the block table
        bs = a.paged
        assert n % bs == 0, "--paged: the block size must divide n here"
        mb = n // bs
        nblk = L * B * mb
        perm = torch.randperm(nblk, device=dev, generator=torch.Generator(device=dev).manual_seed(7))
        table = perm.to(torch.int32).reshape(L * B, mb).contiguous()

        def to_pool(t):        # [L, B, Hkv, n, d] -> [nblk, Hkv, bs, d], logical block j of sequence s at perm[s*mb+j]
            blocks = t.reshape(L * B, Hkv, mb, bs, d).permute(0, 2, 1, 3, 4).reshape(nblk, Hkv, bs, d)
            pool = torch.empty_like(blocks)
            pool[perm.long()] = blocks
            return pool
        k0p, v0p = to_pool(k0), to_pool(v0)
        del k0, v0, k, v
        k0, v0 = k0p, v0p
        k, v = torch.empty_like(k0), torch.empty_like(v0)
        pg_of = lambda l, lb: ea.make_paged(table[l * B:(l + lb) * B], bs, nblk)

    scales = None
    if a.fp8:
        def quant(t):          # [L, B, Hkv, n, d] bf16 -> e4m3 bytes + fp32 scale per (layer, sequence, head)
            sc = (t.abs().amax(dim=(3, 4), keepdim=True).float() / (448.0 * 0.9)).clamp_min(1e-30)
            out = torch.empty(t.shape, dtype=torch.float8_e4m3fn, device=dev)
            for l in range(L):
                out[l] = (t[l].float() / sc[l]).to(torch.float8_e4m3fn)
            return out, sc.reshape(L, B, Hkv).contiguous()
        k8, ksc = quant(k0)
        v8, vsc = quant(v0)
        del k0, v0, k, v
        k0, v0 = k8, v8
        k, v = torch.empty_like(k0), torch.empty_like(v0)
        scales = (ksc, vsc)

    def restore():
        k.copy_(k0)
        v.copy_(v0)

    def step_fp8():
        for i, l in enumerate(range(0, L, LB)):
            ea.compress_layer_fp8(p, q[l:l + LB], w, q_pos0, inv, t_next, k[l:l + LB], v[l:l + LB],
                                  scales[0][l:l + LB], scales[1][l:l + LB], n, n, n_keep, 0, None, None, None,
                                  wss[i % ns], stream=streams[i % ns])

    adapt = None
    if a.adaptive >= 0:
        floor = int(a.adaptive * n_keep)
        adapt = [(torch.empty(B * LB, Hkv, n, dtype=torch.int32, device=dev),
                  torch.empty(B * LB, Hkv, dtype=torch.int32, device=dev)) for _ in range(ns)]

        def step_adaptive():
            for i, l in enumerate(range(0, L, LB)):
                ea.compress_layer_adaptive(p, q[l:l + LB], w, q_pos0, inv, t_next, k[l:l + LB], v[l:l + LB], n, n,
                                           n_keep, floor, None, adapt[i % ns][0], adapt[i % ns][1], wss[i % ns],
                                           stream=streams[i % ns])

    alt = None
    if a.scorer or a.literal:
        sc_b = [torch.empty(B * LB, Hkv, n, dtype=torch.float32, device=dev) for _ in range(ns)]
        ix_b = [torch.empty(B * LB, Hkv, n_keep, dtype=torch.int32, device=dev) for _ in range(ns)]
    if a.scorer:
        kind = {"knorm": ea.SCORER_KNORM, "streaming": ea.SCORER_STREAMING, "keydiff": ea.SCORER_KEYDIFF}[a.scorer]

        def alt():
            for i, l in enumerate(range(0, L, LB)):
                j, st = i % ns, streams[i % ns]
                ea.score_baseline(p, kind, k[l:l + LB], n, n, 4, sc_b[j], wss[j], stream=st)
                ea.select(p, sc_b[j], n, n_keep, ix_b[j], wss[j], stream=st)
                ea.compact(p, k[l:l + LB], v[l:l + LB], n, n, ix_b[j], n_keep, k[l:l + LB], v[l:l + LB], wss[j],
                           stream=st)
    if a.literal:
        dm = a.d_model
        gen = torch.Generator(device=dev).manual_seed(11)
        rnd = lambda *sh: torch.randn(*sh, device=dev, generator=gen)
        hidden = (rnd(L, B, w, dm) * 1.5 + rnd(L, 1, 1, dm)).to(torch.bfloat16)
        w_q = (rnd(L, Hq, d, dm) / dm ** 0.5).to(torch.bfloat16)
        w_o = (rnd(L, Hq, dm, d) / d ** 0.5).to(torch.bfloat16)
        # W_o^T W_o is a constant of the model: taken once per layer, outside the timed region
        gram = torch.empty(L, Hq, d, d, dtype=torch.float32, device=dev)
        for l in range(L):
            ea.wo_gram(p, w_o[l], dm, gram[l])
        mu_b = [torch.empty(B, Hq, d, dtype=torch.float32, device=dev) for _ in range(ns)]
        sg_b = [torch.empty(B, Hq, d, d, dtype=torch.float32, device=dev) for _ in range(ns)]
        wn_b = [torch.empty(B, Hq, n, dtype=torch.float32, device=dev) for _ in range(ns)]

        def alt():
            for l in range(L):
                j, st = l % ns, streams[l % ns]
                ea.query_stats_hidden(p, hidden[l], w_q[l], dm, w, inv, t_next, mu_b[j], sg_b[j], wss[j], stream=st)
                ea.value_norms_wo(p, v[l], n, n, gram[l], wn_b[j], wss[j], stream=st)
                ea.score_wo(p, k[l], v[l], n, n, mu_b[j], sg_b[j], wn_b[j], sc_b[j], wss[j], stream=st)
                ea.select(p, sc_b[j], n, n_keep, ix_b[j], wss[j], stream=st)
                ea.compact(p, k[l], v[l], n, n, ix_b[j], n_keep, k[l], v[l], wss[j], stream=st)

    def step_paged():
        for i, l in enumerate(range(0, L, LB)):
            ea.compress_layer_paged(p, q[l:l + LB], w, q_pos0, inv, t_next, k, v, pg_of(l, LB), n, n_keep, 0, None,
                                    None, None, wss[i % ns], stream=streams[i % ns])

    def step():
        if a.paged:
            return step_paged()
        if a.fp8:
            return step_fp8()
        if adapt is not None:
            return step_adaptive()
        if alt is not None:
            return alt()
        # call i runs on stream i % ns with that stream's workspace; the caller synchronises the
        # device before and after a step
        for i, l in enumerate(range(0, L, LB)):
            ea.compress_layer(p, q[l:l + LB], w, q_pos0, inv, t_next, k[l:l + LB], v[l:l + LB], n, n, n_keep,
                              None, None, wss[i % ns], stream=streams[i % ns])

    def step_layer_by_layer():
        for l in range(L):
            ea.compress_layer(p1, q[l], w, q_pos0, inv, t_next, k[l], v[l], n, n, n_keep, None, None, wss[0])

    if a.graph:
        timed(step, restore, 0, a.warmup, torch)
        cap = torch.cuda.Stream()
        streams = [cap]
        graph = torch.cuda.CUDAGraph()
        restore()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=cap):
            step()
        torch.cuda.synchronize()
        times = timed(graph.replay, restore, a.steps, 0, torch)
    else:
        times = timed(step, restore, a.steps, a.warmup, torch)
    ms_per_step = 1e3 * sum(times) / len(times)
    pairs = L * B * Hkv * n
    f = n_keep / n
    bytes_per_pair = 2 * d * (1 if a.fp8 else 2) * (1 + 2 * f)    # K,V read once + kept rows read+written
    frac = lambda ms: pairs * bytes_per_pair / (ms * 1e-3) / (HBM_PEAK_GBS * 1e9)

    layer_by_layer = None
    if alt is not None:
        if a.scorer:
            bpp = 2 * d * 2 * ((0 if a.scorer == "streaming" else 0.5) + 2 * f)   # K read once (not at all by position)
            what = ("%s scores (ea_score_baseline) + ea_select + ea_compact" % a.scorer)
        else:
            bpp = 2 * d * 2 * (1 + 2 * f)        # V once for ||W_o v||, K once for the logits, kept rows read + written
            what = ("Eq. 5 from hidden states [%d, %d] and W_Q, Eq. 9 with ||W_o v|| (ea_query_stats_hidden, "
                    "ea_value_norms_wo, ea_score_wo, ea_select, ea_compact)" % (w, a.d_model))
        return {"metric": "KV pairs scored+compacted/sec", "value": round(pairs / (ms_per_step * 1e-3) / 1e9, 4),
                "unit": "G pairs/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
                "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
                "dtype": "bf16", "data": "synthetic",
                "config": {"workload": "%s, %s: %d layers x %d KV heads x %d tokens x d%d, ratio %.2f, %d layer(s) per "
                                       "call, %d streams" % (cfg.name, what, L, Hkv * B, n, d, a.ratio, LB, ns),
                           "pairs_per_step": pairs, "bytes_per_pair": bpp},
                "path_hbm_frac": round(pairs * bpp / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9), 4)}
    if a.paged or a.fp8 or adapt is not None:
        out = {"metric": "KV pairs scored+compacted/sec", "value": round(pairs / (ms_per_step * 1e-3) / 1e9, 4),
               "unit": "G pairs/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
               "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
               "dtype": "fp8 cache, fp16 matrix-core operands" if a.fp8 else "bf16", "data": "synthetic",
               "config": {"workload": ("%s, paged: %d layers x %d KV heads x %d tokens x d%d in pools of %d-row blocks "
                                       "behind a shuffled block table, ratio %.2f, %d layer(s) per call, %d streams" %
                                       (cfg.name, L, Hkv * B, n, d, a.paged, a.ratio, LB, ns)) if a.paged else
                                      ("%s, head-adaptive budgets (ea_compress_layer_adaptive, floor %d of %d per head): "
                                       "%d layers x %d KV heads x %d tokens x d%d, ratio %.2f, %d layer(s) per call, %d "
                                       "streams; lengths of the last call %s" %
                                       (cfg.name, int(a.adaptive * n_keep), n_keep, L, Hkv * B, n, d, a.ratio, LB, ns,
                                        adapt[(L // LB - 1) % ns][1][0].tolist())) if adapt is not None else
                                      ("%s, K and V stored as e4m3 bytes with per-head scales: %d layers x %d KV heads x "
                                       "%d tokens x d%d, ratio %.2f, %d layer(s) per call, %d streams" %
                                       (cfg.name, L, Hkv * B, n, d, a.ratio, LB, ns)),
                          "pairs_per_step": pairs, "bytes_per_pair": bytes_per_pair},
               "path_hbm_frac": round(frac(ms_per_step), 4)}
        return out
    if not a.skip_layer_by_layer:
        lbl_times = timed(step_layer_by_layer, restore, max(2, min(a.steps, 3)), 1, torch)
        lbl_ms = 1e3 * sum(lbl_times) / len(lbl_times)
        layer_by_layer = {"ms_per_step": round(lbl_ms, 4), "value": round(pairs / (lbl_ms * 1e-3) / 1e9, 4),
                          "unit": "G pairs/s", "path_hbm_frac": round(frac(lbl_ms), 4),
                          "launch_shape": "1 layer per call, 1 stream"}

    # ---- the same pass with the order-free compaction as its last step (legal by Eq. 2-3: attention
    #      is a sum over cached pairs; about half as many rows move at these ratios).  Reported next
    #      to the headline, never as it: the metric's pass keeps the cache in position order.
    order_free = None
    if not a.skip_layer_by_layer:
        def step_order_free():
            for i, l in enumerate(range(0, L, LB)):
                ea.compress_layer_unordered(p, q[l:l + LB], w, q_pos0, inv, t_next, k[l:l + LB], v[l:l + LB], n, n,
                                            n_keep, None, None, None, wss[i % ns], stream=streams[i % ns])
        of_times = timed(step_order_free, restore, max(2, min(a.steps, 3)), 1, torch)
        of_ms = 1e3 * sum(of_times) / len(of_times)
        order_free = {"ms_per_step": round(of_ms, 4), "value": round(pairs / (of_ms * 1e-3) / 1e9, 4),
                      "unit": "G pairs/s", "note": "ea_compress_layer_unordered, same launch shape; kept rows below "
                      "n_keep stay in place, the others fill the evicted positions"}

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
                                                      v[l:l + LB], n, n, n_keep, wss[0]))
    stage /= nst * ncall                                          # ms per launch (= per call of LB layers)
    score_ms = float(stage[2])
    keys = LB * B * Hkv * n
    score_bytes = keys * 2 * d * 2                                # algorithmic: every K and V row once
    achieved = score_bytes / (score_ms * 1e-3) / 1e9
    G = Hq // Hkv
    fl_exec, fl_dense = score_flops(ea, p1, n, d, G)
    roofline = {"kernel": "score pass A (k_score_hw / k_score_mfma)", "bound": "hbm", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic_from_profile(cfg.name, LB),
                "avg_launch_ms": round(score_ms, 4), "bytes_per_launch": score_bytes,
                "layers_per_launch": LB,
                "mfma_executed_tflops": round(keys * fl_exec / (score_ms * 1e-3) / 1e12, 1),
                "mfma_frac_of_f16_peak": round(keys * fl_exec / (score_ms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4),
                "mfma_dense_equivalent_tflops": round(keys * fl_dense / (score_ms * 1e-3) / 1e12, 1)}
    stage /= LB                                                    # per layer from here on
    compact_bytes = B * Hkv * n_keep * 2 * d * 2 * 2
    stages = {nm: round(float(ms), 4) for nm, ms in zip(ea.STAGE_NAMES, stage)}
    stages["compact_GBs"] = round(compact_bytes / (float(stage[5]) * 1e-3) / 1e9, 1) if stage[5] > 0 else None

    out = {"metric": "KV pairs scored+compacted/sec", "value": round(pairs / (ms_per_step * 1e-3) / 1e9, 4),
           "unit": "G pairs/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
           "ms_per_step": round(ms_per_step, 4), "ms_per_step_p50": round(1e3 * float(np.median(times)), 4),
           "ms_per_step_max": round(1e3 * max(times), 4), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "%s: %d layers x %d KV heads x %d tokens x d%d, Hq %d, window %d, ratio %.2f "
                                  "(keep %d), eps %.2f, in place, %d layer(s) per call, calls spread over %d "
                                  "streams%s" % (cfg.name, L, Hkv * B, n, d, Hq, w, a.ratio, n_keep, a.epsilon, LB,
                                                 ns, ", one step replayed from a HIP graph" if a.graph else ""),
                      "pairs_per_step": pairs, "bytes_per_pair": bytes_per_pair},
           "path_hbm_frac": round(frac(ms_per_step), 4), "layer_by_layer": layer_by_layer,
           "order_free_compaction": order_free,
           "stage_ms_per_layer": stages, "roofline": roofline}
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = oracle_sample(cfg, q, k0, v0, inv, q_pos0, t_next, n_keep, a.epsilon, L, B, Hkv, n)
    return out


# ------------------------------------------------------------------------------ decode schedule
def run_decode(a, torch, ea, cfg):
    """Config 5: positions 2048 -> 32768, a compress pass every 512 generated tokens over all layers:
    statistics from the last 512 queries (absolute positions), cache 4608 -> 4096 pairs per head."""
    import numpy as np
    from ea_inputs.device import make_layer_device
    L = a.layers or cfg.layers
    B, Hq, Hkv, d, w = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.window
    P0, P1, every, budget = 2048, 32768, 512, 4096
    n_cap = budget + every
    LB = max(1, a.layer_batch or 24)
    while L % LB:
        LB -= 1
    p = ea.make_params(B * LB, Hq, Hkv, d, ea.EA_BF16, horizon_T=cfg.horizon_T, epsilon=a.epsilon)
    dev = "cuda"
    kf = torch.empty(L, B, Hkv, P1, d, dtype=torch.bfloat16, device=dev)     # every token the model will produce
    vf = torch.empty_like(kf)
    qf = torch.empty(L, B, Hq, P1, d, dtype=torch.bfloat16, device=dev)
    inv = None
    for l in range(L):
        inv = make_layer_device(cfg, l, n=P1, window=P1, out_k=kf[l], out_v=vf[l], out_q=qf[l])["inv_freq"]
    k = torch.empty(L, B, Hkv, n_cap, d, dtype=torch.bfloat16, device=dev)    # the cache
    v = torch.empty_like(k)
    qw = torch.empty(L, B, Hq, w, d, dtype=torch.bfloat16, device=dev)
    ns = max(1, min(a.streams, L // LB))
    wss = [torch.empty(ea.workspace_bytes(p, n_cap, w), dtype=torch.uint8, device=dev) for _ in range(ns)]
    streams = [torch.cuda.Stream() for _ in range(ns)] if ns > 1 else [None]
    torch.cuda.synchronize()

    def one_pass(n, P):
        for i, l in enumerate(range(0, L, LB)):
            if a.ordered:
                ea.compress_layer(p, qw[l:l + LB], w, P - w, inv, P, k[l:l + LB], v[l:l + LB], n, n_cap, budget,
                                  None, None, wss[i % ns], stream=streams[i % ns])
            else:
                ea.compress_layer_unordered(p, qw[l:l + LB], w, P - w, inv, P, k[l:l + LB], v[l:l + LB], n, n_cap,
                                            budget, None, None, None, wss[i % ns], stream=streams[i % ns])

    def schedule(record):
        """The whole schedule; returns the per-pass seconds of the real passes."""
        n = P0
        k[:, :, :, :P0].copy_(kf[:, :, :, :P0])
        v[:, :, :, :P0].copy_(vf[:, :, :, :P0])
        per_pass, noops = [], 0
        for P in range(P0 + every, P1 + 1, every):
            k[:, :, :, n:n + every].copy_(kf[:, :, :, P - every:P])         # the model appends 512 tokens
            v[:, :, :, n:n + every].copy_(vf[:, :, :, P - every:P])
            n += every
            if n <= budget:
                noops += 1                                                  # within budget: nothing to do
                continue
            qw.copy_(qf[:, :, :, P - w:P])
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            one_pass(n, P)
            torch.cuda.synchronize()
            per_pass.append(time.perf_counter() - t0)
            n = budget
        return per_pass, noops

    for _ in range(max(1, a.warmup) if a.warmup else 0):
        schedule(False)
    steps = []
    for _ in range(a.steps):
        per_pass, noops = schedule(True)
        steps.append(per_pass)
    all_pass = np.array([t for s in steps for t in s])
    npass = len(steps[0])
    ms_per_step = 1e3 * float(np.mean([sum(s) for s in steps]))
    n = n_cap
    pairs_pass = L * B * Hkv * n
    f = budget / n
    bytes_per_pair = 2 * d * 2 * (1 + 2 * f)
    value = npass * pairs_pass / (ms_per_step * 1e-3) / 1e9

    # one more pass with stage timers (one stream), on a full cache
    k[:, :, :, :n].copy_(kf[:, :, :, :n])
    v[:, :, :, :n].copy_(vf[:, :, :, :n])
    qw.copy_(qf[:, :, :, n - w:n])
    torch.cuda.synchronize()
    stage = np.zeros(ea.binding.N_STAGES)
    for l in range(0, L, LB):
        stage += np.array(ea.compress_layer_timed(p, qw[l:l + LB], w, n - w, inv, n, k[l:l + LB], v[l:l + LB], n,
                                                  n_cap, budget, wss[0]))
    stage /= (L // LB)
    score_ms = float(stage[2])
    keys = LB * B * Hkv * n
    score_bytes = keys * 2 * d * 2
    G = Hq // Hkv
    fl_exec, fl_dense = score_flops(ea, p, n, d, G)
    achieved = score_bytes / (score_ms * 1e-3) / 1e9
    roofline = {"kernel": "score pass A (k_score_mfma)", "bound": "hbm", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic_from_profile(cfg.name, LB), "avg_launch_ms": round(score_ms, 4),
                "bytes_per_launch": score_bytes, "layers_per_launch": LB,
                "mfma_executed_tflops": round(keys * fl_exec / (score_ms * 1e-3) / 1e12, 1),
                "mfma_frac_of_f16_peak": round(keys * fl_exec / (score_ms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4),
                "mfma_dense_equivalent_tflops": round(keys * fl_dense / (score_ms * 1e-3) / 1e12, 1)}
    stages = {nm: round(float(ms) / LB, 4) for nm, ms in zip(ea.STAGE_NAMES, stage)}
    out = {"metric": "KV pairs scored+compacted/sec", "value": round(value, 4), "unit": "G pairs/s", "n_gpus": 1,
           "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(ms_per_step, 4),
           "ms_per_pass_mean": round(1e3 * float(all_pass.mean()), 4),
           "ms_per_pass_p50": round(1e3 * float(np.median(all_pass)), 4),
           "ms_per_pass_max": round(1e3 * float(all_pass.max()), 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "%s decode schedule: %d layers x %d KV heads, Hq %d, d%d, positions %d -> %d, a pass "
                                  "every %d tokens (window %d, absolute positions), cache %d -> %d pairs per head, "
                                  "%d real passes + %d within budget per step, %s compaction, eps %.2f, %d layer(s) "
                                  "per call, calls spread over %d streams; appends outside the timed region" %
                                  (cfg.name, L, Hkv * B, Hq, d, P0, P1, every, w, n, budget, npass, noops,
                                   "order-preserving" if a.ordered else "order-free", a.epsilon, LB, ns),
                      "pairs_per_step": npass * pairs_pass, "bytes_per_pair": bytes_per_pair},
           "path_hbm_frac": round(npass * pairs_pass * bytes_per_pair / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9), 4),
           "stage_ms_per_layer": stages, "roofline": roofline}
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = oracle_sample(cfg, qw, k, v, inv, n - w, n, budget, a.epsilon, L, B, Hkv, n)
    return out


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the compress pass "
              "shards by KV head with no exchange); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2510_00636_amd as ea
    from ea_inputs import CONFIGS

    if not os.path.exists(ea.lib_path()):
        import __graft_entry__
        __graft_entry__.build()
    ea.load_library()
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    cfg = CONFIGS[a.workload]
    out = run_decode(a, torch, ea, cfg) if a.workload == "c5" else run_prefill(a, torch, ea, cfg)
    out["hbm_copy_ceiling_GBs"] = round(copy_ceiling(torch), 1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
