#!/usr/bin/env python3
"""Benchmark of the Spotlight decode hot path on one MI355X.

A "step" is one decode step of one attention layer on synthetic, seeded inputs that are already
resident in HBM: append-hash of one new key per head, retrieval (query hash + Hamming scoring +
per-head top-k) and sparse attention over the selected rows.  The headline workload is config C3
(batch 1, 32 heads, 524288 cached tokens, 128-bit codes, top-k 10486, bf16 K/V), the one the
metric (retrieval time at 512K tokens / 32 heads) is quoted on.

Consecutive steps rotate over several independent "layers" (separate code / K / V tensors, at
least 1 GiB of codes in total) so that the 256 MB last-level cache cannot serve the code stream:
the numbers are HBM numbers, as in a model whose every layer is touched once per token.  The
retrieval time with ONE layer (codes that fit the last-level cache) is reported beside it as
`retrieve_us_hot_cache`; only the rotated number is compared with the roofline.

After the headline workload the default run measures the other bandwidth-sized workloads (C2, C4,
C5-128) with fewer steps and reports them under `other_workloads`.

Output: ONE JSON line.
"""
from __future__ import annotations

import argparse
import gc
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="C3", help="C1 | C2 | C3 | C4 | C5-128 | C5-512")
    ap.add_argument("--layers", type=int, default=0, help="independent layers to rotate over (0 = auto)")
    ap.add_argument("--code-bits", type=int, default=0, help="override the workload's code length L")
    ap.add_argument("--hidden", type=int, default=-1, help="override the hash MLP's hidden width (0 = linear hash sign(xR))")
    ap.add_argument("--lsh-init", default="", help="linear hash only: gaussian | rotation")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size")
    ap.add_argument("--no-prepack", action="store_true",
                    help="hash from the weight arrays as stored (no packed copy in the contexts)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-heads", type=int, default=6, help="heads in the oracle's timed sample (headline workload)")
    ap.add_argument("--others", default="auto",
                    help="comma-separated workloads measured after the headline one and reported under "
                         "other_workloads (auto: C2,C4,C5-128 when the headline is the plain C3 run; none: skip)")
    ap.add_argument("--other-steps", type=int, default=40, help="timed steps of each of the other workloads")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run 10 plain device copies of 1 GiB (a kernel of known HBM traffic, for "
                         "scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def gbps(nbytes, us):
    return nbytes / (us * 1e-6) / 1e9 if us else None


def stored_traffic(config_name, kernel):
    """HBM bytes per launch of `kernel` for this workload as rocprofv3's counters gave them in an
    earlier, committed run (profiles/hbm_traffic.txt): a stored figure, not measured by this run."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) == 6 and f[0] == config_name and f[1] == kernel:
            kv = dict(x.split("=") for x in f[2:])
            return int(1024 * (float(kv["fetch_kib"]) * float(kv["fetch_scale"]) +
                               float(kv["write_kib"]) * float(kv["write_scale"])))
    return None


def measure(cfg, args, steps, warmup, with_graph=True, calibrate_copy=False, hot_cache=False):
    """All measurements of one workload; returns a dict of plain numbers.  Tensors are freed on return."""
    import torch
    import workload as wl
    import paper_2508_19740_amd as sp

    dev = torch.device("cuda:0")
    B, Hq, Hkv, N, L, W, k, d = (cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.n_tokens, cfg.code_bits,
                                 cfg.words, cfg.topk, cfg.head_dim)
    esz = 2 if cfg.kv_dtype == "bf16" else 4
    kv_t = torch.bfloat16 if esz == 2 else torch.float32
    w_t = torch.bfloat16 if cfg.weight_dtype == "bf16" else torch.float32
    grow = cfg.extra_tokens > 0                     # C5: the cache grows by one token per step
    code_bytes = B * Hkv * N * L // 8
    layer_bytes = code_bytes + 2 * B * Hkv * cfg.max_tokens * d * esz
    if args.layers > 0:
        n_layers = args.layers
    else:
        n_layers = max(1, min(8, math.ceil((1 << 30) / code_bytes)))
        while n_layers > 1 and n_layers * layer_bytes > 120 * (1 << 30):
            n_layers -= 1

    # ------------------------------------------------------------------ inputs (untimed)
    t_setup = time.time()
    # One context per layer, as a model would hold them: each keeps the packed copy of its layer's
    # hash weights (spotlight_prepack_weights, made once here, untimed like the weights' upload).
    layers = []
    for li in range(n_layers):
        c = cfg.scaled(seed=cfg.seed + 1000 * li)
        w = wl.Workload(c)
        lay = {
            "w": w,
            "K": w.materialize("K", dev),
            "V": w.materialize("V", dev),
            "q": w.q.to(dev),
            "weights": tuple(None if t is None else t.to(dev) for t in w.hash_weights()),
            "codes": torch.zeros(B, Hkv, cfg.max_tokens, W, dtype=torch.int32, device=dev),
            "idx": torch.empty(B, Hq, k, dtype=torch.int32, device=dev),
            "out": torch.empty(B, Hq, d, dtype=torch.float32, device=dev),
            "ctx": sp.Spotlight(B, Hq, Hkv, L, cfg.hidden, cfg.max_tokens, k, kv_dtype=kv_t, weight_dtype=w_t, device=dev),
        }
        if not args.no_prepack:
            lay["ctx"].prepack_weights(*lay["weights"])
        layers.append(lay)
    torch.cuda.synchronize()
    t_gen = time.time() - t_setup

    def profile_enable(on):
        for lay in layers:
            lay["ctx"].profile_enable(on)

    def profile_read():   # totals over the layers' contexts
        tot = {name: [0.0, 0] for name in sp.STAGES}
        for lay in layers:
            for name, (ms, n) in lay["ctx"].profile_read().items():
                tot[name][0] += ms
                tot[name][1] += n
        return tot

    # bulk build of the code caches (setup, timed separately)
    profile_enable(True)
    for lay in layers:
        lay["ctx"].hash_keys(lay["K"], *lay["weights"], 0, N, lay["codes"])
    prof = profile_read()
    bulk_ms = prof["hash_keys"][0] / max(1, prof["hash_keys"][1])
    profile_enable(False)

    def step(i, ev=None, only_layer=None):
        lay = layers[i % n_layers if only_layer is None else only_layer]
        ctx = lay["ctx"]
        n_tok = N
        if grow:                                    # append one key per head, then retrieve over n+1
            j = (i // n_layers) % cfg.extra_tokens
            ctx.hash_keys(lay["K"], *lay["weights"], N + j, 1, lay["codes"])
            n_tok = N + j + 1
        else:                                       # re-hash the newest key in place (same work)
            ctx.hash_keys(lay["K"], *lay["weights"], N - 1, 1, lay["codes"])
        if ev:
            ev[0].record()
        ctx.retrieve_topk(lay["q"], *lay["weights"], lay["codes"], n_tok, k, out_idx=lay["idx"])
        if ev:
            ev[1].record()
        ctx.sparse_decode(lay["q"], lay["K"], lay["V"], lay["idx"], None, out=lay["out"])
        if ev:
            ev[2].record()

    if calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.int32, device=dev).fill_(7)      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()

    # ------------------------------------------------------------------ timed region
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i, evs[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    retr_us = sorted(e[0].elapsed_time(e[1]) * 1e3 for e in evs)
    att_us = sorted(e[1].elapsed_time(e[2]) * 1e3 for e in evs)
    retrieve_us = sum(retr_us) / steps
    attend_us = sum(att_us) / steps

    # ------------------------------------------------------------------ per-kernel durations
    # Same steps again with every kernel launch bracketed by HIP events on the library's stream.
    profile_enable(True)
    stage = {name: [0.0, 0] for name in sp.STAGES}
    done = 0
    while done < steps:
        chunk = min(steps - done, 512)              # at most 8192 recorded launches between reads
        for i in range(done, done + chunk):
            step(i)
        for name, (ms, n) in profile_read().items():
            stage[name] = [ms, n]
        done += chunk
    profile_enable(False)
    stage_us = {name: (ms * 1e3 / n if n else None) for name, (ms, n) in stage.items()}

    # ------------------------------------------------------------------ retrieval calls back to back
    # The same retrieve_topk calls with nothing between them (no append, no attention, no per-call
    # events): what a stream of retrievals costs per call, without the two event records that
    # bracket each call above.
    def retrieve_only(i):
        lay = layers[i % n_layers]
        lay["ctx"].retrieve_topk(lay["q"], *lay["weights"], lay["codes"], N, k, out_idx=lay["idx"])

    for i in range(warmup):
        retrieve_only(i)
    b2b = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    b2b[0].record()
    for i in range(steps):
        retrieve_only(i)
    b2b[1].record()
    torch.cuda.synchronize()
    retrieve_b2b_us = b2b[0].elapsed_time(b2b[1]) * 1e3 / steps

    # ------------------------------------------------------------------ codes that fit the last-level cache
    hot_us = None
    if hot_cache:
        for i in range(warmup):
            step(i, only_layer=0)
        hev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
        for i in range(steps):
            step(i, hev[i], only_layer=0)
        torch.cuda.synchronize()
        hot_us = sum(e[0].elapsed_time(e[1]) * 1e3 for e in hev) / steps

    # ------------------------------------------------------------------ the same step as ONE call
    # spotlight_decode_step: key and query hashed in one launch, then score, select, attend, merge.
    def fused(i):
        lay = layers[i % n_layers]
        n_tok = N + (i // n_layers) % cfg.extra_tokens + 1 if grow else N
        lay["ctx"].decode_step(lay["q"], lay["K"], lay["V"], *lay["weights"], lay["codes"], n_tok, k, 0, 0,
                               out_idx=lay["idx"], out=lay["out"])

    for i in range(warmup):
        fused(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        fused(i)
    torch.cuda.synchronize()
    fused_ms_per_step = (time.perf_counter() - t0) * 1e3 / steps

    # ... and replayed from HIP graphs, one captured step per layer (the call is kernel launches
    # and nothing else).  Only for a fixed context length: a graph freezes n_tokens.
    graph_ms_per_step = None
    if with_graph and not grow:
        side = torch.cuda.Stream()
        graphs = []
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            for li in range(n_layers):
                g = torch.cuda.CUDAGraph()
                g.capture_begin()
                fused(li)
                g.capture_end()
                graphs.append(g)
        torch.cuda.synchronize()
        for i in range(warmup):
            graphs[i % n_layers].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            graphs[i % n_layers].replay()
        torch.cuda.synchronize()
        graph_ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
        del graphs

    # ------------------------------------------------------------------ algorithmic bytes
    # score: every key code read once (L/8 bytes per key per key-value head)
    score_bytes = B * Hkv * N * (L // 8)
    # retrieval as a whole: codes once + indices written + hash weights read for the queries
    wsz = 2 if cfg.weight_dtype == "bf16" else 4
    weight_bytes = Hkv * ((cfg.hidden * d + cfg.hidden + L * cfg.hidden) if cfg.hidden else L * d) * wsz
    retrieve_bytes = score_bytes + B * Hq * k * 4 + weight_bytes
    # attention: K and V row per selected token, its index, q in, out written
    attend_bytes = B * Hq * k * (2 * d * esz + 4) + B * Hq * d * (esz + 4)

    res = {
        "cfg": cfg, "n_layers": n_layers, "esz": esz, "ms_per_step": ms_per_step,
        "retr_us": retr_us, "att_us": att_us, "retrieve_us": retrieve_us, "attend_us": attend_us,
        "stage_us": stage_us, "hot_us": hot_us, "retrieve_b2b_us": retrieve_b2b_us, "fused_ms": fused_ms_per_step, "graph_ms": graph_ms_per_step,
        "bulk_ms": bulk_ms, "t_gen": t_gen, "score_bytes": score_bytes, "retrieve_bytes": retrieve_bytes,
        "attend_bytes": attend_bytes,
        "bulk_gflops": 2.0 * B * Hkv * N * (cfg.hidden * d + L * cfg.hidden if cfg.hidden else L * d) / (bulk_ms * 1e-3) / 1e9,
    }
    if not args.no_cpu_baseline:
        res["cpu"] = cpu_baseline(cfg, layers[0], args.cpu_heads if hot_cache else 2)
    for lay in layers:
        lay["ctx"].close()
    del layers
    gc.collect()
    torch.cuda.empty_cache()
    return res


def workload_text(cfg):
    return (f"{cfg.name}: batch {cfg.batch}, {cfg.n_q_heads} q heads / {cfg.n_kv_heads} kv heads, head_dim {cfg.head_dim}, "
            f"{cfg.n_tokens} cached tokens, {cfg.code_bits}-bit codes (MLP {cfg.head_dim}->{cfg.hidden}->{cfg.code_bits}), "
            f"top-k {cfg.topk}, {cfg.kv_dtype} K/V")


def roofline_of(kind, nbytes, us, traffic):
    kernels = {
        "score": "score_kernel (Hamming distance, histograms, candidate lists)",
        "attend": "attend_kernel (gather + split-k softmax attention; the merge of the partials is a kernel of its "
                  "own, kernel_us.merge)",
    }
    return {
        "kernel": kernels[kind],
        "bound": "hbm",
        "achieved": round(gbps(nbytes, us), 1),
        "peak": HBM_PEAK_GBPS,
        "unit": "GB/s",
        "frac": round(gbps(nbytes, us) / HBM_PEAK_GBPS, 4),
        "traffic": traffic,
        "traffic_source": "stored: rocprofv3 FETCH_SIZE / WRITE_SIZE of an earlier run of this workload "
                          "(profiles/hbm_traffic.txt), not measured by this run" if traffic is not None else None,
        "bytes_per_launch": nbytes,
        "avg_launch_us": round(us, 2),
        "timing": "HIP events around each launch, second pass over the same steps",
    }


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; run it with --gpus 1 (no multi-GPU path exists)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import __graft_entry__
    __graft_entry__.ensure_built()   # builds only if the tree holds no library, or one older than its sources
    import workload as wl
    import paper_2508_19740_amd as sp

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(torch.device("cuda:0"))
    cfg = wl.CONFIGS[args.config]
    variant = ""
    if args.code_bits:
        cfg = cfg.scaled(code_bits=args.code_bits)
        variant += f", L={args.code_bits}"
    if args.hidden >= 0:
        cfg = cfg.scaled(hidden=args.hidden)
        variant += f", hidden={args.hidden}"
    if args.lsh_init:
        cfg = cfg.scaled(lsh_init=args.lsh_init)
        variant += f", {args.lsh_init} LSH"
    if args.batch > 0:
        cfg = cfg.scaled(batch=args.batch)
        variant += f", batch={args.batch}"

    plain_headline = args.config == "C3" and not variant and args.layers == 0
    m = measure(cfg, args, args.steps, args.warmup, with_graph=True, calibrate_copy=args.calibrate_copy,
                hot_cache=True)
    K_steps = args.steps
    stage_us = m["stage_us"]
    esz = m["esz"]

    result = {
        "metric": ("retrieval_us_512k_tokens_32_heads" if args.config == "C3" else f"retrieval_us_{args.config}")
                  + (f" [variant{variant}]" if variant else ""),
        "value": round(m["retrieve_us"], 2),
        "unit": "us",
        "n_gpus": 1,
        "steps": K_steps,
        "warmup": args.warmup,
        "ms_per_step": round(m["ms_per_step"], 4),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",
        "dtype_detail": "u32 xor/popcount and integer counting (retrieval), f32 fma chains (hash MLP), "
                        + ("bf16 K/V with f32 softmax accumulation (attention)" if esz == 2 else "f32 (attention)"),
        "data": "synthetic",
        "config": {
            "workload": workload_text(cfg),
            "layers_rotated": m["n_layers"],
            "hash_weights": "as stored" if args.no_prepack else "prepacked once per layer (spotlight_prepack_weights)",
            "step": "append-hash 1 key/head + retrieve_topk + sparse_decode",
        },
        "library_build_id": sp.build_id(),
        "retrieve_us": {"mean": round(m["retrieve_us"], 2), "median": round(m["retr_us"][K_steps // 2], 2),
                        "min": round(m["retr_us"][0], 2)},
        "retrieve_us_back_to_back": round(m["retrieve_b2b_us"], 2),
        "retrieve_us_hot_cache": None if m["hot_us"] is None else round(m["hot_us"], 2),
        "hot_cache_note": "same call with ONE layer, so the code stream can stay in the 256 MB last-level cache; "
                          "not an HBM number and not compared with the roofline",
        "attend_us": {"mean": round(m["attend_us"], 2), "median": round(m["att_us"][K_steps // 2], 2),
                      "min": round(m["att_us"][0], 2)},
        "retrieve_gbps": round(gbps(m["retrieve_bytes"], m["retrieve_us"]), 1),
        "retrieve_frac_of_hbm_peak": round(gbps(m["retrieve_bytes"], m["retrieve_us"]) / HBM_PEAK_GBPS, 4),
        "attend_gbps": round(gbps(m["attend_bytes"], m["attend_us"]), 1),
        "attend_frac_of_hbm_peak": round(gbps(m["attend_bytes"], m["attend_us"]) / HBM_PEAK_GBPS, 4),
        "decode_step_one_call_ms": round(m["fused_ms"], 4),
        "decode_step_graph_replay_ms": None if m["graph_ms"] is None else round(m["graph_ms"], 4),
        "kernel_us": {kname: (round(v, 2) if v is not None else None) for kname, v in stage_us.items()},
        "bulk_hash_keys_ms_per_layer": round(m["bulk_ms"], 3),
        "bulk_hash_keys_gflops": round(m["bulk_gflops"], 1),
        "setup_s": round(m["t_gen"], 1),
        "roofline": roofline_of("score", m["score_bytes"], stage_us["score"], stored_traffic(args.config, "score_kernel")),
        "roofline_attend": roofline_of("attend", m["attend_bytes"], stage_us["attend"],
                                       stored_traffic(args.config, "attend_kernel")),
    }
    if "cpu" in m:
        result["cpu_baseline"] = m["cpu"]

    # ------------------------------------------------------------------ the other workloads
    names = []
    if args.others == "auto":
        names = ["C2", "C4", "C5-128"] if plain_headline else []
    elif args.others != "none":
        names = [n for n in args.others.split(",") if n]
    others = {}
    for name in names:
        o = measure(wl.CONFIGS[name], args, args.other_steps, min(args.warmup, 10), with_graph=False)
        su = o["stage_us"]
        entry = {
            "workload": workload_text(o["cfg"]),
            "steps": args.other_steps,
            "layers_rotated": o["n_layers"],
            "retrieve_us": round(o["retrieve_us"], 2),
            "retrieve_us_back_to_back": round(o["retrieve_b2b_us"], 2),
            "attend_us": round(o["attend_us"], 2),
            "decode_step_one_call_ms": round(o["fused_ms"], 4),
            "kernel_us": {kname: (round(v, 2) if v is not None else None) for kname, v in su.items()},
            "score": {"bytes_per_launch": o["score_bytes"], "gbps": round(gbps(o["score_bytes"], su["score"]), 1),
                      "frac": round(gbps(o["score_bytes"], su["score"]) / HBM_PEAK_GBPS, 4)},
            "attend": {"bytes_per_launch": o["attend_bytes"], "gbps": round(gbps(o["attend_bytes"], su["attend"]), 1),
                       "frac": round(gbps(o["attend_bytes"], su["attend"]) / HBM_PEAK_GBPS, 4)},
            "bulk_hash_keys_ms_per_layer": round(o["bulk_ms"], 3),
        }
        if name in ("C1", "C2"):
            entry["note"] = "launch-latency-bound: tens of megabytes per launch, a few microseconds per kernel"
        if "cpu" in o:
            entry["cpu_baseline"] = o["cpu"]
        others[name] = entry
    if others:
        result["other_workloads"] = others

    print(json.dumps(result))


def cpu_baseline(cfg, lay, n_heads):
    """Times the CPU oracle on the retrieval of a few heads of the same workload (same seeded K
    rows and weights as layer 0), and scales the per-head time to all heads."""
    import torch
    import oracle

    Hkv, G, N, k = cfg.n_kv_heads, cfg.group, cfg.n_tokens, cfg.topk
    n_heads = max(1, min(n_heads, Hkv))
    w = lay["w"]
    hw = w.hash_weights()
    heads = list(range(n_heads))
    # inputs come from the seeded generator (its device copy), never from the HIP kernels
    hK = lay["K"][0, heads].cpu().unsqueeze(0).contiguous()          # [1, n_heads, Nmax, d]
    hV = lay["V"][0, heads].cpu().unsqueeze(0).contiguous()
    w1, b1, w2 = (None if t is None else t[heads].contiguous() for t in hw)
    q = w.q[0:1, : n_heads * G].contiguous()
    codes = torch.zeros(1, n_heads, cfg.max_tokens, cfg.words, dtype=torch.int32)
    t0 = time.perf_counter()
    oracle.hash_keys(hK, w1, b1, w2, cfg.code_bits, 0, N, codes)         # setup: the oracle's own codes
    t_build = time.perf_counter() - t0
    reps = 3 if n_heads > 2 else 1
    t0 = time.perf_counter()
    for _ in range(reps):
        idx, _, _ = oracle.retrieve_topk(q, w1, b1, w2, codes, N, k)
    t_retr = (time.perf_counter() - t0) / reps
    t0 = time.perf_counter()
    for _ in range(reps):
        oracle.sparse_decode(q, hK, hV, idx, 1.0 / math.sqrt(cfg.head_dim))
    t_att = (time.perf_counter() - t0) / reps
    per_q_head = t_retr / (n_heads * G)
    return {
        "value": round(per_q_head * cfg.batch * cfg.n_q_heads * 1e6, 1),
        "unit": "us",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": f"retrieval (query hash + bit-by-bit Hamming + full sort) of {n_heads * G} of "
                  f"{cfg.batch * cfg.n_q_heads} query heads of layer 0 at full context, mean of {reps} run(s), "
                  f"scaled by heads; the oracle takes heads one after another: its bit-by-bit Hamming loop runs on "
                  f"all {oracle.num_threads()} threads, its full sort (qsort) on ONE; key codes built by the oracle "
                  f"beforehand ({t_build:.1f} s, untimed)",
        "attend_us_scaled": round(t_att / (n_heads * G) * cfg.batch * cfg.n_q_heads * 1e6, 1),
        "hash_keys_us_per_key": round(t_build / (n_heads * N) * 1e6, 3),
    }


if __name__ == "__main__":
    main()
