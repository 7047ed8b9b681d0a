#!/usr/bin/env python3
"""Benchmark of the WindowKV window-selection path on one MI355X.

One *step* is one ``wkv_compress_groups`` call over the whole workload: score the first layer
of every group, pool, select, and gather the kept K/V rows of every layer.  The default
workload is the 32K-token full-model configuration (8 groups of 4 LLaMA-3-8B shaped layers).
Inputs are seeded synthetic tensors, resident in HBM before the timed region starts.

Prints one JSON line:
  value      prefix tokens compressed per second per layer group = L * n_groups / step time
  roofline   the stage that takes the largest share of the step (Eq. 1-2 counts as ONE stage: its
             two launches' durations summed against ONE read of the keys), its algorithmic HBM
             bytes over its mean duration (HIP events on the launch stream, measured here)
  stages     the same for every stage, with the counter-measured traffic where a profile of these
             very kernel sources exists (profiles/traffic.json), else null
  pipeline   the same for the whole step (all kernels, launch gaps included)
  graph_replay  the step replayed from a captured HIP graph (no launch gaps from the host)
  cpu_baseline  the fp64 CPU oracle timed on this host on a bounded sample of the same workload,
             once on one thread and once on all cores the process may use
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E, vendor figure
MFMA_BF16_PEAK_TFLOPS = 2500.0
CSRC = os.path.join(ROOT, "paper_2503_17922_amd", "csrc")


def kernel_sources_sha256():
    """Fingerprint of the kernel sources a traffic profile belongs to."""
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".hip", ".h", ".cpp")):
            h.update(name.encode())
            h.update(open(os.path.join(CSRC, name), "rb").read())
    return h.hexdigest()


def measured_traffic(workload):
    """HBM bytes per launch from rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE, each scaled by
    what the same counter reads for a plain device copy of known size), as recorded in
    profiles/traffic.json together with the fingerprint of the kernel sources they were measured
    on.  A profile of other sources says nothing about these kernels: then every figure is null."""
    try:
        rec = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))["workloads"][workload]
    except (OSError, KeyError, ValueError):
        return {}
    if rec.get("kernel_sources_sha256") != kernel_sources_sha256():
        return {}
    return rec["bytes_per_launch"]


# The paper measures no part of this path by itself; its only speed figures are end-to-end
# generation on other hardware (Table 2), quoted as context.
PAPER_CONTEXT = {
    "hardware": "1x NVIDIA A100-40G (paper, Table 2), LLaMA-3-8B-Instruct, prefill 7950 + 242 generated tokens",
    "end_to_end_tokens_per_s": {"full KV": 764, "WindowKV, KV size 512": 894, "WindowKV + task classifier": 881},
    "end_to_end_ms_per_token": {"full KV": 1.31, "WindowKV, KV size 512": 1.12, "WindowKV + task classifier": 1.14},
    "kv_retained_at_comparable_quality": "about 12 % of the cache (LongBench)",
    "note": "no latency, bandwidth or memory figure for the selection path itself is published: vs_baseline is null",
}


def algorithmic_bytes(w):
    """Bytes each launch / stage must move (what the method needs, not what a kernel happens to
    read).  Eq. 1-2 as a stage and the whole path are charged ONE read of the scored keys,
    although two launches each stream them: the second read is this implementation's cost."""
    e = 4 if w.dtype == "f32" else 2
    d, H = w.head_dim, w.n_kv_heads
    row = d * e
    k_first = sum(w.seq_len) * H * row * w.n_groups                      # K of each scored layer, once
    q = w.batch * w.n_q_heads * w.w_obs * row * w.n_groups
    n_keep = sum(k * wn + w.w_obs for k, wn in zip(w.k_windows, w.win))    # rows kept per KV head
    gather_rw = w.n_layers * 2 * n_keep * H * row                       # read, and the same written
    s_bytes = sum(-(-(L - w.w_obs) // wn) for L, wn in zip(w.seq_len, w.win)) * H * 4 * w.n_groups
    idx_bytes = n_keep * H * 4 * w.n_groups
    return {
        "score_stats": k_first + q,          # launch: the statistics pass reads the keys once
        "score": k_first + q + s_bytes,      # launch: the second read is algorithmic for this kernel alone
        "select": s_bytes + idx_bytes,
        "gather": 2 * gather_rw,
        "score_stage": k_first + q,          # Eq. 1-2 as one stage: the keys once
        "pipeline": k_first + q + 2 * gather_rw,    # the path: keys once + gather read + write
    }


def score_flops(w):
    return 2 * w.n_q_heads * w.w_obs * w.head_dim * sum(w.seq_len) * w.n_groups


def _time_oracle(w, st, budget_s):
    """Whole layer groups of the workload through the oracle until about `budget_s` seconds."""
    import torch
    from oracle import wkv_oracle as O
    from paper_2503_17922_amd import synthetic as P
    done_groups, t_total = 0, 0.0
    for g in (gg % w.n_groups for gg in range(64 * w.n_groups)):
        # stage the group's inputs on the host first: the transfer is not part of the baseline
        G = w.q_per_kv
        q = [[P.host_f64(w, st.q[g][b, h * G:(h + 1) * G]) for h in range(w.n_kv_heads)] for b in range(w.batch)]
        ks = [[[st.k[g * w.gamma + l][b, h, : w.seq_len[b]].cpu() for l in range(w.gamma)]
               for h in range(w.n_kv_heads)] for b in range(w.batch)]
        vs = [[[st.v[g * w.gamma + l][b, h, : w.seq_len[b]].cpu() for l in range(w.gamma)]
               for h in range(w.n_kv_heads)] for b in range(w.batch)]
        bits = (lambda t: t.numpy()) if w.dtype == "f32" else (lambda t: t.view(torch.int16).numpy())
        t0 = time.perf_counter()
        for b in range(w.batch):
            for h in range(w.n_kv_heads):
                k64 = ks[b][h][0].to(torch.float64).numpy()
                _, _, _, idx = O.select_indices(q[b][h], k64, w.win[b], w.top_p[b], w.k_windows[b])
                for l in range(w.gamma):
                    O.gather_rows(bits(ks[b][h][l]), idx)
                    O.gather_rows(bits(vs[b][h][l]), idx)
        t_total += time.perf_counter() - t0
        done_groups += 1
        if t_total >= budget_s:
            break
    return done_groups, t_total


def cpu_baseline(w, st, budget_s=8.0):
    """Time the oracle, as it stands, on whole layer groups of the same workload: once with its
    library routines held to one thread, once on every core the process may use."""
    from threadpoolctl import threadpool_limits
    cores = len(os.sched_getaffinity(0))
    with threadpool_limits(limits=1):
        g1, t1 = _time_oracle(w, st, budget_s)
    gn, tn = _time_oracle(w, st, budget_s)
    unit = "prefix tokens/s per layer group"
    return {"value": sum(w.seq_len) / (tn / gn), "unit": unit, "cores": cores, "kind": "oracle",
            "sample": f"{gn} layer groups of workload {w.name} (its {w.n_groups} groups, repeated in turn: "
                      f"{gn * w.batch * w.n_kv_heads} (sequence, KV head) problems, fp64 numpy, {tn:.1f} s; inputs "
                      f"already on the host)",
            "one_thread": {"value": sum(w.seq_len) / (t1 / g1), "unit": unit, "cores": 1,
                           "sample": f"{g1} layer groups, {t1:.1f} s, numerical libraries limited to one thread"}}


def attention_lse(w, st, g):
    """ln-sum-exp of the observation rows of group g's first layer, [B, Hq, w_obs] float32: the
    by-product of prefill attention that the hand-over variant takes as an input.  Plain torch
    ops on the device, outside every timed region."""
    import torch
    q, k = st.q[g], st.k[g * w.gamma]
    G, a = w.q_per_kv, w.w_obs
    scale = 1.0 / (w.head_dim ** 0.5)
    out = torch.empty((w.batch, w.n_q_heads, a), dtype=torch.float32, device=q.device)
    for b in range(w.batch):
        L = w.seq_len[b]
        pos = torch.arange(L, device=q.device)[None, :]
        visible = pos <= (L - a + torch.arange(a, device=q.device))[:, None]          # causal
        for h in range(w.n_kv_heads):
            kk = k[b, h, :L].float()
            for gq in range(G):
                logits = (q[b, h * G + gq].float() @ kk.T) * scale
                out[b, h * G + gq] = torch.logsumexp(logits.masked_fill(~visible, float("-inf")), dim=1)
    return out


def lse_handoff(args, W, w, st, stream, ab):
    """The same step when the caller hands over the softmax normalisers its prefill attention
    already has: the statistics pass disappears, the rest is unchanged.  Reported beside the
    headline figure, never in place of it."""
    import torch
    lse = [attention_lse(w, st, g) for g in range(w.n_groups)]
    call = W.CompressCall(st.problem, w.n_groups, w.gamma, st.q, lse, st.k, st.v, st.k_out, st.v_out,
                          st.win_idx, st.tok_idx, st.n_keep, st.workspace)
    for _ in range(args.warmup):
        call(stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        call(stream)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    ach = ab["pipeline"] / (ms * 1e-3) / 1e9
    stage_ms = [0.0] * W.WKV_N_STAGES
    for _ in range(5):
        stage_ms = [a + b for a, b in zip(stage_ms, call.profiled(stream))]
    return {"ms_per_step": ms, "value": sum(w.seq_len) * w.n_groups / (ms * 1e-3),
            "unit": "prefix tokens/s per layer group",
            "pipeline": {"achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": round(ach / HBM_PEAK_GBS, 4)},
            "kernels_ms": {n: round(m / 5, 4) for n, m in zip(W.STAGE_NAMES, stage_ms)},
            "note": "inputs additionally include lse_obs [B, Hq, w_obs] per group (a by-product of prefill attention)"}


def decode_leg(W, w, device, stream, steps):
    """One decode step of one layer over retained caches of the workload's size (n_keep rows per
    KV head), for a single sequence (latency) and for 64 sequences (throughput).  Every K and V
    row is read once per step: algorithmic bytes = 2 * batch * Hkv * rows * head_dim * esize.
    The row count is left as it is (WKV_DECODE_KEEP_COUNT), so every step sees the same length."""
    import torch
    torch.manual_seed(1007)                      # seeded N(0,1) caches: the timing does not depend on the values
    out = {}
    kept_rows = w.k_windows[0] * w.win[0] + w.w_obs
    esize = 4 if w.dtype == "f32" else 2
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[w.dtype]
    dt = {"bf16": W.WKV_BF16, "f16": W.WKV_F16, "f32": W.WKV_F32}[w.dtype]
    for batch, n_rows, label in ((1, kept_rows, "batch1"), (64, kept_rows, "batch64"),
                                 (8, w.seq_len[0], "full_cache_batch8")):
        cap = n_rows + 64
        H, d = w.n_kv_heads, w.head_dim
        kc = torch.randn((batch, H, cap, d), device=device, dtype=torch.float32).to(tdt)
        vc = torch.randn((batch, H, cap, d), device=device, dtype=torch.float32).to(tdt)
        q = torch.randn((batch, w.n_q_heads, d), device=device, dtype=torch.float32).to(tdt)
        kn = torch.randn((batch, H, d), device=device, dtype=torch.float32).to(tdt)
        vn = torch.randn((batch, H, d), device=device, dtype=torch.float32).to(tdt)
        res = torch.empty((batch, w.n_q_heads, d), device=device, dtype=torch.float32)
        n_valid = torch.full((batch, H), n_rows, dtype=torch.int32, device=device)
        nbytes = 2 * batch * H * (n_rows + 1) * d * esize
        shape = W.DecodeShape(batch=batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=d, capacity=cap,
                              dtype=dt, flags=W.WKV_DECODE_KEEP_COUNT)
        ws = torch.empty(W.wkv_decode_workspace_bytes(shape), dtype=torch.uint8, device=device)

        def run(n):
            for _ in range(n):
                W.wkv_decode_step(shape, q, kn, vn, kc, vc, n_valid, res, ws, stream)
        run(5)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(steps)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / steps * 1e3
        out[label] = {"ms_per_layer_step": round(ms, 4), "algorithmic_bytes": nbytes,
                      "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1),
                      "frac": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "rows_per_kv_head": n_rows + 1}
    # the method's decode-time gain: attention time per sequence over the whole prefix / over what was kept
    out["attention_speedup_vs_full_cache"] = round((out["full_cache_batch8"]["ms_per_layer_step"] / 8) /
                                                   (out["batch64"]["ms_per_layer_step"] / 64), 2)
    out["note"] = ("wkv_decode_step (two launches: key ranges, merge) on synthetic caches of the retained size (batch1, "
                   "batch64) and of the whole prefix (full_cache_batch8, the same bytes as batch64); batch 1 is bound by "
                   "launch latency and by the host's call overhead")
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c4")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-lse-handoff", action="store_true",
                    help="skip the second measurement (softmax normalisers handed over by the caller)")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode-step measurement")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the same step")
    ap.add_argument("--keep-padding", action="store_true",
                    help="set WKV_KEEP_PADDING: compact-cache rows past n_keep are not zero-filled (matters for "
                         "batches of mixed lengths; the default run zero-fills)")
    ap.add_argument("--score", choices=["auto", "two-pass", "single-read"], default="auto",
                    help="which kernels compute Eq. 1-2: the library's choice (default), or one of the two forced")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy a few times (a known-size reference for hardware counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 (sequences, KV heads and layer groups are independent: shard them across processes)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2503_17922_amd as W
    import wkv_synth as S
    from paper_2503_17922_amd import synthetic as P

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    W.lib()
    device = torch.device("cuda:0")
    w = S.make_workload(args.workload)
    flags = (W.WKV_KEEP_PADDING if args.keep_padding else 0) | \
            {"auto": 0, "two-pass": W.WKV_SCORE_TWO_PASS, "single-read": W.WKV_SCORE_SINGLE_READ}[args.score]
    st = P.DeviceState(w, device, flags=flags)
    call = W.CompressCall(st.problem, w.n_groups, w.gamma, st.q, None, st.k, st.v, st.k_out, st.v_out,
                          st.win_idx, st.tok_idx, st.n_keep, st.workspace)
    stream = torch.cuda.current_stream().cuda_stream

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=device).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        call(stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        call(stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # per-kernel durations: HIP events recorded by the library on the launch stream
    stage_ms = [0.0] * W.WKV_N_STAGES
    n_prof = max(5, min(args.steps, 20))
    for _ in range(n_prof):
        ms = call.profiled(stream)
        stage_ms = [a + b for a, b in zip(stage_ms, ms)]
    stage_ms = [a / n_prof for a in stage_ms]
    stages = dict(zip(W.STAGE_NAMES, stage_ms))

    ab = algorithmic_bytes(w)
    traffic = measured_traffic(w.name)

    def entry(name, ms, nbytes, tr):
        gbs = nbytes / (ms * 1e-3) / 1e9
        return {"name": name, "ms": round(ms, 4), "algorithmic_bytes": nbytes, "GB/s": round(gbs, 1),
                "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": tr,
                "traffic_over_algorithmic": round(tr / nbytes, 3) if tr else None}

    # launches as the library brackets them with events
    kernels = {}
    for name in W.STAGE_NAMES:
        if stages[name] > 0.0015:        # (a stage that launched nothing reads a few hundred ns between two event records)
            kernels[name] = entry(name, stages[name], ab[name], traffic.get(name))
    for name in ("score_stats", "score"):     # each pass computes the whole Q.K^T contraction once
        if name in kernels:
            tf = score_flops(w) / (stages[name] * 1e-3) / 1e12
            kernels[name]["mfma_TFLOP/s"] = round(tf, 1)
            kernels[name]["mfma_frac"] = round(tf / MFMA_BF16_PEAK_TFLOPS, 4)
    # stages of the method: Eq. 1-2 is ONE stage, however many launches compute it, and must read the keys once
    score_traffic = (traffic.get("score_stats", 0) + traffic.get("score", 0)) or None if traffic else None
    stage_list = [entry("score (Eq. 1-2: every launch that reads the scored keys, their durations summed, the keys charged once)",
                        stages["score_stats"] + stages["score"], ab["score_stage"], score_traffic)]
    if "select" in kernels:
        stage_list.append(entry("select (Eq. 3-4 where not pooled by the score launch, Section 2.2.1)", stages["select"], ab["select"], traffic.get("select")))
    stage_list.append(entry("gather (Section 2.2.2)", stages["gather"], ab["gather"], traffic.get("gather")))
    dominant = max(stage_list, key=lambda e: e["ms"])
    # (among the stages that matter for the step time: a tenth of the longest one or more)
    lowest = min((e for e in stage_list if e["ms"] >= 0.1 * dominant["ms"]), key=lambda e: e["frac"])
    roofline = {"kernel": dominant["name"], "bound": "hbm", "achieved": dominant["GB/s"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": dominant["frac"], "traffic": dominant["traffic"],
                "traffic_over_algorithmic": dominant["traffic_over_algorithmic"],
                "algorithmic_bytes": dominant["algorithmic_bytes"], "ms": dominant["ms"],
                "furthest_below": {k: lowest[k] for k in ("name", "ms", "GB/s", "frac", "traffic_over_algorithmic")}}
    pipe_ach = ab["pipeline"] / (ms_per_step * 1e-3) / 1e9
    pipe_traffic = sum(traffic.get(n, 0) for n in kernels) if traffic and all(n in traffic for n in kernels) else None

    # the same step replayed from a captured HIP graph: what remains when the host launches nothing
    graph_ms = None
    if not args.no_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            call(torch.cuda.current_stream().cuda_stream)
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) / args.steps * 1e3

    tokens = sum(w.seq_len)
    out = {
        "metric": "prefix tokens compressed/sec per layer group; achieved HBM GB/s vs peak",
        "value": tokens * w.n_groups / (ms_per_step * 1e-3),
        "unit": "prefix tokens/s per layer group",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"bf16": "bf16", "f16": "f16", "f32": "f32"}[w.dtype], "data": "synthetic",
        "config": {"workload": f"{w.name}: batch {w.batch}, {w.n_groups} groups x {w.gamma} layers, "
                               f"{w.n_q_heads}q/{w.n_kv_heads}kv heads, d={w.head_dim}, L={w.seq_len}, "
                               f"w_obs={w.w_obs}, win={sorted(set(w.win))}, top_p={sorted(set(w.top_p))}, "
                               f"k={w.k_windows}",
                   "ms_per_group": ms_per_step / w.n_groups, "zero_fill_padding": not args.keep_padding,
                   "score_kernels": args.score},
        "roofline": roofline,
        "stages": stage_list,
        "pipeline": {"bound": "hbm", "algorithmic_bytes": ab["pipeline"], "achieved": round(pipe_ach, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(pipe_ach / HBM_PEAK_GBS, 4),
                     "kernel_sum_ms": round(sum(stages.values()), 4),
                     "traffic": pipe_traffic,
                     # the counter-based figure: bytes the kernels really moved over the same step time
                     "traffic_GB/s": round(pipe_traffic / (ms_per_step * 1e-3) / 1e9, 1) if pipe_traffic else None,
                     "traffic_frac": round(pipe_traffic / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if pipe_traffic else None},
        "kernels": kernels,
        "paper_context": PAPER_CONTEXT,
    }
    if graph_ms is not None:
        g_ach = ab["pipeline"] / (graph_ms * 1e-3) / 1e9
        out["graph_replay"] = {"ms_per_step": round(graph_ms, 4), "value": tokens * w.n_groups / (graph_ms * 1e-3),
                               "pipeline_frac": round(g_ach / HBM_PEAK_GBS, 4),
                               "note": "the same call captured once into a HIP graph and replayed; the headline value is the eager call"}
    if not args.no_lse_handoff:
        out["lse_handoff"] = lse_handoff(args, W, w, st, stream, ab)
    if not args.no_decode:
        out["decode"] = decode_leg(W, w, device, stream, max(args.steps, 20))
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, st)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
