#!/usr/bin/env python3
"""Benchmark of the WindowKV window-selection path on one MI355X.

One *step* is one ``wkv_compress_groups`` call over the whole workload: score the first layer
of every group, pool, select, and gather the kept K/V rows of every layer.  The default
workload is the 32K-token full-model configuration (8 groups of 4 LLaMA-3-8B shaped layers).
Inputs are seeded synthetic tensors, resident in HBM before the timed region starts.

Prints one JSON line:
  value      prefix tokens compressed per second per layer group = L * n_groups / step time
  roofline   the kernel that takes the largest share of the step, its algorithmic HBM bytes per
             launch over its mean duration (HIP events on the launch stream, measured here)
  pipeline   the same for the whole step (all kernels, launch gaps included)
  cpu_baseline  the fp64 CPU oracle timed on this host on a bounded sample of the same workload
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E, vendor figure
MFMA_BF16_PEAK_TFLOPS = 2500.0

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, then WRITE_SIZE), each scaled by
# what the same counter reads for a plain 256 MiB device copy (2.0 and 1.0 on this machine); the
# runs are summarised in profiles/compress_groups_c4.md.  Missing key = not measured (null).
MEASURED_TRAFFIC_BYTES = {
    ("c4", "score_pre"): 557.4e6,      # statistics pass
    ("c4", "score"): 560.2e6,          # score pass (folds the statistics, pools its windows)
    ("c4", "topk_windows"): 1.8e6,     # selection on the window scores
    ("c4", "gather"): 1083.2e6,
    ("c4", "pipeline"): 2202.6e6,
}


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
    """Bytes each kernel must move per launch (what the method needs, not what a kernel happens
    to read).  For the whole path the key stream of the scored layers is charged ONCE, although
    the two score kernels each read it: the second read is this implementation's cost."""
    e = 4 if w.dtype == "f32" else 2
    d, H = w.head_dim, w.n_kv_heads
    row = d * e
    k_first = sum(w.seq_len) * H * row * w.n_groups                      # K of each scored layer, once
    q = w.batch * w.n_q_heads * w.w_obs * row * w.n_groups
    n_keep = sum(k * wn + w.w_obs for k, wn in zip(w.k_windows, w.win))    # rows kept per KV head
    gather_rw = w.n_layers * 2 * n_keep * H * row                       # read, and the same written
    t_bytes = sum(L - w.w_obs for L in w.seq_len) * H * 4 * w.n_groups
    return {
        "score_pre": k_first + q,            # two-pass mode: the statistics pass reads the keys once
        "score": k_first + q + t_bytes,      # the second read is algorithmic for this kernel alone
        "window_pool": t_bytes,
        "topk_windows": t_bytes // max(min(w.win), 1),
        "gather": 2 * gather_rw,
        "pipeline": k_first + q + 2 * gather_rw,    # the path: keys once + gather read + write
    }


def score_flops(w):
    return 2 * w.n_q_heads * w.w_obs * w.head_dim * sum(w.seq_len) * w.n_groups


def cpu_baseline(w, st, budget_s=10.0):
    """Time the oracle, as it stands, on whole layer groups of the same workload."""
    import numpy as np
    import torch
    from oracle import wkv_oracle as O
    from paper_2503_17922_amd import synthetic as P
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    done_groups, t_total = 0, 0.0
    # whole layer groups, round after round over the workload, until about `budget_s` of CPU time
    for g in (gg % w.n_groups for gg in range(64 * w.n_groups)):
        # stage the group's inputs on the host first: the transfer is not part of the baseline
        G = w.q_per_kv
        q = [[P.host_f64(w, st.q[g][b, h * G:(h + 1) * G]) for h in range(w.n_kv_heads)] for b in range(w.batch)]
        ks = [[[st.k[g * w.gamma + l][b, h, : w.seq_len[b]].cpu() for l in range(w.gamma)]
               for h in range(w.n_kv_heads)] for b in range(w.batch)]
        vs = [[[st.v[g * w.gamma + l][b, h, : w.seq_len[b]].cpu() for l in range(w.gamma)]
               for h in range(w.n_kv_heads)] for b in range(w.batch)]
        t0 = time.perf_counter()
        for b in range(w.batch):
            for h in range(w.n_kv_heads):
                k64 = ks[b][h][0].to(torch.float64).numpy()
                _, _, _, idx = O.select_indices(q[b][h], k64, w.win[b], w.top_p[b], w.k_windows[b])
                for l in range(w.gamma):
                    O.gather_rows(ks[b][h][l].view(torch.int16).numpy() if w.dtype == "bf16" else ks[b][h][l].numpy(), idx)
                    O.gather_rows(vs[b][h][l].view(torch.int16).numpy() if w.dtype == "bf16" else vs[b][h][l].numpy(), idx)
        t_total += time.perf_counter() - t0
        done_groups += 1
        if t_total >= budget_s:
            break
    per_group = t_total / done_groups
    return {"value": sum(w.seq_len) / per_group, "unit": "prefix tokens/s per layer group", "cores": int(cores),
            "kind": "oracle",
            "sample": f"{done_groups} layer groups of workload {w.name} (its {w.n_groups} groups, repeated in turn: "
                      f"{done_groups * w.batch * w.n_kv_heads} (sequence, KV head) problems, fp64 numpy, "
                      f"{t_total:.1f} s; inputs already on the host)"}


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
    row is read once per step: algorithmic bytes = 2 * batch * Hkv * rows * head_dim * esize."""
    import torch
    torch.manual_seed(1007)                      # seeded N(0,1) caches: the timing does not depend on the values
    out = {}
    kept_rows = w.k_windows[0] * w.win[0] + w.w_obs
    esize = 2 if w.dtype == "bf16" else 4
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    for batch, n_rows, label in ((1, kept_rows, "batch1"), (64, kept_rows, "batch64"),
                                 (8, w.seq_len[0], "full_cache_batch8")):
        cap = n_rows + 64
        shape = W.DecodeShape(batch=batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                              capacity=cap, dtype=W.WKV_BF16 if w.dtype == "bf16" else W.WKV_F32)
        H, d = w.n_kv_heads, w.head_dim
        kc = torch.randn((batch, H, cap, d), device=device, dtype=torch.float32).to(tdt)
        vc = torch.randn((batch, H, cap, d), device=device, dtype=torch.float32).to(tdt)
        q = torch.randn((batch, w.n_q_heads, d), device=device, dtype=torch.float32).to(tdt)
        kn = torch.randn((batch, H, d), device=device, dtype=torch.float32).to(tdt)
        vn = torch.randn((batch, H, d), device=device, dtype=torch.float32).to(tdt)
        res = torch.empty((batch, w.n_q_heads, d), device=device, dtype=torch.float32)
        ws = torch.empty(W.wkv_decode_workspace_bytes(shape), dtype=torch.uint8, device=device)
        n_valid = torch.full((batch, H), n_rows, dtype=torch.int32, device=device)

        def run(n, n_rows=n_rows, n_valid=n_valid):
            for _ in range(n):
                n_valid.fill_(n_rows)            # stay at the same length: the fill is part of the loop for both counts
                W.wkv_decode_step(shape, q, kn, vn, kc, vc, n_valid, res, ws, stream)
        run(5)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(steps)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / steps * 1e3
        nbytes = 2 * batch * H * (n_rows + 1) * d * esize
        out[label] = {"ms_per_layer_step": round(ms, 4), "algorithmic_bytes": nbytes,
                                "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1),
                                "frac": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                "rows_per_kv_head": n_rows + 1}
    # the method's decode-time gain: attention time per sequence over the whole prefix / over what was kept
    out["attention_speedup_vs_full_cache"] = round((out["full_cache_batch8"]["ms_per_layer_step"] / 8) /
                                                   (out["batch64"]["ms_per_layer_step"] / 64), 2)
    out["note"] = ("wkv_decode_step on synthetic caches of the retained size (batch1, batch64) and of the whole prefix "
                   "(full_cache_batch8, the same bytes as batch64); times include one tiny fill kernel per step and "
                   "the launch overhead of 3 kernels (latency-bound at batch 1)")
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
    dominant = max(stages, key=stages.get)
    ach = ab[dominant] / (stages[dominant] * 1e-3) / 1e9
    roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, dominant)),
                "algorithmic_bytes": ab[dominant], "ms": round(stages[dominant], 4)}
    pipe_ach = ab["pipeline"] / (ms_per_step * 1e-3) / 1e9
    kernels = {}
    for name in W.STAGE_NAMES:
        if stages[name] > 0:
            kernels[name] = {"ms": round(stages[name], 4), "algorithmic_bytes": ab[name],
                             "GB/s": round(ab[name] / (stages[name] * 1e-3) / 1e9, 1)}
    for name in ("score_pre", "score"):       # each pass computes the whole Q.K^T contraction once
        if stages[name] > 0:
            tf = score_flops(w) / (stages[name] * 1e-3) / 1e12
            kernels[name]["mfma_TFLOP/s"] = round(tf, 1)
            kernels[name]["mfma_frac"] = round(tf / MFMA_BF16_PEAK_TFLOPS, 4)

    tokens = sum(w.seq_len)
    pipe_traffic = MEASURED_TRAFFIC_BYTES.get((w.name, "pipeline"))
    out = {
        "metric": "prefix tokens compressed/sec per layer group; achieved HBM GB/s vs peak",
        "value": tokens * w.n_groups / (ms_per_step * 1e-3),
        "unit": "prefix tokens/s per layer group",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: batch {w.batch}, {w.n_groups} groups x {w.gamma} layers, "
                               f"{w.n_q_heads}q/{w.n_kv_heads}kv heads, d={w.head_dim}, L={w.seq_len}, "
                               f"w_obs={w.w_obs}, win={sorted(set(w.win))}, top_p={sorted(set(w.top_p))}, "
                               f"k={w.k_windows}",
                   "ms_per_group": ms_per_step / w.n_groups, "zero_fill_padding": not args.keep_padding},
        "roofline": roofline,
        "pipeline": {"bound": "hbm", "algorithmic_bytes": ab["pipeline"], "achieved": round(pipe_ach, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(pipe_ach / HBM_PEAK_GBS, 4),
                     "traffic": pipe_traffic,
                     # the counter-based figure: bytes the kernels really moved over the same step time
                     "traffic_GB/s": round(pipe_traffic / (ms_per_step * 1e-3) / 1e9, 1) if pipe_traffic else None,
                     "traffic_frac": round(pipe_traffic / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if pipe_traffic else None},
        "kernels": kernels,
        "paper_context": PAPER_CONTEXT,
    }
    if not args.no_lse_handoff:
        out["lse_handoff"] = lse_handoff(args, W, w, st, stream, ab)
    if not args.no_decode:
        out["decode"] = decode_leg(W, w, device, stream, max(args.steps, 20))
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, st)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
