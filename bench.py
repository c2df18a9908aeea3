#!/usr/bin/env python3
"""Benchmark of the real-time pre-ranking scoring path on one MI355X.

A step is one pass of the whole hot path -- aif_score_topk = aif_score_batch
(gather -> user fold -> attention + cross -> MLP) followed by aif_topk -- over one batch of
synthetic requests already resident in HBM.  Default workload: configuration
C3 (64 concurrent users x 10^4 candidates, bf16), the batched 10^4-candidate
request shape the metric is quoted on.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C1..C5 | B3]

``--workload B3`` is C3 with the cross block formed by the Bridge Embedding Approximation (Sec. 4.1).

``--workload U1|U3`` times the user-side asynchronous network alone (aif_user_precompute, Sec. 3.1 Eq. 1-3);
``--workload A3`` the two phases of Sec. 3.1 together: the user network of the next batch of users on one stream
beside the real-time scoring of the current batch on another (and, for comparison, both on one stream).
``--workload N3`` times the nearline incremental update of the item table (aif_update_rows, Sec. 3.4): 10^6 rows
of C3's 10^7-row table per step.
``--workload L1..L3`` times the LSH behaviour-modelling path instead (aif_lsh_batch: user-side bit
tables -> LSH-DIN -> SimTier over every candidate x history pair); same JSON contract, its own metric.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0            # MI355X HBM3E
PEAK_MFMA_BF16_TFLOPS = 2500.0   # dense bf16
PEAK_MFMA_I8_TOPS = 5000.0       # dense int8
PEAK_FP32_VALU_TFLOPS = 157.3
# 32-bit integer vector ALU: the fp32 figure counts 2 flops per FMA and 2 lanes per packed instruction
PEAK_INT_VALU_TOPS = PEAK_FP32_VALU_TFLOPS / 4


def algorithmic_work(cfg, k1=None):
    """Per-candidate algorithmic bytes / flops of each kernel (what the method
    needs, not what the implementation moves); amortised per-request terms
    (K/V, weights) are left out.  k1: the contraction layer 1 of the head computes per candidate
    (aif_mlp_layer1_width: D_in - d_user after the user fold, less the cross block where that is folded into the
    user's layer-1 weights as well -- the reduced count: no credit for avoided work)."""
    B = 4 if cfg.dtype == "f32" else 2
    full = cfg.d_in - cfg.d_user
    k1 = full if k1 is None or k1 <= 0 else k1
    d_cross_moved = cfg.d_cross if k1 == full else 0        # a folded cross block is neither written nor read
    dims = cfg.mlp_dims
    mlp = 2 * (k1 * dims[1] + sum(dims[l] * dims[l + 1] for l in range(1, len(dims) - 1)))
    attn = 4 * cfg.seq_len * cfg.d_attn + (2 * cfg.d_item * cfg.d_attn if cfg.use_wq else 0)
    if d_cross_moved == 0:
        pass                                                # folded into the users' weights: no kernel forms the block
    elif cfg.cross_mode == 2:
        attn += 2 * cfg.d_cross * cfg.d_cross_vec
    elif cfg.cross_mode == 1:
        attn += cfg.d_item
    elif cfg.cross_mode == 3:
        attn += 2 * cfg.n_cross * cfg.d_cross_vec
    return {
        "gather": {"bytes": 4 + 2 * cfg.d_item * B},
        "attention": {"flops": attn, "bytes": cfg.d_item * B + (cfg.d_attn + d_cross_moved) * B},
        "mlp": {"flops": mlp, "bytes": k1 * B + 4},
        "topk": {"bytes": 4},
    }


def measured_traffic(workload, stage):
    """HBM bytes per launch of a stage's kernel as rocprofv3's FETCH_SIZE + WRITE_SIZE counters gave them
    (scaled by a copy kernel of known size); read from the committed counter summaries under profiles/, None if none has a
    line for this workload and stage.  Line format: ``traffic_bytes_per_launch <workload> <stage> <bytes>``."""
    folder = os.path.join(ROOT, "profiles")
    try:
        names = sorted(n for n in os.listdir(folder) if n.endswith(".txt"))
    except OSError:
        return None
    for name in names:
        try:
            with open(os.path.join(folder, name)) as f:
                for ln in f:
                    t = ln.split()
                    if len(t) == 4 and t[0] == "traffic_bytes_per_launch" and t[1] == workload and t[2] == stage:
                        TRAFFIC_SOURCE[(workload, stage)] = "profiles/" + name
                        return float(t[3])
        except OSError:
            pass
    return None


TRAFFIC_SOURCE = {}


def traffic_note(workload, stage):
    """Where roofline.traffic came from: the counters are read in profiling runs of their own, not in this run."""
    src = TRAFFIC_SOURCE.get((workload, stage))
    return f"{src}: committed rocprofv3 FETCH_SIZE/WRITE_SIZE summary of the same command, not measured in this run" if src else None


def achievable_peak(kind):
    """What this chip delivered in the calibration loops of paper_2511_12934_amd/profiling/peaks.py (bf16 MFMAs fed
    from LDS with random operands; a plain device copy), from the committed summary under profiles/; None if absent.
    Line format: ``achievable_peak <mfma_bf16|hbm> <value>``."""
    try:
        with open(os.path.join(ROOT, "profiles", "achievable_peaks.txt")) as f:
            for ln in f:
                t = ln.split()
                if len(t) == 3 and t[0] == "achievable_peak" and t[1] == kind:
                    return float(t[2])
    except OSError:
        pass
    return None


def add_achievable(roof):
    """roofline.frac stays against the published peak; beside it the fraction of what the calibration loops reach."""
    kind = {"mfma": "mfma_bf16", "hbm": "hbm"}.get(roof.get("bound"))
    peak = achievable_peak(kind) if kind else None
    if peak:
        roof["achievable_peak"] = peak
        roof["frac_of_achievable"] = roof["achieved"] / peak
        roof["achievable_source"] = "profiles/achievable_peaks.txt (python3 -m paper_2511_12934_amd.profiling.peaks)"
    return roof


def cpu_baseline(cfg, w, seconds_budget=15.0):
    """The oracle as it stands, on the host cores, on a bounded sample of the same workload:
    whole requests of the first few users, as many as fit in about ``seconds_budget`` of wall time."""
    import numpy as np

    import oracle
    threads = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or (os.cpu_count() or 1))

    def run(u, n_c, n_threads=None):
        rows = w.rows_of(u, np.arange(n_c))
        req = w.requests[u]
        t0 = time.perf_counter()
        ref = oracle.score(table=rows, ids=np.arange(n_c, dtype=np.int32), user_vec=req.user.user_vec,
                           seq_keys=req.user.seq_keys, seq_vals=req.user.seq_vals, dims=w.model.dims,
                           weights=w.model.weights, biases=w.model.biases, w_q=w.model.w_q,
                           n_heads=cfg.n_heads, cross_mode=cfg.cross_mode, cross_vecs=req.user.cross_vecs,
                           n_threads=threads if n_threads is None else n_threads)
        oracle.topk(ref.logits, cfg.top_k)
        return time.perf_counter() - t0

    n_probe = min(w.n_cand, 1000)
    per_cand = run(0, n_probe) / n_probe               # probe (also warms the thread pool)
    t_request = per_cand * w.n_cand
    if t_request > seconds_budget:                      # not even one whole request fits: part of one
        n_users, n_c = 1, max(n_probe, int(w.n_cand * seconds_budget / t_request))
    else:
        n_users, n_c = int(min(w.n_users, max(1, seconds_budget // t_request))), w.n_cand
    t = sum(run(u, n_c) for u in range(n_users))
    # the same loop on ONE thread, on about 5 s' worth of one request's candidates
    n_1 = max(64, min(w.n_cand, int(5.0 / (per_cand * threads))))
    t_1 = run(0, n_1, n_threads=1)
    return {"value": n_users * n_c / t, "unit": "candidates/s", "cores": threads, "kind": "oracle",
            "sample": f"{n_users} request(s) x {n_c} candidates of {cfg.name} (oracle score + top-k, "
                      f"{threads} OpenMP threads, {t:.1f} s wall, {t * threads:.0f} core-seconds)",
            "single_thread": {"value": n_1 / t_1, "unit": "candidates/s", "cores": 1,
                              "sample": f"{n_1} candidates of one {cfg.name} request, one thread, {t_1:.1f} s wall"}}


def _percentiles(ts):
    import numpy as np
    ts = np.sort(np.asarray(ts))
    return {"p50_ms": float(ts[len(ts) // 2]), "p99_ms": float(ts[min(len(ts) - 1, int(len(ts) * 0.99))]), "n": int(len(ts))}


def single_request_latency(n_iter=500):
    """p50/p99 of one 10^4-candidate request (configuration C2), host clock from enqueue to completion of top-k, over
    ``n_iter`` timed iterations after 50 untimed ones, 32 distinct requests rotated:
      whole               one aif_score_topk call;
      10x1000             ten 1,000-item mini-batches in one aif_score_batch (the user side staged once) + aif_topk;
      10x1000_ten_streams the ten mini-batches as ten calls on ten streams through ten contexts (Sec. 1 scores the
                          mini-batches separately and in parallel), joined by events before the one aif_topk;
      graph_replay        the whole request as a captured HIP graph of aif_score_topk_static, replayed."""
    import torch

    from paper_2511_12934_amd import runner as R
    from paper_2511_12934_amd import workloads as wl
    cfg = wl.CONFIGS["C2"]
    warm = 50
    out = {}
    idx = torch.empty((1, cfg.top_k), dtype=torch.int32, device="cuda")
    val = torch.empty((1, cfg.top_k), dtype=torch.float32, device="cuda")

    def timed(body):
        ts = []
        for it in range(n_iter + warm):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            body(it)
            torch.cuda.synchronize()
            if it >= warm:
                ts.append((time.perf_counter() - t0) * 1e3)
        return _percentiles(ts)

    from paper_2511_12934_amd import binding as B
    w = R.Workload(cfg, n_users=32)
    # the argument arrays of every call are marshalled beforehand (a Python loop over ten requests would be timed otherwise)
    one = [B.pack_requests([w.launch[u].req]) for u in range(32)]
    out["whole"] = timed(lambda it: w.ctx.aif_score_topk([w.launch[it % 32].req], cfg.top_k, idx, val, packed=one[it % 32]))
    # the same call with nothing allocated and nothing staged through the host, captured once per request and replayed
    side = torch.cuda.Stream()
    graphs = []
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        w.ctx.aif_score_topk_static(w.launch[0].req, cfg.top_k, idx, val)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for u in range(32):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            w.ctx.aif_score_topk_static(w.launch[u].req, cfg.top_k, idx, val)
        graphs.append(g)
    out["graph_replay"] = timed(lambda it: graphs[it % 32].replay())
    out["static_call"] = timed(lambda it: w.ctx.aif_score_topk_static(w.launch[it % 32].req, cfg.top_k, idx, val))
    del graphs

    wm = R.Workload(cfg, n_users=32, minibatch=1000)
    per_user = len(wm.launch) // wm.n_users

    slices = [[d.req for d in wm.launch[u * per_user:(u + 1) * per_user]] for u in range(32)]
    ten = [B.pack_requests(s) for s in slices]

    def sliced(it):
        u = it % 32
        wm.ctx.aif_score_batch(slices[u], packed=ten[u])
        wm.ctx.aif_topk([wm.dev[u].logits], cfg.top_k, idx, val)
    out["10x1000"] = timed(sliced)

    # ten contexts (a context serves one stream at a time), ten streams; the table and the model tensors are shared
    ctxs = [R.make_context(cfg, wm.dmodel, wm.table, max_users=1, max_candidates=1000) for _ in range(per_user)]
    streams = [torch.cuda.Stream() for _ in range(per_user)]
    done = [torch.cuda.Event() for _ in range(per_user)]

    each = [[B.pack_requests([q]) for q in s] for s in slices]

    def ten_streams(it):
        u = it % 32
        main = torch.cuda.current_stream()
        for j in range(per_user):
            with torch.cuda.stream(streams[j]):
                ctxs[j].aif_score_batch(slices[u][j:j + 1], packed=each[u][j])
                done[j].record()
        for j in range(per_user):
            main.wait_event(done[j])
        wm.ctx.aif_topk([wm.dev[u].logits], cfg.top_k, idx, val)
    out["10x1000_ten_streams"] = timed(ten_streams)
    del w, wm, ctxs
    torch.cuda.empty_cache()
    return out


def step_latency(w, n=100):
    """p50/p99 of one batched step, host clock from enqueue to completion, each step synchronised on its own
    (the throughput figure comes from steps enqueued back to back: its inverse is not a latency)."""
    import torch
    ts = []
    for it in range(n + 10):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        w.step()
        torch.cuda.synchronize()
        if it >= 10:
            ts.append((time.perf_counter() - t0) * 1e3)
    return _percentiles(ts)


def wide_model_block(steps=100, warmup=20):
    """The heavier batched 10^4-candidate configuration (C5, the wide model) in the same run: candidates/s and the
    roofline fraction of its dominant kernel, measured as the headline workload is (fewer steps)."""
    import torch

    from paper_2511_12934_amd import runner as R
    from paper_2511_12934_amd import workloads as wl
    cfg = wl.CONFIGS["C5"]
    w = R.Workload(cfg, n_sets=2)
    for _ in range(warmup):
        w.step()
    torch.cuda.synchronize()
    w.ctx.aif_profile_begin_sampled(steps, ["attention", "mlp"], 4)
    t0 = time.perf_counter()
    for _ in range(steps):
        w.step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = w.ctx.aif_profile_end()
    work = algorithmic_work(cfg, w.ctx.aif_mlp_layer1_width())
    cands = w.total_candidates
    kern = {}
    for st in ("attention", "mlp"):
        avg = prof[st][0] / max(prof[st][1], 1)
        kern[st] = {"avg_ms": avg, "tflops": work[st]["flops"] * cands / (avg * 1e-3) / 1e12,
                    "kind": ("generic", "mfma")[w.ctx.aif_stage_kind(st)]}
    dom = max(kern, key=lambda k: kern[k]["avg_ms"])
    roof = {"kernel": dom, "bound": "mfma", "achieved": kern[dom]["tflops"], "peak": PEAK_MFMA_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": kern[dom]["tflops"] / PEAK_MFMA_BF16_TFLOPS, "traffic": measured_traffic("C5", dom),
            "traffic_source": traffic_note("C5", dom), "avg_ms": kern[dom]["avg_ms"]}
    out = {"workload": f"C5: {w.n_users} users x {w.n_cand} candidates, table {cfg.n_items}x{cfg.d_item} bf16, L={cfg.seq_len}, "
                       f"H={cfg.n_heads}, MLP {list(cfg.mlp_dims)}, top-{cfg.top_k}",
           "value": cands * steps / elapsed, "unit": "candidates/s", "steps": steps, "warmup": warmup,
           "ms_per_step": elapsed / steps * 1e3, "roofline": add_achievable(roof), "kernels": kern,
           "mlp_frac_of_mfma_peak": kern["mlp"]["tflops"] / PEAK_MFMA_BF16_TFLOPS}
    del w
    torch.cuda.empty_cache()
    return out


def lsh_pair_ops(cfg):
    """Algorithmic integer operations per (candidate, history item) pair of SimTier: per 32-bit word of the
    signatures one XNOR and one population count (Eq. 6), then tier index (multiply, shift, clamp) and the
    count increment (Eq. 9)."""
    return 2 * (cfg.d_bits // 32) + 4


def lsh_cpu_baseline(cfg, w, seconds_budget=15.0):
    import numpy as np

    import oracle
    threads = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or (os.cpu_count() or 1))

    def run(u, n_c):
        rq = w.requests[u]
        t0 = time.perf_counter()
        oracle.lsh_request(sig_table=w.table_host, ids=rq.ids[:n_c], seq_sig=rq.user.seq_sigs, u_seq=rq.user.seq_emb,
                           n_tiers=cfg.n_tiers, n_threads=threads)
        return time.perf_counter() - t0

    n_probe = min(w.n_cand, 200)
    per_cand = run(0, n_probe) / n_probe                # probe (also warms the thread pool)
    t_request = per_cand * w.n_cand
    if t_request > seconds_budget:
        n_users, n_c = 1, max(n_probe, int(w.n_cand * seconds_budget / t_request))
    else:
        n_users, n_c = int(min(w.n_users, max(1, seconds_budget // t_request))), w.n_cand
    t = sum(run(u, n_c) for u in range(n_users))
    return {"value": n_users * n_c / t, "unit": "candidates/s", "cores": threads, "kind": "oracle",
            "sample": f"{n_users} request(s) x {n_c} candidates of {cfg.name}, history {w.seq_len} (oracle Eq. 6-9, "
                      f"{threads} OpenMP threads, {t:.1f} s wall, {t * threads:.0f} core-seconds)"}


def main_lsh(args):
    import torch

    from paper_2511_12934_amd import runner as R
    from paper_2511_12934_amd import workloads as wl
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    cfg = wl.LSH_CONFIGS[args.workload]
    w = R.LshWorkload(cfg)
    for _ in range(args.warmup):
        w.step()
    torch.cuda.synchronize()
    w.ctx.aif_lsh_profile_begin(args.steps)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        w.step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = w.ctx.aif_lsh_profile_end()
    ms_per_step = elapsed / args.steps * 1e3
    cands = w.total_candidates
    pairs = cands * w.seq_len
    kernels = {st: {"avg_ms": ms / max(n, 1)} for st, (ms, n) in prof.items()}
    kernels["simtier"]["tops"] = lsh_pair_ops(cfg) * pairs / (kernels["simtier"]["avg_ms"] * 1e-3) / 1e12
    kernels["simtier"]["pairs_per_s"] = pairs / (kernels["simtier"]["avg_ms"] * 1e-3)
    # LSH-DIN: bytes the method needs per candidate: id + signature read, d_out fp32 written
    kernels["din"]["gbs"] = (4 + cfg.d_bits // 8 + 4 * cfg.d_out) * cands / (kernels["din"]["avg_ms"] * 1e-3) / 1e9
    dom = max(kernels, key=lambda k: kernels[k]["avg_ms"])
    on_mfma = w.ctx.aif_lsh_simtier_kind() == 1
    if on_mfma:
        # equal-bit counts as int8 dot products on the matrix cores: d' multiply-adds per pair; the tier counting left on
        # the vector ALU is 448 instructions per 256 pairs and lane in the kernel's loop (1.75 per pair)
        t = kernels["simtier"]["avg_ms"] * 1e-3
        kernels["simtier"]["mfma_tops"] = 2.0 * cfg.d_bits * pairs / t / 1e12
        kernels["simtier"]["valu_tops"] = 1.75 * pairs / t / 1e12
        kernels["simtier"]["valu_frac_of_int_peak"] = kernels["simtier"]["valu_tops"] / PEAK_INT_VALU_TOPS
        kernels["simtier"]["tops_note"] = ("tops = the vector-ALU kernel's algorithmic count (2 d'/32 + 4 per pair) over this "
                                           "kernel's time, for comparison with it only")
    if dom == "simtier" and on_mfma:
        roof = {"kernel": "k_lsh_simtier_mfma", "bound": "mfma", "achieved": kernels[dom]["mfma_tops"], "peak": PEAK_MFMA_I8_TOPS,
                "unit": "Top/s", "binding_unit": "vector ALU (tier counting), %.2f of its integer peak"
                                                 % kernels[dom]["valu_frac_of_int_peak"]}
    elif dom == "simtier":
        roof = {"kernel": "k_lsh_simtier", "bound": "alu", "achieved": kernels[dom]["tops"], "peak": PEAK_INT_VALU_TOPS,
                "unit": "Top/s"}
    elif dom == "din":
        roof = {"kernel": "k_lsh_din", "bound": "hbm", "achieved": kernels[dom]["gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s"}
    else:
        flops = 4.0 * cfg.d_bits * cfg.d_out * w.seq_len * w.n_users       # two masked multiply-adds per (t, k, j)
        roof = {"kernel": "k_lsh_user_partial", "bound": "alu", "achieved": flops / (kernels[dom]["avg_ms"] * 1e-3) / 1e12,
                "peak": PEAK_FP32_VALU_TFLOPS / 2, "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = measured_traffic(cfg.name, dom)
    roof["traffic_source"] = traffic_note(cfg.name, dom)
    roof["avg_ms"] = kernels[dom]["avg_ms"]
    line = {
        "metric": "candidates served/sec/GPU by the LSH behaviour modelling (LSH-DIN + SimTier)",
        "value": cands * args.steps / elapsed, "unit": "candidates/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": ("i8" if on_mfma else "u32") if dom == "simtier" else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {w.n_users} users x {w.n_cand} candidates x {w.seq_len} history items, "
                               f"{cfg.d_bits}-bit signatures (table {cfg.n_items} rows), d={cfg.d_out} {cfg.dtype}, "
                               f"{cfg.n_tiers} tiers",
                   "users": w.n_users, "candidates_per_request": w.n_cand, "seq_len": w.seq_len},
        "pairs_per_s": pairs * args.steps / elapsed,
        "roofline": roof, "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = lsh_cpu_baseline(cfg, w)
    print(json.dumps(line))


def user_net_work(cfg):
    """Algorithmic flops per user of the user-side network: Eq. 1 projections, the two attentions (every position
    and the profile over the l positions), the FFN."""
    L, d, dr = cfg.seq_len, cfg.d, cfg.d_raw
    return {"project": 2 * (L + 1) * dr * d, "attention": 4 * (L + 1) * L * d, "ffn_pool": 2 * L * d * d + L * d}


def user_cpu_baseline(cfg, w, seconds_budget=15.0):
    import oracle
    t0 = time.perf_counter()
    n = 0
    for u in w.users:
        oracle.user_network(profile=u.profile, seq=u.seq, w_profile=w.model.w_profile, w_seq=w.model.w_seq,
                            w_ffn=w.model.w_ffn, b_ffn=w.model.b_ffn)
        n += 1
        if time.perf_counter() - t0 > seconds_budget:
            break
    t = time.perf_counter() - t0
    return {"value": n / t, "unit": "users/s", "cores": 1, "kind": "oracle",
            "sample": f"{n} user(s) of {cfg.name}, l = {cfg.seq_len} (oracle Eq. 1-3, one thread, {t:.1f} s wall)"}


def main_user(args):
    import torch

    from paper_2511_12934_amd import runner as R
    from paper_2511_12934_amd import workloads as wl
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    cfg = wl.USER_CONFIGS[args.workload]
    w = R.UserNetWorkload(cfg)
    for _ in range(args.warmup):
        w.step()
    torch.cuda.synchronize()
    w.ctx.aif_user_profile_begin(args.steps)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        w.step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = w.ctx.aif_user_profile_end()
    ms_per_step = elapsed / args.steps * 1e3
    work = user_net_work(cfg)
    mf = w.ctx.aif_user_attention_kind() == 1
    kernels = {}
    for st in ("project", "attention", "ffn_pool"):
        ms, n = prof[st]
        avg = ms / max(n, 1)
        kernels[st] = {"avg_ms": avg, "tflops": work[st] * w.n_users / (avg * 1e-3) / 1e12 if avg > 0 else None}
    kernels["attention"]["kind"] = "mfma" if mf else "generic"
    dom = max(kernels, key=lambda k: kernels[k]["avg_ms"])
    on_mfma = dom == "attention" and mf
    roof = {"kernel": dom, "bound": "mfma" if on_mfma else "alu", "achieved": kernels[dom]["tflops"],
            "peak": PEAK_MFMA_BF16_TFLOPS if on_mfma else PEAK_FP32_VALU_TFLOPS, "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = measured_traffic(cfg.name, dom)
    roof["traffic_source"] = traffic_note(cfg.name, dom)
    roof["avg_ms"] = kernels[dom]["avg_ms"]
    line = {
        "metric": "users served/sec/GPU by the asynchronous user-side network (Eq. 1-3)",
        "value": w.n_users * args.steps / elapsed, "unit": "users/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {w.n_users} users x {cfg.seq_len} positions, raw width {cfg.d_raw}, "
                               f"d = {cfg.d}, {cfg.dtype}", "users": w.n_users, "seq_len": cfg.seq_len},
        "roofline": roof, "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = user_cpu_baseline(cfg, w)
    print(json.dumps(line))


def main_async(args):
    import torch

    from paper_2511_12934_amd import runner as R
    from paper_2511_12934_amd import workloads as wl
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    cfg, ucfg = wl.CONFIGS["A3"], wl.USER_CONFIGS["U3"]
    p = R.AsyncPipeline(cfg, ucfg)

    # the first steps on a stream that has not run yet are slow (tens of ms once): warm both modes up well
    warm = max(args.warmup, 30)
    warm += warm % 2

    def timed(overlap, profile):
        if overlap:
            p.prime()
        for i in range(warm):
            p.step(i, overlap)
        torch.cuda.synchronize()
        if profile:
            p.ctx.aif_profile_begin(args.steps)
            p.uctx.aif_user_profile_begin(args.steps)
        t0 = time.perf_counter()
        for i in range(warm, warm + args.steps):
            p.step(i, overlap)
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        return el, (p.ctx.aif_profile_end(), p.uctx.aif_user_profile_end()) if profile else None

    serial, (prof, uprof) = timed(False, True)
    over, _ = timed(True, False)
    ms_per_step = over / args.steps * 1e3
    work = algorithmic_work(cfg, p.ctx.aif_mlp_layer1_width())
    if p.ctx.aif_stage_kind("gather") == 2:          # the attention kernel indexed the table itself, see main()
        B = 4 if cfg.dtype == "f32" else 2
        work["attention"]["bytes"] += work["gather"]["bytes"] - cfg.d_item * B
        work["gather"]["bytes"] = 0
    cands = p.total_candidates
    kernels = {}
    for stage in ("gather", "attention", "mlp", "topk"):
        ms, n = prof[stage]
        avg_ms = ms / max(n, 1)
        ent = {"avg_ms": avg_ms, "kind": "mfma" if p.ctx.aif_stage_kind(stage) == 1 else "generic"}
        if "flops" in work[stage] and avg_ms > 0:
            ent["tflops"] = work[stage]["flops"] * cands / (avg_ms * 1e-3) / 1e12
        if avg_ms > 0 and work[stage]["bytes"] > 0:
            ent["gbs"] = work[stage]["bytes"] * cands / (avg_ms * 1e-3) / 1e9
        kernels[stage] = ent
    for st in ("project", "attention", "ffn_pool"):
        ms, n = uprof[st]
        kernels["user_" + st] = {"avg_ms": ms / max(n, 1)}
    roof = {"kernel": "mlp", "bound": "mfma", "achieved": kernels["mlp"]["tflops"], "peak": PEAK_MFMA_BF16_TFLOPS,
            "unit": "TFLOP/s", "frac": kernels["mlp"]["tflops"] / PEAK_MFMA_BF16_TFLOPS,
            "traffic": measured_traffic(cfg.name, "mlp"), "avg_ms": kernels["mlp"]["avg_ms"],
            "note": "per-kernel times from the one-stream run (kernels of the two streams share the device in the overlapped one)"}
    line = {
        "metric": "candidates scored/sec/GPU at 10^4-cand requests", "value": cands * args.steps / over,
        "unit": "candidates/s", "n_gpus": 1, "steps": args.steps, "warmup": warm, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"A3: per step the user-side network (Eq. 1-3) of the next {p.n_users} users (l = {ucfg.seq_len}, "
                               f"raw width {ucfg.d_raw}) on one stream beside scoring + top-{cfg.top_k} of {p.n_users} users x "
                               f"{p.n_cand} candidates on another; table {cfg.n_items}x{cfg.d_item} {cfg.dtype}, "
                               f"MLP {list(cfg.mlp_dims)}", "users": p.n_users, "candidates_per_request": p.n_cand,
                   "top_k": cfg.top_k},
        "one_stream_ms_per_step": serial / args.steps * 1e3,
        "user_network_ms": sum(kernels["user_" + st]["avg_ms"] for st in ("project", "attention", "ffn_pool")),
        "roofline": roof, "kernels": kernels,
    }
    print(json.dumps(line))


def main_update(args, n_upd=1_000_000):
    import numpy as np
    import torch

    import oracle
    from paper_2511_12934_amd import runner as R
    from paper_2511_12934_amd import workloads as wl
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    cfg = wl.CONFIGS["C3"]
    w = R.Workload(cfg, n_users=1, n_cand=1000)
    rng = np.random.default_rng(cfg.seed + 77)
    # four id lists taken in turn, so a step does not rewrite the rows the last one left in the caches
    id_sets = [torch.from_numpy(rng.permutation(cfg.n_items)[:n_upd].astype(np.int32)).to("cuda:0") for _ in range(4)]
    rows = (torch.randn((n_upd, cfg.d_item), device="cuda:0") * 0.1).to(torch.bfloat16)
    for i in range(args.warmup):
        w.ctx.aif_update_rows(id_sets[i % 4], rows)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(args.steps):
        w.ctx.aif_update_rows(id_sets[i % 4], rows)
        ev[i + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert w.ctx.aif_poll_device_errors() == 0
    kern_ms = sum(ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps)) / args.steps
    bytes_per_row = 4 + 2 * cfg.d_item * 2
    gbs = bytes_per_row * n_upd / (kern_ms * 1e-3) / 1e9
    line = {
        "metric": "item-table rows updated/sec/GPU (nearline incremental update)", "value": n_upd * args.steps / elapsed,
        "unit": "rows/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"N3: {n_upd} distinct rows of C3's table ({cfg.n_items}x{cfg.d_item} bf16) per step, "
                               "four id lists in turn", "rows_per_step": n_upd},
        "roofline": {"kernel": "k_update_rows", "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": gbs / PEAK_HBM_GBS, "traffic": measured_traffic("N3", "update"), "avg_ms": kern_ms},
    }
    if not args.no_cpu_baseline:
        n_t, n_u = 1_000_000, 200_000
        t = np.zeros((n_t, cfg.d_item), np.float32)
        ids = rng.permutation(n_t)[:n_u].astype(np.int32)
        r = rng.standard_normal((n_u, cfg.d_item)).astype(np.float32)
        reps, c0 = 0, time.perf_counter()
        while time.perf_counter() - c0 < 5.0:
            oracle.update_rows(t, ids, r, inplace=True)
            reps += 1
        ct = time.perf_counter() - c0
        line["cpu_baseline"] = {"value": reps * n_u / ct, "unit": "rows/s", "cores": 1, "kind": "oracle",
                                "sample": f"{reps} update(s) of {n_u} rows of a {n_t}x{cfg.d_item} fp32 table (oracle, one thread, {ct:.1f} s wall)"}
    print(json.dumps(line))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # the board settles at its sustained clocks after some 100 ms of load: 50 steps after 5 read about 4 % slower
    # (the scoring workloads C1..C5, B3; the others keep 50 steps after 5)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3", "C4", "C5", "B3", "A3", "U1", "U3", "N3", "L1", "L2", "L3"])
    ap.add_argument("--id-sets", type=int, default=4,
                    help="distinct candidate lists per user, taken in turn by consecutive steps")
    ap.add_argument("--profile-every", type=int, default=8,
                    help="inside the timed region the dominant kernel of every n-th step is timed with events")
    ap.add_argument("--settle-ms", type=float, default=300.0,
                    help="untimed steps run for this long before the warm-up, so that the board's clocks have settled")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-latency", action="store_true")
    args = ap.parse_args()
    sustained = args.workload[0] in "CB"
    if args.steps is None:
        args.steps = 1000 if sustained else 50
    if args.warmup is None:
        args.warmup = 200 if sustained else 5
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (requests shard by user with no exchange; "
                 "one process per GPU); run with --gpus 1")

    if args.workload.startswith("L"):
        return main_lsh(args)
    if args.workload.startswith("U"):
        return main_user(args)
    if args.workload == "A3":
        return main_async(args)
    if args.workload == "N3":
        return main_update(args)

    import torch

    from paper_2511_12934_amd import runner as R
    from paper_2511_12934_amd import workloads as wl
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    cfg = wl.CONFIGS[args.workload]
    w = R.Workload(cfg, n_sets=args.id_sets)
    # The workload is built on the host for seconds while the device idles at its lowest clocks, and a run of a few
    # dozen steps would be over before the board has settled (its first 100 ms read 4-8 % slow): the same steps are run
    # untimed for --settle-ms first.  They are not part of `warmup` (the W warm-up steps below still run) and are
    # reported as `settle_steps`.
    settle_steps = 0
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
        for _ in range(8):
            w.step()
        torch.cuda.synchronize()
        settle_steps += 8
    for _ in range(args.warmup):
        w.step()
    torch.cuda.synchronize()

    # Every stage's time comes from a few profiled steps BEFORE the timed region (two events per stage cost the
    # stream some microseconds each); inside the timed region only the dominant kernel is bracketed by events,
    # and its time there is the one the roofline line uses.
    n_pre = max(3, min(10, args.steps))
    w.ctx.aif_profile_begin(n_pre)
    for _ in range(n_pre):
        w.step()
    torch.cuda.synchronize()
    prof = w.ctx.aif_profile_end()
    dom = max(("gather", "attention", "mlp"), key=lambda s: prof[s][0] / max(prof[s][1], 1))

    # ... and of it one launch in eight: an event keeps the stream idle for 4-5 us, two per step were 2 % of C3's step
    every = args.profile_every if args.steps >= 8 * args.profile_every else 1
    w.ctx.aif_profile_begin_sampled(args.steps, [dom], every)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        w.step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof[dom] = w.ctx.aif_profile_end()[dom]
    ms_per_step = elapsed / args.steps * 1e3
    value = w.total_candidates * args.steps / elapsed

    work = algorithmic_work(cfg, w.ctx.aif_mlp_layer1_width())
    if w.ctx.aif_stage_kind("gather") == 2:
        # the attention kernel indexed the table itself: id + table row read + item row written are its bytes
        # (in place of the item row it would have read from the workspace); the gather stage moved none
        B = 4 if cfg.dtype == "f32" else 2
        work["attention"]["bytes"] += work["gather"]["bytes"] - cfg.d_item * B
        work["gather"]["bytes"] = 0
    cands = w.total_candidates
    kernels = {}
    for stage in ("gather", "attention", "mlp", "topk"):
        ms, n = prof[stage]
        avg_ms = ms / max(n, 1)
        ent = {"avg_ms": avg_ms,
               "kind": ("generic", "mfma", "inside the attention kernel")[w.ctx.aif_stage_kind(stage)]}
        wk = work[stage]
        if "flops" in wk and avg_ms > 0:
            ent["tflops"] = wk["flops"] * cands / (avg_ms * 1e-3) / 1e12
        if avg_ms > 0 and wk["bytes"] > 0:
            ent["gbs"] = wk["bytes"] * cands / (avg_ms * 1e-3) / 1e9
        kernels[stage] = ent
    for st in kernels:
        kernels[st]["timed_in"] = ("timed region, one launch in %d" % every if st == dom else
                                   "profiled pre-pass of %d steps with events around every stage (reads a few microseconds high)" % n_pre)
    if dom == "gather":
        roof = {"kernel": "k_gather", "bound": "hbm", "achieved": kernels[dom]["gbs"], "peak": PEAK_HBM_GBS,
                "unit": "GB/s"}
    else:
        mf = cfg.dtype == "bf16" and kernels[dom]["kind"] == "mfma"
        roof = {"kernel": dom, "bound": "mfma" if mf else "alu", "achieved": kernels[dom]["tflops"],
                "peak": PEAK_MFMA_BF16_TFLOPS if mf else PEAK_FP32_VALU_TFLOPS, "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = measured_traffic(cfg.name, dom)
    roof["traffic_source"] = traffic_note(cfg.name, dom)
    roof["avg_ms"] = kernels[dom]["avg_ms"]
    add_achievable(roof)
    k1_full, k1_done = cfg.d_in - cfg.d_user, w.ctx.aif_mlp_layer1_width()
    if dom == "mlp":
        # the flops that `achieved` counts: what the kernel computes per candidate, not what the unfused model would
        roof["flops_per_candidate"] = work["mlp"]["flops"]
        roof["layer1_width_per_candidate"] = k1_done
        roof["layer1_width_note"] = (
            "D_in - d_user after the user fold" if k1_done == k1_full else
            f"{k1_done} of the {k1_full} columns left after the user fold: the Hadamard cross block's share is folded into each "
            "user's layer-1 weights once per user, so it is not computed per candidate and not counted")

    line = {
        "metric": "candidates scored/sec/GPU at 10^4-cand requests",
        "value": value, "unit": "candidates/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "settle_steps": settle_steps, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {w.n_users} users x {w.n_cand} candidates, table {cfg.n_items}x{cfg.d_item} "
                               f"{cfg.dtype}, L={cfg.seq_len}, d_attn={cfg.d_attn}, H={cfg.n_heads}, "
                               f"MLP {list(cfg.mlp_dims)}, top-{cfg.top_k}",
                   "users": w.n_users, "candidates_per_request": w.n_cand, "top_k": cfg.top_k,
                   "candidate_lists_rotated": args.id_sets},
        "roofline": roof,
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(cfg, w)
    if not args.no_latency:
        line["step_latency_ms"] = step_latency(w)
        del w
        torch.cuda.empty_cache()
        line["single_request_latency_C2"] = single_request_latency()
        if args.workload == "C3":
            line["wide_model_C5"] = wide_model_block()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
