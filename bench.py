#!/usr/bin/env python3
"""Benchmark of the decode hot path on one MI355X.

One step = one pass of the whole path (centroid scoring -> threshold selection / range compaction ->
split-KV sparse attention over the kept fixed-context keys + the dense user keys -> merge) for one
decode token, through the C ABI (`sq_decode_step`), on seeded synthetic inputs already resident in
HBM.  Steps rotate through `--queries` different query tokens (the paper times 100 different query
tokens per measurement, Appendix "Kernel Benchmarking") and through `--replicas` device copies of
the fixed context, so that the bytes of a step cannot be served from the 256 MB last-level cache.

Prints ONE JSON line: `value` = algorithmic bytes of the whole step / time per step; `roofline` = the dominant
kernel (bytes it has to read / its event-timed duration, against the published 8 TB/s); `cpu_baseline` = the CPU
oracle timed on this host on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0       # MI355X published HBM3E bandwidth
MFMA_F16_PEAK_TFLOPS = 2500.0  # MI355X published dense fp16 matrix rate
METRIC = "decode attn µs/token + achieved HBM GB/s, 32K fixed ctx, keep 1/8, H=32 d=128"


def gpu_score_fn(sq, torch, device):
    """`score_fn` for the workload calibration that runs Eq. 1 through the library (sq_centroid_score)."""
    def fn(q, centroids, sizes, sm_scale):
        nq, d = q.shape
        Cn = centroids.shape[0]
        sh = sq.make_shape(1, 1, 1, Cn, nq, 0, sm_scale)
        tq = torch.from_numpy(np.ascontiguousarray(q)).to(device).view(1, 1, nq, d)
        tc = torch.from_numpy(np.ascontiguousarray(centroids)).to(device).view(1, Cn, d)
        ts = torch.from_numpy(np.ascontiguousarray(sizes, dtype=np.int32)).to(device).view(1, Cn)
        x = torch.empty(1, 1, nq, Cn, dtype=torch.float32, device=device)
        m = torch.empty(1, 1, nq, dtype=torch.float32, device=device)
        D = torch.empty(1, 1, nq, dtype=torch.float32, device=device)
        sq.sq_centroid_score(sh, tq, tc, ts, x, m, D)
        torch.cuda.synchronize()
        x, m, D = (a.cpu().numpy().astype(np.float64) for a in (x, m, D))
        return np.exp(x[0, 0] - m[0, 0][:, None]) / D[0, 0][:, None]
    return fn


def step_bytes(w, n_keys_per_head):
    """Algorithmic HBM bytes of one decode step for the achieved selection (bytes the method must move)."""
    from paper_2411_09688_amd.bytes_model import decode_step_bytes
    return decode_step_bytes(w.H, w.C, w.d, w.U, w.B, n_keys_per_head)


def read_traffic(name):
    """Entries for `roofline`: HBM bytes per launch of the dominant kernel from a committed rocprofv3 --pmc summary
    (`traffic`, None without one), the algorithmic bytes per launch OF THAT SAME RUN, and their ratio.  The counter run covers other query
    tokens than this run, so the counter figure is only ever compared with its own run's byte count."""
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return {"traffic": None}
    vals = {}
    for line in open(path):
        for key in ("traffic_bytes_per_launch", "algorithmic_bytes_per_launch"):
            if line.startswith(key + ":"):
                vals[key] = float(line.split(":", 1)[1])
    t, a = vals.get("traffic_bytes_per_launch"), vals.get("algorithmic_bytes_per_launch")
    if t is None:
        return {"traffic": None}
    return {"traffic": t, "traffic_run_bytes_per_launch": a, "traffic_over_run_bytes": round(t / a, 4) if a else None,
            "traffic_source": "profiles/" + name}


def stream_ceiling(sq, torch, dev, nbytes, reps=30):
    """Measured on this device, in this run: bandwidth of a plain streaming read (sq_probe_stream_read, 512 workgroups,
    non-temporal 16-byte loads) of as many bytes as the dominant kernel moves per launch, rotating through enough
    buffers that the 256 MB last-level cache cannot serve them.  What an HBM-bound kernel of this size can approach."""
    n = int(max(1 << 24, min(int(nbytes), 1 << 30))) & ~255
    nbuf = max(2, min(16, -(-(3 << 28) // n)))
    bufs = [torch.ones(n, dtype=torch.uint8, device=dev) for _ in range(nbuf)]
    sink = torch.zeros(1024, dtype=torch.int32, device=dev)
    for i in range(4):
        sq.sq_probe_stream_read(bufs[i % nbuf], sink, 512, n)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(reps):
            sq.sq_probe_stream_read(bufs[i % nbuf], sink, 512, n)
    g.replay()
    torch.cuda.synchronize()
    e0.record()
    g.replay()
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / reps
    del bufs
    return {"stream_ceiling_GBps": round(n / us / 1e3, 1), "stream_ceiling_bytes": n, "stream_ceiling_us": round(us, 3)}


def cpu_baseline(w_name, seed, budget_s):
    """The CPU oracle, as it stands, timed on this host on a bounded sample of the same workload."""
    import oracle
    from paper_2411_09688_amd import workload as wl
    w = wl.calibrate(wl.make_config(w_name, seed=seed), oracle.scores)
    qs = wl.extra_queries(w, 100)
    n, t_total, nbytes = 0, 0.0, 0
    while n < 100 and t_total < budget_s:
        q = np.ascontiguousarray(qs[n][None, :, None, :])
        t0 = time.perf_counter()
        x, m, D = oracle.centroid_score(q, w.centroids, w.sizes, w.sm_scale)
        mask, ranges, nr, nk = oracle.select(x, m, D, w.thresh, w.sizes, w.offsets)
        oracle.sparse_attn(q, w.K_fixed, w.V_fixed, ranges, nr, w.K_user, w.V_user, w.sm_scale)
        t_total += time.perf_counter() - t0
        nbytes += step_bytes(w, nk)["total"]
        n += 1
    res = dict(value=round(nbytes / t_total / 1e9, 3), unit="GB/s", us_per_token=round(t_total / n * 1e6, 1),
               cores=oracle.num_threads(), kind="oracle",
               sample=f"{n} decode steps (different query tokens) of {w_name}, whole path, same byte model")
    res["selection_quality"] = selection_quality(oracle, w, qs[:4])
    return res


def selection_quality(oracle, w, qs):
    """Diagnostic (untimed, CPU, fp64): the share of the true attention mass over the fixed context that the kept keys
    carry, next to what an ideal lookup with the same key budget would carry (the keys with the highest attention
    scores, found by attending to every key first: the "Ideal" baseline of the paper's appendix)."""
    got, ideal = [], []
    for q in qs:
        qh = np.ascontiguousarray(q[None, :, None, :])
        x, m, D = oracle.centroid_score(qh, w.centroids, w.sizes, w.sm_scale)
        mask, ranges, nr, nk = oracle.select(x, m, D, w.thresh, w.sizes, w.offsets)
        for h in range(w.H):
            s = np.float64(w.sm_scale) * (w.K_fixed[h].astype(np.float64) @ q[h].astype(np.float64))
            p = np.exp(s - s.max())
            p /= p.sum()
            kept = np.zeros(w.L, bool)
            for a, c in ranges[0, h, 0, :nr[0, h, 0]]:
                kept[a:a + c] = True
            k = int(kept.sum())
            got.append(p[kept].sum())
            ideal.append(np.sort(p)[::-1][:k].sum())
    return dict(attention_mass_kept=round(float(np.mean(got)), 4),
                attention_mass_ideal_same_budget=round(float(np.mean(ideal)), 4),
                sample=f"{len(qs)} query tokens x {w.H} heads, fixed-context keys only")


def time_steps(step, args, torch, sq):
    """W warm-up steps, K timed eager steps, the same K steps as one HIP-graph replay, then K steps with the
    library's event hook around the dominant kernel.  step(i, stream_ptr) enqueues step i."""
    import ctypes as C

    def cur_stream():
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)

    st = cur_stream()
    for i in range(args.warmup):
        step(i, st)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, st)
    torch.cuda.synchronize()
    eager_ms = (time.perf_counter() - t0) / args.steps * 1e3

    graph_ms = None
    if not args.no_graph:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            st_cap = cur_stream()
            for i in range(args.steps):
                step(args.warmup + i, st_cap)
        g.replay()                                   # untimed replay (warm-up of the graph itself)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) / args.steps * 1e3
    ms_per_step = min(eager_ms, graph_ms) if graph_ms is not None else eager_ms

    sq.sq_profile_begin(args.steps)
    for i in range(args.steps):
        step(args.warmup + i, st)
    torch.cuda.synchronize()
    return eager_ms, graph_ms, ms_per_step, sq.sq_profile_end()


def base_result(args, metric, value, unit, ms_per_step, eager_ms, graph_ms, tokens):
    return {
        "metric": metric, "value": value, "unit": unit,
        "us_per_token": round(ms_per_step * 1e3 / tokens, 3),
        "us_per_step_eager": round(eager_ms * 1e3, 3),
        "us_per_step_graph": None if graph_ms is None else round(graph_ms * 1e3, 3),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
    }


def bench_prefill(args, torch, sq, wl, dev):
    """Config 4: scores -> per-query masks -> sparse prefill attention; dominant kernel prefill_attn_kernel (MFMA)."""
    import ctypes as C
    w = wl.make_config(args.workload, seed=args.seed, threads=16)
    wl.calibrate(w, gpu_score_fn(sq, torch, dev))
    R = max(1, min(args.replicas, 2))
    Ps = [sq.upload(w, dev) for _ in range(R)]
    shape = Ps[0].shape
    ws = sq.workspace(shape, sq.SQ_CALL_ATTN_PREFILL, dev)
    ws_step = sq.workspace(shape, sq.SQ_CALL_PREFILL_STEP, dev)

    def step(i, stream_ptr):
        P = Ps[i % R]
        if args.separate:
            sq.sq_centroid_score(shape, P.q, P.centroids, P.sizes, P.logits, P.row_max, P.denom)
            sq.sq_select(shape, P.logits, P.row_max, P.denom, P.thresh, P.sizes, P.offsets, P.keep_mask, None,
                         P.n_ranges, P.n_keys)
            sq.sq_sparse_attn_prefill(shape, P.q, P.K_fixed, P.V_fixed, P.offsets, P.keep_mask, P.K_user, P.V_user,
                                      P.out, P.lse, ws)
        else:
            sq.sq_prefill_step(shape, P.q, P.centroids, P.sizes, P.offsets, P.thresh, P.K_fixed, P.V_fixed, P.K_user,
                               P.V_user, P.out, P.lse, None, P.n_keys, ws_step)

    if args.selection == "mean":
        return bench_prefill_mean(args, torch, sq, wl, dev, w, Ps)
    eager_ms, graph_ms, ms, (n_meas, k_avg, k_min, k_max) = time_steps(step, args, torch, sq)
    nk = Ps[0].n_keys.cpu().numpy().astype(np.float64)            # [B,H,Lq]
    t = np.arange(w.Lq)
    user_vis = np.minimum(t + 1, w.U) if w.causal_user else np.full(w.Lq, w.U)
    useful_attn = float((nk.sum() + w.B * w.H * user_vis.sum()) * 4 * w.d)
    score_flops = 2.0 * w.B * w.H * w.Lq * w.C * w.d
    # executed by the attention kernel: every 64-key block of the fixed context and of the visible user keys,
    # for every query of a 64-query workgroup (wave-level skips not subtracted)
    nb_fixed = -(-w.L // 64)
    q0 = np.arange(0, w.Lq, 64)
    nb_user = -(-np.minimum(w.U, q0 + 64) // 64) if w.causal_user else np.full(len(q0), -(-w.U // 64))
    executed = float(w.B * w.H * ((nb_fixed * len(q0) + nb_user.sum()) * 64 * 64) * 4 * w.d)
    tokens = w.B * w.Lq
    res = base_result(args, "sparse prefill attn: useful TFLOP/s (per-query selection), 32K fixed ctx, keep 1/8",
                      round((useful_attn + score_flops) / (ms * 1e-3) / 1e12, 3), "TFLOP/s", ms, eager_ms, graph_ms,
                      tokens)
    res["config"] = {"workload": args.workload, "B": w.B, "H": w.H, "d": w.d, "L": w.L, "C": w.C, "Lq": w.Lq,
                     "U": w.U, "keep_achieved": round(float(nk.mean() / w.L), 5), "replicas": R,
                     "entry": "sq_centroid_score + sq_select + sq_sparse_attn_prefill" if args.separate
                     else "sq_prefill_step"}
    res["flops_per_step"] = {"useful_attention": useful_attn, "scoring": score_flops,
                             "executed_attention_upper_bound": executed}
    res["roofline"] = {"bound": "mfma", "kernel": "prefill_attn_kernel",
                       "achieved": round(useful_attn / (k_avg * 1e-6) / 1e12, 2) if n_meas else None,
                       "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                       "frac": round(useful_attn / (k_avg * 1e-6) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4) if n_meas else None,
                       "executed_TFLOPs": round(executed / (k_avg * 1e-6) / 1e12, 2) if n_meas else None,
                       "executed_frac": round(executed / (k_avg * 1e-6) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4) if n_meas else None,
                       **read_traffic(f"prefill_attn_kernel_{args.workload}_pmc.txt"),
                       "flops_per_launch": useful_attn, "avg_us": round(k_avg, 2), "min_us": round(k_min, 2),
                       "launches": n_meas}
    print(json.dumps(res, ensure_ascii=False))


def bench_prefill_mean(args, torch, sq, wl, dev, w, Ps):
    """Config 4's shape with the paper's own prefill rule (Appendix D): scores averaged over the query tokens ->
    one kept set per (sequence, head) -> attention that gathers only the kept keys."""
    R = len(Ps)
    shape = Ps[0].shape
    W = (w.C + 31) // 32
    mask = torch.zeros(w.B, w.H, W, dtype=torch.int32, device=dev)
    ranges = torch.zeros(w.B, w.H, w.C, 2, dtype=torch.int32, device=dev)
    nr = torch.zeros(w.B, w.H, dtype=torch.int32, device=dev)
    nk = torch.zeros(w.B, w.H, dtype=torch.int32, device=dev)
    ws_s = sq.workspace(shape, sq.SQ_CALL_SELECT_MEAN, dev)
    ws_a = sq.workspace(shape, sq.SQ_CALL_ATTN_PREFILL_SHARED, dev)
    ws_step = sq.workspace(shape, sq.SQ_CALL_PREFILL_MEAN_STEP, dev)
    nk_step = torch.zeros(w.B, w.H, dtype=torch.int32, device=dev)
    # Thresholds on the averaged scores that keep w.keep_frac of the keys per head: bisection on the library's own
    # counts (log domain), untimed.
    P = Ps[0]
    sq.sq_centroid_score(shape, P.q, P.centroids, P.sizes, P.logits, P.row_max, P.denom)
    lo, hi = np.full(w.H, -40.0), np.full(w.H, 0.0)
    thr = torch.zeros(w.H, dtype=torch.float32, device=dev)
    for _ in range(40):
        mid = 0.5 * (lo + hi)
        thr.copy_(torch.from_numpy(np.exp(mid).astype(np.float32)))
        sq.sq_select_mean(shape, P.logits, P.row_max, P.denom, thr, P.sizes, P.offsets, mask, ranges, nr, nk, ws_s)
        kept = nk.cpu().numpy().mean(axis=0)                      # per head
        too_many = kept > w.keep_frac * w.L
        lo = np.where(too_many, mid, lo)
        hi = np.where(too_many, hi, mid)
    thr.copy_(torch.from_numpy(np.exp(hi).astype(np.float32)))

    def step(i, stream_ptr):
        P = Ps[i % R]
        if args.separate:
            sq.sq_centroid_score(shape, P.q, P.centroids, P.sizes, P.logits, P.row_max, P.denom)
            sq.sq_select_mean(shape, P.logits, P.row_max, P.denom, thr, P.sizes, P.offsets, mask, ranges, nr, nk, ws_s)
            sq.sq_sparse_attn_prefill_shared(shape, P.q, P.K_fixed, P.V_fixed, ranges, nr, nk, P.K_user, P.V_user,
                                             P.out, P.lse, ws_a)
        else:
            sq.sq_prefill_mean_step(shape, P.q, P.centroids, P.sizes, P.offsets, thr, P.K_fixed, P.V_fixed, P.K_user,
                                    P.V_user, P.out, P.lse, None, nk_step, ws_step)

    eager_ms, graph_ms, ms, (n_meas, k_avg, k_min, k_max) = time_steps(step, args, torch, sq)
    nkh = (nk if args.separate else nk_step).cpu().numpy().astype(np.float64)   # [B,H]
    t = np.arange(w.Lq)
    user_vis = np.minimum(t + 1, w.U) if w.causal_user else np.full(w.Lq, w.U)
    useful_attn = float((nkh.sum() * w.Lq + w.B * w.H * user_vis.sum()) * 4 * w.d)
    score_flops = 2.0 * w.B * w.H * w.Lq * w.C * w.d
    q0 = np.arange(0, w.Lq, 64)
    nb_user = -(-np.minimum(w.U, q0 + 64) // 64) if w.causal_user else np.full(len(q0), -(-w.U // 64))
    executed = float(((np.ceil(nkh / 64).sum() * len(q0)) + w.B * w.H * nb_user.sum()) * 64 * 64 * 4 * w.d)
    res = base_result(args, "sparse prefill attn: useful TFLOP/s (selection on averaged scores), 32K fixed ctx, keep 1/8",
                      round((useful_attn + score_flops) / (ms * 1e-3) / 1e12, 3), "TFLOP/s", ms, eager_ms, graph_ms,
                      w.B * w.Lq)
    res["config"] = {"workload": args.workload, "selection": "mean", "B": w.B, "H": w.H, "d": w.d, "L": w.L,
                     "C": w.C, "Lq": w.Lq, "U": w.U, "keep_achieved": round(float(nkh.mean() / w.L), 5), "replicas": R,
                     "entry": "sq_centroid_score + sq_select_mean + sq_sparse_attn_prefill_shared" if args.separate
                     else "sq_prefill_mean_step"}
    res["flops_per_step"] = {"useful_attention": useful_attn, "scoring": score_flops, "executed_attention": executed}
    res["roofline"] = {"bound": "mfma", "kernel": "prefill_attn_kernel<shared>",
                       "achieved": round(useful_attn / (k_avg * 1e-6) / 1e12, 2) if n_meas else None,
                       "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                       "frac": round(useful_attn / (k_avg * 1e-6) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4) if n_meas else None,
                       "executed_TFLOPs": round(executed / (k_avg * 1e-6) / 1e12, 2) if n_meas else None,
                       "traffic": None, "flops_per_launch": useful_attn, "avg_us": round(k_avg, 2),
                       "min_us": round(k_min, 2), "launches": n_meas}
    print(json.dumps(res, ensure_ascii=False))


def bench_hier(args, torch, sq, wl, dev):
    """Config 5: two-level lookup + sparse decode attention (sq_hier_decode_step)."""
    w = wl.make_config(args.workload, seed=args.seed, threads=16)
    wl.calibrate(w, gpu_score_fn(sq, torch, dev))
    NQ = args.queries
    P = sq.upload(w, dev)
    shape = P.shape
    qs = wl.extra_queries(w, NQ)
    Q = torch.from_numpy(np.ascontiguousarray(qs[:, None, :, None, :])).to(dev)      # [NQ,1,H,1,d]
    out = torch.zeros(NQ, 1, w.H, 1, w.d, dtype=torch.float16, device=dev)
    lse = torch.zeros(NQ, 1, w.H, 1, dtype=torch.float32, device=dev)
    nkeys = torch.zeros(NQ, 1, w.H, 1, dtype=torch.int32, device=dev)
    ws = sq.workspace(shape, sq.SQ_CALL_HIER_DECODE_STEP, dev)

    def step(i, stream_ptr):
        qi = i % NQ
        sq.sq_hier_decode_step(shape, w.C1, Q[qi], P.centroids1, P.sizes1, P.child_offsets, P.thresh1, P.centroids,
                               P.sizes, P.offsets, P.thresh2, P.K_fixed, P.V_fixed, P.K_user, P.V_user, out[qi],
                               lse[qi], None, nkeys[qi], ws)

    eager_ms, graph_ms, ms, (n_meas, k_avg, k_min, k_max) = time_steps(step, args, torch, sq)
    # candidates per query (for the byte count): one untimed sq_hier_select per query
    m1 = torch.zeros(1, w.H, (w.C1 + 31) // 32, dtype=torch.int32, device=dev)
    m2 = torch.zeros(1, w.H, (w.C + 31) // 32, dtype=torch.int32, device=dev)
    nr = torch.zeros(1, w.H, 1, dtype=torch.int32, device=dev)
    nk1 = torch.zeros(1, w.H, 1, dtype=torch.int32, device=dev)
    ws_h = sq.workspace(shape, sq.SQ_CALL_HIER_SELECT, dev)
    used = sorted({(args.warmup + i) % NQ for i in range(args.steps)})
    fan = np.diff(w.child_offsets, axis=1)
    ncand = {}
    for qi in used:
        sq.sq_hier_select(shape, w.C1, Q[qi], P.centroids1, P.sizes1, P.child_offsets, P.thresh1, P.centroids,
                          P.sizes, P.offsets, P.thresh2, m1, m2, None, nr, nk1, ws_h)
        bits = m1.cpu().numpy().view(np.uint32)[0]
        keep1 = ((bits[:, :, None] >> np.arange(32, dtype=np.uint32)) & 1).reshape(w.H, -1)[:, :w.C1].astype(bool)
        ncand[qi] = int((keep1 * fan).sum())
    nk = nkeys.cpu().numpy()[:, 0, :, 0]
    steps_q = [(args.warmup + i) % NQ for i in range(args.steps)]
    sel = float(np.mean([nk[qi].sum() for qi in steps_q])) * w.d * 4
    cand = float(np.mean([ncand[qi] for qi in steps_q])) * w.d * 2
    coarse = w.H * w.C1 * w.d * 2
    dense = w.H * w.U * w.d * 4
    tot = sel + cand + coarse + dense
    # (the user keys are attended to by extra workgroups of the partial kernel's launch)
    kernel_bytes = sel + dense + w.H * w.d * 2
    res = base_result(args, f"hierarchical decode attn µs/token + achieved HBM GB/s, {w.L // 1024}K fixed ctx, "
                      f"keep {w.keep_frac:.4g}",
                      round(tot / (ms * 1e-3) / 1e9, 2), "GB/s", ms, eager_ms, graph_ms, 1)
    res["config"] = {"workload": args.workload, "H": w.H, "d": w.d, "L": w.L, "C1": w.C1, "C2": w.C, "U": w.U,
                     "fanout_min_max": [int(fan.min()), int(fan.max())],
                     "candidate_fine_fraction": round(float(np.mean([ncand[qi] for qi in steps_q]) / w.H / w.C), 4),
                     "keep_achieved": round(float(np.mean([nk[qi].mean() for qi in steps_q]) / w.L), 5),
                     "queries": NQ, "entry": "sq_hier_decode_step"}
    res["bytes_per_step"] = {"total": round(tot), "coarse_centroids": coarse, "candidate_fine_centroids": round(cand),
                             "selected_kv": round(sel), "dense_kv": dense}
    res["hbm_frac_whole_step"] = round(tot / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)
    res["roofline"] = {"bound": "hbm", "kernel": "decode_attn_index_kernel",
                       "achieved": round(kernel_bytes / (k_avg * 1e-6) / 1e9, 2) if n_meas else None,
                       "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                       "frac": round(kernel_bytes / (k_avg * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4) if n_meas else None,
                       **read_traffic(f"decode_attn_index_kernel_{args.workload}_pmc.txt"),
                       "bytes_per_launch": round(kernel_bytes), "avg_us": round(k_avg, 3), "min_us": round(k_min, 3),
                       "launches": n_meas}
    res["roofline"].update(stream_ceiling(sq, torch, dev, kernel_bytes))
    res["lookup_us"] = hier_lookup_times(args, torch, sq, w, P, shape, Q, dev)
    print(json.dumps(res, ensure_ascii=False))


def hier_lookup_times(args, torch, sq, w, P, shape, Q, dev, reps=100):
    """The centroid lookup alone (no attention), as the paper compares it (appendix "Hierarchical kernel benchmarking"):
    the two-level lookup (sq_hier_select: level-1 scores + selection, level-2 scores + selection over the children of
    the kept coarse clusters) against the one-level lookup over ALL fine centroids (sq_centroid_score + sq_select),
    each as one HIP-graph replay of `reps` lookups on different query tokens."""
    NQ = Q.shape[0]
    i32 = lambda *s: torch.zeros(s, dtype=torch.int32, device=dev)
    m1, m2 = i32(1, w.H, (w.C1 + 31) // 32), i32(1, w.H, (w.C + 31) // 32)
    nr, nk = i32(1, w.H, 1), i32(1, w.H, 1)
    ws_h = sq.workspace(shape, sq.SQ_CALL_HIER_SELECT, dev)
    logits = torch.empty(1, w.H, 1, w.C, dtype=torch.float32, device=dev)
    rmax = torch.empty(1, w.H, 1, dtype=torch.float32, device=dev)
    den = torch.empty_like(rmax)

    def two_level(i):
        sq.sq_hier_select(shape, w.C1, Q[i % NQ], P.centroids1, P.sizes1, P.child_offsets, P.thresh1, P.centroids, P.sizes,
                          P.offsets, P.thresh2, m1, m2, None, nr, nk, ws_h)

    def one_level(i):
        sq.sq_centroid_score(shape, Q[i % NQ], P.centroids, P.sizes, logits, rmax, den)
        sq.sq_select(shape, logits, rmax, den, P.thresh2, P.sizes, P.offsets, m2, None, nr, nk)

    out = {}
    for name, fn in (("two_level", two_level), ("one_level_all_fine_centroids", one_level)):
        for i in range(5):
            fn(i)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(reps):
                fn(i)
        g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        g.replay()
        torch.cuda.synchronize()
        out[name] = round((time.perf_counter() - t0) / reps * 1e6, 2)
    out["two_level_over_one_level"] = round(out["two_level"] / out["one_level_all_fine_centroids"], 3)
    return out


def bench_gqa(args, torch, sq, wl, dev):
    """Grouped-query decode (sq_gqa_decode_step): G query heads per K/V head select independently; one step = one
    token; the union of a group's selections is streamed once."""
    w = wl.make_config(args.workload, seed=args.seed, threads=16)
    wl.calibrate(w, gpu_score_fn(sq, torch, dev))
    G, NQ, R = w.Lq, args.queries, args.replicas
    Hq, W = w.H * G, (w.C + 31) // 32
    tt = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    rep = lambda a: [tt(a) for _ in range(R)]
    Kf, Vf, Ce, Ku, Vu = rep(w.K_fixed), rep(w.V_fixed), rep(w.centroids), rep(w.K_user), rep(w.V_user)
    sizes, offsets, thresh = tt(w.sizes), tt(w.offsets), tt(w.thresh)
    qs = wl.extra_queries(w, NQ + G - 1)                                            # [n, H, d]
    # token i: query head h*G + g of K/V head h is query i + g of that head's stream
    Q = torch.stack([tt(np.ascontiguousarray(qs[i:i + G].transpose(1, 0, 2).reshape(1, Hq, 1, w.d))) for i in range(NQ)])
    out = torch.zeros(NQ, w.B, Hq, 1, w.d, dtype=torch.float16, device=dev)
    lse = torch.zeros(NQ, w.B, Hq, 1, dtype=torch.float32, device=dev)
    nkeys = torch.zeros(NQ, w.B, Hq, 1, dtype=torch.int32, device=dev)
    kmask = torch.zeros(NQ, w.B, Hq, 1, W, dtype=torch.int32, device=dev)
    shape = sq.make_shape(w.B, w.H, w.L, w.C, 1, w.U, w.sm_scale)
    ws = sq.workspace(shape, sq.SQ_CALL_GQA_DECODE_STEP, dev)

    mean = args.selection == "mean"          # one kept set per K/V head from the group's averaged scores
    entry = sq.sq_gqa_mean_decode_step if mean else sq.sq_gqa_decode_step
    if mean:
        ws = sq.workspace(shape, sq.SQ_CALL_GQA_MEAN_DECODE_STEP, dev)

    def step(i, stream_ptr):
        qi, r = i % NQ, i % R
        entry(shape, G, Q[qi], Ce[r], sizes, offsets, thresh, Kf[r], Vf[r], Ku[r], Vu[r], out[qi], lse[qi], kmask[qi],
              nkeys[qi], ws)

    eager_ms, graph_ms, ms, (n_meas, k_avg, k_min, k_max) = time_steps(step, args, torch, sq)
    used = [(args.warmup + i) % NQ for i in range(args.steps)]
    nk = nkeys.cpu().numpy()[:, 0, :, 0]                                            # [NQ, Hq]
    km = kmask.cpu().numpy()[:, 0, :, 0, :].view(np.uint32).reshape(NQ, w.H, G, W)
    union = np.bitwise_or.reduce(km, axis=2)                                        # [NQ, H, W]
    bits = ((union[..., None] >> np.arange(32, dtype=np.uint32)) & 1).reshape(NQ, w.H, -1)[:, :, :w.C]
    uniq = (bits * w.sizes[None]).sum(axis=(1, 2))                                  # keys of the union, per token
    sel = float(np.mean([uniq[qi] for qi in used])) * w.d * 4                       # K + V rows, read once
    sel_req = float(np.mean([nk[qi].sum() for qi in used])) * w.d * 4
    cen = w.H * w.C * w.d * 2
    dense = w.B * w.H * w.U * w.d * 4
    meta = w.H * (2 * w.C + 1) * 4
    tot = sel + cen + dense + meta + 2 * w.B * Hq * w.d * 2      # what the method has to move: every needed byte once
    # The library streams the union once from 8 (sequence, query head) pairs per K/V head on; with fewer, its
    # per-row kernels read a K/V head's selected keys and user keys once per query head.
    shared = mean or w.B * G >= 8
    kernel = "decode_attn_shared_kernel" if shared else "decode_attn_index_kernel"
    # (per-row kernels: every query head reads its own selection and, in extra workgroups of the same launch, the
    # sequence's user keys)
    kernel_bytes = (sel + dense if shared else sel_req + dense * G) + w.B * Hq * w.d * 2
    res = base_result(args, "grouped-query decode attn µs/token + achieved HBM GB/s, 32K fixed ctx, keep 1/8, "
                      "32 query heads over 8 K/V heads, d=128", round(tot / (ms * 1e-3) / 1e9, 2), "GB/s", ms, eager_ms,
                      graph_ms, w.B)
    res["config"] = {"workload": args.workload, "B": w.B, "H_kv": w.H, "G": G, "d": w.d, "L": w.L, "C": w.C, "U": w.U,
                     "keep_target": w.keep_frac, "keep_achieved": round(float(np.mean([nk[qi].mean() for qi in used])) / w.L, 5),
                     "queries": NQ, "replicas": R, "selection": args.selection,
                     "entry": "sq_gqa_mean_decode_step" if mean else "sq_gqa_decode_step"}
    res["bytes_per_step"] = {"total": round(tot), "centroid": cen, "selected_kv": round(sel),
                             "selected_kv_requested": round(sel_req), "dense_kv": dense}
    res["hbm_frac_whole_step"] = round(tot / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)
    res["roofline"] = {"bound": "hbm", "kernel": kernel,
                       "achieved": round(kernel_bytes / (k_avg * 1e-6) / 1e9, 2) if n_meas else None,
                       "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                       "frac": round(kernel_bytes / (k_avg * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4) if n_meas else None,
                       **read_traffic(f"{kernel}_{args.workload}_pmc.txt"),
                       "bytes_per_launch": round(kernel_bytes), "avg_us": round(k_avg, 3), "min_us": round(k_min, 3),
                       "launches": n_meas}
    res["roofline"].update(stream_ceiling(sq, torch, dev, kernel_bytes))
    print(json.dumps(res, ensure_ascii=False))


MFMA_F16_PEAK_TFLOPS = 2500.0


def bench_kmeans(args, torch, sq, wl, dev):
    """Offline clustering (sq_kmeans_step): one step = one Lloyd iteration over every head of the fixed context --
    assignment (the MFMA kernel, 2*L*C*d flops per head), stable grouping by centre, member means."""
    cfg = wl.KMEANS_CONFIGS[args.workload]
    H, L, Cn, d = cfg["H"], cfg["L"], cfg["C"], 128
    K, _, init = wl.clustering_input(args.seed, H, L, Cn)
    shape = sq.make_shape(1, H, L, Cn, 1, 0, 1.0)
    Kg = torch.from_numpy(K).to(dev)
    X = torch.empty_like(Kg)
    sq.sq_kmeans_normalize(shape, Kg, X)
    idx = torch.from_numpy(init).to(dev).long()
    cent = [torch.stack([X[h][idx[h]] for h in range(H)]).contiguous(), None]
    cent[1] = torch.empty_like(cent[0])
    i32 = lambda *s: torch.empty(s, dtype=torch.int32, device=dev)
    assign, sizes, offsets, perm = i32(H, L), i32(H, Cn), i32(H, Cn + 1), i32(H, L)
    ws = sq.workspace(shape, sq.SQ_CALL_KMEANS_STEP, dev)

    def step(i, stream_ptr):                         # centres ping-pong: iteration i reads what i-1 wrote
        sq.sq_kmeans_step(shape, X, cent[i & 1], cent[(i + 1) & 1], assign, sizes, offsets, perm, ws)

    eager_ms, graph_ms, ms, (n_meas, k_avg, k_min, k_max) = time_steps(step, args, torch, sq)
    flops = 2.0 * H * L * Cn * d
    res = base_result(args, "K-means on normalised keys: Lloyd iterations/s over 32 heads x 32K keys x 1024 centres, "
                      "d=128", round(1e3 / ms, 2), "iterations/s", ms, eager_ms, graph_ms, 1)
    del res["us_per_token"]
    res["config"] = {"workload": args.workload, "H": H, "L": L, "C": Cn, "d": d, "entry": "sq_kmeans_step",
                     "largest_cluster": int(sizes.max()), "empty_clusters": int((sizes == 0).sum())}
    res["roofline"] = {"bound": "mfma", "kernel": "kmeans_assign_kernel",
                       "achieved": round(flops / (k_avg * 1e-6) / 1e12, 2) if n_meas else None,
                       "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                       "frac": round(flops / (k_avg * 1e-6) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4) if n_meas else None,
                       "traffic": None, "flops_per_launch": flops, "avg_us": round(k_avg, 3),
                       "min_us": round(k_min, 3), "launches": n_meas}
    if args.cpu_seconds > 0:
        from oracle import clustering as ocl
        Xn, c0 = X.cpu().numpy(), cent[0].cpu().numpy()
        n, t_total = 0, 0.0
        while n < H and t_total < args.cpu_seconds:
            t0 = time.perf_counter()
            ocl.lloyd_step(Xn[n], c0[n])
            t_total += time.perf_counter() - t0
            n += 1
        import os
        res["cpu_baseline"] = dict(value=round(n / t_total / H, 4), unit="iterations/s", cores=os.cpu_count(),
                                   kind="oracle", sample=f"one Lloyd iteration on {n} of the {H} heads, scaled to all heads")
    print(json.dumps(res, ensure_ascii=False))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="cfg2_decode_32k")
    ap.add_argument("--queries", type=int, default=100)
    ap.add_argument("--replicas", type=int, default=8)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget of the CPU-oracle baseline (0 = skip)")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay measurement")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="only run a 256 MiB streaming read and a 256 MiB device copy (known sizes) a few times: "
                         "the reference dispatches that scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings")
    ap.add_argument("--selection", choices=("per_query", "mean"), default="per_query",
                    help="prefill workloads: per-query selection, or the paper's selection on averaged scores")
    ap.add_argument("--separate", action="store_true", help="time the three separate calls instead of sq_decode_step")
    ap.add_argument("--global-threshold", action="store_true",
                    help="decode workloads: heads of different score skewness under ONE threshold for all heads "
                         "(Section 3.2), so that the heads keep very different numbers of keys")
    args = ap.parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU only (no sharding, no collectives); --gpus {args.gpus} is not "
              "supported. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2411_09688_amd import binding as sq, workload as wl
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    sq.lib()
    if args.pmc_calibration:
        src = torch.ones(1 << 28, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        sink = torch.zeros(1024, dtype=torch.int32, device=dev)
        for _ in range(5):
            sq.sq_probe_stream_read(src, sink, 512)
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"pmc_calibration": {"stream_read_bytes": 1 << 28, "copy_bytes_each_way": 1 << 28}}))
        return

    if args.workload in wl.GQA_CONFIGS:
        return bench_gqa(args, torch, sq, wl, dev)
    if args.workload in wl.KMEANS_CONFIGS:
        return bench_kmeans(args, torch, sq, wl, dev)
    cfg = wl.CONFIGS[args.workload] if args.workload in wl.CONFIGS else wl.HIER_SIZING_CONFIGS[args.workload]
    if cfg.get("Lq", 1) > 1:
        return bench_prefill(args, torch, sq, wl, dev)
    if cfg.get("C1", 0):
        return bench_hier(args, torch, sq, wl, dev)
    w = wl.make_config(args.workload, seed=args.seed, threads=16, **({"head_skew": 0.4} if args.global_threshold else {}))
    wl.calibrate(w, gpu_score_fn(sq, torch, dev), global_threshold=args.global_threshold)
    NQ, R = args.queries, args.replicas
    tt = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    rep = lambda a: [tt(a) for _ in range(R)]
    Kf, Vf, Ce, Ku, Vu = rep(w.K_fixed), rep(w.V_fixed), rep(w.centroids), rep(w.K_user), rep(w.V_user)
    sizes, offsets, thresh = tt(w.sizes), tt(w.offsets), tt(w.thresh)
    # queries: NQ tokens; every sequence of a batched workload gets its own rotation of them
    qs = wl.extra_queries(w, NQ + w.B - 1)
    Q = torch.stack([tt(np.ascontiguousarray(qs[i:i + w.B][:, :, None, :])) for i in range(NQ)])  # [NQ,B,H,1,d]
    out = torch.zeros(NQ, w.B, w.H, 1, w.d, dtype=torch.float16, device=dev)
    lse = torch.zeros(NQ, w.B, w.H, 1, dtype=torch.float32, device=dev)
    nkeys = torch.zeros(NQ, w.B, w.H, 1, dtype=torch.int32, device=dev)
    # keep-masks are only requested for a batch: they give the union of the sequences' selections
    kmask = torch.zeros(NQ, w.B, w.H, 1, (w.C + 31) // 32, dtype=torch.int32, device=dev) if w.B > 1 else None
    shape = sq.make_shape(w.B, w.H, w.L, w.C, 1, w.U, w.sm_scale)
    ws = sq.workspace(shape, sq.SQ_CALL_DECODE_STEP, dev)
    if args.separate:
        logits = torch.empty(w.B, w.H, 1, w.C, dtype=torch.float32, device=dev)
        rmax = torch.empty(w.B, w.H, 1, dtype=torch.float32, device=dev)
        den = torch.empty_like(rmax)
        mask = torch.zeros(w.B, w.H, 1, (w.C + 31) // 32, dtype=torch.int32, device=dev)
        ranges = torch.zeros(w.B, w.H, 1, w.C, 2, dtype=torch.int32, device=dev)
        nr = torch.zeros(w.B, w.H, 1, dtype=torch.int32, device=dev)
        ws_a = sq.workspace(shape, sq.SQ_CALL_ATTN_DECODE, dev)

    # Arguments are marshalled once per (query, replica) pair; a step is then one ctypes call.
    import ctypes as C
    L_ = sq.lib()
    sp = C.byref(shape)
    P = lambda t: C.c_void_p(t.data_ptr()) if t is not None else None
    wsp = lambda t: (C.c_void_p(t.data_ptr()), t.numel())
    cycle = int(np.lcm(NQ, R))
    calls = []
    for i in range(cycle):
        qi, r = i % NQ, i % R
        if args.separate:
            calls.append((
                (sp, P(Q[qi]), P(Ce[r]), P(sizes), P(logits), P(rmax), P(den), None, 0),
                (sp, P(logits), P(rmax), P(den), P(thresh), P(sizes), P(offsets), P(mask), P(ranges), P(nr),
                 P(nkeys[qi]), None, 0),
                (sp, P(Q[qi]), P(Kf[r]), P(Vf[r]), P(ranges), P(nr), P(nkeys[qi]), P(Ku[r]), P(Vu[r]), P(out[qi]),
                 P(lse[qi]), *wsp(ws_a))))
        else:
            calls.append((sp, P(Q[qi]), P(Ce[r]), P(sizes), P(offsets), P(thresh), P(Kf[r]), P(Vf[r]), P(Ku[r]),
                          P(Vu[r]), P(out[qi]), P(lse[qi]), P(kmask[qi]) if kmask is not None else None,
                          P(nkeys[qi]), *wsp(ws)))

    def step(i, stream_ptr):
        a = calls[i % cycle]
        if args.separate:
            rc = (L_.sq_centroid_score(*a[0], stream_ptr) or L_.sq_select(*a[1], stream_ptr)
                  or L_.sq_sparse_attn_decode(*a[2], stream_ptr))
        else:
            rc = L_.sq_decode_step(*a, stream_ptr)
        if rc:
            raise sq.SqError(rc, L_.sq_last_error().decode())

    eager_ms, graph_ms, ms_per_step, (n_meas, k_avg_us, k_min_us, k_max_us) = time_steps(step, args, torch, sq)

    nk = nkeys.cpu().numpy()[:, :, :, 0]                       # [NQ, B, H]
    used = [(args.warmup + i) % NQ for i in range(args.steps)]
    per_step = [step_bytes(w, nk[qi]) for qi in used]
    tot = float(np.mean([b["total"] for b in per_step]))
    sel = float(np.mean([b["selected_kv"] for b in per_step]))
    cen = float(per_step[0]["centroid"])
    dense = float(per_step[0]["dense_kv"])
    sel_requested = sel
    if kmask is not None and not args.separate:
        # The sequences of a batch share the fixed context: a key kept by several of them has to leave HBM
        # once.  Unique selected bytes = keys of the union of the sequences' kept clusters, per head.
        km = kmask.cpu().numpy()[:, :, :, 0, :].view(np.uint32)                      # [NQ, B, H, W]
        union = np.bitwise_or.reduce(km, axis=1)                                        # [NQ, H, W]
        bits = ((union[..., None] >> np.arange(32, dtype=np.uint32)) & 1).reshape(NQ, w.H, -1)[:, :, :w.C]
        uniq_keys = (bits * w.sizes[None]).sum(axis=(1, 2))                            # [NQ]
        sel = float(np.mean([uniq_keys[qi] for qi in used])) * w.d * 2 * 2
        tot = tot - sel_requested + sel
    # K/V rows read by the launch of the partial kernel + q: the selected keys and the user keys (in the per-row step
    # the user keys are attended to by extra workgroups of the same launch).
    kernel_bytes = sel + dense + w.B * w.H * w.d * 2
    if w.B > 1 and not args.separate:
        dom_kernel = "decode_attn_shared_kernel"
    elif args.separate:
        dom_kernel = "decode_attn_kernel"
    else:
        dom_kernel = "decode_attn_index_kernel"
    keep = float(np.mean([nk[qi].mean() for qi in used]) / w.L)
    tokens = w.B

    res = {
        "metric": METRIC,
        "value": round(tot / (ms_per_step * 1e-3) / 1e9, 2),
        "unit": "GB/s",
        "us_per_token": round(ms_per_step * 1e3 / tokens, 3),
        "us_per_step_eager": round(eager_ms * 1e3, 3),
        "us_per_step_graph": None if graph_ms is None else round(graph_ms * 1e3, 3),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": args.workload, "B": w.B, "H": w.H, "d": w.d, "L": w.L, "C": w.C, "U": w.U,
                   "keep_target": w.keep_frac, "keep_achieved": round(keep, 5), "queries": NQ, "replicas": R,
                   "threshold": "one for all heads, head skew 0.4" if args.global_threshold else "per head",
                   "keep_per_head_min_max": [round(float(np.mean([nk[qi] for qi in used], axis=(0, 1)).min() / w.L), 4),
                                             round(float(np.mean([nk[qi] for qi in used], axis=(0, 1)).max() / w.L), 4)],
                   "entry": "3 calls" if args.separate else "sq_decode_step"},
        "bytes_per_step": {"total": round(tot), "centroid": round(cen), "selected_kv": round(sel),
                           "selected_kv_requested": round(sel_requested),
                           "dense_kv": round(dense), "centroid_plus_selected_kv": round(cen + sel)},
        "hbm_frac_whole_step": round(tot / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "roofline": {"bound": "hbm", "kernel": dom_kernel,
                     "achieved": round(kernel_bytes / (k_avg_us * 1e-6) / 1e9, 2) if n_meas else None,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(kernel_bytes / (k_avg_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4) if n_meas else None,
                     **read_traffic(f"{dom_kernel}_{args.workload}_pmc.txt"),
                     "bytes_per_launch": round(kernel_bytes), "avg_us": round(k_avg_us, 3),
                     "min_us": round(k_min_us, 3), "launches": n_meas},
    }
    res["roofline"].update(stream_ceiling(sq, torch, dev, kernel_bytes))
    if args.cpu_seconds > 0:
        res["cpu_baseline"] = cpu_baseline(args.workload, args.seed, args.cpu_seconds)
    print(json.dumps(res, ensure_ascii=False))


if __name__ == "__main__":
    main()
