#!/usr/bin/env python3
"""Benchmark of one DASGD worker step (tensair_step) on one MI355X.

A "step" is one pass of the whole hot path over one mini-batch: pair enumeration, negative
sampling, sort/segments, forward, segmented reductions (the own sparse gradient), then the
merged application of the own gradient and the K peer gradients that are resident in HBM.

Procedure
  1. the synthetic workload of the chosen configuration is generated (Zipf token stream);
  2. recording pass (untimed): warmup+steps worker steps are run while the K peer gradients of
     every step -- computed with tensair_sgns_grad on the peers' own mini-batches against model
     snapshots 0..max_stale steps old -- are stored compactly in HBM, and the algorithmic bytes
     of every step are counted from the row counts;
  3. the tables are reset to the initial model; warmup steps, then exactly `steps` calls of
     tensair_step back to back on the stored peers, bracketed by torch.cuda.synchronize() and a
     host clock; being deterministic, the replay computes exactly what the recording pass did;
  4. the library's HIP-event hook times the table-update kernel (the dominant one) inside that
     same timed region;
  5. the CPU oracle is timed on the host for a bounded sample (one step's own gradient + apply).

Prints one JSON line.  --dim, --table-dtype, --batch-centers, --peers and --vocab run a modified copy of the chosen
workload (named so in the line's config.workload): other shapes, not the workload the metric is quoted on.
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

HBM_PEAK = 8.0e12  # bytes/s, MI355X HBM3E


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default: 20 for workload 3; 100/50/10/6 for 1/2/4/5)")
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", type=int, default=3, help="workload 1..5 (3 = the 1M-vocab configuration the metric is quoted on)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prefetch", action="store_true",
                    help="every step self-contained (default: the next mini-batch is handed to tensair_prefetch "
                         "after each step, as it would be waiting in the worker's input queue)")
    ap.add_argument("--row-stride", type=int, default=None,
                    help="elements between table rows (default: the pitch that starts every row on a 128-byte "
                         "line, tensair_aligned_row_stride: 320 for dim 300 in fp32; pass the dim for dense rows)")
    ap.add_argument("--stochastic-rounding", action="store_true",
                    help="bf16 tables rounded stochastically by the table update (a variant; workload 5)")
    ap.add_argument("--resample-negatives", action="store_true",
                    help="negatives equal to the pair's center or context word drawn once more (a variant)")
    ap.add_argument("--breakdown", action="store_true", help="extra pass with an event after every stage (stderr)")
    ap.add_argument("--peer-payload", choices=["f32", "bf16"], default="f32",
                    help="f32: the peers' gradients as the paper sends them (the metric); bf16: as bfloat16 messages "
                         "(tensair_grad_pack / tensair_step_packed, a variant)")
    ap.add_argument("--dim", type=int, default=None, help="other shapes: the named workload with this D (a multiple of 4)")
    ap.add_argument("--table-dtype", choices=["f32", "bf16"], default=None, help="other shapes: element type of the tables")
    ap.add_argument("--batch-centers", type=int, default=None, help="other shapes: centers per mini-batch")
    ap.add_argument("--peers", type=int, default=None, help="other shapes: peer gradients per step (K)")
    ap.add_argument("--vocab", type=int, default=None, help="other shapes: vocabulary size V")
    ap.add_argument("--op", choices=["step", "grad_add", "dense_apply", "lookup", "cosine", "grad_pack"], default="step",
                    help="step: the worker step (the metric); the others time one of the further operations on its own")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build is the one-GPU worker step; there is no multi-GPU path (--gpus must be 1)")
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2211_10280_amd import binding as B
    import workload as W
    from paper_2211_10280_amd.trainer import DasgdWorker

    cfg = W.CONFIGS[args.config]
    if args.stochastic_rounding or args.resample_negatives:
        cfg = cfg.scaled(stochastic_rounding=args.stochastic_rounding, resample=args.resample_negatives)
    other = {k: v for k, v in (("dim", args.dim), ("dtype", args.table_dtype), ("batch", args.batch_centers),
                               ("peers", args.peers), ("vocab", args.vocab)) if v is not None}
    if other:   # not the workload the metric is quoted on: the name in the output line says so
        if args.peers == 0:
            other["max_stale"] = 0
        cfg = cfg.scaled(name=cfg.name + "+" + "+".join(f"{k}={v}" for k, v in other.items() if k != "max_stale"), **other)
    if args.steps is None:
        args.steps = {1: 100, 2: 50, 3: 20, 4: 10, 5: 6}[cfg.idx]   # bounded by the HBM the stored peers take
    if args.warmup is None:
        args.warmup = 2 if cfg.idx == 5 else 3
    K, Wm, S = cfg.peers, args.warmup, args.steps
    total = Wm + S
    t0 = time.perf_counter()
    tok, counts = W.make_stream(cfg)
    log(f"[bench] workload {cfg.name}: stream of {cfg.tokens} tokens in {time.perf_counter() - t0:.1f}s")

    if args.op == "grad_add":
        return bench_grad_add(args, cfg, tok, counts)
    if args.op != "step":
        return bench_streaming(args, cfg, tok, counts)

    worker = DasgdWorker(cfg, tok, counts, prefetch=not args.no_prefetch, row_stride=args.row_stride,
                         bf16_messages=args.peer_payload == "bf16")
    model = worker.model
    theta0 = (model.w_in.clone(), model.w_out.clone())
    D, e = cfg.dim, cfg.elem_bytes
    peer_elem = 2 if args.peer_payload == "bf16" else 4

    # ---- recording pass: peers of every step, algorithmic bytes
    stored, bytes_grad, bytes_apply, pairs = [], [], [], []
    for t in range(total):
        peers = worker.make_peer_grads(t) if K else []
        compact = []
        for pb in peers:
            ui, uo = pb.sizes()
            cb = type(pb)(ui, uo, D)
            cb.in_ids[:ui].copy_(pb.in_ids[:ui]); cb.in_rows[:ui].copy_(pb.in_rows[:ui])
            cb.out_ids[:uo].copy_(pb.out_ids[:uo]); cb.out_rows[:uo].copy_(pb.out_rows[:uo])
            cb.n_rows.copy_(pb.n_rows)
            compact.append(cb)
        begin, n, epoch = worker.step(peers=compact)
        stored.append(compact)
        ui, uo = worker.own.sizes()
        srcs_in = [worker.own.in_ids[:ui]] + [c.in_ids[: c.cap_in] for c in compact]
        srcs_out = [worker.own.out_ids[:uo]] + [c.out_ids[: c.cap_out] for c in compact]
        r_in = int(torch.unique(torch.cat(srcs_in)).numel())
        r_out = int(torch.unique(torch.cat(srcs_out)).numel())
        rows_peers = sum(int(x.numel()) for x in srcs_in[1:]) + sum(int(x.numel()) for x in srcs_out[1:])
        bytes_grad.append((ui + uo) * D * e + (ui + uo) * D * 4)
        # with bfloat16 messages the update also writes the own gradient out as the message this worker sends
        msg_out = (ui + uo) * D * 2 if peer_elem == 2 else 0
        bytes_apply.append((ui + uo) * D * 4 + rows_peers * D * peer_elem + 2 * (r_in + r_out) * D * e + msg_out)
        pairs.append(model.pair_count(cfg.tokens, begin, n))
    model.status()
    torch.cuda.synchronize()
    log(f"[bench] recorded {total} steps; step {total - 1}: U_in={ui} U_out={uo} R_in={r_in} R_out={r_out} "
        f"grad {bytes_grad[-1] / 1e6:.1f} MB apply {bytes_apply[-1] / 1e6:.1f} MB")

    def reset():
        model.w_in.copy_(theta0[0]); model.w_out.copy_(theta0[1])
        worker.restart()

    # ---- replay: warmup, then the timed region
    reset()
    for t in range(Wm):
        worker.step(peers=stored[t])
    B.tensair_profile(model.h, 1)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for t in range(Wm, total):
        worker.step(peers=stored[t])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    recs = B.tensair_profile_read(model.h)
    B.tensair_profile(model.h, 0)
    model.status()
    apply_ms = [ms for tag, ms in recs if tag == "apply_update"]   # one launch of k_apply per step
    assert len(apply_ms) == S, (len(apply_ms), S)
    n_launch = len(apply_ms)

    # ---- streaming ceilings of this machine: 1 GiB per stream; plain copy (also the calibration of the HBM byte
    #      counters), copy around the caches, read only, and three reads per write (the read share of k_apply)
    copy_GBps, ceilings = streaming_ceilings(B, torch)

    n_pairs = sum(pairs[Wm:])
    value = n_pairs / elapsed
    ms_per_step = elapsed / S * 1e3
    step_bytes = sum(bytes_grad[Wm:]) + sum(bytes_apply[Wm:])
    apply_bytes_per_launch = sum(bytes_apply[Wm:]) / n_launch
    apply_avg_s = (sum(apply_ms) / n_launch) * 1e-3
    achieved = apply_bytes_per_launch / apply_avg_s

    # HBM traffic of the dominant kernel: not measured by this run (that takes hardware counters, i.e. rocprofv3
    # around the whole process) but read from the stored summary of such runs on this workload, and said so
    traffic = traffic_source = trace_avg_ms = None
    tname = f"traffic_{cfg.name.replace('+', '_').replace('=', '')}{'_bf16_messages' if peer_elem == 2 else ''}.json"
    tpath = os.path.join(ROOT, "profiles", tname)
    if os.path.exists(tpath):
        try:
            stored = json.load(open(tpath))
            traffic = stored.get("k_apply_hbm_bytes_per_step") / (n_launch // S)
            traffic_source = f"stored: profiles/{tname} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run, not of this one)"
            if stored.get("k_apply_kernel_trace_avg_us"):
                trace_avg_ms = stored["k_apply_kernel_trace_avg_us"] * 1e-3
        except Exception:
            traffic = None

    breakdown = None
    if args.breakdown:
        reset()
        B.tensair_profile(model.h, 2)
        for t in range(total):
            worker.step(peers=stored[t])
            if t == Wm - 1:
                B.tensair_profile_read(model.h)
        torch.cuda.synchronize()
        recs = B.tensair_profile_read(model.h)
        B.tensair_profile(model.h, 0)
        agg = {}
        for tag, ms in recs:
            agg[tag] = agg.get(tag, 0.0) + ms
        breakdown = {k: round(v / S, 4) for k, v in agg.items()}
        log("[bench] per-stage ms/step (events after every stage):", json.dumps(breakdown))

    out = {
        "metric": "training pairs/s per MI355X incl. DASGD apply; % of HBM roofline",
        "value": value,
        "unit": "pairs/s",
        "n_gpus": 1,
        "steps": S,
        "warmup": Wm,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": ("f32" if cfg.dtype == "f32" else "bf16 tables, f32 accumulation") +
                 (", peer gradients as bf16 messages" if peer_elem == 2 else ""),
        "data": "synthetic",
        "config": {"workload": cfg.name, "vocab": cfg.vocab, "dim": cfg.dim, "window": cfg.window,
                   "negatives": cfg.negatives, "batch_centers": cfg.batch, "peers": K,
                   "max_stale": cfg.max_stale, "zipf_s": cfg.zipf_s, "pairs_per_step": n_pairs / S,
                   "next_batch_prefetch": not args.no_prefetch,
                   "row_stride": model.cfg.row_stride, "peer_payload": args.peer_payload,
                   "stochastic_rounding": cfg.stochastic_rounding, "resampled_negatives": cfg.resample},
        "step_hbm_frac": step_bytes / elapsed / HBM_PEAK,
        "measured_copy_GBps": copy_GBps,
        "measured_streaming_GBps": ceilings,
        "step_algorithmic_bytes": step_bytes / S,
        "roofline": {"bound": "hbm", "kernel": "k_apply", "achieved": achieved / 1e9, "peak": HBM_PEAK / 1e9,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK, "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes_per_launch": apply_bytes_per_launch,
                     "avg_launch_ms": apply_avg_s * 1e3, "launches_per_step": n_launch // S,
                     # the same kernel's average in the stored rocprofv3 kernel trace (timed launches), for comparison
                     "stored_kernel_trace_avg_launch_ms": trace_avg_ms},
    }
    if breakdown:
        out["stage_ms_per_step"] = breakdown

    # ---- CPU baseline: the oracle as it stands, one core, a bounded sample of the same workload
    if not args.no_cpu_baseline:
        del stored, worker, theta0
        torch.cuda.empty_cache()
        from oracle.driver import OracleWorker

        t0 = time.perf_counter()
        ow = OracleWorker(cfg, tok, counts, threads=1, bf16_messages=peer_elem == 2)
        n_cpu = {1: 157, 2: 12, 3: 4, 4: 1, 5: 1}[cfg.idx]
        cpu_t, p_cpu = 0.0, 0
        for t in range(n_cpu):
            ow.step()
            cpu_t += ow.t_own + ow.t_apply
            p_cpu += W.pairs_in_batch(cfg, *W.worker_batch(cfg, t, 0)[:2])
        log(f"[bench] oracle: {n_cpu} steps, own gradient + merged apply {cpu_t:.2f}s "
            f"(whole leg incl. init and peer gradients {time.perf_counter() - t0:.1f}s)")
        out["cpu_baseline"] = {"value": p_cpu / cpu_t, "unit": "pairs/s", "cores": 1, "kind": "oracle",
                               "sample": f"steps 0..{n_cpu - 1} of {cfg.name}: own gradient + merged apply of own and "
                                         f"{K} peer gradients ({p_cpu} pairs, {cpu_t:.1f} s); peer gradient synthesis "
                                         f"untimed, as on the GPU",
                               "host_cpus": os.cpu_count()}
    print(json.dumps(out), flush=True)


def streaming_ceilings(B, torch, reps=10):
    """(plain copy GB/s, {mix: GB/s}) of the library's streaming probes over 1 GiB per stream."""
    nbytes = 1 << 30
    src = torch.empty(3 * nbytes, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    moved = {0: 2 * nbytes, 1: 2 * nbytes, 2: nbytes, 3: 4 * nbytes}
    names = {0: "copy", 1: "copy_nontemporal", 2: "read_only", 3: "read3_write1"}
    out = {}
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for mode in (0, 1, 2, 3):
        for _ in range(3):
            B.tensair_stream_probe(dst, src, nbytes, mode)
        ev0.record()
        for _ in range(reps):
            B.tensair_stream_probe(dst, src, nbytes, mode)
        ev1.record()
        torch.cuda.synchronize()
        out[names[mode]] = round(moved[mode] * reps / (ev0.elapsed_time(ev1) * 1e-3) / 1e9, 1)
    del src, dst
    return out["copy"], out


def bench_grad_add(args, cfg, tok, counts):
    """gradients += gradient on two consecutive own gradients of the workload (first sum of a window)."""
    import numpy as np
    import torch

    from paper_2211_10280_amd import binding as B
    import workload as W

    dt = B.F32 if cfg.dtype == "f32" else B.BF16
    m = B.Model(cfg.vocab, cfg.dim, dt, cfg.window, cfg.negatives, cfg.batch, max(cfg.peers, 1), cfg.seed, counts)
    dtok = torch.from_numpy(np.ascontiguousarray(tok, dtype=np.int32)).cuda()
    # W_out away from zero so that both sides carry non-trivial rows (values do not change the traffic)
    m.w_out.copy_(m.w_in)
    g1, g2 = m.grad_buffers(), m.grad_buffers()
    b1, b2 = W.worker_batch(cfg, 0, 0), W.worker_batch(cfg, 1, 0)
    m.sgns_grad(dtok, b1[0], b1[1], b1[2], g1)
    m.sgns_grad(dtok, b2[0], b2[1], b2[2], g2)
    out = B.GradBuffers(min(cfg.vocab, 2 * g1.cap_in), min(cfg.vocab, 2 * g1.cap_out), cfg.dim)
    S = args.steps if args.steps else 50
    Wm = args.warmup if args.warmup is not None else 5
    for _ in range(Wm):
        m.grad_add(g1, g2, out)
    B.tensair_profile(m.h, 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(S):
        m.grad_add(g1, g2, out)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    recs = B.tensair_profile_read(m.h)
    B.tensair_profile(m.h, 0)
    m.status()
    rows_ms = [ms for tag, ms in recs if tag == "add_rows"]
    assert len(rows_ms) == S
    # the plain copy kernel of known size, for the calibration of the HBM byte counters
    nbytes = 1 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    for _ in range(3):
        B.tensair_copy_probe(dst, src, nbytes)
    torch.cuda.synchronize()
    del src, dst
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{cfg.name}_grad_add.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get("k_grad_sum_hbm_bytes_per_launch")
        except Exception:
            traffic = None
    (ua_in, ua_out), (ub_in, ub_out), (uo_in, uo_out) = g1.sizes(), g2.sizes(), out.sizes()
    D = cfg.dim
    # algorithmic bytes of one sum: read both gradients' rows, write the union's rows, ids read and written
    bytes_rows = (ua_in + ua_out + ub_in + ub_out + uo_in + uo_out) * D * 4
    bytes_ids = (ua_in + ua_out + ub_in + ub_out + uo_in + uo_out) * 4
    alg = bytes_rows + bytes_ids
    k_s = sum(rows_ms) / S * 1e-3
    out_json = {
        "metric": "gradient buffer accumulation (gradients += gradient): rows of the sum per second",
        "value": (uo_in + uo_out) / (elapsed / S), "unit": "rows/s", "n_gpus": 1, "steps": S, "warmup": Wm,
        "ms_per_step": elapsed / S * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg.name + ":grad_add", "rows_a": ua_in + ua_out, "rows_b": ub_in + ub_out,
                   "rows_sum": uo_in + uo_out, "dim": D},
        "roofline": {"bound": "hbm", "kernel": "k_grad_sum", "achieved": bytes_rows / k_s / 1e9,
                     "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": bytes_rows / k_s / HBM_PEAK, "traffic": traffic,
                     "algorithmic_bytes_per_launch": bytes_rows, "avg_launch_ms": k_s * 1e3,
                     "whole_call_algorithmic_bytes": alg, "whole_call_frac": alg / (elapsed / S) / HBM_PEAK},
    }
    if not args.no_cpu_baseline:
        import oracle

        (i1, r1), (o1, q1) = g1.to_host()
        (i2, r2), (o2, q2) = g2.to_host()
        t0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t0 < 10.0:
            oracle.grad_add_rows((i1, r1), (i2, r2), D)
            oracle.grad_add_rows((o1, q1), (o2, q2), D)
            reps += 1
        cpu_t = (time.perf_counter() - t0) / reps
        out_json["cpu_baseline"] = {"value": (uo_in + uo_out) / cpu_t, "unit": "rows/s", "cores": 1, "kind": "oracle",
                                    "sample": f"{reps} sums of the same two gradients ({cpu_t:.3f} s each)"}
    print(json.dumps(out_json), flush=True)


def bench_streaming(args, cfg, tok, counts):
    """dense_apply: theta of V*D elements, K+1 gradient blocks; lookup: 1 M random words; cosine: two tables;
    grad_pack: the gradient of the workload's first mini-batch into a bfloat16 message."""
    import numpy as np
    import torch

    import oracle
    from paper_2211_10280_amd import binding as B

    V, D, e = cfg.vocab, cfg.dim, cfg.elem_bytes
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    odt = oracle.F32 if cfg.dtype == "f32" else oracle.BF16
    S = args.steps if args.steps else 20
    Wm = args.warmup if args.warmup is not None else 3
    gen = torch.Generator(device="cuda").manual_seed(cfg.seed)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def to_np(t):
        return t.view(torch.int16).cpu().numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.cpu().numpy()

    if args.op == "dense_apply":
        n, K1 = V * D, cfg.peers + 1
        theta = (torch.randn(n, device="cuda", generator=gen) * 0.1).to(tdt)
        grads = [torch.randn(n, device="cuda", generator=gen) * 0.01 for _ in range(K1)]
        call = lambda: B.tensair_dense_apply(theta, grads, cfg.lr)
        alg = K1 * n * 4 + 2 * n * e
        units, unit, kernel = n, "parameters/s", "k_dense_apply"
        what = {"parameters": n, "gradient_blocks": K1}

        def cpu():
            m = min(n, 4_000_000)
            th = to_np(theta[:m]).copy()
            gs = [g[:m].cpu().numpy() for g in grads]
            t0 = time.perf_counter()
            oracle.dense_apply(th, odt, gs, cfg.lr)
            return m / (time.perf_counter() - t0), f"the first {m} parameters, once"
    elif args.op == "lookup":
        n = 1_000_000
        counts = np.ones(V, np.uint64)
        m = B.Model(V, D, B.F32 if cfg.dtype == "f32" else B.BF16, cfg.window, cfg.negatives, 16, 0, cfg.seed, counts)
        ids = torch.randint(0, V, (n,), device="cuda", generator=gen, dtype=torch.int32)
        out = torch.empty((n, D), device="cuda")
        call = lambda: m.lookup(0, ids, out)
        alg = n * (D * e + D * 4 + 4)
        units, unit, kernel = n, "words/s", "k_lookup"
        what = {"words": n, "dim": D}

        def cpu():
            Wn, idn = to_np(m.w_in), ids.cpu().numpy()
            t0 = time.perf_counter()
            oracle.lookup(Wn, odt, D, idn)
            return n / (time.perf_counter() - t0), "the same lookup, once"
    elif args.op == "grad_pack":
        import workload as W

        m = B.Model(V, D, B.F32 if cfg.dtype == "f32" else B.BF16, cfg.window, cfg.negatives, cfg.batch, 0, cfg.seed, counts)
        m.w_out.copy_(m.w_in)     # W_out away from zero so that both sides carry non-trivial rows
        dtok = torch.from_numpy(np.ascontiguousarray(tok, dtype=np.int32)).cuda()
        g, msg = m.grad_buffers(), m.packed_buffers()
        b0 = W.worker_batch(cfg, 0, 0)
        m.sgns_grad(dtok, b0[0], b0[1], b0[2], g)
        rows = sum(g.sizes())
        call = lambda: m.grad_pack(g, msg)
        alg = rows * (D * 4 + D * 2 + 8)
        units, unit, kernel = rows, "rows/s", "k_grad_pack"
        what = {"rows": rows, "dim": D}

        def cpu():
            (_, ri), (_, ro) = g.to_host()
            t0 = time.perf_counter()
            oracle.grad_pack_rows(ri)
            oracle.grad_pack_rows(ro)
            return rows / (time.perf_counter() - t0), "the same gradient, once"
    else:
        a = (torch.randn((V, D), device="cuda", generator=gen) * 0.1).to(tdt)
        b = (a.float() + torch.randn((V, D), device="cuda", generator=gen) * 0.02).to(tdt)
        diff = torch.empty(V, device="cuda")
        call = lambda: B.tensair_cosine_difference(a, b, D, diff)
        alg = 2 * V * D * e + V * 4
        units, unit, kernel = V, "words/s", "k_cosine_diff"
        what = {"vocab": V, "dim": D}

        def cpu():
            m = min(V, 200_000)
            an, bn = to_np(a[:m]), to_np(b[:m])
            t0 = time.perf_counter()
            oracle.cosine_difference(an, bn, odt, D)
            return m / (time.perf_counter() - t0), f"the first {m} rows, once"

    for _ in range(Wm):
        call()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(S):
        call()
    ev1.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    k_s = ev0.elapsed_time(ev1) * 1e-3 / S      # one kernel per call, back to back on torch's current stream
    # the plain copy kernel of known size, for the calibration of the HBM byte counters
    nbytes = 1 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    for _ in range(3):
        B.tensair_copy_probe(dst, src, nbytes)
    torch.cuda.synchronize()
    del src, dst
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{cfg.name}_{args.op}.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get("hbm_bytes_per_launch")
        except Exception:
            traffic = None
    out_json = {
        "metric": {"dense_apply": "dense-model gradient application (Eq. 1 on every parameter)",
                   "lookup": "embedding lookup (predict path)",
                   "cosine": "cosine difference between two embedding tables",
                   "grad_pack": "sparse gradient into a bfloat16 message"}[args.op],
        "value": units / (elapsed / S), "unit": unit, "n_gpus": 1, "steps": S, "warmup": Wm,
        "ms_per_step": elapsed / S * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if cfg.dtype == "f32" else "bf16 tables, f32 arithmetic", "data": "synthetic",
        "config": {"workload": f"{cfg.name}:{args.op}", **what},
        "roofline": {"bound": "hbm", "kernel": kernel, "achieved": alg / k_s / 1e9, "peak": HBM_PEAK / 1e9,
                     "unit": "GB/s", "frac": alg / k_s / HBM_PEAK, "traffic": traffic,
                     "algorithmic_bytes_per_launch": alg, "avg_launch_ms": k_s * 1e3},
    }
    if not args.no_cpu_baseline:
        v, sample = cpu()
        out_json["cpu_baseline"] = {"value": v, "unit": unit, "cores": 1, "kind": "oracle", "sample": sample}
    print(json.dumps(out_json), flush=True)


if __name__ == "__main__":
    main()
