#!/usr/bin/env python3
"""Benchmark of the DLRM sparse hot path on one MI355X.

One step = one pass of the whole hot path over one mini-batch that is already in
HBM: dense placement, pooled embedding lookup, dot interaction forward, dot
interaction backward, embedding backward with the fused sparse SGD update.
Prints ONE JSON line (metric, roofline of the dominant kernel, CPU-oracle
baseline).  Inputs are seeded and synthetic (workloads/gen.py).

Without --config the line is the batch-2048 multi-hot bandwidth workload (3) and carries a
`per_workload` object with the large one-hot (4) and hot-row stress (5) workloads, timed after it
in the same way with fewer steps."""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "emb-bag fwd+bwd lookups/s & HBM GB/s (% of peak); samples/s at batch 2048"
HBM_PEAK_GBPS = 8000.0
# The upstream gradient dR is drawn N(0,1) (as for the parity tests) and scaled by this power of two
# here.  A step feeds dS = interaction-backward(T, dR) back into the rows that produced T, a linear map
# on the tables whose spectral radius per step is about lr * |dR| * (bag length) * sqrt(F) on the
# multi-hot workload (0.06 unscaled: overflow after ~100 visits of a batch) and, on the hot-row
# workload, where the hottest rows sit in nearly every bag of every sample, about
# lr * |dR| * multiplicity * sqrt(B) * sqrt(K) (~350 unscaled).  Scaled by 2^-20 a 10^4-step run moves
# the tables by a few percent at most.  Kernel time does not depend on values.
DR_SCALE = 2.0 ** -20


def source_digest():
    """Digest of the HIP sources and headers the library is built from: a traffic figure measured with
    rocprofv3 counters is only quoted for the sources it was measured on."""
    h = hashlib.sha256()
    for sub in (os.path.join("paper_1906_00091_amd", "csrc"), "include"):
        for f in sorted(os.listdir(os.path.join(ROOT, sub))):
            h.update(f.encode())
            h.update(open(os.path.join(ROOT, sub, f), "rb").read())
    return h.hexdigest()[:12]


def measured_traffic():
    """HBM bytes per launch from profiles/measured_traffic.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    runs of this script, scaled by the same counters on a plain copy of known size).  Rows:
    | workload | kernel | bytes per launch | source digest |.  Returns {(workload, kernel): (bytes, digest)}."""
    out = {}
    p = os.path.join(ROOT, "profiles", "measured_traffic.md")
    if os.path.exists(p):
        for m in re.finditer(r"^\|\s*(\d+)\s*\|\s*`?(\w+)`?\s*\|\s*([0-9.eE+]+)\s*\|\s*`?([0-9a-f]{12})`?\s*\|",
                             open(p).read(), flags=re.M):
            out[(int(m.group(1)), m.group(2))] = (float(m.group(3)), m.group(4))
    return out


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", type=int, default=0,
                    help="workload 1..5 alone (default: 3 = multi-hot bandwidth, followed by 4 and 5 as per_workload)")
    ap.add_argument("--no-extra", action="store_true", help="without --config: leave workloads 4 and 5 out")
    ap.add_argument("--extra-steps", type=int, default=0,
                    help="timed steps of workloads 4 and 5 in the default run (0 = 100 and 30)")
    ap.add_argument("--algo", default="auto", choices=["auto", "sort", "atomic"])
    ap.add_argument("--optimizer", default="sgd", choices=["sgd", "adagrad"],
                    help="row update of the fused backward (the metric is quoted on sgd)")
    ap.add_argument("--tables", type=int, default=0, metavar="K",
                    help="free-form workload instead of one of the five (any of --tables --rows --dim --batch --bag "
                         "--dist --dtype; what is not given is taken from workload 3): K tables")
    ap.add_argument("--rows", type=int, default=0, help="free-form workload: rows per table")
    ap.add_argument("--dim", type=int, default=0, help="free-form workload: embedding dimension")
    ap.add_argument("--batch", type=int, default=0, help="free-form workload: mini-batch size")
    ap.add_argument("--bag", default="", help="free-form workload: bag length, L (fixed) or LO:HI (uniform, inclusive)")
    ap.add_argument("--dist", default="", help="free-form workload: index distribution, uniform or zipf:ALPHA")
    ap.add_argument("--dtype", default="", choices=["", "f32", "f16", "bf16"], help="free-form workload: table storage")
    ap.add_argument("--locality", type=float, default=0.0, metavar="ALPHA",
                    help="draw the workload's indices with the stack-distance trace generator of Sec. 4.2 from the "
                         "profile of a Zipf(ALPHA) trace instead of the workload's own distribution: same shape, "
                         "more temporal locality the larger ALPHA (a variant; the metric is quoted without)")
    ap.add_argument("--index32", action="store_true", help="int32 index arrays instead of int64")
    ap.add_argument("--weighted", action="store_true",
                    help="per-lookup weights (Eq. (2) in full) instead of sum pooling; the metric is quoted without")
    ap.add_argument("--split-fwd", action="store_true",
                    help="forward as three calls (place_dense, emb_bag_fwd, interact_dot_fwd) even where the "
                         "one-launch forward applies (short bags)")
    ap.add_argument("--keep-t", action="store_true",
                    help="where the forward is the one launch (short bags), still write T and run the interaction "
                         "backward on it, instead of the pair that never materialises T "
                         "(dlrm_emb_interact_fwd with T = NULL, dlrm_emb_interact_bwd)")
    ap.add_argument("--event-every", type=int, default=8,
                    help="an event pair around the dominant kernel is recorded on every N-th timed step")
    ap.add_argument("--self-check", type=int, default=0, metavar="N",
                    help="before anything is timed, run N steps the way they are timed and N steps call by call "
                         "on one stream from the same tables and require identical tables")
    ap.add_argument("--graph", action="store_true",
                    help="capture each distinct batch's step in a HIP graph (through torch) and time replays")
    ap.add_argument("--no-flat", action="store_true",
                    help="always enqueue the segment / hot-row launches of the backward, instead of reading the "
                         "prepared batch's count of oversized row groups on the host and leaving them out at zero")
    ap.add_argument("--no-stamp", action="store_true",
                    help="order the two streams with events only, not with the forward call's start stamp")
    ap.add_argument("--no-overlap", action="store_true",
                    help="group the (row, bag) pairs inside the backward call instead of on a second "
                         "stream beside the forward pass")
    ap.add_argument("--nbatches", type=int, default=0, help="distinct batches cycled (0 = pick)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--copy-calib", action="store_true",
                    help="run a 1 GiB plain copy (place_dense with F=1) before the timed region, as the "
                         "known-size reference for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs")
    ap.add_argument("--ceilings", action="store_true",
                    help="instead of a workload, time the plain memory kernels of libdlrm_ceilings (stream copy and "
                         "read, random whole-row gather and read-modify-write) and print what this board "
                         "sustains for each pattern, one JSON line")
    return ap.parse_args()


def measure_ceilings(torch, ceilings, reps=20):
    """GB/s of the measurement kernels: 4 GiB streamed; 1.5 GB of distinct random rows out of a 2 GiB
    table for the row patterns (HIP events around `reps` back-to-back launches on the current stream)."""
    dev = "cuda:0"
    sink = ceilings.ceiling_sink()

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        b.synchronize()
        return a.elapsed_time(b) / reps   # ms

    out = {}
    n = 1 << 30                                   # fp32 elements: 4 GiB
    src = torch.ones(n, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    out["stream_copy"] = round(2 * 4 * n / timed(lambda: ceilings.dlrm_ceiling_copy(src, dst)) / 1e6, 1)
    out["stream_read"] = round(4 * n / timed(lambda: ceilings.dlrm_ceiling_read(src, sink)) / 1e6, 1)
    del dst
    table = src[: n // 2]                          # 2 GiB
    g = torch.Generator(device=dev).manual_seed(1)
    for row_bytes in (64, 256, 512):
        nrows = table.numel() * 4 // row_bytes
        take = int(1.5e9) // row_bytes
        rows = torch.randperm(nrows, generator=g, device=dev)[:take].to(torch.int32)
        ms = timed(lambda: ceilings.dlrm_ceiling_gather(table, rows, row_bytes, sink))
        out["row_gather_%dB" % row_bytes] = round(take * row_bytes / ms / 1e6, 1)
        if row_bytes != 64:
            ms = timed(lambda: ceilings.dlrm_ceiling_rmw(table, rows, row_bytes))
            out["row_rmw_%dB" % row_bytes] = round(2 * take * row_bytes / ms / 1e6, 1)
        del rows
    del src, table
    torch.cuda.empty_cache()
    return out


def algorithmic_bytes(w, batch, elem_bytes, index_bytes=8, weighted=False):
    """Minimum HBM traffic of the embedding forward / backward for this batch (ideal cache:
    each touched row once, each index, offset, pooled vector and gradient once)."""
    import numpy as np
    U = sum(len(np.unique(batch.indices_of(k))) for k in range(w.K))
    nnz = batch.nnz
    csr = nnz * (index_bytes + (4 if weighted else 0)) + w.K * (w.B + 1) * 8
    pooled = w.K * w.B * w.d * 4
    fwd = U * w.d * elem_bytes + csr + pooled
    bwd = pooled + csr + 2 * U * w.d * elem_bytes
    int_fwd = w.B * (w.F * w.d + w.d + w.P) * 4
    int_bwd = w.B * (2 * w.F * w.d + w.d + w.P) * 4
    return dict(U=U, nnz=nnz, fwd=fwd, bwd=bwd, int_fwd=int_fwd, int_bwd=int_bwd, csr=csr,
                # the one-launch forward that leaves T alone: rows, indices, x in; R out
                fwd_no_t=U * w.d * elem_bytes + csr + w.B * w.d * 4 + w.B * (w.d + w.P) * 4,
                # the backward that pools again: rows, indices, x, dR in; dT out
                bwd_no_t=U * w.d * elem_bytes + csr + w.B * w.d * 4 + w.B * (w.d + w.P) * 4 + w.B * w.F * w.d * 4,
                fwd_logical=nnz * w.d * elem_bytes + csr + pooled)


def stats(xs):
    import numpy as np
    a = np.asarray(xs, dtype=np.float64)
    return {"mean": round(float(a.mean()), 5), "median": round(float(np.median(a)), 5),
            "min": round(float(a.min()), 5), "max": round(float(a.max()), 5), "n": int(a.size)}


def free_form_workload(args):
    """The workload the free-form flags describe (None if none is given); defaults from workload 3."""
    from workloads import gen
    if not (args.tables or args.rows or args.dim or args.batch or args.bag or args.dist or args.dtype):
        return None
    base = gen.WORKLOADS[3]
    bag = base.bag
    if args.bag:
        lo, _, hi = args.bag.partition(":")
        bag = ("uniform", int(lo), int(hi)) if hi else ("fixed", int(lo))
    dist = base.dist
    if args.dist:
        name, _, alpha = args.dist.partition(":")
        dist = ("zipf", float(alpha)) if name == "zipf" else ("uniform",)
    dtype = {"": base.dtype, "f32": gen.F32, "f16": gen.F16, "bf16": gen.BF16}[args.dtype]
    return gen.custom_workload("custom", K=args.tables or base.K, B=args.batch or base.B, d=args.dim or base.d,
                               dtype=dtype, rows=args.rows or int(base.rows[1]), bag=bag, dist=dist)


def run_workload(args, config, steps, warmup, headline, ceil):
    """Times `steps` steps of workload `config` after `warmup`; returns the fields of its JSON object.
    headline: also the CPU-oracle baseline and the self-check; otherwise a shorter record."""
    import ctypes

    import numpy as np
    import torch

    import paper_1906_00091_amd as hot
    from workloads import gen

    dev = "cuda:0"
    w = free_form_workload(args) if config == 0 else gen.WORKLOADS[config]
    if args.locality > 0:
        import dataclasses
        w = dataclasses.replace(w, name="%s_trace_a%g" % (w.name, args.locality), dist=("trace", float(args.locality)))
    print("bench.py: workload %d (%s), %d steps" % (config, w.name, steps), file=sys.stderr, flush=True)
    eb = gen.ELEM_BYTES[w.dtype]
    algo = {"auto": hot.BWD_AUTO, "sort": hot.BWD_SORT, "atomic": hot.BWD_ATOMIC}[args.algo]
    B, F, d, P, K = w.B, w.F, w.d, w.P, w.K

    # ---- inputs, resident in HBM before anything is timed
    rows = gen.table_rows(w)
    first = gen.make_batch(w, rows=rows)
    ab0 = algorithmic_bytes(w, first, eb, 4 if args.index32 else 8, args.weighted)
    nb = args.nbatches
    if nb <= 0:  # enough distinct batches that one batch's rows are out of the 256 MB cache again
        nb = int(min(32, max(2, -(-(1 << 30) // max(ab0["fwd"], 1)))))
    batches = [first] + [gen.make_batch(w, batch_id=i, rows=rows) for i in range(1, nb)]
    abytes = [ab0] + [algorithmic_bytes(w, b, eb, 4 if args.index32 else 8, args.weighted) for b in batches[1:]]
    tdt = {gen.F32: torch.float32, gen.F16: torch.float16, gen.BF16: torch.bfloat16}[w.dtype]
    tables = []
    for k in range(K):
        t = torch.empty((int(rows[k]), d), dtype=tdt, device=dev)
        hot.dlrm_table_init_hash(t, w.dtype, gen.table_key(w.seed, k), float(gen.table_scale(int(rows[k]))))
        tables.append(t)
    dev_batches = []
    for b in batches:
        wts = torch.from_numpy(gen.make_weights(b)).to(dev) if args.weighted else None
        sb = hot.SparseBatch(tables, w.dtype,
                             torch.from_numpy(b.indices.astype(np.int32) if args.index32 else b.indices).to(dev),
                             torch.from_numpy(np.ascontiguousarray(b.offsets)).to(dev),
                             torch.from_numpy(b.tbl_off).to(dev), b.nnz, max_rows=int(rows.max()), weights=wts)
        dev_batches.append((sb, torch.from_numpy(b.x).to(dev), torch.from_numpy(b.dR).to(dev) * DR_SCALE))
    max_nnz = max(b.nnz for b in batches)
    ws_bytes = hot.dlrm_emb_bag_bwd_workspace_bytes(K, B, d, max_nnz, int(rows.max()), w.dtype)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    T = torch.empty((B, F, d), dtype=torch.float32, device=dev)
    R = torch.empty((B, d + P), dtype=torch.float32, device=dev)
    dT = torch.empty((B, F, d), dtype=torch.float32, device=dev)
    lr = float(np.float32(w.lr))
    adagrad = args.optimizer == "adagrad"
    if adagrad:
        assert args.algo != "atomic", "adagrad runs on the sort path only"
        state = [torch.zeros_like(t, dtype=torch.float32) for t in tables]
        state_ptrs = hot.state_pointers(state)
        eps = 1e-8

    # the library's own rule for dlrm_emb_interact_fwd(DLRM_FWD_AUTO), spelled out so the line says which ran
    fused_fwd = (not args.split_fwd and not args.weighted and K <= 64
                 and sum(b.nnz for b in batches) / (len(batches) * K * B) <= 4.0)

    # short bags and a T of at least 16 MiB: the step never writes or reads T (below that the three kernels are
    # latency-bound and the pair measured 1-2 us slower per step on the tiny and click-log workloads)
    no_t = fused_fwd and not args.keep_t and B * F * d * 4 >= (16 << 20)

    def backward(sb, algo_code, ws=ws, red=None):
        """red: a pair of raw HIP events recorded around the dominant kernel of THIS call."""
        if adagrad:
            if red is None:
                hot.dlrm_emb_bag_bwd_adagrad(sb, state_ptrs, dT, F * d, d, lr, eps, ws, algo=algo_code, dS_offset=d)
            else:
                hot.dlrm_emb_bag_bwd_adagrad_timed(sb, state_ptrs, dT, F * d, d, lr, eps, ws, red[0], red[1],
                                                   algo=algo_code, dS_offset=d)
        elif red is None:
            hot.dlrm_emb_bag_bwd_sgd(sb, dT, F * d, d, lr, ws, algo=algo_code, dS_offset=d)
        else:
            hot.dlrm_emb_bag_bwd_sgd_timed(sb, dT, F * d, d, lr, ws, red[0], red[1], algo=algo_code, dS_offset=d)

    stages = ["place_dense", "emb_bag_fwd", "interact_dot_fwd", "interact_dot_bwd", "emb_bag_bwd_sgd"]
    # The grouping of the batch's (row, bag) pairs needs the indices only: it is enqueued on a
    # second stream at the start of the step and meets the main stream before the row update.
    # Below ~200K lookups the grouping is shorter than the cross-stream hand-over costs on the host
    # (measured: the 53K-lookup click-log batch loses 40 us per step to it, the 213K one gains 14).
    overlap = args.algo != "atomic" and not args.no_overlap and max_nnz >= 200_000
    side = torch.cuda.Stream() if overlap else None     # default priority
    prep_done = torch.cuda.Event()   # (inside a captured graph only)
    use_flat = overlap and not args.no_flat and not args.graph
    # raw HIP events (ctypes): the pair recorded around the dominant kernel, and the events
    # that order the two streams.  Neither needs the system-scope fence a default event ends in: the
    # timing pair is created with hipEventDisableSystemFence, the ordering events with
    # hipEventDisableTiming | hipEventReleaseToDevice (both ends are kernels on this device).  (An A/B on
    # one box showed no difference in step time against default events.)
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventCreateWithFlags.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint]
    hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    hip.hipStreamWaitEvent.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint]
    hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
    EV_TIMING, EV_ORDER = 0x20000000, 0x2 | 0x40000000
    all_events = []

    def hip_event(flags=EV_TIMING):
        ev = ctypes.c_void_p()
        assert hip.hipEventCreateWithFlags(ctypes.byref(ev), flags) == 0
        all_events.append(ev)
        return ev

    def ev_record(ev, stream):
        assert hip.hipEventRecord(ev, ctypes.c_void_p(stream.cuda_stream)) == 0

    def ev_wait(stream, ev):
        assert hip.hipStreamWaitEvent(ctypes.c_void_p(stream.cuda_stream), ev, 0) == 0

    def ev_ms(a, b):
        ms = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
        return ms.value

    # With the count in use the grouping runs one step ahead, in the other of two workspaces (the indices
    # of the next batch are there early, Sec. 4.1), so that the host never waits for it.
    ws2 = [ws, torch.empty_like(ws)] if use_flat else [ws]
    n_over = torch.zeros(2, dtype=torch.int32).pin_memory()   # written by the device, read by the host
    n_over_np = n_over.numpy()
    prep_done2 = [hip_event(EV_ORDER), hip_event(EV_ORDER)]
    upd_done2 = [hip_event(EV_ORDER), hip_event(EV_ORDER)]
    prep_done_r, upd_done_r = hip_event(EV_ORDER), hip_event(EV_ORDER)
    main = torch.cuda.current_stream()

    # Stream order without events where the forward is one call: its first kernel stamps a pinned word
    # as it starts, which tells the polling host that the previous step's update is over (an event
    # recorded on the first stream costs the step 6.5 us; the stamp rides in a kernel that runs anyway).
    use_stamp = use_flat and not args.split_fwd and not args.no_stamp
    stamp = torch.zeros(1, dtype=torch.int32).pin_memory()
    stamp_np = stamp.numpy()
    seq = [0]
    cycle = [nb]   # distinct batches the steps cycle through (1 for the same-batch pass)

    def host_wait(cond, what):
        """Spin on pinned memory the device writes (no driver call, no sleep); the time goes to poll_wait."""
        spins = 0
        while not cond():
            spins += 1
            if spins == 1:
                t_poll[0] = time.perf_counter()
            if spins % (1 << 20) == 0 and time.perf_counter() - t_poll[0] > 20.0:
                raise RuntimeError(what + " never arrived")
        if spins:
            poll_wait[0] += time.perf_counter() - t_poll[0]
            poll_wait[1] += 1

    def prepare_ahead(i, after_seq=0):
        """Grouping of step i's batch on the side stream, in workspace i % 2, with its oversized count.
        The workspace was last used by step i - 2: with stamps the host waits until the forward pass of
        step i - 1 has begun, else the side stream waits for the event recorded behind that update."""
        p = i % 2
        if use_stamp:
            host_wait(lambda: stamp_np[0] >= after_seq, "the start stamp of the forward pass")
        else:
            ev_wait(side, upd_done2[p])
        n_over_np[p] = -1
        hot.dlrm_emb_bag_bwd_prepare(dev_batches[i % cycle[0]][0], ws2[p], stream=side)
        hot.dlrm_emb_bag_bwd_prepared_oversized(dev_batches[i % cycle[0]][0], ws2[p], n_over, index=p, stream=side)
        if not use_stamp:
            ev_record(prep_done2[p], side)
    flat_steps = [0]
    t_poll = [0.0]
    poll_wait = [0.0, 0]

    if args.copy_calib:  # 2^22 x 64 fp32 = 1 GiB read + 1 GiB written by a plain copy kernel
        src = torch.empty((1 << 22, 64), dtype=torch.float32, device=dev).normal_()
        dst = torch.empty((1 << 22, 1, 64), dtype=torch.float32, device=dev)
        for _ in range(3):
            hot.dlrm_place_dense(src, dst)
        torch.cuda.synchronize()
        del src, dst

    def step(i, ev=None, red=None, overlap=overlap, capturing=False):
        sb, x, dR = dev_batches[i % cycle[0]]
        ahead = overlap and mode["ahead"] and not capturing and ev is None
        if overlap and not ahead:
            if capturing:  # inside a graph the second stream forks from the capturing one
                side.wait_stream(torch.cuda.current_stream())
            else:
                ev_wait(side, upd_done_r)   # the previous step's update is done with the workspace
            with torch.cuda.stream(side):
                hot.dlrm_emb_bag_bwd_prepare(sb, ws)
                if capturing:
                    prep_done.record(side)
                else:
                    ev_record(prep_done_r, side)
        if ev is not None:
            ev[0].record()
        if not args.split_fwd and ev is None:
            # one call; one launch for short bags, else two (the dense vectors ride in the pooling launch)
            if ahead and use_stamp:
                seq[0] += 1
                hot.dlrm_emb_interact_fwd_stamped(sb, x, None if no_t else T, R,
                                                  hot.FWD_FUSED if fused_fwd else hot.FWD_SPLIT, stamp, seq[0])
            else:
                hot.dlrm_emb_interact_fwd(sb, x, None if no_t else T, R, hot.FWD_FUSED if fused_fwd else hot.FWD_SPLIT)
        else:
            hot.dlrm_place_dense(x, T)
            if ev is not None:
                ev[1].record()
            hot.dlrm_emb_bag_fwd(sb, T, F * d, d, out_offset=d)
            if ev is not None:
                ev[2].record()
            hot.dlrm_interact_dot_fwd(T, R)
            if ev is not None:
                ev[3].record()
        if no_t and ev is None:
            hot.dlrm_emb_interact_bwd(sb, x, dR, dT)   # pools the bags again instead of reading T
        else:
            hot.dlrm_interact_dot_bwd(T, dR, dT)
        if ev is not None:
            ev[4].record()
        if ahead:
            p = i % 2
            # the count arrives behind the grouping on the side stream: once the host has it, the
            # grouping is done and the first stream need not wait for it
            host_wait(lambda: n_over_np[p] >= 0, "the oversized count of step %d" % i)
            code = hot.BWD_SORT_PREPARED
            if n_over_np[p] == 0:
                code = hot.BWD_SORT_PREPARED_FLAT
                flat_steps[0] += 1
            if use_stamp:
                backward(sb, code, ws2[p], red)
                prepare_ahead(i + 1, seq[0])
            else:
                ev_wait(main, prep_done2[p])
                backward(sb, code, ws2[p], red)
                ev_record(upd_done2[p], main)
                prepare_ahead(i + 1)
        elif overlap:
            if capturing:
                torch.cuda.current_stream().wait_event(prep_done)
            else:
                ev_wait(main, prep_done_r)
            backward(sb, hot.BWD_SORT_PREPARED, red=red)
            if not capturing:
                ev_record(upd_done_r, main)
        else:
            backward(sb, algo, red=red)
        if ev is not None:
            ev[5].record()

    mode = {"ahead": use_flat}
    if args.self_check and headline:
        # The steps as they are timed (two streams, events without system fence, the count read from
        # pinned memory, one-call forward) against the same steps issued call by call on one stream:
        # the sort path is bit-reproducible, so the tables must come out identical.
        n_chk = args.self_check
        saved = [t.clone() for t in tables]
        saved_state = [h.clone() for h in state] if adagrad else None
        for ahead_mode in ([True, False] if use_flat else [False]):
            mode["ahead"] = ahead_mode
            if ahead_mode:
                prepare_ahead(0)
            for i in range(n_chk):
                step(i)
            torch.cuda.synchronize()
            piped = [t.clone() for t in tables]
            for t, t0 in zip(tables, saved):
                t.copy_(t0)
            if adagrad:
                for h, h0 in zip(state, saved_state):
                    h.copy_(h0)
            for i in range(n_chk):
                step(i, ev=[torch.cuda.Event() for _ in range(6)], overlap=False)
            torch.cuda.synchronize()
            for k in range(K):
                if not torch.equal(piped[k].view(torch.uint8), tables[k].view(torch.uint8)):
                    raise SystemExit("bench.py --self-check: table %d differs between the timed step "
                                     "sequence (ahead=%s) and the call-by-call one" % (k, ahead_mode))
                if bool((piped[k] != saved[k]).any()) is False and k == 0:
                    raise SystemExit("bench.py --self-check: the steps changed nothing in table 0")
            for t, t0 in zip(tables, saved):
                t.copy_(t0)
            if adagrad:
                for h, h0 in zip(state, saved_state):
                    h.copy_(h0)
            del piped
        del saved, saved_state
        mode["ahead"] = use_flat
        flat_steps[0] = 0
        print("bench.py --self-check: %d steps, tables identical" % n_chk, file=sys.stderr, flush=True)
    if use_flat:
        prepare_ahead(0)
    for i in range(warmup):
        step(i)
    if use_flat and flat_steps[0] == 0:
        # every warm-up batch had oversized row groups (heavy hitters): the count buys nothing, and the
        # grouping overlaps better with the forward pass of its own step than with the previous update
        mode["ahead"] = False
    flat_before = flat_steps[0]
    torch.cuda.synchronize()
    # ---- timed region: exactly `steps` steps; the only events inside are the pairs around the
    # dominant backward kernel, on its launch stream, on every --event-every-th step
    red_ev = {}
    can_red = args.algo != "atomic"
    ev_record(upd_done_r, main)
    torch.cuda.synchronize()
    nxt = warmup   # index of the next step in the sequence
    if args.graph:
        # one graph per distinct batch = one whole step (kernel launches only: the library allocates
        # nothing, sets no memory and never synchronises); replays are what is timed
        graphs = []
        for bi in range(nb):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                step(bi, capturing=True)
            graphs.append(g)
        torch.cuda.synchronize()
        for i in range(min(warmup, 2 * nb)):
            graphs[i % nb].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            graphs[(warmup + i) % nb].replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    else:
        for i in range(0, steps, args.event_every):
            if can_red:
                red_ev[i] = (hip_event(), hip_event())
        t0 = time.perf_counter()
        for i in range(steps):
            step(warmup + i, red=red_ev.get(i))
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        nxt = warmup + steps
    ms_per_step = elapsed * 1e3 / steps
    flat_timed = flat_steps[0] - flat_before
    ids = [(warmup + i) % nb for i in range(steps)]
    red_samples = [ev_ms(a, b_) for a, b_ in red_ev.values()]
    n_red_timed = len(red_samples)

    # ---- more samples of the dominant kernel where the timed region gave fewer than 12: the same
    # step sequence goes on, an event pair on every step (the pairs cost time: these steps are not timed)
    if can_red and not args.graph and len(red_samples) < 12:
        more = [(hip_event(), hip_event()) for _ in range(12 - len(red_samples))]
        for q, pair in enumerate(more):
            step(nxt + q, red=pair)
        torch.cuda.synchronize()
        nxt += len(more)
        red_samples += [ev_ms(a, b_) for a, b_ in more]

    # ---- spread of the step time: the same sequence in 10 chunks, each bracketed by a synchronisation
    chunk_ms = None
    if not args.graph:
        per = max(5, steps // 10)
        chunk_ms = []
        for _ in range(10):
            torch.cuda.synchronize()
            c0 = time.perf_counter()
            for q in range(per):
                step(nxt + q)
            torch.cuda.synchronize()
            chunk_ms.append((time.perf_counter() - c0) * 1e3 / per)
            nxt += per

    # ---- "warm": the same batch over and over (its rows, indices and gradients stay in the caches)
    warm_ms = None
    if not args.graph:
        torch.cuda.synchronize()
        cycle[0] = 1
        nwarm = max(10, steps // 3)
        if mode["ahead"]:
            prepare_ahead(nxt)   # regroup for batch 0 (the pending grouping was for another batch)
        for q in range(3):
            step(nxt + q)
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for q in range(3, 3 + nwarm):
            step(nxt + q)
        torch.cuda.synchronize()
        warm_ms = (time.perf_counter() - c0) * 1e3 / nwarm
        cycle[0] = nb
        nxt += 3 + nwarm

    # ---- per-call breakdown: a separate pass AFTER the timed region, every call on one stream
    # with an event on either side (grouping inside the backward call), same batches in the
    # same order.  Its sum is a little above the step time of an overlapped run.
    nbk = min(steps, 100)
    step(warmup, ev=[torch.cuda.Event() for _ in range(6)], overlap=False)  # first use of the separate forward kernels is not timed
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(nbk)]
    red_bk = [(hip_event(), hip_event()) for _ in range(nbk)] if args.graph and can_red else None
    for i in range(nbk):
        # (with --graph the event pair cannot sit inside the replays: it is recorded here)
        step(warmup + i, ev=events[i], overlap=False, red=red_bk[i] if red_bk else None)
    torch.cuda.synchronize()
    if red_bk:
        red_samples = [ev_ms(a, b_) for a, b_ in red_bk]
    stage_all = {s: [ev[j].elapsed_time(ev[j + 1]) for ev in events] for j, s in enumerate(stages)}
    stage_ms = {s: float(np.mean(v)) for s, v in stage_all.items()}

    # the update on a batch whose grouping is already done (what the timed steps run after the two
    # streams have met), by itself: grouped outside the interval, same algo choice as in the timed steps
    prepared_ms = pair_ms = None
    if overlap:
        pe = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(nbk)]
        # which update every distinct batch takes is found first (a host read), so that the timed calls
        # follow one another without the host in between
        codes = []
        chk = torch.zeros(1, dtype=torch.int32, device=dev)
        for bi in range(nb):
            code = hot.BWD_SORT_PREPARED
            if mode["ahead"]:
                hot.dlrm_emb_bag_bwd_prepare(dev_batches[bi][0], ws)
                hot.dlrm_emb_bag_bwd_prepared_oversized(dev_batches[bi][0], ws, chk)
                if int(chk.item()) == 0:
                    code = hot.BWD_SORT_PREPARED_FLAT
            codes.append(code)
        for i in range(nbk):
            bi = (warmup + i) % nb
            sb = dev_batches[bi][0]
            hot.dlrm_emb_bag_bwd_prepare(sb, ws)
            pe[i][0].record()
            backward(sb, codes[bi])
            pe[i][1].record()
        torch.cuda.synchronize()
        prepared_ms = sum(a.elapsed_time(b_) for a, b_ in pe) / nbk
        # and the pair as the timed steps run it: the pooling call, then the update call on the grouped batch,
        # back to back in one interval (the update then finds the rows the pooling just read in the last-level
        # cache, as it does in a step; the two calls timed apart do not show that)
        pp = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(nbk)]
        for i in range(nbk):
            bi = (warmup + i) % nb
            sb = dev_batches[bi][0]
            hot.dlrm_emb_bag_bwd_prepare(sb, ws)
            pp[i][0].record()
            hot.dlrm_emb_bag_fwd(sb, T, F * d, d, out_offset=d)
            backward(sb, codes[bi])
            pp[i][1].record()
        torch.cuda.synchronize()
        pair_ms = sum(a.elapsed_time(b_) for a, b_ in pp) / nbk

    fused_ms = None
    if fused_fwd:  # the one-launch forward by itself, same batches
        fe = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(nbk)]
        for i in range(nbk):
            sb, x, _ = dev_batches[(warmup + i) % nb]
            fe[i][0].record()
            hot.dlrm_emb_interact_fwd(sb, x, None if no_t else T, R, hot.FWD_FUSED)
            fe[i][1].record()
        torch.cuda.synchronize()
        fused_ms = sum(a.elapsed_time(b_) for a, b_ in fe) / nbk

    not_ms = None
    if no_t:  # the backward that pools again, by itself, same batches
        fe = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(nbk)]
        for i in range(nbk):
            sb, x, dR = dev_batches[(warmup + i) % nb]
            fe[i][0].record()
            hot.dlrm_emb_interact_bwd(sb, x, dR, dT)
            fe[i][1].record()
        torch.cuda.synchronize()
        not_ms = sum(a.elapsed_time(b_) for a, b_ in fe) / nbk
        hot.dlrm_emb_interact_fwd(dev_batches[0][0], dev_batches[0][1], T, R, hot.FWD_FUSED)   # (T for the checks below)

    # ---- the state the steps left behind is finite (the feedback is bounded, see DR_SCALE)
    bad = [n for n, t in (("T", T), ("R", R), ("dT", dT)) if not bool(torch.isfinite(t).all())]
    max_abs = 0.0
    for k in range(K):
        sb0 = dev_batches[0][0]
        a0, a1 = int(batches[0].tbl_off[k]), int(batches[0].tbl_off[k + 1])
        if a1 > a0:
            touched = tables[k].index_select(0, sb0.indices[a0:min(a1, a0 + 200000)].long()).float()
            if not bool(torch.isfinite(touched).all()):
                bad.append("table %d" % k)
            else:
                max_abs = max(max_abs, float(touched.abs().max()))
    finite = not bad
    if not finite:
        raise SystemExit("bench.py: non-finite values after the run of workload %d in: %s" % (config, ", ".join(bad)))

    mean = lambda key: float(np.mean([abytes[i][key] for i in ids]))
    nnz_mean = mean("nnz")
    lookups_per_s = nnz_mean / (ms_per_step * 1e-3)
    emb_ms = stage_ms["emb_bag_fwd"] + stage_ms["emb_bag_bwd_sgd"]
    bwd_bytes = mean("bwd") + (2 * mean("U") * d * 4 if adagrad else 0.0)
    emb_bytes = mean("fwd") + bwd_bytes
    emb_logical = mean("fwd_logical") + bwd_bytes   # every looked-up row counted per lookup in the forward

    # ---- roofline of the dominant kernel.  Both embedding kernels are HBM-bound gathers /
    # scatters; the forward call is one kernel (its call events time it), the backward's
    # bucket_reduce kernel is timed by the event pairs of the timed calls.
    red_ms = float(np.mean(red_samples)) if red_samples else 0.0
    # algorithmic bytes of one bucket_reduce launch: the sorted (row, bag) pairs (8 B per lookup),
    # every pooled-vector gradient once, every touched row read and written once
    # (Adagrad: plus every touched row of the fp32 state read and written once)
    row_rw = d * eb + (d * 4 if adagrad else 0)
    red_bytes = float(np.mean([abytes[i]["nnz"] * 8 + K * B * d * 4 + 2 * abytes[i]["U"] * row_rw for i in ids]))
    fwd_kernel_ms = fused_ms if fused_fwd else stage_ms["emb_bag_fwd"]
    fwd_kernel_bytes = mean("fwd_no_t") if no_t else mean("fwd") + (mean("int_fwd") if fused_fwd else 0.0)
    kernels = {
        ("pooled_interact_fwd_kernel" if fused_fwd else "emb_fwd_kernel"): (fwd_kernel_bytes, fwd_kernel_ms),
        "bucket_reduce_kernel": (red_bytes, red_ms),
        ("pooled_interact_bwd_kernel" if no_t else "interact_bwd_kernel"):
            (mean("bwd_no_t"), not_ms) if no_t else (mean("int_bwd"), stage_ms["interact_dot_bwd"]),
    }
    dom = max(kernels, key=lambda n: kernels[n][1])
    dom_bytes, dom_ms = kernels[dom]
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    traffic, traffic_note = None, "no counter run on record for this workload and kernel"
    rec = measured_traffic().get((config, dom))
    if adagrad or args.weighted or args.index32 or args.locality > 0 or config == 0:
        traffic_note = "counter runs are on record for the five workloads with sum pooling, SGD, int64 indices only"
    elif rec is not None:
        if rec[1] == source_digest():
            traffic, traffic_note = rec[0], "profiles/measured_traffic.md (rocprofv3 --pmc runs on these sources)"
        else:
            traffic_note = ("profiles/measured_traffic.md holds %.4g bytes measured on sources %s; the sources are now %s"
                            % (rec[0], rec[1], source_digest()))
    if dom == "bucket_reduce_kernel":
        timing = ("HIP event pairs recorded on the launch stream around this kernel by the timed calls: every "
                  "%d-th step of the timed region (%d samples; each pair costs its step about 10 us)%s"
                  % (args.event_every, n_red_timed,
                     ", plus %d steps that continue the sequence behind it" % (len(red_samples) - n_red_timed)
                     if len(red_samples) > n_red_timed else "")) if not args.graph else \
                 "event pairs around the kernel in the separate pass after the replays"
    else:
        timing = "events around the call, separate single-stream pass after the timed region"
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                "traffic": traffic, "traffic_source": traffic_note,
                "algorithmic_bytes_per_launch": int(dom_bytes), "avg_launch_ms": round(dom_ms, 5),
                "launch_ms": stats(red_samples) if dom == "bucket_reduce_kernel" and red_samples else None,
                "launch_timing": timing,
                "other_kernels": {n: {"algorithmic_bytes_per_launch": int(v[0]), "avg_launch_ms": round(v[1], 5),
                                      "achieved": round(v[0] / (v[1] * 1e-3) / 1e9, 1) if v[1] > 0 else None}
                                  for n, v in kernels.items() if n != dom}}
    if ceil is not None:
        row_bytes = 512 if d * eb > 256 else 256   # the row patterns are measured at 64, 256 and 512 bytes
        pattern = ("row_rmw_%dB" % row_bytes if dom == "bucket_reduce_kernel" else
                   "stream_copy" if dom == "interact_bwd_kernel" else "row_gather_%dB" % row_bytes)
        # (the pooled-interaction kernels gather rows and stream the rest: held against the gather)
        roofline["board_ceiling"] = {"pattern": pattern, "GBps": ceil[pattern],
                                     "frac": round(achieved / ceil[pattern], 4)}

    def rate(nbytes, ms):
        gbps = nbytes / (ms * 1e-3) / 1e9
        r = {"ms": round(ms, 5), "algorithmic_GBps": round(gbps, 1), "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4)}
        if ceil is not None:
            r["frac_of_measured_copy"] = round(gbps / ceil["stream_copy"], 4)
        return r

    out = {
        "metric": METRIC, "value": round(lookups_per_s, 1), "unit": "lookups/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": gen.DTYPE_NAMES[w.dtype] if w.dtype != gen.F16 else "f16 tables, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": "%d:%s" % (config, w.name), "tables": K, "batch": B, "dim": d,
                   "rows_total": int(rows.sum()), "lookups_per_step": int(round(nnz_mean)),
                   "unique_rows_per_step": int(round(mean("U"))), "distinct_batches": nb,
                   "bwd_algo": args.algo, "optimizer": args.optimizer, "pooling": "weighted" if args.weighted else "sum",
                   "indices": "int32" if args.index32 else "int64",
                   "index_distribution": ("stack-distance generator (Sec. 4.2) on the profile of a Zipf(%g) trace" % args.locality
                                          if args.locality > 0 else {"uniform": "uniform", "zipf": "Zipf(%s)" % (w.dist[1:] or ("",))[0]}[w.dist[0]]), "launch": "hip graph replays" if args.graph else "eager",
                   "lr": w.lr, "upstream_gradient": "N(0,1) x 2^-20 (keeps the fed-back tables finite over 10^4 steps and more)",
                   "forward": ("emb_interact_fwd, one launch, T not written; backward dlrm_emb_interact_bwd pools again" if no_t else
                               "emb_interact_fwd, one launch" if fused_fwd else
                               "place_dense, emb_bag_fwd, interact_dot_fwd" if args.split_fwd else
                               "emb_interact_fwd, two launches (pooling with the dense copy, interaction)"),
                   "grouping": ("second stream, one step ahead (two workspaces)" if mode["ahead"] else
                                "second stream, beside the forward pass" if overlap else "inside the backward call"),
                   "backward_tail": ("left out on steps whose prepared batch reports no oversized row group "
                                     "(%d of the %d timed steps)" % (flat_timed, steps))
                                    if mode["ahead"] else "always enqueued"},
        "samples_per_s": round(B / (ms_per_step * 1e-3), 1),
        "ms_per_step_chunks": None if chunk_ms is None else dict(
            stats(chunk_ms), what="10 further chunks of %d steps of the same sequence, each between two "
                                  "synchronisations; mean step time per chunk" % max(5, steps // 10)),
        "ms_per_step_same_batch": None if warm_ms is None else round(warm_ms, 5),
        "emb_fwd_bwd": dict(rate(emb_bytes, emb_ms), lookups_per_s=round(nnz_mean / (emb_ms * 1e-3), 1),
                            logical_GBps=round(emb_logical / (emb_ms * 1e-3) / 1e9, 1)),
        "stage_ms": {k: round(v, 5) for k, v in stage_ms.items()},
        "stage_ms_median": {k: round(float(np.median(v)), 5) for k, v in stage_all.items()},
        "stage_ms_min": {k: round(float(np.min(v)), 5) for k, v in stage_all.items()},
        "host_poll_wait": {"ms_total": round(poll_wait[0] * 1e3, 3), "steps_that_waited": poll_wait[1]},
        "emb_interact_fwd_ms": None if fused_ms is None else round(fused_ms, 5),
        "emb_interact_bwd_ms": None if not_ms is None else round(not_ms, 5),
        "emb_bag_bwd_prepared_ms": None if prepared_ms is None else round(prepared_ms, 5),
        "emb_fwd_bwd_prepared": None if prepared_ms is None else dict(
            rate(emb_bytes, stage_ms["emb_bag_fwd"] + prepared_ms),
            note="forward call + update call on an already grouped batch, each timed by itself (the grouping runs "
                 "on the second stream in the timed steps)"),
        "emb_fwd_bwd_prepared_pair": None if pair_ms is None else dict(
            rate(emb_bytes, pair_ms),
            note="the same two calls back to back in one interval, as in a timed step"),
        "stage_ms_source": "separate single-stream pass of %d steps after the timed region" % nbk,
        "stage_algorithmic_GBps": {
            "emb_bag_fwd": round(mean("fwd") / (stage_ms["emb_bag_fwd"] * 1e-3) / 1e9, 1),
            "emb_bag_fwd_logical": round(mean("fwd_logical") / (stage_ms["emb_bag_fwd"] * 1e-3) / 1e9, 1),
            "emb_bag_bwd_sgd": round(bwd_bytes / (stage_ms["emb_bag_bwd_sgd"] * 1e-3) / 1e9, 1),
            "interact_dot_fwd": round(mean("int_fwd") / (stage_ms["interact_dot_fwd"] * 1e-3) / 1e9, 1),
            "interact_dot_bwd": round(mean("int_bwd") / (stage_ms["interact_dot_bwd"] * 1e-3) / 1e9, 1)},
        "state_after_run": {"finite": finite, "max_abs_touched_table_value": round(max_abs, 6)},
        "roofline": roofline,
    }

    # ---- CPU baseline: the oracle as it stands, on this machine's host cores, same workload
    if headline and not args.no_cpu_baseline and not args.weighted:
        from oracle import oracle
        b = batches[0]
        host_tables = []
        full = sum(int(r) for r in rows) * d * eb <= 8 << 30
        if full:
            for t in tables:
                a = t.cpu()
                host_tables.append(a.view(torch.int16).numpy().view(np.uint16) if w.dtype == gen.BF16
                                   else a.numpy())
            idx = b.indices
            sample = "whole steps of workload %d on full-size host tables copied from the device" % config
        else:  # tables too large for the host: touched rows only (flatters the CPU's caches)
            idx = np.empty_like(b.indices)
            for k in range(K):
                u = np.unique(b.indices_of(k))
                sel = torch.from_numpy(u).to(dev)
                a = tables[k].index_select(0, sel).cpu()
                host_tables.append(a.view(torch.int16).numpy().view(np.uint16) if w.dtype == gen.BF16
                                   else a.numpy())
                idx[b.tbl_off[k]:b.tbl_off[k + 1]] = np.searchsorted(u, b.indices_of(k))
            sample = "whole steps of workload %d on the touched rows only (compacted tables)" % config
        host_state = [np.zeros(t.shape, dtype=np.float32) for t in host_tables] if adagrad else None
        dRh = (b.dR * np.float32(DR_SCALE)).astype(np.float32)

        def cpu_steps(seconds, max_steps):
            nsteps, t_cpu = 0, 0.0
            while t_cpu < seconds and nsteps < max_steps:
                c0 = time.perf_counter()
                S = oracle.emb_bag_fwd(host_tables, w.dtype, idx, b.offsets, b.tbl_off)
                Th = np.concatenate([b.x[:, None, :], S.astype(np.float32)], axis=1)
                oracle.interact_dot_fwd(Th)
                dTh = oracle.interact_dot_bwd(Th, dRh)
                dSh = np.ascontiguousarray(dTh[:, 1:, :], dtype=np.float32)
                if adagrad:
                    oracle.emb_bag_bwd_adagrad(host_tables, host_state, w.dtype, idx, b.offsets, b.tbl_off, dSh, lr, eps)
                else:
                    oracle.emb_bag_bwd_sgd(host_tables, w.dtype, idx, b.offsets, b.tbl_off, dSh, lr)
                t_cpu += time.perf_counter() - c0
                nsteps += 1
            return nsteps, t_cpu

        threads = oracle.get_threads()
        nsteps, t_cpu = cpu_steps(args.cpu_seconds, 1000)
        out["cpu_baseline"] = {"value": round(b.nnz * nsteps / t_cpu, 1), "unit": "lookups/s",
                               "cores": threads, "kind": "oracle",
                               "sample": "%d %s, %.1f s" % (nsteps, sample, t_cpu)}
        oracle.set_threads(1)
        n1, t1 = cpu_steps(min(4.0, args.cpu_seconds / 3), 3)
        oracle.set_threads(threads)
        out["cpu_baseline"]["single_thread"] = {"value": round(b.nnz * n1 / t1, 1), "unit": "lookups/s", "cores": 1,
                                                "sample": "%d of the same steps, %.1f s" % (n1, t1)}
    torch.cuda.synchronize()
    for ev in all_events:
        hip.hipEventDestroy(ev)
    return out


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "re-run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_1906_00091_amd as hot  # noqa: F401  (fails loudly when the library is missing)
    from paper_1906_00091_amd import ceilings

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.ceilings:
        print(json.dumps({"board_ceilings": measure_ceilings(torch, ceilings), "unit": "GB/s",
                          "what": "bytes read + bytes written per second by the plain memory kernels of "
                                  "libdlrm_ceilings: 4 GiB streamed; 1.5 GB of distinct random rows of a 2 GiB table, "
                                  "four rows in flight per lane group", "nominal_hbm_peak": HBM_PEAK_GBPS}))
        return
    # what this board sustains for plain access patterns (a few seconds, 8 GiB), before the workloads
    ceil = None if args.no_cpu_baseline else measure_ceilings(torch, ceilings)
    custom = free_form_workload(args) is not None
    config = 0 if custom else (args.config if args.config else 3)
    out = run_workload(args, config, args.steps, args.warmup, True, ceil)
    if ceil is not None:
        out["board_ceilings"] = dict(ceil, unit="GB/s", note="plain memory kernels (libdlrm_ceilings) on this board: "
                                     "4 GiB streamed; 1.5 GB of distinct random rows of a 2 GiB table")
    if not args.config and not custom and not args.no_extra and not args.graph and not args.locality > 0:
        keep = ("steps", "warmup", "ms_per_step", "value", "unit", "samples_per_s", "dtype", "ms_per_step_chunks",
                "ms_per_step_same_batch", "emb_fwd_bwd", "emb_fwd_bwd_prepared", "emb_fwd_bwd_prepared_pair", "stage_ms", "stage_ms_median",
                "emb_interact_fwd_ms", "emb_interact_bwd_ms", "emb_bag_bwd_prepared_ms", "stage_algorithmic_GBps", "state_after_run", "roofline")
        per = {}
        for cfg, nsteps in ((4, 100), (5, 30)):
            import gc
            gc.collect()
            torch.cuda.empty_cache()
            nsteps = args.extra_steps or nsteps
            r = run_workload(args, cfg, nsteps, min(args.warmup, 10), False, ceil)
            rec = {k: r[k] for k in keep}
            rec["config"] = {k: r["config"][k] for k in ("tables", "batch", "dim", "rows_total", "lookups_per_step",
                                                         "unique_rows_per_step", "distinct_batches", "forward",
                                                         "grouping", "backward_tail")}
            per[r["config"]["workload"]] = rec
        out["per_workload"] = per
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
