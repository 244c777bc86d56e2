#!/usr/bin/env python3
"""Benchmark of the ROBE-Z hot path on one MI355X.

One "step" is one pass of the whole path over one synthetic batch that is
already resident in HBM: forward gather (+ bag-sum), backward scatter-add and
the Adagrad update, as far as the workload has those phases.  The default
workload is the beyond-LLC multi-hot configuration (1 GB array, d = 128,
Z = 32), the one the target statement is quoted on.

Prints ONE JSON line.  `value` is token lookups per second over whole steps.
`phases` gives forward-only, forward+backward and whole-step rates from
per-kernel HIP-event times taken inside the same timed region; `roofline`
describes the kernel that takes the most time; `cpu_baseline` is the CPU
oracle timed on a bounded sample of the same workload on this machine's host
cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="multihot",
                    help="multihot | training | inference | sweep_z{1,8,32,128} | kaggle_z{1,2,4,8,16} | mixed_dims | inference_bf16 | multihot_fwd_bf16 | tiny")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch (0: as defined)")
    ap.add_argument("--m", type=int, default=0, help="override the array length in floats (0: as defined)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--reproducible", action="store_true",
                    help="time the step with robe_options_t::reproducible set: no float atomics, canonical addition order")
    ap.add_argument("--unfused", action="store_true",
                    help="time robe_backward and robe_adagrad_update as separate calls inside the step "
                         "(default: the fused robe_backward_adagrad; the separate calls are then timed beside it)")
    ap.add_argument("--step-only", action="store_true",
                    help="time the steps only: neither the separate calls beside the fused step nor the "
                         "PCIe-inclusive legs (keeps a profile of the run down to the step's own kernels)")
    ap.add_argument("--graph", action="store_true",
                    help="capture the step (one per id batch) into a HIP graph and time replays beside the eager steps")
    ap.add_argument("--cpu-seconds", type=float, default=6.0, help="target oracle time per phase")
    ap.add_argument("--id-batches", type=int, default=2, help="distinct id batches rotated across steps")
    ap.add_argument("--opt", action="append", default=[], metavar="FIELD=VALUE",
                    help="set a field of the robe_options_t passed to every call (e.g. --opt backward_route=2)")
    ap.add_argument("--copy-calib-mb", type=int, default=0,
                    help="before the warm-up, run one plain device copy of this many MiB: a dispatch of known "
                         "size that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters in a --pmc run")
    return ap.parse_args()


def algorithmic_bytes(w, rows, tokens, touched):
    """Bytes the method itself must move per launch (d floats per vector, 8-byte ids)."""
    if w.array_dtype == "bf16":    # forward only: 2-byte array elements, float32 output
        bags = w.bag_mean is not None
        fwd = tokens * (2 * w.d + 8) + rows * 4 * w.d + (rows + 1) * 8 * bags
        return {"fwd": fwd, "bwd": 0, "adagrad": 0, "sgd": 0, "bwd_adagrad": 0}
    if w.dims is not None:    # single-hot, one vector of dims[f] floats per (sample, table)
        D, F = sum(w.dims), w.n_features
        fwd = w.batch * (8 * D + 8 * F)
        bwd = w.batch * (12 * D + 8 * F)
        return {"fwd": fwd, "bwd": bwd, "adagrad": touched * 24, "sgd": touched * 16, "bwd_adagrad": bwd + touched * 24}
    vec = 4 * w.d
    bags = w.bag_mean is not None
    fwd = tokens * (vec + 8) + rows * vec + (rows + 1) * 8 * bags
    bwd = rows * vec + tokens * (2 * vec + 8) + (rows + 1) * 8 * bags
    ada = touched * 24          # read g, s, M; write s, M, g = 0
    sgd = touched * 16          # read g, M; write M, g = 0
    return {"fwd": fwd, "bwd": bwd, "adagrad": ada, "sgd": sgd, "bwd_adagrad": bwd + ada}


def kernel_sources_hash():
    """Identifies the kernels a profile was taken with: a hash over the HIP sources and the header."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2108_02191_amd", "csrc")
    for path in sorted(os.path.join(csrc, f) for f in os.listdir(csrc)) + [os.path.join(ROOT, "include", "robe.h")]:
        h.update(open(path, "rb").read())
    return h.hexdigest()[:16]


def profile_traffic(workload, unfused):
    """HBM-side bytes per launch from the committed rocprofv3 counter summary of this workload.

    profiles/<workload>_step.md (the default step) and profiles/<workload>_step_separate_calls.md
    (--unfused) carry a line `sources <hash>` (the kernel sources the profile was taken with), lines
    `traffic <phase> <bytes>` per entry-point call and `traffic_kernel <kernel> <bytes>` per launch
    (FETCH_SIZE and WRITE_SIZE of separate --pmc runs of this same script, scaled by the calibration
    copy).  A profile taken with other sources says nothing about these kernels: then nothing is returned."""
    name = workload + ("_step_separate_calls.md" if unfused else "_step.md")
    out = {"phase": {}, "kernel": {}, "kernel_us": {}}
    try:
        lines = open(os.path.join(ROOT, "profiles", name)).read().splitlines()
    except OSError:
        return None
    stamp = [l.split()[1] for l in lines if l.startswith("sources ") and len(l.split()) == 2]
    if not stamp or stamp[0] != kernel_sources_hash():
        return None
    for line in lines:
        parts = line.split()
        if len(parts) == 3 and parts[0] == "traffic":
            out["phase"][parts[1]] = int(parts[2])
        elif len(parts) == 3 and parts[0] == "traffic_kernel":
            out["kernel"][parts[1]] = int(parts[2])
        elif len(parts) == 3 and parts[0] == "duration_us":
            out["kernel_us"][parts[1]] = float(parts[2])
    return out


def token_statistics(w, ids, off):
    """Distinct tokens of a batch, and how many of them occur once (host arithmetic on the inputs)."""
    import numpy as np
    F = w.n_features
    if off is None:
        feat = np.tile(np.arange(F, dtype=np.int64), w.batch)
        flat = ids.ravel()
    else:
        feat = np.repeat(np.arange(w.rows, dtype=np.int64) % F, np.diff(off))
        flat = ids
    key = flat.astype(np.uint64) * np.uint64(64) + feat.astype(np.uint64)
    _, counts = np.unique(key, return_counts=True)
    return int(counts.size), int((counts == 1).sum())


def cpu_baseline(w, M, ids, off, G, target_s):
    """The oracle, as it stands, on a bounded sample: the first `bs` samples of the batch."""
    import numpy as np
    import oracle
    H = oracle.init_hash(w.hash_seed, w.m, w.d, w.Z, w.use_sign)
    threads = max(1, oracle.max_threads())      # every host core the OpenMP runtime offers; the count is reported
    F = w.n_features
    if w.dims is not None or w.array_dtype == "bf16":
        threads = 1             # the oracle's mixed-dimension and bf16 loops are sequential
    Mq = oracle.to_bf16(M) if w.array_dtype == "bf16" else None

    def sub(bs):
        rows = bs * F
        if off is None:
            return ids[:bs], None, G[:bs], rows
        o = off[:rows + 1]
        return ids[:int(o[-1])], o, G[:bs], int(o[-1])

    def run(bs):
        i_, o_, g_, ntok = sub(bs)
        t0 = time.perf_counter()
        if w.array_dtype == "bf16":
            oracle.forward_bf16(H, Mq, i_, o_, bs, F)
        elif w.dims is not None:
            oracle.forward_mixed(H, w.dims, M, i_, o_, bs)
        else:
            oracle.forward(H, M, i_, o_, bs, F, threads=threads)
        t1 = time.perf_counter()
        tb = 0.0
        if "bwd" in w.phases:
            if w.dims is not None:
                oracle.backward_mixed(H, w.dims, g_, i_, o_, bs)
            else:
                oracle.backward(H, g_, i_, o_, bs, F, threads=threads, want_abs=False)
            tb = time.perf_counter() - t1
        return ntok, t1 - t0, tb

    # size the sample from a probe of 1/8 of the batch so that each phase takes about target_s seconds
    probe = max(1, min(w.batch, w.batch // 8))
    ntok, tf, tb = run(probe)
    per_sample = max(tf, tb) / probe
    bs = int(max(probe, min(w.batch, target_s / max(per_sample, 1e-9))))
    ntok, tf, tb = run(bs)
    ta = 0.0
    if "adagrad" in w.phases or "sgd" in w.phases:
        g = np.zeros(w.m, dtype=np.float32)
        g[::3] = 1.0
        Mc, s = M.copy(), np.zeros(w.m, dtype=np.float32)
        t0 = time.perf_counter()
        if "adagrad" in w.phases:
            oracle.adagrad(Mc, s, g, w.lr, w.eps, threads=threads)
        else:
            oracle.sgd(Mc, g, w.lr, threads=threads)
        ta = time.perf_counter() - t0
    return {"sample_tokens": ntok, "sample_batch": bs, "t_fwd": tf, "t_bwd": tb, "t_adagrad_dense_full_m": ta,
            "threads": threads}


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py measures one GPU only (got --gpus {args.gpus}): the ROBE-Z path here has no "
              "multi-GPU part; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads
    import paper_2108_02191_amd as robe

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    robe.lib()  # fail loudly if the HIP library is not built
    dev = "cuda:0"
    torch.cuda.set_device(0)

    w = workloads.get(args.workload)
    if args.batch:
        w = w.scaled(batch=args.batch)
    if args.m:
        w = w.scaled(m=args.m)
    B, F = w.batch, w.n_features
    rows = B * F
    do_bwd = "bwd" in w.phases
    do_ada = "adagrad" in w.phases
    do_sgd = "sgd" in w.phases

    t_gen = time.perf_counter()
    M = workloads.make_array(w.m, 0)
    batches = [workloads.make_indices(w, 1 + k) for k in range(max(1, args.id_batches))]
    G = workloads.make_grad_out(w, 2)
    t_gen = time.perf_counter() - t_gen
    tokens = [int(i.size) for i, _ in batches]

    h = robe.robe_init_hash(w.hash_seed, w.m, w.d, w.Z, w.use_sign)
    Md = torch.from_numpy(M).to(dev)
    bf16 = w.array_dtype == "bf16"
    if bf16:
        if do_bwd:
            print("a bf16 array is forward-only", file=sys.stderr)
            sys.exit(2)
        Mb = robe.robe_array_to_bf16(Md)
        del Md
        Md = None
    dev_batches = [(torch.from_numpy(i).to(dev), None if o is None else torch.from_numpy(o).to(dev)) for i, o in batches]
    Gd = torch.from_numpy(G).to(dev)
    mixed = w.dims is not None
    out = torch.empty((B, sum(w.dims)) if mixed else (B, F, w.d), dtype=torch.float32, device=dev)
    ga = torch.zeros(w.m, dtype=torch.float32, device=dev) if do_bwd else None
    st = torch.zeros(w.m, dtype=torch.float32, device=dev) if do_ada else None
    fields = {k: int(v) for k, v in (kv.split("=", 1) for kv in args.opt)}
    if args.reproducible:
        fields["reproducible"] = 1
    opt = robe.options(**fields) if fields else None
    if do_bwd and w.dims is not None:
        ws_bytes = max(robe.robe_mixed_workspace_bytes(h, w.dims, B, n, opt) for n in tokens)
    else:
        ws_bytes = max(robe.robe_workspace_bytes(h, B, F, n, opt) for n in tokens) if do_bwd else 0
    fused = do_ada and not args.unfused
    fws_bytes = max(robe.robe_fused_workspace_bytes(h, B, F, n, opt) for n in tokens) if fused else 0
    ws = torch.empty(max(ws_bytes, fws_bytes, 1), dtype=torch.uint8, device=dev) if max(ws_bytes, fws_bytes) else None

    stream = torch.cuda.current_stream()

    def step(k, ev=None, opt=opt):
        idd, offd = dev_batches[k % len(dev_batches)]
        if ev:
            ev[0].record(stream)
        if mixed:
            robe.robe_forward_mixed(h, w.dims, Md, idd, offd, B, out=out, options=opt)
        elif bf16:
            robe.robe_forward_bf16(h, Mb, idd, offd, B, F, out=out, options=opt)
        else:
            robe.robe_forward(h, Md, idd, offd, B, F, out=out, options=opt)
        if ev:
            ev[1].record(stream)
        if mixed:
            robe.robe_backward_mixed(h, w.dims, Gd, idd, offd, B, ga, workspace=ws, options=opt)
            if ev:
                ev[2].record(stream)
            ga.zero_()
            if ev:
                ev[3].record(stream)
        elif fused:
            robe.robe_backward_adagrad(h, Gd, idd, offd, B, F, Md, st, w.lr, w.eps, workspace=ws, options=opt)
            if ev:
                ev[3].record(stream)
        elif do_bwd:
            robe.robe_backward(h, Gd, idd, offd, B, F, ga, workspace=ws, options=opt)
            if ev:
                ev[2].record(stream)
            if do_ada:
                robe.robe_adagrad_update(h, Md, st, ga, w.lr, w.eps)
            elif do_sgd:
                robe.robe_sgd_update(h, Md, ga, w.lr)
            else:
                ga.zero_()          # a training loop clears the gradient it has consumed
            if ev:
                ev[3].record(stream)

    # touched slots per step (for the Adagrad algorithmic bytes): one untimed backward
    touched = 0
    if do_bwd:
        idd, offd = dev_batches[0]
        if mixed:
            robe.robe_backward_mixed(h, w.dims, Gd, idd, offd, B, ga, workspace=ws, options=opt)
        else:
            robe.robe_backward(h, Gd, idd, offd, B, F, ga, workspace=ws, options=opt)
        touched = int((ga != 0).sum().item())
        ga.zero_()

    if args.copy_calib_mb > 0:
        n = args.copy_calib_mb * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)              # reads and writes copy_calib_mb MiB each
        torch.cuda.synchronize()
        del src, dst

    # Which kernel inside the backward call to time on its own: the library records two events of ours
    # around one kernel of the sorted routes (options probe_*).  The per-region reduce kernel if the
    # call launches it, else the kernel that combines repeated tokens, else none (direct scatter).
    def probe_options(kernel):
        pb, pe = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        pb.record(stream)
        pe.record(stream)            # (recording creates the handles)
        o = robe.options(**fields, probe_kernel=kernel, probe_begin=pb.cuda_event, probe_end=pe.cuda_event)
        return o, pb, pe

    probe_kernel = robe.PROBE_NONE
    if do_bwd and not mixed:
        for cand in (robe.PROBE_REDUCE, robe.PROBE_COMBINE):
            o, pb, pe = probe_options(cand)
            mark = torch.cuda.Event(enable_timing=True)
            mark.record(stream)
            step(0, opt=o)
            torch.cuda.synchronize()
            if mark.elapsed_time(pb) > 0 and pb.elapsed_time(pe) > 0:     # recorded inside that step
                probe_kernel = cand
                break

    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()

    graph_ms = None
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for k in range(len(dev_batches)):
                step(k)
        torch.cuda.synchronize()
        per_replay = len(dev_batches)
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        n_rep = max(1, args.steps // per_replay)
        t1 = time.perf_counter()
        for _ in range(n_rep):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = 1e3 * (time.perf_counter() - t1) / (n_rep * per_replay)

    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    probes = [probe_options(probe_kernel) if probe_kernel else (opt, None, None) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(k, events[k], opt=probes[k][0])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    probe_ms = [pb.elapsed_time(pe) for _, pb, pe in probes if pb is not None]

    ms_per_step = 1e3 * elapsed / args.steps
    k_ms = {"fwd": [], "bwd": [], "adagrad": [], "sgd": [], "bwd_adagrad": []}
    for ev in events:
        k_ms["fwd"].append(ev[0].elapsed_time(ev[1]))
        if fused:
            k_ms["bwd_adagrad"].append(ev[1].elapsed_time(ev[3]))
        elif do_bwd:
            k_ms["bwd"].append(ev[1].elapsed_time(ev[2]))
            if do_ada:
                k_ms["adagrad"].append(ev[2].elapsed_time(ev[3]))
            if do_sgd:
                k_ms["sgd"].append(ev[2].elapsed_time(ev[3]))
    if fused and not args.step_only:
        # the two separate entry points, timed beside the fused step (not part of the timed steps)
        for k in range(3 + 5):
            idd, offd = dev_batches[k % len(dev_batches)]
            e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            e[0].record(stream)
            robe.robe_backward(h, Gd, idd, offd, B, F, ga, workspace=ws, options=opt)
            e[1].record(stream)
            robe.robe_adagrad_update(h, Md, st, ga, w.lr, w.eps)
            e[2].record(stream)
            torch.cuda.synchronize()
            if k >= 3:
                k_ms["bwd"].append(e[0].elapsed_time(e[1]))
                k_ms["adagrad"].append(e[1].elapsed_time(e[2]))
    mixed_fused = None
    if mixed and do_bwd and not args.step_only:
        # backward + Adagrad in one call over the tables of mixed dimensions, timed beside the step
        # (the step itself stays forward + backward, so that its line compares with earlier ones)
        st_m = torch.zeros(w.m, dtype=torch.float32, device=dev)
        fb = max(robe.robe_fused_mixed_workspace_bytes(h, w.dims, B, n, opt) for n in tokens)
        fws = torch.empty(max(fb, 1), dtype=torch.uint8, device=dev)
        ms = []
        for k in range(3 + 5):
            idd, offd = dev_batches[k % len(dev_batches)]
            e = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            e[0].record(stream)
            robe.robe_backward_adagrad_mixed(h, w.dims, Gd, idd, offd, B, Md, st_m, 0.01, 1e-8, workspace=fws, options=opt)
            e[1].record(stream)
            torch.cuda.synchronize()
            if k >= 3:
                ms.append(e[0].elapsed_time(e[1]))
        mixed_fused = {"entry_point": "robe_backward_adagrad_mixed", "ms": round(sum(ms) / len(ms), 4), "workspace_bytes": fb}
        del st_m, fws
    # The same step with the ids (and CSR offsets) starting in pinned host memory, as the paper times
    # its inference runs (Section 5.4: the batch is sent from RAM to the GPU inside the timed region).
    # Reported beside the headline, never as `value`.
    pinned = [(torch.from_numpy(i).pin_memory(), None if o is None else torch.from_numpy(o).pin_memory())
              for i, o in batches]
    id_bytes = sum(i.numel() * 8 + (0 if o is None else o.numel() * 8) for i, o in pinned) / len(pinned)

    def h2d_step(k):
        hi, ho = pinned[k % len(pinned)]
        di, do_ = dev_batches[k % len(dev_batches)]
        di.copy_(hi, non_blocking=True)
        if ho is not None:
            do_.copy_(ho, non_blocking=True)
        step(k)

    n_h2d = 0 if args.step_only else max(2, min(args.steps, 10))
    for k in range(min(2, n_h2d)):
        h2d_step(k)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for k in range(n_h2d):
        h2d_step(k)
    torch.cuda.synchronize()
    h2d_ms = 1e3 * (time.perf_counter() - t1) / max(n_h2d, 1)

    # The same again with the copy of batch k+1 on a second stream while batch k computes (two device
    # buffers per input, events in both directions).
    copy_stream = torch.cuda.Stream()
    ready = [torch.cuda.Event() for _ in dev_batches]      # batch buffer b holds fresh ids
    drained = [torch.cuda.Event() for _ in dev_batches]    # the step that read buffer b is done
    n_buf = len(dev_batches)

    def enqueue_copy(k):
        b = k % n_buf
        hi, ho = pinned[k % len(pinned)]
        di, do_ = dev_batches[b]
        with torch.cuda.stream(copy_stream):
            copy_stream.wait_event(drained[b])
            di.copy_(hi, non_blocking=True)
            if ho is not None:
                do_.copy_(ho, non_blocking=True)
            ready[b].record(copy_stream)

    h2d_overlap_ms = None
    if n_buf >= 2 and n_h2d:
        for b in range(n_buf):
            drained[b].record(stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        enqueue_copy(0)
        for k in range(n_h2d):
            if k + 1 < n_h2d:
                enqueue_copy(k + 1)
            stream.wait_event(ready[k % n_buf])
            step(k)
            drained[k % n_buf].record(stream)
        torch.cuda.synchronize()
        h2d_overlap_ms = 1e3 * (time.perf_counter() - t1) / n_h2d
    del pinned

    # what this machine's HBM delivers to the simplest streaming kernel: a 1 GiB device-to-device copy
    src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    c_ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for _ in range(2):
        dst.copy_(src)
    c_ev[0].record(stream)
    for _ in range(5):
        dst.copy_(src)
    c_ev[1].record(stream)
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * src.numel() * 4 / (c_ev[0].elapsed_time(c_ev[1]) * 1e-3) / 1e9
    del src, dst
    avg = {k: (sum(v) / len(v) if v else 0.0) for k, v in k_ms.items()}
    tok = sum(tokens[k % len(tokens)] for k in range(args.steps)) / args.steps
    alg = algorithmic_bytes(w, rows, tok, touched)

    def rate(ms):
        return tok / (ms * 1e-3) if ms > 0 else None

    kernels = {}
    for name in ("fwd", "bwd", "adagrad", "sgd", "bwd_adagrad"):
        if avg[name] > 0:
            gbs = alg[name] / (avg[name] * 1e-3) / 1e9
            kernels[name] = {"ms": round(avg[name], 4), "ms_median": round(float(np.median(k_ms[name])), 4),
                             "ms_min": round(min(k_ms[name]), 4), "algorithmic_GB": round(alg[name] / 1e9, 4),
                             "achieved_GBps": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                             "frac_of_device_copy": round(gbs / copy_gbs, 4)}
    in_step = [n for n in kernels if not (fused and n in ("bwd", "adagrad"))]
    phases = {"fwd": {"ms": round(avg["fwd"], 4), "lookups_per_s": rate(avg["fwd"])}}
    if do_bwd and avg["bwd"] > 0:
        phases["fwd_bwd"] = {"ms": round(avg["fwd"] + avg["bwd"], 4), "lookups_per_s": rate(avg["fwd"] + avg["bwd"])}
    if fused:
        t_all = avg["fwd"] + avg["bwd_adagrad"]
        phases["fwd_bwd_adagrad"] = {"ms": round(t_all, 4), "lookups_per_s": rate(t_all),
                                      "how": "robe_forward + fused robe_backward_adagrad"}
        if avg["bwd"] > 0:
            t_sep = avg["fwd"] + avg["bwd"] + avg["adagrad"]
            phases["fwd_bwd_adagrad_separate_calls"] = {"ms": round(t_sep, 4), "lookups_per_s": rate(t_sep)}
    elif do_ada or do_sgd:
        rule = "adagrad" if do_ada else "sgd"
        t_all = avg["fwd"] + avg["bwd"] + avg[rule]
        phases["fwd_bwd_" + rule] = {"ms": round(t_all, 4), "lookups_per_s": rate(t_all)}
    total_alg = sum(alg[n] for n in in_step)

    # ---- what was measured, per entry-point call and for the single kernel that takes the most time ----
    # Per call, three byte counts: `algorithmic` prices every token at the per-unit figures of the
    # workload statement (forward: a read of its d slots; backward: a read and a write of them; 24 bytes
    # per touched slot for Adagrad), whether or not the implementation moves them; `compulsory` is what
    # any implementation of the fused call must move (every gradient row, id and offset once; array and
    # state of the touched slots read and written once); `traffic` is what rocprofv3 counted at the
    # L2 <-> fabric boundary (committed profile of these same kernel sources; absent otherwise).
    prof = profile_traffic(w.name, args.unfused) if not (args.batch or args.m or fields) else None
    distinct, singles = token_statistics(w, *batches[0])
    vec = 4 * w.d
    id_bytes_dev = tok * 8 + ((rows + 1) * 8 if w.bag_mean is not None else 0)
    compulsory = {"fwd": alg["fwd"],
                  "bwd": rows * vec + id_bytes_dev + touched * 8,
                  "adagrad": touched * 24, "sgd": touched * 16,
                  "bwd_adagrad": rows * vec + id_bytes_dev + touched * 16}
    for name, kk in kernels.items():
        if not mixed and not bf16:
            kk["compulsory_GB"] = round(compulsory[name] / 1e9, 4)
        t = prof["phase"].get(name) if prof else None
        kk["traffic_GB"] = None if t is None else round(t / 1e9, 4)
        kk["frac_physical"] = None if t is None else round(t / (kk["ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)

    # Single kernels timed live with events on the launch stream: the forward kernel (the whole
    # robe_forward call), the optimizer kernel (the whole update call), and the kernel the library
    # bracketed with the probe events inside the backward call.  Algorithmic bytes per launch, from the
    # units that launch processes: the reduce kernel reads one summed gradient row per distinct token
    # and reads and writes array and state (fused) or the gradient array (robe_backward) of every
    # touched slot; the combine kernel reads the gradient row of every token that occurs more than once
    # and writes one row per such distinct token (region route), or reads every token's row and reads
    # and writes the slots of every distinct token (atomic route).
    single = {}
    if not mixed:
        single["bag_kernel / single_hot_kernel (robe_forward%s)" % ("_bf16" if bf16 else "")] = (avg["fwd"], alg["fwd"], "fwd_kernel")
    for rule in ("adagrad", "sgd"):
        if avg[rule] > 0 and not fused:      # (beside a fused step the update call is timed for comparison only)
            single["update_kernel (robe_%s_update)" % rule] = (avg[rule], alg[rule], "update_kernel")
    if probe_ms:
        pms = sum(probe_ms) / len(probe_ms)
        multi = distinct - singles
        if probe_kernel == robe.PROBE_REDUCE:
            per_slot = 16 if fused else 8
            single["region_reduce_kernel (inside robe_backward%s)" % ("_adagrad" if fused else "")] = (
                pms, distinct * vec + touched * per_slot, "region_reduce_kernel")
        elif fws_bytes or ws_bytes:
            single["combine_scatter_kernel (inside robe_backward)"] = (pms, tok * vec + distinct * 2 * vec, "combine_scatter_kernel")
    roof = None
    if single:
        dom = max(single, key=lambda k: single[k][0])
        ms_k, bytes_k, tag = single[dom]
        t = prof["kernel"].get(tag) if prof else None
        roof = {"kernel": dom, "bound": "hbm", "achieved": round(bytes_k / (ms_k * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(bytes_k / (ms_k * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                "traffic": t, "frac_physical": None if t is None else round(t / (ms_k * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                "ms": round(ms_k, 4), "algorithmic_bytes": int(bytes_k),
                "ms_rocprofv3": None if not prof or tag not in prof["kernel_us"] else round(prof["kernel_us"][tag] / 1e3, 4),
                "units": {"tokens": tok, "distinct_tokens": distinct, "tokens_occurring_once": singles, "rows": rows,
                          "touched_slots": touched},
                "all_single_kernels_ms": {k: round(v[0], 4) for k, v in single.items()},
                "profile": "profiles/%s_step%s.md" % (w.name, "_separate_calls" if args.unfused else "") if prof else None,
                "kernel_sources": kernel_sources_hash()}
    else:       # tables of mixed dimensions: several launches per call, the call is the unit
        dom = max(in_step, key=lambda n: kernels[n]["ms"])
        roof = {"kernel": ("robe_backward_mixed (whole call: token sort, then one combine kernel over all tables)" if dom == "bwd"
                           else "robe_forward_mixed (whole call: one launch per run of equal dimensions)"),
                "bound": "hbm", "achieved": kernels[dom]["achieved_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": kernels[dom]["frac_of_hbm_peak"], "traffic": prof["phase"].get(dom) if prof else None,
                "ms": kernels[dom]["ms"], "kernel_sources": kernel_sources_hash()}
    result = {
        "metric": "ROBE lookups/sec, whole step (fwd%s%s), d=%d, Z=%d" % (
            "+bwd" if do_bwd else "", "+Adagrad" if do_ada else ("+SGD" if do_sgd else ""), w.d, w.Z)
                  + (" [backward and Adagrad fused]" if fused else ""),
        "value": tok / (ms_per_step * 1e-3),
        "unit": "lookups/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 (array stored as bf16)" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": w.name, "m": w.m, "array_bytes": 4 * w.m, "d": list(w.dims) if w.dims else w.d, "Z": w.Z, "batch": B,
                   "n_features": F, "rows": rows, "tokens_per_step": tok, "bag_mean": w.bag_mean,
                   "ids": f"{w.id_dist}({w.zipf_alpha})" if w.id_dist == "zipf" else w.id_dist,
                   "use_sign": w.use_sign, "phases": w.phases, "id_batches": len(batches),
                   "touched_slots": touched, "reproducible_mode": bool(args.reproducible), "options": fields},
        "effective_GBps_whole_step": total_alg / (ms_per_step * 1e-3) / 1e9,
        "effective_frac_of_hbm_peak": total_alg / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "device_copy_GBps": round(copy_gbs, 1),
        "effective_frac_of_device_copy": total_alg / (ms_per_step * 1e-3) / 1e9 / copy_gbs,
        "phases": phases,
        "kernels": kernels,
        "roofline": roof,
        "pcie_inclusive": None if not n_h2d else {
                           "ms_per_step": round(h2d_ms, 4), "lookups_per_s": tok / (h2d_ms * 1e-3),
                           "host_to_device_bytes_per_step": int(id_bytes), "steps": n_h2d,
                           "what": "ids and CSR offsets copied from pinned host memory inside every step",
                           "ms_per_step_copy_overlapped": None if h2d_overlap_ms is None else round(h2d_overlap_ms, 4),
                           "lookups_per_s_copy_overlapped": None if h2d_overlap_ms is None else tok / (h2d_overlap_ms * 1e-3)},
        "mixed_fused": mixed_fused,
        "graph_replay": None if graph_ms is None else {
            "ms_per_step": round(graph_ms, 5), "lookups_per_s": tok / (graph_ms * 1e-3),
            "what": "the same step captured once per id batch into one HIP graph; value stays the eager figure"},
        "input_generation_s": round(t_gen, 1),
    }

    if not args.no_cpu_baseline:
        idsh, offh = batches[0]
        cb = cpu_baseline(w, M, idsh, offh, G, args.cpu_seconds)
        scale = tok / max(cb["sample_tokens"], 1)
        t_full = (cb["t_fwd"] + cb["t_bwd"]) * scale + cb["t_adagrad_dense_full_m"]
        result["cpu_baseline"] = {
            "value": tok / t_full, "unit": "lookups/s", "cores": cb["threads"], "kind": "oracle",
            "sample": ("first %d of %d batch samples (%d tokens): oracle fwd %.2f s%s, scaled by tokens; "
                       "%s") % (cb["sample_batch"], B, cb["sample_tokens"], cb["t_fwd"],
                                (", bwd %.2f s" % cb["t_bwd"]) if do_bwd else "",
                                ("dense optimizer sweep over all m slots %.3f s, unscaled" % cb["t_adagrad_dense_full_m"])
                                if (do_ada or do_sgd) else "no optimizer phase"),
            "fwd_lookups_per_s": cb["sample_tokens"] / cb["t_fwd"] if cb["t_fwd"] > 0 else None,
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
