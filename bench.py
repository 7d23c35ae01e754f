#!/usr/bin/env python3
"""Benchmark of the VarDrop training hot path on one MI355X.

One step = vardrop_hash -> vardrop_sample -> (read N') -> vardrop_gather_attn_fwd (= vardrop_gather
+ vardrop_attn_fwd) -> vardrop_attn_bwd over one batch of synthetic windows and tokens that already sit in HBM.  The
selection (hash + sample) of batch i+1 is enqueued before the attention of batch i, on a second stream.
Prints ONE JSON line: steps/s, the roofline figure of the dominant kernel, and the CPU
oracle timed on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload traffic] [--no-cpu-baseline]

`--mode bandwidth` instead measures the steady-state HBM bandwidth of the two streaming kernels
(vardrop_hash, vardrop_gather) over enough distinct batches (>= 1 GiB of input) that the 256 MB
last-level cache cannot serve the reads, and prints ONE JSON line with both figures.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3      # MI355X fp32 vector
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E


def algorithmic_work(w, n):
    """Per launch: kernel name -> (bound, algorithmic bytes or flops).  n = kept tokens N'.

    Bytes are what the method must move once (inputs read once, outputs written once); flops are
    those of the contractions the method defines (2 per multiply-add).  The second evaluation of
    S = Q K^T and dP = dO V^T inside the two-part backward of long selections is not counted as useful work.
    """
    B, N, L, d = w.B, w.N, w.L, w.d
    M = B * n
    es = 2 if w.dtype == "bf16" else 4
    mm = "mfma" if w.dtype == "bf16" else "alu"
    return {
        "hash": ("hbm", 4.0 * B * N * L),
        "sample": ("hbm", 8.0 * N + 4.0 * N + 4.0 * n + 8),
        "gather": ("hbm", 2.0 * M * d * es),
        "scatter": ("hbm", (M + B * N) * d * es),
        "gemm_qkv": (mm, 6.0 * M * d * d),
        "sdpa_fwd": (mm, 4.0 * B * n * n * d),
        "gemm_out": (mm, 2.0 * M * d * d),
        "gemm_do": (mm, 2.0 * M * d * d),
        "sdpa_bwd_dq": (mm, 4.0 * B * n * n * d),
        "sdpa_bwd_dkv": (mm, 6.0 * B * n * n * d),
        "sdpa_bwd_dqkv": (mm, 10.0 * B * n * n * d),
        "gemm_dw": (mm, 8.0 * M * d * d),
        "reduce_dw": ("hbm", 4.0 * 4 * d * d * 2),
        "gemm_dxs": (mm, 6.0 * M * d * d),
        "gemm_dw_dxs": (mm, 14.0 * M * d * d),
        "sdpa_bwd": (mm, 10.0 * B * n * n * d + 2.0 * M * d * d),      # includes dO = dy Wo^T
        "qkv_sdpa_fwd": (mm, 6.0 * M * d * d + 4.0 * B * n * n * d),
        "embed_rows": ("hbm", 4.0 * M * L + float(es) * M * L),
        "gemm_embed": (mm, 2.0 * M * L * d),
        "gemm_dwe": (mm, 2.0 * M * L * d),
    }


BRACKET_EVERY = 8      # launches of the dominant kernel per HIP event pair inside the timed region


def recorded_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed hardware-counter summary, or None when the
    kernels have changed since the counters were taken (the summary records a hash of csrc/)."""
    import glob
    import hashlib
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s.txt" % workload)
    if not os.path.exists(path):
        return None
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2501_14183_amd", "csrc", "*"))):
        h.update(open(f, "rb").read())
    lines = open(path).read().splitlines()
    if not lines or ("csrc=" + h.hexdigest()[:16]) not in lines[0]:
        return None
    for line in lines[1:]:
        value, name = line.split("\t")
        if name == kernel:
            return float(value)
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="traffic")
    ap.add_argument("--batches", type=int, default=4, help="distinct pre-generated batches the steps rotate through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--mode", choices=("steps", "bandwidth", "sweep"), default="steps")
    ap.add_argument("--k", type=int, default=0, help="number of dominant frequencies (default: the workload's)")
    ap.add_argument("--gs", type=int, default=0,
                    help="Eq. 1 as printed: a group keeps min(|G|, gs) members (default 0: the workload's keep ratio instead)")
    ap.add_argument("--dense", action="store_true",
                    help="no dropping: one step = attention forward + backward over all N variate tokens of the batch "
                         "(the selection is the identity, Sec. 3.3 at inference); the comparison point for the speed-up")
    ap.add_argument("--embed", action="store_true",
                    help="the tokens are embedded inside the step from the raw windows, for the kept variates only "
                         "(vardrop_embed_fwd / vardrop_embed_bwd; with --dense for all variates), instead of being "
                         "gathered from a pre-embedded batch")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run five plain 256 MiB device copies (reference for hardware byte counters)")
    return ap.parse_args()


def cpu_baseline(w, x_np, tok_np, W_np, seed):
    """The oracle, as it stands, on a bounded sample: the whole path for the first `nb` windows of one batch."""
    import numpy as np
    from oracle import attention as o_attn
    from oracle import kdfh as o_kdfh
    from oracle import sampling as o_samp
    import workloads as wl

    try:
        import threadpoolctl
        cores = max(int(i.get("num_threads", 1)) for i in threadpoolctl.threadpool_info()) if threadpoolctl.threadpool_info() else 1
    except Exception:
        cores = os.cpu_count() or 1
    t0 = time.perf_counter()
    topk, hsh, _ = o_kdfh.kdfh(x_np, w.k)                                   # the hash needs the full batch
    t1 = time.perf_counter()
    gid, sel, G = o_samp.stratified_sample(hsh, 0, w.ratio[0], w.ratio[1], seed, 0)
    t2 = time.perf_counter()
    # attention cost is linear in the batch: time `nb` windows and scale
    per_window = None
    nb = 1
    while True:
        xs = o_attn.gather(tok_np[:nb], sel)
        dy = wl.make_upstream(w, len(sel))[:nb]
        ta = time.perf_counter()
        y, cache = o_attn.mha_forward(xs, *W_np, w.H)
        o_attn.mha_backward(dy, cache)
        tb = time.perf_counter()
        per_window = (tb - ta) / nb
        if (tb - ta) > 3.0 or nb >= w.B:
            break
        nb = min(w.B, nb * 4)
    step_s = (t1 - t0) + (t2 - t1) + per_window * w.B
    note = ("one batch of the same workload: k-DFH and sampling on all %d windows (%.3f s + %.3f s), "
            "gather + attention fwd/bwd timed on %d of %d windows and scaled linearly (%.3f s per window), N'=%d"
            % (w.B, t1 - t0, t2 - t1, nb, w.B, per_window, len(sel)))
    if nb >= w.B and step_s < 5.0:
        # a whole step is cheap enough: repeat whole steps (new selection each) for about ten seconds
        steps, t_start = 0, time.perf_counter()
        while time.perf_counter() - t_start < 10.0:
            steps += 1
            topk, hsh, _ = o_kdfh.kdfh(x_np, w.k)
            gid, sel, G = o_samp.stratified_sample(hsh, 0, w.ratio[0], w.ratio[1], seed, steps)
            xs = o_attn.gather(tok_np, sel)
            y, cache = o_attn.mha_forward(xs, *W_np, w.H)
            o_attn.mha_backward(wl.make_upstream(w, len(sel)), cache)
        step_s = (time.perf_counter() - t_start) / steps
        note = "%d whole steps of the same workload (all %d windows, a new selection each) in %.1f s" % (
            steps, w.B, step_s * steps)
    return {"value": 1.0 / step_s, "unit": "steps/s", "cores": cores, "kind": "oracle", "sample": note}


def steady_bandwidth(args):
    """Kernel time of vardrop_hash and vardrop_gather over M distinct inputs each (M x bytes >= 1 GiB), launched
    back to back on one stream: per-launch durations from HIP events around every launch (library hook), less
    the cost of an empty event pair, and the wall time of the same loop without events."""
    import numpy as np
    import torch
    import paper_2501_14183_amd as vd
    import workloads as wl

    w = wl.WORKLOADS[args.workload]
    td = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    es = 2 if w.dtype == "bf16" else 4
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)
    ctx = vd.Context(0)
    stream = torch.cuda.current_stream()
    gen = torch.Generator(device=dev)
    gen.manual_seed(1234)

    def empty_pair_us():
        e = [torch.cuda.Event(enable_timing=True) for _ in range(64)]
        for i in range(0, 64, 2):
            e[i].record(stream)
            e[i + 1].record(stream)
        torch.cuda.synchronize()
        return float(np.median([e[i].elapsed_time(e[i + 1]) for i in range(0, 64, 2)])) * 1e3

    def measure(kid, launch, count, reps=3):
        for i in range(count):                       # warm-up pass (also builds the hash's table)
            launch(i)
        torch.cuda.synchronize()
        vd.vardrop_profile_stride(ctx, 1)
        vd.vardrop_profile_select(ctx, kid)
        for _ in range(reps):
            for i in range(count):
                launch(i)
        total_ms, launches = vd.vardrop_profile_read(ctx)
        vd.vardrop_profile_select(ctx, -1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            for i in range(count):
                launch(i)
        torch.cuda.synchronize()
        wall_us = (time.perf_counter() - t0) * 1e6 / (reps * count)
        return total_ms * 1e3 / launches - empty_pair_us(), wall_us, launches

    def report(nbytes, us, wall, n, extra):
        # "GB/s" is the conservative figure: launches back to back, dispatch gaps included.  The event figure
        # subtracts an empty bracket of several microseconds and means little for a kernel shorter than that;
        # rocprofv3 --kernel-trace of this same command gives the kernel's own duration.
        d = dict(extra)
        d.update({"bytes_per_launch": nbytes, "back_to_back_us": wall, "GB/s": nbytes / wall * 1e-3,
                  "frac_of_peak": nbytes / wall * 1e-3 / PEAK_HBM_GBS, "event_bracket_us": us,
                  "GB/s_event_bracket": (nbytes / us * 1e-3) if us >= 10.0 else None, "launches": n})
        return d

    kids = {vd.vardrop_kernel_name(k): k for k in range(64) if vd.vardrop_kernel_name(k)}
    out = {}

    # ---- hash: 4 B N L bytes read per launch
    x_bytes = 4 * w.B * w.N * w.L
    M = -(-(1 << 30) // x_bytes)
    xs = [torch.randn((w.B, w.N, w.L), generator=gen, device=dev) for _ in range(M)]
    topk = torch.empty((w.N, w.k), dtype=torch.int32, device=dev)
    hsh = torch.empty(w.N, dtype=torch.int64, device=dev)
    us, wall, n = measure(kids["hash"], lambda i: vd.vardrop_hash(ctx, xs[i], w.k, out=(topk, hsh), stream=stream.cuda_stream), M)
    out["hash"] = report(x_bytes, us, wall, n, {"distinct_inputs": M})
    del xs

    # ---- gather: 2 B N' d es bytes (read + write) per launch, N' = the workload's mean keep
    n_sel = max(1, int(round(w.N * w.ratio[0] / w.ratio[1] * 1.3)))
    g_bytes = 2 * w.B * n_sel * w.d * es
    M = -(-(1 << 30) // g_bytes)
    tok_bytes = w.B * w.N * w.d * es
    M = min(M, max(4, (64 << 30) // tok_bytes))       # at most 64 GiB of token buffers
    toks = [torch.randn((w.B, w.N, w.d), generator=gen, device=dev).to(td) for _ in range(M)]
    sels = []
    for i in range(M):
        pick = torch.randperm(w.N, generator=gen, device=dev)[:n_sel].sort().values.to(torch.int32)
        sel = torch.zeros(w.N, dtype=torch.int32, device=dev)
        sel[:n_sel] = pick
        sels.append(sel)
    dst = [torch.empty((w.B, n_sel, w.d), dtype=td, device=dev) for _ in range(M)]
    us, wall, n = measure(kids["gather"], lambda i: vd.vardrop_gather(ctx, toks[i], sels[i], n_sel, out=dst[i], stream=stream.cuda_stream), M)
    out["gather"] = report(g_bytes, us, wall, n, {"distinct_inputs": M, "kept_tokens": n_sel})
    print(json.dumps({"metric": "steady-state HBM GB/s of vardrop_hash and vardrop_gather", "unit": "GB/s", "n_gpus": 1,
                      "peak": PEAK_HBM_GBS, "data": "synthetic", "dtype": w.dtype,
                      "config": {"workload": "%s-shaped: B=%d N=%d L=%d k=%d d=%d" % (w.name, w.B, w.N, w.L, w.k, w.d)},
                      "kernels": out}))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path; run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    if args.mode == "bandwidth":
        return steady_bandwidth(args)
    import numpy as np
    import torch
    import paper_2501_14183_amd as vd
    import workloads as wl

    import dataclasses
    w = wl.WORKLOADS[args.workload]
    K_MAX = 5                                           # largest k of the sweep (sizes the top-k buffers)
    if args.k:
        w = dataclasses.replace(w, k=args.k)
    gs_cap = args.gs                                    # > 0: Eq. 1 with this cap and no keep ratio
    td = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)
    ctx = vd.Context(0)

    # ---- synthetic inputs, resident in HBM before anything is timed
    xs_dev, tok_dev, host = [], [], None
    for i in range(args.batches):
        x_np, _ = wl.make_signals(w, seed=i)
        tok_np = wl.make_tokens(w, x_np, seed=i)
        if i == 0:
            host = (x_np, tok_np)
        xs_dev.append(torch.from_numpy(x_np).to(dev))
        tok_dev.append(torch.from_numpy(tok_np).to(dev).to(td))
    W_np = wl.make_weights(w, seed=0)
    W_dev = [torch.from_numpy(m).to(dev).to(td) for m in W_np]
    dy_full = torch.from_numpy(wl.make_upstream(w, w.N, seed=0)).to(dev).to(td).reshape(-1)
    stream = torch.cuda.current_stream()
    seed = 0x5EED
    if args.embed:
        gen = torch.Generator(device=dev)
        gen.manual_seed(4321)
        We_dev = (torch.randn((w.L, w.d), generator=gen, device=dev) / w.L ** 0.5).to(td)
        be_dev = (0.1 * torch.randn(w.d, generator=gen, device=dev)).to(td)
        all_idx = torch.arange(w.N, dtype=torch.int32, device=dev)
    saved = ws = None
    stats = {"n_sel": [], "G": []}

    # The selection of a batch depends on its windows only, not on the model, so it runs LOOK batches
    # ahead of the attention and on a stream of its own (default priority): the small k-DFH and sampling
    # kernels then overlap the attention of earlier batches, and the 8-byte read-back of {N', G}
    # that sizes the attention launch is complete when the host needs it.
    # Cross-stream events on the attention stream cost several microseconds each (a marker packet
    # between two kernels), so the attention stream carries none per step: the outputs of the
    # selection live in a ring of RING buffer sets, and the host never runs more than RING - LOOK - FENCE
    # batches ahead of the attention stream (one event every FENCE steps, waited for FENCE steps
    # later), so a set is never rewritten while a gather may still read it.
    LOOK, FENCE, RING = 2, 8, 32
    pinned = [torch.zeros(2, dtype=torch.int32).pin_memory() for _ in range(RING)]
    events = [torch.cuda.Event() for _ in range(RING)]
    side = torch.cuda.Stream(device=dev)
    main_h, side_h = stream.cuda_stream, side.cuda_stream      # raw handles: the binding then skips torch's stream lookup
    sel_bufs = [(torch.empty((w.N, max(w.k, K_MAX)), dtype=torch.int32, device=dev), torch.empty(w.N, dtype=torch.int64, device=dev),
                 torch.empty(w.N, dtype=torch.int32, device=dev), torch.empty(w.N, dtype=torch.int32, device=dev),
                 torch.empty(2, dtype=torch.int32, device=dev)) for _ in range(RING)]
    fences = {}                                         # step -> event recorded on the attention stream after it

    def select(i):
        if args.dense:
            return
        j = i % RING
        topk, hsh, gid, sel, counts = sel_bufs[j]
        vd.vardrop_hash(ctx, xs_dev[i % args.batches], w.k, out=(topk, hsh), stream=side_h)
        num, den = (1, 1) if gs_cap else w.ratio
        vd.vardrop_sample(ctx, hsh, gs_cap, num, den, seed, i, counts_host=pinned[j], out=(gid, sel, counts),
                          stream=side_h)
        events[j].record(side)

    def attend(i):
        nonlocal saved, ws
        j = i % RING
        tok = tok_dev[i % args.batches]
        if args.dense:
            n_sel, G = w.N, w.N
            count = w.B * n_sel * w.d
            shape = (w.B, n_sel, w.d)
            xs = tok
        else:
            sel = sel_bufs[j][3]
            events[j].synchronize()                # N' of batch i (launched LOOK steps earlier)
            n_sel, G = int(pinned[j][0]), int(pinned[j][1])
            count = w.B * n_sel * w.d
            shape = (w.B, n_sel, w.d)
        if args.embed:
            # tokens of the kept variates (all of them with --dense) straight from the raw windows, then attention
            xs, _ = vd.vardrop_embed_fwd(ctx, xs_dev[i % args.batches], all_idx if args.dense else sel, n_sel, We_dev, be_dev,
                                         saved=esaved, out=xs_buf[:count].view(shape), stream=main_h)
            y, saved = vd.vardrop_attn_fwd(ctx, xs, *W_dev, w.H, saved=saved, out=y_buf[:count].view(shape), stream=main_h)
        elif args.dense:
            y, saved = vd.vardrop_attn_fwd(ctx, xs, *W_dev, w.H, saved=saved, out=y_buf[:count].view(shape), stream=main_h)
        else:
            # gather + forward in one call: for N' <= 128 the forward kernel fetches the kept rows itself
            xs, y, saved = vd.vardrop_gather_attn_fwd(ctx, tok, sel, n_sel, *W_dev, w.H, saved=saved,
                                                      out=(xs_buf[:count].view(shape), y_buf[:count].view(shape)), stream=main_h)
        dy = dy_full[:count].view(shape)
        grads = vd.vardrop_attn_bwd(ctx, dy, xs, *W_dev, w.H, saved, ws=ws, out=(dxs_buf[:count].view(shape), *dW_buf),
                                      stream=main_h)
        if args.embed:
            vd.vardrop_embed_bwd(ctx, grads[0], w.L, esaved, ws=ews, out=dWe_buf, stream=main_h)
        stats["n_sel"].append(n_sel)
        stats["G"].append(G)
        return grads

    def run(first, count):
        """`count` whole steps: every batch gets its selection and its attention inside this call."""
        torch.cuda.synchronize()                   # buffer sets are reused from the start: nothing of an earlier call is left
        fences.clear()
        for i in range(first, min(first + LOOK, first + count)):
            select(i)
        for i in range(first, first + count):
            if (i - first) % FENCE == 0:
                old = fences.pop(i - FENCE, None)
                if old is not None:
                    old.synchronize()              # the attention stream has finished step i - FENCE - 1
                ev = torch.cuda.Event()
                ev.record(stream)
                fences[i] = ev
            if i + LOOK < first + count:
                select(i + LOOK)
            attend(i)

    # size the reusable buffers for the largest selection (never re-allocated inside the timed region)
    lib = vd.load_library()
    code = vd.BF16 if w.dtype == "bf16" else vd.F32
    saved = torch.empty(lib.vardrop_attn_saved_bytes(w.B, w.N, w.d, w.H, code), dtype=torch.uint8, device=dev)
    ws = torch.empty(lib.vardrop_attn_workspace_bytes(w.B, w.N, w.d, w.H, code), dtype=torch.uint8, device=dev)

    if args.embed:
        esaved = torch.empty(lib.vardrop_embed_saved_bytes(w.B, w.N, w.L, code), dtype=torch.uint8, device=dev)
        ews = torch.empty(max(lib.vardrop_embed_workspace_bytes(w.B, w.N, w.L, w.d, code), 256), dtype=torch.uint8, device=dev)
        dWe_buf = (torch.empty((w.L, w.d), dtype=torch.float32, device=dev), torch.empty(w.d, dtype=torch.float32, device=dev))

    # outputs of a step, sized for the largest selection as well (every call writes all of what it returns)
    xs_buf, y_buf, dxs_buf = (torch.empty(w.B * w.N * w.d, dtype=td, device=dev) for _ in range(3))
    dW_buf = [torch.empty((w.d, w.d), dtype=torch.float32, device=dev) for _ in range(4)]

    if args.copy_calibration:
        src = torch.zeros(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.mode == "sweep":
        # Sensitivity of the reduction to k and gs (Sec. 4.4, Eq. 1 as printed) on the synthetic workload:
        # groups, kept tokens, delta = 1 - N'/N and whole-step throughput for every pair.
        table = []
        for k in (2, 3, 4, 5):
            for gs in (1, 2, 3, 5, 8, 10, 15, 20):
                w = dataclasses.replace(w, k=k)
                gs_cap = gs
                run(0, 10)
                torch.cuda.synchronize()
                stats = {"n_sel": [], "G": []}
                t0 = time.perf_counter()
                run(10, 60)
                torch.cuda.synchronize()
                dt = (time.perf_counter() - t0) / 60
                n_mean, g_mean = float(np.mean(stats["n_sel"])), float(np.mean(stats["G"]))
                table.append({"k": k, "gs": gs, "groups": g_mean, "kept": n_mean, "delta": 1.0 - n_mean / w.N,
                              "steps_per_s": 1.0 / dt})
        print(json.dumps({"metric": "reduction ratio delta and train steps/s over k and gs (Eq. 1)", "n_gpus": 1,
                          "data": "synthetic", "dtype": w.dtype,
                          "config": {"workload": "%s-shaped: B=%d N=%d L=%d d=%d H=%d" % (w.name, w.B, w.N, w.L, w.d, w.H)},
                          "table": table}))
        return

    run(0, args.warmup)
    torch.cuda.synchronize()

    # ---- which kernel takes the largest share of a step?  (untimed census, HIP events around one kernel at a time)
    census = {}
    for kid in range(64):
        name = vd.vardrop_kernel_name(kid)
        if name is None:
            break
        vd.vardrop_profile_select(ctx, kid)
        run(0, 8)
        total_ms, launches = vd.vardrop_profile_read(ctx)
        if launches:
            census[name] = (kid, total_ms * 1e3 / 8)            # microseconds per step
    # The step time is set by the attention stream; hashing and sampling of the next batch run beside it
    # on the second stream, so the dominant kernel is the largest one on the attention stream.
    on_critical_path = {k: v for k, v in census.items() if k not in ("hash", "sample")}
    dominant = max(on_critical_path, key=lambda k: on_critical_path[k][1])
    # Only this kernel is bracketed while timing, and only every BRACKET_EVERY-th launch of it: an event
    # pair between two kernels costs the attention stream about 7 us, 8 % of a step at this shape.
    vd.vardrop_profile_stride(ctx, BRACKET_EVERY)
    vd.vardrop_profile_select(ctx, census[dominant][0])
    torch.cuda.synchronize()

    stats = {"n_sel": [], "G": []}
    t0 = time.perf_counter()
    run(args.warmup, args.steps)
    t_host = time.perf_counter()                   # every launch of the timed steps has been issued
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms = (t1 - t0) * 1e3 / args.steps
    host_ms = (t_host - t0) * 1e3 / args.steps
    n_mean = float(np.mean(stats["n_sel"]))

    # ---- roofline of the dominant kernel: algorithmic work per launch / mean launch duration (HIP events)
    total_ms, launches = vd.vardrop_profile_read(ctx)
    vd.vardrop_profile_stride(ctx, 1)
    vd.vardrop_profile_select(ctx, -1)
    bound, work = algorithmic_work(w, n_mean)[dominant]
    # an empty event pair on the same stream measures what the bracket itself adds
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    gaps = []
    for _ in range(50):
        e0.record()
        e1.record()
        e1.synchronize()
        gaps.append(e0.elapsed_time(e1))
    gap_ms = float(np.median(gaps))
    avg_s = max(total_ms / max(launches, 1) - gap_ms, 1e-6) * 1e-3
    if bound == "hbm":
        achieved, peak, unit = work / avg_s / 1e9, PEAK_HBM_GBS, "GB/s"
    else:
        achieved, unit = work / avg_s / 1e12, "TFLOP/s"
        peak = PEAK_BF16_TFLOPS if bound == "mfma" else PEAK_FP32_TFLOPS
    roof = {"kernel": dominant, "bound": bound, "achieved": achieved, "peak": peak, "unit": unit,
            "frac": achieved / peak, "traffic": recorded_traffic(w.name, dominant),
            "avg_launch_us": avg_s * 1e6, "event_pair_overhead_us": gap_ms * 1e3, "launches": launches,
            "bracketed_one_launch_in": BRACKET_EVERY,
            "us_per_step_by_kernel": {k: round(v[1], 2) for k, v in census.items()}}

    if args.dense or args.embed:
        args.no_cpu_baseline = True                 # the oracle leg times the dropping path on pre-embedded tokens
    out = {
        "metric": (("dense (no dropping) variate-attn train steps/s (SDPA fwd/bwd over all N tokens)" if args.dense else
                    "variate-attn train steps/s (kDFH+sample+SDPA fwd/bwd), HBM GB/s, MFMA %peak") +
                   (" + token embedding fwd/bwd inside the step" if args.embed else "")),
        "value": 1e3 / ms, "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "host_issue_ms_per_step": host_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": ("%s-shaped, dense: B=%d N=%d d=%d H=%d, selection = identity" % (w.name, w.B, w.N, w.d, w.H))
                               if args.dense else "%s-shaped: B=%d N=%d L=%d k=%d keep=%d/%d d=%d H=%d" %
                               (w.name, w.B, w.N, w.L, w.k, w.ratio[0], w.ratio[1], w.d, w.H),
                   "k": w.k, "gs": gs_cap if gs_cap else None,
                   "kept_tokens_mean": n_mean, "groups_mean": float(np.mean(stats["G"])),
                   "batches": args.batches},
        "roofline": roof,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, host[0], host[1], W_np, seed)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
