#!/usr/bin/env python3
"""Benchmark of the VarDrop training hot path on one MI355X.

One step = vardrop_hash -> vardrop_sample_dev -> vardrop_gather_attn_fwd_dev (= gather + attention forward) ->
vardrop_attn_bwd_dev over one batch of synthetic windows and tokens that already sit in HBM.  The number of kept
tokens N' stays on the device (the kernels read it there), so a step is a fixed sequence of launches with no host
wait.  The selection (hash + sample) of a batch runs on a second stream beside the attention of earlier batches;
where it runs is chosen by a short untimed trial (--launch auto, see Pipeline).  --launch graph instead records each
step once as a HIP graph and replays it (slower with this runtime: a replay costs the host more than issuing the
launches).  Prints ONE JSON line: steps/s, the roofline figures (the dominant kernel, and all kernels), a second
figure at the paper's own sampling rule, and the CPU oracle timed on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload traffic] [--launch auto|eager|burst|graph] [--no-cpu-baseline]

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
        "embed_fused": (mm, 2.0 * M * L * d),
    }


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
    ap.add_argument("--launch", choices=("auto", "eager", "burst", "graph"), default="auto",
                    help="eager: every call of a step issued from the host, the k-DFH and the sampling each placed behind a "
                         "chosen attention kernel or left free (the best placement in a short untimed trial); burst: the same "
                         "calls with the selections in bursts of four on the second stream (less work for the host: "
                         "better when a step is shorter than the host's time to issue it); auto (default): the fastest "
                         "of all three in the trial; graph: one recorded HIP graph per step")
    ap.add_argument("--no-paper-rule", action="store_true",
                    help="skip the second figure at the paper's own sampling rule (Eq. 1 with Table 8's k and gs)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run five plain 256 MiB device copies (reference for hardware byte counters)")
    return ap.parse_args()


def cpu_baseline(w, x_np, tok_np, W_np, seed, gpu_topk=None):
    """The oracle, as it stands, on a bounded sample: the whole path for the first `nb` windows of one batch.
    With the GPU's ranked bins of the same batch it also counts rank disagreements (the inputs are not screened:
    variates whose leading mean amplitudes lie closer than 1e-3 relative may legitimately differ)."""
    import numpy as np
    from oracle import attention as o_attn
    from oracle import kdfh as o_kdfh
    from oracle import sampling as o_samp
    import workloads as wl

    blas = None
    try:
        import threadpoolctl
        info = threadpoolctl.threadpool_info()
        cores = max(int(i.get("num_threads", 1)) for i in info) if info else 1
        blas = ", ".join("%s x%s" % (i.get("internal_api"), i.get("num_threads")) for i in info) or None
    except Exception:
        threadpoolctl = None
        cores = os.cpu_count() or 1
    t0 = time.perf_counter()
    topk, hsh, abar = o_kdfh.kdfh(x_np, w.k)                                # the hash needs the full batch
    t1 = time.perf_counter()
    gid, sel, G = o_samp.stratified_sample(hsh, 0, w.ratio[0], w.ratio[1], seed, 0)
    t2 = time.perf_counter()
    rank_check = None
    if gpu_topk is not None:
        clear = o_kdfh.gap_ok(abar, w.k)
        differs = np.any(np.asarray(gpu_topk)[:, :w.k] != topk, axis=1)
        rank_check = {"variates": int(w.N), "below_the_1e-3_gap": int((~clear).sum()),
                      "rank_flips_among_clear": int((differs & clear).sum()),
                      "rank_flips_below_the_gap": int((differs & ~clear).sum()), "redrawn": 0,
                      "note": "batch 0, unscreened draw: GPU ranked top-k against the fp64 oracle"}
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

    def whole_steps(budget_s, first_step):
        steps, t_start = 0, time.perf_counter()
        while time.perf_counter() - t_start < budget_s:
            steps += 1
            tk, hs, _ = o_kdfh.kdfh(x_np, w.k)
            g_, sl, _ = o_samp.stratified_sample(hs, 0, w.ratio[0], w.ratio[1], seed, first_step + steps)
            xs_ = o_attn.gather(tok_np, sl)
            y_, cache_ = o_attn.mha_forward(xs_, *W_np, w.H)
            o_attn.mha_backward(wl.make_upstream(w, len(sl)), cache_)
        return steps, time.perf_counter() - t_start

    one_thread = None
    if nb >= w.B and step_s < 5.0:
        # a whole step is cheap enough: repeat whole steps (new selection each) for about ten seconds
        steps, took = whole_steps(10.0, 0)
        step_s = took / steps
        note = "%d whole steps of the same workload (all %d windows, a new selection each) in %.1f s" % (steps, w.B, took)
        if threadpoolctl is not None:
            with threadpoolctl.threadpool_limits(limits=1):
                s1, took1 = whole_steps(5.0, 1000)
            one_thread = s1 / took1
    out = {"value": 1.0 / step_s, "unit": "steps/s", "cores": cores, "kind": "oracle", "sample": note,
           "blas_threads": blas, "value_one_thread": one_thread}
    if rank_check is not None:
        out["rank_check"] = rank_check
    return out


def steady_bandwidth(args):
    """Kernel time of vardrop_hash and vardrop_gather over M distinct inputs each (M x bytes >= 1 GiB), launched
    back to back on one stream: per-launch durations from the events the runtime ties to every dispatch (library
    hook: the kernel's own execution time), and the wall time of the same loop without events."""
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
        return total_ms * 1e3 / launches, wall_us, launches

    def report(nbytes, us, wall, n, extra):
        # "GB/s_back_to_back" is the conservative figure: launches back to back, dispatch gaps included; "GB/s" is
        # from the kernel's own execution time, which rocprofv3 --kernel-trace of this same command also reports.
        d = dict(extra)
        d.update({"bytes_per_launch": nbytes, "kernel_us": us, "GB/s": nbytes / us * 1e-3,
                  "frac_of_peak": nbytes / us * 1e-3 / PEAK_HBM_GBS, "back_to_back_us": wall,
                  "GB/s_back_to_back": nbytes / wall * 1e-3, "launches": n})
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


def kernel_rooflines(per_kernel, work, steps=8):
    """{kernel: (summed ms, launches)} of `steps` steps + algorithmic work per launch -> roofline entry per kernel."""
    out = {}
    for name, (ms_sum, launches) in per_kernel.items():
        if name not in work or launches == 0:
            continue
        bound, amount = work[name]
        avg_s = ms_sum * 1e-3 / launches
        if bound == "hbm":
            achieved, peak, unit = amount / avg_s / 1e9, PEAK_HBM_GBS, "GB/s"
        else:
            achieved, unit = amount / avg_s / 1e12, "TFLOP/s"
            peak = PEAK_BF16_TFLOPS if bound == "mfma" else PEAK_FP32_TFLOPS
        out[name] = {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
                     "avg_launch_us": avg_s * 1e6, "launches": launches, "us_per_step": ms_sum * 1e3 / steps}
    return out


class Pipeline:
    """The step on the device-count entry points, for one workload and one sampling rule.

    The selection of a batch (k-DFH, grouping, sampling) depends on its windows only, so it runs on a second
    stream beside the attention of earlier batches.  Nothing of it crosses to the host: the attention kernels read
    N' on the device.
      eager: the selection of step g + LEAD is issued with step g and can be placed beside chosen kernels of it: its
             k-DFH and its sampling each start when a named kernel of step g has finished (the fused forward
             kernel: beside the output projection and what follows; the output projection: beside the attention
             backward kernel; that kernel: beside the gradient GEMM; the gradient GEMM: beside the next step's
             forward kernel), or as soon as the selection stream reaches them.  The two single-launch attention
             kernels need every compute unit at once, and a selection kernel that holds one of them makes such a
             kernel wait a whole round; the GEMMs between them leave compute units and LDS free.  Which placement
             is better depends on the shape; a short trial decides.  A placement uses a completion event that
             rides on the kernel's own dispatch (vardrop_signal_after), so the attention stream carries no event
             packets; it waits for the selection stream once per BURST steps.  A call of `count` steps issues
             exactly `count` selections; one runs ahead of the call's first step and the lead grows by up to two
             per step to LEAD, the attention stream waiting per step until it has (a call of few steps is then
             not held up by a block of selections at its start).
      burst: selections are issued in bursts of BURST steps into a ring of RING buffer sets; the attention
             stream waits for one event per burst (and the selection stream for one per burst before it reuses
             ring sets).  The first bursts of a call hold 1, 1 and 2 steps.
      graph: one recorded HIP graph per step, the selection of the NEXT batch on a branch forked from and joined
             back into the attention stream (ring of two sets).
    """
    BURST, RING, LEAD = 4, 16, 5
    _streams = None
    _side_choice = None        # which candidate the first trial of the process kept

    def __init__(self, vd, ctx, w, xs_dev, tok_dev, W_dev, dy_full, seed, gs_cap=0, dense=False, embed=None):
        import torch
        self.vd, self.ctx, self.w, self.torch = vd, ctx, w, torch
        self.xs_dev, self.tok_dev, self.W_dev, self.dy_full = xs_dev, tok_dev, W_dev, dy_full
        self.nb = len(xs_dev)
        self.seed, self.gs_cap, self.dense = seed, gs_cap, dense
        self.embed = embed                          # (We, be): tokens are embedded from the raw windows inside the step
        self.ratio = (1, 1) if gs_cap else w.ratio
        dev = xs_dev[0].device
        # One pair of streams per process, shared by every pipeline: a later pair from the runtime's pool can end up on one
        # hardware queue, and then the selection does not run beside the attention at all (seen as a step of 78 instead
        # of 56 us in every second to eighth pipeline of a process).
        # The process keeps two more candidates for the selection stream; the trial of --launch auto checks them once.
        if Pipeline._streams is None:
            Pipeline._streams = (torch.cuda.Stream(device=dev), [torch.cuda.Stream(device=dev) for _ in range(3)])
        self.main, self.sides = Pipeline._streams
        self.side = self.sides[Pipeline._side_choice or 0]
        self.side_trials_ms = None
        K_MAX = 5
        self.ring = [(torch.empty((w.N, max(w.k, K_MAX)), dtype=torch.int32, device=dev),
                      torch.empty(w.N, dtype=torch.int64, device=dev), torch.empty(w.N, dtype=torch.int32, device=dev),
                      torch.empty(w.N, dtype=torch.int32, device=dev), torch.empty(2, dtype=torch.int32, device=dev))
                     for _ in range(self.RING)]
        self.events = []
        self.issued = None                         # eager mode: the next selection to draw, kept from call to call
        self.n_drawn = 0                           # selections issued from the host since the counter was last reset
        self.step_dev = torch.zeros(1, dtype=torch.int64, device=dev)
        self.status = torch.zeros(1, dtype=torch.int32, device=dev)
        # ---- N' and G of every batch (they depend on the grouping only, not on the draw): an untimed pass
        self.n_of, self.G_of = [], []
        if dense:
            for r in range(self.RING):
                self.ring[r][3].copy_(torch.arange(w.N, dtype=torch.int32, device=dev))
                self.ring[r][4].copy_(torch.tensor([w.N, w.N], dtype=torch.int32, device=dev))
            self.n_of, self.G_of = [w.N] * self.nb, [w.N] * self.nb
        else:
            for b in range(self.nb):
                self.select(b, 0, self.main)
                self.main.synchronize()
                n_b, G_b = self.ring[0][4].tolist()
                self.n_of.append(n_b)
                self.G_of.append(G_b)
        n_hi = max(self.n_of)
        small = w.dtype == "bf16" and n_hi <= 128
        self.n_max = 128 if small and w.N >= 128 else min(w.N, -(-n_hi // 64) * 64)
        lib = vd.load_library()
        code = vd.BF16 if w.dtype == "bf16" else vd.F32
        td = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        self.saved = torch.empty(lib.vardrop_attn_saved_bytes(w.B, self.n_max, w.d, w.H, code), dtype=torch.uint8, device=dev)
        self.ws = torch.empty(lib.vardrop_attn_workspace_bytes(w.B, self.n_max, w.d, w.H, code), dtype=torch.uint8, device=dev)
        self.xs_buf, self.y_buf, self.dxs_buf = (torch.empty((w.B, self.n_max, w.d), dtype=td, device=dev) for _ in range(3))
        self.dW_buf = [torch.empty((w.d, w.d), dtype=torch.float32, device=dev) for _ in range(4)]
        if embed is not None:
            self.esaved = torch.empty(lib.vardrop_embed_saved_bytes(w.B, self.n_max, w.L, code), dtype=torch.uint8, device=dev)
            self.ews = torch.empty(max(lib.vardrop_embed_workspace_bytes(w.B, self.n_max, w.L, w.d, code), 256), dtype=torch.uint8, device=dev)
            self.dWe_buf = (torch.empty((w.L, w.d), dtype=torch.float32, device=dev), torch.empty(w.d, dtype=torch.float32, device=dev))
        self.graphs = None
        self.gates = None                          # eager mode: ("fwd" | "out" | "bwd" | "pair" | None, the same for the sampling)
        self.gate_kids = None                      # kernel ids a completion signal can ride on, by those names
        self.placed = None
        self.trials_ms = None

    def set_gates(self, hash_after, sample_after):
        """eager mode: the k-DFH and the sampling of a later step's selection start when a kernel of this step has
        finished: "fwd" (forward attention kernel), "out" (output projection), "bwd" (attention backward kernel) or
        "pair" (gradient GEMM); None: when the selection stream gets there."""
        torch = self.torch
        self.gates = (hash_after, sample_after)
        names = ("fwd", "out", "bwd", "pair")
        self.gate_events = []
        for _ in range(len(names) * self.RING):
            ev = torch.cuda.Event()
            ev.record(self.main)                   # creates the underlying event; its handle is reused from here on
            self.gate_events.append(ev)
        self.main.synchronize()
        # raw handles and the runtime's own wait call: two waits per step through torch's wrappers cost the host
        # more than the calls they order
        import ctypes
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipStreamWaitEvent.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint]
        self.hip.hipStreamWaitEvent.restype = ctypes.c_int
        handles = [ev.cuda_event for ev in self.gate_events]
        self.gate_handles = {name: handles[i * self.RING:(i + 1) * self.RING] for i, name in enumerate(names)}

    def side_wait(self, handle):
        if self.hip.hipStreamWaitEvent(self.side.cuda_stream, handle, 0) != 0:
            raise RuntimeError("hipStreamWaitEvent failed")

    def select(self, b, r, stream, hash_gate=None, sample_gate=None):
        """k-DFH + grouping + sampling of batch b into ring set r; the step counter advances on the device.  A gate is
        an event handle the stream waits for before that kernel."""
        vd, w = self.vd, self.w
        topk, hsh, gid, sel, counts = self.ring[r]
        self.n_drawn += 1
        if hash_gate is not None:
            self.side_wait(hash_gate)
        vd.vardrop_hash(self.ctx, self.xs_dev[b], w.k, f_max=-1, out=(topk, hsh), stream=stream.cuda_stream)
        if sample_gate is not None:
            self.side_wait(sample_gate)
        vd.vardrop_sample_dev(self.ctx, hsh, self.gs_cap, self.ratio[0], self.ratio[1], self.seed, self.step_dev, True,
                              (gid, sel, counts), stream=stream.cuda_stream)

    def attend(self, b, r, stream, signals=None):
        """Forward and backward pass of batch b on the selection in ring set r.  signals: {gate name: event handle}
        that the named kernels of this step complete (see set_gates; one request can be pending per kernel)."""
        vd, w = self.vd, self.w
        sel, counts = self.ring[r][3], self.ring[r][4]
        for name, handle in (signals or {}).items():
            vd.vardrop_signal_after(self.ctx, self.gate_kids[name], handle)
        if self.embed is not None:
            # tokens of the kept variates straight from the raw windows (no token tensor of all variates exists)
            vd.vardrop_embed_fwd_dev(self.ctx, self.xs_dev[b], sel, counts, self.n_max, self.embed[0], self.embed[1],
                                     self.xs_buf, self.esaved, status=self.status, stream=stream.cuda_stream)
            vd.vardrop_attn_fwd_dev(self.ctx, self.xs_buf, counts, self.n_max, *self.W_dev, w.H, self.y_buf, self.saved,
                                    status=self.status, stream=stream.cuda_stream)
        else:
            vd.vardrop_gather_attn_fwd_dev(self.ctx, self.tok_dev[b], sel, counts, self.n_max, *self.W_dev, w.H,
                                           self.xs_buf, self.y_buf, self.saved, status=self.status, stream=stream.cuda_stream)
        vd.vardrop_attn_bwd_dev(self.ctx, self.dy_full, self.xs_buf, counts, self.n_max, *self.W_dev, w.H, self.saved,
                                self.ws, (self.dxs_buf, *self.dW_buf), status=self.status, stream=stream.cuda_stream)
        if self.embed is not None:
            vd.vardrop_embed_bwd_dev(self.ctx, self.dxs_buf, counts, self.n_max, w.L, self.esaved, self.ews, self.dWe_buf,
                                     stream=stream.cuda_stream)

    def issue(self, g):
        """Step g: attention of batch g % nb (ring g % 2) beside the selection of the next batch (other ring set)."""
        b, r = g % self.nb, g % 2
        if not self.dense:
            self.side.wait_stream(self.main)                           # fork
            self.select((b + 1) % self.nb, (r + 1) % 2, self.side)
        self.attend(b, r, self.main)
        if not self.dense:
            self.main.wait_stream(self.side)                           # join

    def prime(self):
        """graph mode: the selection of batch 0 into ring set 0, so that the first recorded step finds it."""
        if not self.dense:
            self.select(0, 0, self.main)

    def record(self):
        """One HIP graph per (batch, ring set) combination: nb of them when nb is even, else 2 nb."""
        torch = self.torch
        count = self.nb if self.nb % 2 == 0 else 2 * self.nb
        self.vd.vardrop_profile_select(self.ctx, -1)
        self.graphs = []
        for g in range(count):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=self.main):
                self.issue(g)
            self.graphs.append(graph)
        # the captures advanced nothing (nothing ran), but keep the counter explicit
        torch.cuda.synchronize()

    def event(self, i):
        while len(self.events) <= i:
            self.events.append(self.torch.cuda.Event())
        return self.events[i]

    def run(self, first, count, launch, more=False):
        """`count` whole steps from global step `first`; returns when everything is ISSUED (not finished).
        The caller synchronises the device between two calls (ring sets are reused from the start).
        more: another call continues at step first + count (eager mode keeps its lead of drawn selections for it)."""
        torch = self.torch
        if launch != "eager" or self.gates is None:
            self.issued = None
        if count <= 0:
            return
        if launch == "graph":
            with torch.cuda.stream(self.main):
                G = len(self.graphs)
                for g in range(first, first + count):
                    self.graphs[g % G].replay()
            return
        if self.dense:
            for g in range(first, first + count):
                self.attend(g % self.nb, g % self.RING, self.main)
            return
        end = first + count
        if launch == "eager" and self.gates is not None:
            # One selection runs ahead of the first step; the lead then grows by one selection per step up to LEAD (two
            # selections behind a step's gated kernels while it catches up).  While it grows the attention stream
            # waits for every selection on its own (RAMP steps), afterwards once per BURST steps.  With `more` the
            # lead is kept at the end of the call (the selections of the next LEAD steps are drawn) and the next
            # call carries on from it: every call then draws as many selections as it attends steps.
            B4, LEAD, RAMP = self.BURST, self.LEAD, 2 * self.BURST
            drawn = lambda g: self.event(g % self.RING)  # selection g is drawn (recorded on the selection stream)
            issued = self.issued if first > 0 and self.issued is not None and self.issued > first else first
            ramp = issued - first < LEAD

            def draw(hash_gate=None, sample_gate=None):
                nonlocal issued
                self.select(issued % self.nb, issued % self.RING, self.side, hash_gate, sample_gate)
                drawn(issued).record(self.side)
                issued += 1

            if issued == first:
                draw()
            for g in range(first, end):
                k = g - first
                if ramp and k < RAMP:
                    self.main.wait_event(drawn(g))
                elif k % B4 == 0:
                    self.main.wait_event(drawn(min(g + B4 - 1, end - 1)))
                target = g + 1 + LEAD if more else min(end, g + 1 + LEAD)
                n_new = min(2, target - issued)
                ev = {name: ring[g % self.RING] for name, ring in self.gate_handles.items()}
                ev[None] = None
                used = {name for name in self.gates if name} if n_new > 0 else set()
                # A sampling that waits for no kernel of this step could overwrite a ring set that an attention step
                # far behind the host has yet to read (the host issues faster than the device works).  Every BURST
                # steps this step's backward kernel then carries a signal, and the selection stream waits for the
                # one of BURST steps ago: the steps that read the ring sets drawn next (RING steps back) are over.
                guard = self.gates[1] is None and k % B4 == 0
                if guard:
                    used.add("bwd")
                self.attend(g % self.nb, g % self.RING, self.main, signals={name: ev[name] for name in used})
                if guard and k >= B4:
                    self.side_wait(self.gate_handles["bwd"][(g - B4) % self.RING])
                for i in range(n_new):
                    if i == 0:
                        draw(ev[self.gates[0]], ev[self.gates[1]])
                    else:
                        draw()
            self.issued = issued
            return
        self.issued = None
        blocks, g = [], first
        while g < end:
            # (the bursts grow 1, 1, 2, 4, 4, ...: a burst runs beside the block before it, which must not be shorter)
            size = (1, 1, 2)[len(blocks)] if len(blocks) < 3 else self.BURST
            blocks.append(range(g, min(end, g + size)))
            g += size
        done_sel = lambda j: self.event(2 * j)          # burst j has been drawn (recorded on the selection stream)
        done_att = lambda j: self.event(2 * j + 1)      # block j has been attended (recorded on the attention stream)

        def burst(j):
            if j >= 3:
                self.side.wait_event(done_att(j - 3))   # its ring sets were last read by block j - 3
            for g in blocks[j]:
                self.select(g % self.nb, g % self.RING, self.side)
            done_sel(j).record(self.side)

        burst(0)
        for j, blk in enumerate(blocks):
            if j + 1 < len(blocks):
                burst(j + 1)
            self.main.wait_event(done_sel(j))
            for g in blk:
                self.attend(g % self.nb, g % self.RING, self.main)
            done_att(j).record(self.main)

    def kept(self, first, count):
        ns = [self.n_of[g % self.nb] for g in range(first, first + count)]
        gs = [self.G_of[g % self.nb] for g in range(first, first + count)]
        return sum(ns) / len(ns), sum(gs) / len(gs)


PLACEMENTS = tuple((h, s) for s in (None, "fwd", "out", "bwd", "pair") for h in (None, "fwd", "out", "bwd", "pair"))


def placements(pipe):
    """eager mode: finds the kernels of this pipeline's attention steps that a completion signal can ride on (two
    untimed steps with every launch timed): the forward attention kernel, the output projection, the last attention
    backward kernel and the gradient GEMM.  Returns the (k-DFH after, sampling after) pairs a trial can choose from."""
    import torch
    vd, ctx = pipe.vd, pipe.ctx
    if pipe.dense:
        return []
    pipe.step_dev.zero_()
    vd.vardrop_profile_select(ctx, vd.K_ALL)
    pipe.run(0, 2, "burst")
    torch.cuda.synchronize()
    ran = set(vd.vardrop_profile_read_all(ctx))
    vd.vardrop_profile_select(ctx, -1)
    names = {"fwd": next((name for name in ("qkv_sdpa_fwd", "sdpa_fwd") if name in ran), None),
             "out": "gemm_out" if "gemm_out" in ran else None,
             "bwd": next((name for name in ("sdpa_bwd", "sdpa_bwd_dqkv", "sdpa_bwd_dkv") if name in ran), None),
             "pair": "gemm_dw_dxs" if "gemm_dw_dxs" in ran else None}
    if any(v is None for v in names.values()):
        return []
    kid = {vd.vardrop_kernel_name(k): k for k in range(64) if vd.vardrop_kernel_name(k)}
    pipe.gate_kids = {name: kid[kernel] for name, kernel in names.items()}
    pipe.gate_names = dict(names)
    pipe.gate_names[None] = None
    return list(PLACEMENTS)


def placement_name(gates):
    return "hash:%s,sample:%s" % tuple(g or "free" for g in gates)


def place(pipe, gates):
    """Needs placements(pipe) to have run."""
    pipe.set_gates(*gates)
    pipe.placed = {"hash_starts_after": pipe.gate_names[gates[0]], "sampling_starts_after": pipe.gate_names[gates[1]]}


def choose_launch(pipe, args):
    """--launch auto: tries the burst pipeline and the eager pipeline with every placement of the selection for a
    few untimed steps each and keeps the fastest; --launch eager does the same among the placements only."""
    import copy
    if args.launch in ("burst", "graph") or pipe.dense:
        return "burst" if pipe.dense else args.launch
    cands = placements(pipe)
    if not cands:
        return "burst"
    trial = copy.copy(args)
    trial.steps, trial.warmup = max(40, min(80, args.steps)), 20
    results, by_name = {}, {}
    for gates in cands:
        place(pipe, gates)
        by_name[placement_name(gates)] = gates
        results[placement_name(gates)] = min(timed_steps(pipe, trial, "eager")[0] for _ in range(2))
    if args.launch == "auto":
        results["burst"] = min(timed_steps(pipe, trial, "burst")[0] for _ in range(2))
    best = min(results, key=results.get)
    pipe.trials_ms = results
    launch = "burst" if best == "burst" else "eager"
    if launch == "eager":
        place(pipe, by_name[best])
    if Pipeline._side_choice is None:
        # once per process: is another stream of the runtime's pool a better selection stream?  (Two streams that
        # share a hardware queue do not overlap at all; the first candidate has never been such a one.)
        sides = {0: results[best]}
        for i in range(1, len(pipe.sides)):
            pipe.side = pipe.sides[i]
            sides[i] = min(timed_steps(pipe, trial, launch)[0] for _ in range(2))
        keep = min(sides, key=sides.get)
        if sides[keep] > 0.97 * sides[0]:
            keep = 0                                 # (within the noise of a trial: stay with the first)
        Pipeline._side_choice = keep
        pipe.side = pipe.sides[keep]
        pipe.side_trials_ms = sides
    return launch


def timed_steps(pipe, args, launch):
    """W warm-up steps, then exactly K timed steps, bracketed by device synchronisation on both sides.  The timed call
    issues K selections and K attention steps.  In the eager pipeline the selections run LEAD steps ahead of the
    attention, across the two calls as well: the warm-up call ends with the next LEAD selections drawn, so the timed
    call starts in the steady state, and it draws the selections of the LEAD steps that follow it (checked: at least as
    many selections as steps inside the timed call; the whole-device synchronisation that ends it waits for them too)."""
    import torch
    primed = 0
    if launch == "graph":
        if pipe.graphs is None:
            pipe.run(0, 2, "eager")                 # tables built, function attributes set, before anything is recorded
            torch.cuda.synchronize()
            pipe.record()
        pipe.step_dev.zero_()
        pipe.prime()
        primed = 1
    else:
        pipe.step_dev.zero_()
    pipe.issued, pipe.n_drawn = None, 0
    pipe.run(0, args.warmup, launch, more=True)
    torch.cuda.synchronize()
    drawn_before = pipe.n_drawn
    t0 = time.perf_counter()
    pipe.run(args.warmup, args.steps, launch, more=True)
    t_host = time.perf_counter()                    # every launch of the timed steps has been issued
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    if int(pipe.status[0]) != 0:
        raise RuntimeError("a step found more kept tokens than the bound the launches were sized for")
    if launch != "graph" and not pipe.dense and pipe.n_drawn - drawn_before < args.steps:      # (more while the lead still grows)
        raise RuntimeError("the timed call drew %d selections for %d steps" % (pipe.n_drawn - drawn_before, args.steps))
    expected = primed + args.warmup + args.steps if launch == "graph" else pipe.n_drawn
    if not pipe.dense and int(pipe.step_dev[0]) != expected:
        raise RuntimeError("the device step counter does not match the number of selections drawn")
    return (t1 - t0) * 1e3 / args.steps, (t_host - t0) * 1e3 / args.steps


def steady_hash_gather(vd, ctx, w, stream):
    """Steady-state duration of vardrop_hash and vardrop_gather at this workload's shape over enough distinct inputs
    (>= 1 GiB) that the last-level cache cannot serve them: per-launch durations from dispatch-bound events."""
    import torch
    dev = torch.device("cuda", 0)
    td = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    es = 2 if w.dtype == "bf16" else 4
    gen = torch.Generator(device=dev)
    gen.manual_seed(99)
    out = {}
    x_bytes = 4 * w.B * w.N * w.L
    M = -(-(1 << 30) // x_bytes)
    xs = [torch.randn((w.B, w.N, w.L), generator=gen, device=dev) for _ in range(M)]
    topk = torch.empty((w.N, w.k), dtype=torch.int32, device=dev)
    hsh = torch.empty(w.N, dtype=torch.int64, device=dev)
    kid = {vd.vardrop_kernel_name(k): k for k in range(64) if vd.vardrop_kernel_name(k)}
    with torch.cuda.stream(stream):
        for x in xs:
            vd.vardrop_hash(ctx, x, w.k, f_max=-1, out=(topk, hsh), stream=stream.cuda_stream)
        torch.cuda.synchronize()
        vd.vardrop_profile_select(ctx, kid["hash"])
        for x in xs:
            vd.vardrop_hash(ctx, x, w.k, f_max=-1, out=(topk, hsh), stream=stream.cuda_stream)
        ms, n = vd.vardrop_profile_read(ctx)
    out["hash"] = {"bound": "hbm", "achieved": x_bytes / (ms * 1e-3 / n) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                   "frac": x_bytes / (ms * 1e-3 / n) / 1e9 / PEAK_HBM_GBS, "avg_launch_us": ms * 1e3 / n,
                   "launches": n, "distinct_inputs": M, "bytes_per_launch": x_bytes}
    del xs
    n_sel = max(1, int(round(w.N * w.ratio[0] / w.ratio[1] * 1.3)))
    g_bytes = 2 * w.B * n_sel * w.d * es
    tok_bytes = w.B * w.N * w.d * es
    M = max(4, min(-(-(1 << 30) // g_bytes), (8 << 30) // tok_bytes))
    toks = [torch.randn((w.B, w.N, w.d), generator=gen, device=dev).to(td) for _ in range(M)]
    sel = torch.zeros(w.N, dtype=torch.int32, device=dev)
    sel[:n_sel] = torch.randperm(w.N, generator=gen, device=dev)[:n_sel].sort().values.to(torch.int32)
    dst = torch.empty((w.B, n_sel, w.d), dtype=td, device=dev)
    with torch.cuda.stream(stream):
        for t in toks:
            vd.vardrop_gather(ctx, t, sel, n_sel, out=dst, stream=stream.cuda_stream)
        torch.cuda.synchronize()
        vd.vardrop_profile_select(ctx, kid["gather"])
        for _ in range(3):
            for t in toks:
                vd.vardrop_gather(ctx, t, sel, n_sel, out=dst, stream=stream.cuda_stream)
        ms, n = vd.vardrop_profile_read(ctx)
    vd.vardrop_profile_select(ctx, -1)
    out["gather"] = {"bound": "hbm", "achieved": g_bytes / (ms * 1e-3 / n) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": g_bytes / (ms * 1e-3 / n) / 1e9 / PEAK_HBM_GBS, "avg_launch_us": ms * 1e3 / n,
                     "launches": n, "distinct_inputs": M, "kept_tokens": n_sel, "bytes_per_launch": g_bytes}
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path; run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    if args.mode == "bandwidth":
        return steady_bandwidth(args)
    import dataclasses
    import numpy as np
    import torch
    import paper_2501_14183_amd as vd
    import workloads as wl

    w = wl.WORKLOADS[args.workload]
    if args.k:
        w = dataclasses.replace(w, k=args.k)
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
    seed = 0x5EED

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
        sw = argparse.Namespace(steps=100, warmup=20, launch=args.launch)
        for k in (2, 3, 4, 5):
            for gs in (1, 2, 3, 5, 8, 10, 15, 20):
                wk = dataclasses.replace(w, k=k)
                pipe = Pipeline(vd, ctx, wk, xs_dev, tok_dev, W_dev, dy_full, seed, gs_cap=gs)
                launch = choose_launch(pipe, sw)            # (every cell places its selection by its own trial)
                ms, _ = timed_steps(pipe, sw, launch)
                n_mean, g_mean = pipe.kept(sw.warmup, sw.steps)
                table.append({"k": k, "gs": gs, "groups": g_mean, "kept": n_mean, "delta": 1.0 - n_mean / w.N,
                              "token_bound": pipe.n_max, "steps_per_s": 1e3 / ms, "launch": launch,
                              "selection_placement": pipe.placed if launch == "eager" else None})
                del pipe
        print(json.dumps({"metric": "reduction ratio delta and train steps/s over k and gs (Eq. 1)", "n_gpus": 1,
                          "data": "synthetic", "dtype": w.dtype, "launch": args.launch,
                          "config": {"workload": "%s-shaped: B=%d N=%d L=%d d=%d H=%d" % (w.name, w.B, w.N, w.L, w.d, w.H)},
                          "table": table}))
        return

    embed = None
    if args.embed:
        gen = torch.Generator(device=dev)
        gen.manual_seed(4321)
        embed = ((torch.randn((w.L, w.d), generator=gen, device=dev) / w.L ** 0.5).to(td),
                 (0.1 * torch.randn(w.d, generator=gen, device=dev)).to(td))
    pipe = Pipeline(vd, ctx, w, xs_dev, tok_dev, W_dev, dy_full, seed, gs_cap=args.gs, dense=args.dense, embed=embed)
    launch = choose_launch(pipe, args)
    ms, host_ms = timed_steps(pipe, args, launch)
    n_mean, g_mean = pipe.kept(args.warmup, args.steps)

    # ---- roofline: the same steps once more, issued call by call, every dispatch timed by the events the runtime
    # ties to it (the kernel's own execution time, no extra packet on the stream; launches inside a recorded graph
    # cannot carry them).  Dominant = the kernel with the largest share of a step on the attention stream.
    PROF_STEPS = 8
    pipe.step_dev.zero_()
    pipe.run(0, 4, "burst")
    torch.cuda.synchronize()
    vd.vardrop_profile_select(ctx, vd.K_ALL)
    pipe.run(4, PROF_STEPS, "burst")                 # (a kernel that carries a completion signal cannot be timed)
    torch.cuda.synchronize()
    per_kernel = vd.vardrop_profile_read_all(ctx)
    vd.vardrop_profile_select(ctx, -1)
    n_prof, _ = pipe.kept(4, PROF_STEPS)
    work = algorithmic_work(w, n_prof)
    roof_all = kernel_rooflines(per_kernel, work, PROF_STEPS)
    attn = {k: v for k, v in roof_all.items() if k not in ("hash", "sample")}
    dominant = max(attn, key=lambda k: attn[k]["us_per_step"])
    roof = {"kernel": dominant}
    roof.update({k: roof_all[dominant][k] for k in ("bound", "achieved", "peak", "unit", "frac")})
    roof["traffic"] = recorded_traffic(w.name, dominant)
    roof["avg_launch_us"] = roof_all[dominant]["avg_launch_us"]
    roof["launches"] = roof_all[dominant]["launches"]
    if dominant == "gemm_dw_dxs" and "reduce_dw" not in roof_all:
        roof["note"] = ("one launch for the input gradient and the four weight gradients, each over all of K: no partial "
                        "products and no separate launch that sums K slices (two slices make this launch 3.5 us "
                        "shorter and the step 3 us longer)")
    roof["timing"] = ("events tied to each dispatch of the kernel (hipExtLaunchKernelGGL) over %d steps issued call by call "
                      "right after the timed region" % PROF_STEPS)
    # whole attention (every matrix-core kernel of a step): algorithmic flops of forward + backward over their summed time
    if w.dtype == "bf16":
        flops = sum(work[k][1] * v["launches"] / PROF_STEPS for k, v in attn.items() if v["bound"] == "mfma")
        us = sum(v["us_per_step"] for k, v in attn.items())
        roof_all["attention_fwd_bwd"] = {"bound": "mfma", "achieved": flops / (us * 1e-6) / 1e12, "peak": PEAK_BF16_TFLOPS,
                                         "unit": "TFLOP/s", "frac": flops / (us * 1e-6) / 1e12 / PEAK_BF16_TFLOPS,
                                         "us_per_step": us, "kernels": sorted(attn)}
    if not args.dense and not args.embed:
        steady = steady_hash_gather(vd, ctx, w, pipe.main)
        roof_all["hash_steady_state"] = steady["hash"]
        roof_all["gather_steady_state"] = steady["gather"]

    out = {
        "metric": (("dense (no dropping) variate-attn train steps/s (SDPA fwd/bwd over all N tokens)" if args.dense else
                    "variate-attn train steps/s (kDFH+sample+SDPA fwd/bwd), HBM GB/s, MFMA %peak") +
                   (" + token embedding fwd/bwd of the kept variates inside the step" if args.embed else "")),
        "value": 1e3 / ms, "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "host_issue_ms_per_step": host_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": ("%s-shaped, dense: B=%d N=%d d=%d H=%d, selection = identity" % (w.name, w.B, w.N, w.d, w.H))
                               if args.dense else "%s-shaped: B=%d N=%d L=%d k=%d keep=%s d=%d H=%d" %
                               (w.name, w.B, w.N, w.L, w.k, ("min(|G|,%d)" % args.gs) if args.gs else "%d/%d" % w.ratio, w.d, w.H),
                   "k": w.k, "gs": args.gs if args.gs else None,
                   "kept_tokens_mean": n_mean, "groups_mean": g_mean, "token_bound": pipe.n_max,
                   "batches": args.batches, "launch": launch, "selection_placement": pipe.placed if launch == "eager" else None,
                   "launch_trials_ms_per_step": pipe.trials_ms, "selection_stream_trials_ms_per_step": pipe.side_trials_ms},
        "roofline": roof, "roofline_all": roof_all,
    }
    # ---- the paper's own rule for this dataset shape (Table 8: Traffic k = 4, gs = 10; Electricity k = 3, gs = 10)
    paper_rule = {"traffic": (4, 10), "electricity": (3, 10)}.get(w.name)
    if paper_rule and not (args.dense or args.gs or args.k or args.no_paper_rule or args.embed):
        wk = dataclasses.replace(w, k=paper_rule[0])
        p2 = Pipeline(vd, ctx, wk, xs_dev, tok_dev, W_dev, dy_full, seed, gs_cap=paper_rule[1])
        launch2 = choose_launch(p2, args)
        ms2, host2 = timed_steps(p2, args, launch2)
        n2, g2 = p2.kept(args.warmup, args.steps)
        out["paper_rule"] = {"rule": "Eq. 1, |S_i| = min(|G_i|, gs), with Table 8's k = %d, gs = %d" % paper_rule,
                             "value": 1e3 / ms2, "unit": "steps/s", "ms_per_step": ms2, "host_issue_ms_per_step": host2,
                             "kept_tokens_mean": n2, "groups_mean": g2, "delta": 1.0 - n2 / w.N, "token_bound": p2.n_max,
                             "launch": launch2, "selection_placement": p2.placed if launch2 == "eager" else None}
        del p2
    if not args.dense and not args.embed and not args.no_cpu_baseline:
        gpu_topk = None
        topk0 = torch.empty((w.N, w.k), dtype=torch.int32, device=dev)
        hsh0 = torch.empty(w.N, dtype=torch.int64, device=dev)
        vd.vardrop_hash(ctx, xs_dev[0], w.k, f_max=-1, out=(topk0, hsh0))
        torch.cuda.synchronize()
        gpu_topk = topk0.cpu().numpy()
        out["cpu_baseline"] = cpu_baseline(w, host[0], host[1], W_np, seed, gpu_topk)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
