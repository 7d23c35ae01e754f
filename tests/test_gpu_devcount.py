"""The entry points that read the number of kept tokens on the device (Eq. 2: S, and with it N' = |S|, is data of
the step): against the oracle, against the host-count entry points, at the count's limits, and replayed from a
recorded HIP graph."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import attention as o_attn
from oracle import sampling as o_samp
from util_gpu import SEED, STEP, TOL, oracle_attention, rel_err, to_dev, torch_dtype, workload_inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vd():
    import paper_2501_14183_amd as m
    return m


@pytest.fixture(scope="module")
def ctx(vd):
    return vd.Context(0)


class Buffers:
    """Everything a step writes, sized once for n_max tokens."""

    def __init__(self, vd, B, N, d, H, td, n_max, bias_grads=False):
        lib = vd.load_library()
        code = vd.BF16 if td == torch.bfloat16 else vd.F32
        dev = torch.device("cuda", 0)
        self.n_max = n_max
        self.saved = torch.empty(lib.vardrop_attn_saved_bytes(B, n_max, d, H, code), dtype=torch.uint8, device=dev)
        self.ws = torch.empty(lib.vardrop_attn_workspace_bytes(B, n_max, d, H, code), dtype=torch.uint8, device=dev)
        self.xs, self.y, self.dxs = (torch.full((B, n_max, d), float("nan"), dtype=td, device=dev) for _ in range(3))
        self.dW = [torch.full((d, d), float("nan"), dtype=torch.float32, device=dev) for _ in range(4)]
        self.db = [torch.full((d,), float("nan"), dtype=torch.float32, device=dev) for _ in range(4)] if bias_grads else []
        self.status = torch.zeros(1, dtype=torch.int32, device=dev)

    def packed(self, t, B, n):
        return t.reshape(-1)[:B * n * t.shape[2]].view(B, n, t.shape[2])


def run_dev(vd, ctx, bufs, tok_t, sel, n_dev, W_t, H, dy_packed, b_t=(None,) * 4, stream=None):
    vd.vardrop_gather_attn_fwd_dev(ctx, tok_t, sel, n_dev, bufs.n_max, *W_t, H, bufs.xs, bufs.y, bufs.saved,
                                   *b_t, status=bufs.status, stream=stream)
    vd.vardrop_attn_bwd_dev(ctx, dy_packed, bufs.xs, n_dev, bufs.n_max, *W_t, H, bufs.saved, bufs.ws,
                            (bufs.dxs, *bufs.dW, *bufs.db), status=bufs.status, stream=stream)


@pytest.mark.parametrize("name", wl.ORDER)
def test_step_with_the_count_on_the_device_matches_oracle(vd, ctx, name):
    """hash -> sample -> gather + forward -> backward with N' never leaving the device, at the five workloads:
    integers bit-exact, attention within the tolerance; and bit for bit what the host-count entry points give
    when both take the same kernels (bound = N': always)."""
    w, x, info, want_topk, want_hash, _ = workload_inputs(name)
    td = torch_dtype(w.dtype)
    tok = wl.make_tokens(w, x)
    W = wl.make_weights(w)
    x_t, tok_t = to_dev(x), to_dev(tok, td)
    W_t = [to_dev(m, td) for m in W]
    want_gid, want_sel, want_G = o_samp.stratified_sample(want_hash, 0, w.ratio[0], w.ratio[1], SEED, STEP)
    n = len(want_sel)
    dy = wl.make_upstream(w, n)
    dy_t = to_dev(dy, td)
    want = oracle_attention(tok[:, want_sel, :], W, w.H, dy)
    # bounds: the count itself, the largest the single-kernel path takes (when the count fits), all variates
    bounds = [n, w.N] + ([128] if n <= 128 and w.N >= 128 and w.dtype == "bf16" else [])
    for n_max in bounds:
        bufs = Buffers(vd, w.B, w.N, w.d, w.H, td, n_max)
        topk, hsh, _ = vd.vardrop_hash(ctx, x_t, w.k, f_max=-1)
        step_dev = torch.tensor([STEP], dtype=torch.int64, device="cuda")
        out = (torch.empty(w.N, dtype=torch.int32, device="cuda"), torch.empty(w.N, dtype=torch.int32, device="cuda"),
               torch.empty(2, dtype=torch.int32, device="cuda"))
        gid, sel, counts = vd.vardrop_sample_dev(ctx, hsh, 0, w.ratio[0], w.ratio[1], SEED, step_dev, True, out)
        run_dev(vd, ctx, bufs, tok_t, sel, counts[:1], W_t, w.H, dy_t)
        torch.cuda.synchronize()
        assert int(step_dev[0]) == STEP + 1 and int(bufs.status[0]) == 0
        assert counts.tolist() == [n, want_G]
        assert np.array_equal(topk.cpu().numpy(), want_topk)
        assert np.array_equal(gid.cpu().numpy(), want_gid)
        assert np.array_equal(sel.cpu().numpy()[:n], want_sel)
        xs = bufs.packed(bufs.xs, w.B, n)
        assert np.array_equal(xs.float().cpu().numpy(), tok[:, want_sel, :])
        got = dict(y=bufs.packed(bufs.y, w.B, n), dxs=bufs.packed(bufs.dxs, w.B, n),
                   dWq=bufs.dW[0], dWk=bufs.dW[1], dWv=bufs.dW[2], dWo=bufs.dW[3])
        errs = {k: rel_err(v, want[k]) for k, v in got.items()}
        assert all(e <= TOL[w.dtype] for e in errs.values()), (n_max, errs)
        # nothing past the packed rows was written
        for t in (bufs.xs, bufs.y, bufs.dxs):
            assert torch.isnan(t.reshape(-1)[w.B * n * w.d:].float()).all()
        if n_max == n:
            xs2, y2, saved2 = vd.vardrop_gather_attn_fwd(ctx, tok_t, sel, n, *W_t, w.H)
            g2 = vd.vardrop_attn_bwd(ctx, dy_t, xs2, *W_t, w.H, saved2)
            torch.cuda.synchronize()
            assert torch.equal(got["y"], y2) and torch.equal(got["dxs"], g2[0])
            assert all(torch.equal(a, b) for a, b in zip(bufs.dW, g2[1:]))
        print("%s bound %d: N'=%d errs=%s" % (name, n_max, n, {k: "%.1e" % v for k, v in errs.items()}))


@pytest.mark.parametrize("n_max,counts", [(128, (1, 5, 31, 64, 127, 128)), (300, (1, 63, 128, 129, 188, 200, 256, 300)),
                                          (96, (96, 17))])
def test_ragged_counts_under_one_bound(vd, ctx, n_max, counts):
    """One set of buffers and one bound, many counts (bf16, with biases and bias gradients): every count against
    the oracle, on the single-kernel path (bound <= 128) and on the general path (bound 300, which then also
    serves counts the other path would take)."""
    rng = np.random.default_rng(n_max)
    B, N, d, H = 3, 320, 128, 2
    td = torch.bfloat16
    tok = rng.standard_normal((B, N, d)).astype(np.float32)
    W = [(rng.standard_normal((d, d)) / np.sqrt(d)).astype(np.float32) for _ in range(4)]
    b = [(0.1 * rng.standard_normal(d)).astype(np.float32) for _ in range(4)]
    tok_t, W_t, b_t = to_dev(tok, td), [to_dev(m, td) for m in W], [to_dev(m, td) for m in b]
    tok_r = tok_t.float().cpu().numpy().astype(np.float64)
    W_r = [m.float().cpu().numpy().astype(np.float64) for m in W_t]
    b_r = [m.float().cpu().numpy().astype(np.float64) for m in b_t]
    bufs = Buffers(vd, B, N, d, H, td, n_max, bias_grads=True)
    n_dev = torch.zeros(1, dtype=torch.int32, device="cuda")
    for n in counts:
        sel_np = np.sort(rng.choice(N, size=n, replace=False))
        sel = torch.zeros(N, dtype=torch.int32, device="cuda")
        sel[:n] = to_dev(sel_np.astype(np.int32))
        dy = rng.standard_normal((B, n, d)).astype(np.float32)
        dy_t = to_dev(dy, td)
        n_dev.fill_(n)
        run_dev(vd, ctx, bufs, tok_t, sel, n_dev, W_t, H, dy_t, b_t)
        torch.cuda.synchronize()
        assert int(bufs.status[0]) == 0
        want = oracle_attention(tok_r[:, sel_np, :], W_r, H, dy_t.float().cpu().numpy().astype(np.float64), b_r)
        got = dict(y=bufs.packed(bufs.y, B, n), dxs=bufs.packed(bufs.dxs, B, n), dWq=bufs.dW[0], dWk=bufs.dW[1],
                   dWv=bufs.dW[2], dWo=bufs.dW[3], dbv=bufs.db[2], dbo=bufs.db[3])
        errs = {k: rel_err(v, want[k]) for k, v in got.items()}
        assert all(e <= TOL["bf16"] for e in errs.values()), (n, errs)
        assert torch.equal(bufs.packed(bufs.xs, B, n), tok_t[:, to_dev(sel_np), :])


def test_count_outside_the_bound_raises_the_status_and_writes_nothing(vd, ctx):
    rng = np.random.default_rng(5)
    B, N, d, H = 2, 200, 128, 2
    td = torch.bfloat16
    tok_t = to_dev(rng.standard_normal((B, N, d)).astype(np.float32), td)
    W_t = [to_dev((rng.standard_normal((d, d)) / np.sqrt(d)).astype(np.float32), td) for _ in range(4)]
    sel = torch.arange(N, dtype=torch.int32, device="cuda")
    for n_max in (64, 150):                                   # single-kernel path, general path
        for bad in (n_max + 1, -1, 2 ** 31 - 1):
            bufs = Buffers(vd, B, N, d, H, td, n_max)
            n_dev = torch.tensor([bad], dtype=torch.int32, device="cuda")
            dy_t = torch.ones((B, n_max, d), dtype=td, device="cuda")
            run_dev(vd, ctx, bufs, tok_t, sel, n_dev, W_t, H, dy_t)
            torch.cuda.synchronize()
            assert int(bufs.status[0]) == 1
            for t in (bufs.xs, bufs.y, bufs.dxs, *bufs.dW):
                assert torch.isnan(t.float()).all()
        # a count of zero is valid: nothing is attended, the weight gradients are zero
        bufs = Buffers(vd, B, N, d, H, td, n_max)
        n_dev = torch.zeros(1, dtype=torch.int32, device="cuda")
        run_dev(vd, ctx, bufs, tok_t, sel, n_dev, W_t, H, torch.ones((B, n_max, d), dtype=td, device="cuda"))
        torch.cuda.synchronize()
        assert int(bufs.status[0]) == 0
        assert all(t.eq(0).all() for t in bufs.dW)
        assert torch.isnan(bufs.y.float()).all() and torch.isnan(bufs.dxs.float()).all()


def test_fp32_back_end_with_the_count_on_the_device(vd, ctx):
    rng = np.random.default_rng(6)
    B, N, d, H = 2, 50, 64, 2
    tok = rng.standard_normal((B, N, d)).astype(np.float32)
    W = [(rng.standard_normal((d, d)) / np.sqrt(d)).astype(np.float32) for _ in range(4)]
    tok_t, W_t = to_dev(tok), [to_dev(m) for m in W]
    bufs = Buffers(vd, B, N, d, H, torch.float32, 40, bias_grads=True)
    n_dev = torch.zeros(1, dtype=torch.int32, device="cuda")
    for n in (40, 1, 33):
        sel_np = np.sort(rng.choice(N, size=n, replace=False))
        sel = torch.zeros(N, dtype=torch.int32, device="cuda")
        sel[:n] = to_dev(sel_np.astype(np.int32))
        dy = rng.standard_normal((B, n, d)).astype(np.float32)
        n_dev.fill_(n)
        run_dev(vd, ctx, bufs, tok_t, sel, n_dev, W_t, H, to_dev(dy))
        torch.cuda.synchronize()
        want = oracle_attention(tok[:, sel_np, :].astype(np.float64), [m.astype(np.float64) for m in W], H, dy.astype(np.float64))
        got = dict(y=bufs.packed(bufs.y, B, n), dxs=bufs.packed(bufs.dxs, B, n), dWq=bufs.dW[0], dWk=bufs.dW[1],
                   dWv=bufs.dW[2], dWo=bufs.dW[3], dbv=bufs.db[2], dbo=bufs.db[3])
        errs = {k: rel_err(v, want[k]) for k, v in got.items()}
        assert all(e <= TOL["fp32"] for e in errs.values()), (n, errs)
    n_dev.fill_(41)
    run_dev(vd, ctx, bufs, tok_t, sel, n_dev, W_t, H, to_dev(dy))
    torch.cuda.synchronize()
    assert int(bufs.status[0]) == 1


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_gather_and_scatter_with_the_count_on_the_device(vd, ctx, dtype):
    rng = np.random.default_rng(8)
    B, N, d, n_max = 3, 40, 24, 30
    tok = torch.from_numpy(rng.standard_normal((B, N, d)).astype(np.float32)).to(dtype).cuda()
    out = torch.full((B, n_max, d), float("nan"), dtype=dtype, device="cuda")
    back = torch.full((B, N, d), float("nan"), dtype=dtype, device="cuda")
    n_dev = torch.zeros(1, dtype=torch.int32, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    for n in (30, 7, 1):
        sel_np = np.sort(rng.choice(N, size=n, replace=False)).astype(np.int32)
        sel = torch.zeros(N, dtype=torch.int32, device="cuda")
        sel[:n] = torch.from_numpy(sel_np).cuda()
        n_dev.fill_(n)
        vd.vardrop_gather_dev(ctx, tok, sel, n_dev, n_max, out, status=status)
        packed = out.reshape(-1)[:B * n * d].view(B, n, d)
        vd.vardrop_scatter_dev(ctx, packed, sel, n_dev, n_max, back, status=status)
        torch.cuda.synchronize()
        assert np.array_equal(packed.float().cpu().numpy(), o_attn.gather(tok.float().cpu().numpy(), sel_np))
        assert np.array_equal(back.float().cpu().numpy(), o_attn.scatter_add(packed.float().cpu().numpy(), sel_np, N))
    assert int(status[0]) == 0
    n_dev.fill_(31)
    vd.vardrop_gather_dev(ctx, tok, sel, n_dev, n_max, out, status=status)
    torch.cuda.synchronize()
    assert int(status[0]) == 1


def test_sampling_draws_anew_at_every_replay_of_a_recorded_step(vd, ctx):
    """The whole step of the Traffic-shaped workload recorded once as a HIP graph (selection on a forked branch
    beside the attention, as the benchmark records it) and replayed: every replay draws the selection of the next
    step counter and must equal the same step issued eagerly, with the program's own eager work and
    synchronisations between the replays."""
    w, x, info, want_topk, want_hash, _ = workload_inputs("traffic")
    td = torch_dtype(w.dtype)
    tok = wl.make_tokens(w, x)
    W = wl.make_weights(w)
    x_t, tok_t = to_dev(x), to_dev(tok, td)
    W_t = [to_dev(m, td) for m in W]
    n_max = 128
    dy_t = to_dev(wl.make_upstream(w, n_max), td)                      # the first B * N' * d elements are the step's dy
    bufs, ref = Buffers(vd, w.B, w.N, w.d, w.H, td, n_max), Buffers(vd, w.B, w.N, w.d, w.H, td, n_max)
    sel_out = [tuple((torch.empty((w.N, w.k), dtype=torch.int32, device="cuda"), torch.empty(w.N, dtype=torch.int64, device="cuda"),
                      torch.empty(w.N, dtype=torch.int32, device="cuda"), torch.empty(w.N, dtype=torch.int32, device="cuda"),
                      torch.empty(2, dtype=torch.int32, device="cuda"))) for _ in range(2)]
    step_dev = torch.tensor([STEP], dtype=torch.int64, device="cuda")

    def step(bf, so, main, side):
        """selection (hash + sample) on `side`, attention forward + backward of the selection on `main`"""
        topk, hsh, gid, sel, counts = so
        side.wait_stream(main)
        vd.vardrop_hash(ctx, x_t, w.k, out=(topk, hsh), stream=side.cuda_stream)
        vd.vardrop_sample_dev(ctx, hsh, 0, w.ratio[0], w.ratio[1], SEED, step_dev, True, (gid, sel, counts),
                              stream=side.cuda_stream)
        main.wait_stream(side)
        run_dev(vd, ctx, bf, tok_t, sel, counts[:1], W_t, w.H, dy_t, stream=main.cuda_stream)

    main, side = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(main):
        step(bufs, sel_out[0], main, side)                             # eager warm-up: tables built, attributes set
    torch.cuda.synchronize()
    step_dev.fill_(STEP)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=main):
        step(bufs, sel_out[0], main, side)
    torch.cuda.synchronize()
    seen = set()
    for r in range(4):
        s = STEP + r
        step_dev.fill_(s)
        graph.replay()
        torch.cuda.synchronize()
        assert int(step_dev[0]) == s + 1
        _, want_sel, _ = o_samp.stratified_sample(want_hash, 0, w.ratio[0], w.ratio[1], SEED, s)
        n = len(want_sel)
        assert sel_out[0][4].tolist()[0] == n and np.array_equal(sel_out[0][3].cpu().numpy()[:n], want_sel)
        seen.add(tuple(want_sel.tolist()))
        # the same step, eagerly, into the other buffers (this is also the eager work between two replays)
        step_dev.fill_(s)
        with torch.cuda.stream(main):
            step(ref, sel_out[1], main, side)
        torch.cuda.synchronize()
        for a, b in zip((bufs.xs, bufs.y, bufs.dxs, *bufs.dW), (ref.xs, ref.y, ref.dxs, *ref.dW)):
            a, b = a.reshape(-1), b.reshape(-1)
            k = w.B * n * w.d if a.numel() == w.B * n_max * w.d else a.numel()
            assert torch.equal(a[:k], b[:k]), r
        if r == 0:
            dy = dy_t.reshape(-1)[:w.B * n * w.d].view(w.B, n, w.d).float().cpu().numpy().astype(np.float64)
            want = oracle_attention(tok[:, want_sel, :], W, w.H, dy)
            errs = {"y": rel_err(bufs.packed(bufs.y, w.B, n), want["y"]), "dWq": rel_err(bufs.dW[0], want["dWq"]),
                    "dxs": rel_err(bufs.packed(bufs.dxs, w.B, n), want["dxs"])}
            assert all(e <= TOL[w.dtype] for e in errs.values()), errs
    assert len(seen) == 4


def test_embedding_of_the_kept_windows_with_the_count_on_the_device(vd, ctx):
    """Raw windows -> embedding of the kept variates -> attention forward / backward -> embedding gradients, every
    call reading the count on the device; tokens, outputs and all gradients against the oracle for several counts
    under one bound."""
    from oracle import embedding as o_emb
    rng = np.random.default_rng(11)
    B, N, L, d, H, n_max = 3, 150, 96, 128, 2, 128
    td = torch.bfloat16
    x = (rng.standard_normal((B, N, L)) * rng.uniform(0.1, 5.0, size=(1, N, 1)) + rng.uniform(-3, 3, size=(1, N, 1))).astype(np.float32)
    We = wl.quantise(rng.standard_normal((L, d)) / np.sqrt(L), "bf16")
    be = wl.quantise(0.1 * rng.standard_normal(d), "bf16")
    W = [wl.quantise(rng.standard_normal((d, d)) / np.sqrt(d), "bf16") for _ in range(4)]
    x_t, We_t, be_t, W_t = to_dev(x), to_dev(We, td), to_dev(be, td), [to_dev(m, td) for m in W]
    lib = vd.load_library()
    bufs = Buffers(vd, B, N, d, H, td, n_max)
    esaved = torch.empty(lib.vardrop_embed_saved_bytes(B, n_max, L, vd.BF16), dtype=torch.uint8, device="cuda")
    ews = torch.empty(lib.vardrop_embed_workspace_bytes(B, n_max, L, d, vd.BF16), dtype=torch.uint8, device="cuda")
    dWe = torch.empty((L, d), dtype=torch.float32, device="cuda")
    dbe = torch.empty((d,), dtype=torch.float32, device="cuda")
    n_dev = torch.zeros(1, dtype=torch.int32, device="cuda")
    for n in (128, 1, 77):
        sel_np = np.sort(rng.choice(N, size=n, replace=False))
        sel = torch.zeros(N, dtype=torch.int32, device="cuda")
        sel[:n] = to_dev(sel_np.astype(np.int32))
        dy = wl.quantise(rng.standard_normal((B, n, d)), "bf16")
        n_dev.fill_(n)
        vd.vardrop_embed_fwd_dev(ctx, x_t, sel, n_dev, n_max, We_t, be_t, bufs.xs, esaved, status=bufs.status)
        vd.vardrop_attn_fwd_dev(ctx, bufs.xs, n_dev, n_max, *W_t, H, bufs.y, bufs.saved, status=bufs.status)
        vd.vardrop_attn_bwd_dev(ctx, to_dev(dy, td), bufs.xs, n_dev, n_max, *W_t, H, bufs.saved, bufs.ws,
                                (bufs.dxs, *bufs.dW), status=bufs.status)
        vd.vardrop_embed_bwd_dev(ctx, bufs.dxs, n_dev, n_max, L, esaved, ews, (dWe, dbe))
        torch.cuda.synchronize()
        assert int(bufs.status[0]) == 0
        want_xs = o_emb.embed_forward(x, sel_np, We, be, True)
        xs = bufs.packed(bufs.xs, B, n)
        assert rel_err(xs, want_xs) <= TOL["bf16"]
        xs_r = xs.float().cpu().numpy().astype(np.float64)                # the attention sees the rounded tokens
        want = oracle_attention(xs_r, W, H, dy)
        got = dict(y=bufs.packed(bufs.y, B, n), dxs=bufs.packed(bufs.dxs, B, n), dWq=bufs.dW[0], dWo=bufs.dW[3])
        errs = {k: rel_err(v, want[k]) for k, v in got.items()}
        assert all(e <= TOL["bf16"] for e in errs.values()), (n, errs)
        dxs_r = bufs.packed(bufs.dxs, B, n).float().cpu().numpy().astype(np.float64)
        want_dWe, want_dbe = o_emb.embed_backward(x, sel_np, dxs_r, True)
        assert rel_err(dWe, want_dWe) <= TOL["bf16"] and rel_err(dbe, want_dbe) <= TOL["bf16"], n
    n_dev.fill_(129)
    vd.vardrop_embed_fwd_dev(ctx, x_t, sel, n_dev, n_max, We_t, be_t, bufs.xs, esaved, status=bufs.status)
    torch.cuda.synchronize()
    assert int(bufs.status[0]) == 1


def test_the_benchmark_pipeline_computes_the_same_steps_in_every_launch_mode(vd, ctx):
    """bench.py's Pipeline at the Traffic shape: the burst pipeline, the eager pipeline with every placement of the
    k-DFH and the sampling behind the attention kernels (completion signals) and the recorded graph all draw
    selection g with Philox step g and leave the same last step behind, bit for bit; that step is checked against
    the oracle."""
    import argparse
    import bench
    from oracle import sampling as o_samp
    w = wl.WORKLOADS["traffic"]
    td = torch.bfloat16
    dev = torch.device("cuda", 0)
    xs_dev, tok_dev, tok_np = [], [], []
    for i in range(2):
        x_np, _ = wl.make_signals(w, seed=i)
        t_np = wl.make_tokens(w, x_np, seed=i)
        xs_dev.append(torch.from_numpy(x_np).to(dev))
        tok_dev.append(torch.from_numpy(t_np).to(dev).to(td))
        tok_np.append(t_np)
    W_np = wl.make_weights(w, seed=0)
    W_dev = [torch.from_numpy(m).to(dev).to(td) for m in W_np]
    dy_np = wl.make_upstream(w, w.N, seed=0)
    dy_full = torch.from_numpy(dy_np).to(dev).to(td).reshape(-1)
    seed, K = 0x5EED, 9
    pipe = bench.Pipeline(vd, ctx, w, xs_dev, tok_dev, W_dev, dy_full, seed)
    args = argparse.Namespace(steps=K - 2, warmup=2)
    gates = bench.placements(pipe)
    assert len(gates) == len(bench.PLACEMENTS) and ("fwd", "bwd") in gates
    runs = [("burst", None)] + [("eager", g) for g in gates] + [("graph", None)]
    first = None
    for mode, gate in runs:
        if gate:
            bench.place(pipe, gate)
        for t in (pipe.y_buf, pipe.dxs_buf, pipe.xs_buf, *pipe.dW_buf):
            t.fill_(float("nan"))
        bench.timed_steps(pipe, args, mode)                    # (checks the status word and the step counter itself)
        torch.cuda.synchronize()
        g = K - 1
        r = g % (2 if mode == "graph" else pipe.RING)
        n, G = pipe.ring[r][4].tolist()
        sel = pipe.ring[r][3][:n].cpu().numpy()
        hsh = pipe.ring[r][1].cpu().numpy().view(np.uint64)
        _, want_sel, want_G = o_samp.stratified_sample(hsh, 0, w.ratio[0], w.ratio[1], seed, g)
        assert (n, G) == (len(want_sel), want_G) and np.array_equal(sel, want_sel), (mode, gate)
        cnt = w.B * n * w.d
        got = dict(y=pipe.y_buf.reshape(-1)[:cnt].view(w.B, n, w.d).clone(), dxs=pipe.dxs_buf.reshape(-1)[:cnt].view(w.B, n, w.d).clone(),
                   dWq=pipe.dW_buf[0].clone(), dWk=pipe.dW_buf[1].clone(), dWv=pipe.dW_buf[2].clone(), dWo=pipe.dW_buf[3].clone())
        if first is None:
            first = got
            b = g % 2
            tok_r = tok_dev[b].float().cpu().numpy().astype(np.float64)
            W_r = [m.float().cpu().numpy().astype(np.float64) for m in W_dev]
            dy_r = dy_full[:cnt].view(w.B, n, w.d).float().cpu().numpy().astype(np.float64)
            want = oracle_attention(tok_r[:, want_sel, :], W_r, w.H, dy_r)
            errs = {k: rel_err(v, want[k]) for k, v in got.items()}
            assert all(e <= TOL["bf16"] for e in errs.values()), errs
        else:
            for k in got:
                assert torch.equal(got[k], first[k]), (mode, gate, k)
