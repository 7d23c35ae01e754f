"""The whole hot path through the C ABI, as the benchmark runs it, against the oracle."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import sampling as o_samp
from util_gpu import SEED, STEP, TOL, elem_err, oracle_attention, rel_err, to_dev, torch_dtype, workload_inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vd():
    import paper_2501_14183_amd as m
    return m


@pytest.fixture(scope="module")
def ctx(vd):
    return vd.Context(0)


@pytest.mark.parametrize("name", wl.ORDER)
def test_step_matches_oracle(vd, ctx, name):
    w, x, info, want_topk, want_hash, _ = workload_inputs(name)
    td = torch_dtype(w.dtype)
    tok = wl.make_tokens(w, x)
    W = wl.make_weights(w)
    x_t, tok_t = to_dev(x), to_dev(tok, td)
    W_t = [to_dev(m, td) for m in W]
    pinned = torch.zeros(2, dtype=torch.int32).pin_memory()

    topk, hsh, _ = vd.vardrop_hash(ctx, x_t, w.k)
    gid, sel, counts = vd.vardrop_sample(ctx, hsh, 0, w.ratio[0], w.ratio[1], SEED, STEP, counts_host=pinned)
    torch.cuda.current_stream().synchronize()
    n_sel, G = int(pinned[0]), int(pinned[1])
    xs = vd.vardrop_gather(ctx, tok_t, sel, n_sel)
    y, saved = vd.vardrop_attn_fwd(ctx, xs, *W_t, w.H)
    dy = wl.make_upstream(w, n_sel)
    dxs, dWq, dWk, dWv, dWo = vd.vardrop_attn_bwd(ctx, to_dev(dy, td), xs, *W_t, w.H, saved)
    dtok = vd.vardrop_scatter(ctx, dxs, sel, n_sel, w.N)
    torch.cuda.synchronize()

    want_gid, want_sel, want_G = o_samp.stratified_sample(want_hash, 0, w.ratio[0], w.ratio[1], SEED, STEP)
    assert np.array_equal(topk.cpu().numpy(), want_topk)
    assert np.array_equal(hsh.cpu().numpy().view(np.uint64), want_hash)
    assert (n_sel, G) == (len(want_sel), want_G)
    assert np.array_equal(gid.cpu().numpy(), want_gid)
    assert np.array_equal(sel.cpu().numpy()[:n_sel], want_sel)
    assert np.array_equal(xs.float().cpu().numpy(), tok[:, want_sel, :])
    want = oracle_attention(tok[:, want_sel, :], W, w.H, dy)
    got = dict(y=y, dxs=dxs, dWq=dWq, dWk=dWk, dWv=dWv, dWo=dWo)
    errs = {k: rel_err(v, want[k]) for k, v in got.items()}
    assert all(e <= TOL[w.dtype] for e in errs.values()), errs
    kept = np.zeros(w.N, dtype=bool)
    kept[want_sel] = True
    d_np = dtok.float().cpu().numpy()
    assert np.all(d_np[:, ~kept] == 0) and np.array_equal(d_np[:, kept], dxs.float().cpu().numpy())
    print("%s: G=%d N'=%d redrawn=%d errs=%s" % (name, G, n_sel, info["redrawn"], {k: "%.1e" % v for k, v in errs.items()}))


@pytest.mark.parametrize("name", wl.ORDER)
def test_gather_fused_into_the_forward_pass(vd, ctx, name):
    """vardrop_gather_attn_fwd: the kept tokens and the attention output against the oracle, and bit for bit
    against vardrop_gather followed by vardrop_attn_fwd (short selections gather inside the forward kernel,
    long ones and fp32 run the two steps)."""
    w, x, info, _, want_hash, _ = workload_inputs(name)
    td = torch_dtype(w.dtype)
    tok = wl.make_tokens(w, x)
    W = wl.make_weights(w)
    b = wl.make_biases(w)
    tok_t = to_dev(tok, td)
    W_t = [to_dev(m, td) for m in W]
    b_t = [to_dev(m, td) for m in b]
    _, want_sel, _ = o_samp.stratified_sample(want_hash, 0, w.ratio[0], w.ratio[1], SEED, STEP)
    cases = [want_sel, want_sel[:1], np.arange(min(w.N, 128)), np.arange(min(w.N, 129)), np.array([w.N - 1])]
    for sel_np in cases:
        n = len(sel_np)
        sel = torch.zeros(w.N, dtype=torch.int32, device="cuda")
        sel[:n] = torch.from_numpy(np.asarray(sel_np, dtype=np.int32)).cuda()
        xs, y, saved = vd.vardrop_gather_attn_fwd(ctx, tok_t, sel, n, *W_t, w.H, *b_t)
        xs2 = vd.vardrop_gather(ctx, tok_t, sel, n)
        y2, saved2 = vd.vardrop_attn_fwd(ctx, xs2, *W_t, w.H, *b_t)
        torch.cuda.synchronize()
        assert np.array_equal(xs.float().cpu().numpy(), tok[:, sel_np, :])
        assert torch.equal(xs, xs2) and torch.equal(y, y2)
        from oracle import attention as o_att
        want, _ = o_att.mha_forward(tok[:, sel_np, :].astype(np.float64), *[m.astype(np.float64) for m in W], w.H,
                                    *[m.astype(np.float64) for m in b])
        assert rel_err(y, want) <= TOL[w.dtype]
        fine = elem_err(y, want, w.dtype)
        assert fine[0] <= 1.0 and fine[1] <= 1.0, fine
        # the backward pass reads the kept tokens the fused call wrote
        dy = to_dev(wl.make_upstream(w, n), td)
        g1 = vd.vardrop_attn_bwd(ctx, dy, xs, *W_t, w.H, saved)
        g2 = vd.vardrop_attn_bwd(ctx, dy, xs2, *W_t, w.H, saved2)
        torch.cuda.synchronize()
        assert all(torch.equal(u, v) for u, v in zip(g1, g2))


def test_out_of_range_index_gives_a_zero_row_in_the_fused_gather(vd, ctx):
    """An index outside [0, N) stands for a zero row, inside the forward kernel (short selections) as in the gather
    kernel (long ones): the fused call equals the two separate calls, no row of another batch element is read,
    and the zero rows attend like tokens of zeros."""
    rng = np.random.default_rng(3)
    B, N, d, H = 2, 300, 128, 2
    tok = to_dev(rng.standard_normal((B, N, d)).astype(np.float32), torch.bfloat16)
    W = [to_dev((rng.standard_normal((d, d)) / np.sqrt(d)).astype(np.float32), torch.bfloat16) for _ in range(4)]
    for n in (40, 128, 200):
        sel_np = np.sort(rng.choice(N, size=n, replace=False)).astype(np.int32)
        bad = [0, n // 2, n - 1]
        sel_np[bad] = [-1, N, 2 ** 31 - 1]
        sel = to_dev(sel_np)
        xs, y, _ = vd.vardrop_gather_attn_fwd(ctx, tok, sel, n, *W, H)
        xs2 = vd.vardrop_gather(ctx, tok, sel, n)
        y2, _ = vd.vardrop_attn_fwd(ctx, xs2, *W, H)
        torch.cuda.synchronize()
        assert xs[:, bad].eq(0).all() and torch.equal(xs, xs2)
        assert torch.equal(y, y2)
        clean = tok.clone()
        sel_ok = sel_np.copy()
        sel_ok[bad] = [0, 1, 2]
        want_xs = clean[:, to_dev(sel_ok.astype(np.int64))]
        want_xs[:, bad] = 0
        assert torch.equal(xs, want_xs)


def test_gather_fused_error_codes(vd, ctx):
    tok = torch.zeros((2, 10, 128), dtype=torch.bfloat16, device="cuda")
    W = [torch.zeros((128, 128), dtype=torch.bfloat16, device="cuda") for _ in range(4)]
    sel = torch.arange(10, dtype=torch.int32, device="cuda")
    with pytest.raises(vd.VarDropError) as e:
        vd.vardrop_gather_attn_fwd(ctx, tok, sel, 11, *W, 2)              # more kept rows than variates
    assert e.value.code == -1
    with pytest.raises(vd.VarDropError) as e:
        vd.vardrop_gather_attn_fwd(ctx, tok, None, 4, *W, 2)
    assert e.value.code == -1
    xs, y, _ = vd.vardrop_gather_attn_fwd(ctx, tok, sel, 0, *W, 2)       # nothing kept: a no-op
    assert xs.shape == (2, 0, 128)


def test_pipelined_steps_in_the_benchmark_configuration(vd, ctx):
    """Traffic-shaped batch, launched the way bench.py launches it: selection on a second stream a step ahead
    through raw stream handles, a ring of selection buffers, outputs written into buffers sized for all N
    variates and viewed at N'; three consecutive steps (new selection each), every one against the oracle."""
    w, x, info, want_topk, want_hash, _ = workload_inputs("traffic")
    td = torch_dtype(w.dtype)
    tok = wl.make_tokens(w, x)
    W = wl.make_weights(w)
    x_t, tok_t = to_dev(x), to_dev(tok, td)
    W_t = [to_dev(m, td) for m in W]
    dev = x_t.device
    main, side = torch.cuda.current_stream(), torch.cuda.Stream(device=dev)
    main_h, side_h = main.cuda_stream, side.cuda_stream
    lib = vd.load_library()
    saved = torch.empty(lib.vardrop_attn_saved_bytes(w.B, w.N, w.d, w.H, vd.BF16), dtype=torch.uint8, device=dev)
    ws = torch.empty(lib.vardrop_attn_workspace_bytes(w.B, w.N, w.d, w.H, vd.BF16), dtype=torch.uint8, device=dev)
    xs_buf, y_buf, dxs_buf = (torch.empty(w.B * w.N * w.d, dtype=td, device=dev) for _ in range(3))
    dW_buf = [torch.empty((w.d, w.d), dtype=torch.float32, device=dev) for _ in range(4)]
    ring = 3
    bufs = [(torch.empty((w.N, w.k), dtype=torch.int32, device=dev), torch.empty(w.N, dtype=torch.int64, device=dev),
             torch.empty(w.N, dtype=torch.int32, device=dev), torch.empty(w.N, dtype=torch.int32, device=dev),
             torch.empty(2, dtype=torch.int32, device=dev)) for _ in range(ring)]
    pinned = [torch.zeros(2, dtype=torch.int32).pin_memory() for _ in range(ring)]
    events = [torch.cuda.Event() for _ in range(ring)]
    torch.cuda.synchronize()

    def select(i):
        topk, hsh, gid, sel, counts = bufs[i % ring]
        vd.vardrop_hash(ctx, x_t, w.k, out=(topk, hsh), stream=side_h)
        vd.vardrop_sample(ctx, hsh, 0, w.ratio[0], w.ratio[1], SEED, STEP + i, counts_host=pinned[i % ring],
                          out=(gid, sel, counts), stream=side_h)
        events[i % ring].record(side)

    steps = 3
    select(0)
    for i in range(steps):
        if i + 1 < steps:
            select(i + 1)
        events[i % ring].synchronize()
        n_sel, G = int(pinned[i % ring][0]), int(pinned[i % ring][1])
        sel = bufs[i % ring][3]
        count, shape = w.B * n_sel * w.d, (w.B, n_sel, w.d)
        xs, y, _ = vd.vardrop_gather_attn_fwd(ctx, tok_t, sel, n_sel, *W_t, w.H, saved=saved,
                                              out=(xs_buf[:count].view(shape), y_buf[:count].view(shape)), stream=main_h)
        dy = wl.make_upstream(w, n_sel)
        grads = vd.vardrop_attn_bwd(ctx, to_dev(dy, td), xs, *W_t, w.H, saved, ws=ws,
                                    out=(dxs_buf[:count].view(shape), *dW_buf), stream=main_h)
        torch.cuda.synchronize()          # the check below reads the buffers the next step reuses
        want_gid, want_sel, want_G = o_samp.stratified_sample(want_hash, 0, w.ratio[0], w.ratio[1], SEED, STEP + i)
        assert (n_sel, G) == (len(want_sel), want_G)
        assert np.array_equal(bufs[i % ring][0].cpu().numpy(), want_topk)
        assert np.array_equal(sel.cpu().numpy()[:n_sel], want_sel)
        assert np.array_equal(xs.float().cpu().numpy(), tok[:, want_sel, :])
        want = oracle_attention(tok[:, want_sel, :], W, w.H, dy)
        got = dict(zip(("dxs", "dWq", "dWk", "dWv", "dWo"), grads), y=y)
        errs = {k: rel_err(v, want[k]) for k, v in got.items()}
        assert all(e <= TOL[w.dtype] for e in errs.values()), (i, errs)


def test_completion_signal_rides_on_the_kernel_and_is_one_shot(vd, ctx):
    """vardrop_signal_after: the event completes with the named kernel's launch, a second stream that waits for it
    sees the kernel's output, the request is consumed by one launch, and an unknown id is refused."""
    torch.manual_seed(3)
    B, N, d, n = 4, 640, 512, 200
    tok = torch.randn(B, N, d, device="cuda").to(torch.bfloat16)
    sel = torch.sort(torch.randperm(N, device="cuda")[:n]).values.to(torch.int32)
    kid = {vd.vardrop_kernel_name(k): k for k in range(64) if vd.vardrop_kernel_name(k)}
    main, side = torch.cuda.Stream(), torch.cuda.Stream()
    ev = torch.cuda.Event()
    ev.record(main)                                   # creates the event; its handle is what the library is given
    main.synchronize()
    out = torch.zeros(B, n, d, dtype=torch.bfloat16, device="cuda")
    copy = torch.zeros_like(out)
    torch.cuda.synchronize()
    for _ in range(3):
        out.zero_()
        copy.zero_()
        torch.cuda.synchronize()
        vd.vardrop_signal_after(ctx, kid["gather"], ev.cuda_event)
        vd.vardrop_gather(ctx, tok, sel, n, out=out, stream=main.cuda_stream)
        side.wait_event(ev)
        with torch.cuda.stream(side):
            copy.copy_(out)
        side.synchronize()
        assert ev.query()
        assert torch.equal(copy, tok[:, sel.long(), :])
    # consumed: the next launch carries nothing and can be timed as usual
    vd.vardrop_profile_select(ctx, kid["gather"])
    vd.vardrop_gather(ctx, tok, sel, n, out=out, stream=main.cuda_stream)
    main.synchronize()
    ms, launches = vd.vardrop_profile_read(ctx)
    vd.vardrop_profile_select(ctx, -1)
    assert launches == 1 and ms > 0
    with pytest.raises(vd.VarDropError):
        vd.vardrop_signal_after(ctx, 1000, ev.cuda_event)
    vd.vardrop_signal_after(ctx, kid["gather"], None)      # cancelling is allowed


def test_two_kernels_of_one_call_can_each_carry_a_signal(vd, ctx):
    """One request can be pending per kernel id: the forward attention kernel and the output projection of one
    vardrop_attn_fwd call each complete their own event, in launch order, and a request for a kernel the call does
    not launch stays pending without disturbing it."""
    w = wl.WORKLOADS["electricity"]
    td = torch_dtype(w.dtype)
    rng = np.random.default_rng(11)
    n = 96
    xs = to_dev(wl.quantise(rng.standard_normal((w.B, n, w.d)), w.dtype), td)
    W_t = [to_dev(m, td) for m in wl.make_weights(w)]
    kid = {vd.vardrop_kernel_name(k): k for k in range(64) if vd.vardrop_kernel_name(k)}
    main = torch.cuda.Stream()
    events = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    for ev in events:
        ev.record(main)
    main.synchronize()
    y0, _ = vd.vardrop_attn_fwd(ctx, xs, *W_t, w.H)
    torch.cuda.synchronize()
    lib = vd.load_library()
    code = vd.BF16
    saved = torch.empty(lib.vardrop_attn_saved_bytes(w.B, n, w.d, w.H, code), dtype=torch.uint8, device="cuda")
    y = torch.empty_like(y0)
    vd.vardrop_signal_after(ctx, kid["qkv_sdpa_fwd"], events[0].cuda_event)
    vd.vardrop_signal_after(ctx, kid["gemm_out"], events[1].cuda_event)
    vd.vardrop_signal_after(ctx, kid["scatter"], events[2].cuda_event)         # not launched by this call
    vd.vardrop_attn_fwd(ctx, xs, *W_t, w.H, saved=saved, out=y, stream=main.cuda_stream)
    events[1].synchronize()
    assert events[0].query() and events[1].query()
    assert events[0].elapsed_time(events[1]) > 0                                # the projection finished later
    main.synchronize()
    assert torch.equal(y, y0)
    vd.vardrop_signal_after(ctx, kid["scatter"], None)
