"""The whole hot path through the C ABI, as the benchmark runs it, against the oracle."""
import numpy as np
import pytest
import torch

import workloads as wl
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
