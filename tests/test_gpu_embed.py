"""GPU embedding of the kept variates (vardrop_embed_fwd / bwd) against the fp64 oracle."""
import numpy as np
import pytest
import torch

import util_gpu
import workloads as wl
from oracle import embedding as o_emb
from oracle import sampling as o_samp
from util_gpu import SEED, STEP, TOL, rel_err, to_dev, torch_dtype

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vd():
    import paper_2501_14183_amd as m
    return m


@pytest.fixture(scope="module")
def ctx(vd):
    return vd.Context(0)


def embedding_weights(L, d, dtype, seed):
    """Seeded L x d map and bias, already representable in `dtype` (the oracle gets the same values)."""
    rng = np.random.default_rng([0xE3BED, seed, L, d])
    We = wl.quantise(rng.standard_normal((L, d)) / np.sqrt(L), dtype)
    be = wl.quantise(0.1 * rng.standard_normal(d), dtype)
    return We, be


def check(vd, ctx, x, sel, d, dtype, standardise=True, bias=True, seed=0):
    B, N, L = x.shape
    n_sel = len(sel)
    We, be = embedding_weights(L, d, dtype, seed)
    rng = np.random.default_rng([0xD75, seed])
    dxs = wl.quantise(rng.standard_normal((B, n_sel, d)), dtype)
    td = torch_dtype(dtype)
    xd, seld = to_dev(x), to_dev(np.asarray(sel, dtype=np.int32))
    xs, saved = vd.vardrop_embed_fwd(ctx, xd, seld, n_sel, to_dev(We, td), to_dev(be, td) if bias else None, standardise)
    dWe, dbe = vd.vardrop_embed_bwd(ctx, to_dev(dxs, td), L, saved, want_bias=bias)
    torch.cuda.synchronize()
    want = o_emb.embed_forward(x, sel, We, be if bias else None, standardise)
    want_dWe, want_dbe = o_emb.embed_backward(x, sel, dxs, standardise)
    tol = TOL[dtype]
    assert rel_err(xs, want) <= tol
    assert rel_err(dWe, want_dWe) <= tol
    if bias:
        assert rel_err(dbe, want_dbe) <= tol
    return xs


@pytest.mark.parametrize("name", wl.ORDER)
def test_five_workloads(vd, ctx, name):
    """The kept variates of each workload (oracle selection), embedded from the raw windows."""
    w, x, info, topk, hsh, abar = util_gpu.workload_inputs(name)
    gid, sel, G = o_samp.stratified_sample(hsh, 0, w.ratio[0], w.ratio[1], SEED, STEP)
    if name == "stress":
        x, sel = x[:2], sel[:400]                       # (the fp64 oracle loops over every kept window)
    check(vd, ctx, x, np.asarray(sel), w.d, w.dtype)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("B,N,L,d,n_sel", [(1, 5, 8, 8, 1), (3, 40, 96, 64, 7), (2, 70, 200, 136, 65), (5, 9, 1024, 24, 9),
                                            (2, 300, 336, 512, 130)])
def test_ragged_shapes_raw_and_standardised(vd, ctx, dtype, B, N, L, d, n_sel):
    rng = np.random.default_rng([B, N, L, d])
    x = (rng.standard_normal((B, N, L)) * rng.uniform(0.1, 10, (1, N, 1)) + rng.uniform(-3, 3, (1, N, 1))).astype(np.float32)
    sel = np.sort(rng.choice(N, n_sel, replace=False))
    check(vd, ctx, x, sel, d, dtype, standardise=True, bias=True, seed=1)
    check(vd, ctx, x, sel, d, dtype, standardise=False, bias=False, seed=2)


def test_kept_only_equals_gather_of_the_full_embedding(vd, ctx):
    """Rows of the kept-only embedding are bit-identical to the same rows of the all-variate embedding."""
    rng = np.random.default_rng(3)
    B, N, L, d = 4, 50, 96, 128
    x = to_dev(rng.standard_normal((B, N, L)).astype(np.float32))
    We, be = embedding_weights(L, d, "bf16", 0)
    Wd, bd = to_dev(We, torch.bfloat16), to_dev(be, torch.bfloat16)
    sel = np.sort(rng.choice(N, 11, replace=False)).astype(np.int32)
    full, _ = vd.vardrop_embed_fwd(ctx, x, to_dev(np.arange(N, dtype=np.int32)), N, Wd, bd)
    kept, _ = vd.vardrop_embed_fwd(ctx, x, to_dev(sel), len(sel), Wd, bd)
    torch.cuda.synchronize()
    assert torch.equal(kept, full[:, torch.from_numpy(sel).long().cuda(), :])


def test_strided_batch_constant_window_and_bad_index(vd, ctx):
    rng = np.random.default_rng(4)
    big = rng.standard_normal((3, 12, 100)).astype(np.float32)
    big[:, 5, :] = 2.5                                                     # a constant variate: zeros after standardisation
    view = to_dev(big)[:, 1:11, :96]                                       # non-contiguous rows
    sel = np.array([0, 4, 7], dtype=np.int32)                              # row 4 of the view is variate 5
    We, be = embedding_weights(96, 64, "fp32", 0)
    xs, _ = vd.vardrop_embed_fwd(ctx, view, to_dev(sel), 3, to_dev(We), to_dev(be))
    torch.cuda.synchronize()
    want = o_emb.embed_forward(big[:, 1:11, :96], sel, We, be)
    assert rel_err(xs, want) <= TOL["fp32"]
    assert np.allclose(xs[:, 1].cpu().numpy(), be, atol=1e-6)
    bad = to_dev(np.array([2, 99], dtype=np.int32))                        # 99 is outside 0..N-1: a zero window
    xs, _ = vd.vardrop_embed_fwd(ctx, view, bad, 2, to_dev(We), None, standardise=False)
    torch.cuda.synchronize()
    assert torch.count_nonzero(xs[:, 1]) == 0


def test_empty_selection_and_error_codes(vd, ctx):
    x = torch.zeros((2, 6, 96), device="cuda")
    We = torch.zeros((96, 64), device="cuda", dtype=torch.bfloat16)
    sel = torch.zeros((6,), device="cuda", dtype=torch.int32)
    xs, saved = vd.vardrop_embed_fwd(ctx, x, sel, 0, We)
    assert xs.shape == (2, 0, 64)
    dWe, dbe = vd.vardrop_embed_bwd(ctx, xs, 96, saved)
    torch.cuda.synchronize()
    assert torch.count_nonzero(dWe) == 0 and torch.count_nonzero(dbe) == 0
    with pytest.raises(vd.VarDropError) as e:
        vd.vardrop_embed_fwd(ctx, x, sel, 7, We)                           # more kept variates than variates
    assert e.value.code == -1
    with pytest.raises(vd.VarDropError) as e:
        vd.vardrop_embed_fwd(ctx, torch.zeros((2, 6, 100), device="cuda"), sel, 3,
                             torch.zeros((100, 60), device="cuda", dtype=torch.bfloat16))   # d, L not multiples of 8
    assert e.value.code == -4
    with pytest.raises(vd.VarDropError) as e:
        vd.vardrop_embed_fwd(ctx, torch.zeros((1, 2, 2048), device="cuda"), sel, 1, torch.zeros((2048, 64), device="cuda"))
    assert e.value.code == -4
