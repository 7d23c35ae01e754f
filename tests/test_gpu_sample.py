"""GPU grouping + stratified sampling (vardrop_sample) against the oracle: bit-exact."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import sampling as o_samp

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vd():
    import paper_2501_14183_amd as m
    return m


@pytest.fixture(scope="module")
def ctx(vd):
    return vd.Context(0)


def run(vd, ctx, hashes, gs, num, den, seed, step, pinned=None):
    h = torch.from_numpy(np.asarray(hashes, dtype=np.uint64).view(np.int64)).cuda()
    gid, sel, counts = vd.vardrop_sample(ctx, h, gs, num, den, seed, step, counts_host=pinned)
    torch.cuda.synchronize()
    n_sel, G = (int(v) for v in counts.cpu())
    return gid.cpu().numpy().astype(np.int64), sel.cpu().numpy()[:n_sel].astype(np.int64), n_sel, G


def check(vd, ctx, hashes, gs, num, den, seed, step):
    want_gid, want_sel, want_G = o_samp.stratified_sample(hashes, gs, num, den, seed, step)
    gid, sel, n_sel, G = run(vd, ctx, hashes, gs, num, den, seed, step)
    assert G == want_G and n_sel == len(want_sel)
    assert np.array_equal(gid, want_gid)
    assert np.array_equal(sel, want_sel)
    return gid, sel


@pytest.mark.parametrize("name", wl.ORDER)
def test_five_workloads_bit_exact(vd, ctx, name):
    from util_gpu import workload_inputs, SEED, STEP
    w, x, info, topk, hsh, abar = workload_inputs(name)
    gid, sel = check(vd, ctx, hsh, 0, w.ratio[0], w.ratio[1], SEED, STEP)           # the configured keep ratio
    sizes = np.bincount(gid)
    kept = np.bincount(gid[sel], minlength=len(sizes))
    assert np.all(kept >= 1)
    assert kept.tolist() == [o_samp.keep_count(int(g), 0, *w.ratio) for g in sizes]
    for gs in (1, 5, 10, 20):                                                       # Eq. 1 as printed
        gid, sel = check(vd, ctx, hsh, gs, 1, 1, SEED, STEP + gs)
        kept = np.bincount(gid[sel], minlength=len(sizes))
        assert kept.tolist() == [min(int(g), gs) for g in sizes]
    print("%s: G=%d N'=%d delta=%.4f" % (name, len(sizes), len(sel), o_samp.reduction_ratio(w.N, len(sel))))


@pytest.mark.parametrize("N,n_distinct", [(1, 1), (2, 1), (3, 3), (64, 5), (65, 7), (129, 129), (1000, 40),
                                          (4097, 300), (8192, 1), (8192, 8192), (8191, 977)])
def test_sizes_and_degenerate_groupings(vd, ctx, N, n_distinct):
    rng = np.random.default_rng(N + n_distinct)
    pool = rng.integers(0, 2 ** 63, size=n_distinct, dtype=np.uint64)
    if n_distinct == N:
        hashes = rng.permutation(np.unique(rng.integers(0, 2 ** 63, size=4 * N, dtype=np.uint64))[:N])
    else:
        hashes = pool[rng.integers(0, n_distinct, size=N)]
    check(vd, ctx, hashes, 0, 1, 10, seed=N, step=3)
    check(vd, ctx, hashes, 3, 1, 1, seed=2 ** 63 + 5, step=2 ** 40 + N)
    check(vd, ctx, hashes, 7, 2, 3, seed=1, step=0)
    gid, sel = check(vd, ctx, hashes, 0, 1, 1, seed=1, step=1)
    assert sel.tolist() == list(range(N))                                           # nothing dropped


def test_extreme_hash_values_and_new_selection_every_step(vd, ctx):
    hashes = np.array([2 ** 64 - 1, 0, 2 ** 63, 2 ** 64 - 1, 0, 1, 2 ** 64 - 2] * 9, dtype=np.uint64)
    check(vd, ctx, hashes, 2, 1, 1, 11, 12)
    sels = set()
    for step in range(20):
        _, sel = check(vd, ctx, hashes, 2, 1, 1, 99, step)
        sels.add(tuple(sel.tolist()))
    assert len(sels) > 10


def test_counts_reach_pinned_host_memory_and_runs_are_deterministic(vd, ctx):
    rng = np.random.default_rng(0)
    hashes = rng.integers(0, 50, size=3000).astype(np.uint64)
    pinned = torch.zeros(2, dtype=torch.int32).pin_memory()
    a = run(vd, ctx, hashes, 4, 1, 3, 5, 6, pinned=pinned)
    assert pinned.tolist() == [a[2], a[3]]
    b = run(vd, ctx, hashes, 4, 1, 3, 5, 6)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_error_codes(vd, ctx):
    h = torch.zeros(10, dtype=torch.int64, device="cuda")
    for args, code in [((0, 2, 1, 0, 0), -1), ((0, 1, 0, 0, 0), -1)]:
        with pytest.raises(vd.VarDropError) as e:
            vd.vardrop_sample(ctx, h, *args)
        assert e.value.code == code
    with pytest.raises(vd.VarDropError) as e:
        vd.vardrop_sample(ctx, torch.zeros(8193, dtype=torch.int64, device="cuda"), 0, 1, 1, 0, 0)
    assert e.value.code == -4
