"""GPU k-DFH (vardrop_hash) against the fp64 oracle: ranked top-k and hash bit-exact."""
import numpy as np
import pytest
import torch

import util_gpu
import workloads as wl
from oracle import kdfh as o_kdfh

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vd():
    import paper_2501_14183_amd as m
    return m


@pytest.fixture(scope="module")
def ctx(vd):
    return vd.Context(0)


def run(vd, ctx, x, k, f_min=1, f_max=None):
    xt = x if isinstance(x, torch.Tensor) else torch.from_numpy(np.ascontiguousarray(x)).cuda()
    topk, hsh, abar = vd.vardrop_hash(ctx, xt, k, f_min, f_max, want_abar=True)
    torch.cuda.synchronize()
    return topk.cpu().numpy().astype(np.int64), hsh.cpu().numpy().view(np.uint64), abar.cpu().numpy()


def compare(vd, ctx, x, k, f_min=1, f_max=None):
    L = x.shape[-1]
    fm = o_kdfh.default_cutoff(L) if f_max is None else f_max
    want_topk, want_hash, want_abar = o_kdfh.kdfh(x, k, f_min, fm)
    topk, hsh, abar = run(vd, ctx, x, k, f_min, f_max)
    scale = np.abs(want_abar).max(axis=1, keepdims=True)
    scale[scale == 0] = 1.0
    assert np.all(np.abs(abar - want_abar) <= 2e-5 * scale)
    ok = o_kdfh.gap_ok(want_abar, k)
    flips = int((topk != want_topk).any(axis=1).sum())
    flips_screened = int((topk[ok] != want_topk[ok]).any(axis=1).sum())
    return topk, hsh, want_topk, want_hash, flips, flips_screened, ok


@pytest.mark.parametrize("name", wl.ORDER)
def test_five_workloads_bit_exact(vd, ctx, name):
    from util_gpu import workload_inputs
    w, x, info, want_topk, want_hash, want_abar = workload_inputs(name)
    assert info["unresolved"] == 0
    topk, hsh, abar = run(vd, ctx, x, w.k)
    assert np.array_equal(topk, want_topk)
    assert np.array_equal(hsh, want_hash)
    scale = np.abs(want_abar).max(axis=1, keepdims=True)
    assert np.all(np.abs(abar - want_abar) <= 2e-5 * scale)
    # the unscreened draw of the same workload: rank flips may only occur below the 1e-3 gap
    w, xu, _, tu, hu, au = workload_inputs(name, screened=False)
    t2, h2, _ = run(vd, ctx, xu, w.k)
    ok = o_kdfh.gap_ok(au, w.k)
    assert np.array_equal(t2[ok], tu[ok])
    below = int((t2[~ok] != tu[~ok]).any(axis=1).sum())
    print("%s: %d variates below the gap, %d rank flips among them" % (name, int((~ok).sum()), below))


def test_planted_sinusoids_and_order(vd, ctx):
    L = 96
    t = np.arange(L)
    x = np.zeros((4, 3, L), dtype=np.float32)
    for n, (fs, amps) in enumerate([((4, 12, 8), (3, 2, 1)), ((12, 4, 8), (3, 2, 1)), ((5, 24, 1), (1.0, 0.8, 0.5))]):
        for b in range(4):
            x[b, n] = sum(a * np.sin(2 * np.pi * f * t / L + 0.37 * b + f) for f, a in zip(fs, amps))
    topk, hsh, _ = run(vd, ctx, x, 3)
    assert topk.tolist() == [[4, 12, 8], [12, 4, 8], [5, 24, 1]]
    assert hsh[0] != hsh[1] and int(hsh[0]) == (4 * 49 + 12) * 49 + 8


def test_flat_variate_hashes_to_lowest_bins(vd, ctx):
    topk, hsh, abar = run(vd, ctx, np.zeros((8, 5, 96), dtype=np.float32), 3)
    assert topk.tolist() == [[1, 2, 3]] * 5 and np.all(abar == 0)
    topk, _, _ = run(vd, ctx, np.zeros((2, 3, 512), dtype=np.float32), 5)
    assert topk.tolist() == [[1, 2, 3, 4, 5]] * 3


@pytest.mark.parametrize("B,N,L,k", [(1, 7, 96, 3), (5, 13, 96, 3), (32, 3, 96, 2), (33, 5, 96, 3), (70, 4, 64, 4),
                                      (3, 40, 97, 3), (6, 9, 98, 2), (2, 5, 10, 2), (4, 3, 2, 1), (16, 37, 336, 4),
                                      (8, 11, 512, 5), (33, 2, 896, 6)])
def test_shapes_and_ragged_edges(vd, ctx, B, N, L, k):
    rng = np.random.default_rng(B * 1000 + L)
    x = rng.standard_normal((B, N, L)).astype(np.float32)
    t = np.arange(L)
    for n in range(N):                                   # a few dominant lines on top of the noise
        for j, f in enumerate(rng.choice(np.arange(1, max(2, L // 4)), size=min(3, max(1, L // 4 - 1)), replace=False)):
            x[:, n] += (4.0 / (1 + j)) * np.sin(2 * np.pi * f * t / L + rng.uniform(0, 6, size=(B, 1))).astype(np.float32)
    topk, hsh, want_topk, want_hash, flips, flips_screened, ok = compare(vd, ctx, x, k)
    assert flips_screened == 0
    assert np.array_equal(hsh[ok], want_hash[ok])
    assert flips <= (~ok).sum()


@pytest.mark.parametrize("B,N,L,k,f_min,f_max", [(8, 4099, 512, 5, 1, None), (40, 530, 448, 4, 1, None),
                                                  (3, 8200, 384, 3, 1, None), (16, 2060, 512, 4, 0, 256),
                                                  (8, 4100, 400, 3, 3, 66)])
def test_long_windows_with_many_row_blocks_per_compute_unit(vd, ctx, B, N, L, k, f_min, f_max):
    """Shapes that take the pipelined kernel (long aligned windows, at least four row blocks per compute unit): a
    ragged last group, more than 32 windows per variate (two row blocks per group), groups of 8 variates, candidate
    ranges with and without the mean and the Nyquist bin and with one or two bins beside the tiles."""
    rng = np.random.default_rng(B * 1000 + L + N)
    x = rng.standard_normal((B, N, L)).astype(np.float32)
    t = np.arange(L)
    lo, hi = max(f_min, 1), (o_kdfh.default_cutoff(L) if f_max is None else min(f_max, L // 2 - 1))
    lines = rng.integers(lo, hi + 1, size=(N, 3))
    phase = rng.uniform(0, 6, size=(B, N, 3))
    for j in range(3):
        x += ((4.0 / (1 + j)) * np.sin(2 * np.pi * lines[None, :, j, None] * t[None, None, :] / L + phase[:, :, j, None])).astype(np.float32)
    x *= np.exp(rng.uniform(-3, 3, size=(1, N, 1))).astype(np.float32)            # per-variate scale
    topk, hsh, want_topk, want_hash, flips, flips_screened, ok = compare(vd, ctx, x, k, f_min=f_min, f_max=f_max)
    assert flips_screened == 0 and ok.sum() >= N // 2
    assert np.array_equal(hsh[ok], want_hash[ok])
    assert flips <= (~ok).sum()


def test_candidate_range_parameters(vd, ctx):
    rng = np.random.default_rng(3)
    x = (rng.standard_normal((4, 6, 96)) + 2.0).astype(np.float32)        # large mean: bin 0 dominates when allowed
    topk, hsh, want_topk, want_hash, flips, fs, ok = compare(vd, ctx, x, 3, f_min=0, f_max=48)
    assert fs == 0 and np.all(topk[:, 0] == 0)
    topk, hsh, want_topk, want_hash, flips, fs, ok = compare(vd, ctx, x, 10, f_min=7, f_max=16)
    assert fs == 0 and topk.min() >= 7 and topk.max() <= 16 and sorted(topk[0].tolist()) == list(range(7, 17))


@pytest.mark.parametrize("f_min,f_max,k", [(0, 128, 4), (1, 64, 3), (2, 63, 5), (7, 40, 6), (5, 5, 1), (64, 128, 3)])
def test_candidate_range_on_a_long_window(vd, ctx, f_min, f_max, k):
    """Even and odd first bins, ranges that end inside a tile of 32, the DC and the Nyquist bin, at a window
    length where the kernel splits the bins by parity."""
    rng = np.random.default_rng(100 * f_min + f_max)
    B, N, L = 8, 10, 256
    t = np.arange(L)
    x = 0.3 * rng.standard_normal((B, N, L)) + 0.5
    for n in range(N):
        for j, f in enumerate(rng.choice(np.arange(f_min, f_max + 1), size=min(k, f_max - f_min + 1), replace=False)):
            x[:, n] += (3.0 / (1 + j)) * np.cos(2 * np.pi * f * t / L + rng.uniform(0, 6, size=(B, 1)))
    topk, hsh, want_topk, want_hash, flips, fs, ok = compare(vd, ctx, x.astype(np.float32), k, f_min=f_min, f_max=f_max)
    assert fs == 0 and ok.sum() >= N // 2
    assert topk.min() >= f_min and topk.max() <= f_max
    assert np.array_equal(hsh[ok], want_hash[ok])


def test_strided_input_and_determinism(vd, ctx):
    rng = np.random.default_rng(5)
    big = torch.from_numpy(rng.standard_normal((6, 20, 128)).astype(np.float32)).cuda()
    view = big[1:5, 2:19, :96]                                         # non-contiguous, unaligned rows
    want = o_kdfh.kdfh(view.cpu().numpy(), 3)
    topk, hsh, _ = run(vd, ctx, view, 3)
    ok = o_kdfh.gap_ok(want[2], 3)
    assert np.array_equal(topk[ok], want[0][ok])
    again = run(vd, ctx, view, 3)
    assert np.array_equal(topk, again[0]) and np.array_equal(hsh, again[1])


def test_window_order_and_scale_invariance(vd, ctx):
    from util_gpu import workload_inputs
    w, x, _, want_topk, _, _ = workload_inputs("electricity")
    topk, _, _ = run(vd, ctx, x[::-1].copy(), w.k)
    assert np.array_equal(topk, want_topk)
    topk, _, _ = run(vd, ctx, (x * np.float32(8.0)), w.k)              # exact power-of-two scaling
    assert np.array_equal(topk, want_topk)


def test_dynamic_range_of_windows(vd, ctx):
    """Every window has its own magnitude, from 1e-30 to 1e30: the per-window scaling of the kernel must keep
    the fp32 quality of the spectrum whatever the scale, also next to an all-zero window."""
    rng = np.random.default_rng(11)
    B, N, L = 8, 24, 336
    t = np.arange(L)
    x = 0.05 * rng.standard_normal((B, N, L))
    for n in range(N):
        for j, f in enumerate(rng.choice(np.arange(1, 80), size=4, replace=False)):
            x[:, n] += (3.0 / (1 + j)) * np.sin(2 * np.pi * f * t / L + rng.uniform(0, 6, size=(B, 1)))
    mag = 10.0 ** rng.uniform(-30, 30, size=(B, N, 1))
    mag[:, :4] = 10.0 ** rng.uniform(-30, 30, size=(1, 4, 1))            # four variates with one scale for all windows
    x = (x * mag).astype(np.float32)
    x[3, 7] = 0.0
    x[:, 9] = 0.0
    topk, hsh, want_topk, want_hash, flips, flips_screened, ok = compare(vd, ctx, x, 4)
    assert flips_screened == 0 and ok.sum() >= N - 4
    assert topk[9].tolist() == [1, 2, 3, 4]


def test_longest_window(vd, ctx):
    rng = np.random.default_rng(12)
    B, N, L = 2, 5, 1024
    t = np.arange(L)
    x = 0.1 * rng.standard_normal((B, N, L))
    for n in range(N):
        for j, f in enumerate(rng.choice(np.arange(1, 257), size=6, replace=False)):
            x[:, n] += (3.0 / (1 + j)) * np.sin(2 * np.pi * f * t / L + rng.uniform(0, 6, size=(B, 1)))
    topk, hsh, want_topk, want_hash, flips, flips_screened, ok = compare(vd, ctx, x.astype(np.float32), 6)
    assert flips_screened == 0 and np.array_equal(hsh[ok], want_hash[ok]) and ok.sum() >= 3


@pytest.mark.parametrize("name", ["tiny", "traffic", "long"])
def test_time_major_batches(vd, ctx, name):
    """[B][L][N] input (time stride N, variate stride 1): same result as the time-contiguous layout, bit for bit,
    and equal to the oracle wherever the amplitude gap holds."""
    w, x, info, want_topk, want_hash, abar = util_gpu.workload_inputs(name)
    xt = torch.from_numpy(np.ascontiguousarray(x.transpose(0, 2, 1))).cuda()           # [B][L][N]
    view = xt.transpose(1, 2)                                                          # [B][N][L], strides (L N, 1, N)
    assert view.stride() == (w.L * w.N, 1, w.N)
    topk, hsh, _ = run(vd, ctx, view, w.k)
    ref = run(vd, ctx, torch.from_numpy(x).cuda(), w.k)
    assert np.array_equal(topk, ref[0]) and np.array_equal(hsh, ref[1])
    assert np.array_equal(topk, want_topk) and np.array_equal(hsh, want_hash)


def test_time_strided_ragged_shapes(vd, ctx):
    rng = np.random.default_rng(11)
    for B, N, L, k in [(3, 37, 50, 2), (33, 5, 96, 3), (1, 70, 200, 4)]:
        base = torch.from_numpy(rng.standard_normal((B, L + 3, N + 2)).astype(np.float32)).cuda()
        view = base[:, 1:L + 1, 1:N + 1].transpose(1, 2)                               # offset, padded, time-major
        want = o_kdfh.kdfh(view.cpu().numpy(), k)
        topk, hsh, _ = run(vd, ctx, view, k)
        ok = o_kdfh.gap_ok(want[2], k)
        assert np.array_equal(topk[ok], want[0][ok]) and np.array_equal(hsh[ok], want[1][ok])
        ref = run(vd, ctx, view.contiguous(), k)
        assert np.array_equal(topk, ref[0]) and np.array_equal(hsh, ref[1])


def test_error_codes(vd, ctx):
    x = torch.zeros((2, 3, 96), device="cuda")
    for kwargs, code in [(dict(k=30), -1), (dict(k=0), -1), (dict(k=3, f_min=5, f_max=4), -1),
                         (dict(k=3, f_max=49), -1)]:
        with pytest.raises(vd.VarDropError) as e:
            vd.vardrop_hash(ctx, x, **kwargs)
        assert e.value.code == code
    with pytest.raises(vd.VarDropError) as e:
        vd.vardrop_hash(ctx, torch.zeros((2, 3, 2048), device="cuda"), 3)
    assert e.value.code == -4
    with pytest.raises(vd.VarDropError) as e:                      # 32 variates x 257 bins of sums + operands > LDS
        vd.vardrop_hash(ctx, torch.zeros((1, 2, 1024), device="cuda"), 6)
    assert e.value.code == -4
    with pytest.raises(vd.VarDropError) as e:                      # time stride != 1 needs the workspace
        vd.vardrop_hash(ctx, torch.zeros((2, 96, 3), device="cuda").transpose(1, 2), 3,
                        ws=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.code == -2                                        # EWORKSPACE
    with pytest.raises(vd.VarDropError) as e:
        vd.vardrop_hash(ctx, torch.zeros((1, 1, 1024), device="cuda"), 8, 1, 512)          # 513**8 >= 2**63
    assert e.value.code == -1
