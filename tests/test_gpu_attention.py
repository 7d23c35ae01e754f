"""GPU multi-head attention forward/backward against the fp64 oracle.

Tolerance (per tensor): max|gpu - oracle| / max|oracle| <= 2e-2 for bf16, 1e-5 for fp32, and on top of that the
element-wise bounds of util_gpu.elem_err (RMS of the difference, and every element against a relative term plus a
floor proportional to the tensor's RMS), so that small elements are constrained as well.
The oracle receives the same bf16- (or fp32-) representable inputs, converted to fp64.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from util_gpu import TOL, elem_err, oracle_attention, rel_err, to_dev, torch_dtype

pytestmark = pytest.mark.gpu

GRADS = ("dxs", "dWq", "dWk", "dWv", "dWo")


@pytest.fixture(scope="module")
def vd():
    import paper_2501_14183_amd as m
    return m


@pytest.fixture(scope="module")
def ctx(vd):
    return vd.Context(0)


def run_gpu(vd, ctx, xs, W, H, dy, dtype, biases=None):
    td = torch_dtype(dtype)
    xs_t, dy_t = to_dev(xs, td), to_dev(dy, td)
    W_t = [to_dev(w, td) for w in W]
    b_t = [to_dev(b, td) for b in biases] if biases else [None] * 4
    y, saved = vd.vardrop_attn_fwd(ctx, xs_t, *W_t, H, *b_t)
    out = vd.vardrop_attn_bwd(ctx, dy_t, xs_t, *W_t, H, saved, bias_grads=biases is not None)
    torch.cuda.synchronize()
    names = GRADS + (("dbq", "dbk", "dbv", "dbo") if biases else ())
    res = dict(zip(names, out))
    res["y"] = y
    return res


def random_case(seed, B, n, d, dtype, bias):
    rng = np.random.default_rng(seed)
    xs = wl.quantise(rng.standard_normal((B, n, d)), dtype)
    W = [wl.quantise(rng.standard_normal((d, d)) / np.sqrt(d), dtype) for _ in range(4)]
    dy = wl.quantise(rng.standard_normal((B, n, d)), dtype)
    b = [wl.quantise(0.2 * rng.standard_normal(d), dtype) for _ in range(4)] if bias else None
    return xs, W, dy, b


def compare(got, want, dtype, names):
    errs = {k: rel_err(got[k], want[k]) for k in names}
    if "dbk" in names:
        # Softmax does not see a shift of all logits of a row, so the key-bias gradient is identically zero
        # (and with a single token the query-bias gradient too): measure both against a scale that does
        # not vanish, the larger of their own, the query-bias and 1% of the value-bias gradient.
        floor = max(np.abs(want["dbq"]).max(), 1e-2 * np.abs(want["dbv"]).max())
        for k in ("dbq", "dbk"):
            diff = np.abs(got[k].float().cpu().numpy() - want[k]).max()
            errs[k] = float(diff / max(np.abs(want[k]).max(), floor))
    bad = {k: v for k, v in errs.items() if not v <= TOL[dtype]}
    assert not bad, "relative errors above %g: %s (all: %s)" % (TOL[dtype], bad, errs)
    # element-wise (the two bias gradients that vanish identically or nearly so keep the scale chosen above)
    fine = {k: elem_err(got[k], want[k], dtype) for k in names if k not in ("dbq", "dbk")}
    bad = {k: v for k, v in fine.items() if v is not None and not (v[0] <= 1.0 and v[1] <= 1.0)}
    assert not bad, "element-wise bounds exceeded (rms ratio, element ratio; both must be <= 1): %s (all: %s)" % (bad, fine)
    return errs


@pytest.mark.parametrize("name", wl.ORDER)
def test_five_workloads(vd, ctx, name):
    """Tokens of the workload, gathered at the oracle's selection, through attention fwd + bwd."""
    from util_gpu import workload_inputs, workload_selection
    w, x, *_ = workload_inputs(name)
    gid, sel, G = workload_selection(name)
    tok = wl.make_tokens(w, x)
    xs = tok[:, sel, :]
    W = wl.make_weights(w)
    dy = wl.make_upstream(w, len(sel))
    want = oracle_attention(xs, W, w.H, dy)
    got = run_gpu(vd, ctx, xs, W, w.H, dy, w.dtype)
    errs = compare(got, want, w.dtype, ("y",) + GRADS)
    print("%s: n=%d %s" % (name, len(sel), {k: "%.2e" % v for k, v in errs.items()}))


@pytest.mark.parametrize("n", [1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 130, 257, 300])
def test_bf16_ragged_token_counts_with_biases(vd, ctx, n):
    xs, W, dy, b = random_case(n, 3, n, 128, "bf16", bias=True)
    want = oracle_attention(xs, W, 2, dy, tuple(b))
    got = run_gpu(vd, ctx, xs, W, 2, dy, "bf16", biases=b)
    compare(got, want, "bf16", ("y",) + GRADS + ("dbq", "dbk", "dbv", "dbo"))


@pytest.mark.parametrize("n", [129, 188, 192, 200, 256, 257, 321])
def test_bf16_ragged_token_counts_in_the_wide_launch_shape(vd, ctx, n):
    """Enough (batch, head) pairs that the long-selection kernels run with four wavefronts and 128 rows per
    workgroup (the shape the large workloads use), at token counts that end a block of 64 and of 128 early, the first
    count past the single-kernel path (129) and the token count the paper reports for Traffic (188, Table 3)."""
    xs, W, dy, b = random_case(1000 + n, 32, n, 512, "bf16", bias=False)
    want = oracle_attention(xs, W, 8, dy)
    got = run_gpu(vd, ctx, xs, W, 8, dy, "bf16")
    compare(got, want, "bf16", ("y",) + GRADS)


@pytest.mark.parametrize("B,n,d,H", [(4, 150, 192, 3), (8, 100, 320, 5), (6, 90, 64, 1), (2, 130, 64, 1), (3, 200, 320, 5)])
def test_bf16_model_widths_off_the_tile_grid(vd, ctx, B, n, d, H):
    """d is a multiple of 64 but not of the 128-wide GEMM tiles; B*n large enough for sliced weight gradients; more
    than 128 tokens with one head and with an odd head count (the dO product then forms the row sums of dO * O)."""
    xs, W, dy, b = random_case(7 * d + n, B, n, d, "bf16", bias=True)
    want = oracle_attention(xs, W, H, dy, tuple(b))
    got = run_gpu(vd, ctx, xs, W, H, dy, "bf16", biases=b)
    compare(got, want, "bf16", ("y",) + GRADS + ("dbq", "dbk", "dbv", "dbo"))


@pytest.mark.parametrize("B,n,d,H", [(1, 5, 16, 1), (2, 70, 64, 2), (3, 33, 128, 2), (2, 9, 128, 1), (4, 10, 64, 2)])
def test_fp32_head_sizes_and_biases(vd, ctx, B, n, d, H):
    xs, W, dy, b = random_case(d + n, B, n, d, "fp32", bias=True)
    want = oracle_attention(xs, W, H, dy, tuple(b))
    got = run_gpu(vd, ctx, xs, W, H, dy, "fp32", biases=b)
    compare(got, want, "fp32", ("y",) + GRADS + ("dbq", "dbk", "dbv", "dbo"))


def test_dense_mode_equals_identity_selection(vd, ctx):
    """Inference path of the paper: no variate dropped, all N tokens attend."""
    w = wl.WORKLOADS["electricity"]
    from util_gpu import workload_inputs
    _, x, *_ = workload_inputs("electricity")
    tok = wl.make_tokens(w, x)[:4]
    W = wl.make_weights(w)
    dy = wl.make_upstream(w, w.N)[:4]
    want = oracle_attention(tok, W, w.H, dy)
    got = run_gpu(vd, ctx, tok, W, w.H, dy, "bf16")
    compare(got, want, "bf16", ("y",) + GRADS)


def test_softmax_with_large_logits_stays_finite(vd, ctx):
    xs, W, dy, _ = random_case(1, 2, 40, 64, "bf16", bias=False)
    xs = wl.quantise(xs * 30.0, "bf16")                     # logits of a few hundred: one-hot-like rows
    want = oracle_attention(xs, W, 1, dy)
    got = run_gpu(vd, ctx, xs, W, 1, dy, "bf16")
    assert all(torch.isfinite(v.float()).all() for v in got.values())
    assert rel_err(got["y"], want["y"]) <= 5e-2             # near-ties between keys amplify bf16 rounding of Q, K


def test_determinism(vd, ctx):
    xs, W, dy, _ = random_case(9, 4, 130, 512, "bf16", bias=False)
    a = run_gpu(vd, ctx, xs, W, 8, dy, "bf16")
    b = run_gpu(vd, ctx, xs, W, 8, dy, "bf16")
    for k in a:
        assert torch.equal(a[k], b[k]), k


def test_empty_and_error_cases(vd, ctx):
    d, H = 64, 1
    W = [torch.zeros((d, d), dtype=torch.bfloat16, device="cuda") for _ in range(4)]
    xs = torch.zeros((2, 0, d), dtype=torch.bfloat16, device="cuda")
    y, saved = vd.vardrop_attn_fwd(ctx, xs, *W, H)
    out = vd.vardrop_attn_bwd(ctx, xs, xs, *W, H, saved)
    assert y.shape == (2, 0, d) and all(float(t.abs().sum()) == 0 for t in out[1:])
    with pytest.raises(vd.VarDropError) as e:                                   # d_k = 32 is not built for bf16
        vd.vardrop_attn_fwd(ctx, torch.zeros((1, 4, 64), dtype=torch.bfloat16, device="cuda"), *W, 2)
    assert e.value.code == -4
    with pytest.raises(vd.VarDropError) as e:                                   # H does not divide d
        vd.vardrop_attn_fwd(ctx, torch.zeros((1, 4, 64), dtype=torch.bfloat16, device="cuda"), *W, 3)
    assert e.value.code == -1


def test_bf16_backward_is_bit_reproducible(vd, ctx):
    """Sliced weight gradients are summed in a fixed order, whichever workgroup finishes last: equal bits on every call."""
    xs, W, dy, _ = random_case(77, 8, 113, 512, "bf16", bias=False)
    first = run_gpu(vd, ctx, xs, W, 8, dy, "bf16")
    for _ in range(3):
        again = run_gpu(vd, ctx, xs, W, 8, dy, "bf16")
        for k in GRADS + ("y",):
            assert torch.equal(first[k], again[k]), k
