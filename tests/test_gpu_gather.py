"""GPU gather / scatter against the oracle: exact copies."""
import numpy as np
import pytest
import torch

from oracle import attention as o_attn

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vd():
    import paper_2501_14183_amd as m
    return m


@pytest.fixture(scope="module")
def ctx(vd):
    return vd.Context(0)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("B,N,d,n_sel", [(4, 32, 64, 10), (32, 862, 512, 113), (3, 17, 5, 4), (2, 9, 24, 9),
                                          (1, 1, 8, 1), (5, 40, 768, 0)])
def test_gather_and_scatter_exact(vd, ctx, dtype, B, N, d, n_sel):
    rng = np.random.default_rng(N * d + n_sel)
    tok = torch.from_numpy(rng.standard_normal((B, N, d)).astype(np.float32)).to(dtype).cuda()
    sel_np = np.sort(rng.choice(N, size=n_sel, replace=False)).astype(np.int32)
    sel = torch.from_numpy(sel_np).cuda()
    out = vd.vardrop_gather(ctx, tok, sel, n_sel)
    want = o_attn.gather(tok.float().cpu().numpy(), sel_np)
    assert out.shape == (B, n_sel, d)
    assert np.array_equal(out.float().cpu().numpy(), want)
    g = torch.from_numpy(rng.standard_normal((B, n_sel, d)).astype(np.float32)).to(dtype).cuda()
    back = vd.vardrop_scatter(ctx, g, sel, n_sel, N)
    want_back = o_attn.scatter_add(g.float().cpu().numpy(), sel_np, N)
    assert np.array_equal(back.float().cpu().numpy(), want_back)


def test_unaligned_rows_take_the_narrow_path(vd, ctx):
    rng = np.random.default_rng(1)
    base = torch.from_numpy(rng.standard_normal(4 * 11 * 24 + 1).astype(np.float32)).to(torch.bfloat16).cuda()
    tok = base[1:].view(4, 11, 24)                                   # 2-byte aligned only
    sel_np = np.array([0, 5, 10], dtype=np.int32)
    out = vd.vardrop_gather(ctx, tok, torch.from_numpy(sel_np).cuda(), 3)
    assert np.array_equal(out.float().cpu().numpy(), o_attn.gather(tok.float().cpu().numpy(), sel_np))


def test_out_of_range_index_gives_a_zero_row(vd, ctx):
    tok = torch.ones((2, 4, 8), device="cuda")
    sel = torch.tensor([1, 9], dtype=torch.int32, device="cuda")
    out = vd.vardrop_gather(ctx, tok, sel, 2)
    assert out[:, 0].eq(1).all() and out[:, 1].eq(0).all()


def test_error_codes(vd, ctx):
    tok = torch.ones((2, 4, 8), device="cuda")
    sel = torch.tensor([1, 2, 3, 0, 1], dtype=torch.int32, device="cuda")
    with pytest.raises(vd.VarDropError) as e:
        vd.vardrop_gather(ctx, tok, sel, 5)                          # n_sel > N
    assert e.value.code == -1
