"""The entry point that allocates nothing (vardrop_sample_nearest_noalloc, static device scratch) against the entry
point it is a variant of (vardrop_sample_nearest, caller workspace): identical integer outputs, on two calls in a row,
the second with a smaller input, through the C ABI."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def spectra(rng, N, F, n_groups):
    h = rng.integers(0, n_groups, size=N).astype(np.uint64) * np.uint64(977) + np.uint64(5)
    centre = rng.uniform(1.0, 9.0, (n_groups, F))
    A = np.abs(centre[(h // np.uint64(977)).astype(np.int64) % n_groups] + 0.3 * rng.standard_normal((N, F)))
    return h, A.astype(np.float32)


def test_static_scratch_equals_caller_workspace_on_two_calls_in_a_row():
    import paper_2501_14183_amd as vd
    lib = vd.load_library()
    ctx = vd.Context(0)
    rng = np.random.default_rng(2024)
    stream = torch.cuda.current_stream().cuda_stream
    # a large call (the stress shape: 8192 variates, 128 bins = the whole scratch), then a smaller one that leaves
    # most of the array holding the first call's contents
    for N, F, n_groups, gs, num, den in ((8192, 128, 700, 0, 1, 20), (1000, 25, 40, 3, 1, 1), (37, 7, 5, 1, 1, 1)):
        h, A = spectra(rng, N, F, n_groups)
        h_t = torch.from_numpy(h.view(np.int64)).cuda()
        A_t = torch.from_numpy(A).cuda()
        outs = []
        for which in ("noalloc", "workspace"):
            gid = torch.full((N,), -7, dtype=torch.int32, device="cuda")
            sel = torch.full((N,), -7, dtype=torch.int32, device="cuda")
            counts = torch.full((2,), -7, dtype=torch.int32, device="cuda")
            if which == "noalloc":
                rc = lib.vardrop_sample_nearest_noalloc(ctx.handle, h_t.data_ptr(), A_t.data_ptr(), N, F, gs, num, den,
                                                        gid.data_ptr(), sel.data_ptr(), counts.data_ptr(), stream)
            else:
                ws = torch.empty(lib.vardrop_sample_nearest_workspace_bytes(N, F), dtype=torch.uint8, device="cuda")
                rc = lib.vardrop_sample_nearest(ctx.handle, h_t.data_ptr(), A_t.data_ptr(), N, F, gs, num, den,
                                                gid.data_ptr(), sel.data_ptr(), counts.data_ptr(), None,
                                                ws.data_ptr(), ws.numel(), stream)
            assert rc == 0, (which, rc)
            torch.cuda.synchronize()
            outs.append((gid.cpu().numpy(), sel.cpu().numpy(), counts.cpu().numpy()))
        (g1, s1, c1), (g2, s2, c2) = outs
        assert np.array_equal(c1, c2) and c1[0] >= 1 and c1[1] >= 1
        assert np.array_equal(g1, g2)
        assert np.array_equal(s1[:c1[0]], s2[:c2[0]])
    # sizes beyond the static array are refused with a clear error, before anything is launched
    big = torch.zeros(8192, dtype=torch.int64, device="cuda")
    out = [torch.empty(8192, dtype=torch.int32, device="cuda") for _ in range(2)] + [torch.empty(2, dtype=torch.int32, device="cuda")]
    A_big = torch.ones((8192, 129), device="cuda")
    rc = lib.vardrop_sample_nearest_noalloc(ctx.handle, big.data_ptr(), A_big.data_ptr(), 8192, 129, 0, 1, 1,
                                            out[0].data_ptr(), out[1].data_ptr(), out[2].data_ptr(), stream)
    assert rc == -4
    assert lib.vardrop_strerror(rc).decode() == "request outside the implemented range"
