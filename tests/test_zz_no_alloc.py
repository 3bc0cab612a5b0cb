"""dash_block_norms_static -- the entry point for callers that cannot allocate -- against dash_block_norms:
same kernels, so the scales must agree bit for bit; two calls in a row on the one static scratch array, the
second on a smaller input; limits are refused with a clear error."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dash():
    from paper_2602_02016_amd import Dash
    d = Dash(0)
    yield d
    d.close()


def _stack(n, b, seed):
    import torch
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    G = torch.randn(n, b, b, device="cuda", generator=gen)
    return (G + G.transpose(1, 2)).contiguous() * 0.05 + torch.eye(b, device="cuda")


@pytest.mark.parametrize("scaling", ["frobenius", "trace", "none"])
def test_static_scratch_matches_workspace_path_twice(dash, scaling):
    import torch
    eps = 1e-3
    big, small = _stack(37, 256, 11), _stack(5, 128, 12)
    out_big = torch.full((37,), -1.0, device="cuda")
    out_small = torch.full((5,), -1.0, device="cuda")
    # two calls in a row on the same static array, the second with fewer and smaller blocks
    dash.block_norms_static(big, out_big, eps=eps, scaling=scaling)
    dash.block_norms_static(small, out_small, eps=eps, scaling=scaling)
    torch.cuda.synchronize()
    ref_big = dash.block_norms(big, eps=eps, scaling=scaling)
    ref_small = dash.block_norms(small, eps=eps, scaling=scaling)
    torch.cuda.synchronize()
    assert np.array_equal(out_big.cpu().numpy(), ref_big.cpu().numpy())
    assert np.array_equal(out_small.cpu().numpy(), ref_small.cpu().numpy())
    # and against the definition, in float64 on the host
    for A, out in ((big, out_big), (small, out_small)):
        Ad = A.cpu().numpy().astype(np.float64) + eps * np.eye(A.shape[1])
        want = {"frobenius": np.sqrt((Ad ** 2).sum(axis=(1, 2))), "trace": np.trace(Ad, axis1=1, axis2=2),
                "none": np.ones(A.shape[0])}[scaling]
        assert np.allclose(out.cpu().numpy(), want, rtol=2e-6, atol=0)


def test_static_scratch_limits_are_refused(dash):
    import torch
    from paper_2602_02016_amd.binding import DashError, ERR_INVALID_ARG, ERR_UNSUPPORTED
    A = _stack(2, 64, 3)
    out = torch.zeros(2, device="cuda")
    with pytest.raises(DashError) as e:
        dash.block_norms_static(A, out, scaling="pi")
    assert e.value.status == ERR_UNSUPPORTED
    # one block more than the scratch holds: refused before anything is launched (the pointer is never read)
    import ctypes as C
    st = dash.lib.dash_block_norms_static(dash.h, C.c_void_p(A.data_ptr()), 16385, 64, 0.0, 0, C.c_void_p(out.data_ptr()))
    assert st == ERR_INVALID_ARG
    assert b"16384" in dash.lib.dash_last_error(dash.h)
    # the largest accepted size runs (64 x 64 blocks: 256 MiB)
    n = 16384
    big = torch.ones(n, 64, 64, device="cuda")
    out = torch.zeros(n, device="cuda")
    dash.block_norms_static(big, out, scaling="frobenius")
    torch.cuda.synchronize()
    assert float(out.min()) == 64.0 and float(out.max()) == 64.0
