"""The entry point that allocates nothing (dq_whip_loss_grad_noalloc) against the entry point it is a variant of
(dq_whip_loss_grad), through the C ABI: two calls in a row, the second on a smaller input, so that whatever the first
call left in the library's fixed device array must not leak into the second."""

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2511_04063_amd import binding as B  # noqa: E402


def block(b, T, n, seed, dtype=torch.float32):
    g = np.random.Generator(np.random.Philox(seed))
    Y = (g.standard_t(3.0, size=(b, T, n)) * 2.0).astype(np.float32)
    Y[0, 0, 0] = 0.0
    return torch.from_numpy(Y).cuda()


@pytest.mark.parametrize("bf16", [True, False])
def test_noalloc_matches_whip_loss_grad_twice(bf16):
    ctx = B.Context()
    ctx.ensure_workspace(1, 64, 64, B.DQ_F32)
    try:
        # first call: three problems of 1500 x 1024 (the dense fast path, many workgroups);
        # second call: one problem of 37 x 101 (ragged rows, few workgroups): far fewer partial sums than the first
        for (b, T, n, red) in ((3, 1500, 1024, B.DQ_REDUCE_TOKEN_MEAN), (1, 37, 101, B.DQ_REDUCE_SUM)):
            Y = block(b, T, n, 9100 + T)
            if n % 8:
                buf = torch.full((b, T, n + (8 - n % 8)), float("nan"), device="cuda")
                buf[:, :, :n] = Y
                Y = buf[:, :, :n]
            dt = torch.bfloat16 if bf16 else torch.float32
            code = B.DQ_BF16 if bf16 else B.DQ_F32
            ld = Y.stride(-2)
            outs = []
            for _ in range(2):
                dbuf = torch.full((b, T, ld), float("nan"), device="cuda", dtype=dt)
                outs.append((torch.full((b,), float("nan"), device="cuda"), dbuf[:, :, :n]))
            ctx.dq_whip_loss_grad(Y, red, outs[0][0], outs[0][1], code)
            B.dq_whip_loss_grad_noalloc(torch.cuda.current_stream(), Y, red, outs[1][0], outs[1][1], code)
            torch.cuda.synchronize()
            assert torch.isfinite(outs[1][0]).all()
            # same kernels, same launch shape: the gradient bit for bit, the loss to the last bit of its fp64 sum
            assert torch.equal(outs[0][1], outs[1][1])
            assert torch.equal(outs[0][0], outs[1][0])
            # and against the definition, on the host in fp64
            Yh = Y.double().cpu().numpy()
            c = 1.0 / T if red == B.DQ_REDUCE_TOKEN_MEAN else 1.0
            ref = c * np.exp(-np.abs(Yh)).sum(axis=(1, 2))
            assert np.abs(outs[1][0].cpu().numpy() - ref).max() <= 1e-5 * np.abs(ref).max()
    finally:
        torch.cuda.synchronize()
        ctx.close()


def test_noalloc_rejects_what_it_cannot_hold():
    Y = torch.zeros((4, 8), device="cuda")
    dY = torch.full((4, 8), 7.0, device="cuda")
    loss = torch.full((1,), 5.0, device="cuda")
    lib = B.load_library()
    st = lib.dq_whip_loss_grad_noalloc(None, 8193, 4, 8, Y.data_ptr(), 8, B.DQ_REDUCE_SUM, loss.data_ptr(),
                                       dY.data_ptr(), B.DQ_F32, 8)
    assert st == B.DQ_ERR_UNSUPPORTED
    st = lib.dq_whip_loss_grad_noalloc(None, 1, 4, 8, Y.data_ptr(), 6, B.DQ_REDUCE_SUM, loss.data_ptr(),
                                       dY.data_ptr(), B.DQ_F32, 8)
    assert st == B.DQ_ERR_SHAPE
    torch.cuda.synchronize()
    assert loss.item() == 5.0 and torch.all(dY == 7.0)
