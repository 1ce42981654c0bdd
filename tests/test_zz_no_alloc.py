"""qsv_measure_static (the entry point that allocates nothing and keeps its partial results in the
library's fixed scratch array) against qsv_measure (partials in the caller's workspace): same kernels,
so the outputs must agree bit for bit, on two calls in a row, the second on a smaller input, and a
request beyond the array's size must be refused before anything runs."""
import numpy as np
import pytest

from paper_2602_13140_amd import binding as qb
from paper_2602_13140_amd import workloads as wl
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

RY, RZ, RING = 2, 3, 1


def prepare(ctx, n, B, seed):
    g = np.random.Generator(np.random.PCG64(seed))
    spec = wl.CircuitSpec(2, (RY, RZ), RING, 0)
    params = wl.draw_params(spec, n, seed + 1)
    x = g.standard_normal((B, (1 << n) - 3)).astype(np.float32)
    xd, pd = gu.dev(x), gu.dev(params)
    circ = qb.circuit_from_spec(spec)

    def run():
        ctx.qsv_amp_encode(xd)
        ctx.qsv_apply_layers(circ, pd, None, 0)
    return run, xd, g.random((B, 37))


def both(ctx, kind, shape, dtype="float32", rerun=None, **kw):
    """The same request through both entry points (the state re-prepared before each when the request
    modifies it)."""
    torch = gu.torch_cuda()
    outs = []
    for static in (False, True):
        if rerun:
            rerun()
        out = torch.full(shape, -7.0 if dtype == "float32" else -7, dtype=getattr(torch, dtype), device="cuda")
        (ctx.qsv_measure_static if static else ctx.qsv_measure)(kind, out, **kw)
        torch.cuda.synchronize()
        outs.append((out.cpu().numpy(), gu.state_np(ctx)))
    return outs


def test_static_scratch_entry_point_matches_the_workspace_one(oracle):
    torch = gu.torch_cuda()
    for n, B, seed in ((14, 3, 900), (9, 2, 901)):          # the second call is the smaller one
        ctx = gu.make_ctx(n, B)
        run, xd, u = prepare(ctx, n, B, seed)
        run()
        ud = gu.dev(u)
        mask = (1 << (n - 1)) | 0b101
        cases = [
            (qb.QSV_M_EXPZ_ALL, (B, n), "float32", {}, False),
            (qb.QSV_M_EXPZ_ONE, (B,), "float32", {"qubit": n - 2}, False),
            (qb.QSV_M_MARGINAL, (B, 8), "float32", {"mask": mask}, False),
            (qb.QSV_M_FIDELITY, (B,), "float32", {"x": xd}, False),
            (qb.QSV_M_SAMPLE, (B, u.shape[1]), "int64", {"uniforms": ud}, False),
            (qb.QSV_M_PROBS, (B, 1 << n), "float32", {}, False),
            (qb.QSV_M_PROJECT_ZERO, (B,), "float32", {"mask": mask, "renormalise": 1}, True),
        ]
        for kind, shape, dtype, kw, modifies in cases:
            (a, sa), (b, sb) = both(ctx, kind, shape, dtype, rerun=run if modifies else None, **kw)
            assert np.array_equal(a, b), (n, kind)
            assert np.array_equal(sa, sb), (n, kind)
            assert not np.any(a == -7), (n, kind)           # every output element was written
        # and the values are the oracle's (the contract's tolerance), not merely equal to each other
        ref, _ = oracle.amp_encode(xd.cpu().numpy(), n)
        spec = wl.CircuitSpec(2, (RY, RZ), RING, 0)
        oracle.apply_layers(ref, oracle.make_circuit(2, [RY, RZ], RING), wl.draw_params(spec, n, seed + 1))
        z = torch.zeros((B, n), dtype=torch.float32, device="cuda")
        run()
        ctx.qsv_measure_static(qb.QSV_M_EXPZ_ALL, z)
        torch.cuda.synchronize()
        assert np.abs(z.cpu().numpy() - oracle.expz_all(ref)).max() <= 1e-5
        ctx.close()


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    torch = gu.torch_cuda()
    n = 20
    ctx = gu.make_ctx(n, 1)
    ctx.state.zero_()
    ctx.state[0, 0, 0] = 1.0
    out = torch.zeros((1, 1 << n), dtype=torch.float32, device="cuda")
    with pytest.raises(qb.QsvError) as ei:                   # 2^20 outcomes x 8 bytes of partials > 4 MiB
        ctx.qsv_measure_static(qb.QSV_M_MARGINAL, out, mask=(1 << n) - 1)
    assert ei.value.status == qb.QSV_ERR_WORKSPACE and "fixed array" in str(ei.value)
    ctx.qsv_measure(qb.QSV_M_MARGINAL, out, mask=(1 << n) - 1)          # the workspace entry point takes it
    torch.cuda.synchronize()
    assert out[0, 0].item() == 1.0 and out.sum().item() == 1.0
    ctx.close()
