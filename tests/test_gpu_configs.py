"""GPU parity at the five workload configs' full sizes, in the launch configuration bench.py
times (default tile, fused passes).  Where the oracle cannot finish the whole output in a test's
time (config 2's 164 096 circuits) sampled outputs are compared one by one."""
import numpy as np
import pytest

from paper_2602_13140_amd import binding as qb
from paper_2602_13140_amd import workloads as wl
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def ocirc(oracle, spec):
    return oracle.make_circuit(spec.n_layers, list(spec.rot), spec.entangler, spec.reupload)


def test_config0_autoencoder_roundtrip(oracle):
    w = wl.config(0)
    ctx = gu.make_ctx(w.n, w.batch)
    circ = qb.circuit_from_spec(w.circuit)
    xd, pd = gu.dev(w.x), gu.dev(w.params)
    ctx.qsv_amp_encode(xd)
    ctx.qsv_apply_layers(circ, pd, None, 0)
    mid = gu.state_np(ctx)
    ref, _ = oracle.amp_encode(w.x, w.n)
    oracle.apply_layers(ref, ocirc(oracle, w.circuit), w.params)
    assert np.abs(mid - ref).max() <= 2e-6
    ctx.qsv_apply_layers(circ, pd, None, 1)
    p = gu.measure(ctx, qb.QSV_M_PROBS, (w.batch, 1 << w.n))
    oracle.apply_layers(ref, ocirc(oracle, w.circuit), w.params, inverse=True)
    gu.prob_checks(p, oracle.probs(ref))
    xd64 = w.x.astype(np.float64)
    assert np.abs(p - xd64 ** 2 / (xd64 ** 2).sum(1, keepdims=True)).max() <= 1e-5   # closed form
    # the same step in one launch
    torch = gu.torch_cuda()
    p1 = torch.full((w.batch, 1 << w.n), -7.0, dtype=torch.float32, device="cuda")
    ctx.state.fill_(9.0)
    ctx.qsv_forward_small(xd, circ, pd, None, 1, qb.QSV_M_PROBS, p1)
    gu.prob_checks(p1.cpu().numpy(), oracle.probs(ref))
    assert np.abs(gu.state_np(ctx) - ref).max() <= 2e-6
    ctx.close()


def test_config1_reupload_expz(oracle):
    w = wl.config(1)
    ctx = gu.make_ctx(w.n, w.batch)
    ctx.qsv_amp_encode(gu.dev(w.x))
    ctx.qsv_apply_layers(qb.circuit_from_spec(w.circuit), gu.dev(w.params), gu.dev(w.feats), 0)
    z = gu.measure(ctx, qb.QSV_M_EXPZ_ALL, (w.batch, w.n))
    ref, _ = oracle.amp_encode(w.x, w.n)
    oracle.apply_layers(ref, ocirc(oracle, w.circuit), w.params, w.feats)
    assert np.abs(z - oracle.expz_all(ref)).max() <= 1e-5
    assert np.abs(gu.state_np(ctx) - ref).max() <= 1e-5
    # the same step in one launch, with every number of amplitudes per thread
    torch = gu.torch_cuda()
    circ, xd, pd, fd = qb.circuit_from_spec(w.circuit), gu.dev(w.x), gu.dev(w.params), gu.dev(w.feats)
    for regs in (0, 2, 3, 4):
        ctx.qsv_set_option("small_regs", regs)
        z1 = torch.full((w.batch, w.n), -7.0, dtype=torch.float32, device="cuda")
        ctx.state.fill_(9.0)
        ctx.qsv_forward_small(xd, circ, pd, fd, 0, qb.QSV_M_EXPZ_ALL, z1)
        assert np.abs(z1.cpu().numpy() - oracle.expz_all(ref)).max() <= 1e-5, regs
        assert np.abs(gu.state_np(ctx) - ref).max() <= 1e-5, regs
    ctx.close()


@pytest.mark.parametrize("rot,layered", [((wl.RY, wl.RZ), 1), ((wl.RY, wl.RZ), 0), ((wl.RX, wl.RY, wl.RZ), 1),
                                         ((wl.RY, wl.RZ), -1), ((wl.RX, wl.RY, wl.RZ), -1)])
def test_config2_gradient_sampled(oracle, rot, layered):
    """Full 256 x P gradient on the GPU; the oracle recomputes two samples x 12 random parameters
    (plus their losses).  The three-rotation variant is the reading that gives ~480 params.
    layered = 1: workspace with room for the per-layer states, so shifted circuits start from them;
    layered = 0: the minimum workspace, every shifted circuit runs whole; layered = -1: the
    reverse-mode entry point qsv_adjoint_grad, which must give the same values."""
    torch = gu.torch_cuda()
    w = wl.config(2)
    spec = wl.CircuitSpec(w.circuit.n_layers, rot, w.circuit.entangler)
    P = spec.num_params(w.n)
    params = wl.draw_params(spec, w.n, 2002)
    circ = qb.circuit_from_spec(spec)
    ctx = gu.make_ctx(w.n, w.batch, ws_bytes=qb.qsv_grad_workspace_bytes(w.n, w.batch, circ) if layered > 0 else None)
    loss = torch.zeros(w.batch, dtype=torch.float32, device="cuda")
    grad = torch.zeros((w.batch, P), dtype=torch.float32, device="cuda")
    mg = torch.zeros(P, dtype=torch.float32, device="cuda")
    call = ctx.qsv_adjoint_grad if layered < 0 else ctx.qsv_param_shift_grad
    call(circ, gu.dev(w.x), gu.dev(params), None, 0, loss, grad, None, mg)
    torch.cuda.synchronize()
    gg, ll = grad.cpu().numpy(), loss.cpu().numpy()
    g = np.random.Generator(np.random.PCG64(5))
    rows = sorted(g.choice(w.batch, 2, replace=False).tolist())
    sub = sorted(g.choice(P, 12, replace=False).tolist()) + [0, P - 1]
    lref, gref = oracle.param_shift_grad(w.x[rows], w.n, ocirc(oracle, spec), params, None, 0, subset=sub)
    assert np.abs(ll[rows] - lref).max() <= 1e-5
    assert np.abs(gg[rows][:, sub] - gref).max() <= 1e-4
    assert np.linalg.norm(gg[rows][:, sub] - gref) <= 1e-3 * np.linalg.norm(gref)
    assert np.abs(mg.cpu().numpy() - gg.astype(np.float64).mean(0)).max() <= 1e-6
    assert np.all(np.abs(gg) <= 1.0) and np.all(np.abs(ll) <= 1.0)
    ctx.close()


def test_config2_gradient_wide(oracle, capsys):
    """Config 2 at full size through all three entry points (shift rule layer by layer, shift rule with
    whole circuits, reverse mode): every one of the 256 x 320 entries must agree between them, and the
    oracle recomputes all 320 parameters for two samples (the first and one from the last chunk of
    rows) and 8 seeded parameters for all 256 samples, so every chunk boundary of the full-size
    launches is covered."""
    torch = gu.torch_cuda()
    w = wl.config(2)
    spec = w.circuit
    P = spec.num_params(w.n)
    params = wl.draw_params(spec, w.n, 2002)
    circ = qb.circuit_from_spec(spec)
    xd, pd = gu.dev(w.x), gu.dev(params)
    got = {}
    for name in ("layered", "whole", "adjoint"):
        ctx = gu.make_ctx(w.n, w.batch,
                          ws_bytes=None if name == "whole" else qb.qsv_grad_workspace_bytes(w.n, w.batch, circ))
        loss = torch.zeros(w.batch, dtype=torch.float32, device="cuda")
        grad = torch.zeros((w.batch, P), dtype=torch.float32, device="cuda")
        (ctx.qsv_adjoint_grad if name == "adjoint" else ctx.qsv_param_shift_grad)(circ, xd, pd, None, 0, loss, grad)
        torch.cuda.synchronize()
        got[name] = (loss.cpu().numpy().astype(np.float64), grad.cpu().numpy().astype(np.float64))
        ctx.close()
        with capsys.disabled():
            print(" [c2 %s done]" % name, end="", flush=True)
    l0, g0 = got["layered"]
    for name in ("whole", "adjoint"):
        l1, g1 = got[name]
        assert np.abs(l1 - l0).max() <= 1e-5, name
        assert np.abs(g1 - g0).max() <= 1e-4, name
        assert np.linalg.norm(g1 - g0) <= 1e-3 * np.linalg.norm(g0), name
    oc = ocirc(oracle, spec)
    g = np.random.Generator(np.random.PCG64(77))
    rows = [0, int(g.integers(w.batch - 16, w.batch))]
    lref, gref = oracle.param_shift_grad(w.x[rows], w.n, oc, params, None, 0)
    with capsys.disabled():
        print(" [c2 oracle: all parameters of 2 samples]", end="", flush=True)
    # <Z_0> behind a CZ ladder only sees the parameters inside qubit 0's light cone; the others have
    # gradient zero (the oracle returns 1e-17).  Six seeded parameters from inside it, two from outside.
    live = np.flatnonzero(np.abs(gref).max(0) > 1e-4)
    dead = np.flatnonzero(np.abs(gref).max(0) < 1e-12)
    assert live.size >= 6 and dead.size >= 2
    sub = sorted(g.choice(live, 6, replace=False).tolist() + g.choice(dead, 2, replace=False).tolist())
    lall, gall = oracle.param_shift_grad(w.x, w.n, oc, params, None, 0, subset=sub)
    with capsys.disabled():
        print(" [c2 oracle: 8 parameters of all samples]", end="", flush=True)
    for name, (ll, gg) in got.items():
        assert np.abs(ll[rows] - lref).max() <= 1e-5, name
        assert np.abs(gg[rows] - gref).max() <= 1e-4, name
        assert np.linalg.norm(gg[rows] - gref) <= 1e-3 * np.linalg.norm(gref), name
        assert np.abs(ll - lall).max() <= 1e-5, name
        assert np.abs(gg[:, sub] - gall).max() <= 1e-4, name
        assert np.linalg.norm(gg[:, sub] - gall) <= 1e-3 * np.linalg.norm(gall), name


def test_config3_autoencoder_full(oracle, capsys):
    w = wl.config(3)
    n, B = w.n, w.batch
    ctx = gu.make_ctx(n, B)
    circ = qb.circuit_from_spec(w.circuit)
    xd, pd = gu.dev(w.x), gu.dev(w.params)
    ctx.qsv_amp_encode(xd)
    ctx.qsv_apply_layers(circ, pd, None, 0)
    m = bin(w.trash_mask).count("1")
    marg = gu.measure(ctx, qb.QSV_M_MARGINAL, (B, 1 << m), mask=w.trash_mask)
    p0 = gu.measure(ctx, qb.QSV_M_PROJECT_ZERO, (B,), mask=w.trash_mask, renormalise=1)
    ctx.qsv_apply_layers(circ, pd, None, 1)
    F = gu.measure(ctx, qb.QSV_M_FIDELITY, (B,), x=xd)
    final = gu.state_np(ctx)
    oc = ocirc(oracle, w.circuit)
    ref, _ = oracle.amp_encode(w.x, n)
    oracle.apply_layers(ref, oc, w.params)
    with capsys.disabled():
        print(" [c3 oracle encoder done]", end="", flush=True)
    mref = oracle.marginal(ref, w.trash_mask)
    p0ref = oracle.project_zero(ref, w.trash_mask, renormalise=True)
    oracle.apply_layers(ref, oc, w.params, inverse=True)
    Fref = oracle.fidelity(ref, w.x)
    assert np.abs(marg - mref).max() <= 1e-5
    assert np.abs(p0 - p0ref).max() <= 1e-5
    assert np.abs(F - Fref).max() <= 1e-5
    assert np.abs(F - p0).max() <= 1e-5                     # invariant: F = P0 after renormalising
    d = np.abs(final - ref)
    assert d.max() <= 1e-5
    assert (d ** 2).sum(1).max() <= 1e-9                    # relative l2 error of the final state
    ctx.close()


def test_config4_full(oracle, capsys):
    torch = gu.torch_cuda()
    w = wl.config(4)
    n = w.n
    ctx = gu.make_ctx(n, 1)
    circ = qb.circuit_from_spec(w.circuit)
    xd, pd = gu.dev(w.x), gu.dev(w.params)
    ctx.qsv_amp_encode(xd)
    ctx.qsv_apply_layers(circ, pd, None, 0)
    p32 = gu.measure(ctx, qb.QSV_M_PROBS, (1, 1 << n))
    s = gu.measure(ctx, qb.QSV_M_SAMPLE, (1, w.uniforms.shape[1]), dtype="int64", uniforms=gu.dev(w.uniforms))
    assert abs(p32.astype(np.float64).sum() - 1.0) <= 1e-5
    assert np.array_equal(s, oracle.sample(p32, w.uniforms))        # bit-exact sampling
    # oracle, five layers at a time so that the run keeps reporting progress
    ref, _ = oracle.amp_encode(w.x, n)
    per = w.circuit.slots() * n
    for l0 in range(0, w.circuit.n_layers, 5):
        sub = oracle.make_circuit(5, list(w.circuit.rot), w.circuit.entangler, 0)
        oracle.apply_layers(ref, sub, w.params[l0 * per:(l0 + 5) * per])
        with capsys.disabled():
            print(" [c4 oracle layer %d]" % (l0 + 5), end="", flush=True)
    pref = oracle.probs(ref)
    gu.prob_checks(p32, pref)
    d = np.abs(gu.state_np(ctx) - ref)
    assert d.max() <= 1e-5 and (d ** 2).sum() <= 1e-9
    # the same circuit with every CNOT a register operation (the default defers those whose target
    # lies outside a pass's tile): the other plan, the same state
    ctx.qsv_set_option("defer_cnots", 0)
    ctx.qsv_amp_encode(xd)
    ctx.qsv_apply_layers(circ, pd, None, 0)
    d = np.abs(gu.state_np(ctx) - ref)
    assert d.max() <= 1e-5 and (d ** 2).sum() <= 1e-9
    ctx.qsv_set_option("defer_cnots", -1)
    del ref, pref, d
    # the inverse brings the state back to the encoded input
    ctx.qsv_apply_layers(circ, pd, None, 1)
    F = gu.measure(ctx, qb.QSV_M_FIDELITY, (1,), x=xd)
    assert abs(F[0] - 1.0) <= 1e-5
    ctx.close()


def test_largest_state_30_qubits_one_layer(oracle, capsys):
    """Maximum size the boundary accepts (n = 30: 8 GiB of state).  Only here does a tile span 2^29
    elements or more, which takes the pass kernel off its 32-bit addressing path.  One layer of
    RX,RY,RZ + CNOT ring and its inverse; the comparison walks the state in slices."""
    torch = gu.torch_cuda()
    n = 30
    spec = wl.CircuitSpec(1, (wl.RX, wl.RY, wl.RZ), wl.ENT_CNOT_RING)
    params = wl.draw_params(spec, n, 2030)
    g = np.random.Generator(np.random.PCG64(1030))
    x = g.random(1 << n, dtype=np.float32)[None, :] - np.float32(0.5)
    ctx = gu.make_ctx(n, 1)
    xd = gu.dev(x)
    ctx.qsv_amp_encode(xd)
    ctx.qsv_apply_layers(qb.circuit_from_spec(spec), gu.dev(params), None, 0)
    z = gu.measure(ctx, qb.QSV_M_EXPZ_ALL, (1, n))
    torch.cuda.synchronize()
    got = ctx.state.cpu().numpy()                      # [1][2^n][2] float32
    with capsys.disabled():
        print(" [n=30 gpu done]", end="", flush=True)
    ref, _ = oracle.amp_encode(x, n)
    oracle.apply_layers(ref, oracle.make_circuit(1, list(spec.rot), spec.entangler, 0), params)
    with capsys.disabled():
        print(" [n=30 oracle done]", end="", flush=True)
    assert np.abs(z - oracle.expz_all(ref)).max() <= 1e-5
    worst, err2, norm2 = 0.0, 0.0, 0.0
    step = 1 << 26
    for lo in range(0, 1 << n, step):
        r = ref[0, lo:lo + step]
        dr = got[0, lo:lo + step, 0].astype(np.float64) - r.real
        di = got[0, lo:lo + step, 1].astype(np.float64) - r.imag
        worst = max(worst, np.abs(dr).max(), np.abs(di).max())
        err2 += float((dr * dr).sum() + (di * di).sum())
        norm2 += float((got[0, lo:lo + step].astype(np.float64) ** 2).sum())
    assert worst <= 1e-7 and err2 <= 1e-10            # amplitudes are about 3e-5 in size
    assert abs(norm2 - 1.0) <= 1e-5
    del ref, got
    ctx.qsv_apply_layers(qb.circuit_from_spec(spec), gu.dev(params), None, 1)
    F = gu.measure(ctx, qb.QSV_M_FIDELITY, (1,), x=xd)
    assert abs(F[0] - 1.0) <= 1e-5
    ctx.close()


def test_config3_training_step_sampled(oracle):
    """Config 3 as a training step: loss 1 - P0 on the four trash qubits after the 20-layer encoder,
    its gradient for all 800 parameters and 32 samples in reverse mode, one Adam step.  The oracle
    recomputes the loss of two samples and their gradient for six parameters by the shift rule."""
    torch = gu.torch_cuda()
    w = wl.config(3)
    n, B = w.n, w.batch
    circ = qb.circuit_from_spec(w.circuit)
    P = w.circuit.num_params(n)
    ctx = gu.make_ctx(n, B, ws_bytes=qb.qsv_grad_workspace_bytes(n, B, circ))
    xd, pd = gu.dev(w.x), gu.dev(w.params)
    loss = torch.zeros(B, dtype=torch.float32, device="cuda")
    grad = torch.zeros((B, P), dtype=torch.float32, device="cuda")
    ml = torch.zeros(1, dtype=torch.float32, device="cuda")
    mg = torch.zeros(P, dtype=torch.float32, device="cuda")
    ctx.qsv_loss_grad(circ, xd, pd, None, qb.QSV_LOSS_TRASH, loss, grad, ml, mg, mask=w.trash_mask)
    torch.cuda.synchronize()
    gg, ll = grad.cpu().numpy(), loss.cpu().numpy()
    g = np.random.Generator(np.random.PCG64(6))
    rows = sorted(g.choice(B, 2, replace=False).tolist())
    sub = sorted(g.choice(P, 4, replace=False).tolist()) + [0, P - 1]
    lref, gref = oracle.loss_grad(w.x[rows], n, ocirc(oracle, w.circuit), w.params, kind=oracle.LOSS_TRASH,
                                  mask=w.trash_mask, subset=sub)
    assert np.abs(ll[rows] - lref).max() <= 1e-5
    assert np.abs(gg[rows][:, sub] - gref).max() <= 1e-4
    assert np.linalg.norm(gg[rows][:, sub] - gref) <= 1e-3 * np.linalg.norm(gref)
    assert abs(ml.item() - ll.astype(np.float64).mean()) <= 1e-6
    assert np.abs(mg.cpu().numpy() - gg.astype(np.float64).mean(0)).max() <= 1e-6
    m = torch.zeros(P, dtype=torch.float32, device="cuda")
    v = torch.zeros(P, dtype=torch.float32, device="cuda")
    ctx.qsv_adam_step(pd, mg, m, v, 1, 0.01)
    torch.cuda.synchronize()
    want, _, _ = oracle.adam_step(w.params, mg.cpu().numpy(), np.zeros(P), np.zeros(P), 1, 0.01)
    assert np.abs(pd.cpu().numpy() - want).max() <= 1e-6
    ctx.close()


def test_config1_training_step(oracle):
    """Config 1 as a training step: mean squared error of <Z_q> against seeded targets, gradient
    for all 180 parameters (re-upload weights included) and 1024 samples.  The oracle recomputes
    16 samples in full."""
    torch = gu.torch_cuda()
    w = wl.config(1)
    n, B = w.n, w.batch
    circ = qb.circuit_from_spec(w.circuit)
    P = w.circuit.num_params(n)
    y = np.random.Generator(np.random.PCG64(4001)).uniform(-1, 1, (B, n)).astype(np.float32)
    ctx = gu.make_ctx(n, B)
    loss = torch.zeros(B, dtype=torch.float32, device="cuda")
    grad = torch.zeros((B, P), dtype=torch.float32, device="cuda")
    mg = torch.zeros(P, dtype=torch.float32, device="cuda")
    ctx.qsv_loss_grad(circ, gu.dev(w.x), gu.dev(w.params), gu.dev(w.feats), qb.QSV_LOSS_MSE_Z, loss, grad,
                      None, mg, targets=gu.dev(y))
    torch.cuda.synchronize()
    gg, ll = grad.cpu().numpy(), loss.cpu().numpy()
    rows = list(range(0, B, 64))
    lref, gref = oracle.loss_grad(w.x[rows], n, ocirc(oracle, w.circuit), w.params, w.feats[rows],
                                  kind=oracle.LOSS_MSE_Z, targets=y[rows])
    assert np.abs(ll[rows] - lref).max() <= 1e-5
    assert np.abs(gg[rows] - gref).max() <= 1e-4
    assert np.linalg.norm(gg[rows] - gref) <= 1e-3 * np.linalg.norm(gref)
    assert np.abs(mg.cpu().numpy() - gg.astype(np.float64).mean(0)).max() <= 1e-6
    ctx.close()


def test_config3_true_reset_fidelity_sampled(oracle):
    """Config 3 with a real reset of the four trash qubits (16 decoder runs per sample); the oracle
    recomputes two samples from the GPU's encoder output."""
    torch = gu.torch_cuda()
    w = wl.config(3)
    n, B = w.n, w.batch
    circ = qb.circuit_from_spec(w.circuit)
    ctx = gu.make_ctx(n, B, ws_bytes=qb.qsv_grad_workspace_bytes(n, B, circ))
    xd, pd = gu.dev(w.x), gu.dev(w.params)
    ctx.qsv_amp_encode(xd)
    ctx.qsv_apply_layers(circ, pd, None, 0)
    F = torch.zeros(B, dtype=torch.float32, device="cuda")
    ctx.qsv_reset_fidelity(circ, pd, None, w.trash_mask, xd, F)
    p0 = gu.measure(ctx, qb.QSV_M_MARGINAL, (B, 16), mask=w.trash_mask)[:, 0]
    Fg = F.cpu().numpy()
    rows = [3, 20]
    enc = gu.state_np(ctx)[rows]
    want = oracle.reset_fidelity(np.ascontiguousarray(enc), ocirc(oracle, w.circuit), w.params, None,
                                 w.trash_mask, w.x[rows])
    assert np.abs(Fg[rows] - want).max() <= 1e-5
    # the t = 0 term alone is P0^2 (projection without renormalising), so F >= P0^2
    assert np.all(Fg >= p0.astype(np.float64) ** 2 - 1e-5) and np.all(Fg <= 1 + 1e-5)
    ctx.close()
