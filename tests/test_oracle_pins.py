"""Pins for the CPU oracle: closed forms, truth tables, dense brute force, finite differences.

None of these re-types the oracle's own loops: each compares it with something fixed by the
mathematics (a closed form, an integer bit permutation, a Kronecker-product matrix, a central
finite difference, an analytic identity), so that a dropped term, wrong sign, wrong qubit order or
transposed matrix anywhere in the oracle fails at least one of them.
"""
import itertools
import os

import numpy as np
import pytest

from tests import dense_bruteforce as dense

RX, RY, RZ = 1, 2, 3
NONE, RING, LADDER = 0, 1, 2
HERE = os.path.dirname(os.path.abspath(__file__))


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ------------------------------------------------------------------ encoding
def test_encode_closed_form_and_padding(oracle):
    x = rng(1).standard_normal((5, 11)).astype(np.float32)
    st, nrm = oracle.amp_encode(x, 4)
    xd = x.astype(np.float64)
    assert np.allclose(nrm, np.sqrt((xd ** 2).sum(1)), rtol=1e-14)
    p = oracle.probs(st)
    assert np.allclose(p[:, :11], xd ** 2 / (xd ** 2).sum(1, keepdims=True), atol=1e-15)
    assert np.all(p[:, 11:] == 0.0) and np.all(st.imag == 0.0)
    assert np.allclose(p.sum(1), 1.0, atol=1e-14)
    # sign of the amplitudes is the sign of x
    assert np.all(np.sign(st.real[:, :11]) == np.sign(xd))


def test_encode_idempotent_and_zero_vector(oracle):
    x = rng(2).standard_normal((3, 8)).astype(np.float32)
    st, _ = oracle.amp_encode(x, 3)
    st2, _ = oracle.amp_encode((3.5 * x).astype(np.float32), 3)
    assert np.allclose(st, st2, atol=1e-7)
    x[1] = 0.0
    st, nrm = oracle.amp_encode(x, 3)
    assert nrm[1] == 0.0 and np.all(st[1] == 0.0) and not np.isnan(st).any()


def test_encode_rejects_bad_dim(oracle):
    with pytest.raises(ValueError):
        oracle.amp_encode(np.ones((1, 9), np.float32), 3)


# ------------------------------------------------------------------ single gates, closed forms
@pytest.mark.parametrize("theta", [0.0, 0.3, 1.0, np.pi / 2, 2.5, np.pi, 4.0, 6.0])
def test_ry_closed_form(oracle, theta):
    st = oracle.zero_state(1, 3)
    oracle.gate_rot(st, RY, 1, theta)
    p = oracle.probs(st)[0]
    assert abs(p[0] - np.cos(theta / 2) ** 2) < 1e-15      # P(0) = cos^2(theta/2)
    assert abs(p[2] - np.sin(theta / 2) ** 2) < 1e-15      # qubit 1 <-> index bit 1
    assert abs(oracle.expz_all(st)[0, 1] - np.cos(theta)) < 1e-15
    assert abs(st[0, 2].real - np.sin(theta / 2)) < 1e-15 and st[0, 2].imag == 0.0  # sign of s


@pytest.mark.parametrize("theta", [0.4, np.pi / 2, np.pi, 5.0])
def test_rx_closed_form(oracle, theta):
    st = oracle.zero_state(1, 2)
    oracle.gate_rot(st, RX, 0, theta)
    assert abs(oracle.probs(st)[0, 1] - np.sin(theta / 2) ** 2) < 1e-15
    assert abs(st[0, 1] - (-1j * np.sin(theta / 2))) < 1e-15  # RX(pi)|0> = -i|1>
    assert abs(st[0, 0] - np.cos(theta / 2)) < 1e-15


@pytest.mark.parametrize("phi", [0.3, 1.7, np.pi, 4.4])
def test_rz_phase(oracle, phi):
    x = rng(3).standard_normal((2, 8)).astype(np.float32)
    st, _ = oracle.amp_encode(x, 3)
    p0 = oracle.probs(st)
    ref = st.copy()
    oracle.gate_rot(st, RZ, 2, phi)
    assert np.allclose(oracle.probs(st), p0, atol=1e-15)   # diagonal: probabilities unchanged
    # amplitudes with qubit 2 = 0 pick up e^{-i phi/2}, the others e^{+i phi/2}
    assert np.allclose(st[:, :4], ref[:, :4] * np.exp(-0.5j * phi), atol=1e-15)
    assert np.allclose(st[:, 4:], ref[:, 4:] * np.exp(+0.5j * phi), atol=1e-15)
    oracle.gate_rot(st, RZ, 2, -phi)
    assert np.allclose(st, ref, atol=1e-15)
    # relative phase seen through RY(pi/2) RZ(phi) RY(-pi/2) on |0>: P(0) = cos^2(phi/2)
    s = oracle.zero_state(1, 1)
    oracle.gate_rot(s, RY, 0, -np.pi / 2)
    oracle.gate_rot(s, RZ, 0, phi)
    oracle.gate_rot(s, RY, 0, np.pi / 2)
    assert abs(oracle.probs(s)[0, 0] - np.cos(phi / 2) ** 2) < 1e-15


def test_rotation_matrix_orientation(oracle):
    """RY on |1> gives (-s, c): catches a transposed 2x2."""
    st = np.zeros((1, 2), dtype=np.complex128)
    st[0, 1] = 1.0
    oracle.gate_rot(st, RY, 0, 0.7)
    assert np.allclose(st[0], [-np.sin(0.35), np.cos(0.35)], atol=1e-15)


# ------------------------------------------------------------------ entanglers
def test_cnot_truth_table(oracle):
    n = 3
    for ctrl, tgt in itertools.permutations(range(n), 2):
        for k in range(1 << n):
            st = np.zeros((1, 1 << n), dtype=np.complex128)
            st[0, k] = 1.0
            oracle.gate_cnot(st, ctrl, tgt)
            k2 = k ^ (1 << tgt) if (k >> ctrl) & 1 else k
            assert st[0, k2] == 1.0 and np.count_nonzero(st) == 1


def ring_image(k, n):
    """Image of basis state k under CNOT(0,1), CNOT(1,2), ..., CNOT(n-1,0), by bit operations."""
    b = [(k >> q) & 1 for q in range(n)]
    for q in range(n):
        b[(q + 1) % n] ^= b[q]
    return sum(v << q for q, v in enumerate(b))


@pytest.mark.parametrize("n", [2, 3, 4, 5, 7])
@pytest.mark.parametrize("mode", [1, 2])
def test_cnot_ring_permutation(oracle, n, mode):
    circ = oracle.make_circuit(1, [], RING)
    N = 1 << n
    st = np.eye(N, dtype=np.complex128)          # sample k = basis state k
    oracle.apply_layers(st, circ, np.zeros(0), mode=mode)
    for k in range(N):
        assert st[k, ring_image(k, n)] == 1.0 and np.count_nonzero(st[k]) == 1
    # closed form of the ring: prefix XOR, then bit 0 ^= parity of all bits
    k = 0b1011 if n >= 4 else 0b11
    b = [(k >> q) & 1 for q in range(n)]
    pre = np.bitwise_xor.accumulate(b)
    pre[0] = b[0] ^ pre[n - 1]
    assert ring_image(k, n) == sum(int(v) << q for q, v in enumerate(pre))
    oracle.apply_layers(st, circ, np.zeros(0), inverse=True, mode=mode)
    assert np.array_equal(st, np.eye(N))


def test_ghz_from_chain(oracle):
    n = 4
    st = oracle.zero_state(1, n)
    oracle.gate_rot(st, RY, 0, np.pi / 2)
    for q in range(n - 1):
        oracle.gate_cnot(st, q, q + 1)
    p = oracle.probs(st)[0]
    assert abs(p[0] - 0.5) < 1e-15 and abs(p[-1] - 0.5) < 1e-15
    assert np.allclose(oracle.expz_all(st), 0.0, atol=1e-15)
    gold = np.loadtxt(os.path.join(HERE, "golden", "ghz4_probs.txt"))
    assert np.allclose(p, gold, atol=1e-15)


@pytest.mark.parametrize("n", [2, 3, 5])
@pytest.mark.parametrize("mode", [1, 2])
def test_cz_ladder(oracle, n, mode):
    circ = oracle.make_circuit(1, [], LADDER)
    st = np.eye(1 << n, dtype=np.complex128)
    oracle.apply_layers(st, circ, np.zeros(0), mode=mode)
    for k in range(1 << n):
        sign = (-1) ** bin(k & (k >> 1)).count("1")
        assert st[k, k] == sign and np.count_nonzero(st[k]) == 1
    plus = oracle.zero_state(1, n)
    for q in range(n):
        oracle.gate_rot(plus, RY, q, np.pi / 2)
    oracle.apply_layers(plus, circ, np.zeros(0), mode=mode)
    assert np.allclose(oracle.probs(plus), 2.0 ** -n, atol=1e-15)
    assert np.allclose(oracle.expz_all(plus), 0.0, atol=1e-15)


# ------------------------------------------------------------------ whole circuits, dense brute force
CASES = [
    (2, 2, (RY, RZ), RING, 0), (3, 2, (RY, RZ), RING, 0), (4, 2, (RY, RZ), RING, 0),
    (5, 3, (RX, RY, RZ), RING, 0), (6, 2, (RX, RY, RZ), RING, 0),
    (4, 3, (RY, RZ), LADDER, 0), (6, 2, (RY, RZ), LADDER, 0),
    (3, 2, (RZ, RX), NONE, 0), (1, 3, (RX, RY, RZ), RING, 0),
    (4, 3, (RY, RZ), RING, 1), (5, 2, (RY, RZ), LADDER, 1), (3, 2, (), RING, 1),
]


@pytest.mark.parametrize("n,L,rot,ent,reup", CASES)
@pytest.mark.parametrize("inverse", [False, True])
@pytest.mark.parametrize("mode", [1, 2])          # one thread per sample; pair loops split (the n >= 18 path)
def test_circuit_vs_dense(oracle, n, L, rot, ent, reup, inverse, mode):
    g = rng(100 + n * 7 + L + ent + reup)
    circ = oracle.make_circuit(L, list(rot), ent, reup)
    P = oracle.num_params(circ, n)
    assert P == L * (reup + len(rot)) * n
    params = g.uniform(0, 2 * np.pi, P)
    B = 3
    x = g.standard_normal((B, 1 << n)).astype(np.float32)
    feats = g.standard_normal((B, n)) if reup else None
    st, _ = oracle.amp_encode(x, n)
    start = st.copy()
    oracle.apply_layers(st, circ, params, feats, inverse=inverse, mode=mode)
    for b in range(B):
        U = dense.circuit_unitary(n, L, rot, ent, reup, params, feats[b] if reup else None)
        if inverse:
            U = U.conj().T
        assert np.allclose(st[b], U @ start[b], atol=1e-13)
    assert np.allclose(oracle.probs(st).sum(1), 1.0, atol=1e-12)     # norm preservation


@pytest.mark.parametrize("n,L,rot,ent,reup", CASES)
def test_encoder_times_inverse_is_identity(oracle, n, L, rot, ent, reup):
    g = rng(200 + n)
    circ = oracle.make_circuit(L, list(rot), ent, reup)
    params = g.uniform(0, 2 * np.pi, oracle.num_params(circ, n))
    x = g.standard_normal((4, 1 << n)).astype(np.float32)
    feats = g.standard_normal((4, n)) if reup else None
    st, _ = oracle.amp_encode(x, n)
    start = st.copy()
    oracle.apply_layers(st, circ, params, feats)
    assert not np.allclose(st, start, atol=1e-3) or L == 0
    oracle.apply_layers(st, circ, params, feats, inverse=True)
    assert np.allclose(st, start, atol=1e-13)
    xd = x.astype(np.float64)
    assert np.allclose(oracle.probs(st), xd ** 2 / (xd ** 2).sum(1, keepdims=True), atol=1e-13)


def test_larger_n_unitarity_and_inverse(oracle):
    """n = 12: too large for the dense check, pinned by norm and by U^-1 U = I."""
    n, g = 12, rng(7)
    circ = oracle.make_circuit(4, [RX, RY, RZ], RING)
    params = g.uniform(0, 2 * np.pi, oracle.num_params(circ, n))
    x = g.standard_normal((2, 1 << n)).astype(np.float32)
    st, _ = oracle.amp_encode(x, n)
    start = st.copy()
    oracle.apply_layers(st, circ, params)
    assert np.allclose(oracle.probs(st).sum(1), 1.0, atol=1e-12)
    oracle.apply_layers(st, circ, params, inverse=True)
    assert np.allclose(st, start, atol=1e-12)


# ------------------------------------------------------------------ measurement
def test_expz_from_probs_and_range(oracle):
    n, g = 6, rng(8)
    circ = oracle.make_circuit(2, [RY, RZ], RING)
    st, _ = oracle.amp_encode(g.standard_normal((3, 1 << n)).astype(np.float32), n)
    oracle.apply_layers(st, circ, g.uniform(0, 6.28, oracle.num_params(circ, n)))
    p, z = oracle.probs(st), oracle.expz_all(st)
    k = np.arange(1 << n)
    for q in range(n):
        assert np.allclose(z[:, q], (p * (1 - 2 * ((k >> q) & 1))).sum(1), atol=1e-14)
    assert np.all(np.abs(z) <= 1.0 + 1e-14)


@pytest.mark.parametrize("mask", [0b000001, 0b110000, 0b101010, 0b011110, 0b111111])
def test_marginal_and_projection(oracle, mask):
    n, g = 6, rng(9)
    circ = oracle.make_circuit(2, [RY, RZ], RING)
    x = g.standard_normal((3, 1 << n)).astype(np.float32)
    params = g.uniform(0, 6.28, oracle.num_params(circ, n))
    st, _ = oracle.amp_encode(x, n)
    oracle.apply_layers(st, circ, params)
    p = oracle.probs(st)
    marg = oracle.marginal(st, mask)
    assert np.allclose(marg.sum(1), 1.0, atol=1e-13)
    # brute force by string manipulation of the index
    bits = [q for q in range(n) if (mask >> q) & 1]
    ref = np.zeros_like(marg)
    for k in range(1 << n):
        v = sum(((k >> q) & 1) << j for j, q in enumerate(bits))
        ref[:, v] += p[:, k]
    assert np.allclose(marg, ref, atol=1e-14)
    # projection with and without renormalisation; fidelity invariants F = P0, P0^2, 1
    keep = (np.arange(1 << n) & mask) == 0
    for renorm, power in ((True, 1), (False, 2)):
        s2 = st.copy()
        p0 = oracle.project_zero(s2, mask, renormalise=renorm)
        assert np.allclose(p0, marg[:, 0], atol=1e-14)
        assert np.all(s2[:, ~keep] == 0)
        scale = 1 / np.sqrt(p0)[:, None] if renorm else 1.0
        assert np.allclose(s2[:, keep], st[:, keep] * scale, atol=1e-14)
        oracle.apply_layers(s2, circ, params, inverse=True)
        assert np.allclose(oracle.fidelity(s2, x), p0 ** power, atol=1e-13)
    s3 = st.copy()
    oracle.apply_layers(s3, circ, params, inverse=True)
    assert np.allclose(oracle.fidelity(s3, x), 1.0, atol=1e-13)


def test_fidelity_definition(oracle):
    g = rng(10)
    x = g.standard_normal((2, 8)).astype(np.float32)
    st = (g.standard_normal((2, 8)) + 1j * g.standard_normal((2, 8)))
    st /= np.linalg.norm(st, axis=1, keepdims=True)
    st = np.ascontiguousarray(st)
    xd = x.astype(np.float64)
    ain = xd / np.linalg.norm(xd, axis=1, keepdims=True)
    ref = np.abs((ain.conj() * st).sum(1)) ** 2
    assert np.allclose(oracle.fidelity(st, x), ref, atol=1e-14)


# ------------------------------------------------------------------ parameter shift
def test_param_shift_single_ry_closed_form(oracle):
    circ = oracle.make_circuit(1, [RY], NONE)
    x = np.array([[1.0, 0.0]], dtype=np.float32)          # |0>
    for theta in (0.2, 1.1, 2.9, 5.0):
        loss, grad = oracle.param_shift_grad(x, 1, circ, [theta])
        assert abs(loss[0] - np.cos(theta)) < 1e-15
        assert abs(grad[0, 0] + np.sin(theta)) < 1e-15     # d cos / d theta = -sin


@pytest.mark.parametrize("n,L,rot,ent,reup", [
    (3, 2, (RY, RZ), LADDER, 0), (4, 2, (RX, RY, RZ), RING, 0), (3, 2, (RY, RZ), RING, 1)])
def test_param_shift_vs_finite_difference(oracle, n, L, rot, ent, reup):
    g = rng(11 + n + reup)
    circ = oracle.make_circuit(L, list(rot), ent, reup)
    P = oracle.num_params(circ, n)
    params = g.uniform(0, 2 * np.pi, P)
    B = 2
    x = g.standard_normal((B, 1 << n)).astype(np.float32)
    feats = g.standard_normal((B, n)) if reup else None
    obs = 1
    loss, grad = oracle.param_shift_grad(x, n, circ, params, feats, obs_qubit=obs)

    def f(pv):
        st, _ = oracle.amp_encode(x, n)
        oracle.apply_layers(st, circ, pv, feats)
        return oracle.expz_all(st)[:, obs]

    assert np.allclose(loss, f(params), atol=1e-14)
    h = 1e-4
    for p in range(P):
        e = np.zeros(P)
        e[p] = h
        fd = (f(params + e) - f(params - e)) / (2 * h)
        assert np.allclose(grad[:, p], fd, atol=1e-7), p
    # subset interface returns the same columns
    sub = [P - 1, 0, 3]
    _, gs = oracle.param_shift_grad(x, n, circ, params, feats, obs_qubit=obs, subset=sub)
    assert np.array_equal(gs, grad[:, sub])


# ------------------------------------------------------------------ sampler
def test_sampler_uniform_closed_form(oracle):
    n = 10
    p = np.full((2, 1 << n), 2.0 ** -n, dtype=np.float32)
    u = rng(12).random((2, 500))
    s = oracle.sample(p, u)
    assert np.array_equal(s, np.floor(u * (1 << n)).astype(np.int64))


def test_sampler_basis_state_and_zero_weights(oracle):
    n = 8
    p = np.zeros((1, 1 << n), dtype=np.float32)
    p[0, 77] = 1.0
    u = rng(13).random((1, 100))
    assert np.all(oracle.sample(p, u) == 77)
    p[0, 77] = 0.25
    p[0, 200] = 0.75
    s = oracle.sample(p, np.array([[0.0, 0.2499999, 0.25, 0.9999999]]))
    assert s.tolist() == [[77, 77, 200, 200]]
    p[:] = 0
    assert np.all(oracle.sample(p, u) == -1)


def test_sampler_matches_python_integers_and_histogram(oracle):
    n, g = 7, rng(14)
    w = g.random(1 << n)
    w[g.random(1 << n) < 0.2] = 0.0
    p = (w / w.sum()).astype(np.float32)[None, :]
    u = g.random((1, 20000))
    s = oracle.sample(p, u)
    # exact rule re-done with Python's arbitrary-precision integers
    wk = [int(np.floor(np.ldexp(np.float64(v), 60))) for v in p[0]]
    cum = np.cumsum(np.array(wk, dtype=object))
    total = int(cum[-1])
    for j in range(0, 20000, 37):
        r = int(np.floor(np.ldexp(u[0, j], 53)))
        t = (r * total) >> 53
        k = next(i for i, c in enumerate(cum) if c > t)
        assert s[0, j] == k
    assert not np.any(p[0, s[0]] == 0.0)                       # zero-weight outcomes never drawn
    hist = np.bincount(s[0], minlength=1 << n) / 20000.0
    sigma = np.sqrt(p[0] * (1 - p[0]) / 20000.0)
    assert np.all(np.abs(hist - p[0]) <= 5 * sigma + 1e-9)


# ------------------------------------------------------------------ threading, and the large-n path
def test_threads_do_not_change_results(oracle):
    g = rng(15)
    for n, ent in ((5, RING), (18, RING), (18, LADDER)):
        circ = oracle.make_circuit(2, [RX, RY, RZ], ent)
        params = g.uniform(0, 6.28, oracle.num_params(circ, n))
        x = g.standard_normal((2, 1 << n)).astype(np.float32)
        outs = []
        for t in (1, oracle.max_threads()):
            oracle.set_threads(t)
            st, _ = oracle.amp_encode(x, n)
            oracle.apply_layers(st, circ, params)
            outs.append(st)
        oracle.set_threads(oracle.max_threads())
        assert np.array_equal(outs[0], outs[1])


def apply_gate_by_gate(oracle, st, n, L, rot, ent, reup, params, feats, inverse):
    """The circuit through the single-gate entry points (oracle_gate_rot / cnot / cz), in the order
    the benchmark spec gives; the gate entry points are the ones the closed forms above pin."""
    slots = reup + len(rot)
    p = np.asarray(params, dtype=np.float64).reshape(L, slots, n)

    def angle(l, slot, q, b):
        return p[l, slot, q] * (feats[b, q] if (reup and slot == 0) else 1.0)

    for b in range(st.shape[0]):
        row = st[b:b + 1]
        if not inverse:
            for l in range(L):
                for slot in range(slots):
                    axis = RX if (reup and slot == 0) else rot[slot - reup]
                    for q in range(n):
                        oracle.gate_rot(row, axis, q, angle(l, slot, q, b))
                if ent == RING and n >= 2:
                    for q in range(n):
                        oracle.gate_cnot(row, q, (q + 1) % n)
                if ent == LADDER:
                    for q in range(n - 1):
                        oracle.gate_cz(row, q, q + 1)
        else:
            for l in reversed(range(L)):
                if ent == RING and n >= 2:
                    for q in reversed(range(n)):
                        oracle.gate_cnot(row, q, (q + 1) % n)
                if ent == LADDER:
                    for q in reversed(range(n - 1)):
                        oracle.gate_cz(row, q, q + 1)
                for slot in reversed(range(slots)):
                    axis = RX if (reup and slot == 0) else rot[slot - reup]
                    for q in reversed(range(n)):
                        oracle.gate_rot(row, axis, q, -angle(l, slot, q, b))


@pytest.mark.parametrize("rot,ent,reup", [((RX, RY, RZ), RING, 0), ((RY, RZ), LADDER, 0), ((RZ, RX), RING, 1)])
@pytest.mark.parametrize("inverse", [False, True])
def test_large_n_path_equals_gate_by_gate(oracle, rot, ent, reup, inverse):
    """n = 18 is where apply_layers switches to pair-parallel gates (the path that judges the 20-,
    26- and 30-qubit GPU runs): it must give, bit for bit, what the single-gate entry points give,
    and what the per-sample mode gives."""
    n, L, B = 18, 2, 2
    g = rng(160 + ent + reup)
    circ = oracle.make_circuit(L, list(rot), ent, reup)
    params = g.uniform(0, 2 * np.pi, oracle.num_params(circ, n))
    x = g.standard_normal((B, 1 << n)).astype(np.float32)
    feats = g.standard_normal((B, n)) if reup else None
    st, _ = oracle.amp_encode(x, n)
    ref = st.copy()
    per_sample = st.copy()
    oracle.apply_layers(st, circ, params, feats, inverse=inverse)            # auto: pair-parallel at n = 18
    oracle.apply_layers(per_sample, circ, params, feats, inverse=inverse, mode=1)
    apply_gate_by_gate(oracle, ref, n, L, rot, ent, reup, params, feats, inverse)
    assert np.array_equal(st, ref)
    assert np.array_equal(st, per_sample)


def test_small_n_modes_agree_bit_for_bit(oracle):
    n, g = 5, rng(170)
    for ent in (RING, LADDER):
        circ = oracle.make_circuit(3, [RX, RY, RZ], ent, 1)
        params = g.uniform(0, 2 * np.pi, oracle.num_params(circ, n))
        feats = g.standard_normal((3, n))
        st, _ = oracle.amp_encode(g.standard_normal((3, 1 << n)).astype(np.float32), n)
        a, b = st.copy(), st.copy()
        oracle.apply_layers(a, circ, params, feats, mode=1)
        oracle.apply_layers(b, circ, params, feats, mode=2)
        assert np.array_equal(a, b)


def test_large_n_closed_forms(oracle):
    """Closed forms at n = 18 through the pair-parallel path."""
    n = 18
    N = 1 << n
    # (1) GHZ: RY(pi/2) on qubit 0, then the ring.  The chain CNOT(0,1)..CNOT(16,17) spreads qubit 0 over
    # all qubits; the closing CNOT(17,0) then clears qubit 0 in the |1..1> branch: (|0..0> + |01..1>)/sqrt 2
    # in index order (qubit 0 = lowest bit), i.e. indices 0 and 2^18 - 2.
    circ = oracle.make_circuit(1, [RY], RING)
    params = np.zeros(n)
    params[0] = np.pi / 2
    st = oracle.zero_state(1, n)
    oracle.apply_layers(st, circ, params)
    p = oracle.probs(st)[0]
    assert abs(p[0] - 0.5) < 1e-15 and abs(p[N - 2] - 0.5) < 1e-15 and np.count_nonzero(p) == 2
    z = oracle.expz_all(st)[0]
    assert abs(z[0] - 1.0) < 1e-15 and np.allclose(z[1:], 0.0, atol=1e-15)
    # (2) the ring as a permutation of basis states, from integer bit operations
    ring = oracle.make_circuit(1, [], RING)
    ks = [1, 2, 0b1011, N - 1, N >> 1, 0x2A5A5, 0x15A5A]
    st = np.zeros((len(ks), N), dtype=np.complex128)
    for i, k in enumerate(ks):
        st[i, k] = 1.0
    oracle.apply_layers(st, ring, np.zeros(0))
    for i, k in enumerate(ks):
        assert st[i, ring_image(k, n)] == 1.0 and np.count_nonzero(st[i]) == 1
    oracle.apply_layers(st, ring, np.zeros(0), inverse=True)
    for i, k in enumerate(ks):
        assert st[i, k] == 1.0 and np.count_nonzero(st[i]) == 1
    # (3) CZ ladder: sign (-1)^popcount(k & (k >> 1)) on basis states; |+..+> stays uniform
    lad = oracle.make_circuit(1, [], LADDER)
    st = np.zeros((len(ks), N), dtype=np.complex128)
    for i, k in enumerate(ks):
        st[i, k] = 1.0
    oracle.apply_layers(st, lad, np.zeros(0))
    for i, k in enumerate(ks):
        assert st[i, k] == (-1) ** bin(k & (k >> 1)).count("1") and np.count_nonzero(st[i]) == 1
    plus = oracle.make_circuit(1, [RY], LADDER)
    st = oracle.zero_state(1, n)
    oracle.apply_layers(st, plus, np.full(n, np.pi / 2))
    assert np.allclose(oracle.probs(st), 2.0 ** -n, atol=1e-18)
    # (4) one RY, RX, RZ on a high qubit: P(bit set) = sin^2(theta/2); RZ leaves probabilities alone
    for axis, q, theta in ((RY, 17, 0.7), (RX, 9, 2.1)):
        one = oracle.make_circuit(1, [axis], NONE)
        params = np.zeros(n)
        params[q] = theta
        st = oracle.zero_state(1, n)
        oracle.apply_layers(st, one, params)
        p = oracle.probs(st)[0]
        assert abs(p[0] - np.cos(theta / 2) ** 2) < 1e-15 and abs(p[1 << q] - np.sin(theta / 2) ** 2) < 1e-15
        want = np.sin(theta / 2) if axis == RY else -1j * np.sin(theta / 2)
        assert abs(st[0, 1 << q] - want) < 1e-15
    # (5) encoder then decoder is the identity; norm preserved in between
    g = rng(171)
    circ = oracle.make_circuit(2, [RX, RY, RZ], RING)
    params = g.uniform(0, 2 * np.pi, oracle.num_params(circ, n))
    st, _ = oracle.amp_encode(g.standard_normal((1, N)).astype(np.float32), n)
    start = st.copy()
    oracle.apply_layers(st, circ, params)
    assert abs(oracle.probs(st).sum() - 1.0) < 1e-12 and not np.allclose(st, start, atol=1e-3)
    oracle.apply_layers(st, circ, params, inverse=True)
    assert np.allclose(st, start, atol=1e-13)


# ------------------------------------------------------------------ training losses and optimisers
def test_loss_grad_single_ry_closed_forms(oracle):
    """|0> -> RY(theta): P(qubit reads 0) = cos^2(theta/2), <Z> = cos(theta)."""
    circ = oracle.make_circuit(1, [RY], NONE)
    x = np.array([[1.0, 0.0]], dtype=np.float32)
    for theta in (0.3, 1.2, 2.5, 4.4):
        loss, grad = oracle.loss_grad(x, 1, circ, [theta], kind=oracle.LOSS_TRASH, mask=1)
        assert abs(loss[0] - np.sin(theta / 2) ** 2) < 1e-15
        assert abs(grad[0, 0] - 0.5 * np.sin(theta)) < 1e-15
        y = np.array([[0.37]])
        loss, grad = oracle.loss_grad(x, 1, circ, [theta], kind=oracle.LOSS_MSE_Z, targets=y)
        assert abs(loss[0] - (np.cos(theta) - 0.37) ** 2) < 1e-15
        assert abs(grad[0, 0] + 2 * (np.cos(theta) - 0.37) * np.sin(theta)) < 1e-15


@pytest.mark.parametrize("n,L,rot,ent,reup,kind", [
    (3, 2, (RY, RZ), LADDER, 0, 1), (4, 2, (RX, RY, RZ), RING, 0, 1), (3, 2, (RY, RZ), RING, 1, 1),
    (3, 2, (RY, RZ), LADDER, 0, 2), (4, 1, (RX, RY, RZ), RING, 0, 2), (3, 2, (RY, RZ), RING, 1, 2)])
def test_loss_grad_vs_finite_difference(oracle, n, L, rot, ent, reup, kind):
    """The loss is recomputed here from separately pinned pieces (apply_layers, marginal, expz_all),
    and its central finite difference must match the shift-rule gradient."""
    g = rng(70 + n + 2 * reup + kind)
    circ = oracle.make_circuit(L, list(rot), ent, reup)
    P = oracle.num_params(circ, n)
    params = g.uniform(0, 2 * np.pi, P)
    B = 2
    x = g.standard_normal((B, 1 << n)).astype(np.float32)
    feats = g.standard_normal((B, n)) if reup else None
    mask = 0b101 if kind == 1 else 0
    y = g.uniform(-1, 1, (B, n)) if kind == 2 else None
    loss, grad = oracle.loss_grad(x, n, circ, params, feats, kind=kind, mask=mask, targets=y)

    def f(pv):
        st, _ = oracle.amp_encode(x, n)
        oracle.apply_layers(st, circ, pv, feats)
        if kind == 1:
            return 1.0 - oracle.marginal(st, mask)[:, 0]
        return ((oracle.expz_all(st) - y) ** 2).mean(1)

    assert np.allclose(loss, f(params), atol=1e-14)
    h = 1e-4
    for p in range(P):
        e = np.zeros(P)
        e[p] = h
        fd = (f(params + e) - f(params - e)) / (2 * h)
        assert np.allclose(grad[:, p], fd, atol=2e-7), p
    sub = [P - 1, 0, 2]
    _, gs = oracle.loss_grad(x, n, circ, params, feats, kind=kind, mask=mask, targets=y, subset=sub)
    assert np.array_equal(gs, grad[:, sub])


def test_loss_grad_special_cases(oracle):
    g = rng(77)
    n = 3
    circ = oracle.make_circuit(2, [RY, RZ], RING)
    P = oracle.num_params(circ, n)
    params = g.uniform(0, 2 * np.pi, P)
    x = g.standard_normal((2, 8)).astype(np.float32)
    # targets equal to the circuit's own <Z_q>: the loss and its gradient vanish
    st, _ = oracle.amp_encode(x, n)
    oracle.apply_layers(st, circ, params)
    loss, grad = oracle.loss_grad(x, n, circ, params, kind=oracle.LOSS_MSE_Z, targets=oracle.expz_all(st))
    assert np.all(np.abs(loss) < 1e-28) and np.all(np.abs(grad) < 1e-14)
    # one trash qubit q: 1 - P0 = (1 - <Z_q>) / 2, so the gradient is minus half the <Z_q> gradient
    for q in range(n):
        lt, gt = oracle.loss_grad(x, n, circ, params, kind=oracle.LOSS_TRASH, mask=1 << q)
        lz, gz = oracle.param_shift_grad(x, n, circ, params, obs_qubit=q)
        assert np.allclose(lt, 0.5 * (1 - lz), atol=1e-14) and np.allclose(gt, -0.5 * gz, atol=1e-14)
    assert np.all((lt >= 0) & (lt <= 1))


def test_optimiser_steps_closed_forms(oracle):
    p = np.array([1.0, -2.0, 0.5], dtype=np.float32)
    g = np.array([0.25, -4.0, 0.0], dtype=np.float32)
    assert np.array_equal(oracle.sgd_step(p, g, 0.5), np.array([0.875, 0.0, 0.5], dtype=np.float32))
    # first Adam step from zero moments: m_hat = g, v_hat = g^2, so the step is lr * g / (|g| + eps)
    lr, eps = 0.01, 1e-8
    p1, m1, v1 = oracle.adam_step(p, g, np.zeros(3), np.zeros(3), 1, lr, 0.9, 0.999, eps)
    want = p.astype(np.float64) - lr * g / (np.abs(g) + eps)
    assert np.allclose(p1, want, atol=1e-7) and p1[2] == p[2]
    assert np.allclose(m1, 0.1 * g, atol=1e-9) and np.allclose(v1, 0.001 * g.astype(np.float64) ** 2, atol=1e-9)
    # constant gradient: the bias-corrected moments stay at g and g^2, every step has the same size
    q, m, v = p.copy(), np.zeros(3), np.zeros(3)
    for t in range(1, 6):
        q, m, v = oracle.adam_step(q, g, m, v, t, lr)
    assert np.allclose(q, p - 5 * lr * np.sign(g), atol=1e-5)


# ------------------------------------------------------------------ Pauli strings
def test_pauli_single_qubit_closed_forms(oracle):
    x = np.array([[1.0, 0.0]], dtype=np.float32)
    for theta in (0.4, 1.3, 2.2, 5.1):
        st, _ = oracle.amp_encode(x, 1)
        oracle.gate_rot(st, RY, 0, theta)                   # cos(t/2)|0> + sin(t/2)|1>
        assert abs(oracle.pauli_expect(st, xmask=1)[0] - np.sin(theta)) < 1e-15
        assert abs(oracle.pauli_expect(st, ymask=1)[0]) < 1e-15
        assert abs(oracle.pauli_expect(st, zmask=1)[0] - np.cos(theta)) < 1e-15
        st, _ = oracle.amp_encode(x, 1)
        oracle.gate_rot(st, RX, 0, theta)                   # cos(t/2)|0> - i sin(t/2)|1>
        assert abs(oracle.pauli_expect(st, ymask=1)[0] + np.sin(theta)) < 1e-15
        assert abs(oracle.pauli_expect(st, xmask=1)[0]) < 1e-15


def test_pauli_strings_on_ghz(oracle):
    """(|0..0> + |1..1>)/sqrt(2): <X..X> = 1, <Z_i Z_j> = 1, <Z_i> = 0; for the Bell pair <YY> = -1;
    an X string with an even number of X replaced by Y picks up (-1)^(pairs)."""
    n = 4
    x = np.zeros((1, 16), dtype=np.float32)
    x[0, 0] = x[0, 15] = 1.0
    st, _ = oracle.amp_encode(x, n)
    assert abs(oracle.pauli_expect(st, xmask=0b1111)[0] - 1.0) < 1e-15
    assert abs(oracle.pauli_expect(st, zmask=0b0101)[0] - 1.0) < 1e-15
    assert abs(oracle.pauli_expect(st, zmask=0b0100)[0]) < 1e-15
    assert abs(oracle.pauli_expect(st, xmask=0b0011, ymask=0b1100)[0] + 1.0) < 1e-15
    assert abs(oracle.pauli_expect(st, ymask=0b1111)[0] - 1.0) < 1e-15
    assert abs(oracle.pauli_expect(st, xmask=0b0111)[0]) < 1e-15       # not all qubits flipped
    bell = np.zeros((1, 4), dtype=np.float32)
    bell[0, 0] = bell[0, 3] = 1.0
    sb, _ = oracle.amp_encode(bell, 2)
    assert abs(oracle.pauli_expect(sb, ymask=0b11)[0] + 1.0) < 1e-15


def test_pauli_strings_vs_dense_kronecker(oracle):
    g = rng(120)
    paulis = {"I": np.eye(2), "X": np.array([[0, 1], [1, 0]]), "Y": np.array([[0, -1j], [1j, 0]]),
              "Z": np.diag([1.0, -1.0])}
    for n in (1, 2, 3, 5):
        st = (g.standard_normal((3, 1 << n)) + 1j * g.standard_normal((3, 1 << n)))
        st /= np.linalg.norm(st, axis=1, keepdims=True)
        st = np.ascontiguousarray(st)
        for _ in range(12):
            letters = g.choice(list("IXYZ"), n)
            full = np.eye(1)
            for q in range(n):                                # qubit n-1 is the leftmost factor
                full = np.kron(paulis[letters[q]], full)
            masks = {c: sum(1 << q for q in range(n) if letters[q] == c) for c in "XYZ"}
            re, im = oracle.pauli_expect(st, masks["X"], masks["Y"], masks["Z"], with_imag=True)
            want = np.einsum("bi,ij,bj->b", st.conj(), full, st)
            assert np.allclose(re, want.real, atol=1e-13) and np.allclose(im, 0, atol=1e-13)
            assert np.allclose(want.imag, 0, atol=1e-13)
    # Z-only strings are parity sums of the probabilities, and single Z reproduces expz_all
    p = oracle.probs(st)
    k = np.arange(1 << n)
    par = lambda m: 1 - 2 * (np.array([bin(int(v) & m).count("1") for v in k]) & 1)
    assert np.allclose(oracle.pauli_expect(st, zmask=0b10110), (p * par(0b10110)).sum(1), atol=1e-13)
    z = oracle.expz_all(st)
    for q in range(n):
        assert np.allclose(oracle.pauli_expect(st, zmask=1 << q), z[:, q], atol=1e-13)
    with pytest.raises(ValueError):
        oracle.pauli_expect(st, xmask=1, zmask=1)


# ------------------------------------------------------------------ trash reset, finite shots
@pytest.mark.parametrize("n,mask,ent", [(3, 0b100, RING), (4, 0b1010, LADDER), (5, 0b11000, RING), (4, 0b0001, RING)])
def test_reset_fidelity_vs_density_matrix(oracle, n, mask, ent):
    """F = <a_in| D rho D^dagger |a_in> with rho = (partial trace over the trash qubits) (x) |0><0|,
    everything built densely with numpy."""
    g = rng(140 + n)
    L, rot = 2, (RY, RZ)
    circ = oracle.make_circuit(L, list(rot), ent)
    P = oracle.num_params(circ, n)
    params = g.uniform(0, 2 * np.pi, P)
    B = 3
    x = g.standard_normal((B, 1 << n)).astype(np.float32)
    st, _ = oracle.amp_encode(x, n)
    a_in = st.copy()
    oracle.apply_layers(st, circ, params)                       # encoder output
    F = oracle.reset_fidelity(st, circ, params, None, mask, x)
    U = dense.circuit_unitary(n, L, rot, ent, 0, params)
    D = U.conj().T
    k = np.arange(1 << n)
    keep = (k & mask) == 0
    for b in range(B):
        rho = np.zeros((1 << n, 1 << n), dtype=np.complex128)
        for t in sorted(set((k & mask).tolist())):
            v = np.zeros(1 << n, dtype=np.complex128)
            v[keep] = st[b][k[keep] | t]                         # psi_t with the trash moved to 0
            rho += np.outer(v, v.conj())
        assert abs(np.trace(rho).real - 1.0) < 1e-12
        want = (a_in[b].conj() @ D @ rho @ D.conj().T @ a_in[b]).real
        assert abs(F[b] - want) < 1e-12
    # never below the post-selected, unnormalised value (the t = 0 term alone)
    st0 = st.copy()
    oracle.project_zero(st0, mask, renormalise=False)
    oracle.apply_layers(st0, circ, params, inverse=True)
    assert np.all(F >= oracle.fidelity(st0, x) - 1e-14)


def test_reset_fidelity_is_one_when_trash_is_already_zero(oracle):
    """If the encoder already leaves the trash qubit in |0>, the reset changes nothing and the decoder
    returns the input: F = 1.  The input must be real (it is amplitude-encoded), so the circuit is
    RY-only with the ring, a real orthogonal matrix: the decoder applied to a real state with qubit 3
    in |0> is then a real input whose encoder output has that property."""
    n, mask = 4, 0b1000
    circ = oracle.make_circuit(2, [RY], RING)
    params = rng(150).uniform(0, 2 * np.pi, oracle.num_params(circ, n))
    v = rng(151).standard_normal((3, 8)).astype(np.float32)
    st, _ = oracle.amp_encode(v, n)                              # amplitudes 8..15 are zero
    oracle.apply_layers(st, circ, params, inverse=True)          # the input state a_in
    assert np.all(st.imag == 0.0)
    x = st.real.astype(np.float32)                               # float rounding: 1e-7 relative
    enc, _ = oracle.amp_encode(x, n)
    oracle.apply_layers(enc, circ, params)
    assert np.allclose(oracle.marginal(enc, mask)[:, 0], 1.0, atol=1e-6)
    F = oracle.reset_fidelity(enc, circ, params, None, mask, x)
    assert np.allclose(F, 1.0, atol=1e-6)
    # and with the trash qubit entangled the reset loses fidelity
    w, _ = oracle.amp_encode(rng(152).standard_normal((3, 16)).astype(np.float32), n)
    xw = w.real.astype(np.float32)
    oracle.apply_layers(w, circ, params)
    assert np.all(oracle.reset_fidelity(w, circ, params, None, mask, xw) < 0.999)


def test_shot_expz_closed_forms(oracle):
    s = np.array([[0, 0, 0, 0], [5, 5, 5, 5], [0, 7, -1, -1], [-1, -1, -1, -1]], dtype=np.int64)
    z = oracle.shot_expz(s, 3)
    assert np.array_equal(z[0], [1, 1, 1])
    assert np.array_equal(z[1], [-1, 1, -1])                     # 5 = 0b101
    assert np.array_equal(z[2], [0, 0, 0])                       # one shot each way, two skipped
    assert np.array_equal(z[3], [0, 0, 0])
    # many shots from a known distribution approach the exact expectation
    g = rng(152)
    p = g.random(16); p /= p.sum()
    smp = g.choice(16, size=(1, 200000), p=p)
    exact = np.array([(p * (1 - 2 * ((np.arange(16) >> q) & 1))).sum() for q in range(4)])
    assert np.abs(oracle.shot_expz(smp, 4)[0] - exact).max() < 5 / np.sqrt(200000)
