"""Dense 2^n x 2^n brute force for n <= 6, used only to pin the CPU oracle.

Independent of the oracle's amplitude loops: every gate is built as a full matrix with Kronecker
products (qubit 0 = least-significant index bit, so U_total = G_{n-1} (x) ... (x) G_0) or as an
explicit permutation matrix from integer bit operations, and the circuit is their product.
"""
import numpy as np

I2 = np.eye(2, dtype=np.complex128)


def rot_matrix(axis, theta):
    c, s = np.cos(theta / 2.0), np.sin(theta / 2.0)
    if axis == 1:
        return np.array([[c, -1j * s], [-1j * s, c]], dtype=np.complex128)
    if axis == 2:
        return np.array([[c, -s], [s, c]], dtype=np.complex128)
    if axis == 3:
        return np.array([[np.exp(-0.5j * theta), 0], [0, np.exp(0.5j * theta)]],
                        dtype=np.complex128)
    raise ValueError(axis)


def single(n, q, g):
    """g on qubit q: kron(I, ..., g, ..., I) with qubit n-1 leftmost."""
    m = np.array([[1.0 + 0j]])
    for j in range(n - 1, -1, -1):
        m = np.kron(m, g if j == q else I2)
    return m


def cnot(n, ctrl, tgt):
    N = 1 << n
    m = np.zeros((N, N), dtype=np.complex128)
    for k in range(N):
        k2 = k ^ (1 << tgt) if (k >> ctrl) & 1 else k
        m[k2, k] = 1.0
    return m


def cz(n, q0, q1):
    N = 1 << n
    d = np.ones(N, dtype=np.complex128)
    for k in range(N):
        if (k >> q0) & 1 and (k >> q1) & 1:
            d[k] = -1.0
    return np.diag(d)


def layer_unitary(n, rot, entangler, reupload, layer_params, feat):
    """layer_params: [slots][n] float64; feat: [n] or None.  Returns the 2^n x 2^n layer matrix."""
    N = 1 << n
    U = np.eye(N, dtype=np.complex128)
    slot = 0
    if reupload:
        for q in range(n):
            U = single(n, q, rot_matrix(1, layer_params[0][q] * feat[q])) @ U
        slot = 1
    for r, axis in enumerate(rot):
        for q in range(n):
            U = single(n, q, rot_matrix(axis, layer_params[slot + r][q])) @ U
    if entangler == 1 and n >= 2:
        for q in range(n):
            U = cnot(n, q, (q + 1) % n) @ U
    elif entangler == 2:
        for q in range(n - 1):
            U = cz(n, q, q + 1) @ U
    return U


def circuit_unitary(n, n_layers, rot, entangler, reupload, params, feat=None):
    slots = int(reupload) + len(rot)
    p = np.asarray(params, dtype=np.float64).reshape(n_layers, slots, n)
    U = np.eye(1 << n, dtype=np.complex128)
    for l in range(n_layers):
        U = layer_unitary(n, rot, entangler, reupload, p[l], feat) @ U
    return U
