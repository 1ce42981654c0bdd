"""ctypes loader and numpy-facing wrappers for the C++ oracle (test infrastructure only).

The circuit, measurement, sampling and gradient functions only marshal arguments: their numbers
come from ``qsv_oracle.cpp``.  Three small definitions are written here in numpy instead
(``shot_expz``, ``sgd_step``, ``adam_step``); each is pinned by closed forms in the CPU tests like
the C++ functions.  States are numpy complex128 arrays of shape [B, 2**n]; parameters and features
are converted to float64 exactly (they are float32 on the GPU side).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qsv_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")

RX, RY, RZ = 1, 2, 3
ENT_NONE, ENT_CNOT_RING, ENT_CZ_LADDER = 0, 1, 2


class Circuit(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("reupload", ctypes.c_int32),
                ("n_rot", ctypes.c_int32), ("rot", ctypes.c_int32 * 3),
                ("entangler", ctypes.c_int32)]


def make_circuit(n_layers, rot, entangler, reupload=0):
    c = Circuit()
    c.n_layers = n_layers
    c.reupload = int(reupload)
    c.n_rot = len(rot)
    for i, r in enumerate(rot):
        c.rot[i] = r
    c.entangler = entangler
    return c


def build(force=False):
    """Compile the oracle with g++ (OpenMP).  Rebuilds when the source is newer."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["g++", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c++17", _SRC, "-o", _LIB]
    subprocess.check_call(cmd)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.oracle_num_params.restype = ctypes.c_int64
        L.oracle_max_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def max_threads():
    return int(lib().oracle_max_threads())


def set_threads(t):
    lib().oracle_set_threads(ctypes.c_int(int(t)))


def num_params(circ, n):
    return int(lib().oracle_num_params(ctypes.byref(circ), ctypes.c_int(n)))


def _state(state):
    assert state.dtype == np.complex128 and state.flags.c_contiguous and state.ndim == 2
    B, N = state.shape
    n = int(N).bit_length() - 1
    assert (1 << n) == N
    return B, n


def amp_encode(x, n):
    x = np.ascontiguousarray(x, dtype=np.float32)
    B, dim = x.shape
    state = np.empty((B, 1 << n), dtype=np.complex128)
    norm = np.empty(B, dtype=np.float64)
    rc = lib().oracle_amp_encode(_p(x), ctypes.c_int64(B), ctypes.c_int64(dim), ctypes.c_int(n),
                                 _p(state), _p(norm))
    if rc:
        raise ValueError("oracle_amp_encode rc=%d" % rc)
    return state, norm


def zero_state(B, n):
    s = np.zeros((B, 1 << n), dtype=np.complex128)
    s[:, 0] = 1.0
    return s


def gate_rot(state, axis, q, theta):
    B, n = _state(state)
    rc = lib().oracle_gate_rot(_p(state), ctypes.c_int64(B), ctypes.c_int(n), ctypes.c_int(axis),
                               ctypes.c_int(q), ctypes.c_double(theta))
    if rc:
        raise ValueError("oracle_gate_rot rc=%d" % rc)


def gate_cnot(state, ctrl, tgt):
    B, n = _state(state)
    rc = lib().oracle_gate_cnot(_p(state), ctypes.c_int64(B), ctypes.c_int(n), ctypes.c_int(ctrl),
                                ctypes.c_int(tgt))
    if rc:
        raise ValueError("oracle_gate_cnot rc=%d" % rc)


def gate_cz(state, q0, q1):
    B, n = _state(state)
    rc = lib().oracle_gate_cz(_p(state), ctypes.c_int64(B), ctypes.c_int(n), ctypes.c_int(q0),
                              ctypes.c_int(q1))
    if rc:
        raise ValueError("oracle_gate_cz rc=%d" % rc)


MODE_AUTO, MODE_PER_SAMPLE, MODE_PER_PAIR = 0, 1, 2


def apply_layers(state, circ, params, feats=None, inverse=False, mode=MODE_AUTO):
    """mode only chooses how the work is spread over threads (one thread per sample, or every
    gate's pair loop split across threads; auto = the latter from 18 qubits on)."""
    B, n = _state(state)
    params = np.ascontiguousarray(params, dtype=np.float64).ravel()
    assert params.size == num_params(circ, n), (params.size, num_params(circ, n))
    f = None
    if feats is not None:
        f = np.ascontiguousarray(feats, dtype=np.float64)
        assert f.shape == (B, n)
    rc = lib().oracle_apply_layers_mode(_p(state), ctypes.c_int64(B), ctypes.c_int(n),
                                        ctypes.byref(circ), _p(params),
                                        _p(f) if f is not None else None, ctypes.c_int(int(inverse)),
                                        ctypes.c_int(int(mode)))
    if rc:
        raise ValueError("oracle_apply_layers rc=%d" % rc)


def probs(state):
    B, n = _state(state)
    p = np.empty((B, 1 << n), dtype=np.float64)
    lib().oracle_probs(_p(state), ctypes.c_int64(B), ctypes.c_int(n), _p(p))
    return p


def expz_all(state):
    B, n = _state(state)
    z = np.empty((B, n), dtype=np.float64)
    lib().oracle_expz_all(_p(state), ctypes.c_int64(B), ctypes.c_int(n), _p(z))
    return z


def marginal(state, mask):
    B, n = _state(state)
    m = bin(mask).count("1")
    out = np.empty((B, 1 << m), dtype=np.float64)
    rc = lib().oracle_marginal(_p(state), ctypes.c_int64(B), ctypes.c_int(n),
                               ctypes.c_uint64(mask), _p(out))
    if rc:
        raise ValueError("oracle_marginal rc=%d" % rc)
    return out


def project_zero(state, mask, renormalise=True):
    B, n = _state(state)
    p0 = np.empty(B, dtype=np.float64)
    rc = lib().oracle_project_zero(_p(state), ctypes.c_int64(B), ctypes.c_int(n),
                                   ctypes.c_uint64(mask), ctypes.c_int(int(renormalise)), _p(p0))
    if rc:
        raise ValueError("oracle_project_zero rc=%d" % rc)
    return p0


def fidelity(state, x):
    B, n = _state(state)
    x = np.ascontiguousarray(x, dtype=np.float32)
    assert x.shape[0] == B
    F = np.empty(B, dtype=np.float64)
    rc = lib().oracle_fidelity(_p(state), ctypes.c_int64(B), ctypes.c_int(n), _p(x),
                               ctypes.c_int64(x.shape[1]), _p(F))
    if rc:
        raise ValueError("oracle_fidelity rc=%d" % rc)
    return F


def reset_fidelity(state, circ, params, feats, mask, x):
    """Fidelity with the input after a true reset of the trash qubits and the decoder (circ inverse)."""
    B, n = _state(state)
    params = np.ascontiguousarray(params, dtype=np.float64).ravel()
    assert params.size == num_params(circ, n)
    f = None
    if feats is not None:
        f = np.ascontiguousarray(feats, dtype=np.float64)
        assert f.shape == (B, n)
    x = np.ascontiguousarray(x, dtype=np.float32)
    assert x.shape[0] == B
    F = np.empty(B, dtype=np.float64)
    rc = lib().oracle_reset_fidelity(_p(state), ctypes.c_int64(B), ctypes.c_int(n), ctypes.byref(circ),
                                     _p(params), _p(f) if f is not None else None, ctypes.c_uint64(mask),
                                     _p(x), ctypes.c_int64(x.shape[1]), _p(F))
    if rc:
        raise ValueError("oracle_reset_fidelity rc=%d" % rc)
    return F


def shot_expz(samples, n):
    """Finite-shot estimate of <Z_q> from basis-state samples [B, shots] (entries -1 are skipped):
    the mean of (1 - 2 bit_q) over the valid shots; a row without valid shots gives 0."""
    s = np.asarray(samples, dtype=np.int64)
    out = np.zeros((s.shape[0], n), dtype=np.float64)
    for b in range(s.shape[0]):
        v = s[b][s[b] >= 0]
        if v.size:
            for q in range(n):
                out[b, q] = np.mean(1.0 - 2.0 * ((v >> q) & 1))
    return out


def pauli_expect(state, xmask=0, ymask=0, zmask=0, with_imag=False):
    """<P> for the Pauli string with X on xmask, Y on ymask, Z on zmask (bit q = qubit q)."""
    B, n = _state(state)
    re = np.empty(B, dtype=np.float64)
    im = np.empty(B, dtype=np.float64)
    rc = lib().oracle_pauli_expect(_p(state), ctypes.c_int64(B), ctypes.c_int(n), ctypes.c_uint64(xmask),
                                   ctypes.c_uint64(ymask), ctypes.c_uint64(zmask), _p(re), _p(im))
    if rc:
        raise ValueError("oracle_pauli_expect rc=%d" % rc)
    return (re, im) if with_imag else re


def sample(p32, uniforms):
    """p32: float32 [B, 2**n]; uniforms: float64 [B, shots] in [0,1).  Returns int64 [B, shots]."""
    p32 = np.ascontiguousarray(p32, dtype=np.float32)
    B, N = p32.shape
    n = int(N).bit_length() - 1
    u = np.ascontiguousarray(uniforms, dtype=np.float64).reshape(B, -1)
    out = np.empty(u.shape, dtype=np.int64)
    lib().oracle_sample(_p(p32), ctypes.c_int64(B), ctypes.c_int(n), _p(u),
                        ctypes.c_int64(u.shape[1]), _p(out))
    return out


def param_shift_grad(x, n, circ, params, feats=None, obs_qubit=0, subset=None):
    x = np.ascontiguousarray(x, dtype=np.float32)
    B, dim = x.shape
    params = np.ascontiguousarray(params, dtype=np.float64).ravel()
    P = num_params(circ, n)
    assert params.size == P
    f = None
    if feats is not None:
        f = np.ascontiguousarray(feats, dtype=np.float64)
        assert f.shape == (B, n)
    sub = None
    nl = P
    if subset is not None:
        sub = np.ascontiguousarray(subset, dtype=np.int64)
        nl = sub.size
    loss = np.empty(B, dtype=np.float64)
    grad = np.empty((B, nl), dtype=np.float64)
    rc = lib().oracle_param_shift_grad(
        _p(x), ctypes.c_int64(B), ctypes.c_int64(dim), ctypes.c_int(n), ctypes.byref(circ),
        _p(params), _p(f) if f is not None else None, ctypes.c_int(obs_qubit),
        _p(sub) if sub is not None else None, ctypes.c_int64(nl), _p(loss), _p(grad))
    if rc:
        raise ValueError("oracle_param_shift_grad rc=%d" % rc)
    return loss, grad


LOSS_TRASH, LOSS_MSE_Z = 1, 2


def loss_grad(x, n, circ, params, feats=None, kind=LOSS_TRASH, mask=0, targets=None, subset=None):
    """Per-sample training loss and its gradient by the shift rule (see oracle_loss_grad)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    B, dim = x.shape
    params = np.ascontiguousarray(params, dtype=np.float64).ravel()
    P = num_params(circ, n)
    assert params.size == P
    f = None
    if feats is not None:
        f = np.ascontiguousarray(feats, dtype=np.float64)
        assert f.shape == (B, n)
    y = None
    if targets is not None:
        y = np.ascontiguousarray(targets, dtype=np.float64)
        assert y.shape == (B, n)
    sub, nl = None, P
    if subset is not None:
        sub = np.ascontiguousarray(subset, dtype=np.int64)
        nl = sub.size
    loss = np.empty(B, dtype=np.float64)
    grad = np.empty((B, nl), dtype=np.float64)
    rc = lib().oracle_loss_grad(
        _p(x), ctypes.c_int64(B), ctypes.c_int64(dim), ctypes.c_int(n), ctypes.byref(circ),
        _p(params), _p(f) if f is not None else None, ctypes.c_int(kind), ctypes.c_uint64(mask),
        _p(y) if y is not None else None, _p(sub) if sub is not None else None, ctypes.c_int64(nl),
        _p(loss), _p(grad))
    if rc:
        raise ValueError("oracle_loss_grad rc=%d" % rc)
    return loss, grad


def sgd_step(params, grad, lr):
    """theta <- theta - lr * g, in double, stored as float32 (the optimiser the training step uses)."""
    p = np.asarray(params, dtype=np.float64) - float(lr) * np.asarray(grad, dtype=np.float64)
    return p.astype(np.float32)


def adam_step(params, grad, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8):
    """One Adam update (Kingma & Ba, Algorithm 1) in double; returns float32 params, m, v.
    t is the 1-based step count."""
    g = np.asarray(grad, dtype=np.float64)
    m = beta1 * np.asarray(m, dtype=np.float64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, dtype=np.float64) + (1.0 - beta2) * g * g
    mh = m / (1.0 - beta1 ** t)
    vh = v / (1.0 - beta2 ** t)
    p = np.asarray(params, dtype=np.float64) - lr * mh / (np.sqrt(vh) + eps)
    return p.astype(np.float32), m.astype(np.float32), v.astype(np.float32)
