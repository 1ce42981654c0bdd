"""Thin ctypes binding over libqsv.so with the C ABI's names.

Argument marshalling only: every step of the path runs in the HIP kernels.  torch is used for
device memory and the current stream; there is no CPU fallback, and a missing library is an
error, not a reason to compute elsewhere.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqsv.so")

QSV_OK, QSV_ERR_INVALID_ARG, QSV_ERR_UNSUPPORTED, QSV_ERR_ZERO_NORM, QSV_ERR_WORKSPACE, QSV_ERR_HIP = range(6)
QSV_RX, QSV_RY, QSV_RZ = 1, 2, 3
QSV_ENT_NONE, QSV_ENT_CNOT_RING, QSV_ENT_CZ_LADDER = 0, 1, 2
(QSV_M_PROBS, QSV_M_EXPZ_ALL, QSV_M_EXPZ_ONE, QSV_M_MARGINAL, QSV_M_PROJECT_ZERO, QSV_M_FIDELITY,
 QSV_M_SAMPLE) = range(1, 8)


class qsv_circuit(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("reupload", ctypes.c_int32),
                ("n_rot", ctypes.c_int32), ("rot", ctypes.c_int32 * 3),
                ("entangler", ctypes.c_int32)]


class qsv_measure_req(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("qubit", ctypes.c_int32), ("mask", ctypes.c_uint64),
                ("renormalise", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("x_dev", ctypes.c_void_p), ("dim", ctypes.c_int64),
                ("uniforms_dev", ctypes.c_void_p), ("shots", ctypes.c_int64),
                ("out_dev", ctypes.c_void_p)]


class qsv_loss(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("reserved", ctypes.c_int32), ("mask", ctypes.c_uint64),
                ("targets_dev", ctypes.c_void_p)]


QSV_LOSS_TRASH, QSV_LOSS_MSE_Z = 1, 2


class QsvError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("qsv status %d: %s" % (status, message))
        self.status = status


_lib = None


def load():
    """Loads libqsv.so (built in-tree by build.py).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s not found: build it with `python -m paper_2602_13140_amd.build` "
            "(there is no fallback path)" % LIB_PATH)
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    L.qsv_num_params.restype = i64
    L.qsv_num_params.argtypes = [ctypes.POINTER(qsv_circuit), i32]
    L.qsv_workspace_bytes.restype = ctypes.c_size_t
    L.qsv_workspace_bytes.argtypes = [i32, i32]
    L.qsv_grad_workspace_bytes.restype = ctypes.c_size_t
    L.qsv_grad_workspace_bytes.argtypes = [i32, i32, ctypes.POINTER(qsv_circuit)]
    L.qsv_create.restype = i32
    L.qsv_create.argtypes = [ctypes.POINTER(vp), i32, i32, i32, vp, vp, vp, ctypes.c_size_t]
    L.qsv_destroy.restype = None
    L.qsv_destroy.argtypes = [vp]
    L.qsv_last_error.restype = ctypes.c_char_p
    L.qsv_last_error.argtypes = [vp]
    L.qsv_amp_encode.restype = i32
    L.qsv_amp_encode.argtypes = [vp, vp, i64, vp]
    L.qsv_apply_layers.restype = i32
    L.qsv_apply_layers.argtypes = [vp, ctypes.POINTER(qsv_circuit), vp, vp, i32]
    L.qsv_measure.restype = i32
    L.qsv_measure.argtypes = [vp, ctypes.POINTER(qsv_measure_req)]
    L.qsv_forward_small.restype = i32
    L.qsv_forward_small.argtypes = [vp, vp, i64, ctypes.POINTER(qsv_circuit), vp, vp, i32, i32, vp, vp]
    L.qsv_measure_static.restype = i32
    L.qsv_measure_static.argtypes = [vp, ctypes.POINTER(qsv_measure_req)]
    L.qsv_param_shift_grad.restype = i32
    L.qsv_param_shift_grad.argtypes = [vp, ctypes.POINTER(qsv_circuit), vp, i64, vp, vp, ctypes.c_int32,
                                       vp, vp, vp, vp]
    L.qsv_adjoint_grad.restype = i32
    L.qsv_adjoint_grad.argtypes = [vp, ctypes.POINTER(qsv_circuit), vp, i64, vp, vp, ctypes.c_int32,
                                       vp, vp, vp, vp]
    L.qsv_loss_grad.restype = i32
    L.qsv_loss_grad.argtypes = [vp, ctypes.POINTER(qsv_circuit), vp, i64, vp, vp, ctypes.POINTER(qsv_loss),
                                vp, vp, vp, vp]
    L.qsv_sgd_step.restype = i32
    L.qsv_sgd_step.argtypes = [vp, vp, vp, i64, ctypes.c_double]
    L.qsv_adam_step.restype = i32
    L.qsv_adam_step.argtypes = [vp, vp, vp, vp, vp, i64, i64, ctypes.c_double, ctypes.c_double,
                                ctypes.c_double, ctypes.c_double]
    L.qsv_reset_fidelity.restype = i32
    L.qsv_reset_fidelity.argtypes = [vp, ctypes.POINTER(qsv_circuit), vp, vp, ctypes.c_uint64, vp, i64, vp]
    L.qsv_shot_expz.restype = i32
    L.qsv_shot_expz.argtypes = [vp, vp, i64, vp]
    L.qsv_pauli_expect.restype = i32
    L.qsv_pauli_expect.argtypes = [vp, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64, vp]
    L.qsv_plan_describe.restype = i64
    L.qsv_plan_describe.argtypes = [ctypes.POINTER(qsv_circuit), i32, i32, i32, i32, ctypes.c_char_p, i64]
    L.qsv_probe_pass.restype = i32
    L.qsv_probe_pass.argtypes = [vp, i32, i32, i32]
    L.qsv_set_option.restype = i32
    L.qsv_set_option.argtypes = [vp, ctypes.c_char_p, i64]
    _lib = L
    return L


def make_circuit(n_layers, rot, entangler, reupload=0):
    c = qsv_circuit()
    c.n_layers = int(n_layers)
    c.reupload = int(reupload)
    c.n_rot = len(rot)
    for i, r in enumerate(rot):
        c.rot[i] = int(r)
    c.entangler = int(entangler)
    return c


def circuit_from_spec(spec):
    """spec: workloads.CircuitSpec."""
    return make_circuit(spec.n_layers, spec.rot, spec.entangler, spec.reupload)


def qsv_num_params(circ, n):
    return int(load().qsv_num_params(ctypes.byref(circ), n))


def qsv_workspace_bytes(n, batch):
    return int(load().qsv_workspace_bytes(n, batch))


def qsv_grad_workspace_bytes(n, batch, circ):
    return int(load().qsv_grad_workspace_bytes(n, batch, ctypes.byref(circ)))


def qsv_plan_describe(circ, n, batch=1, inverse=0, tile_log2=0):
    L = load()
    need = L.qsv_plan_describe(ctypes.byref(circ), n, batch, inverse, tile_log2, None, 0)
    if need < 0:
        raise ValueError("bad circuit descriptor")
    buf = ctypes.create_string_buffer(need + 1)
    L.qsv_plan_describe(ctypes.byref(circ), n, batch, inverse, tile_log2, buf, need + 1)
    return buf.value.decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


class Context:
    """Owns a qsv_ctx plus the torch tensors that back its state and workspace."""

    def __init__(self, n, batch, device=0, ws_bytes=None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("qsv needs a GPU: torch.cuda.is_available() is False")
        self.L = load()
        self.n, self.batch = n, batch
        self.dev = torch.device("cuda", device)
        self.state = torch.zeros((batch, 1 << n, 2), dtype=torch.float32, device=self.dev)
        need = qsv_workspace_bytes(n, batch)
        ws_bytes = need if ws_bytes is None else ws_bytes
        self.ws = torch.empty(ws_bytes + 256, dtype=torch.uint8, device=self.dev)
        off = (-self.ws.data_ptr()) % 256
        self.stream = torch.cuda.current_stream(self.dev)
        h = ctypes.c_void_p()
        st = self.L.qsv_create(ctypes.byref(h), n, batch, device,
                               ctypes.c_void_p(self.stream.cuda_stream),
                               ctypes.c_void_p(self.state.data_ptr()),
                               ctypes.c_void_p(self.ws.data_ptr() + off), ws_bytes)
        if st != QSV_OK:
            raise QsvError(st, self.L.qsv_last_error(None).decode())
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.L.qsv_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st):
        if st != QSV_OK:
            raise QsvError(st, self.L.qsv_last_error(self.h).decode())

    def qsv_set_option(self, name, value):
        self._check(self.L.qsv_set_option(self.h, name.encode(), int(value)))

    def qsv_probe_pass(self, low_bits, window_start, transposes=0):
        self._check(self.L.qsv_probe_pass(self.h, low_bits, window_start, transposes))

    def qsv_amp_encode(self, x, norm_out=None):
        assert x.is_cuda and x.dtype.is_floating_point and x.is_contiguous() and x.shape[0] == self.batch
        self._check(self.L.qsv_amp_encode(self.h, _ptr(x), x.shape[1], _ptr(norm_out)))

    def qsv_apply_layers(self, circ, params, feats=None, inverse=0):
        self._check(self.L.qsv_apply_layers(self.h, ctypes.byref(circ), _ptr(params), _ptr(feats),
                                            int(inverse)))

    def qsv_forward_small(self, x, circ, params, feats, decode, kind, out, norm_out=None):
        assert x.is_cuda and x.is_contiguous() and x.shape[0] == self.batch and out.is_cuda and out.is_contiguous()
        self._check(self.L.qsv_forward_small(self.h, _ptr(x), x.shape[1], ctypes.byref(circ), _ptr(params),
                                             _ptr(feats), int(decode), int(kind), _ptr(out), _ptr(norm_out)))

    def qsv_measure_static(self, kind, out, **kw):
        self.qsv_measure(kind, out, entry=self.L.qsv_measure_static, **kw)

    def qsv_measure(self, kind, out, qubit=0, mask=0, renormalise=0, x=None, uniforms=None, entry=None):
        r = qsv_measure_req()
        r.kind, r.qubit, r.mask, r.renormalise, r.reserved = kind, qubit, mask, int(renormalise), 0
        r.x_dev = x.data_ptr() if x is not None else None
        r.dim = x.shape[1] if x is not None else 0
        r.uniforms_dev = uniforms.data_ptr() if uniforms is not None else None
        r.shots = uniforms.shape[1] if uniforms is not None else 0
        r.out_dev = out.data_ptr()
        self._check((entry or self.L.qsv_measure)(self.h, ctypes.byref(r)))

    def qsv_loss_grad(self, circ, x, params, feats, kind, loss, grad, mean_loss=None, mean_grad=None,
                      mask=0, targets=None):
        spec = qsv_loss(kind, 0, mask, None if targets is None else targets.data_ptr())
        self._check(self.L.qsv_loss_grad(self.h, ctypes.byref(circ), _ptr(x), x.shape[1], _ptr(params),
                                         _ptr(feats), ctypes.byref(spec), _ptr(loss), _ptr(grad),
                                         _ptr(mean_loss), _ptr(mean_grad)))

    def qsv_reset_fidelity(self, circ, params, feats, mask, x, out):
        self._check(self.L.qsv_reset_fidelity(self.h, ctypes.byref(circ), _ptr(params), _ptr(feats), mask,
                                              _ptr(x), x.shape[1], _ptr(out)))

    def qsv_shot_expz(self, samples, out):
        self._check(self.L.qsv_shot_expz(self.h, _ptr(samples), samples.shape[1], _ptr(out)))

    def qsv_pauli_expect(self, out, xmask=0, ymask=0, zmask=0):
        self._check(self.L.qsv_pauli_expect(self.h, xmask, ymask, zmask, _ptr(out)))

    def qsv_sgd_step(self, params, grad, lr):
        self._check(self.L.qsv_sgd_step(self.h, _ptr(params), _ptr(grad), params.numel(), lr))

    def qsv_adam_step(self, params, grad, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8):
        self._check(self.L.qsv_adam_step(self.h, _ptr(params), _ptr(grad), _ptr(m), _ptr(v), params.numel(),
                                         t, lr, beta1, beta2, eps))

    def qsv_adjoint_grad(self, circ, x, params, feats, obs_qubit, loss, grad, mean_loss=None,
                         mean_grad=None):
        self._check(self.L.qsv_adjoint_grad(self.h, ctypes.byref(circ), _ptr(x), x.shape[1],
                                            _ptr(params), _ptr(feats), obs_qubit, _ptr(loss),
                                            _ptr(grad), _ptr(mean_loss), _ptr(mean_grad)))

    def qsv_param_shift_grad(self, circ, x, params, feats, obs_qubit, loss, grad, mean_loss=None,
                             mean_grad=None):
        self._check(self.L.qsv_param_shift_grad(self.h, ctypes.byref(circ), _ptr(x), x.shape[1],
                                                _ptr(params), _ptr(feats), obs_qubit, _ptr(loss),
                                                _ptr(grad), _ptr(mean_loss), _ptr(mean_grad)))
