"""Seeded synthetic inputs for the five workload configs (and scaled-down variants of them).

This module holds no arithmetic of the method: it only draws random inputs with numpy's
``Generator(PCG64(seed))`` and describes each circuit as plain Python data.  Both the HIP path
and the CPU oracle are fed from here, byte-identical float32 arrays.

Recipe per config (task statement, workload configs 0-4):
  c0: n=4,  B=64,   x ~ N(0,1)^16 L2-normalised per row; 2 layers RY,RZ + CNOT ring; decoder = inverse
  c1: n=10, B=1024, x ~ N(0,1)^1024; 6 layers re-upload RX(w*x_i) + RY,RZ + CNOT ring; w ~ N(0,1)
  c2: n=16, B=256,  x ~ U(-1,1)^65536; 10 layers RY,RZ + CZ ladder; <Z_0> loss + full gradient
  c3: n=20, B=32,   x ~ N(0,1)^(2^20); 20 layers RY,RZ + CNOT ring; trash mask = 4 highest qubits
  c4: n=26, B=1,    x ~ N(0,1)^(2^26); 30 layers RX,RY,RZ + CNOT ring; 4096 uniforms for sampling
Rotation angles are U(0, 2*pi) throughout.
"""
from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np

RX, RY, RZ = 1, 2, 3
ENT_NONE, ENT_CNOT_RING, ENT_CZ_LADDER = 0, 1, 2


@dataclass
class CircuitSpec:
    n_layers: int
    rot: Tuple[int, ...]
    entangler: int
    reupload: int = 0

    def slots(self):
        return self.reupload + len(self.rot)

    def num_params(self, n):
        return self.n_layers * self.slots() * n

    def gates_per_layer(self, n):
        ent = 0
        if self.entangler == ENT_CNOT_RING and n >= 2:
            ent = n
        elif self.entangler == ENT_CZ_LADDER:
            ent = n - 1
        return self.slots() * n + ent


@dataclass
class Workload:
    name: str
    n: int
    batch: int
    dim: int
    circuit: CircuitSpec
    x: np.ndarray                      # float32 [batch, dim]
    params: np.ndarray                 # float32 [P]
    feats: Optional[np.ndarray] = None  # float32 [batch, n]
    trash_mask: int = 0
    obs_qubit: int = 0
    uniforms: Optional[np.ndarray] = None  # float64 [batch, shots]
    extra: dict = field(default_factory=dict)


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def draw_params(spec, n, seed):
    """Angles U(0, 2*pi); re-upload weights (slot 0 of each layer) N(0,1)."""
    rng = _rng(seed)
    slots = spec.slots()
    p = rng.uniform(0.0, 2.0 * np.pi, size=(spec.n_layers, slots, n))
    if spec.reupload:
        p[:, 0, :] = rng.standard_normal(size=(spec.n_layers, n))
    return p.astype(np.float32).ravel()


def draw_x(batch, dim, seed, dist="normal", l2_normalise=False):
    rng = _rng(seed)
    if dist == "normal":
        x = rng.standard_normal(size=(batch, dim), dtype=np.float32)
    elif dist == "uniform":
        x = (rng.random(size=(batch, dim), dtype=np.float32) * 2.0 - 1.0).astype(np.float32)
    else:
        raise ValueError(dist)
    if l2_normalise:
        x = (x / np.linalg.norm(x.astype(np.float64), axis=1, keepdims=True)).astype(np.float32)
    return np.ascontiguousarray(x, dtype=np.float32)


def config(idx, n=None, batch=None, n_layers=None, shots=None):
    """Workload config ``idx`` (0..4).  n / batch / n_layers / shots override the full sizes so
    that tests can run the same recipe at a size the oracle finishes in seconds."""
    if idx == 0:
        n = 4 if n is None else n
        batch = 64 if batch is None else batch
        spec = CircuitSpec(2 if n_layers is None else n_layers, (RY, RZ), ENT_CNOT_RING)
        x = draw_x(batch, 1 << n, 1000, "normal", l2_normalise=True)
        return Workload("c0", n, batch, 1 << n, spec, x, draw_params(spec, n, 2000))
    if idx == 1:
        n = 10 if n is None else n
        batch = 1024 if batch is None else batch
        spec = CircuitSpec(6 if n_layers is None else n_layers, (RY, RZ), ENT_CNOT_RING, 1)
        x = draw_x(batch, 1 << n, 1001, "normal")
        feats = np.ascontiguousarray(x[:, :n])
        return Workload("c1", n, batch, 1 << n, spec, x, draw_params(spec, n, 2001), feats=feats)
    if idx == 2:
        n = 16 if n is None else n
        batch = 256 if batch is None else batch
        spec = CircuitSpec(10 if n_layers is None else n_layers, (RY, RZ), ENT_CZ_LADDER)
        x = draw_x(batch, 1 << n, 1002, "uniform")
        return Workload("c2", n, batch, 1 << n, spec, x, draw_params(spec, n, 2002), obs_qubit=0)
    if idx == 3:
        n = 20 if n is None else n
        batch = 32 if batch is None else batch
        spec = CircuitSpec(20 if n_layers is None else n_layers, (RY, RZ), ENT_CNOT_RING)
        x = draw_x(batch, 1 << n, 1003, "normal")
        m = min(4, n - 1)
        mask = ((1 << m) - 1) << (n - m)
        return Workload("c3", n, batch, 1 << n, spec, x, draw_params(spec, n, 2003),
                        trash_mask=mask)
    if idx == 4:
        n = 26 if n is None else n
        batch = 1 if batch is None else batch
        spec = CircuitSpec(30 if n_layers is None else n_layers, (RX, RY, RZ), ENT_CNOT_RING)
        x = draw_x(batch, 1 << n, 1004, "normal")
        shots = 4096 if shots is None else shots
        u = _rng(3004).random(size=(batch, shots))
        return Workload("c4", n, batch, 1 << n, spec, x, draw_params(spec, n, 2004), uniforms=u)
    raise ValueError("config index must be 0..4")


def nominal_updates(spec, n, circuits):
    """Gate-amplitude updates as written in the circuit: every gate counts 2**n."""
    return circuits * spec.n_layers * spec.gates_per_layer(n) * (1 << n)
