#!/usr/bin/env python3
"""Benchmark of the qsv hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of the headline workload (config 4:
26 qubits, batch 1: amplitude encoding, 30 layers RX/RY/RZ + CNOT ring, the full 2^26
probability vector, 4096 seeded samples), inputs resident in HBM.  `value` is nominal
gate-amplitude updates per second (every gate of the circuit as written counts 2^n) over the
whole step.  The other configs are timed too and reported under "others".

Prints ONE JSON line.  `roofline` is for the dominant kernel (the fused gate pass): algorithmic
bytes per launch = one read + one write of the state, divided by the pass kernel's average
duration measured with events on the stream the kernels run on.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes per pass (config 3: a pair of launches) from rocprofv3 FETCH_SIZE / WRITE_SIZE, each scaled by what the same
# counter reads for the load/store-only probe pass of known size (FETCH_SIZE x 2.000, WRITE_SIZE x
# 1.000); the runs and their figures are in profiles/k_pass_hbm_traffic_counters.md.
TRAFFIC_BYTES_PER_LAUNCH = {"c4": 1073974797, "c3": 537444482}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--configs", default="4,3,2,1,0", help="which configs to time (4 is the headline)")
    ap.add_argument("--tile", type=int, default=0, help="force the pass kernel's tile_log2 (0 = default)")
    ap.add_argument("--defer", type=int, default=-1,
                    help="qsv_apply_layers defers CNOTs whose target lies outside a pass's tile (1), keeps every CNOT in "
                         "registers (0), or decides itself (-1, the default: it defers when it can)")
    ap.add_argument("--prio", type=int, default=-1, help="load_store_priority option of the pass kernel (0 or 1)")
    ap.add_argument("--low", type=int, default=0, help="force the planner's minimum number of low index bits per tile")
    ap.add_argument("--planes", type=int, default=0, help="force the pass kernel's LDS planes (1 or 2; 0 = default)")
    ap.add_argument("--nt", type=int, default=-1, help="force nontemporal tile stores (1) or ordinary ones (0)")
    ap.add_argument("--probe", action="store_true",
                    help="only time the load/store-only probe pass on config 4's state (streaming ceiling "
                         "of the pass kernel's access pattern; also the known-size copy used to scale "
                         "rocprofv3's FETCH_SIZE/WRITE_SIZE counters)")
    ap.add_argument("--rev", type=int, default=-1, help="every other pass takes its tiles in descending order (1) or not (0)")
    ap.add_argument("--probe-transposes", type=int, default=0,
                    help="probe pass: moves of the register run through LDS between the tile's load and its store")
    ap.add_argument("--probe-layout", type=int, default=-1,
                    help="probe pass: start of the register run the tile is loaded and stored in (-1 = highest)")
    ap.add_argument("--c3-batch", type=int, default=0,
                    help="with --configs 3 alone: run config 3's circuit at this batch instead of 32 (128 = 1 GiB of "
                         "state, beyond the memory-side cache)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-classic", action="store_true", help="skip the extra run of config 4 without deferred CNOTs")
    ap.add_argument("--cpu-layers", type=int, default=20, help="layers of config 4 the oracle is timed on")
    return ap.parse_args()


def n_passes(qb, circ, n, batch, inverse, tile, defer=False):
    text = qb.qsv_plan_describe(circ, n, batch, inverse, tile | (0x100 if defer else 0))
    return sum(1 for ln in text.split("\n") if ln.startswith("P "))


class Timer:
    """Event pairs on torch's current stream (the stream the library launches on)."""

    def __init__(self, torch):
        self.torch = torch
        self.pairs = {}

    def span(self, name):
        t = self.torch
        a, b = t.cuda.Event(enable_timing=True), t.cuda.Event(enable_timing=True)
        self.pairs.setdefault(name, []).append((a, b))
        return a, b

    def total_ms(self, name):
        return sum(a.elapsed_time(b) for a, b in self.pairs.get(name, []))


def run_steps(torch, step, steps, warmup):
    for _ in range(warmup):
        step(None)
    torch.cuda.synchronize()
    tm = Timer(torch)
    t0 = time.perf_counter()
    for _ in range(steps):
        step(tm)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps, tm


def graph_replay_ms(torch, build, steps):
    """One step captured into a HIP graph on a stream of its own (after two eager steps, which upload
    the plans), then replayed `steps` times: what a launch-bound small configuration costs when the
    host issues one graph launch per step instead of one launch per kernel."""
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ctx, step = build()                      # the context binds the side stream
        step(None)
        step(None)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step(None)
        for _ in range(3):
            graph.replay()
        side.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        side.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        ctx.close()
    return ms


def bench_c4(torch, qb, wl, args, apply_only=False):
    w = wl.config(4)
    n = w.n
    ctx = qb.Context(n, 1)
    if args.tile:
        ctx.qsv_set_option("tile_log2", args.tile)
    if args.defer >= 0:
        ctx.qsv_set_option("defer_cnots", args.defer)
    if args.prio >= 0:
        ctx.qsv_set_option("load_store_priority", args.prio)
    if args.low:
        ctx.qsv_set_option("low_bits", args.low)
    if args.planes:
        ctx.qsv_set_option("lds_planes", args.planes)
    if args.nt >= 0:
        ctx.qsv_set_option("nt_store", args.nt)
    if args.rev >= 0:
        ctx.qsv_set_option("reverse_passes", args.rev)
    circ = qb.circuit_from_spec(w.circuit)
    xd = torch.from_numpy(w.x).cuda()
    pd = torch.from_numpy(w.params).cuda()
    ud = torch.from_numpy(w.uniforms).cuda()
    probs = torch.empty((1, 1 << n), dtype=torch.float32, device="cuda")
    shots = torch.empty(w.uniforms.shape, dtype=torch.int64, device="cuda")

    def step(tm):
        ctx.qsv_amp_encode(xd)
        if tm:
            a, b = tm.span("apply")
            a.record()
        ctx.qsv_apply_layers(circ, pd, None, 0)
        if tm:
            b.record()
        ctx.qsv_measure(qb.QSV_M_PROBS, probs)
        ctx.qsv_measure(qb.QSV_M_SAMPLE, shots, uniforms=ud)

    ms, tm = run_steps(torch, step, args.steps, args.warmup)
    passes = n_passes(qb, circ, n, 1, 0, args.tile, args.defer != 0)
    apply_ms = tm.total_ms("apply") / args.steps
    updates = wl.nominal_updates(w.circuit, n, 1)
    state_bytes = 8 * (1 << n)
    res = {
        "workload": "c4: 26 qubits, batch 1, 30 layers RX/RY/RZ + CNOT ring, probs + 4096 samples",
        "ms_per_step": ms, "apply_ms": apply_ms, "passes": passes, "updates": updates,
        "updates_per_s": updates / (ms * 1e-3), "apply_updates_per_s": updates / (apply_ms * 1e-3),
        "pass_avg_ms": apply_ms / passes, "pass_bytes": 2 * state_bytes,
        "pass_gbs": 2 * state_bytes / (apply_ms / passes * 1e-3) / 1e9,
        "unitary_flops": 13.0 * w.circuit.n_layers * n * (1 << n),
    }
    if apply_only:
        ctx.close()
        return res, w
    # a Pauli-string expectation on the final state: one read pass (8 bytes per amplitude)
    ev = torch.empty(1, dtype=torch.float32, device="cuda")
    xm, ym, zm = 0x0092492, 0x1124924, 0x2249249          # X, Y, Z on every third qubit each

    def pauli(tm):
        ctx.qsv_pauli_expect(ev, xm, ym, zm)

    pms, _ = run_steps(torch, pauli, max(args.steps, 5), 1)
    res["pauli_string"] = {"ms": pms, "gbs": state_bytes / (pms * 1e-3) / 1e9,
                           "what": "<P> of a 26-qubit mixed X/Y/Z string on the final state, 8 B per amplitude"}
    ctx.close()
    return res, w


def bench_c3(torch, qb, wl, args, batch=None):
    """batch = None: config 3 as given (32 samples, 256 MiB of state: as large as the chip's memory-side
    cache, so part of every pass is served from it).  A larger batch is the same circuit on a state the
    cache cannot hold (supplementary: shows the pass kernel's rate against HBM alone)."""
    w = wl.config(3) if batch is None else wl.config(3, batch=batch)
    n, B = w.n, w.batch
    ctx = qb.Context(n, B)
    if args.tile:
        ctx.qsv_set_option("tile_log2", args.tile)
    if args.defer >= 0:
        ctx.qsv_set_option("defer_cnots", args.defer)
    if args.prio >= 0:
        ctx.qsv_set_option("load_store_priority", args.prio)
    if args.low:
        ctx.qsv_set_option("low_bits", args.low)
    if args.planes:
        ctx.qsv_set_option("lds_planes", args.planes)
    if args.nt >= 0:
        ctx.qsv_set_option("nt_store", args.nt)
    if args.rev >= 0:
        ctx.qsv_set_option("reverse_passes", args.rev)
    circ = qb.circuit_from_spec(w.circuit)
    xd = torch.from_numpy(w.x).cuda()
    pd = torch.from_numpy(w.params).cuda()
    p0 = torch.empty(B, dtype=torch.float32, device="cuda")
    marg = torch.empty((B, 16), dtype=torch.float32, device="cuda")
    fid = torch.empty(B, dtype=torch.float32, device="cuda")

    def step(tm):
        ctx.qsv_amp_encode(xd)
        if tm:
            a, b = tm.span("apply")
            a.record()
        ctx.qsv_apply_layers(circ, pd, None, 0)
        if tm:
            b.record()
        ctx.qsv_measure(qb.QSV_M_MARGINAL, marg, mask=w.trash_mask)
        ctx.qsv_measure(qb.QSV_M_PROJECT_ZERO, p0, mask=w.trash_mask, renormalise=1)
        if tm:
            a, b = tm.span("apply")
            a.record()
        ctx.qsv_apply_layers(circ, pd, None, 1)
        if tm:
            b.record()
        ctx.qsv_measure(qb.QSV_M_FIDELITY, fid, x=xd)

    ms, tm = run_steps(torch, step, args.steps, args.warmup)
    passes = n_passes(qb, circ, n, B, 0, args.tile, args.defer != 0) + n_passes(qb, circ, n, B, 1, args.tile, args.defer != 0)
    apply_ms = tm.total_ms("apply") / args.steps
    updates = 2 * wl.nominal_updates(w.circuit, n, B)
    state_bytes = 8 * B * (1 << n)
    extra = {}
    if batch is None:
        # the same autoencoder with a true reset of the trash qubits: 16 decoder runs per sample
        ctx.qsv_amp_encode(xd)
        ctx.qsv_apply_layers(circ, pd, None, 0)

        def reset_step(tm):
            ctx.qsv_reset_fidelity(circ, pd, None, w.trash_mask, xd, fid)

        reset_ms, _ = run_steps(torch, reset_step, 3, 1)
        reset_updates = 16 * wl.nominal_updates(w.circuit, n, B)
        extra["true_reset"] = {"what": "qsv_reset_fidelity: sum over the 16 trash outcomes, 16 decoder runs per sample",
                               "ms": reset_ms, "updates": reset_updates,
                               "updates_per_s": reset_updates / (reset_ms * 1e-3)}
    else:
        extra["note"] = ("supplementary, not one of the five configs: config 3's circuit at batch %d, %d MiB of "
                         "state, which the 256 MiB memory-side cache cannot hold" % (B, state_bytes >> 20))
    ctx.close()
    return dict(extra, **{
        "workload": "c3: 20 qubits, batch %d, 20-layer encoder + trash projection + decoder + fidelity" % B,
        "ms_per_step": ms, "apply_ms": apply_ms, "passes": passes, "updates": updates,
        "updates_per_s": updates / (ms * 1e-3), "apply_updates_per_s": updates / (apply_ms * 1e-3),
        # states of two rows or more go through a pass as two launches (halves of the rows) side by
        # side on two streams: the per-pass figures below are for the pair
        "launches_per_pass": 2 if B >= 2 else 1,
        "pass_avg_ms": apply_ms / passes, "pass_bytes": 2 * state_bytes,
        "pass_gbs": 2 * state_bytes / (apply_ms / passes * 1e-3) / 1e9,
        "pass_hbm_frac": 2 * state_bytes / (apply_ms / passes * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "state_mib": state_bytes >> 20,
        "memory_side_cache": "state <= 256 MiB: passes are partly served by the memory-side cache, the figure is "
                             "bandwidth between L2 and the fabric, not HBM alone" if state_bytes <= (256 << 20)
                             else "state larger than the 256 MiB memory-side cache: HBM bandwidth",
    })


def bench_c2(torch, qb, wl, args):
    """Config 2: the full parameter-shift gradient, timed twice: layer by layer from kept states
    (the default when the workspace has room for them) and with every shifted circuit run whole."""
    w = wl.config(2)
    n, B = w.n, w.batch
    P = w.circuit.num_params(n)
    circ = qb.circuit_from_spec(w.circuit)
    ctx = qb.Context(n, B, ws_bytes=qb.qsv_grad_workspace_bytes(n, B, circ))
    if args.tile:
        ctx.qsv_set_option("tile_log2", args.tile)
    if args.defer >= 0:
        ctx.qsv_set_option("defer_cnots", args.defer)
    if args.prio >= 0:
        ctx.qsv_set_option("load_store_priority", args.prio)
    if args.low:
        ctx.qsv_set_option("low_bits", args.low)
    if args.planes:
        ctx.qsv_set_option("lds_planes", args.planes)
    if args.nt >= 0:
        ctx.qsv_set_option("nt_store", args.nt)
    if args.rev >= 0:
        ctx.qsv_set_option("reverse_passes", args.rev)
    xd = torch.from_numpy(w.x).cuda()
    pd = torch.from_numpy(w.params).cuda()
    loss = torch.empty(B, dtype=torch.float32, device="cuda")
    grad = torch.empty((B, P), dtype=torch.float32, device="cuda")
    mg = torch.empty(P, dtype=torch.float32, device="cuda")

    def step(tm):
        ctx.qsv_param_shift_grad(circ, xd, pd, None, 0, loss, grad, None, mg)

    steps = max(1, min(args.steps, 3))
    circuits = B * (2 * P + 1)
    updates = wl.nominal_updates(w.circuit, n, circuits)
    L = w.circuit.n_layers
    layer_updates = wl.nominal_updates(w.circuit, n, 1) // L      # gate-amplitude updates of one layer
    per_layer = 2 * P // L                                         # shifted circuits per sample and layer
    executed = B * layer_updates * (L + sum(per_layer * (L - l) for l in range(L)))
    ms, _ = run_steps(torch, step, steps, 1)
    ctx.qsv_set_option("grad_layered", 0)
    ms_whole, _ = run_steps(torch, step, steps, 1)

    def step_adj(tm):
        ctx.qsv_adjoint_grad(circ, xd, pd, None, 0, loss, grad, None, mg)

    ms_adj, _ = run_steps(torch, step_adj, max(steps, 5), 1)
    ctx.close()

    # The other reading of "about 480 parameters": three rotations (RX, RY, RZ) per qubit and layer.
    spec3 = wl.CircuitSpec(L, (wl.RX, wl.RY, wl.RZ), w.circuit.entangler)
    P3 = spec3.num_params(n)
    circ3 = qb.circuit_from_spec(spec3)
    ctx3 = qb.Context(n, B, ws_bytes=qb.qsv_grad_workspace_bytes(n, B, circ3))
    p3d = torch.from_numpy(wl.draw_params(spec3, n, 2002)).cuda()
    grad3 = torch.empty((B, P3), dtype=torch.float32, device="cuda")
    mg3 = torch.empty(P3, dtype=torch.float32, device="cuda")
    ms3, _ = run_steps(torch, lambda tm: ctx3.qsv_param_shift_grad(circ3, xd, p3d, None, 0, loss, grad3, None, mg3),
                       1, 1)
    ms3_adj, _ = run_steps(torch, lambda tm: ctx3.qsv_adjoint_grad(circ3, xd, p3d, None, 0, loss, grad3, None, mg3),
                           max(steps, 5), 1)
    ctx3.close()
    updates3 = wl.nominal_updates(spec3, n, B * (2 * P3 + 1))
    return {"workload": "c2: 16 qubits, batch 256, 10 layers RY,RZ + CZ ladder, full parameter-shift gradient",
            "method": "layer by layer from kept states: a circuit that shifts a parameter of layer l runs layers l..L-1",
            "ms_per_step": ms, "steps": steps, "circuits": circuits, "params": P, "updates": updates,
            "updates_per_s": updates / (ms * 1e-3),
            "executed_updates": executed, "executed_updates_per_s": executed / (ms * 1e-3),
            "whole_circuits": {"ms_per_step": ms_whole, "executed_updates": updates,
                               "executed_updates_per_s": updates / (ms_whole * 1e-3)},
            "adjoint": {"method": "qsv_adjoint_grad: same loss and gradient in reverse mode (one forward run, "
                                  "psi and lambda taken back layer by layer, 2x2 transition sums per qubit)",
                        "ms_per_step": ms_adj, "speedup_over_shift_rule": ms / ms_adj},
            "three_rotations": {"workload": "same with RX,RY,RZ per layer: 480 parameters", "params": P3,
                                "circuits": B * (2 * P3 + 1), "updates": updates3, "ms_per_step": ms3,
                                "updates_per_s": updates3 / (ms3 * 1e-3), "adjoint_ms_per_step": ms3_adj}}


def bench_c1(torch, qb, wl, args):
    w = wl.config(1)
    n, B = w.n, w.batch
    circ = qb.circuit_from_spec(w.circuit)
    xd, pd, fd = (torch.from_numpy(a).cuda() for a in (w.x, w.params, w.feats))
    z = torch.empty((B, n), dtype=torch.float32, device="cuda")

    def build():
        ctx = qb.Context(n, B)
        if args.tile:
            ctx.qsv_set_option("tile_log2", args.tile)
        if args.defer >= 0:
            ctx.qsv_set_option("defer_cnots", args.defer)
        if args.prio >= 0:
            ctx.qsv_set_option("load_store_priority", args.prio)
        if args.planes:
            ctx.qsv_set_option("lds_planes", args.planes)

        def step(tm):
            ctx.qsv_amp_encode(xd)
            ctx.qsv_apply_layers(circ, pd, fd, 0)
            ctx.qsv_measure(qb.QSV_M_EXPZ_ALL, z)
        return ctx, step

    ctx, step = build()
    ms, _ = run_steps(torch, step, args.steps, args.warmup)
    updates = wl.nominal_updates(w.circuit, n, B)
    fms, _ = run_steps(torch, lambda tm: ctx.qsv_forward_small(xd, circ, pd, fd, 0, qb.QSV_M_EXPZ_ALL, z),
                       max(args.steps, 50), args.warmup)
    ctx.close()
    gms = graph_replay_ms(torch, build, max(args.steps, 50))
    return {"workload": "c1: 10 qubits, batch 1024, 6 re-uploading layers, <Z_q> for every qubit",
            "ms_per_step": ms, "updates": updates, "updates_per_s": updates / (ms * 1e-3),
            "one_launch_ms_per_step": fms, "one_launch_updates_per_s": updates / (fms * 1e-3),
            "graph_replay_ms_per_step": gms, "graph_replay_updates_per_s": updates / (gms * 1e-3),
            "what": "ms_per_step: qsv_amp_encode + qsv_apply_layers + qsv_measure; one_launch: qsv_forward_small; "
                    "graph_replay: the separate calls captured into one HIP graph"}


def bench_train(torch, qb, wl, args, idx):
    """A training step on config 3 (loss 1 - P0 on the trash qubits after the encoder) or config 1
    (mean squared error of <Z_q> against seeded targets): loss and gradient of every sample for
    every parameter in reverse mode, batch means, one Adam step, all on the device."""
    import numpy as np
    w = wl.config(idx)
    n, B = w.n, w.batch
    circ = qb.circuit_from_spec(w.circuit)
    P = w.circuit.num_params(n)
    ctx = qb.Context(n, B, ws_bytes=qb.qsv_grad_workspace_bytes(n, B, circ))
    xd = torch.from_numpy(w.x).cuda()
    pd = torch.from_numpy(w.params.copy()).cuda()
    fd = torch.from_numpy(w.feats).cuda() if w.feats is not None else None
    y = np.random.Generator(np.random.PCG64(4001)).uniform(-1, 1, (B, n)).astype(np.float32)
    yd = torch.from_numpy(y).cuda()
    loss = torch.empty(B, dtype=torch.float32, device="cuda")
    grad = torch.empty((B, P), dtype=torch.float32, device="cuda")
    ml = torch.empty(1, dtype=torch.float32, device="cuda")
    mg = torch.empty(P, dtype=torch.float32, device="cuda")
    m = torch.zeros(P, dtype=torch.float32, device="cuda")
    v = torch.zeros(P, dtype=torch.float32, device="cuda")
    t = [0]

    def step(tm):
        if idx == 3:
            ctx.qsv_loss_grad(circ, xd, pd, None, qb.QSV_LOSS_TRASH, loss, grad, ml, mg, mask=w.trash_mask)
        else:
            ctx.qsv_loss_grad(circ, xd, pd, fd, qb.QSV_LOSS_MSE_Z, loss, grad, ml, mg, targets=yd)
        t[0] += 1
        ctx.qsv_adam_step(pd, mg, m, v, t[0], 0.01)

    steps = max(1, min(args.steps, 5))
    ms, _ = run_steps(torch, step, steps, 1)
    torch.cuda.synchronize()
    out = {"workload": ("c3 training step: 20 qubits, batch 32, 20-layer encoder, loss 1 - P0 on 4 trash qubits"
                        if idx == 3 else
                        "c1 training step: 10 qubits, batch 1024, 6 re-uploading layers, squared error on <Z_q>"),
           "method": "qsv_loss_grad (reverse mode) + qsv_adam_step", "params": P, "steps": steps,
           "ms_per_step": ms, "mean_loss_after": float(ml.item()),
           "shift_rule_circuits_replaced": B * (2 * P + 1)}
    ctx.close()
    return out


def bench_c0(torch, qb, wl, args):
    w = wl.config(0)
    n, B = w.n, w.batch
    circ = qb.circuit_from_spec(w.circuit)
    xd, pd = torch.from_numpy(w.x).cuda(), torch.from_numpy(w.params).cuda()
    p = torch.empty((B, 1 << n), dtype=torch.float32, device="cuda")

    def build():
        ctx = qb.Context(n, B)

        def step(tm):
            ctx.qsv_amp_encode(xd)
            ctx.qsv_apply_layers(circ, pd, None, 0)
            ctx.qsv_apply_layers(circ, pd, None, 1)
            ctx.qsv_measure(qb.QSV_M_PROBS, p)
        return ctx, step

    ctx, step = build()
    ms, _ = run_steps(torch, step, args.steps, args.warmup)
    updates = 2 * wl.nominal_updates(w.circuit, n, B)
    fms, _ = run_steps(torch, lambda tm: ctx.qsv_forward_small(xd, circ, pd, None, 1, qb.QSV_M_PROBS, p),
                       max(args.steps, 50), args.warmup)
    ctx.close()
    gms = graph_replay_ms(torch, build, max(args.steps, 50))
    return {"workload": "c0: 4 qubits, batch 64, 2-layer encoder + decoder, basis probabilities",
            "ms_per_step": ms, "updates": updates, "updates_per_s": updates / (ms * 1e-3),
            "one_launch_ms_per_step": fms, "one_launch_updates_per_s": updates / (fms * 1e-3),
            "graph_replay_ms_per_step": gms, "graph_replay_updates_per_s": updates / (gms * 1e-3),
            "what": "ms_per_step: qsv_amp_encode + 2 x qsv_apply_layers + qsv_measure; one_launch: "
                    "qsv_forward_small; graph_replay: the separate calls captured into one HIP graph"}


def probe(torch, qb, args):
    """Load/store-only passes over a 2^26-amplitude state (512 MiB read + 512 MiB written per
    launch), for a few tile geometries (low bits c, window start w)."""
    n = 26
    ctx = qb.Context(n, 1)
    if args.tile:
        ctx.qsv_set_option("tile_log2", args.tile)
    if args.defer >= 0:
        ctx.qsv_set_option("defer_cnots", args.defer)
    if args.prio >= 0:
        ctx.qsv_set_option("load_store_priority", args.prio)
    if args.nt >= 0:
        ctx.qsv_set_option("nt_store", args.nt)
    if args.rev >= 0:
        ctx.qsv_set_option("reverse_passes", args.rev)
    if args.probe_layout >= 0:
        ctx.qsv_set_option("probe_layout", args.probe_layout)
    tile = args.tile or 12
    ctx.state.normal_()
    nbytes = 2 * 8 * (1 << n)
    out = []
    for c, w in ((tile, tile), (8, n - (tile - 8)), (6, n - (tile - 6)), (5, n - (tile - 5)), (4, 10), (4, n - (tile - 4))):
        for _ in range(3):
            ctx.qsv_probe_pass(c, w, args.probe_transposes)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(args.steps):
            ctx.qsv_probe_pass(c, w, args.probe_transposes)
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / args.steps
        out.append({"low_bits": c, "window_start": w, "ms": ms, "gbs": nbytes / ms / 1e6})
    ctx.close()
    return {"probe": "load/store-only pass, 26 qubits", "bytes_per_launch": nbytes, "tile_log2": tile,
            "geometries": out}


def cpu_baseline(wl, w4, layers):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample of config 4:
    encode + the first `layers` layers on the same 2^26-amplitude state."""
    from oracle import cpu
    cpu.build()
    spec = w4.circuit
    per = spec.slots() * w4.n
    circ = cpu.make_circuit(layers, list(spec.rot), spec.entangler, 0)
    t0 = time.perf_counter()
    st, _ = cpu.amp_encode(w4.x, w4.n)
    cpu.apply_layers(st, circ, w4.params[:layers * per])
    dt = time.perf_counter() - t0
    updates = layers * spec.gates_per_layer(w4.n) * (1 << w4.n)
    return {"value": updates / dt, "unit": "updates/s", "cores": cpu.max_threads(), "kind": "oracle",
            "sample": "config 4 state (2^26 amplitudes, complex128): amplitude encoding + first %d of 30 "
                      "layers (%d gates), %.1f s" % (layers, layers * spec.gates_per_layer(w4.n), dt)}


def alu_view(head):
    if "unitary_flops" not in head:
        return None
    tf = head["unitary_flops"] / (head["apply_ms"] * 1e-3) / 1e12
    # one FMA per lane and cycle: 256 CUs x 4 SIMDs x 16 lanes x 2 flops x 2.4 GHz
    one_per_lane = 256 * 4 * 16 * 2 * 2.4e9 / 1e12
    return {"achieved": tf, "peak": 157.3, "unit": "TFLOP/s", "frac": tf / 157.3,
            "peak_without_packed_instructions": one_per_lane, "frac_without_packed_instructions": tf / one_per_lane,
            "note": "fp32 vector peak of the data sheet (reached with packed instructions only, which this build does not "
                    "use); with one FMA per lane and cycle the same units give 78.6 TFLOP/s; flops are those of the "
                    "unitaries alone (26 per amplitude pair), about 87 % of the vector instructions of a pass"}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2602_13140_amd import binding as qb
    from paper_2602_13140_amd import workloads as wl
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    qb.load()  # fails loudly if libqsv.so is missing: there is no fallback path
    if args.probe:
        print(json.dumps(probe(torch, qb, args)))
        return
    which = [int(c) for c in args.configs.split(",") if c != ""]
    others = {}
    w4 = None
    if 4 in which or not which:
        head, w4 = bench_c4(torch, qb, wl, args)
    elif which[0] == 3:
        head = bench_c3(torch, qb, wl, args, batch=args.c3_batch or None)   # profiling aid: config 3 as the only workload
    else:
        print("bench.py: --configs must include 4 (the headline) or start with 3", file=sys.stderr)
        sys.exit(2)
    if 3 in which and w4 is not None:
        others["c3"] = bench_c3(torch, qb, wl, args)
        others["c3_batch128"] = bench_c3(torch, qb, wl, args, batch=128)
        if args.defer != 0 and not args.no_classic:
            cargs = argparse.Namespace(**vars(args))
            cargs.defer, cargs.steps, cargs.warmup = 0, 5, 1
            others["c3_batch128_no_deferral"] = bench_c3(torch, qb, wl, cargs, batch=128)
        others["c3_train"] = bench_train(torch, qb, wl, args, 3)
    if w4 is not None and args.defer != 0 and not args.no_classic:
        # config 4 with every CNOT a register operation (the plan without deferral): more, lighter passes
        cargs = argparse.Namespace(**vars(args))
        cargs.defer, cargs.steps, cargs.warmup = 0, 5, 1
        c4c, _ = bench_c4(torch, qb, wl, cargs, apply_only=True)
        others["c4_no_deferral"] = {k: c4c[k] for k in ("apply_ms", "passes", "apply_updates_per_s", "pass_avg_ms",
                                                        "pass_gbs")}
        others["c4_no_deferral"]["pass_hbm_frac"] = c4c["pass_gbs"] / HBM_PEAK_GBS
        others["c4_no_deferral"]["what"] = ("config 4's 30 layers with defer_cnots = 0: every CNOT in registers, "
                                            "more and lighter passes over the state")
    if 2 in which:
        others["c2"] = bench_c2(torch, qb, wl, args)
    if 1 in which:
        others["c1"] = bench_c1(torch, qb, wl, args)
        others["c1_train"] = bench_train(torch, qb, wl, args, 1)
    if 0 in which:
        others["c0"] = bench_c0(torch, qb, wl, args)
    cpu = None
    if not args.no_cpu and w4 is not None:
        cpu = cpu_baseline(wl, w4, args.cpu_layers)
    out = {
        "metric": "gate-amplitude updates/sec (batched, complex64) + achieved HBM GB/s vs peak",
        "value": head["updates_per_s"], "unit": "updates/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": head["workload"], "tile_log2": args.tile, "passes": head["passes"],
                   "apply_ms": head["apply_ms"], "apply_updates_per_s": head["apply_updates_per_s"]},
        "roofline": {"bound": "hbm", "kernel": "k_pass (fused gate pass)", "achieved": head["pass_gbs"],
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": head["pass_gbs"] / HBM_PEAK_GBS,
                     "traffic": TRAFFIC_BYTES_PER_LAUNCH.get(head["workload"][:2]),
                     "traffic_source": "rocprofv3 FETCH_SIZE / WRITE_SIZE of an earlier run of this command, scaled by "
                                       "a load/store-only pass of known size (profiles/k_pass_hbm_traffic_counters.md); "
                                       "not re-measured in this run",
                     "bytes_per_launch": head["pass_bytes"], "avg_launch_ms": head["pass_avg_ms"],
                     "launches_per_pass": head.get("launches_per_pass", 1),
                     # the same launches against the vector-ALU roofline: a fused unitary is 26 flops per amplitude
                     # pair (2 multiplies + 12 FMAs), CNOTs and transposes move data and count nothing
                     "alu_view": alu_view(head)},
        "cpu_baseline": cpu,
        "others": dict(others, **{k: head[k] for k in ("pauli_string", "true_reset") if k in head}),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
