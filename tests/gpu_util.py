"""Helpers for the GPU parity tests: run the HIP path through the C ABI on seeded inputs and
fetch results as numpy arrays.  No arithmetic of the method happens here."""
import numpy as np


def torch_cuda():
    import torch
    return torch


def dev(a):
    torch = torch_cuda()
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def state_np(ctx):
    torch = torch_cuda()
    torch.cuda.synchronize()
    s = ctx.state.cpu().numpy()
    return (s[..., 0].astype(np.float64) + 1j * s[..., 1].astype(np.float64))


def make_ctx(n, batch, tile=0, naive=0, planes=0, ws_bytes=None):
    from paper_2602_13140_amd import binding as qb
    ctx = qb.Context(n, batch, ws_bytes=ws_bytes)
    if tile:
        ctx.qsv_set_option("tile_log2", tile)
    if planes:
        ctx.qsv_set_option("lds_planes", planes)
    if naive:
        ctx.qsv_set_option("naive", 1)
    return ctx


def measure(ctx, kind, shape, dtype="float32", **kw):
    torch = torch_cuda()
    out = torch.full(shape, -7.0 if dtype == "float32" else -7,
                     dtype=getattr(torch, dtype), device="cuda")
    ctx.qsv_measure(kind, out, **kw)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def prob_checks(p_gpu, p_ref):
    """Contract tolerance (1e-5 absolute) plus relative checks that stay meaningful when the
    probabilities themselves are tiny."""
    p_gpu = np.asarray(p_gpu, dtype=np.float64)
    d = np.abs(p_gpu - p_ref)
    assert d.max() <= 1e-5, d.max()
    assert d.sum(axis=-1).max() <= 1e-4, d.sum(axis=-1).max()
    assert (d.max(axis=-1) / p_ref.max(axis=-1)).max() <= 1e-3
