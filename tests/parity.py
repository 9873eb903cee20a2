"""Helpers for the GPU parity tests: move seeded host arrays to the device bit for bit, call the
library through its C ABI, bring the result back as fp64, and compare with the CPU oracle under
the stated tolerances."""
from __future__ import annotations

import numpy as np

import workloads as wl
from paper_1910_00078_amd import cvx

DT_CODE = {wl.F32: cvx.CVX_F32, wl.F16: cvx.CVX_F16, wl.BF16: cvx.CVX_BF16}


def to_device(stored: np.ndarray, dtype: str):
    import torch
    if dtype == wl.BF16:
        return torch.from_numpy(stored.view(np.int16).copy()).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(stored)).cuda()


def to_host_f64(t, dtype: str) -> np.ndarray:
    import torch
    if dtype == wl.BF16:
        bits = t.view(torch.int16).cpu().numpy().view(np.uint16)
        return wl.to_f64(bits, dtype)
    return t.cpu().numpy().astype(np.float64)


def tolerance_ok(gpu: np.ndarray, ref: np.ndarray, dtype: str):
    """fp32: relative L2 error <= 1e-5.  fp16 / bf16: every element within 1e-2*|ref| + 1e-3*rms(ref).
    Returns (ok, message)."""
    gpu = gpu.astype(np.float64).ravel()
    ref = ref.astype(np.float64).ravel()
    if not np.all(np.isfinite(gpu)):
        return False, "non-finite values in GPU output"
    if dtype == wl.F32:
        den = np.linalg.norm(ref)
        rel = np.linalg.norm(gpu - ref) / den if den > 0 else np.linalg.norm(gpu - ref)
        return rel <= 1e-5, "relative L2 error %.3e (limit 1e-5)" % rel
    rms = float(np.sqrt(np.mean(ref * ref)))
    err = np.abs(gpu - ref)
    lim = 1e-2 * np.abs(ref) + 1e-3 * rms
    bad = err > lim
    worst = int(np.argmax(err - lim))
    return (not bad.any(),
            "%d of %d outside tolerance; worst at %d: gpu %.6g ref %.6g (limit %.3g, rms %.3g)"
            % (int(bad.sum()), err.size, worst, gpu[worst], ref[worst], lim[worst], rms))


def run_gpu(w: wl.ConvWorkload, x, wt, b, *, act=cvx.CVX_ACT_RELU, alpha=0.0, policy=0, bias_f32=False,
            bn=None, eps=1e-5, use_bias=True, pin=None, offsets=(0, 0, 0)):
    """x, wt, b in storage representation (host).  Returns (y as fp64 host array, name of the kernel the
    call enqueued).  pin is the developer kernel pin; offsets moves
    x, w, y that many elements off their allocations' (16-byte-aligned) starts."""
    import torch
    dx, dw = to_device(x, w.dtype), to_device(wt, w.dtype)
    if offsets[0]:
        dx = _shifted(dx, offsets[0])
    if offsets[1]:
        dw = _shifted(dw, offsets[1])
    db = None
    if use_bias:
        db = torch.from_numpy(wl.to_f64(b, w.dtype).astype(np.float32)).cuda() if bias_f32 else to_device(b, w.dtype)
    dbn = None if bn is None else tuple(torch.from_numpy(np.asarray(t, np.float32)).cuda() for t in bn)
    # every output element starts as NaN: one the kernel never writes fails the comparison instead of
    # showing whatever the allocator left there (possibly an earlier case's correct result)
    y = torch.full((w.N, w.K, w.Ho, w.Wo), float("nan"), dtype=dx.dtype, device="cuda")
    if offsets[2]:
        y = _shifted(y, offsets[2], fill=float("nan"))
    info = {}
    cvx.conv_fwd_fused(dx, dw, db, pad=w.pad, stride=w.stride, dil=w.dil, groups=w.groups, act=act,
                       alpha=alpha, bn=dbn, eps=eps, policy=policy, out=y, pin=pin, info=info)
    torch.cuda.synchronize()
    return to_host_f64(y, w.dtype), info["kernel"]


def _shifted(t, elements: int, fill=0.0):
    """A contiguous copy of t that starts `elements` elements into a fresh allocation."""
    import torch
    buf = torch.full((t.numel() + elements,), fill, dtype=t.dtype, device=t.device)
    view = buf[elements:].view(t.shape)
    view.copy_(t)
    return view


def run_oracle(w: wl.ConvWorkload, x, wt, b, *, act=1, alpha=0.0, bn=None, eps=1e-5, use_bias=True):
    from oracle import conv_oracle
    return conv_oracle.conv_fwd(wl.to_f64(x, w.dtype), wl.to_f64(wt, w.dtype),
                                wl.to_f64(b, w.dtype) if use_bias else None,
                                pad=w.pad, stride=w.stride, dil=w.dil, groups=w.groups, act=act, alpha=alpha,
                                bn=bn, eps=eps)
