"""Helpers shared by the GPU parity tests: device upload/download, the error metric and
schedule forcing.  Holds none of the method's arithmetic."""
import contextlib
import os

import numpy as np
import torch

import paper_2006_16236_amd as la
import workloads as wl

DEV = "cuda:0"

# Tolerances of the benchmark spec: max|gpu - ref| / max|ref| per output tensor.
TOL_F32 = 1e-4          # fp32, N <= 4096
TOL_F32_LONG = 1e-3     # fp32, N > 4096
TOL_BF16 = 2e-2         # bf16 tensors, fp32 accumulation


def tol_for(N, bf16=False):
    if bf16:
        return TOL_BF16
    return TOL_F32 if N <= 4096 else TOL_F32_LONG


def rel_err(got, ref, floor=0.0):
    """max|got - ref| / max(max|ref|, floor).  `floor` matters only where the exact result
    vanishes by cancellation (see grad_errs)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape
    assert np.all(np.isfinite(got)), "non-finite values in the GPU result"
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), floor, 1e-300))


def err_report(got, ref):
    """Three views of the same difference (ref: fp64 oracle):
    max_norm     max|d| / max|ref|                          (the gate of the benchmark spec)
    elementwise  max over elements of |d| / (|ref| + 1e-3 max|ref|): every element against its
                 own size, floored so that exact zeros do not divide by nothing.  The causal
                 output shrinks like 1/sqrt(i) along a long sequence; this view keeps the late
                 tokens honest where the max-norm only sees the early ones
    rms          sqrt(mean d^2) / sqrt(mean ref^2)"""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape and np.all(np.isfinite(got))
    d = np.abs(got - ref)
    top = max(float(np.abs(ref).max()), 1e-300)
    return {"max_norm": float(d.max() / top),
            "elementwise": float((d / (np.abs(ref) + 1e-3 * top)).max()),
            "rms": float(np.sqrt(np.mean(d * d)) / max(np.sqrt(np.mean(ref * ref)), 1e-300))}


def grad_errs(got, ref):
    """Errors of (dQ, dK, dV).  Each tensor is scaled by its own max|ref|, but never by less
    than 1e-3 of the largest of the three: for N = 1 (and for constant V) the exact dQ, dK
    are zero up to eps, every term cancels, and a scale of their own would be meaningless."""
    floor = 1e-3 * max(float(np.abs(r).max()) for r in ref)
    return [rel_err(a, b, floor) for a, b in zip(got, ref)]


def to_dev(x, bf16=False):
    """float32 host array -> device tensor (bf16: the values must already be bf16-exact)."""
    t = torch.from_numpy(np.ascontiguousarray(x)).to(DEV)
    return t.to(torch.bfloat16) if bf16 else t


def to_host(t):
    return t.detach().to(torch.float32).cpu().numpy()


@contextlib.contextmanager
def schedule(target_waves=None, min_seg_chunks=None, fold_max_segs=None, bwd_seg_group=None,
             stream_loads=None):
    """Force the segment schedule (and the kind of loads) of the library through its environment
    knobs."""
    keys = {"LA_TARGET_WAVES": target_waves, "LA_MIN_SEG_CHUNKS": min_seg_chunks,
            "LA_FOLD_MAX_SEGS": fold_max_segs, "LA_BWD_SEG_GROUP": bwd_seg_group,
            "LA_STREAM_LOADS": stream_loads}
    old = {k: os.environ.get(k) for k in keys}
    try:
        for k, v in keys.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = str(v)
        la.la_tuning_reload()
        yield
    finally:
        for k, v in old.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v
        la.la_tuning_reload()


SCHEDULES = {
    "default": dict(),
    "one_segment": dict(target_waves=1),
    "many_segments": dict(target_waves=1 << 20, min_seg_chunks=1),
    "three_chunk_segments": dict(target_waves=1 << 20, min_seg_chunks=3),
    # few segments per sequence, their totals added up by the consumers (no scan kernel) ...
    "folded_totals": dict(target_waves=24, min_seg_chunks=1, fold_max_segs=64),
    # ... and the same few segments through the scan kernel
    "few_segments_scanned": dict(target_waves=24, min_seg_chunks=1, fold_max_segs=1),
}


def maybe_bf16(arrs, bf16):
    return [wl.round_to_bf16(a) for a in arrs] if bf16 else list(arrs)
