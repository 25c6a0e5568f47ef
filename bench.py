#!/usr/bin/env python3
"""Benchmark of the linear-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One "step" is one pass of the whole training hot path over one batch of synthetic
input: la_causal_fwd followed by la_causal_bwd (every kernel they launch) on the
metric's workload: B=2, H=8, N=65536, D=M=64, fp32, Q/K/V/dO i.i.d. N(0,1) from
a fixed seed, already resident in HBM when the clock starts.  Prints ONE JSON line:
throughput in Mtokens/s (a token = all 8 heads), the roofline fraction of the
dominant kernel (HIP events around its launches inside the timed region) and the
fp64 CPU oracle timed on this machine's host cores on a bounded sample.

`--workload NAME` runs another workload instead of the metric's (same output format, its own
metric name; for per-kernel profiles of the other kernel families): headline_bf16, global,
global_bf16, cfg2, cfg3, cfg3_bf16 (forward + backward), decode_B64, decode_B4096 (one
la_recurrent_step per step), decode_B64_multi (one la_recurrent_steps launch of 3072 steps).

`--table PATH` additionally times the other workloads (sequence-length sweep, the
MNIST/CIFAR-shaped configs, bf16, the non-causal pair and the decode loop) and writes
them to PATH as JSON; it is a reporting aid and prints no extra stdout line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
MFMA_F32_PEAK_TFLOPS = 157.3     # MI355X dense fp32 matrix, published


# HBM bytes per launch at the metric's workload, measured with rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE and scaled by a copy kernel of known size: read from the tracked summary of that
# run (the table in profiles/), so that the figure on the bench line cannot drift from it.
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "hbm_traffic_and_pipe_counters_N65536_B2_H8_D64_f32.md")
TRAFFIC_ROW = {"causal_pass_fwd": "causal_pass_kernel<0", "pass_dq": "dq_causal_kernel",
               "reverse_pass_dv_dk": "reverse_pass_kernel", "segment_state_kv": "segment_state_kernel",
               "scan_states": "scan_states_kernel"}


def measured_traffic_bytes(path: str = TRAFFIC_SUMMARY) -> dict:
    """{bench kernel name: bytes read + written per launch} from the traffic table of the
    profile summary (columns: kernel | FETCH_SIZE KiB | WRITE_SIZE KiB | read MB (scaled) |
    written MB (scaled) | ...); {} if the file or the table is missing."""
    out = {}
    try:
        with open(path) as f:
            lines = f.read().splitlines()
    except OSError:
        return out
    for line in lines:
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) < 5:
            continue
        for name, key in TRAFFIC_ROW.items():
            if key in cells[0] and name not in out:
                try:
                    out[name] = float(round((float(cells[3]) + float(cells[4])) * 1e6))
                except ValueError:
                    pass
    return out


def kernel_bytes(name: str, D: int, M: int, e: int) -> float:
    """Algorithmic HBM bytes per token-head of one launch of `name`: the tensors it must
    read and write once (e = bytes per element of the N-sized tensors; den, 1/den and
    delta are fp32 scalars per token-head)."""
    return {
        "causal_pass_fwd": e * (2 * D + 2 * M) + 4,     # Q K V -> O, den
        "pass_dq": e * (3 * D + 2 * M) + 12,            # dO V K Q, den -> dQ, 1/den, delta
        "reverse_pass_dv_dk": e * (3 * D + 3 * M) + 8,  # Q K V dO, 1/den, delta -> dV, dK
        "segment_state_kv": e * (D + M),                # K V
        "global_readout": e * (D + M) + 4,              # Q -> O, den
        "pass_dq_global": e * (2 * D + M) + 4,          # Q dO, den -> dQ (non-causal)
        "global_bwd_readouts": e * (2 * D + 2 * M),     # K V -> dV, dK
        "recurrent_step": 2 * 4 * D * (M + 1) + e * (2 * D + 2 * M),   # S, z read and written; q k v out
        "recurrent_steps": e * (2 * D + 2 * M),         # per step of a multi-step launch: q k v out
                                                        # (the state stays in registers)
    }.get(name, 0.0)


def kernel_flops(name: str, D: int, M: int) -> float:
    """Algorithmic flops per token-head: the state update and the state read-out
    (2*D*(M+1) each, ones column included) that the pass performs."""
    full = 4.0 * D * (M + 1)
    return {"causal_pass_fwd": full, "pass_dq": 1.5 * full, "reverse_pass_dv_dk": 1.5 * full,
            "segment_state_kv": full / 2, "global_readout": full / 2, "pass_dq_global": full / 2,
            "global_bwd_readouts": full, "recurrent_step": full, "recurrent_steps": full}.get(name, 0.0)


class FwdBwd:
    """Device buffers and the step function for one workload."""

    def __init__(self, w, bf16=False, token_major=False, group=0, poly2=False):
        """group > 0: the (batch, head) sequences are processed `group` at a time (forward and
        backward of one group, then the next): a schedule experiment, see --groups.
        poly2: Q and K hold 8 raw values per token and the library applies the degree-2
        polynomial map (section 3.2) to 64 features; eps 0.5."""
        import torch

        import paper_2006_16236_amd as la
        import workloads as wl
        self.la, self.torch, self.w, self.bf16 = la, torch, w, bf16
        dev = "cuda:0"
        host = wl.qkvg(w)
        if bf16:
            host = [wl.round_to_bf16(x) for x in host]
        self.feat = False
        self.eps = w.eps
        if poly2:       # the first 8 of the 64 columns of Q and K are the raw vectors
            host = [host[0][..., :8].copy(), host[1][..., :8].copy(), host[2], host[3]]
            self.feat, self.eps = "poly2", 0.5
        self.host = host
        dt = torch.bfloat16 if bf16 else torch.float32
        self.Q, self.K, self.V, self.G = (torch.from_numpy(x).to(dev).to(dt) for x in host)
        self.token_major = token_major
        if token_major:      # [B, H, N, .] -> [B, N, H, .], the entry points for that layout
            self.Q, self.K, self.V, self.G = (x.transpose(1, 2).contiguous()
                                              for x in (self.Q, self.K, self.V, self.G))
        self.O = torch.empty_like(self.V)
        self.den = torch.empty(w.B, w.H, w.N, dtype=torch.float32, device=dev)
        self.dQ, self.dK, self.dV = (torch.empty_like(x) for x in (self.Q, self.K, self.V))
        code = la.LA_F32_POLY2 if poly2 else la.LA_BF16 if bf16 else la.LA_F32
        Dq = 8 if poly2 else w.D
        nf = la.la_causal_fwd_workspace(w.B, w.H, w.N, Dq, w.M, code)
        nb = la.la_causal_bwd_workspace(w.B, w.H, w.N, Dq, w.M, code)
        self.ws_f = torch.empty(max(nf, 16), dtype=torch.uint8, device=dev)
        self.ws_b = torch.empty(max(nb, 16), dtype=torch.uint8, device=dev)
        self.groups = None
        if group > 0 and not token_major:
            BH = w.B * w.H
            flat = [x.view(BH, *x.shape[2:]) for x in (self.Q, self.K, self.V, self.G, self.O, self.den,
                                                       self.dQ, self.dK, self.dV)]
            self.groups = []
            for i in range(0, BH, group):
                n = min(group, BH - i)
                views = [x[i:i + n].unsqueeze(0) for x in flat]      # [1, n, N, .]: contiguous slices
                wf = torch.empty(max(la.la_causal_fwd_workspace(1, n, w.N, w.D, w.M, code), 16),
                                 dtype=torch.uint8, device=dev)
                wb = torch.empty(max(la.la_causal_bwd_workspace(1, n, w.N, w.D, w.M, code), 16),
                                 dtype=torch.uint8, device=dev)
                self.groups.append((views, wf, wb))

    def step(self):
        la, w = self.la, self.w
        if self.groups is not None:
            for (Q, K, V, G, O, den, dQ, dK, dV), wf, wb in self.groups:
                la.la_causal_fwd(Q, K, V, O, den, w.eps, ws=wf)
                la.la_causal_bwd(Q, K, V, O, den, G, dQ, dK, dV, w.eps, ws=wb, fwd_ws=wf)
            return
        fwd = la.la_causal_fwd_bnhd if self.token_major else la.la_causal_fwd
        bwd = la.la_causal_bwd_bnhd if self.token_major else la.la_causal_bwd
        fwd(self.Q, self.K, self.V, self.O, self.den, self.eps, ws=self.ws_f, features=self.feat)
        bwd(self.Q, self.K, self.V, self.O, self.den, self.G, self.dQ, self.dK,
            self.dV, self.eps, ws=self.ws_b, fwd_ws=self.ws_f, features=self.feat)

    def fwd_only(self):
        fwd = self.la.la_causal_fwd_bnhd if self.token_major else self.la.la_causal_fwd
        fwd(self.Q, self.K, self.V, self.O, self.den, self.eps, ws=self.ws_f, features=self.feat)


# The GPU needs some tens of milliseconds of back-to-back work to settle its clocks: the first
# 20 steps after a pause run ~7 % slower than the following ones.  Hence the default warm-up of the
# headline run (--warmup 50) and of every row of the table.
TABLE_WARMUP = 30
SETTLE_STEPS = 50


def time_steps(fn, steps, warmup, torch):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def profile_kernels(la, fn, steps, torch, mask=None):
    torch.cuda.synchronize()
    la.la_profile_begin() if mask is None else la.la_profile_begin(mask)
    for _ in range(steps):
        fn()
    prof = la.la_profile_end()
    return {k: (ms / n, n // steps) for k, (ms, n) in prof.items()}   # avg ms per launch, launches/step


def cpu_baseline(w, host, sample_tokens, causal=True):
    """The oracle as it stands (fp64, OpenMP over the (b, h) slabs), forward + backward, on
    the first `sample_tokens` tokens of every slab of the same workload."""
    import numpy as np

    from oracle import la_oracle
    Q, K, V, G = (np.ascontiguousarray(x[:, :, :sample_tokens], dtype=np.float64) for x in host)
    threads = min(la_oracle.max_threads(), w.B * w.H)
    fwd = la_oracle.causal_fwd_prefix if causal else la_oracle.global_fwd_linear
    bwd = la_oracle.causal_bwd_linear if causal else la_oracle.global_bwd_linear
    t0 = time.perf_counter()
    fwd(Q, K, V, w.eps)
    bwd(Q, K, V, G, w.eps)
    dt = time.perf_counter() - t0
    # one thread on one (batch, head) sequence, first 16384 tokens: the per-core rate
    n1 = min(sample_tokens, 16384)
    one = [np.ascontiguousarray(x[:1, :1, :n1]) for x in (Q, K, V, G)]
    nmax = la_oracle.max_threads()
    la_oracle.set_threads(1)
    t1 = time.perf_counter()
    fwd(*one[:3], w.eps)
    bwd(*one, w.eps)
    dt1 = time.perf_counter() - t1
    la_oracle.set_threads(nmax)
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            model = next(l.split(":", 1)[1].strip() for l in f if l.startswith("model name"))
    except (OSError, StopIteration):
        pass
    return {"value": w.B * sample_tokens / dt / 1e6, "unit": "Mtokens/s", "cores": threads,
            "kind": "oracle", "cpu_model": model,
            "single_thread_mtok_s": n1 / w.H / dt1 / 1e6,   # one head of n1 tokens = n1/H tokens

            "sample": f"fp64 oracle forward+backward on the first {sample_tokens} of {w.N} tokens of "
                      f"all {w.B * w.H} (batch, head) sequences of the same inputs, one run, "
                      f"{dt:.1f} s wall x {threads} threads = {dt * threads:.0f} s of CPU work; OpenMP "
                      f"over sequences ({nmax} threads available, {threads} busy)"}


class GlobalFwdBwd(FwdBwd):
    """The same buffers, stepping the non-causal pair (la_global_fwd + la_global_bwd)."""

    def __init__(self, w, bf16=False):
        super().__init__(w, bf16)
        la, torch = self.la, self.torch
        code = la.LA_BF16 if bf16 else la.LA_F32
        self.ws_f = torch.empty(la.la_global_fwd_workspace(w.B, w.H, w.N, w.D, w.M, code),
                                dtype=torch.uint8, device="cuda:0")
        self.ws_b = torch.empty(la.la_global_bwd_workspace(w.B, w.H, w.N, w.D, w.M, code),
                                dtype=torch.uint8, device="cuda:0")

    def step(self):
        la, w = self.la, self.w
        la.la_global_fwd(self.Q, self.K, self.V, self.O, w.eps, ws=self.ws_f, den=self.den)
        la.la_global_bwd(self.Q, self.K, self.V, self.O, self.den, self.G, self.dQ, self.dK, self.dV,
                         w.eps, ws=self.ws_b, fwd_ws=self.ws_f)


class Decode:
    """Recurrent decode (eq. 16-20): B sequences, one token per head per step; `multi` > 0:
    one la_recurrent_steps launch of that many steps."""

    def __init__(self, d, B, multi=0):
        import torch

        import paper_2006_16236_amd as la
        self.la, self.d, self.B, self.multi, self.t = la, d, B, multi, 0
        T = multi if multi else 8
        g = torch.Generator(device="cuda:0").manual_seed(d.seed)
        self.q = torch.randn(T, B, d.H, d.D, device="cuda:0", generator=g)
        self.k = torch.randn(T, B, d.H, d.D, device="cuda:0", generator=g)
        self.v = torch.randn(T, B, d.H, d.M, device="cuda:0", generator=g)
        self.S = torch.zeros(B, d.H, d.D, d.M, device="cuda:0")
        self.z = torch.zeros(B, d.H, d.D, device="cuda:0")
        self.out = torch.empty(T if multi else 1, B, d.H, d.M, device="cuda:0")

    def step(self):
        la, d = self.la, self.d
        if self.multi:
            la.la_recurrent_steps(self.q, self.k, self.v, self.S, self.z, self.out, d.eps)
        else:
            t = self.t = (self.t + 1) % 8
            la.la_recurrent_step(self.q[t], self.k[t], self.v[t], self.S, self.z, self.out[0], d.eps)


WORKLOADS = ("headline", "headline_bf16", "headline_poly2", "global", "global_bf16", "cfg2", "cfg3", "cfg3_bf16",
             "decode_B64", "decode_B4096", "decode_B64_multi")


def make_workload(name, group=0):
    """-> (object with .step(), description dict).  tokens: tokens per step (a token = all H
    heads); path_bytes: compulsory HBM bytes per token-head of one step (the tensors that must be
    read and written once), None where a step is not one pass over tensors."""
    import workloads as wl
    if name.startswith("decode"):
        d = wl.CFG5
        B = 4096 if "4096" in name else d.B
        multi = d.T if name.endswith("_multi") else 0
        obj = Decode(d, B, multi)
        steps_per = multi if multi else 1
        return obj, {"metric": "recurrent decode Mtokens/s (H=8,D=M=64)", "tokens": B * steps_per,
                     "H": d.H, "D": d.D, "M": d.M, "e": 4, "dtype": "f32", "host": None,
                     "path_bytes": kernel_bytes("recurrent_steps" if multi else "recurrent_step", d.D, d.M, 4),
                     "w": None,
                     "config": {"workload": name, "B": B, "H": d.H, "D": d.D, "M": d.M, "eps": d.eps,
                                "step": f"la_recurrent_steps, T={multi}" if multi else "la_recurrent_step",
                                "seed": d.seed},
                     "rename": {"recurrent_step": "recurrent_steps"} if multi else {}}
    bf16 = name.endswith("_bf16")
    poly2 = name.endswith("_poly2")
    base = name[:-5] if bf16 else name[:-6] if poly2 else name
    w = {"headline": wl.HEADLINE, "global": wl.HEADLINE, "cfg2": wl.CFG2, "cfg3": wl.CFG3}[base]
    glob = base == "global"
    obj = GlobalFwdBwd(w, bf16) if glob else FwdBwd(w, bf16, group=group, poly2=poly2)
    e = 2 if bf16 else 4
    metric = ("non-causal" if glob else "causal") + f" linear-attn fwd+bwd Mtokens/s (H={w.H},D={w.D},M={w.M},N={w.N})"
    if name == "headline":
        metric = "causal linear-attn fwd+bwd Mtokens/s (H=8,D=M=64,N=2^16)"
    if poly2:
        metric = "causal linear-attn fwd+bwd Mtokens/s, degree-2 polynomial map of 8 raw dims (H=8,C=M=64,N=2^16)"
    # D: elements per token of Q, K (sizes the bytes); C: feature width (sizes the flops)
    return obj, {"metric": metric, "tokens": w.B * w.N, "H": w.H, "D": 8 if poly2 else w.D, "C": w.D, "M": w.M, "e": e,
                 "dtype": "bf16" if bf16 else "f32", "host": obj.host, "w": None if poly2 else w,
                 # (polynomial map: Q, K and their gradients are 8 wide, 4 of the 12 tensors)
                 "path_bytes": e * (6 * w.M + 4 * 8) if poly2 else e * (6 * w.D + 6 * w.M),
                 "config": {"workload": w.name + ("_bf16" if bf16 else "") + ("_noncausal" if glob else "")
                            + ("_poly2_map_of_8_raw_dims" if poly2 else ""),
                            "B": w.B, "H": w.H, "N": w.N, "D": 8 if poly2 else w.D, "M": w.M, "eps": obj.eps,
                            "step": "la_global_fwd + la_global_bwd" if glob else "la_causal_fwd + la_causal_bwd",
                            "seed": w.seed},
                 # the non-causal dQ kernel reads fewer tensors than the causal one
                 "rename": {"pass_dq": "pass_dq_global"} if glob else {}}


def run_workload(args):
    import statistics

    import torch

    import paper_2006_16236_amd as la

    obj, info = make_workload(args.workload, args.groups)
    if args.groups:
        info["config"]["sequences_per_group"] = args.groups
    step = obj.step
    # the first --warmup steps, on clocks as they are after a pause: timed, reported beside the
    # settled figure, not part of it
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    unsettled = (time.perf_counter() - t0) / max(args.warmup, 1)
    # clocks settle only after ~50 ms of back-to-back work (see TABLE_WARMUP): when the caller
    # asks for a shorter warm-up, run the difference as well, untimed, and say so in the output
    settle = max(0, SETTLE_STEPS - args.warmup)
    for _ in range(settle):
        step()
    # untimed look at every kernel, to find the dominant one
    prof_all = profile_kernels(la, step, 3, torch)
    per_step = {k: ms * n for k, (ms, n) in prof_all.items()}
    dominant = max(per_step, key=per_step.get)
    kid = [la.la_kernel_name(i) for i in range(la.binding.LA_K_COUNT)].index(dominant)

    # the timed region: exactly `steps` steps between two synchronisations (wall clock: the
    # mean), HIP events on the launch stream at up to 20 evenly spaced step borders (their
    # differences give a median), events inside the library only around the dominant kernel
    groups = max(1, min(args.steps, 20))
    border = [round(i * args.steps / groups) for i in range(groups + 1)]
    marks = [torch.cuda.Event(enable_timing=True) for _ in border]
    torch.cuda.synchronize()
    la.la_profile_begin(1 << kid)
    t0 = time.perf_counter()
    nxt = 0
    for i in range(args.steps):
        if i == border[nxt]:
            marks[nxt].record()
            nxt += 1
        step()
    marks[nxt].record()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    dom_ms, dom_n = la.la_profile_end()[dominant]
    dom_ms /= dom_n
    per_group = [marks[i].elapsed_time(marks[i + 1]) / (border[i + 1] - border[i]) for i in range(groups)]
    median_ms = statistics.median(per_group)

    D, M, e, H = info["D"], info["M"], info["e"], info["H"]
    tokens = info["tokens"]
    th = tokens * H
    value = tokens / sec / 1e6
    kname = info["rename"].get(dominant, dominant)
    launches_per_step = prof_all[dominant][1]
    th_per_launch = th / launches_per_step if args.workload.startswith("decode") else th
    if args.workload.endswith("_multi"):
        th_per_launch = th
    ach_gbs = kernel_bytes(kname, D, M, e) * th_per_launch / (dom_ms * 1e-3) / 1e9
    ach_tf = kernel_flops(kname, info.get("C", D), M) * th_per_launch / (dom_ms * 1e-3) / 1e12
    hbm_ceiling = HBM_PEAK_GBS * 1e9 / (H * info["path_bytes"]) / 1e6
    traffic = measured_traffic_bytes().get(dominant) if args.workload == "headline" else None
    out = {
        "metric": info["metric"],
        "value": round(value, 3), "unit": "Mtokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "settle_steps": settle, "ms_per_step": round(sec * 1e3, 4),
        "ms_per_step_median": round(median_ms, 4),
        "unsettled_ms_per_step": round(unsettled * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": info["dtype"], "data": "synthetic",
        "config": info["config"],
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": round(ach_gbs, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach_gbs / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "avg_kernel_ms": round(dom_ms, 4),
                     "mfma_f32_tflops_algorithmic": round(ach_tf, 2),
                     "mfma_f32_frac": round(ach_tf / MFMA_F32_PEAK_TFLOPS, 4)},
        "path_frac_of_hbm_roofline": round(value / hbm_ceiling, 4),
        "path_hbm_ceiling_mtok_s": round(hbm_ceiling, 1),
        "kernels_ms_per_step": {k: round(v, 4) for k, v in sorted(per_step.items(), key=lambda kv: -kv[1])},
    }
    if not args.no_cpu_baseline and info["w"] is not None:
        w = info["w"]
        out["cpu_baseline"] = cpu_baseline(w, info["host"], min(args.cpu_sample_tokens, w.N),
                                           causal="global" not in args.workload)
    return out, obj


def run_table(args):
    """Everything else worth a number; written to the file `--table` names."""
    import torch

    import paper_2006_16236_amd as la
    import workloads as wl
    rows = []

    def fwdbwd_row(w, bf16=False, steps=20, token_major=False):
        fb = FwdBwd(w, bf16, token_major)
        sec = time_steps(fb.step, steps, TABLE_WARMUP, torch)
        secf = time_steps(fb.fwd_only, steps, TABLE_WARMUP, torch)
        prof = profile_kernels(la, fb.step, 3, torch)
        e = 2 if bf16 else 4
        ceiling = HBM_PEAK_GBS * 1e9 / (w.H * e * (6 * w.D + 6 * w.M)) / 1e6
        rows.append({"workload": w.name + ("_bf16" if bf16 else "") + ("_layout_BNHD" if token_major else ""),
                     "tokens": w.B * w.N,
                     "fwd_bwd_ms": sec * 1e3, "fwd_ms": secf * 1e3,
                     "fwd_bwd_mtok_s": w.B * w.N / sec / 1e6, "fwd_mtok_s": w.B * w.N / secf / 1e6,
                     "hbm_ceiling_mtok_s": ceiling, "frac": w.B * w.N / sec / 1e6 / ceiling,
                     "kernels_ms": {k: round(ms * n, 4) for k, (ms, n) in prof.items()}})
        if not args.no_cpu_baseline and not token_major:      # the oracle on the same inputs, beside it
            cb = cpu_baseline(w, fb.host, w.N)
            rows[-1]["oracle_mtok_s"] = cb["value"]
            rows[-1]["oracle_cores"] = cb["cores"]
        print("table:", json.dumps(rows[-1]), file=sys.stderr, flush=True)
        return fb

    for w in (wl.CFG2, wl.CFG3):
        fwdbwd_row(w, steps=200)
    fwdbwd_row(wl.CFG3, bf16=True, steps=200)
    fwdbwd_row(wl.sweep_point(16), bf16=True)
    fwdbwd_row(wl.sweep_point(16), token_major=True)
    fwdbwd_row(wl.sweep_point(16), bf16=True, token_major=True)
    for n in range(9, 17):
        w = wl.sweep_point(n)
        fb = fwdbwd_row(w)
        # the non-causal forward on the same tensors
        ws = torch.empty(la.la_global_fwd_workspace(w.B, w.H, w.N, w.D, w.M), dtype=torch.uint8,
                         device="cuda:0")
        sec = time_steps(lambda: la.la_global_fwd(fb.Q, fb.K, fb.V, fb.O, w.eps, ws=ws), 20, TABLE_WARMUP, torch)
        rows.append({"workload": w.name + "_global_fwd", "tokens": w.B * w.N, "fwd_ms": sec * 1e3,
                     "fwd_mtok_s": w.B * w.N / sec / 1e6,
                     "hbm_ceiling_mtok_s": HBM_PEAK_GBS * 1e9 / (w.H * 4 * (2 * w.D + 2 * w.M)) / 1e6})
        print("table:", json.dumps(rows[-1]), file=sys.stderr, flush=True)
        # ... and forward + backward of the non-causal form
        deng = torch.empty(w.B, w.H, w.N, dtype=torch.float32, device="cuda:0")
        wsb = torch.empty(la.la_global_bwd_workspace(w.B, w.H, w.N, w.D, w.M), dtype=torch.uint8,
                          device="cuda:0")

        def global_step():
            la.la_global_fwd(fb.Q, fb.K, fb.V, fb.O, w.eps, ws=ws, den=deng)
            la.la_global_bwd(fb.Q, fb.K, fb.V, fb.O, deng, fb.G, fb.dQ, fb.dK, fb.dV, w.eps, ws=wsb,
                             fwd_ws=ws)
        sec = time_steps(global_step, 20, TABLE_WARMUP, torch)
        prof = profile_kernels(la, global_step, 3, torch)
        rows.append({"workload": w.name + "_global_fwd_bwd", "tokens": w.B * w.N,
                     "fwd_bwd_ms": sec * 1e3, "fwd_bwd_mtok_s": w.B * w.N / sec / 1e6,
                     "hbm_ceiling_mtok_s": HBM_PEAK_GBS * 1e9 / (w.H * 4 * (6 * w.D + 6 * w.M)) / 1e6,
                     "kernels_ms": {k: round(ms * n, 4) for k, (ms, n) in prof.items()}})
        print("table:", json.dumps(rows[-1]), file=sys.stderr, flush=True)
        del fb, ws, wsb, deng
    # recurrent decode: 3072 sequential steps, one token per head per step
    for B in (wl.CFG5.B, 4096):
        d = wl.CFG5
        T = d.T if B == d.B else 64
        q = torch.randn(8, B, d.H, d.D, device="cuda:0")
        k = torch.randn(8, B, d.H, d.D, device="cuda:0")
        v = torch.randn(8, B, d.H, d.M, device="cuda:0")
        S = torch.zeros(B, d.H, d.D, d.M, device="cuda:0")
        z = torch.zeros(B, d.H, d.D, device="cuda:0")
        out = torch.empty(B, d.H, d.M, device="cuda:0")
        for t in range(8):
            la.la_recurrent_step(q[t % 8], k[t % 8], v[t % 8], S, z, out, d.eps)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(T):
            la.la_recurrent_step(q[t % 8], k[t % 8], v[t % 8], S, z, out, d.eps)
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t0) / T
        bytes_step = B * d.H * (2 * 4 * d.D * (d.M + 1) + 4 * (2 * d.D + 2 * d.M))
        rows.append({"workload": f"decode_B{B}_H8_D64", "steps": T, "us_per_step": sec * 1e6,
                     "tokens_per_s": B / sec, "achieved_GBs": bytes_step / sec / 1e9,
                     "frac_hbm": bytes_step / sec / 1e9 / HBM_PEAK_GBS})
        print("table:", json.dumps(rows[-1]), file=sys.stderr, flush=True)
    # per-step launches recorded once into a HIP graph of 64 steps, replayed 48 times
    d = wl.CFG5
    q = torch.randn(64, d.B, d.H, d.D, device="cuda:0")
    k = torch.randn(64, d.B, d.H, d.D, device="cuda:0")
    v = torch.randn(64, d.B, d.H, d.M, device="cuda:0")
    S = torch.zeros(d.B, d.H, d.D, d.M, device="cuda:0")
    z = torch.zeros(d.B, d.H, d.D, device="cuda:0")
    out = torch.empty(64, d.B, d.H, d.M, device="cuda:0")

    def steps64():
        for t in range(64):
            la.la_recurrent_step(q[t], k[t], v[t], S, z, out[t], d.eps)
    steps64()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        steps64()
    sec = time_steps(graph.replay, d.T // 64, 4, torch)
    rows.append({"workload": f"decode_B{d.B}_H8_D64_graph_of_64_steps", "steps": d.T,
                 "us_per_step": sec * 1e6 / 64, "tokens_per_s": d.B * 64 / sec})
    print("table:", json.dumps(rows[-1]), file=sys.stderr, flush=True)
    # the same 3072 steps in one launch (tokens known in advance)
    d = wl.CFG5
    q = torch.randn(d.T, d.B, d.H, d.D, device="cuda:0")
    k = torch.randn(d.T, d.B, d.H, d.D, device="cuda:0")
    v = torch.randn(d.T, d.B, d.H, d.M, device="cuda:0")
    S = torch.zeros(d.B, d.H, d.D, d.M, device="cuda:0")
    z = torch.zeros(d.B, d.H, d.D, device="cuda:0")
    out = torch.empty_like(v)
    sec = time_steps(lambda: la.la_recurrent_steps(q, k, v, S, z, out, d.eps), 5, 2, torch)
    rows.append({"workload": f"decode_B{d.B}_H8_D64_{d.T}_steps_one_launch", "steps": d.T,
                 "us_per_step": sec * 1e6 / d.T, "tokens_per_s": d.B * d.T / sec})
    print("table:", json.dumps(rows[-1]), file=sys.stderr, flush=True)
    os.makedirs(os.path.dirname(os.path.abspath(args.table)), exist_ok=True)
    with open(args.table, "w") as f:
        json.dump(rows, f, indent=1)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=65536)
    ap.add_argument("--workload", choices=WORKLOADS, default="headline",
                    help="which workload to step (default: the metric's)")
    ap.add_argument("--groups", type=int, default=0, metavar="G",
                    help="schedule experiment (causal workloads): process the B*H sequences G at a time, "
                         "forward and backward of one group before the next, so that a group's tensors "
                         "could stay in the 256 MB memory-side cache between its kernels")
    ap.add_argument("--table", metavar="PATH", default=None,
                    help="also time the other workloads and write them to PATH (JSON)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a 1 GiB device-to-device copy first (a kernel of known traffic, "
                         "to calibrate rocprofv3's FETCH_SIZE / WRITE_SIZE counters in the same run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    out, obj = run_workload(args)
    del obj
    if args.table:
        run_table(args)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
