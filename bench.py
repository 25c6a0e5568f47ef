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


# HBM bytes per launch at the metric's workload, measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# and scaled by a copy kernel of known size (factors 2.000 / 1.000); the runs and their commands are
# in profiles/hbm_traffic_and_pipe_counters_N65536_B2_H8_D64_f32.md.  Read + written, in bytes.
MEASURED_TRAFFIC_BYTES = {
    "causal_pass_fwd": (839.6 + 273.7) * 1e6,
    "pass_dq": (1095.7 + 296.5) * 1e6,
    "reverse_pass_dv_dk": (1101.7 + 536.9) * 1e6,
    "segment_state_kv": (532.8 + 33.8) * 1e6,
    "scan_states": (34.5 + 25.6) * 1e6,
}


def kernel_bytes(name: str, D: int, M: int, e: int) -> float:
    """Algorithmic HBM bytes per token-head of one launch of `name`: the tensors it must
    read and write once (e = bytes per element of the N-sized tensors; den, 1/den and
    delta are fp32 scalars per token-head)."""
    return {
        "causal_pass_fwd": e * (2 * D + 2 * M) + 4,     # Q K V -> O, den
        "pass_dq": e * (3 * D + 2 * M) + 12,            # dO V K Q, den -> dQ, 1/den, delta
        "reverse_pass_dv_dk": e * (3 * D + 3 * M) + 8,  # Q K V dO, 1/den, delta -> dV, dK
        "segment_state_kv": e * (D + M),                # K V
        "global_readout": e * (D + M),                  # Q -> O
    }.get(name, 0.0)


def kernel_flops(name: str, D: int, M: int) -> float:
    """Algorithmic flops per token-head: the state update and the state read-out
    (2*D*(M+1) each, ones column included) that the pass performs."""
    full = 4.0 * D * (M + 1)
    return {"causal_pass_fwd": full, "pass_dq": 1.5 * full, "reverse_pass_dv_dk": 1.5 * full,
            "segment_state_kv": full / 2, "global_readout": full / 2}.get(name, 0.0)


class FwdBwd:
    """Device buffers and the step function for one workload."""

    def __init__(self, w, bf16=False, token_major=False):
        import torch

        import paper_2006_16236_amd as la
        import workloads as wl
        self.la, self.torch, self.w, self.bf16 = la, torch, w, bf16
        dev = "cuda:0"
        host = wl.qkvg(w)
        if bf16:
            host = [wl.round_to_bf16(x) for x in host]
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
        code = la.LA_BF16 if bf16 else la.LA_F32
        nf = la.la_causal_fwd_workspace(w.B, w.H, w.N, w.D, w.M, code)
        nb = la.la_causal_bwd_workspace(w.B, w.H, w.N, w.D, w.M, code)
        self.ws_f = torch.empty(max(nf, 16), dtype=torch.uint8, device=dev)
        self.ws_b = torch.empty(max(nb, 16), dtype=torch.uint8, device=dev)

    def step(self):
        la, w = self.la, self.w
        fwd = la.la_causal_fwd_bnhd if self.token_major else la.la_causal_fwd
        bwd = la.la_causal_bwd_bnhd if self.token_major else la.la_causal_bwd
        fwd(self.Q, self.K, self.V, self.O, self.den, w.eps, ws=self.ws_f)
        bwd(self.Q, self.K, self.V, self.O, self.den, self.G, self.dQ, self.dK,
            self.dV, w.eps, ws=self.ws_b, fwd_ws=self.ws_f)

    def fwd_only(self):
        fwd = self.la.la_causal_fwd_bnhd if self.token_major else self.la.la_causal_fwd
        fwd(self.Q, self.K, self.V, self.O, self.den, self.w.eps, ws=self.ws_f)


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


def cpu_baseline(w, host, sample_tokens):
    """The oracle as it stands (fp64, OpenMP over the (b, h) slabs), forward + backward, on
    the first `sample_tokens` tokens of every slab of the same workload."""
    import numpy as np

    from oracle import la_oracle
    Q, K, V, G = (np.ascontiguousarray(x[:, :, :sample_tokens], dtype=np.float64) for x in host)
    threads = min(la_oracle.max_threads(), w.B * w.H)
    t0 = time.perf_counter()
    la_oracle.causal_fwd_prefix(Q, K, V, w.eps)
    la_oracle.causal_bwd_linear(Q, K, V, G, w.eps)
    dt = time.perf_counter() - t0
    # one thread on one (batch, head) sequence, first 16384 tokens: the per-core rate
    n1 = min(sample_tokens, 16384)
    one = [np.ascontiguousarray(x[:1, :1, :n1]) for x in (Q, K, V, G)]
    nmax = la_oracle.max_threads()
    la_oracle.set_threads(1)
    t1 = time.perf_counter()
    la_oracle.causal_fwd_prefix(*one[:3], w.eps)
    la_oracle.causal_bwd_linear(*one, w.eps)
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


def run_headline(args):
    import torch

    import paper_2006_16236_amd as la
    import workloads as wl

    w = wl.HEADLINE
    fb = FwdBwd(w)
    # clocks settle only after ~50 ms of back-to-back work (see TABLE_WARMUP): when the caller
    # asks for a shorter warm-up, run the difference as well, untimed, and say so in the output
    settle = max(0, SETTLE_STEPS - args.warmup)
    for _ in range(args.warmup + settle):
        fb.step()
    # untimed look at every kernel, to find the dominant one
    prof_all = profile_kernels(la, fb.step, 3, torch)
    per_step = {k: ms * n for k, (ms, n) in prof_all.items()}
    dominant = max(per_step, key=per_step.get)
    kid = [la.la_kernel_name(i) for i in range(la.binding.LA_K_COUNT)].index(dominant)

    # the timed region: exactly `steps` steps, events only around the dominant kernel
    torch.cuda.synchronize()
    la.la_profile_begin(1 << kid)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        fb.step()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    dom_ms, dom_n = la.la_profile_end()[dominant]
    dom_ms /= dom_n

    tokens = w.B * w.N
    th = tokens * w.H
    value = tokens / sec / 1e6
    ach_gbs = kernel_bytes(dominant, w.D, w.M, 4) * th / (dom_ms * 1e-3) / 1e9
    ach_tf = kernel_flops(dominant, w.D, w.M) * th / (dom_ms * 1e-3) / 1e12
    hbm_ceiling = HBM_PEAK_GBS * 1e9 / (w.H * 4 * (6 * w.D + 6 * w.M)) / 1e6
    out = {
        "metric": "causal linear-attn fwd+bwd Mtokens/s (H=8,D=M=64,N=2^16)",
        "value": round(value, 3), "unit": "Mtokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "settle_steps": settle, "ms_per_step": round(sec * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "N": w.N, "D": w.D, "M": w.M,
                   "eps": w.eps, "step": "la_causal_fwd + la_causal_bwd", "seed": w.seed},
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": round(ach_gbs, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach_gbs / HBM_PEAK_GBS, 4),
                     "traffic": MEASURED_TRAFFIC_BYTES.get(dominant), "avg_kernel_ms": round(dom_ms, 4),
                     "mfma_f32_tflops_algorithmic": round(ach_tf, 2),
                     "mfma_f32_frac": round(ach_tf / MFMA_F32_PEAK_TFLOPS, 4)},
        "path_frac_of_hbm_roofline": round(value / hbm_ceiling, 4),
        "path_hbm_ceiling_mtok_s": round(hbm_ceiling, 1),
        "kernels_ms_per_step": {k: round(v, 4) for k, v in sorted(per_step.items(), key=lambda kv: -kv[1])},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, fb.host, args.cpu_sample_tokens)
    return out, fb


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
    out, fb = run_headline(args)
    del fb
    if args.table:
        run_table(args)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
