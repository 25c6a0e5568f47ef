"""Host-side input recipe: determinism, shapes, and exact bf16 rounding (checked against
torch's own float32 -> bfloat16 conversion as an independent library routine)."""
import numpy as np
import torch

import workloads as wl


def test_shapes_and_determinism():
    Q, K, V, G = wl.qkvg(wl.CFG1)
    assert Q.shape == (1, 1, 256, 32) and V.shape == (1, 1, 256, 32) and Q.dtype == np.float32
    Q2, K2, V2, G2 = wl.qkvg(wl.CFG1)
    assert np.array_equal(Q, Q2) and np.array_equal(G, G2)
    assert not np.array_equal(Q, K)
    w = wl.sweep_point(16)
    assert (w.B, w.H, w.N, w.D, w.M) == (2, 8, 65536, 64, 64)
    assert all(wl.sweep_point(n).B * wl.sweep_point(n).N == 1 << 17 for n in range(9, 17))
    q, k, v = wl.decode_streams(wl.CFG5, T=3)
    assert q.shape == (3, 64, 8, 64) and v.shape == (3, 64, 8, 64)


def test_config3_scaling():
    Q, K, V, G = wl.qkvg(wl.Workload("t", 1, 1, 4096, 64, 64, 3, scale=0.125))
    assert abs(Q.std() - 0.125) < 0.01 and abs(V.std() - 0.125) < 0.01 and abs(G.std() - 1.0) < 0.05


def test_bf16_rounding_matches_library():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(10000).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.0078125, 1.01171875, 3.3895314e38,
                                  1e-40, np.inf, -np.inf], dtype=np.float32)])
    r = wl.round_to_bf16(x)
    t = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(r, t.to(torch.float32).numpy())
    bits = wl.bf16_bits(r)
    assert np.array_equal(bits, t.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(wl.bf16_bits_to_f32(bits), r)


def test_bench_traffic_figures_come_from_the_tracked_profile_summary():
    """bench.py's roofline.traffic is read from the table in profiles/ (no literal to go
    stale), and the measured bytes of every pass kernel equal the tensors it must read and
    write once within a few percent."""
    import bench
    t = bench.measured_traffic_bytes()
    w = wl.HEADLINE
    th = w.B * w.H * w.N
    for k in ("causal_pass_fwd", "pass_dq", "reverse_pass_dv_dk", "segment_state_kv"):
        assert k in t, k
        alg = bench.kernel_bytes(k, w.D, w.M, 4) * th
        assert 0.98 * alg <= t[k] <= 1.08 * alg, (k, t[k], alg)
    assert bench.measured_traffic_bytes("/nonexistent/file.md") == {}
