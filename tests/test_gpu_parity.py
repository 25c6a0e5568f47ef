"""GPU parity: every entry point of the C ABI against the fp64 oracle, element by element,
on the same seeded inputs.  Sizes span several 16-token chunks, several segments and ragged
tails; every schedule of the segment scan is forced in turn."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import (DEV, SCHEDULES, grad_errs, maybe_bf16, rel_err, schedule, to_dev, to_host,
                      tol_for)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def la():
    import paper_2006_16236_amd as la_mod
    assert torch.cuda.is_available()
    return la_mod


def run_fwd(la, Q, K, V, eps, bf16=False, want_den=True):
    dq, dk, dv = (to_dev(x, bf16) for x in (Q, K, V))
    O = torch.full_like(dv, float("nan"))
    den = torch.full(Q.shape[:-1], float("nan"), dtype=torch.float32, device=DEV) if want_den else None
    la.la_causal_fwd(dq, dk, dv, O, den, eps)
    torch.cuda.synchronize()
    return to_host(O), (den.cpu().numpy() if want_den else None)


def run_bwd(la, Q, K, V, G, eps, bf16=False, reuse_fwd=True, reuse_states=True):
    dq, dk, dv, dg = (to_dev(x, bf16) for x in (Q, K, V, G))
    O = den = fwd_ws = None
    if reuse_fwd:
        O = torch.empty_like(dv)
        den = torch.empty(Q.shape[:-1], dtype=torch.float32, device=DEV)
        fwd_ws = la.la_causal_fwd(dq, dk, dv, O, den, eps)
    gq = torch.full_like(dq, float("nan"))
    gk = torch.full_like(dk, float("nan"))
    gv = torch.full_like(dv, float("nan"))
    la.la_causal_bwd(dq, dk, dv, O, den, dg, gq, gk, gv, eps,
                     fwd_ws=fwd_ws if reuse_states else None)
    torch.cuda.synchronize()
    return to_host(gq), to_host(gk), to_host(gv)


EDGE_N = [1, 15, 16, 17, 63, 64, 65, 257, 784, 1000]


@pytest.mark.parametrize("sched", list(SCHEDULES))
@pytest.mark.parametrize("N", EDGE_N)
def test_causal_fwd_edge_lengths(la, oracle, N, sched):
    B, H, D, M = 2, 3, 64, 64
    Q, K, V = wl.random_case(100 + N, B, H, N, D, M)[:3]
    ref, dref = oracle.causal_fwd_prefix(Q, K, V, 1e-6, return_den=True)
    with schedule(**SCHEDULES[sched]):
        O, den = run_fwd(la, Q, K, V, 1e-6)
    assert rel_err(O, ref) <= tol_for(N)
    assert rel_err(den, dref) <= tol_for(N)


@pytest.mark.parametrize("D,M", [(32, 32), (32, 64), (64, 32), (64, 64)])
@pytest.mark.parametrize("sched", ["default", "many_segments", "folded_totals"])
def test_causal_fwd_bwd_all_head_sizes(la, oracle, D, M, sched):
    B, H, N = 2, 2, 203
    Q, K, V, G = wl.random_case(200 + D + 2 * M, B, H, N, D, M)
    eps = 1e-6
    ref = oracle.causal_fwd_prefix(Q, K, V, eps)
    gref = oracle.causal_bwd_linear(Q, K, V, G, eps)
    with schedule(**SCHEDULES[sched]):
        O, _ = run_fwd(la, Q, K, V, eps)
        got = run_bwd(la, Q, K, V, G, eps)
    assert rel_err(O, ref) <= tol_for(N)
    for e, name in zip(grad_errs(got, gref), ("dQ", "dK", "dV")):
        assert e <= tol_for(N), name


@pytest.mark.parametrize("D,M", [(64, 64), (32, 64)])
@pytest.mark.parametrize("sched", ["default", "many_segments"])
def test_elements_of_widely_different_magnitude(la, oracle, D, M, sched):
    """Every tile mixes elements from 2^-10 to 2^10 times a Gaussian.  Part of the fp32 products
    run on bf16 matrix instructions with operands cut into three bf16 pieces; the cut is per
    element, so the accuracy must not depend on how the magnitudes inside a tile compare."""
    B, H, N = 2, 2, 419
    Q, K, V, G = wl.wide_range_case(4242 + D, B, H, N, D, M)
    eps = 1e-6
    ref = oracle.causal_fwd_prefix(Q, K, V, eps)
    gref = oracle.causal_bwd_linear(Q, K, V, G, eps)
    gl_ref = oracle.global_bwd_linear(Q, K, V, G, eps)
    with schedule(**SCHEDULES[sched]):
        O, _ = run_fwd(la, Q, K, V, eps)
        got = run_bwd(la, Q, K, V, G, eps)
        dq, dk, dv, dg = (to_dev(x) for x in (Q, K, V, G))
        Og = torch.empty_like(dv)
        deng = torch.empty(Q.shape[:-1], dtype=torch.float32, device=DEV)
        gws = la.la_global_fwd(dq, dk, dv, Og, eps, den=deng)
        gq, gk, gv = torch.empty_like(dq), torch.empty_like(dk), torch.empty_like(dv)
        la.la_global_bwd(dq, dk, dv, Og, deng, dg, gq, gk, gv, eps, fwd_ws=gws)
        torch.cuda.synchronize()
    assert rel_err(O, ref) <= 1e-5
    for e, name in zip(grad_errs(got, gref), ("dQ", "dK", "dV")):
        assert e <= 1e-5, name
    assert rel_err(to_host(Og), oracle.global_fwd_linear(Q, K, V, eps)) <= 1e-5
    for e, name in zip(grad_errs([to_host(x) for x in (gq, gk, gv)], gl_ref), ("dQ", "dK", "dV")):
        assert e <= 1e-5, "non-causal " + name


def test_elements_of_widely_different_magnitude_bf16(la, oracle):
    """The same kind of input as bf16 tensors (products on 16-bit operands, two bf16 pieces per
    value in the backward): the bf16 gate must hold whatever the spread inside a tile."""
    B, H, N, D, M = 2, 2, 419, 64, 64
    host = maybe_bf16(wl.wide_range_case(4343, B, H, N, D, M, log2_spread=6), True)
    Q, K, V, G = host
    eps = 1e-6
    ref = oracle.causal_fwd_prefix(Q, K, V, eps)
    gref = oracle.causal_bwd_linear(Q, K, V, G, eps)
    with schedule(**SCHEDULES["many_segments"]):
        O, _ = run_fwd(la, Q, K, V, eps, bf16=True)
        got = run_bwd(la, Q, K, V, G, eps, bf16=True)
    assert rel_err(O, ref) <= tol_for(N, True)
    for e, name in zip(grad_errs(got, gref), ("dQ", "dK", "dV")):
        assert e <= tol_for(N, True), name


@pytest.mark.parametrize("sched", list(SCHEDULES))
@pytest.mark.parametrize("N", EDGE_N)
def test_causal_bwd_edge_lengths(la, oracle, N, sched):
    B, H, D, M = 1, 3, 64, 64
    Q, K, V, G = wl.random_case(300 + N, B, H, N, D, M)
    gref = oracle.causal_bwd_linear(Q, K, V, G, 1e-6)
    with schedule(**SCHEDULES[sched]):
        got = run_bwd(la, Q, K, V, G, 1e-6)
    for e, name in zip(grad_errs(got, gref), ("dQ", "dK", "dV")):
        assert e <= tol_for(N), name


def test_causal_bwd_recomputes_forward_when_not_given(la, oracle):
    B, H, N, D, M = 2, 2, 333, 64, 64
    Q, K, V, G = wl.random_case(401, B, H, N, D, M)
    gref = oracle.causal_bwd_linear(Q, K, V, G, 1e-6)
    for sched in ("default", "many_segments"):
        with schedule(**SCHEDULES[sched]):
            a = run_bwd(la, Q, K, V, G, 1e-6, reuse_fwd=False)
            b = run_bwd(la, Q, K, V, G, 1e-6, reuse_fwd=True)
            c = run_bwd(la, Q, K, V, G, 1e-6, reuse_fwd=True, reuse_states=False)
        assert all(np.array_equal(x, y) for x, y in zip(a, b))
        assert all(np.array_equal(x, y) for x, y in zip(a, c))
        assert max(grad_errs(a, gref)) <= tol_for(N)


@pytest.mark.parametrize("eps", [0.0, 1e-6, 0.5])
def test_eps_values(la, oracle, eps):
    B, H, N, D, M = 1, 2, 100, 32, 32
    Q, K, V, G = wl.random_case(402, B, H, N, D, M)
    ref = oracle.causal_fwd_prefix(Q, K, V, eps)
    gref = oracle.causal_bwd_linear(Q, K, V, G, eps)
    O, _ = run_fwd(la, Q, K, V, eps)
    assert rel_err(O, ref) <= tol_for(N)
    assert max(grad_errs(run_bwd(la, Q, K, V, G, eps), gref)) <= tol_for(N)


@pytest.mark.parametrize("sched", ["default", "one_segment", "many_segments", "folded_totals"])
@pytest.mark.parametrize("N", [1, 17, 64, 257, 1000])
def test_global_fwd(la, oracle, N, sched):
    B, H, D, M = 2, 2, 64, 64
    Q, K, V = wl.random_case(500 + N, B, H, N, D, M)[:3]
    ref = oracle.global_fwd_linear(Q, K, V, 1e-6)
    dq, dk, dv = (to_dev(x) for x in (Q, K, V))
    O = torch.full_like(dv, float("nan"))
    with schedule(**SCHEDULES[sched]):
        la.la_global_fwd(dq, dk, dv, O, 1e-6)
    torch.cuda.synchronize()
    assert rel_err(to_host(O), ref) <= tol_for(N)


def run_global(la, Q, K, V, G, eps, bf16=False, reuse_fwd=True, reuse_states=True):
    """Non-causal forward (with den) and backward; returns O, den, (dQ, dK, dV) on the host."""
    dq, dk, dv, dg = (to_dev(x, bf16) for x in (Q, K, V, G))
    O = torch.full_like(dv, float("nan"))
    den = torch.full(Q.shape[:-1], float("nan"), dtype=torch.float32, device=DEV)
    fwd_ws = la.la_global_fwd(dq, dk, dv, O, eps, den=den)
    gq = torch.full_like(dq, float("nan"))
    gk = torch.full_like(dk, float("nan"))
    gv = torch.full_like(dv, float("nan"))
    la.la_global_bwd(dq, dk, dv, O if reuse_fwd else None, den if reuse_fwd else None, dg, gq, gk,
                     gv, eps, fwd_ws=fwd_ws if reuse_states else None)
    torch.cuda.synchronize()
    return to_host(O), den.cpu().numpy(), (to_host(gq), to_host(gk), to_host(gv))


@pytest.mark.parametrize("B,H,N,D,M,sched,eps", [(3, 4, 14, 32, 32, "one_segment", 1e-3),
                                                  (2, 2, 593, 32, 64, "default", 0.0),
                                                  (1, 4, 3793, 32, 64, "many_segments", 1e-6)])
def test_bf16_backward_on_small_inputs(la, oracle, B, H, N, D, M, sched, eps):
    """bf16 tensors scaled by 1/8: the features are 1 + (something small) and the gradients with
    respect to Q are differences of nearly equal terms.  The sums over K, V that the backward
    passes start from must then be good to more than bf16's 8 bits: with plain bf16 products in
    them these cases sat at 1.4e-2 .. 2.04e-2."""
    host = maybe_bf16(wl.random_case(50000 + N, B, H, N, D, M, scale=0.125), True)
    Q, K, V, G = host
    with schedule(**SCHEDULES[sched]):
        grads = run_bwd(la, Q, K, V, G, eps, bf16=True)
        _, _, ggrads = run_global(la, Q, K, V, G, eps, bf16=True)
    for e, name in zip(grad_errs(grads, oracle.causal_bwd_linear(Q, K, V, G, eps)), ("dQ", "dK", "dV")):
        assert e <= 1e-2, name
    for e, name in zip(grad_errs(ggrads, oracle.global_bwd_linear(Q, K, V, G, eps)), ("dQ", "dK", "dV")):
        assert e <= 1e-2, "non-causal " + name


@pytest.mark.parametrize("sched", ["default", "one_segment", "many_segments", "folded_totals"])
@pytest.mark.parametrize("N", [1, 15, 16, 17, 64, 257, 1000])
def test_global_bwd_edge_lengths(la, oracle, N, sched):
    B, H, D, M = 2, 2, 64, 64
    Q, K, V, G = wl.random_case(520 + N, B, H, N, D, M)
    gref = oracle.global_bwd_linear(Q, K, V, G, 1e-6)
    with schedule(**SCHEDULES[sched]):
        O, den, grads = run_global(la, Q, K, V, G, 1e-6)
    assert rel_err(O, oracle.global_fwd_linear(Q, K, V, 1e-6)) <= tol_for(N)
    # the denominator of eq. 5-6: phi(Q_i) . sum_j phi(K_j) + eps, here from the oracle's phi
    dref = np.einsum("bhnd,bhd->bhn", oracle.phi(Q), oracle.phi(K).sum(axis=2)) + 1e-6
    assert rel_err(den, dref) <= tol_for(N)
    assert max(grad_errs(grads, gref)) <= tol_for(N)


@pytest.mark.parametrize("D,M", [(32, 32), (32, 64), (64, 32)])
@pytest.mark.parametrize("reuse", ["all", "no_states", "recompute"])
def test_global_bwd_head_sizes_and_recompute(la, oracle, D, M, reuse):
    B, H, N = 1, 3, 333
    Q, K, V, G = wl.random_case(560 + D + 2 * M, B, H, N, D, M)
    gref = oracle.global_bwd_linear(Q, K, V, G, 1e-6)
    with schedule(**SCHEDULES["three_chunk_segments"]):
        _, _, grads = run_global(la, Q, K, V, G, 1e-6, reuse_fwd=reuse != "recompute",
                                 reuse_states=reuse == "all")
    assert max(grad_errs(grads, gref)) <= tol_for(N)


def test_global_bwd_quadratic_definition_and_bf16(la, oracle):
    B, H, N, D, M = 1, 2, 200, 64, 64
    Q, K, V, G = wl.random_case(590, B, H, N, D, M)
    gref = oracle.global_bwd_quadratic(Q, K, V, G, 1e-6)
    _, _, grads = run_global(la, Q, K, V, G, 1e-6)
    assert max(grad_errs(grads, gref)) <= tol_for(N)
    Qb, Kb, Vb, Gb = (wl.round_to_bf16(x) for x in (Q, K, V, G))
    gref = oracle.global_bwd_linear(Qb, Kb, Vb, Gb, 1e-6)
    _, _, grads = run_global(la, Qb, Kb, Vb, Gb, 1e-6, bf16=True)
    assert max(grad_errs(grads, gref)) <= tol_for(N, bf16=True)


@pytest.mark.parametrize("D,M", [(32, 32), (32, 64), (64, 32), (64, 64)])
def test_recurrent_steps_against_oracle_and_causal_fwd(la, oracle, D, M):
    B, H, T = 3, 2, 40
    w = wl.DecodeWorkload("t", B, H, D, M, T, 600 + D + 2 * M)
    q, k, v = wl.decode_streams(w)
    S = torch.zeros(B, H, D, M, device=DEV)
    z = torch.zeros(B, H, D, device=DEV)
    dq, dk, dv = (to_dev(x) for x in (q, k, v))
    out = torch.empty(T, B, H, M, device=DEV)
    for t in range(T):
        la.la_recurrent_step(dq[t], dk[t], dv[t], S, z, out[t], 1e-6)
    torch.cuda.synchronize()
    So = np.zeros((B, H, D, M)); zo = np.zeros((B, H, D))
    ref = np.stack([oracle.recurrent_step(q[t], k[t], v[t], So, zo, 1e-6) for t in range(T)])
    assert rel_err(to_host(out), ref) <= 1e-4
    assert rel_err(S.cpu().numpy(), So) <= 1e-4
    assert rel_err(z.cpu().numpy(), zo) <= 1e-4
    # the same tokens stacked as one sequence through the parallel kernel (eq. 12 == eq. 20)
    Qs, Ks, Vs = (np.ascontiguousarray(np.moveaxis(x, 0, 2)) for x in (q, k, v))
    O, _ = run_fwd(la, Qs, Ks, Vs, 1e-6)
    assert rel_err(O, np.moveaxis(ref, 0, 2)) <= 1e-4


def test_entry_points_under_hip_graph_capture(la):
    """The entry points only enqueue kernels on the caller's stream (no allocation, no memset,
    no synchronisation), so they can be recorded into a HIP graph.  A graph of 8 decode steps
    plus a causal forward + backward is replayed several times, with eager work and
    synchronisations in between, and every replay must equal the eager result bit for bit."""
    B, H, T, N, D, M = 4, 2, 8, 300, 64, 64
    w = wl.DecodeWorkload("g", B, H, D, M, 4 * T, 660)
    q, k, v = (to_dev(x) for x in wl.decode_streams(w))
    Q, K, V, G = (to_dev(x) for x in wl.random_case(661, B, H, N, D, M))
    # static buffers of the graph
    qs, ks, vs = torch.empty_like(q[:T]), torch.empty_like(k[:T]), torch.empty_like(v[:T])
    S = torch.zeros(B, H, D, M, device=DEV); z = torch.zeros(B, H, D, device=DEV)
    outs = torch.empty(T, B, H, M, device=DEV)
    O = torch.empty_like(V); den = torch.empty(B, H, N, device=DEV)
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    ws_f = torch.empty(max(la.la_causal_fwd_workspace(B, H, N, D, M), 16), dtype=torch.uint8, device=DEV)
    ws_b = torch.empty(la.la_causal_bwd_workspace(B, H, N, D, M), dtype=torch.uint8, device=DEV)

    def work():
        for t in range(T):
            la.la_recurrent_step(qs[t], ks[t], vs[t], S, z, outs[t], 1e-6)
        la.la_causal_fwd(Q, K, V, O, den, 1e-6, ws=ws_f)
        la.la_causal_bwd(Q, K, V, None, den, G, dQ, dK, dV, 1e-6, ws=ws_b, fwd_ws=ws_f)

    # eager reference: four rounds of T steps, the state carried across rounds
    S_e = torch.zeros_like(S); z_e = torch.zeros_like(z)
    eager_outs = []
    for r in range(4):
        o = torch.empty(T, B, H, M, device=DEV)
        for t in range(T):
            la.la_recurrent_step(q[r * T + t], k[r * T + t], v[r * T + t], S_e, z_e, o[t], 1e-6)
        eager_outs.append(o)
    work()                                             # warm-up on static buffers, also gives
    torch.cuda.synchronize()                           # the eager forward / backward results
    ref = [x.clone() for x in (O, den, dQ, dK, dV)]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        work()
    S.zero_(); z.zero_()
    for r in range(4):
        qs.copy_(q[r * T:(r + 1) * T]); ks.copy_(k[r * T:(r + 1) * T]); vs.copy_(v[r * T:(r + 1) * T])
        for x in (O, den, dQ, dK, dV):
            x.fill_(float("nan"))                      # eager work between the replays
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(outs, eager_outs[r]), r
        assert all(torch.equal(a, b) for a, b in zip((O, den, dQ, dK, dV), ref)), r
    assert torch.equal(S, S_e) and torch.equal(z, z_e)


@pytest.mark.parametrize("D,M", [(32, 32), (32, 64), (64, 32), (64, 64)])
@pytest.mark.parametrize("bf16", [False, True])
def test_multi_step_decode_equals_single_steps_bit_for_bit(la, oracle, D, M, bf16):
    B, H, T = 2, 3, 37
    w = wl.DecodeWorkload("t", B, H, D, M, T, 650 + D + 2 * M)
    q, k, v = maybe_bf16(wl.decode_streams(w), bf16)
    dq, dk, dv = (to_dev(x, bf16) for x in (q, k, v))
    S1 = torch.zeros(B, H, D, M, device=DEV); z1 = torch.zeros(B, H, D, device=DEV)
    out1 = torch.empty_like(dv)
    for t in range(T):
        la.la_recurrent_step(dq[t], dk[t], dv[t], S1, z1, out1[t], 1e-6)
    S2 = torch.zeros_like(S1); z2 = torch.zeros_like(z1); out2 = torch.full_like(dv, float("nan"))
    la.la_recurrent_steps(dq[:20], dk[:20], dv[:20], S2, z2, out2[:20], 1e-6)     # two launches:
    la.la_recurrent_steps(dq[20:], dk[20:], dv[20:], S2, z2, out2[20:], 1e-6)     # the state carries over
    torch.cuda.synchronize()
    assert torch.equal(out1, out2) and torch.equal(S1, S2) and torch.equal(z1, z2)
    So = np.zeros((B, H, D, M)); zo = np.zeros((B, H, D))
    ref = np.stack([oracle.recurrent_step(q[t], k[t], v[t], So, zo, 1e-6) for t in range(T)])
    assert rel_err(to_host(out2), ref) <= (2e-2 if bf16 else 1e-4)
    assert rel_err(S2.cpu().numpy(), So) <= 1e-4


@pytest.mark.parametrize("sched", ["default", "many_segments", "folded_totals"])
def test_bf16_tensors_fp32_state(la, oracle, sched):
    B, H, N, D, M = 2, 2, 300, 64, 64
    Q, K, V, G = maybe_bf16(wl.random_case(700, B, H, N, D, M, scale=0.125), True)
    eps = 1e-6
    ref = oracle.causal_fwd_prefix(Q, K, V, eps)
    with schedule(**SCHEDULES[sched]):
        O, _ = run_fwd(la, Q, K, V, eps, bf16=True)
        got = run_bwd(la, Q, K, V, G, eps, bf16=True)
    assert rel_err(O, ref) <= tol_for(N, True)
    # the backward consumes the bf16-rounded O of the forward, as a training step would
    gref = oracle.causal_bwd_linear(Q, K, V, G, eps)
    for e, name in zip(grad_errs(got, gref), ("dQ", "dK", "dV")):
        assert e <= tol_for(N, True), name


@pytest.mark.parametrize("sched", ["default", "one_segment", "many_segments", "folded_totals"])
def test_forward_with_state_in_and_out(la, oracle, sched):
    """A sequence processed in two pieces through la_causal_fwd_state, then continued token by
    token with la_recurrent_step, reproduces the one-shot causal forward (eq. 12 == eq. 20)."""
    B, H, D, M = 2, 2, 64, 32
    N1, N2, N3 = 150, 333, 5
    N = N1 + N2 + N3
    Q, K, V = wl.random_case(900, B, H, N, D, M)[:3]
    ref = oracle.causal_fwd_prefix(Q, K, V, 1e-6)
    dq, dk, dv = (to_dev(x) for x in (Q, K, V))
    O = torch.full_like(dv, float("nan"))
    Sa = torch.empty(B, H, D, M, device=DEV); za = torch.empty(B, H, D, device=DEV)
    Sb = torch.empty_like(Sa); zb = torch.empty_like(za)
    piece = lambda t, a, b: t[:, :, a:b].contiguous()
    with schedule(**SCHEDULES[sched]):
        O1 = torch.empty(B, H, N1, M, device=DEV)
        la.la_causal_fwd_state(piece(dq, 0, N1), piece(dk, 0, N1), piece(dv, 0, N1), O1, None,
                               None, None, Sa, za, 1e-6)
        O2 = torch.empty(B, H, N2, M, device=DEV)
        la.la_causal_fwd_state(piece(dq, N1, N1 + N2), piece(dk, N1, N1 + N2), piece(dv, N1, N1 + N2),
                               O2, None, Sa, za, Sb, zb, 1e-6)
    O3 = torch.empty(B, H, N3, M, device=DEV)
    for t in range(N3):
        i = N1 + N2 + t
        step_out = torch.empty(B, H, M, device=DEV)
        la.la_recurrent_step(dq[:, :, i].contiguous(), dk[:, :, i].contiguous(),
                             dv[:, :, i].contiguous(), Sb, zb, step_out, 1e-6)
        O3[:, :, t] = step_out
    torch.cuda.synchronize()
    got = np.concatenate([to_host(O1), to_host(O2), to_host(O3)], axis=2)
    assert rel_err(got, ref) <= 1e-4
    fk = oracle.phi(K.astype(np.float64))
    assert rel_err(Sb.cpu().numpy(), np.einsum("bhnd,bhnm->bhdm", fk, V.astype(np.float64))) <= 1e-4
    assert rel_err(zb.cpu().numpy(), fk.sum(2)) <= 1e-4


@pytest.mark.parametrize("group", [1, 2])
@pytest.mark.parametrize("D,M", [(32, 32), (64, 64), (64, 32)])
@pytest.mark.parametrize("cut", ["scanned", "folded"])
def test_backward_takes_segments_singly_or_in_pairs(la, oracle, D, M, group, cut):
    """The backward's workgroups take the forward's segments one by one (the default at
    D = M = 32) or in pairs (the default otherwise): both groupings, for either head size, on
    scanned and on folded segment totals, causal and non-causal, against the oracle."""
    B, H, N = 2, 2, 1000
    Q, K, V, G = wl.random_case(990 + D + M, B, H, N, D, M)
    ref = oracle.causal_bwd_linear(Q, K, V, G, 1e-6)
    gref = oracle.global_bwd_linear(Q, K, V, G, 1e-6)
    dq, dk, dv, dg = (to_dev(x) for x in (Q, K, V, G))
    kw = dict(target_waves=1 << 20, min_seg_chunks=3) if cut == "scanned" else dict(target_waves=24, min_seg_chunks=1, fold_max_segs=64)
    with schedule(bwd_seg_group=group, **kw):
        O = torch.empty_like(dv); den = torch.empty(B, H, N, device=DEV)
        ws = la.la_causal_fwd(dq, dk, dv, O, den, 1e-6)
        got = [torch.full_like(x, float("nan")) for x in (dq, dk, dv)]
        la.la_causal_bwd(dq, dk, dv, None, den, dg, got[0], got[1], got[2], 1e-6, fwd_ws=ws)
        Og = torch.empty_like(dv); deng = torch.empty(B, H, N, device=DEV)
        wsg = la.la_global_fwd(dq, dk, dv, Og, 1e-6, den=deng)
        ggot = [torch.full_like(x, float("nan")) for x in (dq, dk, dv)]
        la.la_global_bwd(dq, dk, dv, None, deng, dg, ggot[0], ggot[1], ggot[2], 1e-6, fwd_ws=wsg)
        torch.cuda.synchronize()
    assert max(grad_errs([to_host(x) for x in got], ref)) <= tol_for(N)
    assert max(grad_errs([to_host(x) for x in ggot], gref)) <= tol_for(N)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("D,M", [(32, 32), (64, 64)])
def test_non_temporal_loads_change_no_bit(la, oracle, D, M, bf16):
    """LA_STREAM_LOADS=1 makes every kernel fetch its tiles with non-temporal loads (plain loads
    are the default): the same values arrive, so causal and non-causal forward and backward must
    come out bit for bit the same, and equal to the oracle's within the gate; ragged length,
    several segments per sequence."""
    B, H, N = 2, 2, 1000
    host = maybe_bf16(wl.random_case(7100 + D, B, H, N, D, M, scale=0.5 if bf16 else 1.0), bf16)
    Q, K, V, G = host
    ref_o = oracle.causal_fwd_prefix(Q, K, V, 1e-6)
    ref_g = oracle.causal_bwd_linear(Q, K, V, G, 1e-6)
    gref = oracle.global_bwd_linear(Q, K, V, G, 1e-6)
    res = []
    for nt in (0, 1):
        with schedule(target_waves=1 << 20, min_seg_chunks=3, stream_loads=nt):
            O, den = run_fwd(la, Q, K, V, 1e-6, bf16=bf16)
            grads = run_bwd(la, Q, K, V, G, 1e-6, bf16=bf16)
            Og, deng, ggrads = run_global(la, Q, K, V, G, 1e-6, bf16=bf16)
        res.append([O, den, *grads, Og, deng, *ggrads])
    for a, b in zip(*res):
        assert np.array_equal(a, b)
    O, den, gq, gk, gv, Og, deng, hq, hk, hv = res[1]
    assert rel_err(O, ref_o) <= tol_for(N, bf16)
    assert max(grad_errs((gq, gk, gv), ref_g)) <= tol_for(N, bf16)
    assert max(grad_errs((hq, hk, hv), gref)) <= tol_for(N, bf16)


def _state_case(seed, B, H, N, D, M):
    """Inputs plus a non-zero initial state and a non-zero gradient arriving at the final state
    (the state is that of P imaginary earlier tokens: positive z0, S0 of matching size)."""
    Q, K, V, G = wl.random_case(seed, B, H, N, D, M)
    rng = np.random.default_rng(seed + 7)
    S0 = (rng.standard_normal((B, H, D, M)) * 3.0).astype(np.float32)
    z0 = rng.uniform(2.0, 9.0, (B, H, D)).astype(np.float32)
    dS1 = (rng.standard_normal((B, H, D, M)) * 0.5).astype(np.float32)
    dz1 = (rng.standard_normal((B, H, D)) * 0.5).astype(np.float32)
    return Q, K, V, G, S0, z0, dS1, dz1


def _gpu_bwd_state(la, Q, K, V, G, S0, z0, dS1, dz1, eps, reuse="all", want_state_grad=True):
    dq, dk, dv, dg = (to_dev(x) for x in (Q, K, V, G))
    s0, zz0, ds1, dzz1 = (None if x is None else to_dev(x) for x in (S0, z0, dS1, dz1))
    B, H, N, D = Q.shape
    M = V.shape[-1]
    O = torch.empty_like(dv)
    den = torch.empty(B, H, N, device=DEV)
    fwd_ws = la.la_causal_fwd_state(dq, dk, dv, O, den, s0, zz0, None, None, eps)
    gq, gk, gv = (torch.full_like(x, float("nan")) for x in (dq, dk, dv))
    ds0 = torch.full((B, H, D, M), float("nan"), device=DEV) if want_state_grad else None
    dzz0 = torch.full((B, H, D), float("nan"), device=DEV) if want_state_grad else None
    la.la_causal_bwd_state(dq, dk, dv, O if reuse != "recompute" else None,
                           den if reuse != "recompute" else None, dg, gq, gk, gv, s0, zz0, ds1, dzz1,
                           ds0, dzz0, eps, fwd_ws=fwd_ws if reuse == "all" else None)
    torch.cuda.synchronize()
    out = [to_host(gq), to_host(gk), to_host(gv)]
    if want_state_grad:
        out += [ds0.cpu().numpy(), dzz0.cpu().numpy()]
    return out


@pytest.mark.parametrize("sched", list(SCHEDULES))
@pytest.mark.parametrize("N", [1, 16, 17, 100, 257, 1000])
def test_backward_with_state_gradient_in_and_out(la, oracle, N, sched):
    B, H, D, M = 2, 2, 64, 64
    Q, K, V, G, S0, z0, dS1, dz1 = _state_case(930 + N, B, H, N, D, M)
    ref = oracle.causal_bwd_state(Q, K, V, G, S0, z0, dS1, dz1, 1e-6)
    with schedule(**SCHEDULES[sched]):
        got = _gpu_bwd_state(la, Q, K, V, G, S0, z0, dS1, dz1, 1e-6)
    assert max(grad_errs(got[:3], ref[:3])) <= tol_for(N)
    assert rel_err(got[3], ref[3]) <= tol_for(N)
    assert rel_err(got[4], ref[4]) <= tol_for(N)


@pytest.mark.parametrize("D,M", [(32, 32), (32, 64), (64, 32)])
@pytest.mark.parametrize("reuse", ["all", "no_states", "recompute"])
def test_backward_with_state_head_sizes_and_recompute(la, oracle, D, M, reuse):
    B, H, N = 1, 3, 333
    Q, K, V, G, S0, z0, dS1, dz1 = _state_case(960 + D + 2 * M, B, H, N, D, M)
    ref = oracle.causal_bwd_state(Q, K, V, G, S0, z0, dS1, dz1, 1e-6)
    for sched in ("one_segment", "three_chunk_segments"):
        with schedule(**SCHEDULES[sched]):
            got = _gpu_bwd_state(la, Q, K, V, G, S0, z0, dS1, dz1, 1e-6, reuse=reuse)
        assert max(grad_errs(got[:3], ref[:3])) <= tol_for(N), sched
        assert rel_err(got[3], ref[3]) <= tol_for(N) and rel_err(got[4], ref[4]) <= tol_for(N), sched


@pytest.mark.parametrize("sched", ["default", "one_segment", "many_segments", "folded_totals"])
def test_backward_chained_over_two_pieces_equals_the_uncut_sequence(la, oracle, sched):
    """Forward piece by piece through the state, backward piece by piece in reverse through the
    state gradient: the gradients equal those of the uncut sequence (oracle: Algorithm 1 backward
    on the whole sequence, which knows nothing of pieces)."""
    B, H, D, M = 2, 2, 64, 64
    N1, N2 = 200, 350
    Q, K, V, G = wl.random_case(990, B, H, N1 + N2, D, M)
    ref = oracle.causal_bwd_linear(Q, K, V, G, 1e-6)
    a = [np.ascontiguousarray(x[:, :, :N1]) for x in (Q, K, V, G)]
    b = [np.ascontiguousarray(x[:, :, N1:]) for x in (Q, K, V, G)]
    with schedule(**SCHEDULES[sched]):
        da = [to_dev(x) for x in a[:3]]
        Oa = torch.empty_like(da[2])
        Sa = torch.empty(B, H, D, M, device=DEV); za = torch.empty(B, H, D, device=DEV)
        la.la_causal_fwd_state(*da, Oa, None, None, None, Sa, za, 1e-6)
        torch.cuda.synchronize()
        gb = _gpu_bwd_state(la, *b, Sa.cpu().numpy(), za.cpu().numpy(), None, None, 1e-6)
        ga = _gpu_bwd_state(la, *a, None, None, gb[3], gb[4], 1e-6, want_state_grad=False)
    got = [np.concatenate([x, y], axis=2) for x, y in zip(ga[:3], gb[:3])]
    assert max(grad_errs(got, ref)) <= tol_for(N1 + N2)


@pytest.mark.parametrize("sched", ["default", "one_segment", "three_chunk_segments"])
def test_backward_needs_den_but_not_O(la, oracle, sched):
    """The backward rebuilds dO.O from its own read-out: O may be NULL, or hold anything."""
    B, H, N, D, M = 2, 2, 300, 64, 64
    Q, K, V, G = wl.random_case(995, B, H, N, D, M)
    gref = oracle.causal_bwd_linear(Q, K, V, G, 1e-6)
    ggref = oracle.global_bwd_linear(Q, K, V, G, 1e-6)
    dq, dk, dv, dg = (to_dev(x) for x in (Q, K, V, G))
    with schedule(**SCHEDULES[sched]):
        O = torch.empty_like(dv)
        den = torch.empty(B, H, N, device=DEV)
        fwd_ws = la.la_causal_fwd(dq, dk, dv, O, den, 1e-6)
        junk = torch.full_like(dv, float("nan"))
        for o_arg in (None, junk):
            gq, gk, gv = (torch.full_like(x, float("nan")) for x in (dq, dk, dv))
            la.la_causal_bwd(dq, dk, dv, o_arg, den, dg, gq, gk, gv, 1e-6, fwd_ws=fwd_ws)
            torch.cuda.synchronize()
            assert max(grad_errs([to_host(gq), to_host(gk), to_host(gv)], gref)) <= tol_for(N)
        gws = la.la_global_fwd(dq, dk, dv, O, 1e-6, den=den)
        gq, gk, gv = (torch.full_like(x, float("nan")) for x in (dq, dk, dv))
        la.la_global_bwd(dq, dk, dv, None, den, dg, gq, gk, gv, 1e-6, fwd_ws=gws)
        torch.cuda.synchronize()
        assert max(grad_errs([to_host(gq), to_host(gk), to_host(gv)], ggref)) <= tol_for(N)


@pytest.mark.parametrize("causal", [True, False])
def test_autograd_front_end(la, oracle, causal):
    """The torch.autograd wrappers run the library's forward and backward: loss = sum(G * O)."""
    B, H, N, D, M = 2, 2, 333, 64, 32
    Q, K, V, G = wl.random_case(997, B, H, N, D, M)
    tq, tk, tv = (to_dev(x).requires_grad_(True) for x in (Q, K, V))
    fn = la.causal_linear_attention if causal else la.linear_attention
    O = fn(tq, tk, tv, 1e-6)
    (O * to_dev(G)).sum().backward()
    torch.cuda.synchronize()
    if causal:
        ref, gref = oracle.causal_fwd_prefix(Q, K, V, 1e-6), oracle.causal_bwd_linear(Q, K, V, G, 1e-6)
    else:
        ref, gref = oracle.global_fwd_linear(Q, K, V, 1e-6), oracle.global_bwd_linear(Q, K, V, G, 1e-6)
    assert rel_err(to_host(O), ref) <= tol_for(N)
    assert max(grad_errs([to_host(t.grad) for t in (tq, tk, tv)], gref)) <= tol_for(N)


def _random_shapes(count, seed):
    rng = np.random.default_rng(seed)
    sched_names = list(SCHEDULES)
    for i in range(count):
        yield (int(rng.integers(1, 4)), int(rng.integers(1, 5)), int(rng.integers(1, 700)),
               int(rng.choice([32, 64])), int(rng.choice([32, 64])),
               sched_names[int(rng.integers(len(sched_names)))], float(rng.choice([0.0, 1e-6, 1e-2])),
               2000 + i)


@pytest.mark.parametrize("B,H,N,D,M,sched,eps,seed", list(_random_shapes(24, 31337)))
def test_random_shapes_all_entry_points(la, oracle, B, H, N, D, M, sched, eps, seed):
    """Seeded random sizes, head widths, schedules and eps: causal forward + backward (with a
    state handed in and out) and the non-causal pair, each against the oracle."""
    Q, K, V, G, S0, z0, dS1, dz1 = _state_case(seed, B, H, N, D, M)
    tol = tol_for(N)
    with schedule(**SCHEDULES[sched]):
        O, den = run_fwd(la, Q, K, V, eps)
        grads = run_bwd(la, Q, K, V, G, eps)
        gs = _gpu_bwd_state(la, Q, K, V, G, S0, z0, dS1, dz1, eps)
        Og, deng, gg = run_global(la, Q, K, V, G, eps)
    ref, dref = oracle.causal_fwd_prefix(Q, K, V, eps, return_den=True)
    assert rel_err(O, ref) <= tol and rel_err(den, dref) <= tol
    assert max(grad_errs(grads, oracle.causal_bwd_linear(Q, K, V, G, eps))) <= tol
    rs = oracle.causal_bwd_state(Q, K, V, G, S0, z0, dS1, dz1, eps)
    assert max(grad_errs(gs[:3], rs[:3])) <= tol
    assert rel_err(gs[3], rs[3]) <= tol and rel_err(gs[4], rs[4]) <= tol
    assert rel_err(Og, oracle.global_fwd_linear(Q, K, V, eps)) <= tol
    assert max(grad_errs(gg, oracle.global_bwd_linear(Q, K, V, G, eps))) <= tol


# ---- token-major tensors [B, N, H, .] --------------------------------------------------------

def _token_major(x, bf16=False):
    """[B, H, N, F] host array -> contiguous [B, N, H, F] device tensor."""
    return to_dev(np.ascontiguousarray(np.transpose(x, (0, 2, 1, 3))), bf16)


def _head_major(t):
    return to_host(t).transpose(0, 2, 1, 3)


@pytest.mark.parametrize("B,H,N,D,M,bf16,sched,reuse", [
    (2, 3, 333, 64, 64, False, "default", "all"),
    (1, 8, 1000, 64, 32, False, "many_segments", "den"),
    (3, 2, 77, 32, 64, False, "three_chunk_segments", "none"),
    (2, 5, 16, 32, 32, False, "one_segment", "all"),
    (2, 1, 129, 64, 64, False, "default", "all"),
    (2, 4, 500, 64, 64, True, "default", "all"),
    (1, 6, 47, 32, 64, True, "many_segments", "den"),
])
def test_token_major_layout(la, oracle, B, H, N, D, M, bf16, sched, reuse):
    """la_causal_fwd_bnhd / la_causal_bwd_bnhd on [B, N, H, .] tensors: against the oracle, and
    bit for bit against the [B, H, N, .] entry points (same arithmetic, other addresses)."""
    host = maybe_bf16(wl.random_case(8800 + N, B, H, N, D, M), bf16)
    Q, K, V, G = host
    eps = 1e-6
    tq, tk, tv, tg = (_token_major(x, bf16) for x in host)
    with schedule(**SCHEDULES[sched]):
        O = torch.full_like(tv, float("nan"))
        den = torch.full((B, H, N), float("nan"), dtype=torch.float32, device=DEV)
        ws = la.la_causal_fwd_bnhd(tq, tk, tv, O, den, eps)
        gq, gk, gv = (torch.full_like(x, float("nan")) for x in (tq, tk, tv))
        la.la_causal_bwd_bnhd(tq, tk, tv, None, den if reuse != "none" else None, tg, gq, gk, gv, eps,
                              fwd_ws=ws if reuse == "all" else None)
        torch.cuda.synchronize()
        O2, den2 = run_fwd(la, Q, K, V, eps, bf16=bf16)
        g2 = run_bwd(la, Q, K, V, G, eps, bf16=bf16, reuse_fwd=reuse != "none",
                     reuse_states=reuse == "all")
    tol = tol_for(N, bf16)
    ref, dref = oracle.causal_fwd_prefix(Q, K, V, eps, return_den=True)
    assert rel_err(_head_major(O), ref) <= tol and rel_err(den.cpu().numpy(), dref) <= tol
    got = [_head_major(x) for x in (gq, gk, gv)]
    assert max(grad_errs(got, oracle.causal_bwd_linear(Q, K, V, G, eps))) <= tol
    assert np.array_equal(_head_major(O), O2) and np.array_equal(den.cpu().numpy(), den2)
    for a, b in zip(got, g2):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("B,H,N,D,M,sched", [(2, 3, 333, 64, 64, "default"), (1, 4, 1000, 32, 64, "many_segments"),
                                             (2, 2, 100, 64, 32, "folded_totals"), (3, 2, 16, 32, 32, "one_segment")])
def test_token_major_layout_with_state(la, oracle, B, H, N, D, M, sched):
    """la_causal_fwd_state_bnhd / la_causal_bwd_state_bnhd: state in and out on [B, N, H, .]
    tensors, against the oracle and bit for bit against the [B, H, N, .] entry points."""
    Q, K, V, G, S0, z0, dS1, dz1 = _state_case(9900 + N, B, H, N, D, M)
    eps = 1e-6
    tq, tk, tv, tg = (_token_major(x, False) for x in (Q, K, V, G))
    s0, zz0, ds1, dzz1 = (to_dev(x) for x in (S0, z0, dS1, dz1))
    with schedule(**SCHEDULES[sched]):
        O = torch.full_like(tv, float("nan"))
        den = torch.full((B, H, N), float("nan"), dtype=torch.float32, device=DEV)
        S1 = torch.full((B, H, D, M), float("nan"), device=DEV)
        z1 = torch.full((B, H, D), float("nan"), device=DEV)
        ws = la.la_causal_fwd_state(tq, tk, tv, O, den, s0, zz0, S1, z1, eps, token_major=True)
        gq, gk, gv = (torch.full_like(x, float("nan")) for x in (tq, tk, tv))
        ds0 = torch.full((B, H, D, M), float("nan"), device=DEV)
        dzz0 = torch.full((B, H, D), float("nan"), device=DEV)
        la.la_causal_bwd_state(tq, tk, tv, None, den, tg, gq, gk, gv, s0, zz0, ds1, dzz1, ds0, dzz0, eps,
                               fwd_ws=ws, token_major=True)
        torch.cuda.synchronize()
        # the same through the [B, H, N, .] entry points
        hq, hk, hv = (to_dev(x) for x in (Q, K, V))
        O2 = torch.empty_like(hv)
        den2 = torch.empty(B, H, N, device=DEV)
        S12, z12 = torch.empty_like(S1), torch.empty_like(z1)
        la.la_causal_fwd_state(hq, hk, hv, O2, den2, s0, zz0, S12, z12, eps)
        g2 = _gpu_bwd_state(la, Q, K, V, G, S0, z0, dS1, dz1, eps)
    tol = tol_for(N)
    ref_O, ref_den, ref_S1, ref_z1 = oracle.causal_fwd_state(Q, K, V, S0, z0, eps)
    assert rel_err(_head_major(O), ref_O) <= tol and rel_err(den.cpu().numpy(), ref_den) <= tol
    assert rel_err(S1.cpu().numpy(), ref_S1) <= tol and rel_err(z1.cpu().numpy(), ref_z1) <= tol
    ref = oracle.causal_bwd_state(Q, K, V, G, S0, z0, dS1, dz1, eps)
    got = [_head_major(gq), _head_major(gk), _head_major(gv), ds0.cpu().numpy(), dzz0.cpu().numpy()]
    assert max(grad_errs(got[:3], ref[:3])) <= tol
    assert rel_err(got[3], ref[3]) <= tol and rel_err(got[4], ref[4]) <= tol
    assert np.array_equal(_head_major(O), to_host(O2)) and torch.equal(den, den2)
    assert torch.equal(S1, S12) and torch.equal(z1, z12)
    for a, b in zip(got, g2):
        assert np.array_equal(a, b)


def test_backward_workspace_holds_no_token_sized_matrix(la, oracle):
    """The constant-memory backward (section 3.3.1): besides the segment states its workspace is
    three fp32 scalars per token, also when the denominators are recomputed (the forward is then
    run for its denominators only)."""
    B, H, N, D, M = 2, 4, 700, 64, 64
    Q, K, V, G = wl.random_case(5151, B, H, N, D, M)
    with schedule(**SCHEDULES["one_segment"]):
        need = la.la_causal_bwd_workspace(B, H, N, D, M)
        assert need <= 3 * (B * H * N * 4 + 256)
        got = run_bwd(la, Q, K, V, G, 1e-6, reuse_fwd=False)
    assert la.la_global_bwd_workspace(B, H, N, D, M) <= \
        2 * la.la_global_fwd_workspace(B, H, N, D, M) + B * H * N * 4 + 256
    assert max(grad_errs(got, oracle.causal_bwd_linear(Q, K, V, G, 1e-6))) <= tol_for(N)


@pytest.mark.parametrize("B,H,N,D,M,bf16,sched", [
    (2, 3, 333, 64, 64, False, "default"),
    (1, 8, 1000, 64, 32, False, "many_segments"),
    (3, 2, 77, 32, 64, True, "one_segment"),
])
def test_token_major_layout_non_causal(la, oracle, B, H, N, D, M, bf16, sched):
    host = maybe_bf16(wl.random_case(8700 + N, B, H, N, D, M), bf16)
    Q, K, V, G = host
    eps = 1e-6
    tq, tk, tv, tg = (_token_major(x, bf16) for x in host)
    with schedule(**SCHEDULES[sched]):
        O = torch.full_like(tv, float("nan"))
        den = torch.full((B, H, N), float("nan"), dtype=torch.float32, device=DEV)
        ws = la.la_global_fwd_bnhd(tq, tk, tv, O, eps, den=den)
        gq, gk, gv = (torch.full_like(x, float("nan")) for x in (tq, tk, tv))
        la.la_global_bwd_bnhd(tq, tk, tv, None, den, tg, gq, gk, gv, eps, fwd_ws=ws)
        torch.cuda.synchronize()
        O2, den2, g2 = run_global(la, Q, K, V, G, eps, bf16=bf16)
    tol = tol_for(N, bf16)
    assert rel_err(_head_major(O), oracle.global_fwd_linear(Q, K, V, eps)) <= tol
    got = [_head_major(x) for x in (gq, gk, gv)]
    assert max(grad_errs(got, oracle.global_bwd_linear(Q, K, V, G, eps))) <= tol
    assert np.array_equal(_head_major(O), O2) and np.array_equal(den.cpu().numpy(), den2)
    for a, b in zip(got, g2):
        assert np.array_equal(a, b)


def test_token_major_autograd(la, oracle):
    B, H, N, D, M = 2, 4, 210, 64, 64
    Q, K, V, G = wl.random_case(8899, B, H, N, D, M)
    tq, tk, tv = (_token_major(x).requires_grad_() for x in (Q, K, V))
    O = la.causal_linear_attention(tq, tk, tv, 1e-6, layout="bnhd")
    O.backward(_token_major(G))
    torch.cuda.synchronize()
    assert rel_err(_head_major(O), oracle.causal_fwd_prefix(Q, K, V, 1e-6)) <= tol_for(N)
    got = [_head_major(x.grad) for x in (tq, tk, tv)]
    assert max(grad_errs(got, oracle.causal_bwd_linear(Q, K, V, G, 1e-6))) <= tol_for(N)
    for x in (tq, tk, tv):
        x.grad = None
    O = la.linear_attention(tq, tk, tv, 1e-6, layout="bnhd")
    O.backward(_token_major(G))
    torch.cuda.synchronize()
    assert rel_err(_head_major(O), oracle.global_fwd_linear(Q, K, V, 1e-6)) <= tol_for(N)
    got = [_head_major(x.grad) for x in (tq, tk, tv)]
    assert max(grad_errs(got, oracle.global_bwd_linear(Q, K, V, G, 1e-6))) <= tol_for(N)


# ---- Q and K as feature values of a map the caller applied ---------------------------------

@pytest.fixture
def oracle_features(oracle):
    oracle.set_feature_map(1)
    yield oracle
    oracle.set_feature_map(0)


def _feature_case(seed, B, H, N, D, M):
    """Non-negative features (some below one, some exactly zero) in place of Q and K."""
    rng = np.random.default_rng(seed)
    FQ = rng.gamma(1.5, 0.6, (B, H, N, D)).astype(np.float32)
    FK = rng.gamma(1.5, 0.6, (B, H, N, D)).astype(np.float32)
    FK[rng.random(FK.shape) < 0.1] = 0.0
    V = rng.standard_normal((B, H, N, M)).astype(np.float32)
    G = rng.standard_normal((B, H, N, M)).astype(np.float32)
    return FQ, FK, V, G


@pytest.mark.parametrize("sched", ["default", "one_segment", "three_chunk_segments"])
@pytest.mark.parametrize("D,M,N", [(64, 64, 300), (32, 64, 77), (64, 32, 1000)])
def test_caller_supplied_features_against_oracle(la, oracle_features, D, M, N, sched):
    o = oracle_features
    B, H = 2, 2
    FQ, FK, V, G = _feature_case(1100 + N, B, H, N, D, M)
    eps = 1e-5
    dq, dk, dv, dg = (to_dev(x) for x in (FQ, FK, V, G))
    with schedule(**SCHEDULES[sched]):
        O = torch.empty_like(dv); den = torch.empty(B, H, N, device=DEV)
        ws = la.la_causal_fwd(dq, dk, dv, O, den, eps, features=True)
        gq, gk, gv = (torch.empty_like(x) for x in (dq, dk, dv))
        la.la_causal_bwd(dq, dk, dv, None, den, dg, gq, gk, gv, eps, fwd_ws=ws, features=True)
        Og = torch.empty_like(dv); deng = torch.empty(B, H, N, device=DEV)
        wsg = la.la_global_fwd(dq, dk, dv, Og, eps, den=deng, features=True)
        hq, hk, hv = (torch.empty_like(x) for x in (dq, dk, dv))
        la.la_global_bwd(dq, dk, dv, None, deng, dg, hq, hk, hv, eps, fwd_ws=wsg, features=True)
    torch.cuda.synchronize()
    tol = tol_for(N)
    ref, dref = o.causal_fwd_prefix(FQ, FK, V, eps, return_den=True)
    assert rel_err(to_host(O), ref) <= tol and rel_err(den.cpu().numpy(), dref) <= tol
    assert max(grad_errs([to_host(x) for x in (gq, gk, gv)], o.causal_bwd_linear(FQ, FK, V, G, eps))) <= tol
    assert rel_err(to_host(Og), o.global_fwd_linear(FQ, FK, V, eps)) <= tol
    assert max(grad_errs([to_host(x) for x in (hq, hk, hv)], o.global_bwd_linear(FQ, FK, V, G, eps))) <= tol


def test_degree_two_polynomial_kernel_through_the_feature_interface(la, oracle_features):
    """The polynomial kernel of degree 2 (section 3.2: a finite feature map, sim(q, k) = (q . k)^2):
    phi(x) = vec(x x^T), 64 features of an 8-vector, handed in as features (signed values).
    The oracle on these features must equal attention with (q . k)^2 written out, and the GPU
    must equal the oracle, forward and backward, causal and not."""
    o = oracle_features
    rng = np.random.default_rng(2468)
    B, H, N, d, M = 2, 3, 333, 8, 64
    xq, xk = (rng.standard_normal((B, H, N, d)) for _ in range(2))
    V, G = (rng.standard_normal((B, H, N, M)).astype(np.float32) for _ in range(2))
    FQ = np.einsum("...i,...j->...ij", xq, xq).reshape(B, H, N, d * d).astype(np.float32)
    FK = np.einsum("...i,...j->...ij", xk, xk).reshape(B, H, N, d * d).astype(np.float32)
    # (q . k)^2 can be arbitrarily small, and where den is tiny its rounding error in fp32 is
    # amplified by 1/den^2 in the gradients (token 0 of a causal sequence has a single term):
    # a sizeable eps keeps the case well conditioned; the point here is the interface
    eps = 0.5
    # the definition, from the float32 features' own inner products
    A = np.einsum("bhic,bhjc->bhij", FQ.astype(np.float64), FK.astype(np.float64))
    np.testing.assert_allclose(A, np.einsum("bhid,bhjd->bhij", xq, xk) ** 2, rtol=2e-5, atol=2e-5)
    Ac = np.tril(A)
    ref_c = (Ac @ V) / (Ac.sum(-1, keepdims=True) + eps)
    ref_g = (A @ V) / (A.sum(-1, keepdims=True) + eps)
    np.testing.assert_allclose(o.causal_fwd_prefix(FQ, FK, V, eps), ref_c, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(o.global_fwd_linear(FQ, FK, V, eps), ref_g, rtol=1e-9, atol=1e-11)
    dq, dk, dv, dg = (to_dev(x) for x in (FQ, FK, V, G))
    O = torch.empty_like(dv); den = torch.empty(B, H, N, device=DEV)
    ws = la.la_causal_fwd(dq, dk, dv, O, den, eps, features=True)
    gq, gk, gv = (torch.empty_like(x) for x in (dq, dk, dv))
    la.la_causal_bwd(dq, dk, dv, None, den, dg, gq, gk, gv, eps, fwd_ws=ws, features=True)
    Og = torch.empty_like(dv); deng = torch.empty(B, H, N, device=DEV)
    wsg = la.la_global_fwd(dq, dk, dv, Og, eps, den=deng, features=True)
    hq, hk, hv = (torch.empty_like(x) for x in (dq, dk, dv))
    la.la_global_bwd(dq, dk, dv, None, deng, dg, hq, hk, hv, eps, fwd_ws=wsg, features=True)
    torch.cuda.synchronize()
    tol = tol_for(N)
    assert rel_err(to_host(O), ref_c) <= tol and rel_err(to_host(Og), ref_g) <= tol
    assert max(grad_errs([to_host(x) for x in (gq, gk, gv)], o.causal_bwd_linear(FQ, FK, V, G, eps))) <= tol
    assert max(grad_errs([to_host(x) for x in (hq, hk, hv)], o.global_bwd_linear(FQ, FK, V, G, eps))) <= tol


def test_random_fourier_features_through_the_feature_interface(la, oracle_features):
    """Random Fourier features (the paper's conclusion names them as a feature map to explore):
    phi(x) = sqrt(1/R) [cos(Wx), sin(Wx)] with R = 32 Gaussian directions, so that
    phi(q) . phi(k) = mean_r cos(w_r . (q - k)), the Monte Carlo estimate of the RBF kernel
    exp(-|q - k|^2 / 2).  The map needs a projection, which the caller applies; the 64 signed
    features go through the feature interface.  The oracle on these features must equal
    attention with that similarity written out, which in turn is the RBF kernel up to the
    Monte Carlo error; the GPU must equal the oracle, forward and backward, causal and not."""
    o = oracle_features
    rng = np.random.default_rng(1357)
    B, H, N, d, R, M = 2, 2, 300, 16, 32, 64
    xq, xk = (0.1 * rng.standard_normal((B, H, N, d)) for _ in range(2))
    W = rng.standard_normal((R, d))
    V, G = (rng.standard_normal((B, H, N, M)).astype(np.float32) for _ in range(2))
    feat = lambda x: (np.concatenate([np.cos(x @ W.T), np.sin(x @ W.T)], axis=-1) / np.sqrt(R)).astype(np.float32)
    FQ, FK = feat(xq), feat(xk)
    eps = 1e-6
    diff = xq[:, :, :, None, :] - xk[:, :, None, :, :]
    A_def = np.cos(diff @ W.T).mean(-1)                     # the similarity, written out
    A = np.einsum("bhic,bhjc->bhij", FQ.astype(np.float64), FK.astype(np.float64))
    np.testing.assert_allclose(A, A_def, rtol=0, atol=5e-7)
    rbf = np.exp(-0.5 * (diff ** 2).sum(-1))
    assert np.abs(A_def - rbf).max() < 0.3 and np.abs(A_def - rbf).mean() < 0.04 and A.min() > 0.3
    Ac = np.tril(A)
    ref_c = (Ac @ V) / (Ac.sum(-1, keepdims=True) + eps)
    ref_g = (A @ V) / (A.sum(-1, keepdims=True) + eps)
    np.testing.assert_allclose(o.causal_fwd_prefix(FQ, FK, V, eps), ref_c, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(o.global_fwd_linear(FQ, FK, V, eps), ref_g, rtol=1e-9, atol=1e-11)
    dq, dk, dv, dg = (to_dev(x) for x in (FQ, FK, V, G))
    O = torch.empty_like(dv); den = torch.empty(B, H, N, device=DEV)
    ws = la.la_causal_fwd(dq, dk, dv, O, den, eps, features=True)
    gq, gk, gv = (torch.empty_like(x) for x in (dq, dk, dv))
    la.la_causal_bwd(dq, dk, dv, None, den, dg, gq, gk, gv, eps, fwd_ws=ws, features=True)
    Og = torch.empty_like(dv); deng = torch.empty(B, H, N, device=DEV)
    wsg = la.la_global_fwd(dq, dk, dv, Og, eps, den=deng, features=True)
    hq, hk, hv = (torch.empty_like(x) for x in (dq, dk, dv))
    la.la_global_bwd(dq, dk, dv, None, deng, dg, hq, hk, hv, eps, fwd_ws=wsg, features=True)
    torch.cuda.synchronize()
    tol = tol_for(N)
    assert rel_err(to_host(O), ref_c) <= tol and rel_err(to_host(Og), ref_g) <= tol
    assert max(grad_errs([to_host(x) for x in (gq, gk, gv)], o.causal_bwd_linear(FQ, FK, V, G, eps))) <= tol
    assert max(grad_errs([to_host(x) for x in (hq, hk, hv)], o.global_bwd_linear(FQ, FK, V, G, eps))) <= tol


def test_caller_supplied_features_decode_and_bf16(la, oracle_features):
    o = oracle_features
    B, H, T, D, M = 3, 2, 25, 64, 64
    FQ, FK, V, G = _feature_case(1150, B, H, T, D, M)
    # decode, token by token and in one launch (layout [T, B, H, .])
    q, k, v = (np.ascontiguousarray(np.moveaxis(x, 2, 0)) for x in (FQ, FK, V))
    dq, dk, dv = (to_dev(x) for x in (q, k, v))
    S = torch.zeros(B, H, D, M, device=DEV); z = torch.zeros(B, H, D, device=DEV)
    out = torch.empty(T, B, H, M, device=DEV)
    for t in range(T):
        la.la_recurrent_step(dq[t], dk[t], dv[t], S, z, out[t], 1e-6, features=True)
    S2 = torch.zeros_like(S); z2 = torch.zeros_like(z); out2 = torch.empty_like(out)
    la.la_recurrent_steps(dq, dk, dv, S2, z2, out2, 1e-6, features=True)
    torch.cuda.synchronize()
    ref = o.causal_fwd_prefix(FQ, FK, V, 1e-6)
    assert rel_err(np.moveaxis(to_host(out), 0, 2), ref) <= 1e-4
    assert torch.equal(out, out2) and torch.equal(S, S2) and torch.equal(z, z2)
    # bf16 tensors
    FQb, FKb, Vb, Gb = (wl.round_to_bf16(x) for x in (FQ, FK, V, G))
    bq, bk, bv, bg = (to_dev(x, True) for x in (FQb, FKb, Vb, Gb))
    O = torch.empty_like(bv); den = torch.empty(B, H, T, device=DEV)
    ws = la.la_causal_fwd(bq, bk, bv, O, den, 1e-6, features=True)
    gq, gk, gv = (torch.empty_like(x) for x in (bq, bk, bv))
    la.la_causal_bwd(bq, bk, bv, None, den, bg, gq, gk, gv, 1e-6, fwd_ws=ws, features=True)
    torch.cuda.synchronize()
    assert rel_err(to_host(O), o.causal_fwd_prefix(FQb, FKb, Vb, 1e-6)) <= 2e-2
    gref = o.causal_bwd_linear(FQb, FKb, Vb, Gb, 1e-6)
    assert max(grad_errs([to_host(x) for x in (gq, gk, gv)], gref)) <= 2e-2


def test_features_equal_the_elu_map_on_shifted_inputs_bit_for_bit(la):
    """elu(x) + 1 = x + 1 with slope 1 for x > 0, and x + 1 is exact for x on a coarse grid: the
    same call on raw x (map inside) and on features x + 1 (map outside) must agree in every bit,
    for every entry point including the state-carrying ones."""
    B, H, N, D, M = 2, 2, 200, 64, 64
    rng = np.random.default_rng(1160)
    Xq = (rng.integers(1, 256, (B, H, N, D)) / 64.0).astype(np.float32)
    Xk = (rng.integers(1, 256, (B, H, N, D)) / 64.0).astype(np.float32)
    _, _, V, G, S0, z0, dS1, dz1 = _state_case(1161, B, H, N, D, M)
    res = []
    for Qh, Kh, feat in ((Xq, Xk, False), (Xq + 1.0, Xk + 1.0, True)):
        dq, dk, dv, dg = (to_dev(x) for x in (Qh, Kh, V, G))
        s0, zz0, ds1, dzz1 = (to_dev(x) for x in (S0, z0, dS1, dz1))
        O = torch.empty_like(dv); den = torch.empty(B, H, N, device=DEV)
        S1 = torch.empty(B, H, D, M, device=DEV); z1 = torch.empty(B, H, D, device=DEV)
        with schedule(**SCHEDULES["three_chunk_segments"]):
            ws = la.la_causal_fwd_state(dq, dk, dv, O, den, s0, zz0, S1, z1, 1e-6, features=feat)
            gq, gk, gv = (torch.empty_like(x) for x in (dq, dk, dv))
            ds0 = torch.empty_like(S1); dzz0 = torch.empty_like(z1)
            la.la_causal_bwd_state(dq, dk, dv, None, den, dg, gq, gk, gv, s0, zz0, ds1, dzz1, ds0, dzz0,
                                   1e-6, fwd_ws=ws, features=feat)
        torch.cuda.synchronize()
        res.append([x.clone() for x in (O, den, S1, z1, gq, gk, gv, ds0, dzz0)])
    for a, b in zip(*res):
        assert torch.equal(a, b)


def test_bitwise_determinism_and_slab_independence(la):
    B, H, N, D, M = 2, 4, 500, 64, 64
    Q, K, V, G = wl.random_case(800, B, H, N, D, M)
    with schedule(**SCHEDULES["three_chunk_segments"]):
        O1, d1 = run_fwd(la, Q, K, V, 1e-6)
        O2, d2 = run_fwd(la, Q, K, V, 1e-6)
        g1 = run_bwd(la, Q, K, V, G, 1e-6)
        g2 = run_bwd(la, Q, K, V, G, 1e-6)
        perm = [1, 0]
        O3, _ = run_fwd(la, Q[perm], K[perm], V[perm], 1e-6)
    assert np.array_equal(O1, O2) and np.array_equal(d1, d2)
    assert all(np.array_equal(a, b) for a, b in zip(g1, g2))
    assert np.array_equal(O3, O1[perm])


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("future", ["huge", "inf", "nan"])
def test_causality_future_does_not_leak(la, future, bf16):
    """Outputs before token t are bit-identical whatever follows it, finite or not: the mask is a
    select on the scores, so 1e30-sized (or NaN) scores of future tokens contribute an exact
    zero, and V is made finite when its tile is parked, so that the zero is not multiplied by an
    Inf or a NaN of a later token of the same 16-token tile."""
    B, H, N, D, M = 1, 2, 200, 64, 64
    Q, K, V = maybe_bf16(wl.random_case(801, B, H, N, D, M)[:3], bf16)
    t = 77                                     # inside a chunk: 77 = 4*16 + 13
    dev = [to_dev(x, bf16) for x in (Q, K, V)]
    O = torch.empty_like(dev[2]); den = torch.empty(B, H, N, device=DEV)
    la.la_causal_fwd(dev[0], dev[1], dev[2], O, den, 1e-6)
    Q2, K2, V2 = Q.copy(), K.copy(), V.copy()
    if future == "huge":
        V2[:, :, t:] = 1e30; Q2[:, :, t:] = -3.0; K2[:, :, t:] = 50.0
    elif future == "inf":
        V2[:, :, t:] = np.inf; V2[:, :, t + 1::2] = -np.inf; Q2[:, :, t:] = np.inf; K2[:, :, t:] = np.inf
    else:
        V2[:, :, t:] = np.nan; Q2[:, :, t:] = np.nan; K2[:, :, t:] = np.nan
    dq, dk, dv = (to_dev(x, bf16) for x in (Q2, K2, V2))
    O2 = torch.empty_like(dv); den2 = torch.empty_like(den)
    la.la_causal_fwd(dq, dk, dv, O2, den2, 1e-6)
    torch.cuda.synchronize()
    assert torch.equal(O2[:, :, :t], O[:, :, :t]) and torch.equal(den2[:, :, :t], den[:, :, :t])
    assert bool(torch.isfinite(O2[:, :, :t].float()).all())


def test_outputs_stay_inside_their_buffers(la):
    """Guard bands around every output keep their NaN fill for a ragged N."""
    B, H, N, D, M = 2, 2, 77, 32, 64
    Q, K, V, G = wl.random_case(802, B, H, N, D, M)
    dq, dk, dv, dg = (to_dev(x) for x in (Q, K, V, G))
    pad = 1024

    def guarded(shape):
        n = int(np.prod(shape))
        buf = torch.full((n + 2 * pad,), float("nan"), device=DEV)
        return buf, buf[pad:pad + n].view(*shape)

    bO, O = guarded(dv.shape); bd, den = guarded(Q.shape[:-1])
    bq, gq = guarded(dq.shape); bk, gk = guarded(dk.shape); bv, gv = guarded(dv.shape)
    with schedule(**SCHEDULES["many_segments"]):
        la.la_causal_fwd(dq, dk, dv, O, den, 1e-6)
        la.la_causal_bwd(dq, dk, dv, O, den, dg, gq, gk, gv, 1e-6)
    torch.cuda.synchronize()
    for buf, view in ((bO, O), (bd, den), (bq, gq), (bk, gk), (bv, gv)):
        assert torch.isnan(buf[:pad]).all() and torch.isnan(buf[-pad:]).all()
        assert torch.isfinite(view).all()


def test_underflowed_keys_give_zero_rows(la):
    B, H, N, D, M = 1, 1, 40, 32, 32
    Q, K, V = wl.random_case(803, B, H, N, D, M)[:3]
    K[:, :, :20] = -200.0                     # exp underflows to 0 in fp32
    O, den = run_fwd(la, Q, K, V, 1e-6)
    assert np.all(O[:, :, :20] == 0.0)
    assert np.all(np.isfinite(O))


# ---- fused degree-2 polynomial map (section 3.2): Q, K hold 8 raw values per token ---------------

def _poly2_case(seed, B, H, N, M):
    rng = np.random.default_rng(seed)
    Q, K = (rng.standard_normal((B, H, N, 8)).astype(np.float32) for _ in range(2))
    V, G = (rng.standard_normal((B, H, N, M)).astype(np.float32) for _ in range(2))
    return Q, K, V, G


# (q . k)^2 can be arbitrarily small, and where den is tiny its rounding error in fp32 is amplified
# by 1/den^2 in the gradients (token 0 of a causal sequence has a single term): a sizeable eps
# keeps the cases well conditioned
POLY_EPS = 0.5


@pytest.mark.parametrize("sched", list(SCHEDULES))
@pytest.mark.parametrize("N,M", [(1, 64), (16, 32), (17, 64), (100, 64), (257, 32), (1000, 64)])
def test_poly2_map_causal_forward_backward(la, oracle, N, M, sched):
    B, H = 2, 3
    Q, K, V, G = _poly2_case(7000 + N, B, H, N, M)
    ref, dref = oracle.causal_fwd_poly2(Q, K, V, POLY_EPS, return_den=True)
    gref = oracle.causal_bwd_poly2(Q, K, V, G, POLY_EPS)
    dq, dk, dv, dg = (to_dev(x) for x in (Q, K, V, G))
    with schedule(**SCHEDULES[sched]):
        O = torch.full_like(dv, float("nan"))
        den = torch.full((B, H, N), float("nan"), device=DEV)
        ws = la.la_causal_fwd(dq, dk, dv, O, den, POLY_EPS, features="poly2")
        gq, gk, gv = (torch.full_like(x, float("nan")) for x in (dq, dk, dv))
        la.la_causal_bwd(dq, dk, dv, None, den, dg, gq, gk, gv, POLY_EPS, fwd_ws=ws, features="poly2")
        # and without anything kept from the forward
        rq, rk, rv = (torch.full_like(x, float("nan")) for x in (dq, dk, dv))
        la.la_causal_bwd(dq, dk, dv, None, None, dg, rq, rk, rv, POLY_EPS, features="poly2")
        torch.cuda.synchronize()
    tol = tol_for(N)
    assert gq.shape == (B, H, N, 8)
    assert rel_err(to_host(O), ref) <= tol and rel_err(den.cpu().numpy(), dref) <= tol
    assert max(grad_errs([to_host(x) for x in (gq, gk, gv)], gref)) <= tol
    assert torch.equal(gq, rq) and torch.equal(gk, rk) and torch.equal(gv, rv)


@pytest.mark.parametrize("sched", ["default", "one_segment", "many_segments", "folded_totals"])
@pytest.mark.parametrize("N,M", [(1, 32), (17, 64), (300, 64), (1000, 32)])
def test_poly2_map_non_causal_forward_backward(la, oracle, N, M, sched):
    B, H = 2, 2
    Q, K, V, G = _poly2_case(7100 + N, B, H, N, M)
    ref = oracle.global_fwd_poly2(Q, K, V, POLY_EPS)
    gref = oracle.global_bwd_poly2(Q, K, V, G, POLY_EPS)
    dq, dk, dv, dg = (to_dev(x) for x in (Q, K, V, G))
    with schedule(**SCHEDULES[sched]):
        O = torch.full_like(dv, float("nan"))
        den = torch.full((B, H, N), float("nan"), device=DEV)
        ws = la.la_global_fwd(dq, dk, dv, O, POLY_EPS, den=den, features="poly2")
        gq, gk, gv = (torch.full_like(x, float("nan")) for x in (dq, dk, dv))
        la.la_global_bwd(dq, dk, dv, None, den, dg, gq, gk, gv, POLY_EPS, fwd_ws=ws, features="poly2")
        torch.cuda.synchronize()
    tol = tol_for(N)
    assert rel_err(to_host(O), ref) <= tol
    assert max(grad_errs([to_host(x) for x in (gq, gk, gv)], gref)) <= tol


def test_poly2_map_equals_the_feature_interface_and_decode(la, oracle):
    """The fused map against the same call on host-built features (LA_F32_FEATURES): same
    products, so the outputs agree to rounding of the features; token-major layout bit for bit;
    decode step by step and in one launch against the oracle's recurrence."""
    B, H, N, M = 2, 4, 203, 64
    Q, K, V, G = _poly2_case(7200, B, H, N, M)
    dq, dk, dv, dg = (to_dev(x) for x in (Q, K, V, G))
    O = torch.empty_like(dv)
    la.la_causal_fwd(dq, dk, dv, O, None, POLY_EPS, features="poly2")
    FQ = (dq[..., :, None] * dq[..., None, :]).reshape(B, H, N, 64).contiguous()      # fp32 products,
    FK = (dk[..., :, None] * dk[..., None, :]).reshape(B, H, N, 64).contiguous()      # as in the kernel
    O2 = torch.empty_like(dv)
    la.la_causal_fwd(FQ, FK, dv, O2, None, POLY_EPS, features=True)
    torch.cuda.synchronize()
    assert torch.equal(O, O2)
    # token-major tensors
    tq, tk, tv, tg = (x.transpose(1, 2).contiguous() for x in (dq, dk, dv, dg))
    Ot = torch.empty_like(tv); den = torch.empty(B, H, N, device=DEV)
    ws = la.la_causal_fwd_bnhd(tq, tk, tv, Ot, den, POLY_EPS, features="poly2")
    gq, gk, gv = (torch.empty_like(x) for x in (tq, tk, tv))
    la.la_causal_bwd_bnhd(tq, tk, tv, None, den, tg, gq, gk, gv, POLY_EPS, fwd_ws=ws, features="poly2")
    hq, hk, hv = (torch.empty_like(x) for x in (dq, dk, dv))
    la.la_causal_bwd(dq, dk, dv, None, den, dg, hq, hk, hv, POLY_EPS, features="poly2")
    torch.cuda.synchronize()
    assert torch.equal(Ot.transpose(1, 2), O)
    for a, b in ((gq, hq), (gk, hk), (gv, hv)):
        assert torch.equal(a.transpose(1, 2), b)
    # decode: state sized by the 64 features
    T = 40
    q, k, v = (x[:, :, :T].permute(2, 0, 1, 3).contiguous() for x in (dq, dk, dv))
    S = torch.zeros(B, H, 64, M, device=DEV); z = torch.zeros(B, H, 64, device=DEV)
    out = torch.empty(T, B, H, M, device=DEV)
    for t in range(T):
        la.la_recurrent_step(q[t], k[t], v[t], S, z, out[t], POLY_EPS, features="poly2")
    S2 = torch.zeros_like(S); z2 = torch.zeros_like(z); out2 = torch.empty_like(out)
    la.la_recurrent_steps(q, k, v, S2, z2, out2, POLY_EPS, features="poly2")
    torch.cuda.synchronize()
    assert torch.equal(out, out2) and torch.equal(S, S2) and torch.equal(z, z2)
    So, zo = np.zeros((B, H, 64, M)), np.zeros((B, H, 64))
    qh, kh, vh = (to_host(x) for x in (q, k, v))
    for t in range(T):
        ref = oracle.recurrent_step_poly2(qh[t], kh[t], vh[t], So, zo, POLY_EPS)
        assert rel_err(to_host(out[t]), ref) <= 1e-4
    assert rel_err(S.cpu().numpy(), So) <= 1e-4 and rel_err(z.cpu().numpy(), zo) <= 1e-4
    assert rel_err(to_host(out), np.moveaxis(to_host(O[:, :, :T]), 2, 0)) <= 1e-4     # decode == parallel


@pytest.mark.parametrize("sched", ["default", "many_segments", "folded_totals"])
def test_poly2_map_sequence_in_two_pieces_through_the_state(la, oracle, sched):
    """The state interface with the polynomial map: the state is sized by the 64 features, not by
    the 8 raw values.  Forward in two pieces (the first one's final state starts the second),
    backward in reverse (the second one's state gradient arrives at the first): outputs and
    gradients must be those of the uncut sequence."""
    B, H, N1, N2, M = 2, 2, 130, 275, 64
    N = N1 + N2
    Q, K, V, G = _poly2_case(7300, B, H, N, M)
    ref = oracle.causal_fwd_poly2(Q, K, V, POLY_EPS)
    gref = oracle.causal_bwd_poly2(Q, K, V, G, POLY_EPS)
    dev = [to_dev(x) for x in (Q, K, V, G)]
    a = [x[:, :, :N1].contiguous() for x in dev]
    b = [x[:, :, N1:].contiguous() for x in dev]
    S1 = torch.full((B, H, 64, M), float("nan"), device=DEV); z1 = torch.full((B, H, 64), float("nan"), device=DEV)
    kw = dict(features="poly2")
    with schedule(**SCHEDULES[sched]):
        Oa = torch.empty_like(a[2]); dena = torch.empty(B, H, N1, device=DEV)
        wsa = la.la_causal_fwd_state(a[0], a[1], a[2], Oa, dena, None, None, S1, z1, POLY_EPS, **kw)
        Ob = torch.empty_like(b[2]); denb = torch.empty(B, H, N2, device=DEV)
        wsb = la.la_causal_fwd_state(b[0], b[1], b[2], Ob, denb, S1, z1, None, None, POLY_EPS, **kw)
        gb = [torch.full_like(x, float("nan")) for x in b[:3]]
        dS = torch.full_like(S1, float("nan")); dz = torch.full_like(z1, float("nan"))
        la.la_causal_bwd_state(b[0], b[1], b[2], Ob, denb, b[3], gb[0], gb[1], gb[2], S1, z1, None, None,
                               dS, dz, POLY_EPS, fwd_ws=wsb, **kw)
        ga = [torch.full_like(x, float("nan")) for x in a[:3]]
        la.la_causal_bwd_state(a[0], a[1], a[2], None, None, a[3], ga[0], ga[1], ga[2], None, None, dS, dz,
                               None, None, POLY_EPS, **kw)
        torch.cuda.synchronize()
    assert ga[0].shape == (B, H, N1, 8)
    tol = tol_for(N)
    assert rel_err(np.concatenate([to_host(Oa), to_host(Ob)], axis=2), ref) <= tol
    got = [np.concatenate([to_host(x), to_host(y)], axis=2) for x, y in zip(ga, gb)]
    assert max(grad_errs(got, gref)) <= tol
    fk = oracle.poly2_features(K[:, :, :N1].astype(np.float64))
    assert rel_err(S1.cpu().numpy(), np.einsum("bhnd,bhnm->bhdm", fk, V[:, :, :N1].astype(np.float64))) <= tol
    assert rel_err(z1.cpu().numpy(), fk.sum(2), floor=1.0) <= tol


def test_two_host_threads_on_their_own_streams(la):
    """The header's thread-safety claim: calls from several host threads are safe as long as
    they share no output or workspace buffer.  Two threads, each with its own stream and
    buffers, run forward + backward + decode steps repeatedly at the same time; every result
    must be bit for bit what the same calls give one after the other."""
    import threading
    cases = [wl.random_case(1800 + i, 2, 3, 700 + 37 * i, 64, 64) for i in range(2)]

    def work(i, stream, rounds, out):
        Q, K, V, G = (to_dev(x) for x in cases[i])
        B, H, N = Q.shape[:3]
        with torch.cuda.stream(stream):
            for _ in range(rounds):
                O = torch.empty_like(V); den = torch.empty(B, H, N, device=DEV)
                ws = la.la_causal_fwd(Q, K, V, O, den, 1e-6)
                g = [torch.empty_like(x) for x in (Q, K, V)]
                la.la_causal_bwd(Q, K, V, None, den, G, g[0], g[1], g[2], 1e-6, fwd_ws=ws)
                S = torch.zeros(B, H, 64, 64, device=DEV); z = torch.zeros(B, H, 64, device=DEV)
                o = torch.empty(B, H, 64, device=DEV)
                for t in range(8):
                    la.la_recurrent_step(Q[:, :, t].contiguous(), K[:, :, t].contiguous(),
                                         V[:, :, t].contiguous(), S, z, o, 1e-6)
            stream.synchronize()
        out[i] = [O, den] + g + [S, z, o]

    serial, parallel = {}, {}
    for i in range(2):
        work(i, torch.cuda.Stream(), 1, serial)
    threads = [threading.Thread(target=work, args=(i, torch.cuda.Stream(), 20, parallel)) for i in range(2)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    torch.cuda.synchronize()
    for i in range(2):
        assert len(parallel[i]) == len(serial[i])
        for a, b in zip(parallel[i], serial[i]):
            assert torch.equal(a, b)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("sched", ["default", "many_segments", "folded_totals"])
def test_padded_keys_are_masked_by_minus_infinity(la, oracle, sched, bf16):
    """Sequences of different lengths in one batch of the non-causal calls: the padded tail of a
    sequence is taken out of the sums of eq. 5-6 by K = -inf there (phi(-inf) = 0 and phi' = 0,
    exactly), with a zero upstream gradient on the padded queries.  Every sequence must then
    equal the oracle on the sequence cut to its own length, forward and backward, and the padded
    rows of dK and dV must be exact zeros."""
    B, H, N, D, M = 3, 2, 700, 64, 64
    lengths = [700, 517, 130]
    Q, K, V, G = wl.random_case(1900, B, H, N, D, M)
    for b, n in enumerate(lengths):
        K[b, :, n:] = -np.inf
        G[b, :, n:] = 0.0
    Q, K, V, G = maybe_bf16([Q, K, V, G], bf16)
    with schedule(**SCHEDULES[sched]):
        O, den, grads = run_global(la, Q, K, V, G, 1e-6, bf16=bf16)
    tol = tol_for(N, bf16)
    for b, n in enumerate(lengths):
        cut = [x[b:b + 1, :, :n] for x in (Q, K, V, G)]
        assert rel_err(O[b:b + 1, :, :n], oracle.global_fwd_linear(*cut[:3], 1e-6)) <= tol
        ref = oracle.global_bwd_linear(*cut, 1e-6)
        assert max(grad_errs([g[b:b + 1, :, :n] for g in grads], ref)) <= tol
        assert np.all(grads[0][b, :, n:] == 0) and np.all(grads[1][b, :, n:] == 0) and np.all(grads[2][b, :, n:] == 0)
    assert np.all(np.isfinite(O)) and all(np.all(np.isfinite(g)) for g in grads)
