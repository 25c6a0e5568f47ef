"""ctypes front end of the fp64 CPU oracle (oracle/la_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module
and this module never imports the product package.

All functions take and return numpy float64 arrays shaped [B, H, N, feature]
(or [BH, N, feature]); any leading dimensions are flattened into independent
slabs.  See the C file for which equation each function follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "la_oracle.c")
_LIB = os.path.join(_HERE, "liblaoracle.so")

_dp = ctypes.POINTER(ctypes.c_double)
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP over slabs).  -O2 without
    fast-math: summation order stays exactly as written in the source."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.la_oracle_phi.restype = ctypes.c_double
        _lib.la_oracle_phi.argtypes = [ctypes.c_double]
        _lib.la_oracle_dphi.restype = ctypes.c_double
        _lib.la_oracle_dphi.argtypes = [ctypes.c_double]
        _lib.la_oracle_max_threads.restype = ctypes.c_int
    return _lib


def _c(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(_dp)


def _slabs(Q, V):
    N, D = Q.shape[-2], Q.shape[-1]
    M = V.shape[-1]
    BH = int(np.prod(Q.shape[:-2], dtype=np.int64)) if Q.ndim > 2 else 1
    return BH, N, D, M


def max_threads() -> int:
    return int(_load().la_oracle_max_threads())


def set_threads(n: int) -> None:
    _load().la_oracle_set_threads(ctypes.c_int(int(n)))


def set_feature_map(which: int) -> None:
    """0: phi(x) = elu(x) + 1 (eq. 7, the default); 1: identity (Q, K hold feature values)."""
    _load().la_oracle_set_feature_map(ctypes.c_int(int(which)))


def phi(x):
    lib = _load()
    return np.vectorize(lambda t: lib.la_oracle_phi(float(t)), otypes=[np.float64])(np.asarray(x))


def dphi(x):
    lib = _load()
    return np.vectorize(lambda t: lib.la_oracle_dphi(float(t)), otypes=[np.float64])(np.asarray(x))


def _fwd(name, Q, K, V, eps, want_den):
    lib = _load()
    BH, N, D, M = _slabs(Q, V)
    Q, pq = _c(Q); K, pk = _c(K); V, pv = _c(V)
    O = np.empty(V.shape, dtype=np.float64)
    den = np.empty(Q.shape[:-1], dtype=np.float64)
    getattr(lib, name)(pq, pk, pv, O.ctypes.data_as(_dp), den.ctypes.data_as(_dp),
                       ctypes.c_int(BH), ctypes.c_int(N), ctypes.c_int(D), ctypes.c_int(M),
                       ctypes.c_double(eps))
    return (O, den) if want_den else O


def causal_fwd_quadratic(Q, K, V, eps=1e-6, return_den=False):
    """eq. 8 with sim = phi^T phi; O(N^2)."""
    return _fwd("la_oracle_causal_fwd_quadratic", Q, K, V, eps, return_den)


def causal_fwd_prefix(Q, K, V, eps=1e-6, return_den=False):
    """eq. 10-12 (running sums); O(N D M)."""
    return _fwd("la_oracle_causal_fwd_prefix", Q, K, V, eps, return_den)


def causal_weights(Q, K, eps=1e-6):
    """Row-normalised weights of eq. 8 for a single [N, D] slab -> [N, N]."""
    lib = _load()
    Q, pq = _c(Q); K, pk = _c(K)
    assert Q.ndim == 2
    N, D = Q.shape
    W = np.empty((N, N), dtype=np.float64)
    lib.la_oracle_causal_weights(pq, pk, W.ctypes.data_as(_dp), ctypes.c_int(N), ctypes.c_int(D),
                                 ctypes.c_double(eps))
    return W


def recurrent_step(q, k, v, S, z, eps=1e-6, return_den=False):
    """eq. 16-20 for one token per slab.  S [..., D, M] and z [..., D] are
    float64 C-contiguous arrays updated IN PLACE; returns out [..., M]."""
    lib = _load()
    assert S.dtype == np.float64 and S.flags.c_contiguous
    assert z.dtype == np.float64 and z.flags.c_contiguous
    D, M = S.shape[-2], S.shape[-1]
    BH = int(np.prod(S.shape[:-2], dtype=np.int64)) if S.ndim > 2 else 1
    q, pq = _c(q); k, pk = _c(k); v, pv = _c(v)
    out = np.empty(v.shape, dtype=np.float64)
    den = np.empty(z.shape[:-1], dtype=np.float64)
    lib.la_oracle_recurrent_step(pq, pk, pv, S.ctypes.data_as(_dp), z.ctypes.data_as(_dp),
                                 out.ctypes.data_as(_dp), den.ctypes.data_as(_dp),
                                 ctypes.c_int(BH), ctypes.c_int(D), ctypes.c_int(M),
                                 ctypes.c_double(eps))
    return (out, den) if return_den else out


def _gfwd(name, Q, K, V, eps):
    lib = _load()
    BH, N, D, M = _slabs(Q, V)
    Q, pq = _c(Q); K, pk = _c(K); V, pv = _c(V)
    O = np.empty(V.shape, dtype=np.float64)
    getattr(lib, name)(pq, pk, pv, O.ctypes.data_as(_dp),
                       ctypes.c_int(BH), ctypes.c_int(N), ctypes.c_int(D), ctypes.c_int(M),
                       ctypes.c_double(eps))
    return O


def global_fwd_quadratic(Q, K, V, eps=1e-6):
    """eq. 3 with sim = phi^T phi; O(N^2)."""
    return _gfwd("la_oracle_global_fwd_quadratic", Q, K, V, eps)


def global_fwd_linear(Q, K, V, eps=1e-6):
    """eq. 5-6; O(N D M)."""
    return _gfwd("la_oracle_global_fwd_linear", Q, K, V, eps)


def causal_numerator_fwd(fQ, fK, V):
    """The numerator of eq. 9 on already-mapped phi(Q), phi(K) (what Algorithm 1's forward returns)."""
    lib = _load()
    BH, N, C, M = _slabs(fQ, V)
    fQ, pq = _c(fQ); fK, pk = _c(fK); V, pv = _c(V)
    Vbar = np.empty(V.shape, dtype=np.float64)
    lib.la_oracle_causal_numerator_fwd(pq, pk, pv, Vbar.ctypes.data_as(_dp), ctypes.c_int(BH),
                                       ctypes.c_int(N), ctypes.c_int(C), ctypes.c_int(M))
    return Vbar


def causal_numerator_bwd(fQ, fK, V, G):
    """eq. 13-15: gradients of that numerator for phi(Q), phi(K), V."""
    lib = _load()
    BH, N, C, M = _slabs(fQ, V)
    fQ, pq = _c(fQ); fK, pk = _c(fK); V, pv = _c(V); G, pg = _c(G)
    gQ = np.empty(fQ.shape, dtype=np.float64)
    gK = np.empty(fK.shape, dtype=np.float64)
    gV = np.empty(V.shape, dtype=np.float64)
    lib.la_oracle_causal_numerator_bwd(pq, pk, pv, pg, gQ.ctypes.data_as(_dp),
                                       gK.ctypes.data_as(_dp), gV.ctypes.data_as(_dp),
                                       ctypes.c_int(BH), ctypes.c_int(N), ctypes.c_int(C),
                                       ctypes.c_int(M))
    return gQ, gK, gV


def _bwd(name, Q, K, V, G, eps):
    lib = _load()
    BH, N, D, M = _slabs(Q, V)
    Q, pq = _c(Q); K, pk = _c(K); V, pv = _c(V); G, pg = _c(G)
    dQ = np.empty(Q.shape, dtype=np.float64)
    dK = np.empty(K.shape, dtype=np.float64)
    dV = np.empty(V.shape, dtype=np.float64)
    getattr(lib, name)(pq, pk, pv, pg, dQ.ctypes.data_as(_dp), dK.ctypes.data_as(_dp),
                       dV.ctypes.data_as(_dp), ctypes.c_int(BH), ctypes.c_int(N),
                       ctypes.c_int(D), ctypes.c_int(M), ctypes.c_double(eps))
    return dQ, dK, dV


def causal_bwd_quadratic(Q, K, V, G, eps=1e-6):
    """Gradient of eq. 8 by brute force; O(N^2)."""
    return _bwd("la_oracle_causal_bwd_quadratic", Q, K, V, G, eps)


def causal_bwd_linear(Q, K, V, G, eps=1e-6):
    """eq. 13-15 on ones-augmented values + chain rule; O(N D M)."""
    return _bwd("la_oracle_causal_bwd_linear", Q, K, V, G, eps)


def global_bwd_quadratic(Q, K, V, G, eps=1e-6):
    """Gradient of eq. 3 (non-causal) by brute force; O(N^2)."""
    return _bwd("la_oracle_global_bwd_quadratic", Q, K, V, G, eps)


def global_bwd_linear(Q, K, V, G, eps=1e-6):
    """Gradient of eq. 5-6 from the two global sums; O(N D M)."""
    return _bwd("la_oracle_global_bwd_linear", Q, K, V, G, eps)


def _opt(a):
    if a is None:
        return None, None
    return _c(a)


def causal_fwd_state(Q, K, V, S0=None, Z0=None, eps=1e-6):
    """eq. 10-12 started from (S0 [..., D, M], Z0 [..., D]) (None: zero).
    Returns O, den, S_N, Z_N."""
    lib = _load()
    BH, N, D, M = _slabs(Q, V)
    Q, pq = _c(Q); K, pk = _c(K); V, pv = _c(V)
    S0, ps0 = _opt(S0); Z0, pz0 = _opt(Z0)
    O = np.empty(V.shape, dtype=np.float64)
    den = np.empty(Q.shape[:-1], dtype=np.float64)
    S1 = np.empty(Q.shape[:-2] + (D, M), dtype=np.float64)
    Z1 = np.empty(Q.shape[:-2] + (D,), dtype=np.float64)
    lib.la_oracle_causal_fwd_state(pq, pk, pv, ps0, pz0, O.ctypes.data_as(_dp),
                                   den.ctypes.data_as(_dp), S1.ctypes.data_as(_dp),
                                   Z1.ctypes.data_as(_dp), ctypes.c_int(BH), ctypes.c_int(N),
                                   ctypes.c_int(D), ctypes.c_int(M), ctypes.c_double(eps))
    return O, den, S1, Z1


def causal_bwd_state(Q, K, V, G, S0=None, Z0=None, dS1=None, dZ1=None, eps=1e-6):
    """Backpropagation through time with the state gradient handed in (dS1, dZ1 at the
    final state; None: zero) and out.  Returns dQ, dK, dV, dS0, dZ0."""
    lib = _load()
    BH, N, D, M = _slabs(Q, V)
    Q, pq = _c(Q); K, pk = _c(K); V, pv = _c(V); G, pg = _c(G)
    S0, ps0 = _opt(S0); Z0, pz0 = _opt(Z0); dS1, pds1 = _opt(dS1); dZ1, pdz1 = _opt(dZ1)
    dQ = np.empty(Q.shape, dtype=np.float64)
    dK = np.empty(K.shape, dtype=np.float64)
    dV = np.empty(V.shape, dtype=np.float64)
    dS0 = np.empty(Q.shape[:-2] + (D, M), dtype=np.float64)
    dZ0 = np.empty(Q.shape[:-2] + (D,), dtype=np.float64)
    lib.la_oracle_causal_bwd_state(pq, pk, pv, ps0, pz0, pg, pds1, pdz1, dQ.ctypes.data_as(_dp),
                                   dK.ctypes.data_as(_dp), dV.ctypes.data_as(_dp),
                                   dS0.ctypes.data_as(_dp), dZ0.ctypes.data_as(_dp),
                                   ctypes.c_int(BH), ctypes.c_int(N), ctypes.c_int(D),
                                   ctypes.c_int(M), ctypes.c_double(eps))
    return dQ, dK, dV, dS0, dZ0


# ---- degree-2 polynomial kernel (section 3.2) -------------------------------------------------
# sim(q, k) = (q . k)^2 has the finite feature map phi(x) = vec(x x^T): d raw dimensions give
# C = d^2 features, phi(q) . phi(k) = sum_ij q_i q_j k_i k_j = (q . k)^2, and the cost of the
# linear form becomes O(N d^2 M).  The functions below are that definition written out: map the
# raw vectors, run the functions above with the identity feature map on the mapped values, and
# carry the gradients back to the raw vectors by the chain rule of x -> x x^T.

def poly2_features(X):
    """[..., d] -> [..., d*d]: feature d*i + j = x_i x_j."""
    X = np.asarray(X, dtype=np.float64)
    return (X[..., :, None] * X[..., None, :]).reshape(X.shape[:-1] + (X.shape[-1] ** 2,))


def poly2_chain(X, dF):
    """Gradient with respect to the features [..., d*d] -> gradient with respect to x [..., d]:
    d(x_i x_j)/dx_k = delta_ik x_j + delta_jk x_i, so dx_k = sum_j (dF[k, j] + dF[j, k]) x_j."""
    X = np.asarray(X, dtype=np.float64)
    d = X.shape[-1]
    G = np.asarray(dF, dtype=np.float64).reshape(X.shape[:-1] + (d, d))
    return np.einsum("...kj,...j->...k", G + np.swapaxes(G, -1, -2), X)


class _identity_map:
    """Run the C functions with Q, K taken as feature values (and put the switch back)."""

    def __enter__(self):
        set_feature_map(1)

    def __exit__(self, *exc):
        set_feature_map(0)


def causal_fwd_poly2(Q, K, V, eps=1e-6, return_den=False):
    """eq. 10-12 with phi(x) = vec(x x^T)."""
    with _identity_map():
        return causal_fwd_prefix(poly2_features(Q), poly2_features(K), V, eps, return_den)


def causal_bwd_poly2(Q, K, V, G, eps=1e-6):
    """Gradients of the above for the raw Q, K and for V."""
    with _identity_map():
        dFq, dFk, dV = causal_bwd_linear(poly2_features(Q), poly2_features(K), V, G, eps)
    return poly2_chain(Q, dFq), poly2_chain(K, dFk), dV


def global_fwd_poly2(Q, K, V, eps=1e-6):
    """eq. 5-6 with phi(x) = vec(x x^T)."""
    with _identity_map():
        return global_fwd_linear(poly2_features(Q), poly2_features(K), V, eps)


def global_bwd_poly2(Q, K, V, G, eps=1e-6):
    with _identity_map():
        dFq, dFk, dV = global_bwd_linear(poly2_features(Q), poly2_features(K), V, G, eps)
    return poly2_chain(Q, dFq), poly2_chain(K, dFk), dV


def recurrent_step_poly2(q, k, v, S, z, eps=1e-6):
    """eq. 16-20 with phi(x) = vec(x x^T); S [..., d*d, M], z [..., d*d] updated in place."""
    with _identity_map():
        return recurrent_step(poly2_features(q), poly2_features(k), v, S, z, eps)
