"""la_causal_fwd_noalloc (the forward whose segment states live in the library's built-in
scratch array) against la_causal_fwd, through the C ABI: two calls in a row, the second on a
smaller input, so that the second call runs on an array that still holds the first call's
states.  Collected last on purpose (file name)."""
import pytest
import torch

import workloads as wl
from gpu_util import DEV, rel_err, to_dev, to_host, tol_for

pytestmark = pytest.mark.gpu


def _pair(la, w, bf16=False):
    Q, K, V = (to_dev(wl.round_to_bf16(x) if bf16 else x, bf16) for x in wl.qkvg(w, with_grad=False))
    code = la.LA_BF16 if bf16 else la.LA_F32
    need = la.la_causal_fwd_workspace(w.B, w.H, w.N, w.D, w.M, code)
    O_ref = torch.full_like(V, float("nan"))
    den_ref = torch.full((w.B, w.H, w.N), float("nan"), dtype=torch.float32, device=DEV)
    la.la_causal_fwd(Q, K, V, O_ref, den_ref, w.eps)
    O = torch.full_like(V, float("nan"))
    den = torch.full_like(den_ref, float("nan"))
    la.la_causal_fwd_noalloc(Q, K, V, O, den, w.eps)
    torch.cuda.synchronize()
    return need, O, den, O_ref, den_ref


def test_noalloc_forward_matches_the_workspace_forward_twice_in_a_row():
    import paper_2006_16236_amd as la
    from paper_2006_16236_amd import binding
    assert torch.cuda.is_available()
    big = wl.Workload("noalloc_big", 2, 8, 8192, 64, 64, 1601)       # 128 segments per sequence
    small = wl.Workload("noalloc_small", 1, 3, 1000, 64, 32, 1602)   # ragged tail, fewer states
    tiny = wl.Workload("noalloc_tiny", 2, 2, 16, 32, 32, 1603)       # one chunk: no states at all
    needs = []
    for w, bf16 in ((big, False), (small, False), (small, True), (tiny, False)):
        need, O, den, O_ref, den_ref = _pair(la, w, bf16)
        needs.append(need)
        assert need <= binding.LA_NOALLOC_SCRATCH_BYTES
        tol = tol_for(w.N, bf16)
        assert rel_err(to_host(O), to_host(O_ref)) <= tol, w.name
        assert rel_err(den.cpu().numpy(), den_ref.cpu().numpy()) <= tol, w.name
        # same kernels, same schedule, deterministic sums: the results are in fact identical
        assert torch.equal(O, O_ref) and torch.equal(den, den_ref), w.name
    assert needs[0] > needs[1] > 0 and needs[3] == 0


def test_noalloc_forward_refuses_what_does_not_fit():
    from paper_2006_16236_amd import binding
    w = wl.Workload("noalloc_too_big", 125, 8, 4096, 64, 64, 1604)   # 3000 states of 16.6 KB
    assert binding.la_causal_fwd_workspace(w.B, w.H, w.N, w.D, w.M) > binding.LA_NOALLOC_SCRATCH_BYTES
    x = torch.zeros(16, device=DEV)       # never dereferenced: the sizes are refused on the host
    st = binding.raw().la_causal_fwd_noalloc(x.data_ptr(), x.data_ptr(), x.data_ptr(), x.data_ptr(),
                                             None, w.B, w.H, w.N, w.D, w.M, 1e-6, 0, None)
    assert st == binding.LA_ERR_SCRATCH
