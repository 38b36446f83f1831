"""GPU tests of the value-distillation loss (Sec. 3.3, Eq. "vd_loss") through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import hybrid_attn_oracle as O
from paper_2509_24899_amd import hybrid_attn as ha
from paper_2509_24899_amd import workloads as W
from tests.test_gpu_parity import REL_L2, SMALL, SMALL64, oracle_map, record

pytestmark = pytest.mark.gpu


def run_loss(inp, R, layout="bhnd", **kw):
    w = inp.workload
    q, k, v, fq, fk = ha.to_device(inp)
    if layout == "bnhd":
        q, k, v = (t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in (q, k, v))
    loss, yt, ys = ha.hybrid_attn_value_distill_loss(q, k, v, fq if R != 1 else None, fk if R != 1 else None, R,
                                                     w.block_size, w.scale, **kw)
    torch.cuda.synchronize()
    return loss.cpu().numpy(), yt, ys, (q, k, v, fq, fk)


@pytest.mark.parametrize("wl,R", [(W.TINY, 4), (SMALL, 4), (SMALL, 0), (SMALL64, 3)])
def test_loss_against_the_oracle(wl, R):
    """The GPU loss differs from the fp64 loss only through the errors of its two forwards:
    |L_gpu - L| <= ||dy||_1 + ||dy_hat||_1 <= sqrt(n) (||dy||_2 + ||dy_hat||_2), and each forward is held
    to rel-L2 <= 5e-3, so the bound is sqrt(n) 5e-3 (||y||_2 + ||y_hat||_2) with n the element count."""
    inp = W.make_inputs(wl)
    got, yt, ys, _ = run_loss(inp, R)
    fq, fk = oracle_map(inp.phi_q), oracle_map(inp.phi_k)
    y = O.hybrid_attn(inp.q, inp.k, inp.v, None, None, 1, wl.scale)
    yh = O.hybrid_attn(inp.q, inp.k, inp.v, fq, fk, R, wl.scale)
    ref = O.value_distill_loss(inp.q, inp.k, inp.v, fq, fk, R, wl.scale)
    bound = np.sqrt(y.size) * REL_L2 * (np.linalg.norm(y) + np.linalg.norm(yh))
    record(f"vd_loss_{wl.name}_R{R}", abs(got[0] - ref), abs(got[0] - ref) / ref, bound=float(bound), loss=float(ref))
    assert abs(got[0] - ref) <= bound
    assert abs(got[0] - ref) <= 2e-2 * ref          # in practice far inside the bound
    per = np.array([[np.abs(y[b, h] - yh[b, h]).sum() for h in range(wl.H)] for b in range(wl.B)]).ravel()
    np.testing.assert_allclose(got[1:], per, rtol=3e-2)
    np.testing.assert_allclose(got[1:].sum(), got[0], rtol=1e-14)


@pytest.mark.parametrize("layout", ("bhnd", "bnhd"))
def test_reduction_is_exact_on_its_own_inputs(layout):
    """The reduction alone: against a float64 sum of |y - y_hat| over the very tensors the kernel read."""
    inp = W.make_inputs(SMALL)
    got, yt, ys, _ = run_loss(inp, 4, layout)
    want = (yt.double() - ys.double()).abs().sum(dim=(2, 3)).cpu().numpy().ravel()
    np.testing.assert_allclose(got[1:], want, rtol=1e-5)
    np.testing.assert_allclose(got[0], want.sum(), rtol=1e-5)


def test_teacher_equals_student_at_rate_one_and_cached_teacher():
    inp = W.make_inputs(SMALL)
    got, yt, ys, (q, k, v, fq, fk) = run_loss(inp, 1)
    assert got[0] == 0.0 and (got[1:] == 0.0).all()      # same kernel twice: bitwise equal outputs
    first, yt, _, _ = run_loss(inp, 4)
    again, _, _ = ha.hybrid_attn_value_distill_loss(q, k, v, fq, fk, 4, SMALL.block_size, SMALL.scale,
                                                    y_teacher=yt, teacher_is_cached=True)
    torch.cuda.synchronize()
    assert (again.cpu().numpy() == first).all()           # bitwise reproducible, teacher forward skipped


def test_headline_shape_against_torch_reduction():
    """480p / 81 frames, R = 4: the reduction against torch's own float64 reduction of the same tensors."""
    w = W.WAN_480P_81F
    gen = torch.Generator(device="cuda").manual_seed(3)
    s = w.d ** -0.5
    q, k, v = ((torch.randn(w.B, w.H, w.N, w.d, generator=gen, device="cuda") * s).to(torch.bfloat16) for _ in range(3))

    def dmap():
        return ha.FeatureMap((torch.randn(w.H, w.d_hidden, w.d, generator=gen, device="cuda") * s).to(torch.bfloat16),
                             torch.randn(w.H, w.d_hidden, generator=gen, device="cuda") * 0.1,
                             (torch.randn(w.H, w.d_feat, w.d_hidden, generator=gen, device="cuda") * s).to(torch.bfloat16),
                             torch.randn(w.H, w.d_feat, generator=gen, device="cuda") * 0.1, w.poly_degree)
    loss, yt, ys = ha.hybrid_attn_value_distill_loss(q, k, v, dmap(), dmap(), w.R, w.block_size, w.scale)
    torch.cuda.synchronize()
    want = (yt.double() - ys.double()).abs().sum(dim=(2, 3)).ravel()
    got = loss.cpu().numpy()
    np.testing.assert_allclose(got[1:], want.cpu().numpy(), rtol=1e-5)
    np.testing.assert_allclose(got[0], float(want.sum()), rtol=1e-5)
    assert got[0] > 0
