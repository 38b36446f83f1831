"""GPU tests of the value-distillation gradient for the feature maps beyond d -> d -> d (Tab. "phi": wider and three-layer maps)."""
import numpy as np
import pytest
import torch

from oracle import value_distill_grad_oracle as G
from paper_2509_24899_amd import hybrid_attn as ha
from paper_2509_24899_amd import workloads as W
from tests.test_gpu_parity import SMALL
from tests.test_gpu_value_distill_grad import (GRAD_REL_L2, LOGIT_STD1, NAMES, bf16_representable, compare,
                                               oracle_forward_pieces, round_io)

pytestmark = pytest.mark.gpu

WIDE_CASES = [
    (W.replace(SMALL, name="vdg_paper_width", B=2, H=2, d_hidden=256, d_feat=256, poly_degree=2, seed=90), 4),
    (W.replace(SMALL, name="vdg_P3", B=1, H=2, d_hidden=384, d_feat=384, poly_degree=3, seed=91), 4),
    (W.replace(SMALL, name="vdg_256_128", B=2, H=2, N=700, d_hidden=256, d_feat=128, poly_degree=1, seed=92), 3),
    (W.replace(LOGIT_STD1, name="vdg_P4_linear", B=1, H=2, N=515, d_hidden=512, d_feat=512, poly_degree=4, seed=93), 0),
    (W.replace(SMALL, name="vdg_128_384_f32", B=1, H=2, N=450, dtype="f32", d_hidden=128, d_feat=384, poly_degree=3, seed=94), 2),
    # three layers: the P = 6 row of Tab. "phi", unequal widths, and the smallest shape
    (W.replace(SMALL, name="vdg_P6_3layer", B=1, H=2, N=600, d_hidden=768, d_mid=768, d_feat=768, poly_degree=6, seed=95), 4),
    (W.replace(SMALL, name="vdg_3layer_256_128_384", B=2, H=2, N=500, d_hidden=256, d_mid=128, d_feat=384, poly_degree=3, seed=96), 3),
    (W.replace(LOGIT_STD1, name="vdg_3layer_128", B=1, H=2, N=333, d_hidden=128, d_mid=128, d_feat=128, poly_degree=2, seed=97), 0),
]


@pytest.mark.parametrize("wl,R", WIDE_CASES, ids=[c[0].name for c in WIDE_CASES])
def test_wide_map_gradient_against_the_oracle(wl, R):
    """Backward pass alone, signs from the same stored outputs on both sides."""
    inp = bf16_representable(W.make_inputs(wl))
    fq, fk, y, yh, den = oracle_forward_pieces(inp, R)
    y_r, yh_r = round_io(y, wl.dtype), round_io(yh, wl.dtype)
    want = G.value_distill_grad(inp.q, inp.k, inp.v, fq, fk, R, wl.scale, sign_from=(y_r, yh_r))
    q, k, v, dq, dk = ha.to_device(inp)
    dt = q.dtype
    yt_d = torch.from_numpy(y_r).to(device="cuda", dtype=dt).contiguous()
    ys_d = torch.from_numpy(yh_r).to(device="cuda", dtype=dt).contiguous()
    den_d = torch.from_numpy(den).to(device="cuda", dtype=torch.float32).contiguous()
    print(f"  case {wl.name} R={R}", flush=True)
    loss, gq, gk, _, _, _ = ha.hybrid_attn_value_distill_grad(q, k, v, dq, dk, R, wl.block_size, wl.scale, y_teacher=yt_d,
                                                             teacher_is_cached=True, y_student=ys_d, row_den=den_d,
                                                             student_is_cached=True)
    torch.cuda.synchronize()
    worst = compare(f"{wl.name}_R{R}", (gq, gk), want)
    assert worst <= GRAD_REL_L2
    np.testing.assert_allclose(loss.cpu().numpy()[0], float(np.abs(y_r - yh_r).sum()), rtol=1e-5)


def test_wide_map_whole_step_and_replay():
    """Teacher, student, loss and backward in one call at the paper's default width; a second call on the stored
    student outputs reproduces every gradient bit for bit."""
    wl, R = WIDE_CASES[0]
    inp = W.make_inputs(wl)
    fq, fk, y, yh, den = oracle_forward_pieces(inp, R)
    want = G.value_distill_grad(inp.q, inp.k, inp.v, fq, fk, R, wl.scale)
    q, k, v, dq, dk = ha.to_device(inp)
    print(f"  case whole step {wl.name} R={R}", flush=True)
    loss, gq, gk, yt, ys, rd = ha.hybrid_attn_value_distill_grad(q, k, v, dq, dk, R, wl.block_size, wl.scale)
    torch.cuda.synchronize()
    np.testing.assert_allclose(rd.cpu().numpy(), den, rtol=5e-3)
    assert abs(loss.cpu().numpy()[0] - want[2]) <= 2e-2 * want[2]
    assert compare(f"whole_step_{wl.name}_R{R}", (gq, gk), want) <= 6e-2
    loss2, gq2, gk2, _, _, _ = ha.hybrid_attn_value_distill_grad(q, k, v, dq, dk, R, wl.block_size, wl.scale, y_teacher=yt,
                                                                teacher_is_cached=True, y_student=ys, row_den=rd,
                                                                student_is_cached=True)
    torch.cuda.synchronize()
    for a, b in ((gq, gq2), (gk, gk2)):
        for n in NAMES:
            assert torch.equal(a[n], b[n])
    assert torch.equal(loss, loss2)


def test_three_layer_whole_step():
    """Teacher, student, loss and backward in one call for a three-layer map."""
    wl, R = WIDE_CASES[6]
    inp = W.make_inputs(wl)
    fq, fk, y, yh, den = oracle_forward_pieces(inp, R)
    want = G.value_distill_grad(inp.q, inp.k, inp.v, fq, fk, R, wl.scale)
    q, k, v, dq, dk = ha.to_device(inp)
    print(f"  case whole step {wl.name} R={R}", flush=True)
    loss, gq, gk, yt, ys, rd = ha.hybrid_attn_value_distill_grad(q, k, v, dq, dk, R, wl.block_size, wl.scale)
    torch.cuda.synchronize()
    np.testing.assert_allclose(rd.cpu().numpy(), den, rtol=5e-3)
    assert abs(loss.cpu().numpy()[0] - want[2]) <= 2e-2 * want[2]
    assert compare(f"whole_step_{wl.name}_R{R}", (gq, gk), want) <= 6e-2
