"""GPU tests of the block-granular variant of the token split (not the paper's method: Sec. 3.2 splits per token;
this is the other reading of a "block rate"): groups of g consecutive tokens, every R-th group softmax tokens.
Everything downstream of the split is the same code, so each entry point is run once more on it."""
import numpy as np
import pytest
import torch

from oracle import hybrid_attn_oracle as O
from oracle import value_distill_grad_oracle as G
from paper_2509_24899_amd import hybrid_attn as ha
from paper_2509_24899_amd import workloads as W
from tests.test_gpu_parity import MAX_ABS, REL_L2, SMALL, SMALL64, metrics, oracle_map, record
from tests.test_gpu_value_distill_grad import GRAD_REL_L2, LOGIT_STD1, bf16_representable, compare, round_io

pytestmark = pytest.mark.gpu


def forward_case(name, inp, R, g, block_size=128, rows=None):
    w = inp.workload
    q, k, v, fq, fk = ha.to_device(inp)
    print(f"  case {name} R={R} g={g}", flush=True)
    y = ha.hybrid_attn_forward(q, k, v, fq, fk, (R, g), block_size, w.scale)
    torch.cuda.synchronize()
    y = y.float().cpu().numpy()
    ref = O.hybrid_attn(inp.q, inp.k, inp.v, oracle_map(inp.phi_q), oracle_map(inp.phi_k), O.BlockSplit(R, g), w.scale, rows=rows)
    if rows is not None:
        y = y[:, :, rows]
    assert np.isfinite(y).all()
    ma, rl = metrics(y, ref)
    record(name, ma, rl, R=R, g=g, N=w.N)
    assert ma <= MAX_ABS and rl <= REL_L2, (name, ma, rl)
    return y


@pytest.mark.parametrize("R,g", [(4, 32), (4, 128), (3, 7), (2, 64), (8, 100), (0, 16), (1, 16), (4, 1), (2, 1337), (5, 300)])
def test_forward_block_split(R, g):
    """Group sizes below, at and above the kernels' 32- and 128-token tiles, a last group that is cut short inside its
    softmax part (g = 300, 1337) or inside its linear part, and the degenerate rates."""
    forward_case(f"blocksplit_R{R}_g{g}", W.make_inputs(SMALL), R, g)
    forward_case(f"blocksplit_R{R}_g{g}_bs64", W.make_inputs(SMALL), R, g, block_size=64)


def test_granularity_one_is_the_token_rule():
    inp = W.make_inputs(SMALL)
    q, k, v, fq, fk = ha.to_device(inp)
    a = ha.hybrid_attn_forward(q, k, v, fq, fk, 4, 128, SMALL.scale)
    b = ha.hybrid_attn_forward(q, k, v, fq, fk, (4, 1), 128, SMALL.scale)
    c = ha.hybrid_attn_forward(q, k, v, fq, fk, (4, 0), 128, SMALL.scale)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(a, c)


def test_other_paths_block_split():
    """d_head = 64, the 256-wide fused map, a layer-by-layer map, [B, N, H, d] memory and the state tap."""
    forward_case("blocksplit_d64", W.make_inputs(SMALL64), 3, 48, block_size=64)
    w = W.replace(SMALL, B=1, H=2, d_hidden=256, d_feat=256, seed=50)
    forward_case("blocksplit_phi256", W.make_inputs(w), 4, 64)
    w = W.replace(SMALL, name="phi_P3", B=1, H=2, d_hidden=384, d_feat=384, poly_degree=3, seed=63)
    inp = W.make_inputs(w)
    forward_case("blocksplit_phi384", inp, 4, 50)
    _, k, v, _, fk = ha.to_device(inp)
    S, z = ha.hybrid_attn_linear_state(k, v, fk, (4, 50))
    torch.cuda.synchronize()
    for h in range(w.H):
        Sr, zr = O.linear_state(inp.k[0, h], inp.v[0, h], oracle_map(inp.phi_k), h, O.BlockSplit(4, 50))
        assert metrics(S.cpu().numpy()[0, h], Sr)[1] <= REL_L2 and metrics(z.cpu().numpy()[0, h], zr)[1] <= REL_L2


@pytest.mark.parametrize("wl,R,g", [(SMALL, 4, 32), (LOGIT_STD1, 2, 100),
                                     (W.replace(SMALL, name="vdg_bs_256", B=1, H=2, d_hidden=256, d_feat=256, seed=98), 3, 64)])
def test_value_distill_loss_and_gradient_block_split(wl, R, g):
    """Loss and gradient on the variant split: stored outputs decide the signs on both sides."""
    inp = bf16_representable(W.make_inputs(wl))
    fq, fk = oracle_map(inp.phi_q), oracle_map(inp.phi_k)
    split = O.BlockSplit(R, g)
    y = O.hybrid_attn(inp.q, inp.k, inp.v, None, None, 1, wl.scale)
    yh = O.hybrid_attn(inp.q, inp.k, inp.v, fq, fk, split, wl.scale)
    den = np.empty((wl.B, wl.H, wl.N))
    for b in range(wl.B):
        for h in range(wl.H):
            _, l, _ = O.softmax_part(inp.q[b, h], inp.k[b, h], inp.v[b, h], split, wl.scale)
            _, z = O.linear_state(inp.k[b, h], inp.v[b, h], fk, h, split)
            den[b, h] = l + O.feature_map(inp.q[b, h], fq, h) @ z
    y_r, yh_r = round_io(y, wl.dtype), round_io(yh, wl.dtype)
    want = G.value_distill_grad(inp.q, inp.k, inp.v, fq, fk, split, wl.scale, sign_from=(y_r, yh_r))
    q, k, v, dq, dk = ha.to_device(inp)
    dt = q.dtype
    yt_d = torch.from_numpy(y_r).to(device="cuda", dtype=dt).contiguous()
    ys_d = torch.from_numpy(yh_r).to(device="cuda", dtype=dt).contiguous()
    den_d = torch.from_numpy(den).to(device="cuda", dtype=torch.float32).contiguous()
    print(f"  case gradient {wl.name} R={R} g={g}", flush=True)
    loss, gq, gk, _, _, _ = ha.hybrid_attn_value_distill_grad(q, k, v, dq, dk, (R, g), wl.block_size, wl.scale, y_teacher=yt_d,
                                                             teacher_is_cached=True, y_student=ys_d, row_den=den_d,
                                                             student_is_cached=True)
    torch.cuda.synchronize()
    assert compare(f"blocksplit_{wl.name}_R{R}_g{g}", (gq, gk), want) <= GRAD_REL_L2
    np.testing.assert_allclose(loss.cpu().numpy()[0], float(np.abs(y_r - yh_r).sum()), rtol=1e-5)
    # the loss entry point from q, k, v
    loss2, _, ys2 = ha.hybrid_attn_value_distill_loss(q, k, v, dq, dk, (R, g), wl.block_size, wl.scale)
    torch.cuda.synchronize()
    ref = O.value_distill_loss(inp.q, inp.k, inp.v, fq, fk, split, wl.scale)
    assert abs(loss2.cpu().numpy()[0] - ref) <= 2e-2 * ref


def test_headline_shape_block_split_sampled_rows():
    """480p / 81 frames, groups of 128 tokens at R = 4: sampled query rows against the oracle."""
    wl = W.replace(W.WAN_480P_81F, H=2, seed=77)
    inp = W.make_inputs(wl)
    rows = np.concatenate([np.array([0, 127, 128, 511, 512, 640, 16383, 32759]), W.sample_rows(wl, n_random=48)])
    forward_case("blocksplit_headline_R4_g128", inp, 4, 128, rows=rows)
