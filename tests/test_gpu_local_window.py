"""GPU tests of the local-window variant (the design Sec. 3.2 sets its uniform stride against, in a blocked form): the
softmax tokens of a query are its own tile of 2 * block_size tokens and W tokens on either side, every other token is
a linear token."""
import numpy as np
import pytest
import torch

from oracle import hybrid_attn_oracle as O
from paper_2509_24899_amd import hybrid_attn as ha
from paper_2509_24899_amd import workloads as W
from tests.test_gpu_parity import MAX_ABS, REL_L2, SMALL, SMALL64, metrics, oracle_map, record

pytestmark = pytest.mark.gpu


def window_case(name, inp, Wtok, block_size=128, rows=None, layout="bhnd"):
    w = inp.workload
    q, k, v, fq, fk = ha.to_device(inp)
    if layout == "bnhd":
        q, k, v = (t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in (q, k, v))
    T = 2 * block_size
    print(f"  case {name} W={Wtok} bs={block_size}", flush=True)
    y = ha.hybrid_attn_forward(q, k, v, fq, fk, (0, 0, 0, Wtok), block_size, w.scale)
    torch.cuda.synchronize()
    y = y.float().cpu().numpy()
    ref = O.hybrid_attn_local_window(inp.q, inp.k, inp.v, oracle_map(inp.phi_q), oracle_map(inp.phi_k), w.scale, T, Wtok // T, rows=rows)
    if rows is not None:
        y = y[:, :, rows]
    assert np.isfinite(y).all()
    ma, rl = metrics(y, ref)
    record(name, ma, rl, W=Wtok, N=w.N)
    assert ma <= MAX_ABS and rl <= REL_L2, (name, ma, rl)
    return y


@pytest.mark.parametrize("Wtok,bs", [(256, 128), (512, 128), (128, 64), (384, 64), (1024, 128), (2048, 128)])
def test_forward_local_window(Wtok, bs):
    """Windows of one to several tiles on either side at 1337 tokens (a short last tile), up to a window that covers the
    whole sequence for every query (then nothing is left for the linear part)."""
    window_case(f"window_W{Wtok}_bs{bs}", W.make_inputs(SMALL), Wtok, block_size=bs)


def test_window_over_everything_is_softmax_attention():
    inp = W.make_inputs(SMALL)
    q, k, v, fq, fk = ha.to_device(inp)
    a = ha.hybrid_attn_forward(q, k, v, None, None, 1, 128, SMALL.scale)
    b = ha.hybrid_attn_forward(q, k, v, fq, fk, (0, 0, 0, 1536), 128, SMALL.scale)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_other_paths_local_window():
    """d_head = 64, fp32 io, the 256-wide fused map, [B, N, H, d] memory, logits of unit scale."""
    window_case("window_d64", W.make_inputs(SMALL64), 128, block_size=64)
    window_case("window_tiny_f32", W.make_inputs(W.TINY), 256)
    w = W.replace(SMALL, B=1, H=2, d_hidden=256, d_feat=256, seed=50)
    window_case("window_phi256", W.make_inputs(w), 256)
    window_case("window_bnhd", W.make_inputs(SMALL), 256, layout="bnhd")
    window_case("window_logit_std1", W.make_inputs(W.replace(SMALL, seed=21, qk_gain=float(128 ** 0.5))), 256)


@pytest.mark.parametrize("N", (19, 128, 129, 257, 600))
def test_short_sequences_local_window(N):
    """Fewer tokens than one tile, exactly one tile, one token more, and a few tiles; window of one tile on either side."""
    w = W.replace(SMALL, N=N, B=1, H=2, seed=300 + N)
    window_case(f"window_N{N}", W.make_inputs(w), 128, block_size=64)
    window_case(f"window_N{N}_bs128", W.make_inputs(w), 256, block_size=128)


def test_local_window_rejected_where_it_has_no_kernels():
    inp = W.make_inputs(SMALL)
    q, k, v, fq, fk = ha.to_device(inp)
    with pytest.raises(ha.HybridAttnError):
        ha.hybrid_attn_forward(q, k, v, fq, fk, (4, 0, 0, 256), 128, SMALL.scale)         # needs rate 0
    with pytest.raises(ha.HybridAttnError):
        ha.hybrid_attn_forward(q, k, v, fq, fk, (0, 0, 0, 200), 128, SMALL.scale)         # not whole tiles
    with pytest.raises(ha.HybridAttnError):
        ha.hybrid_attn_value_distill_loss(q, k, v, fq, fk, (0, 0, 0, 256), 128, SMALL.scale)


def test_headline_shape_local_window_sampled_rows():
    """480p / 81 frames with a window of 1024 tokens on either side: sampled rows (first, last and interior tiles)."""
    wl = W.replace(W.WAN_480P_81F, H=2, seed=79)
    inp = W.make_inputs(wl)
    rows = np.unique(np.concatenate([np.array([0, 255, 256, 1279, 1280, 16383, 31487, 31488, 32759]), W.sample_rows(wl, n_random=40)]))
    window_case("window_headline_W1024", inp, 1024, rows=rows)
