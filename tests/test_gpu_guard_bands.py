"""Memory safety of every entry point, shown without faulting anything: each buffer the library WRITES (outputs and the
workspace) is carved out of a larger allocation with sentinel-filled guard bands on both sides; the workspace is filled
with NaN bit patterns before the run (the header says its contents are undefined, so nothing may be read before it is
written).  After the run the bands must be untouched, the outputs finite, and equal bit for bit to those of an ordinary
call.  Sizes: the degenerate ones (single token, fewer tokens than a wave / a tile, one past a tile, ragged tails), both
block sizes, both head widths and io dtypes, every feature-map path, the three variants of the token split, and the
480p / 81-frame configuration at full size."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2509_24899_amd import hybrid_attn as ha
from paper_2509_24899_amd import workloads as W

pytestmark = pytest.mark.gpu

BAND = 1 << 16          # bytes of guard on either side of every carved buffer
SENTINEL = 0xA5


class Carved:
    """`nbytes` of device memory with a guard band before and after it."""

    def __init__(self, nbytes, fill=None):
        self.nbytes = int(nbytes)
        pad = (-self.nbytes) % 256
        self.buf = torch.full((BAND + self.nbytes + pad + BAND,), SENTINEL, dtype=torch.uint8, device="cuda")
        assert self.buf.data_ptr() % 256 == 0
        self.payload = self.buf[BAND:BAND + self.nbytes]
        if fill is not None:
            self.payload.fill_(fill)

    def ptr(self):
        return self.payload.data_ptr()

    def tensor(self, dtype, shape):
        return self.payload.view(dtype).view(shape)

    def check(self, what):
        lo, hi = self.buf[:BAND], self.buf[BAND + self.nbytes:]
        assert bool((lo == SENTINEL).all()), f"{what}: bytes BEFORE the buffer were written"
        assert bool((hi == SENTINEL).all()), f"{what}: bytes AFTER the buffer were written"


def carved_like(t):
    c = Carved(t.numel() * t.element_size(), fill=0xFF)
    return c, c.tensor(t.dtype, t.shape)


def poisoned_workspace(nbytes):
    return Carved(max(int(nbytes), 256), fill=0xFF)       # 0xFF.. is a NaN in bf16, fp32 and fp64


def run_forward(w, rate=None, act=ha.HA_ACT_SOFTMAX):
    inp = W.make_inputs(w)
    q, k, v, fq, fk = ha.to_device(inp)
    fq.out_act = fk.out_act = act
    rate = w.rate if rate is None else rate
    R = rate[0] if isinstance(rate, tuple) else rate
    if R == 1 and not (isinstance(rate, tuple) and len(rate) == 4):
        fq = fk = None
    want = ha.hybrid_attn_forward(q, k, v, fq, fk, rate, w.block_size, w.scale)
    prob = ha.make_problem(q, rate, w.block_size, w.scale)
    ws = poisoned_workspace(ha.hybrid_attn_workspace_bytes(prob, fq, fk))
    oc, out = carved_like(q)
    ha.hybrid_attn_forward(q, k, v, fq, fk, rate, w.block_size, w.scale, out=out, workspace=ws.payload)
    torch.cuda.synchronize()
    ws.check(f"{w.name}: workspace")
    oc.check(f"{w.name}: out")
    assert torch.isfinite(out.float()).all().item(), w.name
    assert torch.equal(out, want), w.name
    # the static-scratch entry point writes `out` only
    if ha.hybrid_attn_workspace_bytes(prob, fq, fk) <= ha.hybrid_attn_static_scratch_bytes():
        oc2, out2 = carved_like(q)
        ha.hybrid_attn_forward_static(q, k, v, fq, fk, rate, out2, w.block_size, w.scale)
        torch.cuda.synchronize()
        oc2.check(f"{w.name}: out (static scratch)")
        assert torch.equal(out2, want), w.name


BASE = W.Workload("guard", 1, 2, 300, 128, "bf16", 128, 4, 128, 128, seed=400)


@pytest.mark.parametrize("N,R", [(1, 1), (1, 0), (2, 2), (5, 2), (31, 4), (32, 3), (33, 33), (64, 1), (65, 64), (127, 0), (128, 4),
                                 (129, 4), (130, 4), (255, 8), (256, 2), (257, 0), (300, 7), (1337, 4)])
@pytest.mark.parametrize("bs", (64, 128))
def test_forward_degenerate_sizes(N, R, bs):
    print(f"  case guard N={N} R={R} bs={bs}", flush=True)
    run_forward(W.replace(BASE, N=N, R=R, block_size=bs, seed=400 + N))


@pytest.mark.parametrize("d,dtype", [(64, "bf16"), (64, "f32"), (128, "f32")])
@pytest.mark.parametrize("N,R", [(1, 0), (33, 4), (131, 3), (777, 1)])
def test_forward_other_head_widths_and_dtypes(d, dtype, N, R):
    print(f"  case guard d={d} {dtype} N={N} R={R}", flush=True)
    run_forward(W.replace(BASE, B=2, N=N, R=R, d=d, d_hidden=d, d_feat=d, dtype=dtype, seed=500 + N))


@pytest.mark.parametrize("Hd,F,Dm,P", [(256, 256, 0, 2), (384, 384, 0, 3), (512, 256, 0, 2), (768, 768, 768, 6), (256, 128, 128, 1)])
@pytest.mark.parametrize("N,R", [(19, 4), (161, 0), (700, 3)])
def test_forward_every_feature_map_path(Hd, F, Dm, P, N, R):
    print(f"  case guard map {Hd}/{Dm}/{F} N={N} R={R}", flush=True)
    run_forward(W.replace(BASE, N=N, R=R, d_hidden=Hd, d_feat=F, d_mid=Dm, poly_degree=P, seed=600 + N))
    run_forward(W.replace(BASE, N=N, R=R, d_hidden=Hd, d_feat=F, d_mid=Dm, poly_degree=P, seed=600 + N, block_size=64),
                act=ha.HA_ACT_RELU)


@pytest.mark.parametrize("bs", (64, 128))
def test_forward_variants_of_the_split(bs):
    T = 2 * bs
    for N in (T - 1, T + 1, 5 * T + 17):
        print(f"  case guard variants N={N} bs={bs}", flush=True)
        run_forward(W.replace(BASE, N=N, R=3, block_size=bs, split_granularity=8, seed=700 + N))
        run_forward(W.replace(BASE, N=N, R=2, block_size=bs, split_granularity=bs + 3, seed=701 + N))
        run_forward(W.replace(BASE, N=N, R=4, block_size=bs, causal_chunk=T, seed=702 + N))
        run_forward(W.replace(BASE, N=N, R=4, block_size=bs, causal_chunk=2 * T, split_granularity=5, seed=703 + N))
        run_forward(W.replace(BASE, N=N, R=0, block_size=bs, local_window=T, seed=704 + N))
        run_forward(W.replace(BASE, N=N, R=0, block_size=bs, local_window=3 * T, d_hidden=256, d_feat=256, seed=705 + N))


def test_forward_full_size_config():
    """480p / 81 frames, 12 heads, R = 4, block 128: the configuration bench.py times."""
    print("  case guard full size", flush=True)
    run_forward(W.WAN_480P_81F)


def test_forward_strided_layout_writes_only_its_rows():
    """[B, H, N, d] views over [B, N, H, d] memory: `out` is the strided view of a carved buffer."""
    w = W.replace(BASE, B=2, H=3, N=333, seed=800)
    q, k, v, fq, fk = ha.to_device(W.make_inputs(w))
    q, k, v = (t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in (q, k, v))
    want = ha.hybrid_attn_forward(q, k, v, fq, fk, w.R, w.block_size, w.scale)
    oc = Carved(q.numel() * 2, fill=0xFF)
    out = oc.tensor(torch.bfloat16, (w.B, w.N, w.H, w.d)).permute(0, 2, 1, 3)
    ws = poisoned_workspace(ha.hybrid_attn_workspace_bytes(ha.make_problem(q, w.R, w.block_size, w.scale), fq, fk))
    ha.hybrid_attn_forward(q, k, v, fq, fk, w.R, w.block_size, w.scale, out=out, workspace=ws.payload)
    torch.cuda.synchronize()
    oc.check("strided out")
    ws.check("strided workspace")
    assert torch.equal(out, want)


def _fm(fm):
    s = fm.c_struct()
    return s, ctypes.byref(s)


@pytest.mark.parametrize("N,R,Hd", [(1, 0, 128), (33, 4, 128), (300, 3, 128), (300, 0, 256), (131, 2, 384)])
def test_linear_state_tap(N, R, Hd):
    w = W.replace(BASE, N=N, R=R, d_hidden=Hd, d_feat=Hd, poly_degree=Hd // 128, seed=900 + N)
    _, k, v, _, fk = ha.to_device(W.make_inputs(w))
    S_want, z_want = ha.hybrid_attn_linear_state(k, v, fk, R)
    prob = ha.make_problem(k, R, w.block_size, 1.0)
    sk, pk = _fm(fk)
    ws = poisoned_workspace(ha.hybrid_attn_workspace_bytes(prob, fk, fk))
    Sc, S = carved_like(S_want)
    zc, z = carved_like(z_want)
    st = ha._lib().hybrid_attn_linear_state(ctypes.byref(prob), k.data_ptr(), v.data_ptr(), pk, S.data_ptr(), z.data_ptr(), ws.ptr(),
                                            ws.nbytes, torch.cuda.current_stream().cuda_stream)
    assert st == ha.HA_OK
    torch.cuda.synchronize()
    for c, what in ((ws, "workspace"), (Sc, "S"), (zc, "z")):
        c.check(f"linear_state {what}")
    assert torch.equal(S, S_want) and torch.equal(z, z_want)


@pytest.mark.parametrize("N,R,Hd,Dm,dtype", [(1, 0, 128, 0, "bf16"), (37, 4, 128, 0, "bf16"), (300, 3, 128, 0, "f32"), (161, 2, 256, 0, "bf16"),
                                             (131, 4, 384, 0, "bf16"), (200, 4, 256, 128, "bf16"), (64, 1, 128, 0, "bf16")])
def test_value_distill_loss_and_gradient(N, R, Hd, Dm, dtype):
    """Teacher, student, loss, row denominators, all gradient tensors and both workspaces carved."""
    F = 128 if Dm else Hd
    w = W.replace(BASE, N=N, R=R, d_hidden=Hd, d_feat=F, d_mid=Dm, poly_degree=2 if F % 2 == 0 else 1, dtype=dtype, seed=1000 + N)
    q, k, v, fq, fk = ha.to_device(W.make_inputs(w))
    print(f"  case guard distill N={N} R={R} map {Hd}/{Dm}/{F} {dtype}", flush=True)
    want = ha.hybrid_attn_value_distill_grad(q, k, v, fq, fk, R, w.block_size, w.scale)
    torch.cuda.synchronize()
    lib = ha._lib()
    prob = ha.make_problem(q, R, w.block_size, w.scale)
    sq, pq = _fm(fq)
    sk, pk = _fm(fk)
    stream = torch.cuda.current_stream().cuda_stream
    # loss entry point
    ws = poisoned_workspace(lib.hybrid_attn_value_distill_workspace_bytes(ctypes.byref(prob), pq, pk))
    ytc, yt = carved_like(q)
    ysc, ys = carved_like(q)
    lc, loss = carved_like(want[0])
    st = lib.hybrid_attn_value_distill_loss(ctypes.byref(prob), q.data_ptr(), k.data_ptr(), v.data_ptr(), pq if R != 1 else None,
                                            pk if R != 1 else None, 0, yt.data_ptr(), ys.data_ptr(), loss.data_ptr(), ws.ptr(),
                                            ws.nbytes, stream)
    assert st == ha.HA_OK
    torch.cuda.synchronize()
    for c, what in ((ws, "workspace"), (ytc, "y_teacher"), (ysc, "y_student"), (lc, "loss")):
        c.check(f"value_distill_loss {what}")
    assert torch.equal(loss, want[0]) and torch.equal(yt, want[3]) and torch.equal(ys, want[4])
    # gradient entry point
    ws = poisoned_workspace(lib.hybrid_attn_value_distill_grad_workspace_bytes(ctypes.byref(prob), pq, pk))
    ytc, yt = carved_like(q)
    ysc, ys = carved_like(q)
    lc, loss = carved_like(want[0])
    dc, den = carved_like(want[5])
    carved, structs = [], []
    for g in (want[1], want[2]):
        cs = {n: carved_like(t) for n, t in g.items()}
        carved.append(cs)
        structs.append(ha.ha_feature_map_grad(cs["w1"][1].data_ptr(), cs["b1"][1].data_ptr(), cs["w2"][1].data_ptr(), cs["b2"][1].data_ptr(),
                                              cs["w_mid"][1].data_ptr() if "w_mid" in cs else None,
                                              cs["b_mid"][1].data_ptr() if "b_mid" in cs else None))
    st = lib.hybrid_attn_value_distill_grad(ctypes.byref(prob), q.data_ptr(), k.data_ptr(), v.data_ptr(), pq, pk, 0, 0, yt.data_ptr(),
                                            ys.data_ptr(), den.data_ptr(), loss.data_ptr(), ctypes.byref(structs[0]),
                                            ctypes.byref(structs[1]), ws.ptr(), ws.nbytes, stream)
    assert st == ha.HA_OK
    torch.cuda.synchronize()
    for c, what in ((ws, "workspace"), (ytc, "y_teacher"), (ysc, "y_student"), (lc, "loss"), (dc, "row_den")):
        c.check(f"value_distill_grad {what}")
    assert torch.equal(loss, want[0]) and torch.equal(ys, want[4])
    if R != 1:
        assert torch.equal(den, want[5])
    for cs, g, side in ((carved[0], want[1], "phi_q"), (carved[1], want[2], "phi_k")):
        for n, (c, t) in cs.items():
            c.check(f"value_distill_grad grad {side}.{n}")
            assert torch.isfinite(t).all().item()
            assert torch.equal(t, g[n]), (side, n)


@pytest.mark.parametrize("n", (1, 7, 255, 256, 257, 128 * 128 + 3))
@pytest.mark.parametrize("kind", (ha.HA_OPT_SGD, ha.HA_OPT_ADAMW))
def test_param_update(n, kind):
    gen = torch.Generator(device="cuda").manual_seed(n)
    src = [torch.randn(n, generator=gen, device="cuda") for _ in range(2)]
    cm, master = carved_like(src[0])
    master.copy_(src[0])
    cmm, m = carved_like(src[0])
    cv, v = carved_like(src[0])
    m.zero_()
    v.zero_()
    cio, io = Carved(n * 2, fill=0xFF), None
    io = cio.tensor(torch.bfloat16, (n,))
    ha.hybrid_attn_param_update(master, src[1], 1e-2, kind=kind, m=m if kind == ha.HA_OPT_ADAMW else None,
                                v=v if kind == ha.HA_OPT_ADAMW else None, step=1, param_io=io)
    torch.cuda.synchronize()
    for c, what in ((cm, "master"), (cmm, "m"), (cv, "v"), (cio, "param_io")):
        c.check(f"param_update {what}")
    assert torch.isfinite(master).all().item() and torch.equal(io, master.to(torch.bfloat16))
