"""GPU tests of the parameter update (Sec. 3.3, Alg. 1: phi <- phi - eta grad_phi L; AdamW per the training details)
and of the inner loop it closes: repeated student updates on a cached teacher output."""
import numpy as np
import pytest
import torch

from oracle import hybrid_attn_oracle as O
from oracle import param_update_oracle as U
from oracle import value_distill_grad_oracle as G
from paper_2509_24899_amd import hybrid_attn as ha
from paper_2509_24899_amd import workloads as W
from tests.test_gpu_parity import SMALL, oracle_map
from tests.test_gpu_value_distill_grad import LOGIT_STD1

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n", (1, 255, 256, 257, 100003))
@pytest.mark.parametrize("io", ("bf16", "f32", None))
def test_update_rules_against_the_oracle(n, io):
    """Six steps of both rules, elementwise.  fp32 arithmetic against fp64: 1e-6 relative to the size of the numbers
    involved.  The io copy is a rounding decision: it is held to the round-to-nearest-even of the very master value the
    kernel stored."""
    rng = np.random.default_rng(n)
    p0 = rng.standard_normal(n)
    grads = [rng.standard_normal(n) * s for s in (1.0, 0.1, 3.0, 1e-3, 1.0, 0.5)]
    dev = "cuda"
    for kind in (ha.HA_OPT_SGD, ha.HA_OPT_ADAMW):
        master = torch.tensor(p0, dtype=torch.float32, device=dev)
        m, v = torch.zeros_like(master), torch.zeros_like(master)
        copy = None if io is None else torch.empty(n, dtype=torch.bfloat16 if io == "bf16" else torch.float32, device=dev)
        ref, rm, rv = master.cpu().numpy().astype(np.float64), np.zeros(n), np.zeros(n)
        for t, g in enumerate(grads, start=1):
            g32 = torch.tensor(g, dtype=torch.float32, device=dev)
            g64 = g32.cpu().numpy().astype(np.float64)
            if kind == ha.HA_OPT_SGD:
                ha.hybrid_attn_param_update(master, g32, 0.05, grad_scale=0.25, param_io=copy)
                ref = U.sgd_step(ref, g64, 0.05, grad_scale=0.25)
            else:
                ha.hybrid_attn_param_update(master, g32, 0.02, kind=kind, m=m, v=v, step=t, grad_scale=0.5, beta1=0.8, beta2=0.95,
                                            eps=1e-6, weight_decay=0.3, param_io=copy)
                ref, rm, rv = U.adamw_step(ref, g64, rm, rv, t, 0.02, np.float32(0.8), np.float32(0.95), np.float32(1e-6),
                                           np.float32(0.3), grad_scale=0.5)
            torch.cuda.synchronize()
            got = master.cpu().numpy().astype(np.float64)
            np.testing.assert_allclose(got, ref, rtol=2e-6, atol=2e-6)
            if kind == ha.HA_OPT_ADAMW:
                np.testing.assert_allclose(m.cpu().numpy(), rm, rtol=2e-6, atol=1e-7)
                np.testing.assert_allclose(v.cpu().numpy(), rv, rtol=2e-6, atol=1e-7)
            if copy is not None:
                assert torch.equal(copy, master.to(copy.dtype))


@pytest.mark.parametrize("kind", (ha.HA_OPT_SGD, ha.HA_OPT_ADAMW))
def test_inner_loop_of_the_distillation_reduces_the_loss(kind):
    """Alg. 1's inner loop on one cached batch: U student updates (forward, loss, gradient, update), fp32 master
    weights, bf16 weights for the forward.  The oracle runs the same loop in fp64 with its own gradients; the two loss
    curves are held to one per cent of each other (measured: 1e-3) (the signs of y_hat - y are decided on slightly different numbers, and each
    trajectory feeds on its own updates) and the loss goes down."""
    wl, R, steps = W.replace(LOGIT_STD1, B=1, H=2, N=300, seed=31), 4, 8
    inp = W.make_inputs(wl)
    q, k, v, dq, dk = ha.to_device(inp)
    fq, fk = oracle_map(inp.phi_q), oracle_map(inp.phi_k)
    names = ("w1", "b1", "w2", "b2")
    lr = 100.0 if kind == ha.HA_OPT_SGD else 1e-3      # the plain step needs a rate that suits the mean-scaled gradient; AdamW: the paper's 1e-3
    scale_g = 1.0 / (wl.N * wl.d)          # a mean instead of Alg. 1's plain sum over one sample: keeps the step sizes sane
    gpu_state = {}
    for tag, fm in (("q", dq), ("k", dk)):
        for n in names:
            t = getattr(fm, n)
            gpu_state[tag, n] = dict(master=t.float().clone() if t.dtype != torch.float32 else t,
                                     m=torch.zeros(t.shape, dtype=torch.float32, device="cuda"),
                                     v=torch.zeros(t.shape, dtype=torch.float32, device="cuda"))
    ref_state = {(tag, n): dict(m=np.zeros_like(getattr(fm, n)), v=np.zeros_like(getattr(fm, n)))
                 for tag, fm in (("q", fq), ("k", fk)) for n in names}
    yt = None
    gpu_loss, ref_loss = [], []
    for step in range(1, steps + 1):
        loss, gq, gk, yt, _, _ = ha.hybrid_attn_value_distill_grad(q, k, v, dq, dk, R, wl.block_size, wl.scale, y_teacher=yt,
                                                                   teacher_is_cached=yt is not None)
        gpu_loss.append(float(loss[0].item()))
        for tag, fm, g in (("q", dq, gq), ("k", dk, gk)):
            for n in names:
                s = gpu_state[tag, n]
                t = getattr(fm, n)
                ha.hybrid_attn_param_update(s["master"], g[n], lr, kind=kind, m=s["m"], v=s["v"], step=step, grad_scale=scale_g,
                                            param_io=None if t is s["master"] else t)
        rq, rk, rl = G.value_distill_grad(inp.q, inp.k, inp.v, fq, fk, R, wl.scale)
        ref_loss.append(rl)
        for tag, fm, g in (("q", fq, rq), ("k", fk, rk)):
            for n in names:
                arr = getattr(fm, n)
                if kind == ha.HA_OPT_SGD:
                    arr[...] = U.sgd_step(arr, g[n], lr, grad_scale=scale_g)
                else:
                    s = ref_state[tag, n]
                    arr[...], s["m"], s["v"] = U.adamw_step(arr, g[n], s["m"], s["v"], step, lr, grad_scale=scale_g)
    torch.cuda.synchronize()
    print("  gpu loss", [round(x, 2) for x in gpu_loss], flush=True)
    print("  ref loss", [round(x, 2) for x in ref_loss], flush=True)
    assert gpu_loss[-1] < 0.97 * gpu_loss[0] and ref_loss[-1] < 0.97 * ref_loss[0]
    np.testing.assert_allclose(gpu_loss, ref_loss, rtol=1e-2)


def test_student_update_under_hip_graph_capture():
    """One whole student update (student forward, loss, gradient, plain-step update of the eight parameter tensors) is a
    fixed sequence of launches on the caller's stream with no host synchronisation and no memset, so it can be captured
    into a HIP graph once and replayed per update.  Three replays, with eager work and synchronisations in between,
    must reproduce three eager updates bit for bit: the loss of every step and the final parameters."""
    wl, R, lr = W.replace(LOGIT_STD1, B=1, H=2, N=300, seed=32), 4, 50.0
    inp = W.make_inputs(wl)
    q, k, v, dq, dk = ha.to_device(inp)
    names = ("w1", "b1", "w2", "b2")
    scale_g = 1.0 / (wl.N * wl.d)
    prob = ha.make_problem(q, R, wl.block_size, wl.scale)
    ws = torch.empty(ha.hybrid_attn_value_distill_grad_workspace_bytes(prob, dq, dk), dtype=torch.uint8, device="cuda")
    start = {(tag, n): getattr(fm, n).clone() for tag, fm in (("q", dq), ("k", dk)) for n in names}
    masters = {key: (t.float().clone() if t.dtype != torch.float32 else None) for key, t in start.items()}
    _, _, _, yt, ys, rd = ha.hybrid_attn_value_distill_grad(q, k, v, dq, dk, R, wl.block_size, wl.scale, workspace=ws)
    torch.cuda.synchronize()

    def reset():
        for (tag, n), t in start.items():
            getattr(dq if tag == "q" else dk, n).copy_(t)
            if masters[tag, n] is not None:
                masters[tag, n].copy_(t.float())

    def one_update():
        loss, gq, gk, _, _, _ = ha.hybrid_attn_value_distill_grad(q, k, v, dq, dk, R, wl.block_size, wl.scale, y_teacher=yt,
                                                                  teacher_is_cached=True, y_student=ys, row_den=rd, workspace=ws,
                                                                  stream=torch.cuda.current_stream())
        for tag, fm, g in (("q", dq, gq), ("k", dk, gk)):
            for n in names:
                t = getattr(fm, n)
                m = masters[tag, n]
                ha.hybrid_attn_param_update(m if m is not None else t, g[n], lr, grad_scale=scale_g,
                                            param_io=t if m is not None else None, stream=torch.cuda.current_stream())
        return loss

    reset()
    eager_losses = []
    for _ in range(3):
        eager_losses.append(one_update().clone())
    torch.cuda.synchronize()
    eager_final = {(tag, n): getattr(dq if tag == "q" else dk, n).clone() for (tag, n) in start}
    assert eager_losses[2][0] < eager_losses[0][0]

    reset()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        one_update()                                    # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    reset()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        loss_g = one_update()
    reset()                                             # capture runs nothing; start the replays from the initial weights
    for rep in range(3):
        ws.random_(0, 255)                              # eager work between replays: the workspace holds garbage
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(loss_g, eager_losses[rep]), f"replay {rep}: loss differs from the eager update"
    for (tag, n), t in eager_final.items():
        assert torch.equal(getattr(dq if tag == "q" else dk, n), t), (tag, n)
