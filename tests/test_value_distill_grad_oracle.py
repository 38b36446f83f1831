"""Pins for the oracle's gradient of the value-distillation loss with respect to the feature maps
(Sec. 3.3, Alg. "distil": phi <- phi - eta grad_phi L with L of Eq. "vd_loss")."""
import importlib.util
import inspect
import sys

import numpy as np
import pytest
import torch

from oracle import hybrid_attn_oracle as O
from oracle import value_distill_grad_oracle as G
from tests.test_oracle_pins import _rand_map

NAMES = ("w1", "b1", "w2", "b2")


def _inputs(seed, B=2, H=2, N=13, d=6):
    rng = np.random.default_rng(seed)
    return rng, tuple(rng.standard_normal((B, H, N, d)) for _ in range(3))


def _names(fm):
    return NAMES + (("w_mid", "b_mid") if fm.w_mid is not None else ())


def _with_mid(rng, fm, Dm):
    """The same map with one more hidden layer Hd -> Dm in front of the last layer (Tab. "phi", three layers)."""
    H, F, Hd = fm.w2.shape
    return O.FeatureMap(fm.w1, fm.b1, rng.standard_normal((H, F, Dm)) / np.sqrt(Dm), fm.b2, fm.P, fm.act,
                        w_mid=rng.standard_normal((H, Dm, Hd)) / np.sqrt(Hd), b_mid=rng.standard_normal((H, Dm)) * 0.3)


def _torch_loss_and_grads(q, k, v, fq, fk, R, scale):
    """The loss written once more with torch ops on float64 tensors (library softmax for the teacher, one
    concatenated weight matrix for the student) and differentiated by torch's reverse-mode autograd."""
    tq, tk, tv = (torch.tensor(t, dtype=torch.float64) for t in (q, k, v))
    B, H, N, d = q.shape
    par = {}
    for tag, fm in (("q", fq), ("k", fk)):
        par[tag] = [torch.tensor(getattr(fm, n), dtype=torch.float64, requires_grad=True) for n in _names(fm)]

    def phi(x, tag, fm, h):
        w1, b1, w2, b2 = par[tag][:4]
        hid = torch.relu(x @ w1[h].T + b1[h])
        if fm.w_mid is not None:
            hid = torch.relu(torch.nn.functional.linear(hid, par[tag][4][h], par[tag][5][h]))
        u = hid @ w2[h].T + b2[h]
        if fm.act == O.ACT_SOFTMAX:
            t = torch.softmax(u, dim=-1)
        elif fm.act == O.ACT_EXP:
            t = torch.exp(u)
        else:
            t = torch.relu(u)
        parts = torch.chunk(t, fm.P, dim=-1)
        return torch.cat([c ** (i + 1) for i, c in enumerate(parts)], dim=-1)

    is_s = torch.zeros(N, dtype=torch.bool) if R == 0 else (torch.arange(N) % R == 0)
    loss = torch.zeros((), dtype=torch.float64)
    for b in range(B):
        for h in range(H):
            logits = scale * tq[b, h] @ tk[b, h].T                              # [N, N]
            teacher = torch.softmax(logits, dim=-1) @ tv[b, h]
            w = torch.zeros(N, N, dtype=torch.float64)
            if is_s.any():
                ls = logits[:, is_s]
                w[:, is_s] = torch.exp(ls - ls.max(dim=1, keepdim=True).values)
            if (~is_s).any():
                w[:, ~is_s] = phi(tq[b, h], "q", fq, h) @ phi(tk[b, h][~is_s], "k", fk, h).T
            student = (w @ tv[b, h]) / w.sum(dim=1, keepdim=True)
            loss = loss + (teacher - student).abs().sum()
    if loss.requires_grad:
        loss.backward()
    grads = {tag: {n: (p.grad.numpy() if p.grad is not None else np.zeros(p.shape)) for n, p in zip(_names(fm), par[tag])}
             for tag, fm in (("q", fq), ("k", fk))}
    return float(loss.detach()), grads


def pin_against_autograd(M, seeds=(0, 1), acts=(O.ACT_SOFTMAX, O.ACT_EXP, O.ACT_RELU), rates=(0, 2, 3), three_layers=False):
    for seed in seeds:
        for act in acts:
            for R in rates:
                rng, (q, k, v) = _inputs(seed)
                fq, fk = _rand_map(rng, 2, 6, 8, 6, 3, act), _rand_map(rng, 2, 6, 8, 6, 2, act)
                if three_layers:
                    fq, fk = _with_mid(rng, fq, 5), _with_mid(rng, fk, 7)
                gq, gk, loss = M.value_distill_grad(q, k, v, fq, fk, R, 0.45)
                want_loss, want = _torch_loss_and_grads(q, k, v, fq, fk, R, 0.45)
                np.testing.assert_allclose(loss, want_loss, rtol=1e-11)
                for got, tag, fm in ((gq, "q", fq), (gk, "k", fk)):
                    assert set(got) == set(_names(fm))
                    for n in _names(fm):
                        scale_ = np.abs(want[tag][n]).max() + 1e-30
                        np.testing.assert_allclose(got[n], want[tag][n], rtol=1e-8, atol=1e-9 * scale_,
                                                   err_msg=f"seed {seed} act {act} R {R} phi_{tag}.{n}")


def test_matches_reverse_mode_autograd():
    pin_against_autograd(G)


def test_three_layer_map_matches_reverse_mode_autograd():
    """Tab. "phi", three-layer row: one more ReLU layer between the two (unequal widths 8 -> 5 / 7 -> 6)."""
    pin_against_autograd(G, three_layers=True)


THREE_LAYER_MUTATIONS = [
    ("dpre2 = (du @ fm.w2[head]) * (hidden2 > 0.0)", "dpre2 = du @ fm.w2[head]"),                    # second ReLU gate
    ("mid = (dpre2.T @ hidden, dpre2.sum(axis=0))", "mid = (dpre2.T @ hidden2[:, :1] * 0 + dpre2.T @ hidden * 2, dpre2.sum(axis=0))"),
    ("dhidden = dpre2 @ fm.w_mid[head]", "dhidden = dpre2 @ np.abs(fm.w_mid[head])"),               # wrong weights on the way down
    ("dw2 = du.T @ hidden2", "dw2 = du.T @ (hidden2 + 0.1)"),                                        # wrong activations
]


@pytest.mark.parametrize("old,new", THREE_LAYER_MUTATIONS)
def test_three_layer_planted_mistakes_are_caught(old, new):
    _mutant_must_fail(old, new, three_layers=True)


def test_matches_central_finite_differences_of_the_loss():
    """d loss / d theta for a handful of single parameters, from the loss oracle alone (which has its own
    pins).  The loss is piecewise smooth; the step is small enough that no |.| changes branch."""
    rng, (q, k, v) = _inputs(5, B=1)
    fq, fk = _rand_map(rng, 2, 6, 8, 6, 2), _rand_map(rng, 2, 6, 8, 6, 2)
    R, scale, eps = 3, 0.5, 1e-6
    gq, gk, loss = G.value_distill_grad(q, k, v, fq, fk, R, scale)
    np.testing.assert_allclose(loss, O.value_distill_loss(q, k, v, fq, fk, R, scale), rtol=1e-12)
    pick = np.random.default_rng(9)
    for fm, grads in ((fq, gq), (fk, gk)):
        for n in NAMES:
            arr = getattr(fm, n)
            for _ in range(3):
                idx = tuple(int(pick.integers(s)) for s in arr.shape)
                keep = arr[idx]
                arr[idx] = keep + eps
                up = O.value_distill_loss(q, k, v, fq, fk, R, scale)
                arr[idx] = keep - eps
                dn = O.value_distill_loss(q, k, v, fq, fk, R, scale)
                arr[idx] = keep
                fd = (up - dn) / (2 * eps)
                assert abs(fd - grads[n][idx]) <= 2e-5 * max(1.0, abs(fd)), (n, idx, fd, grads[n][idx])


@pytest.mark.parametrize("rows_per_chunk", (1, 4, 5, 13, 64))
def test_row_chunked_driver_equals_the_whole_head(rows_per_chunk):
    """head_gradients_by_row_chunks (rows taken a chunk at a time, for sequences whose N x N_S weights do not fit)
    against head_gradients on the same head: every tensor and the loss to rounding, for chunk lengths that divide N,
    that do not, of one row, and longer than N; with the sign pattern computed and handed in; R = 0, 1, 3."""
    rng, (q, k, v) = _inputs(5, B=1, H=2, N=13, d=6)
    fq, fk = _rand_map(rng, 2, 6, 7, 8, 2), _rand_map(rng, 2, 6, 7, 8, 2)
    for R in (0, 1, 3):
        for h in (0, 1):
            want_q, want_k, want_loss = G.head_gradients(q[0, h], k[0, h], v[0, h], fq, fk, h, R, 0.4)
            got_q, got_k, got_loss = G.head_gradients_by_row_chunks(q[0, h], k[0, h], v[0, h], fq, fk, h, R, 0.4,
                                                                    rows_per_chunk=rows_per_chunk)
            assert got_loss == pytest.approx(want_loss, rel=1e-12)
            for a, b in zip(got_q + got_k, want_q + want_k):
                np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-13)
            sign = rng.choice([-1.0, 0.0, 1.0], size=q[0, h].shape)
            want_q, want_k, _ = G.head_gradients(q[0, h], k[0, h], v[0, h], fq, fk, h, R, 0.4, sign)
            got_q, got_k, none = G.head_gradients_by_row_chunks(q[0, h], k[0, h], v[0, h], fq, fk, h, R, 0.4, sign,
                                                                rows_per_chunk=rows_per_chunk)
            assert none is None or R == 1
            for a, b in zip(got_q + got_k, want_q + want_k):
                np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-13)


def test_no_linear_tokens_no_gradient():
    """R = 1: T_L is empty, the student never evaluates phi, every gradient is exactly zero."""
    rng, (q, k, v) = _inputs(2)
    fq, fk = _rand_map(rng, 2, 6, 8, 6, 2), _rand_map(rng, 2, 6, 8, 6, 2)
    gq, gk, loss = G.value_distill_grad(q, k, v, fq, fk, 1, 0.4)
    assert loss == 0.0
    for g in (gq, gk):
        for n in NAMES:
            assert g[n].shape == getattr(fq, n).shape and not g[n].any()


def test_softmax_shift_invariance():
    """Adding one constant to all F second-layer biases of a head leaves a softmax map unchanged, so the b2
    gradient of every head sums to zero; phi_k's first-layer gradient vanishes for heads whose hidden units are
    all switched off (b1 very negative)."""
    rng, (q, k, v) = _inputs(3)
    fq, fk = _rand_map(rng, 2, 6, 8, 6, 2), _rand_map(rng, 2, 6, 8, 6, 3)
    fk.b1[1] = -1e3
    gq, gk, _ = G.value_distill_grad(q, k, v, fq, fk, 2, 0.4)
    for g in (gq, gk):
        assert np.abs(g["b2"].sum(axis=1)).max() <= 1e-12 * np.abs(g["b2"]).max()
    assert not gk["w1"][1].any() and not gk["b1"][1].any() and not gk["w2"][1].any()
    assert gk["b2"][1].any() and gk["w1"][0].any()


def test_batch_additivity_and_sign_override():
    """Parameters are shared over the batch: the gradient is the sum of per-sample gradients.  Handing in the
    exact outputs as `sign_from` changes nothing; flipping them flips every gradient."""
    rng, (q, k, v) = _inputs(4, B=2)
    fq, fk = _rand_map(rng, 2, 6, 8, 6, 2), _rand_map(rng, 2, 6, 8, 6, 2)
    R, scale = 4, 0.4
    gq, gk, loss = G.value_distill_grad(q, k, v, fq, fk, R, scale)
    parts = [G.value_distill_grad(q[b:b + 1], k[b:b + 1], v[b:b + 1], fq, fk, R, scale) for b in range(2)]
    y = O.hybrid_attn(q, k, v, None, None, 1, scale)
    y_hat = O.hybrid_attn(q, k, v, fq, fk, R, scale)
    same = G.value_distill_grad(q, k, v, fq, fk, R, scale, sign_from=(y, y_hat))
    flipped = G.value_distill_grad(q, k, v, fq, fk, R, scale, sign_from=(y_hat, y))
    for i, g in enumerate((gq, gk)):
        for n in NAMES:
            np.testing.assert_allclose(parts[0][i][n] + parts[1][i][n], g[n], rtol=1e-12, atol=1e-15)
            np.testing.assert_allclose(same[i][n], g[n], rtol=1e-13, atol=0)
            np.testing.assert_allclose(flipped[i][n], -g[n], rtol=1e-13, atol=0)


MUTATIONS = [
    ("dden = -(g * y_hat).sum(axis=1) / den", "dden = (g * y_hat).sum(axis=1) / den"),                 # sign of the denominator path
    ("dfq = dnum @ S.T + dden[:, None] * z[None, :]", "dfq = dnum @ S.T"),                             # dropped term
    ("dfk = v[idx_l] @ dS.T + dz[None, :]", "dfk = v[idx_l] @ dS + dz[None, :]"),                      # transposed operand
    ("du = t * (dt - (t * dt).sum(axis=-1, keepdims=True))", "du = t * dt"),                           # softmax Jacobian without its rank-one part
    ("dt[:, sl] = dphi[:, sl] * p * t[:, sl] ** (p - 1)", "dt[:, sl] = dphi[:, sl] * t[:, sl] ** (p - 1)"),  # power rule without p
    ("dpre = dhidden * (hidden > 0.0)", "dpre = dhidden"),                                             # ReLU gate
    ("dw2 = du.T @ hidden\n", "dw2 = du.T @ np.maximum(hidden, 0.1)\n"),                                   # wrong activations
    ("dS = fq.T @ dnum", "dS = fq.T @ g"),                                                             # missing 1/den
]


@pytest.mark.parametrize("old,new", MUTATIONS)
def test_planted_mistakes_are_caught(old, new):
    """A copy of the oracle's source with one mistake must fail the autograd pin."""
    _mutant_must_fail(old, new)


def _mutant_must_fail(old, new, three_layers=False):
    src = inspect.getsource(G)
    assert src.count(old) == 1, "mutation target not found: " + old
    spec = importlib.util.spec_from_loader("oracle._mutant_grad", loader=None)
    mod = importlib.util.module_from_spec(spec)
    mod.__package__ = "oracle"
    sys.modules["oracle._mutant_grad"] = mod
    try:
        exec(compile(src.replace(old, new), "<mutant>", "exec"), mod.__dict__)
        with pytest.raises((AssertionError, ValueError)):
            pin_against_autograd(mod, seeds=(0,), acts=(O.ACT_SOFTMAX,), rates=(2,), three_layers=three_layers)
    finally:
        del sys.modules["oracle._mutant_grad"]
