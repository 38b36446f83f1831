"""Pins for the oracle's value-distillation loss (Sec. 3.3, Eq. "vd_loss"): || y - y_hat ||_1 between softmax
attention and hybrid attention of the same q, k, v."""
import numpy as np
import pytest

from oracle import hybrid_attn_oracle as O
from tests.test_oracle_pins import _const_map, _rand_map


def _inputs(seed, B=1, H=2, N=19, d=6):
    rng = np.random.default_rng(seed)
    return rng, tuple(rng.standard_normal((B, H, N, d)) for _ in range(3))


def test_teacher_against_itself_is_zero():
    """R = 1 makes the student the teacher (T_L empty): the loss is exactly 0."""
    rng, (q, k, v) = _inputs(0)
    fq, fk = _rand_map(rng, 2, 6, 8, 6, 2), _rand_map(rng, 2, 6, 8, 6, 2)
    assert O.value_distill_loss(q, k, v, fq, fk, 1, 0.4) == 0.0


def test_closed_form_with_constant_feature_map():
    """q = 0: the teacher output is the plain mean of all v rows; with a zero second layer the student is
    (sum_S v + kappa sum_L v) / (N_S + kappa N_L) for every row (Eq. "hybrid" with all softmax weights 1 and
    all linear weights kappa = D' sum_p F^(-2p)).  Both are the same for all N rows, so the loss is
    N x the 1-norm of their difference, summed over heads."""
    rng = np.random.default_rng(1)
    N, d, R, F, P, H = 14, 5, 4, 6, 2, 2
    q = np.zeros((1, H, N, d))
    k = rng.standard_normal((1, H, N, d))
    v = rng.standard_normal((1, H, N, d)) + np.arange(N)[None, None, :, None]
    fm = _const_map(H, d, 4, F, P)
    kappa = (F // P) * sum(float(F) ** (-2 * p) for p in range(1, P + 1))
    s_tok = [j for j in range(N) if j % R == 0]
    l_tok = [j for j in range(N) if j % R != 0]
    want = 0.0
    for h in range(H):
        teacher = v[0, h].mean(0)
        student = (v[0, h, s_tok].sum(0) + kappa * v[0, h, l_tok].sum(0)) / (len(s_tok) + kappa * len(l_tok))
        want += N * np.abs(teacher - student).sum()
    got = O.value_distill_loss(q, k, v, fm, fm, R, 0.5)
    np.testing.assert_allclose(got, want, rtol=1e-12)
    assert want > 0.1          # the case is not degenerate


def test_equals_the_loop_form():
    """Teacher and student outputs from the entry-by-entry N x N loop form, absolute differences added one
    by one in Python."""
    rng, (q, k, v) = _inputs(2, B=2, H=2, N=11, d=4)
    fq, fk = _rand_map(rng, 2, 4, 5, 6, 3), _rand_map(rng, 2, 4, 5, 6, 3)
    for R in (0, 2, 3):
        want = 0.0
        for b in range(2):
            for h in range(2):
                y = O.hybrid_attn_dense_loops(q[b, h], k[b, h], v[b, h], None, None, h, 1, 0.7)
                yh = O.hybrid_attn_dense_loops(q[b, h], k[b, h], v[b, h], fq, fk, h, R, 0.7)
                for i in range(y.shape[0]):
                    for c in range(y.shape[1]):
                        want += abs(float(y[i, c]) - float(yh[i, c]))
        np.testing.assert_allclose(O.value_distill_loss(q, k, v, fq, fk, R, 0.7), want, rtol=1e-11)


def test_scaling_and_additivity():
    """Both outputs are linear in v, so the loss is absolutely homogeneous in v; it is a sum over batch
    entries and heads, so it adds up over a split of the batch."""
    rng, (q, k, v) = _inputs(3, B=2)
    fq, fk = _rand_map(rng, 2, 6, 8, 6, 2), _rand_map(rng, 2, 6, 8, 6, 2)
    base = O.value_distill_loss(q, k, v, fq, fk, 4, 0.4)
    assert base > 0
    np.testing.assert_allclose(O.value_distill_loss(q, k, -2.5 * v, fq, fk, 4, 0.4), 2.5 * base, rtol=1e-12)
    parts = sum(O.value_distill_loss(q[b:b + 1], k[b:b + 1], v[b:b + 1], fq, fk, 4, 0.4) for b in range(2))
    np.testing.assert_allclose(parts, base, rtol=1e-12)


@pytest.mark.parametrize("kind", ["l2", "signed", "student_only"])
def test_planted_mistakes_are_caught(kind):
    """Variants with one mistake each must fail the closed-form pin."""
    rng = np.random.default_rng(1)
    N, d, R, F, P, H = 14, 5, 4, 6, 2, 2
    q = np.zeros((1, H, N, d))
    k = rng.standard_normal((1, H, N, d))
    v = rng.standard_normal((1, H, N, d)) + np.arange(N)[None, None, :, None]
    fm = _const_map(H, d, 4, F, P)
    good = O.value_distill_loss(q, k, v, fm, fm, R, 0.5)
    y = O.hybrid_attn(q, k, v, None, None, 1, 0.5)
    yh = O.hybrid_attn(q, k, v, fm, fm, R, 0.5)
    bad = {"l2": float(np.sqrt(((y - yh) ** 2).sum())), "signed": float((y - yh).sum()),
           "student_only": float(np.abs(yh).sum())}[kind]
    assert abs(bad - good) > 1e-3 * good
