"""Pins for the oracle's parameter update (Sec. 3.3, Alg. "distil", update line; AdamW per the appendix's training details)."""
import importlib.util
import inspect
import sys

import numpy as np
import pytest
import torch

from oracle import param_update_oracle as U


def _torch_run(opt_name, p0, grads, **kw):
    p = torch.nn.Parameter(torch.tensor(p0, dtype=torch.float64))
    opt = getattr(torch.optim, opt_name)([p], **kw)
    out = []
    for g in grads:
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        out.append(p.detach().numpy().copy())
    return out


def pin_against_torch(M):
    rng = np.random.default_rng(0)
    p0 = rng.standard_normal((5, 7))
    grads = [rng.standard_normal((5, 7)) * s for s in (1.0, 0.1, 3.0, 1e-3, 1.0, 0.5)]
    ref = _torch_run("SGD", p0, grads, lr=0.05)
    p = p0
    for g, r in zip(grads, ref):
        p = M.sgd_step(p, 4.0 * g, 0.05, grad_scale=0.25)
        np.testing.assert_allclose(p, r, rtol=1e-13, atol=1e-15)
    for kw in (dict(lr=1e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.01), dict(lr=0.02, betas=(0.8, 0.95), eps=1e-6, weight_decay=0.3)):
        ref = _torch_run("AdamW", p0, grads, **kw)
        p, m, v = p0, np.zeros_like(p0), np.zeros_like(p0)
        for t, (g, r) in enumerate(zip(grads, ref), start=1):
            p, m, v = M.adamw_step(p, 2.0 * g, m, v, t, kw["lr"], kw["betas"][0], kw["betas"][1], kw["eps"], kw["weight_decay"],
                                   grad_scale=0.5)
            np.testing.assert_allclose(p, r, rtol=1e-11, atol=1e-14)


def test_matches_torch_optimizers():
    pin_against_torch(U)


def test_first_adamw_step_closed_form():
    """With zero eps and decay the first step moves every entry by exactly lr against the sign of its gradient."""
    rng = np.random.default_rng(1)
    p0, g = rng.standard_normal(11), rng.standard_normal(11)
    p, m, v = U.adamw_step(p0, g, np.zeros(11), np.zeros(11), 1, 0.125, eps=0.0, weight_decay=0.0)
    np.testing.assert_allclose(p, p0 - 0.125 * np.sign(g), rtol=1e-13)
    np.testing.assert_allclose(m, 0.1 * g, rtol=1e-13)
    np.testing.assert_allclose(v, 0.001 * g * g, rtol=1e-12)
    with pytest.raises(ValueError):
        U.adamw_step(p0, g, m, v, 0, 0.1)


MUTATIONS = [
    ("p = p * (1.0 - lr * weight_decay)", "p = p - lr * weight_decay * g"),                      # coupled decay
    ("m_hat = m / (1.0 - beta1 ** step)", "m_hat = m"),                                          # no bias correction
    ("v_hat = v / (1.0 - beta2 ** step)", "v_hat = v / (1.0 - beta1 ** step)"),                  # wrong beta
    ("p = p - lr * m_hat / (np.sqrt(v_hat) + eps)", "p = p - lr * m_hat / np.sqrt(v_hat + eps)"),  # eps inside the root
    ("v = beta2 * np.asarray(v, dtype=np.float64) + (1.0 - beta2) * g * g", "v = beta2 * np.asarray(v, dtype=np.float64) + (1.0 - beta2) * np.abs(g)"),
    ("- lr * (grad_scale * np.asarray(grad, dtype=np.float64))", "- lr * np.asarray(grad, dtype=np.float64)"),   # scale dropped
]


@pytest.mark.parametrize("old,new", MUTATIONS)
def test_planted_mistakes_are_caught(old, new):
    src = inspect.getsource(U)
    assert src.count(old) == 1, "mutation target not found: " + old
    spec = importlib.util.spec_from_loader("oracle._mutant_update", loader=None)
    mod = importlib.util.module_from_spec(spec)
    sys.modules["oracle._mutant_update"] = mod
    try:
        exec(compile(src.replace(old, new), "<mutant>", "exec"), mod.__dict__)
        with pytest.raises(AssertionError):
            pin_against_torch(mod)
    finally:
        del sys.modules["oracle._mutant_update"]
