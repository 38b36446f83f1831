"""fp64 CPU oracle for the gradient of the value-distillation objective with respect to the
feature maps (Sec. 3.3: Alg. "distil", the update of phi = (phi_q, phi_k); Eq. "vd_loss").

TEST INFRASTRUCTURE ONLY.  Plain chain rule, written out step by step in float64.  It shares no
code with the GPU library and must never be imported by the product path.

What it computes.  With q, k, v fixed (in the distillation stage everything but phi is frozen, so
the attention inputs of the isolated layer are constants), the loss is

    L = sum_{b,h,i,c} | y_i,c - y_hat_i,c |,     y = softmax attention (Eq. "softmax"),
                                                  y_hat = hybrid attention (Eq. "hybrid")

and y_hat_i = num_i / den_i with num_i = a_i + phi_q(q_i) S, den_i = l_i + phi_q(q_i) . z,
S = sum_{T_L} phi_k(k_j)^T v_j, z = sum_{T_L} phi_k(k_j); a_i, l_i (the softmax-token sums) do
not depend on phi.  The derivative is taken where it exists; at y_hat = y the subgradient 0 is
used (sign(0) = 0).  Returned are dL/dW1, dL/db1, dL/dW2, dL/db2 (and dL/dW_mid, dL/db_mid for the
three-layer map of Tab. "phi") of phi_q and of phi_k per head, summed over the batch (the parameters are shared by the batch; Alg. "distil" then divides by the
number of samples, which is left to the caller).

Readings taken: the loss is the plain sum (no mean); phi_q and phi_k are separate parameter sets;
the sign pattern may be handed in (`sign_from`) as the pair of tensors both sides of a parity test
look at, so that the one discontinuous decision of the gradient is taken from the same numbers.

Pins (tests/test_value_distill_grad_oracle.py): reverse-mode automatic differentiation of an
independent torch expression of the loss; central finite differences of the pinned loss oracle;
exact zeros at R = 1; the shift invariance of the channel softmax (the b2 gradient sums to zero
per head); planted mistakes that these must reject.  No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

from . import hybrid_attn_oracle as O


def feature_map_with_trace(x, fm: O.FeatureMap, head: int):
    """phi(x) of Sec. 3.2 together with what its derivative needs: rows x [n, d] ->
    (phi [n, F], hidden [n, Hd], pre-activation u [n, F], positive output t [n, F], second hidden
    layer [n, Dm] of a three-layer map or None)."""
    x = np.asarray(x, dtype=np.float64)
    pre = x @ fm.w1[head].T + fm.b1[head]
    hidden = np.maximum(pre, 0.0)
    hidden2 = None
    if fm.w_mid is not None:
        hidden2 = np.maximum(hidden @ fm.w_mid[head].T + fm.b_mid[head], 0.0)
    last_in = hidden if hidden2 is None else hidden2
    u = last_in @ fm.w2[head].T + fm.b2[head]
    if fm.act == O.ACT_SOFTMAX:
        e = np.exp(u - u.max(axis=-1, keepdims=True))
        t = e / e.sum(axis=-1, keepdims=True)
    elif fm.act == O.ACT_EXP:
        t = np.exp(u)
    elif fm.act == O.ACT_RELU:
        t = np.maximum(u, 0.0)
    else:
        raise ValueError("unknown activation")
    Dp = fm.F // fm.P
    phi = np.empty_like(t)
    for p in range(1, fm.P + 1):
        sl = slice((p - 1) * Dp, p * Dp)
        phi[:, sl] = t[:, sl] ** p
    return phi, hidden, u, t, hidden2


def feature_map_backward(x, fm: O.FeatureMap, head: int, dphi):
    """Given dL/dphi [n, F] for rows x [n, d], the gradient with respect to the parameters of the
    map of this head: (dW1 [Hd, d], db1 [Hd], dW2 [F, Hd or Dm], db2 [F]) and, for a three-layer map,
    (dW_mid [Dm, Hd], db_mid [Dm]) behind them."""
    x = np.asarray(x, dtype=np.float64)
    _, hidden, u, t, hidden2 = feature_map_with_trace(x, fm, head)
    Dp = fm.F // fm.P
    dt = np.empty_like(t)
    for p in range(1, fm.P + 1):                         # phi_c = t_c ** p on slice p
        sl = slice((p - 1) * Dp, p * Dp)
        dt[:, sl] = dphi[:, sl] * p * t[:, sl] ** (p - 1)
    if fm.act == O.ACT_SOFTMAX:                           # t = softmax(u) over the F channels
        du = t * (dt - (t * dt).sum(axis=-1, keepdims=True))
    elif fm.act == O.ACT_EXP:
        du = dt * t
    else:                                                 # ReLU
        du = dt * (u > 0.0)
    db2 = du.sum(axis=0)
    if hidden2 is None:
        dw2 = du.T @ hidden
        dhidden = du @ fm.w2[head]
        mid = ()
    else:                                                 # one more ReLU layer between the two
        dw2 = du.T @ hidden2
        dpre2 = (du @ fm.w2[head]) * (hidden2 > 0.0)
        mid = (dpre2.T @ hidden, dpre2.sum(axis=0))
        dhidden = dpre2 @ fm.w_mid[head]
    dpre = dhidden * (hidden > 0.0)
    dw1 = dpre.T @ x
    db1 = dpre.sum(axis=0)
    return (dw1, db1, dw2, db2) + mid


def param_names(fm: O.FeatureMap):
    """Names of the parameter tensors of a map, in the order feature_map_backward returns their gradients."""
    return ("w1", "b1", "w2", "b2") + (("w_mid", "b_mid") if fm.w_mid is not None else ())


def head_gradients(q, k, v, phi_q, phi_k, head, R, scale, sign=None):
    """One (batch, head): q, k, v [N, d] -> (grads of phi_q, grads of phi_k, loss), each grads a tuple
    (dW1, db1, dW2, db2[, dW_mid, db_mid]).  `sign` [N, d], if given, replaces sign(y_hat - y)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    N, d = q.shape
    _, idx_l = O.token_split(N, R)
    a_t, l_t, _ = O.softmax_part(q, k, v, 1, scale)                 # teacher: every token a softmax token
    y = a_t / l_t[:, None]
    a, l, _ = O.softmax_part(q, k, v, R, scale)                     # student's softmax-token sums
    if idx_l.size == 0:                                             # no linear tokens: phi is unused
        zq = tuple(np.zeros_like(getattr(phi_q, n)[head]) for n in param_names(phi_q))
        zk = tuple(np.zeros_like(getattr(phi_k, n)[head]) for n in param_names(phi_k))
        return zq, zk, float(np.abs(y - a / l[:, None]).sum())
    fk = O.feature_map(k[idx_l], phi_k, head)                       # [N_L, F]
    S = fk.T @ v[idx_l]
    z = fk.sum(axis=0)
    fq = O.feature_map(q, phi_q, head)                              # [N, F]
    num = a + fq @ S
    den = l + fq @ z
    y_hat = num / den[:, None]
    g = np.sign(y_hat - y) if sign is None else np.asarray(sign, dtype=np.float64)   # dL/dy_hat
    dnum = g / den[:, None]                                         # y_hat = num / den
    dden = -(g * y_hat).sum(axis=1) / den
    dfq = dnum @ S.T + dden[:, None] * z[None, :]                   # through num and den to phi_q(q_i)
    dS = fq.T @ dnum
    dz = fq.T @ dden
    dfk = v[idx_l] @ dS.T + dz[None, :]                             # through S and z to phi_k(k_j), j in T_L
    gq = feature_map_backward(q, phi_q, head, dfq)
    gk = feature_map_backward(k[idx_l], phi_k, head, dfk)
    return gq, gk, float(np.abs(y - y_hat).sum())


def head_gradients_by_row_chunks(q, k, v, phi_q, phi_k, head, R, scale, sign=None, rows_per_chunk=2048):
    """head_gradients for sequences too long to hold the N x N_S weights at once.  Every sum over the query tokens i
    (the state gradients dS, dz and the parameter gradients of phi_q) is a plain sum of per-row terms, so the rows are
    taken `rows_per_chunk` at a time and their contributions added up; S, z and the key-side chain are as in
    head_gradients.  Same return value; with `sign` given the teacher is not evaluated and the loss is None.
    Pinned against head_gradients on small inputs with chunk lengths that do and do not divide N."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    N, d = q.shape
    _, idx_l = O.token_split(N, R)
    if idx_l.size == 0:
        return head_gradients(q, k, v, phi_q, phi_k, head, R, scale, sign)
    fk = O.feature_map(k[idx_l], phi_k, head)
    S = fk.T @ v[idx_l]
    z = fk.sum(axis=0)
    dS = np.zeros_like(S)
    dz = np.zeros_like(z)
    gq = None
    loss = 0.0 if sign is None else None
    for lo in range(0, N, rows_per_chunk):
        rows = slice(lo, min(lo + rows_per_chunk, N))
        a, l, _ = O.softmax_part(q[rows], k, v, R, scale)
        fq = O.feature_map(q[rows], phi_q, head)
        den = l + fq @ z
        y_hat = (a + fq @ S) / den[:, None]
        if sign is None:
            a_t, l_t, _ = O.softmax_part(q[rows], k, v, 1, scale)
            y = a_t / l_t[:, None]
            g = np.sign(y_hat - y)
            loss += float(np.abs(y - y_hat).sum())
        else:
            g = np.asarray(sign[rows], dtype=np.float64)
        dnum_rows = g / den[:, None]
        dden_rows = -(g * y_hat).sum(axis=1) / den
        dS += fq.T @ dnum_rows
        dz += fq.T @ dden_rows
        part = feature_map_backward(q[rows], phi_q, head, dnum_rows @ S.T + dden_rows[:, None] * z[None, :])
        gq = part if gq is None else tuple(x + y_ for x, y_ in zip(gq, part))
    gk = feature_map_backward(k[idx_l], phi_k, head, v[idx_l] @ dS.T + dz[None, :])
    return gq, gk, loss


def value_distill_grad(q, k, v, phi_q, phi_k, R, scale, sign_from=None):
    """Gradient of the value-distillation loss for q, k, v [B, H, N, d].

    `sign_from` = (y_teacher, y_student), both [B, H, N, d]: when given, dL/dy_hat is the sign of
    their difference (student minus teacher) instead of the sign of the float64 values computed here.
    Returns (grads_q, grads_k, loss): grads_* is a dict with w1 [H, Hd, d], b1 [H, Hd], w2 [H, F, Hd],
    b2 [H, F] (three-layer maps: w2 [H, F, Dm], w_mid [H, Dm, Hd], b_mid [H, Dm]), summed over the batch."""
    B, H, N, d = q.shape

    def zeros(fm):
        return {n: np.zeros_like(getattr(fm, n)) for n in param_names(fm)}

    out_q, out_k, loss = zeros(phi_q), zeros(phi_k), 0.0
    for b in range(B):
        for h in range(H):
            sign = None
            if sign_from is not None:
                sign = np.sign(np.asarray(sign_from[1][b, h], dtype=np.float64) - np.asarray(sign_from[0][b, h], dtype=np.float64))
            gq, gk, l_bh = head_gradients(q[b, h], k[b, h], v[b, h], phi_q, phi_k, h, R, scale, sign)
            for out, g, fm in ((out_q, gq, phi_q), (out_k, gk, phi_k)):
                for name, t in zip(param_names(fm), g):
                    out[name][h] += t
            loss += l_bh
    return out_q, out_k, loss
