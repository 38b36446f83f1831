"""Pins for the fp64 oracle: everything the paper and the mathematics fix without any GPU code.

Each `pin_*` function takes the oracle module and asserts one fact.  They run against the real
oracle (must pass) and against planted-mistake variants of it (at least one pin must fail for
every mistake), which shows that the pin set can tell a wrong oracle from a right one.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import torch

from oracle import hybrid_attn_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_map(rng, H, d, Hd, F, P, act=O.ACT_SOFTMAX, gain=1.0, mod=O):
    return mod.FeatureMap(rng.standard_normal((H, Hd, d)) * gain / np.sqrt(d), rng.standard_normal((H, Hd)) * 0.3,
                          rng.standard_normal((H, F, Hd)) * gain / np.sqrt(Hd), rng.standard_normal((H, F)) * 0.3, P, act)


def _const_map(H, d, Hd, F, P, mod=O):
    """Second layer all zero => softmax output is exactly 1/F in every channel."""
    return mod.FeatureMap(np.ones((H, Hd, d)), np.zeros((H, Hd)), np.zeros((H, F, Hd)), np.zeros((H, F)), P)


# ----------------------------------------------------------------------------- library pins

def pin_r1_is_library_softmax_attention(M):
    """R = 1 is full softmax attention (Eq. "softmax"; Sec. 3.3 lists rate 1 as full softmax):
    compare with torch's scaled_dot_product_attention and with scipy's softmax, both fp64."""
    rng = np.random.default_rng(1)
    B, H, N, d = 2, 3, 37, 10
    q, k, v = (rng.standard_normal((B, H, N, d)) * 1.5 for _ in range(3))
    scale = 0.37
    y = M.hybrid_attn(q, k, v, None, None, 1, scale)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q), torch.from_numpy(k), torch.from_numpy(v), scale=scale).numpy()
    np.testing.assert_allclose(y, ref, rtol=1e-11, atol=1e-13)
    ref2 = scipy.special.softmax(np.einsum("bhid,bhjd->bhij", q, k) * scale, axis=-1) @ v
    np.testing.assert_allclose(y, ref2, rtol=1e-11, atol=1e-13)


def pin_feature_map_is_grouped_conv(M):
    """The embedding network is a per-head MLP "implemented as grouped 1x1 convolutions"
    (Sec. 3.2): run torch's conv1d with groups = H over all heads at once, ReLU between the
    layers, softmax over each head's F channels, then chunk / pow / cat for the P slices."""
    rng = np.random.default_rng(2)
    H, d, Hd, n = 3, 6, 10, 17
    for P, F in ((1, 8), (2, 8), (3, 9), (4, 8)):
        fm = _rand_map(rng, H, d, Hd, F, P, mod=M)
        x = rng.standard_normal((H, n, d))
        xt = torch.from_numpy(x).permute(0, 2, 1).reshape(1, H * d, n)           # [1, H*d, n]
        h1 = torch.nn.functional.conv1d(xt, torch.from_numpy(fm.w1).reshape(H * Hd, d, 1),
                                        torch.from_numpy(fm.b1).reshape(-1), groups=H)
        h1 = torch.relu(h1)
        u = torch.nn.functional.conv1d(h1, torch.from_numpy(fm.w2).reshape(H * F, Hd, 1),
                                       torch.from_numpy(fm.b2).reshape(-1), groups=H)
        t = torch.softmax(u.reshape(H, F, n), dim=1)
        parts = torch.chunk(t, P, dim=1)
        ref = torch.cat([torch.pow(part, p + 1) for p, part in enumerate(parts)], dim=1)   # [H, F, n]
        for h in range(H):
            got = M.feature_map(x[h], fm, h)
            np.testing.assert_allclose(got, ref[h].T.numpy(), rtol=1e-11, atol=1e-300)
            assert (got > 0).all()                        # phi must be non-negative (Sec. 3.1)


@pytest.mark.parametrize("act", ("exp", "relu"))
def test_alternate_output_activations_against_library_ops(act):
    """The two optional output activations of the feature map (exp, ReLU) elementwise against torch: grouped 1x1
    convolutions, torch.exp / torch.relu on the pre-activations, chunk / pow / cat for the P slices.  ReLU outputs may
    be exactly zero, exp outputs are strictly positive; a swapped or missing branch fails the comparison."""
    rng = np.random.default_rng(31)
    H, d, Hd, n = 3, 6, 10, 17
    code = {"exp": O.ACT_EXP, "relu": O.ACT_RELU}[act]
    for P, F in ((1, 8), (2, 8), (3, 9)):
        fm = O.FeatureMap(rng.standard_normal((H, Hd, d)) / np.sqrt(d), rng.standard_normal((H, Hd)) * 0.3,
                          rng.standard_normal((H, F, Hd)) / np.sqrt(Hd), rng.standard_normal((H, F)) * 0.3, P, code)
        x = rng.standard_normal((H, n, d))
        xt = torch.from_numpy(x).permute(0, 2, 1).reshape(1, H * d, n)
        conv = torch.nn.functional.conv1d
        h1 = torch.relu(conv(xt, torch.from_numpy(fm.w1).reshape(H * Hd, d, 1), torch.from_numpy(fm.b1).reshape(-1), groups=H))
        u = conv(h1, torch.from_numpy(fm.w2).reshape(H * F, Hd, 1), torch.from_numpy(fm.b2).reshape(-1), groups=H).reshape(H, F, n)
        t = torch.exp(u) if act == "exp" else torch.relu(u)
        ref = torch.cat([torch.pow(part, p + 1) for p, part in enumerate(torch.chunk(t, P, dim=1))], dim=1)
        for h in range(H):
            got = O.feature_map(x[h], fm, h)
            np.testing.assert_allclose(got, ref[h].T.numpy(), rtol=1e-11, atol=1e-300)
            assert (got > 0).all() if act == "exp" else ((got >= 0).all() and (got == 0).any())
            # the three activations differ from one another on the same pre-activations
            other = O.FeatureMap(fm.w1, fm.b1, fm.w2, fm.b2, P, O.ACT_SOFTMAX if act == "exp" else O.ACT_EXP)
            assert not np.allclose(O.feature_map(x[h], other, h), got)


def test_three_layer_feature_map_is_grouped_conv():
    """The three-layer map of Tab. "phi" (its P = 6 row): three grouped 1x1 convolutions with a ReLU after the
    first two, same output stage; and its parameter count through n_params() (15.4 M at d = 128, 12 heads)."""
    rng = np.random.default_rng(12)
    H, d, Hd, Dm, F, P, n = 3, 6, 10, 7, 9, 3, 17
    fm = O.FeatureMap(rng.standard_normal((H, Hd, d)) / np.sqrt(d), rng.standard_normal((H, Hd)) * 0.3,
                      rng.standard_normal((H, F, Dm)) / np.sqrt(Dm), rng.standard_normal((H, F)) * 0.3, P,
                      w_mid=rng.standard_normal((H, Dm, Hd)) / np.sqrt(Hd), b_mid=rng.standard_normal((H, Dm)) * 0.3)
    x = rng.standard_normal((H, n, d))
    xt = torch.from_numpy(x).permute(0, 2, 1).reshape(1, H * d, n)
    conv = torch.nn.functional.conv1d
    h1 = torch.relu(conv(xt, torch.from_numpy(fm.w1).reshape(H * Hd, d, 1), torch.from_numpy(fm.b1).reshape(-1), groups=H))
    h2 = torch.relu(conv(h1, torch.from_numpy(fm.w_mid).reshape(H * Dm, Hd, 1), torch.from_numpy(fm.b_mid).reshape(-1), groups=H))
    u = conv(h2, torch.from_numpy(fm.w2).reshape(H * F, Dm, 1), torch.from_numpy(fm.b2).reshape(-1), groups=H)
    t = torch.softmax(u.reshape(H, F, n), dim=1)
    ref = torch.cat([torch.pow(part, p + 1) for p, part in enumerate(torch.chunk(t, P, dim=1))], dim=1)
    for h in range(H):
        np.testing.assert_allclose(O.feature_map(x[h], fm, h), ref[h].T.numpy(), rtol=1e-11, atol=1e-300)
    # dropping the middle layer must change the result (the pin is sensitive to it)
    two = O.FeatureMap(fm.w1, fm.b1, rng.standard_normal((H, F, Hd)), fm.b2, P)
    assert not np.allclose(O.feature_map(x[0], two, 0), ref[0].T.numpy())
    big = O.FeatureMap(np.zeros((12, 768, 128)), np.zeros((12, 768)), np.zeros((12, 768, 768)), np.zeros((12, 768)), 6,
                       w_mid=np.zeros((12, 768, 768)), b_mid=np.zeros((12, 768)))
    assert round(big.n_params() / 1e6, 1) == 15.4


# ----------------------------------------------------------------------------- closed forms

def pin_two_token_golden(M):
    """tests/golden/two_token_case.txt: one softmax token + one linear token, worked by hand.
    The softmax weight is exactly 1 whatever q.k is (c_i is that row's only exponent)."""
    vals = [int(t) for line in open(os.path.join(GOLDEN, "two_token_case.txt")) if not line.startswith("#")
            for t in line.split()]
    wn, wd, y0n, y0d, y1n, y1d = vals
    rng = np.random.default_rng(3)
    d = 2
    q = rng.standard_normal((1, 1, 2, d)) * 3.0          # large logits: exp(q.k) would be far from 1
    k = rng.standard_normal((1, 1, 2, d)) * 3.0
    v = np.array([[[[1.0, -2.0], [3.0, 5.0]]]])
    fm = _const_map(1, d, 3, 4, 2, mod=M)
    g = M.feature_map(q[0, 0], fm, 0)
    np.testing.assert_allclose(g @ g[0], float(Fraction(wn, wd)), rtol=1e-14)
    y = M.hybrid_attn(q, k, v, fm, fm, 2, 1.0 / np.sqrt(d))
    want = np.array([float(Fraction(y0n, y0d)), float(Fraction(y1n, y1d))])
    np.testing.assert_allclose(y[0, 0, 0], want, rtol=1e-13)
    np.testing.assert_allclose(y[0, 0, 1], want, rtol=1e-13)


def pin_constant_phi_closed_form(M):
    """q = 0 makes every softmax weight exp(0 - 0) = 1; a zero second layer makes every linear
    weight kappa = D' * sum_p F^(-2p).  Then y_i = (sum_S v + kappa sum_L v) / (N_S + kappa N_L).
    Distinct v rows make the result sensitive to which tokens land in T_S."""
    rng = np.random.default_rng(4)
    for (N, R, F, P) in ((13, 4, 6, 2), (16, 3, 6, 3), (9, 2, 4, 1), (11, 0, 8, 2), (7, 1, 4, 2), (20, 8, 4, 4)):
        d = 5
        q = np.zeros((1, 2, N, d))
        k = rng.standard_normal((1, 2, N, d))
        v = rng.standard_normal((1, 2, N, d)) + np.arange(N)[None, None, :, None]
        fm = _const_map(2, d, 4, F, P, mod=M)
        y = M.hybrid_attn(q, k, v, fm, fm, R, 0.5)
        Dp = F // P
        kappa = Dp * sum(float(F) ** (-2 * p) for p in range(1, P + 1))
        s_tok = [j for j in range(N) if R >= 1 and j % R == 0]      # tokens 1, R+1, 2R+1, ... 1-indexed
        l_tok = [j for j in range(N) if j not in s_tok]
        for h in range(2):
            num = v[0, h, s_tok].sum(0) + kappa * v[0, h, l_tok].sum(0)
            den = len(s_tok) + kappa * len(l_tok)
            np.testing.assert_allclose(y[0, h], np.broadcast_to(num / den, (N, d)), rtol=1e-12)


def pin_r0_is_linear_attention_nxn(M):
    """No softmax tokens: y = (phi_q(Q) phi_k(K)^T) V / rowsum, the un-reassociated N x N form of
    the linear-attention equation of Sec. 3.1."""
    rng = np.random.default_rng(5)
    H, N, d, F = 2, 29, 7, 6
    q, k, v = (rng.standard_normal((1, H, N, d)) for _ in range(3))
    fq, fk = _rand_map(rng, H, d, 9, F, 2, mod=M), _rand_map(rng, H, d, 9, F, 2, mod=M)
    y = M.hybrid_attn(q, k, v, fq, fk, 0, 1.0)
    for h in range(H):
        A = M.feature_map(q[0, h], fq, h) @ M.feature_map(k[0, h], fk, h).T         # [N, N]
        np.testing.assert_allclose(y[0, h], (A @ v[0, h]) / A.sum(1, keepdims=True), rtol=1e-11)


# ----------------------------------------------------------------------------- brute force

def pin_dense_loops(M):
    """The explicit N x N loop form of Eq. "hybrid" on tiny inputs, all rates, P in {1,2,3}."""
    rng = np.random.default_rng(6)
    for R in (0, 1, 2, 3, 4, 5, 8):
        for P, F in ((1, 4), (2, 6), (3, 6)):
            N, d, H = 19, 4, 2
            q, k, v = (rng.standard_normal((1, H, N, d)) * 1.3 for _ in range(3))
            fq, fk = _rand_map(rng, H, d, 5, F, P, mod=M), _rand_map(rng, H, d, 5, F, P, mod=M)
            y = M.hybrid_attn(q, k, v, fq, fk, R, 0.7)
            for h in range(H):
                ref = O.hybrid_attn_dense_loops(q[0, h], k[0, h], v[0, h], fq, fk, h, R, 0.7)
                np.testing.assert_allclose(y[0, h], ref, rtol=1e-11, atol=1e-13)


# ----------------------------------------------------------------------------- invariants

def pin_invariants(M):
    rng = np.random.default_rng(7)
    H, N, d, F, R = 2, 41, 6, 8, 4
    q, k, v = (rng.standard_normal((1, H, N, d)) for _ in range(3))
    fq, fk = _rand_map(rng, H, d, 7, F, 2, mod=M), _rand_map(rng, H, d, 7, F, 2, mod=M)
    y = M.hybrid_attn(q, k, v, fq, fk, R, 0.4)
    # convex combination of value rows (all weights >= 0, one shared normaliser)
    assert (y <= v.max(axis=2, keepdims=True) + 1e-12).all() and (y >= v.min(axis=2, keepdims=True) - 1e-12).all()
    vc = np.broadcast_to(rng.standard_normal((1, H, 1, d)), v.shape)
    np.testing.assert_allclose(M.hybrid_attn(q, k, vc, fq, fk, R, 0.4), vc, rtol=1e-12)
    # permuting (k, v) pairs inside T_S and inside T_L changes nothing
    s_idx, l_idx = M.token_split(N, R)
    perm = np.arange(N)
    perm[s_idx] = rng.permutation(s_idx)
    perm[l_idx] = rng.permutation(l_idx)
    np.testing.assert_allclose(M.hybrid_attn(q, k[:, :, perm], v[:, :, perm], fq, fk, R, 0.4), y, rtol=1e-11)
    # a row depends on its own q only; sampled rows equal the full result
    rows = np.array([0, 3, 17, 40])
    np.testing.assert_allclose(M.hybrid_attn(q, k, v, fq, fk, R, 0.4, rows=rows), y[:, :, rows], rtol=1e-13)
    q2 = q.copy()
    q2[:, :, 5] += 1.0
    y2 = M.hybrid_attn(q2, k, v, fq, fk, R, 0.4)
    assert np.array_equal(np.delete(y2, 5, axis=2), np.delete(y, 5, axis=2)) and not np.allclose(y2[:, :, 5], y[:, :, 5])
    # largest softmax weight per row is exactly 1 and l_i in [1, N_S]
    a, l, c = M.softmax_part(q[0, 0], k[0, 0], v[0, 0], R, 0.4)
    assert (l >= 1.0).all() and (l <= len(s_idx)).all()
    # R = 1: softmax shift invariance (same vector added to every key)
    y1 = M.hybrid_attn(q, k, v, None, None, 1, 0.4)
    np.testing.assert_allclose(M.hybrid_attn(q, k + rng.standard_normal((1, H, 1, d)), v, None, None, 1, 0.4), y1, rtol=1e-10)


def pin_split_rule(M):
    """T_S = {i | i mod R = 1} with 1-indexed tokens (Sec. 3.2); rate 3 as in Fig. "method"."""
    s, l = M.token_split(10, 3)
    assert [i + 1 for i in s] == [1, 4, 7, 10] and [i + 1 for i in l] == [2, 3, 5, 6, 8, 9]
    s, l = M.token_split(5, 1)
    assert list(s) == [0, 1, 2, 3, 4] and len(l) == 0
    s, l = M.token_split(5, 0)
    assert len(s) == 0 and list(l) == [0, 1, 2, 3, 4]
    s, _ = M.token_split(32760, 4)
    assert len(s) == 8190


def pin_block_granular_split(M):
    """The block-granular variant: explicit index lists, block = 1 equals the paper's rule, the closed form for a
    constant feature map (sensitive to which tokens are softmax tokens) and the loop form with its own counting."""
    s, l = M.token_split(11, M.BlockSplit(3, 2))
    assert list(s) == [0, 1, 6, 7] and list(l) == [2, 3, 4, 5, 8, 9, 10]
    s, l = M.token_split(7, M.BlockSplit(2, 4))
    assert list(s) == [0, 1, 2, 3] and list(l) == [4, 5, 6]
    assert len(M.token_split(9, M.BlockSplit(0, 4))[0]) == 0 and len(M.token_split(9, M.BlockSplit(1, 4))[1]) == 0
    for N, R in ((10, 3), (17, 4), (5, 1), (6, 0)):
        for a, b in zip(M.token_split(N, M.BlockSplit(R, 1)), M.token_split(N, R)):
            assert list(a) == list(b)
    rng = np.random.default_rng(14)
    N, d, F, P, R, blk = 23, 5, 6, 2, 3, 4
    q = np.zeros((1, 2, N, d))
    k = rng.standard_normal((1, 2, N, d))
    v = rng.standard_normal((1, 2, N, d)) + np.arange(N)[None, None, :, None]
    fm = _const_map(2, d, 4, F, P, mod=M)
    y = M.hybrid_attn(q, k, v, fm, fm, M.BlockSplit(R, blk), 0.5)
    kappa = (F // P) * sum(float(F) ** (-2 * p) for p in range(1, P + 1))
    s_tok = [0, 1, 2, 3, 12, 13, 14, 15]                          # blocks 0 and 3 of four tokens
    l_tok = [j for j in range(N) if j not in s_tok]
    for h in range(2):
        num = v[0, h, s_tok].sum(0) + kappa * v[0, h, l_tok].sum(0)
        np.testing.assert_allclose(y[0, h], np.broadcast_to(num / (len(s_tok) + kappa * len(l_tok)), (N, d)), rtol=1e-12)
    q, k, v = (rng.standard_normal((1, 2, 19, 4)) * 1.3 for _ in range(3))
    fq, fk = _rand_map(rng, 2, 4, 5, 6, 2, mod=M), _rand_map(rng, 2, 4, 5, 6, 2, mod=M)
    for R, blk in ((2, 3), (4, 2), (3, 8), (0, 2), (1, 5)):
        y = M.hybrid_attn(q, k, v, fq, fk, M.BlockSplit(R, blk), 0.7)
        for h in range(2):
            ref = O.hybrid_attn_dense_loops(q[0, h], k[0, h], v[0, h], fq, fk, h, O.BlockSplit(R, blk), 0.7)
            np.testing.assert_allclose(y[0, h], ref, rtol=1e-11, atol=1e-13)


def pin_chunk_causal(M):
    """The chunk-causal variant against an N x N weight matrix built entry by entry with the visibility rule written
    as a mask (own loops, own split rule), against library causal softmax attention at R = 1 with chunks of one
    token, and its reductions: one chunk covering everything is Eq. "hybrid"; the last chunk's rows equal Eq. "hybrid"
    on the whole sequence; the first chunk's rows equal Eq. "hybrid" on the first chunk alone."""
    rng = np.random.default_rng(15)
    H, N, d, F = 2, 23, 4, 6
    q, k, v = (rng.standard_normal((1, H, N, d)) * 1.2 for _ in range(3))
    fq, fk = _rand_map(rng, H, d, 5, F, 2, mod=M), _rand_map(rng, H, d, 5, F, 2, mod=M)
    for R, C in ((3, 5), (2, 8), (4, 4), (0, 6), (1, 7)):
        y = M.hybrid_attn_chunk_causal(q, k, v, fq, fk, R, 0.6, C)
        for h in range(H):
            gq, gk = M.feature_map(q[0, h], fq, h), M.feature_map(k[0, h], fk, h)
            for i in range(N):
                vis = [j for j in range(N) if j // C <= i // C]
                soft = [j for j in vis if R >= 1 and j % R == 0]
                c = max((0.6 * float(q[0, h, i] @ k[0, h, j]) for j in soft), default=0.0)
                num, den = np.zeros(d), 0.0
                for j in vis:
                    w = np.exp(0.6 * float(q[0, h, i] @ k[0, h, j]) - c) if j in soft else float(gq[i] @ gk[j])
                    num += w * v[0, h, j]
                    den += w
                np.testing.assert_allclose(y[0, h, i], num / den, rtol=1e-10, atol=1e-13)
    y1 = M.hybrid_attn_chunk_causal(q, k, v, None, None, 1, 0.6, 1)
    ref = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q), torch.from_numpy(k), torch.from_numpy(v),
                                                           is_causal=True, scale=0.6).numpy()
    np.testing.assert_allclose(y1, ref, rtol=1e-10, atol=1e-13)
    full = M.hybrid_attn(q, k, v, fq, fk, 3, 0.6)
    np.testing.assert_allclose(M.hybrid_attn_chunk_causal(q, k, v, fq, fk, 3, 0.6, N), full, rtol=1e-13)
    yc = M.hybrid_attn_chunk_causal(q, k, v, fq, fk, 3, 0.6, 6)
    np.testing.assert_allclose(yc[:, :, 18:], full[:, :, 18:], rtol=1e-13)
    np.testing.assert_allclose(yc[:, :, :6], M.hybrid_attn(q[:, :, :6], k[:, :, :6], v[:, :, :6], fq, fk, 3, 0.6), rtol=1e-13)
    rows = np.array([0, 5, 6, 17, 22])
    np.testing.assert_allclose(M.hybrid_attn_chunk_causal(q, k, v, fq, fk, 3, 0.6, 6, rows=rows), yc[:, :, rows], rtol=1e-13)


def pin_local_window(M):
    """The local-window variant against an N x N weight matrix built entry by entry (own loops), and its reductions: a
    window that covers every tile is plain softmax attention; with constant feature maps and q = 0 the closed form
    (sum over the window + kappa sum over the rest) / (window size + kappa rest size)."""
    rng = np.random.default_rng(16)
    H, N, d, F = 2, 22, 4, 6
    q, k, v = (rng.standard_normal((1, H, N, d)) * 1.2 for _ in range(3))
    fq, fk = _rand_map(rng, H, d, 5, F, 2, mod=M), _rand_map(rng, H, d, 5, F, 2, mod=M)
    for T, W in ((4, 1), (5, 0), (3, 2), (8, 1)):
        y = M.hybrid_attn_local_window(q, k, v, fq, fk, 0.6, T, W)
        for h in range(H):
            gq, gk = M.feature_map(q[0, h], fq, h), M.feature_map(k[0, h], fk, h)
            for i in range(N):
                soft = [j for j in range(N) if abs(j // T - i // T) <= W]
                c = max(0.6 * float(q[0, h, i] @ k[0, h, j]) for j in soft)
                num, den = np.zeros(d), 0.0
                for j in range(N):
                    w = np.exp(0.6 * float(q[0, h, i] @ k[0, h, j]) - c) if j in soft else float(gq[i] @ gk[j])
                    num += w * v[0, h, j]
                    den += w
                np.testing.assert_allclose(y[0, h, i], num / den, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(M.hybrid_attn_local_window(q, k, v, fq, fk, 0.6, 4, 6), M.hybrid_attn(q, k, v, None, None, 1, 0.6),
                               rtol=1e-12)
    rows = np.array([0, 3, 4, 11, 21])
    np.testing.assert_allclose(M.hybrid_attn_local_window(q, k, v, fq, fk, 0.6, 4, 1, rows=rows),
                               M.hybrid_attn_local_window(q, k, v, fq, fk, 0.6, 4, 1)[:, :, rows], rtol=1e-13)
    fm = _const_map(2, d, 4, F, 2, mod=M)
    vv = rng.standard_normal((1, 2, N, d)) + np.arange(N)[None, None, :, None]
    y = M.hybrid_attn_local_window(np.zeros((1, 2, N, d)), k, vv, fm, fm, 0.5, 4, 1)
    kappa = (F // 2) * sum(float(F) ** (-2 * p) for p in (1, 2))
    for i in (0, 5, 13, 21):
        win = [j for j in range(N) if abs(j // 4 - i // 4) <= 1]
        rest = [j for j in range(N) if j not in win]
        for h in range(2):
            ref = (vv[0, h, win].sum(0) + kappa * vv[0, h, rest].sum(0)) / (len(win) + kappa * len(rest))
            np.testing.assert_allclose(y[0, h, i], ref, rtol=1e-12)


PINS = [pin_r1_is_library_softmax_attention, pin_feature_map_is_grouped_conv, pin_two_token_golden,
        pin_constant_phi_closed_form, pin_r0_is_linear_attention_nxn, pin_dense_loops, pin_invariants,
        pin_split_rule, pin_block_granular_split, pin_chunk_causal, pin_local_window]


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_pin(pin):
    pin(O)


def test_tab_phi_parameter_counts():
    """Tab. "phi": printed parameter counts (in M) of one feature map at d = 128, 12 heads."""
    for line in open(os.path.join(GOLDEN, "tab_phi_params.txt")):
        if line.startswith("#") or not line.strip():
            continue
        P, layers, printed = line.split()
        P, layers, printed = int(P), int(layers), float(printed)
        H, d = 12, 128
        if layers == 2:
            fm = O.FeatureMap(np.zeros((H, P * d, d)), np.zeros((H, P * d)), np.zeros((H, P * d, P * d)),
                              np.zeros((H, P * d)), P)
            n = fm.n_params()
        else:  # the 3-layer map of the ablation has one more P*d x P*d layer with bias
            n = H * (d * P * d + P * d + 2 * (P * d * P * d + P * d))
        assert round(n / 1e6, 1) == printed, (P, layers, n)


# ----------------------------------------------------------------------------- planted mistakes

def _mut_split_off_by_one(mp):
    good = O.token_split

    def bad(N, R):
        if isinstance(R, O.BlockSplit):
            return good(N, R)
        idx = np.arange(N)
        is_s = (idx % R) == (1 % R) if R else np.zeros(N, bool)
        return idx[is_s], idx[~is_s]
    mp.setattr(O, "token_split", bad)


def _mut_block_split_counts_tokens_not_blocks(mp):
    """The variant's rule with the block index dropped: the first token of every R-th block only."""
    good = O.token_split

    def bad(N, R):
        if not isinstance(R, O.BlockSplit):
            return good(N, R)
        idx = np.arange(N)
        is_s = (idx % (R.R * R.block)) == 0 if R.R else np.zeros(N, bool)
        return idx[is_s], idx[~is_s]
    mp.setattr(O, "token_split", bad)


def _mut_causal_per_token(mp):
    """Token-causal instead of chunk-causal: a query sees only the tokens up to itself inside its own chunk."""
    def bad(q, k, v, phi_q, phi_k, R, scale, chunk, rows=None):
        B, H, N, d = q.shape
        sel = np.arange(N) if rows is None else np.asarray(rows)
        y = np.empty((B, H, sel.size, d))
        for n, i in enumerate(sel):
            for b in range(B):
                for h in range(H):
                    y[b, h, n] = O.hybrid_attn_head(q[b, h, :i + 1], k[b, h, :i + 1], v[b, h, :i + 1], phi_q, phi_k, h, R, scale,
                                                    rows=[i])[0]
        return y
    mp.setattr(O, "hybrid_attn_chunk_causal", bad)


def _mut_window_one_sided(mp):
    """The window reaching back only (tiles t - w .. t), as a causal language model would have it."""
    def bad(q, k, v, phi_q, phi_k, scale, tile, w_tiles, rows=None):
        B, H, N, d = q.shape
        sel = np.arange(N) if rows is None else np.asarray(rows)
        y = np.empty((B, H, sel.size, d))
        tok = np.arange(N)
        for n, i in enumerate(sel):
            in_win = (tok // tile >= i // tile - w_tiles) & (tok // tile <= i // tile)
            for b_ in range(B):
                for h in range(H):
                    s_ = (q[b_, h, i] @ k[b_, h, in_win].T) * scale
                    p_ = np.exp(s_ - s_.max())
                    num, den = p_ @ v[b_, h, in_win], p_.sum()
                    if (~in_win).any():
                        fk = O.feature_map(k[b_, h, ~in_win], phi_k, h)
                        g = O.feature_map(q[b_, h, i:i + 1], phi_q, h)[0]
                        num, den = num + g @ (fk.T @ v[b_, h, ~in_win]), den + g @ fk.sum(axis=0)
                    y[b_, h, n] = num / den
        return y
    mp.setattr(O, "hybrid_attn_local_window", bad)


def _mut_softmax_per_slice(mp):
    def bad(x, fm, head):
        x = np.asarray(x, dtype=np.float64)
        u = np.maximum(x @ fm.w1[head].T + fm.b1[head], 0.0) @ fm.w2[head].T + fm.b2[head]
        Dp = fm.F // fm.P
        out = np.empty_like(u)
        for p in range(1, fm.P + 1):
            sl = slice((p - 1) * Dp, p * Dp)
            out[:, sl] = scipy.special.softmax(u[:, sl], axis=-1) ** p
        return out
    mp.setattr(O, "feature_map", bad)


def _mut_no_powers(mp):
    def bad(x, fm, head):
        x = np.asarray(x, dtype=np.float64)
        u = np.maximum(x @ fm.w1[head].T + fm.b1[head], 0.0) @ fm.w2[head].T + fm.b2[head]
        return scipy.special.softmax(u, axis=-1)
    mp.setattr(O, "feature_map", bad)


def _mut_powers_from_zero(mp):
    def bad(x, fm, head):
        x = np.asarray(x, dtype=np.float64)
        u = np.maximum(x @ fm.w1[head].T + fm.b1[head], 0.0) @ fm.w2[head].T + fm.b2[head]
        t = scipy.special.softmax(u, axis=-1)
        Dp = fm.F // fm.P
        return np.concatenate([t[:, p * Dp:(p + 1) * Dp] ** p for p in range(fm.P)], axis=1)
    mp.setattr(O, "feature_map", bad)


def _mut_no_relu(mp):
    def bad(x, fm, head):
        x = np.asarray(x, dtype=np.float64)
        u = (x @ fm.w1[head].T + fm.b1[head]) @ fm.w2[head].T + fm.b2[head]
        t = scipy.special.softmax(u, axis=-1)
        Dp = fm.F // fm.P
        return np.concatenate([t[:, p * Dp:(p + 1) * Dp] ** (p + 1) for p in range(fm.P)], axis=1)
    mp.setattr(O, "feature_map", bad)


def _mut_no_scale(mp):
    good = O.softmax_part
    mp.setattr(O, "softmax_part", lambda q, k, v, R, scale: good(q, k, v, R, 1.0))


def _mut_unstabilised(mp):
    """The other reading of c_i: true exp(q.k) weights next to the linear ones, i.e. the linear
    terms effectively scaled by exp(-c_i)."""
    good = O.softmax_part

    def bad(q, k, v, R, scale):
        a, l, c = good(q, k, v, R, scale)
        e = np.where(np.isfinite(c), np.exp(c), 1.0)
        return a * e[:, None], l * e, c
    mp.setattr(O, "softmax_part", bad)


def _mut_max_over_all_tokens(mp):
    good = O.softmax_part

    def bad(q, k, v, R, scale):
        a, l, c = good(q, k, v, R, scale)
        if not np.isfinite(c).all():
            return a, l, c
        call = (np.asarray(q) @ np.asarray(k).T * scale).max(axis=1)
        e = np.exp(c - call)
        return a * e[:, None], l * e, call
    mp.setattr(O, "softmax_part", bad)


def _mut_drop_z(mp):
    good = O.linear_state

    def bad(k, v, fm, head, R):
        S, z = good(k, v, fm, head, R)
        return S, np.ones_like(z)
    mp.setattr(O, "linear_state", bad)


def _mut_state_over_all_tokens(mp):
    good = O.linear_state
    mp.setattr(O, "linear_state", lambda k, v, fm, head, R: good(k, v, fm, head, 0))


def _mut_phi_sees_scaled_input(mp):
    good = O.feature_map
    mp.setattr(O, "feature_map", lambda x, fm, head: good(np.asarray(x) * 0.5, fm, head))


MUTATIONS = [_mut_split_off_by_one, _mut_block_split_counts_tokens_not_blocks, _mut_causal_per_token, _mut_window_one_sided,
             _mut_softmax_per_slice, _mut_no_powers, _mut_powers_from_zero, _mut_no_relu,
             _mut_no_scale, _mut_unstabilised, _mut_max_over_all_tokens, _mut_drop_z, _mut_state_over_all_tokens,
             _mut_phi_sees_scaled_input]


@pytest.mark.parametrize("mutate", MUTATIONS, ids=lambda f: f.__name__)
def test_planted_mistake_is_caught(mutate, monkeypatch):
    mutate(monkeypatch)
    caught = []
    for pin in PINS:
        try:
            pin(O)
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, "no pin noticed the planted mistake"
