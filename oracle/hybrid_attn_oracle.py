"""fp64 CPU oracle for the hybrid-attention forward of "Attention Surgery" (arXiv 2509.24899).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the HIP path is
checked against.  It shares no code with the GPU library and must never be imported by the
product path: only tests, the smoke check and the benchmark's CPU-baseline leg may call it.

What it computes (Sec. 3.2, Eq. "hybrid"): for every query token i of one head

            sum_{j in T_S} exp(scale * q_i.k_j - c_i) v_j  +  phi_q(q_i) . S
    y_i  =  -------------------------------------------------------------------
            sum_{j in T_S} exp(scale * q_i.k_j - c_i)      +  phi_q(q_i) . z

    S = sum_{j in T_L} phi_k(k_j)^T v_j   (F x d),     z = sum_{j in T_L} phi_k(k_j)   (F)

with T_S the uniformly strided softmax tokens, T_L the rest, c_i the largest exponent of row i
over T_S, and phi the learnable polynomial feature map of Sec. 3.2 ("Characterization of phi").

Readings of the paper taken here (each is a decision, listed again in the design notes):
  * T_S = {i | i mod R = 1} over 1-indexed tokens  ==  0-indexed j % R == 0  (Sec. 3.2).
  * R = 1 is "full softmax" (Sec. 3.3, block-rate optimisation): T_S = all tokens, T_L empty.
  * R = 0 encodes a purely linear block (Tab. "vsnodist" rows "Linear"): T_S empty, no c_i.
  * c_i is subtracted inside the softmax exponents only, exactly as Eq. "hybrid" is printed;
    the linear terms are NOT multiplied by exp(-c_i).  The maximum runs over T_S only.
  * Attention is per head; scale is passed in (1/sqrt(d_head) for the paper's operator);
    the feature maps see the unscaled q and k.
  * phi: per-head 2-layer MLP (a grouped 1x1 convolution per layer; optionally 3 layers, as in
    the P = 6 row of Tab. "phi") with ReLU between the layers; the output is made positive by a softmax over all F output channels of the token,
    then split into P contiguous slices and slice p (1-based) is raised elementwise to the
    power p and the slices are concatenated in channel order.

Variant (not the paper's method, which Sec. 3.2 states per token): `BlockSplit(R, block)` in place of the integer
R makes whole blocks of `block` consecutive tokens softmax tokens, every R-th block, the other reading of a
"block rate"; everything downstream of the split is unchanged.

Second variant (the paper names causal attention as future work and defines none): `hybrid_attn_chunk_causal`
cuts the sequence into chunks of `chunk` consecutive tokens; a query sees the keys of its own and of all earlier
chunks, softmax tokens and linear tokens alike, so S and z become prefix sums over chunks.  It is written as the
pinned non-causal function applied to every prefix of the sequence.

Third variant: `hybrid_attn_local_window`, the design Sec. 3.2 sets its uniform stride against: the softmax tokens of
a query are a local window around it, every other token is a linear token.  Blocked form: the sequence is cut into
tiles of `tile` tokens and the window of a query is its own tile and `w_tiles` tiles on either side.

All arithmetic is float64; nothing is rounded inside.  Inputs are whatever the caller hands in
(already rounded to the io dtype of the GPU path and widened).

Pins (tests/test_oracle_pins.py): R=1 against library softmax attention; the feature map against
torch's grouped conv1d; closed forms for constant feature maps and for the two-token case; the
explicit N x N loop form `hybrid_attn_dense_loops`; convexity / permutation / row-independence
invariants; planted-mistake variants that the pins must reject.  `value_distill_loss` is pinned
in tests/test_value_distill_oracle.py (zero at R = 1, a closed form, the loop form, scaling).  No
function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

ACT_SOFTMAX = 0
ACT_EXP = 1
ACT_RELU = 2


class FeatureMap:
    """Parameters of one feature map (phi_q or phi_k) for all heads.

    w1: [H, Hd, d]   b1: [H, Hd]   w2: [H, F, Hd]   b2: [H, F]   (Sec. 3.2: per-head embedding
    network realised as grouped 1x1 convolutions), P = polynomial degree, act = output
    positivity (softmax over the F channels by default).  Tab. "phi" also has a three-layer map
    (its P = 6 row): then w_mid [H, Dm, Hd], b_mid [H, Dm] sit between the two, with a ReLU after
    each hidden layer, and w2 is [H, F, Dm].
    """

    def __init__(self, w1, b1, w2, b2, poly_degree=2, act=ACT_SOFTMAX, w_mid=None, b_mid=None):
        self.w1 = np.asarray(w1, dtype=np.float64)
        self.w2 = np.asarray(w2, dtype=np.float64)
        H, Hd, _ = self.w1.shape
        F = self.w2.shape[1]
        self.b1 = np.zeros((H, Hd)) if b1 is None else np.asarray(b1, dtype=np.float64)
        self.b2 = np.zeros((H, F)) if b2 is None else np.asarray(b2, dtype=np.float64)
        self.w_mid = None if w_mid is None else np.asarray(w_mid, dtype=np.float64)
        self.b_mid = None
        if self.w_mid is not None:
            Dm = self.w_mid.shape[1]
            self.b_mid = np.zeros((H, Dm)) if b_mid is None else np.asarray(b_mid, dtype=np.float64)
        self.P = int(poly_degree)
        self.act = int(act)
        if F % self.P != 0:
            raise ValueError("poly_degree must divide the feature width F")

    @property
    def F(self):
        return self.w2.shape[1]

    def n_params(self):
        """Learnable parameter count of this one map over all heads (weights and biases)."""
        n = self.w1.size + self.b1.size + self.w2.size + self.b2.size
        if self.w_mid is not None:
            n += self.w_mid.size + self.b_mid.size
        return n


class BlockSplit:
    """Block-granular variant of the token split: token j (0-based) is a softmax token when its block
    j // block is a multiple of R.  Accepted wherever a rate R is; block = 1 is the paper's rule."""

    def __init__(self, R: int, block: int):
        if R < 0 or block < 1:
            raise ValueError("R must be >= 0 and block >= 1")
        self.R, self.block = int(R), int(block)


def token_split(N: int, R):
    """Index sets (0-based) of softmax tokens T_S and linear tokens T_L (Sec. 3.2)."""
    if isinstance(R, BlockSplit):
        idx = np.arange(N)
        if R.R == 0:
            is_s = np.zeros(N, dtype=bool)
        else:
            is_s = ((idx // R.block) % R.R) == 0
        return idx[is_s], idx[~is_s]
    if R < 0:
        raise ValueError("R must be >= 0")
    idx = np.arange(N)
    if R == 0:
        is_s = np.zeros(N, dtype=bool)
    else:
        is_s = (idx % R) == 0  # 1-indexed "i mod R = 1"; for R = 1 every token (full softmax)
    return idx[is_s], idx[~is_s]


def feature_map(x, fm: FeatureMap, head: int):
    """phi(x) for rows x [n, d] of one head -> [n, F]  (Sec. 3.2, "Characterization of phi")."""
    x = np.asarray(x, dtype=np.float64)
    hidden = np.maximum(x @ fm.w1[head].T + fm.b1[head], 0.0)        # [n, Hd], ReLU
    if fm.w_mid is not None:                                         # three-layer map: one more hidden layer
        hidden = np.maximum(hidden @ fm.w_mid[head].T + fm.b_mid[head], 0.0)
    u = hidden @ fm.w2[head].T + fm.b2[head]                         # [n, F]
    if fm.act == ACT_SOFTMAX:
        u = u - u.max(axis=-1, keepdims=True)
        t = np.exp(u)
        t = t / t.sum(axis=-1, keepdims=True)
    elif fm.act == ACT_EXP:
        t = np.exp(u)
    elif fm.act == ACT_RELU:
        t = np.maximum(u, 0.0)
    else:
        raise ValueError("unknown activation")
    Dp = fm.F // fm.P
    out = np.empty_like(t)
    for p in range(1, fm.P + 1):                                     # psi_p(x) ** p
        sl = slice((p - 1) * Dp, p * Dp)
        out[:, sl] = t[:, sl] ** p
    return out


def linear_state(k, v, phi_k: FeatureMap, head: int, R: int):
    """S = sum_{j in T_L} phi_k(k_j)^T v_j  [F, d]  and  z = sum_{j in T_L} phi_k(k_j)  [F]."""
    N, d = k.shape
    _, idx_l = token_split(N, R)
    if idx_l.size == 0:
        F = phi_k.F if phi_k is not None else 0
        return np.zeros((F, d)), np.zeros(F)
    f = feature_map(k[idx_l], phi_k, head)                           # [N_L, F]
    return f.T @ np.asarray(v, dtype=np.float64)[idx_l], f.sum(axis=0)


def softmax_part(q_rows, k, v, R: int, scale: float):
    """a_i = sum_{T_S} exp(s_ij - c_i) v_j, l_i = sum_{T_S} exp(s_ij - c_i), c_i = max_j s_ij."""
    N, d = k.shape
    idx_s, _ = token_split(N, R)
    n = q_rows.shape[0]
    if idx_s.size == 0:
        return np.zeros((n, d)), np.zeros(n), np.full(n, -np.inf)
    ks = np.asarray(k, dtype=np.float64)[idx_s]
    vs = np.asarray(v, dtype=np.float64)[idx_s]
    s = (np.asarray(q_rows, dtype=np.float64) @ ks.T) * scale       # [n, N_S]
    c = s.max(axis=1)
    p = np.exp(s - c[:, None])
    return p @ vs, p.sum(axis=1), c


def hybrid_attn_head(q, k, v, phi_q, phi_k, head, R, scale, rows=None, row_chunk=2048):
    """Eq. "hybrid" for one (batch, head): q,k,v [N, d] -> y [N or len(rows), d]."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    N, d = q.shape
    sel = np.arange(N) if rows is None else np.asarray(rows)
    _, idx_l = token_split(N, R)
    has_linear = idx_l.size > 0
    if has_linear:
        S, z = linear_state(k, v, phi_k, head, R)
    out = np.empty((sel.size, d))
    for lo in range(0, sel.size, row_chunk):
        r = sel[lo:lo + row_chunk]
        a, l, _ = softmax_part(q[r], k, v, R, scale)
        num, den = a, l
        if has_linear:
            g = feature_map(q[r], phi_q, head)                      # [n, F]
            num = num + g @ S
            den = den + g @ z
        out[lo:lo + row_chunk] = num / den[:, None]
    return out


def hybrid_attn(q, k, v, phi_q, phi_k, R, scale, rows=None):
    """Eq. "hybrid" for q,k,v [B, H, N, d] -> y [B, H, N or len(rows), d] (float64).

    `rows` (optional, 1-D indices) restricts the per-query part to a sample of query rows; the
    state S, z always runs over every linear key.
    """
    B, H, N, d = q.shape
    n_out = N if rows is None else len(rows)
    y = np.empty((B, H, n_out, d))
    for b in range(B):
        for h in range(H):
            y[b, h] = hybrid_attn_head(q[b, h], k[b, h], v[b, h], phi_q, phi_k, h, R, scale, rows)
    return y


def hybrid_attn_chunk_causal(q, k, v, phi_q, phi_k, R, scale, chunk: int, rows=None):
    """Chunk-causal variant of Eq. "hybrid" for q, k, v [B, H, N, d]: query i attends to the tokens j with
    j // chunk <= i // chunk; among those the split into softmax and linear tokens is the usual one (position in the
    whole sequence decides).  For the queries of chunk c this is Eq. "hybrid" on the first (c + 1) chunk tokens, and
    that is how it is computed.  `rows` (optional, sorted 1-D indices) restricts the output to those queries."""
    if chunk < 1:
        raise ValueError("chunk must be >= 1")
    B, H, N, d = q.shape
    sel = np.arange(N) if rows is None else np.asarray(rows)
    y = np.empty((B, H, sel.size, d))
    for c in range(-(-N // chunk)):
        end = min((c + 1) * chunk, N)
        pos = np.nonzero((sel >= c * chunk) & (sel < end))[0]
        if pos.size == 0:
            continue
        for b in range(B):
            for h in range(H):
                y[b, h, pos] = hybrid_attn_head(q[b, h, :end], k[b, h, :end], v[b, h, :end], phi_q, phi_k, h, R, scale,
                                                rows=sel[pos])
    return y


def hybrid_attn_local_window(q, k, v, phi_q, phi_k, scale, tile: int, w_tiles: int, rows=None):
    """Local-window variant of Eq. "hybrid" for q, k, v [B, H, N, d]: for a query in tile t (tiles of `tile`
    consecutive tokens) T_S is the set of tokens in tiles t - w_tiles .. t + w_tiles and T_L is every other token;
    with those sets the equation is evaluated as printed (c_i over the window only).  `rows` (optional, sorted
    1-D indices) restricts the output to those queries."""
    if tile < 1 or w_tiles < 0:
        raise ValueError("tile must be >= 1 and w_tiles >= 0")
    B, H, N, d = q.shape
    sel = np.arange(N) if rows is None else np.asarray(rows)
    y = np.empty((B, H, sel.size, d))
    tok = np.arange(N)
    for t in range(-(-N // tile)):
        pos = np.nonzero((sel >= t * tile) & (sel < (t + 1) * tile))[0]
        if pos.size == 0:
            continue
        in_win = (tok // tile >= t - w_tiles) & (tok // tile <= t + w_tiles)
        win, rest = tok[in_win], tok[~in_win]
        for b in range(B):
            for h in range(H):
                qs = np.asarray(q[b, h], dtype=np.float64)[sel[pos]]
                kk = np.asarray(k[b, h], dtype=np.float64)
                vv = np.asarray(v[b, h], dtype=np.float64)
                s = (qs @ kk[win].T) * scale
                p = np.exp(s - s.max(axis=1, keepdims=True))
                num, den = p @ vv[win], p.sum(axis=1)
                if rest.size:
                    fk = feature_map(kk[rest], phi_k, h)
                    g = feature_map(qs, phi_q, h)
                    num = num + g @ (fk.T @ vv[rest])
                    den = den + g @ fk.sum(axis=0)
                y[b, h, pos] = num / den[:, None]
    return y


def value_distill_loss(q, k, v, phi_q, phi_k, R, scale):
    """Value-distillation objective of Sec. 3.3 (Eq. "vd_loss"): || y - y_hat ||_1 with y the softmax
    attention of Eq. "softmax" (the teacher: every token a softmax token) and y_hat the hybrid
    attention of Eq. "hybrid" at rate R (the student), summed over every batch entry, head, token
    and channel of q, k, v [B, H, N, d].  (Alg. 1 averages this over the samples of a batch: divide
    by B.)  Returns a float."""
    y = hybrid_attn(q, k, v, None, None, 1, scale)
    y_hat = hybrid_attn(q, k, v, phi_q, phi_k, R, scale)
    total = 0.0
    for b in range(y.shape[0]):
        for h in range(y.shape[1]):
            total += float(np.abs(y[b, h] - y_hat[b, h]).sum())
    return total


def hybrid_attn_dense_loops(q, k, v, phi_q, phi_k, head, R, scale):
    """Second, independent form for tiny inputs: the N x N weight matrix of Eq. "hybrid" built
    entry by entry with Python loops, no cached state and no matrix products.

    w_ij = exp(scale q_i.k_j - c_i) if j is a softmax token, phi_q(q_i).phi_k(k_j) otherwise;
    y_i = sum_j w_ij v_j / sum_j w_ij.
    """
    N, d = q.shape
    if isinstance(R, BlockSplit):                                    # variant: every R-th block of tokens, counted in loops
        is_s, j = [], 0
        while j < N:
            for blk in range(max(R.R, 1)):
                for _ in range(R.block):
                    if j < N:
                        is_s.append(R.R >= 1 and blk == 0)
                        j += 1
    else:
        is_s = [(R >= 1 and (j + 1) % R == (1 % R)) for j in range(N)]   # the rule in 1-indexed form
    gq = feature_map(q, phi_q, head) if phi_q is not None else None
    fk = feature_map(k, phi_k, head) if phi_k is not None else None
    y = np.zeros((N, d))
    for i in range(N):
        logits = {}
        for j in range(N):
            if is_s[j]:
                acc = 0.0
                for t in range(d):
                    acc += float(q[i, t]) * float(k[j, t])
                logits[j] = acc * scale
        c = max(logits.values()) if logits else 0.0
        den = 0.0
        num = [0.0] * d
        for j in range(N):
            if is_s[j]:
                w = float(np.exp(logits[j] - c))
            else:
                w = 0.0
                for f in range(gq.shape[1]):
                    w += float(gq[i, f]) * float(fk[j, f])
            den += w
            for t in range(d):
                num[t] += w * float(v[j, t])
        for t in range(d):
            y[i, t] = num[t] / den
    return y
