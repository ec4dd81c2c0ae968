"""Float64 CPU oracle for the SQuat key-quantization path (arxiv 2503.24358).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, numpy-only
restatement of what the paper defines, kept independent of the HIP library: it
shares no code, tables or helpers with it and never imports it.  Only the test
suite, the smoke check and the CPU-baseline leg of the benchmark may call it.

Every function names the passage of the paper it follows.  Where the paper is
silent the reading taken is stated in the docstring (and listed in the design
notes of the repository).

Notation follows the paper: d hidden size of one head, r subspace dimension,
Qhat (r x d) the scaled top-r right singular vectors of the prompt queries,
lambda the penalty weight, g the number of channels frozen per iteration,
T = d / g iterations, G the quantization group size, b the bit width.

Parity status of each function:
  gram, subspace                pinned (library SVD, planted spectrum, Eckart-Young)
  gram_update, iteration_start,
  subspace_iteration            pinned (Gram of the concatenated queries; fixed point at the exact
                                eigenvectors; converged limit = library eigh; residual and Ritz
                                values against their definitions; monotone Ritz values; the
                                convergence rate (lambda_{p+1} / lambda_r)^k on a planted spectrum)
  update_matrix_*               pinned (three routes + brute-force constrained LS,
                                g=1 against the one-coordinate rule of Prop. 1)
  rtn_group, quantize_keys      pinned (hand-worked fixture, r=0 fixed point,
                                per-step optimality against a generic solver,
                                soft and hard invariants), both grouping axes
  CacheOracle                   pinned (counts against l mod R by hand, stores
                                against one-shot quantization of the prefix; scores_rope:
                                zero frequencies = scores, hand-rotated cached keys,
                                both key groupings)
  key_scores_rope, rope_rotate  pinned (norm preservation, relative-position identity, explicit
                                2x2 rotations, zero angle = key_scores; per-channel grouping:
                                element loops)
  key_scores                    pinned (element loops, one-hot queries, closed
                                form for constant codes)
  dequantize_keys, pack/unpack  pinned (definition of deq; pack o unpack = id,
                                single-code layout checks), both layouts
  exact integer codes for a concrete key under lambda>0: parity unpinned by the
  paper (it prints no worked numeric example); pinned only through the
  invariants above.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "gram", "subspace", "subspace_svd", "deviation_from_subspace",
    "gram_update", "iteration_start", "subspace_iteration",
    "update_matrix_lemma", "update_matrix_kkt", "update_matrix_lowrank",
    "rtn_group", "quantize_keys", "dequantize_keys",
    "pack_codes", "unpack_codes", "pack_codes_tokens", "unpack_codes_tokens",
    "replay_classify", "key_scores", "key_scores_rope", "rope_rotate", "CacheOracle",
]


# --------------------------------------------------------------------------- #
# Step 1: query subspace  (Section 3.2; Algorithm 1, prefill phase, SVD lines)
# --------------------------------------------------------------------------- #

def _pool(Q) -> np.ndarray:
    """Stack the queries of all query heads that share one KV head row-wise.

    Appendix "Details of Our Main Algorithm": for grouped-query attention the
    queries of the associated query heads are concatenated before the SVD.
    Accepts (n, d) or (q_per_kv, n, d) or a list of (n_i, d) arrays.
    """
    if isinstance(Q, (list, tuple)):
        return np.concatenate([np.asarray(q, dtype=np.float64) for q in Q], axis=0)
    Q = np.asarray(Q, dtype=np.float64)
    if Q.ndim == 3:
        return Q.reshape(-1, Q.shape[-1])
    return Q


def gram(Q) -> np.ndarray:
    """Gram matrix Q^T Q (d x d) of the pooled prompt queries.

    The right singular vectors of Q are the eigenvectors of Q^T Q and the
    squared singular values are its eigenvalues, so this is the sufficient
    statistic of the SVD in Algorithm 1.  No centering, no 1/n, no row
    normalisation (the normalisation in Definition 1 is for the plot only).
    """
    Qp = _pool(Q)
    return Qp.T @ Qp


def subspace(Q, r: int):
    """Qhat = diag(Sigma[:r]) V[:r]  via the eigen-decomposition of Q^T Q.

    Section 3.2 (last sentence) and Algorithm 1: the top r right singular
    vectors scaled by their singular values.  Rows are ordered by descending
    singular value; each row's sign is fixed so that its largest-magnitude
    component is positive (the paper leaves sign free; nothing downstream
    depends on it).  Zero singular values give zero rows.

    Returns (Qhat (r, d), eig (r,)) with eig the eigenvalues of Q^T Q
    (= squared singular values).
    """
    Gm = gram(Q)
    d = Gm.shape[0]
    w, V = np.linalg.eigh(Gm)            # ascending
    order = np.argsort(w)[::-1]
    w = np.maximum(w[order], 0.0)
    V = V[:, order]
    r_eff = min(r, d)
    Qhat = np.zeros((r, d))
    eig = np.zeros((r,))
    for i in range(r_eff):
        v = V[:, i]
        j = int(np.argmax(np.abs(v)))
        if v[j] < 0:
            v = -v
        Qhat[i] = np.sqrt(w[i]) * v
        eig[i] = w[i]
    return Qhat, eig


def subspace_svd(Q, r: int):
    """Same object through the library SVD of Q itself (Algorithm 1 verbatim).

    Used only to cross-check `subspace`.
    """
    Qp = _pool(Q)
    _, s, Vt = np.linalg.svd(Qp, full_matrices=False)
    k = min(r, s.shape[0])
    Qhat = np.zeros((r, Qp.shape[1]))
    for i in range(k):
        v = Vt[i]
        j = int(np.argmax(np.abs(v)))
        if v[j] < 0:
            v = -v
        Qhat[i] = s[i] * v
    eig = np.zeros((r,))
    eig[:k] = s[:k] ** 2
    return Qhat, eig


def deviation_from_subspace(q: np.ndarray, basis: np.ndarray) -> np.ndarray:
    """Definition 1: || q - Proj_P(q) ||_2 for each row of q.

    `basis` holds (not necessarily orthonormal) spanning rows, e.g. Qhat.
    """
    q = np.asarray(q, dtype=np.float64)
    B = np.asarray(basis, dtype=np.float64)
    # orthonormalise the span with a library QR
    Qo, _ = np.linalg.qr(B.T)
    proj = (q @ Qo) @ Qo.T
    return np.linalg.norm(q - proj, axis=-1)


# --------------------------------------------------------------------------- #
# Step 1, cheaper: block power iteration on the Gram matrix, and its refresh
# (Algorithm 1, the remark on the SVD line: the decomposition "can be
# accelerated using block power method")
# --------------------------------------------------------------------------- #

def gram_update(G: np.ndarray, Q_new) -> np.ndarray:
    """Gram matrix after more queries have arrived: Q^T Q of the old and new rows together is the sum of
    the two Gram matrices (the same identity that pools the query heads of one KV head)."""
    return np.asarray(G, dtype=np.float64) + gram(Q_new)


def iteration_start(Qhat_prev, d: int = 128, p: int = 32) -> np.ndarray:
    """Start block X0 (d x p) of the iteration.

    Warm start: the directions of a previous Qhat (its non-zero rows, normalised) come first; the block is
    completed to p columns with coordinate vectors e_c, c = 0, s, 2 s, ... with s = d // (p - k) for the
    p - k missing columns (after one multiplication by the Gram matrix these are columns of it, i.e.
    a range-finder start).  Cold start (Qhat_prev None or empty): all p columns are coordinate vectors,
    s = d // p.  This is this build's choice (the paper does not spell an initialisation out); both sides
    of the parity tests use it.
    """
    cols = []
    if Qhat_prev is not None:
        for row in np.asarray(Qhat_prev, dtype=np.float64):
            nrm = np.linalg.norm(row)
            if nrm > 0.0 and len(cols) < p:
                cols.append(row / nrm)
    k = len(cols)
    if k < p:
        step = d // (p - k)
        for j in range(p - k):
            e = np.zeros(d)
            e[j * step] = 1.0
            cols.append(e)
    return np.stack(cols, axis=1)


def subspace_iteration(G: np.ndarray, X0: np.ndarray, iterations: int, r: int):
    """Block power (orthogonal / subspace) iteration on the Gram matrix followed by a Rayleigh-Ritz step.

    X <- orth(X0); `iterations` times X <- orth(G X); then T = X^T G X is diagonalised, T = W diag(theta) W^T,
    and the Ritz pairs (theta_i, x_i = X w_i) with the r largest theta stand in for the eigenpairs:
    Qhat[i] = sqrt(theta_i) x_i^T with the sign convention of `subspace`.  The block may be wider than r
    (oversampling): the iteration then converges like (lambda_{p+1} / lambda_r)^iterations.

    Returns (Qhat (r, d), theta (r,), resid (r,)) with resid_i = ||G x_i - theta_i x_i||_2 / theta_1, the
    relative residual of each Ritz pair (zero at an exact eigenpair).
    """
    G = np.asarray(G, dtype=np.float64)
    d = G.shape[0]
    X, _ = np.linalg.qr(np.asarray(X0, dtype=np.float64))
    for _ in range(iterations):
        X, _ = np.linalg.qr(G @ X)
    Y = G @ X
    T = X.T @ Y
    T = 0.5 * (T + T.T)
    theta, W = np.linalg.eigh(T)
    order = np.argsort(theta)[::-1]
    theta = theta[order]
    Xr = X @ W[:, order]
    Yr = Y @ W[:, order]
    top = max(theta[0], 0.0)
    Qhat = np.zeros((r, d))
    th = np.zeros(r)
    resid = np.zeros(r)
    for i in range(min(r, Xr.shape[1])):
        v = Xr[:, i]
        resid[i] = np.linalg.norm(Yr[:, i] - theta[i] * v) / top if top > 0 else 0.0
        j = int(np.argmax(np.abs(v)))
        if v[j] < 0:
            v = -v
        th[i] = max(theta[i], 0.0)
        Qhat[i] = np.sqrt(th[i]) * v
    return Qhat, th, resid


# --------------------------------------------------------------------------- #
# Step 2: the update matrix  (Prop. 1-2, Lemma 2, Lemma 3 and its Remark)
# --------------------------------------------------------------------------- #
#
# All three routes return U (d x d), strictly block-lower-triangular, with
#     U[t g :, (t-1) g : t g] = B_t H_t        for t = 1 .. T-1
# so that the block update of Lemma 2 reads  k[t g:] += U[t g:, blk] @ dvec.

def _check_block(d: int, g: int) -> int:
    if g <= 0 or d % g:
        raise ValueError("d must be divisible by g")
    return d // g


def update_matrix_lemma(Qhat: np.ndarray, lam: float, g: int) -> np.ndarray:
    """Route (i), the paper's own: P_inv, the A_t^{-1} chain, then B_t H_t.

    Lemma 2 defines P_inv = (I + lambda Qhat^T Qhat)^{-1}, A_t its top-left
    (tg x tg) block, B_t the block below A_t, H_t the last g columns of
    A_t^{-1}.  The Remark after Lemma 3 starts the chain at A_T^{-1} = P and
    Lemma 3 removes one block at a time: with A_{t+1}^{-1} = [[M, N^T],[N, O]],
    A_t^{-1} = M - N^T O^{-1} N.
    """
    Qhat = np.asarray(Qhat, dtype=np.float64)
    d = Qhat.shape[1]
    T = _check_block(d, g)
    P = np.eye(d) + lam * (Qhat.T @ Qhat)
    P_inv = np.linalg.inv(P)
    A_inv = {T: P}
    for t in range(T - 1, 0, -1):
        full = A_inv[t + 1]
        M = full[: t * g, : t * g]
        N = full[t * g:, : t * g]
        O = full[t * g:, t * g:]
        A_inv[t] = M - N.T @ np.linalg.inv(O) @ N
    U = np.zeros((d, d))
    for t in range(1, T):
        B_t = P_inv[t * g:, : t * g]
        H_t = A_inv[t][:, -g:]
        U[t * g:, (t - 1) * g: t * g] = B_t @ H_t
    return U


def update_matrix_kkt(Qhat: np.ndarray, lam: float, g: int) -> np.ndarray:
    """Route (ii), the plain definition: solve Lemma 2's problem generically.

    Column j of panel t is the tail of  argmin delta^T P delta  subject to
    delta[:tg] = unit vector at (t-1)g + j.  The equality-constrained quadratic
    programme is solved through its KKT linear system with a library solver;
    nothing of the paper's closed form is used.
    """
    Qhat = np.asarray(Qhat, dtype=np.float64)
    d = Qhat.shape[1]
    T = _check_block(d, g)
    P = np.eye(d) + lam * (Qhat.T @ Qhat)
    U = np.zeros((d, d))
    for t in range(1, T):
        nfix = t * g
        Tm = np.zeros((nfix, d))
        Tm[:, :nfix] = np.eye(nfix)
        KKT = np.zeros((d + nfix, d + nfix))
        KKT[:d, :d] = 2.0 * P
        KKT[:d, d:] = -Tm.T
        KKT[d:, :d] = Tm
        for j in range(g):
            rhs = np.zeros(d + nfix)
            rhs[d + (t - 1) * g + j] = 1.0
            sol = np.linalg.solve(KKT, rhs)
            U[nfix:, (t - 1) * g + j] = sol[nfix:d]
    return U


def update_matrix_lowrank(Qhat: np.ndarray, lam: float, g: int) -> np.ndarray:
    """Route (iii): rank-r closed form of the same matrix, incl. lambda = +inf.

    Eliminating the free tail of Lemma 2's problem gives
        W_t = -P[tg:, tg:]^{-1} P[tg:, blk],
    and with P = I + lambda Qhat^T Qhat the Woodbury identity (the paper's
    footnote on O(r d^2)) turns this into
        W_t = -Qr^T (I/lambda + Qr Qr^T)^{-1} Qb,
    Qb = Qhat[:, blk], Qr = Qhat[:, tg:].  For lambda = +inf (the equality
    constraint of Eq. (1)) the limit is  -pinv(Qr) Qb, the minimum-norm
    least-squares tail, also when the constraint cannot be met exactly.
    """
    Qhat = np.asarray(Qhat, dtype=np.float64)
    r, d = Qhat.shape
    T = _check_block(d, g)
    U = np.zeros((d, d))
    if r == 0 or lam == 0:
        return U
    for t in range(1, T):
        Qb = Qhat[:, (t - 1) * g: t * g]
        Qr = Qhat[:, t * g:]
        if np.isinf(lam):
            W = -np.linalg.pinv(Qr) @ Qb
        else:
            S = np.eye(r) / lam + Qr @ Qr.T
            W = -Qr.T @ np.linalg.solve(S, Qb)
        U[t * g:, (t - 1) * g: t * g] = W
    return U


# --------------------------------------------------------------------------- #
# Step 3: the quantizer  (Section 2 "Quantization"; Algorithm 1, function Quant)
# --------------------------------------------------------------------------- #

def rtn_group(x: np.ndarray, bits: int, axis: int = -1):
    """Asymmetric min/max round-to-nearest of one group (Section 2).

    m = min, M = max, Delta = (M - m) / (2^b - 1), code = round((x - m)/Delta),
    deq = code * Delta + m.  Readings where the paper is silent: Delta and m
    are rounded to fp16 BEFORE use (they are what is stored), ties round to
    even, codes are clamped to [0, 2^b - 1] (needed once m is rounded), and a
    constant group (Delta = 0) gets code 0.

    Returns (codes uint8, scale fp16, zero fp16, xhat float64); scale/zero keep
    a singleton `axis`.
    """
    x = np.asarray(x, dtype=np.float64)
    levels = float((1 << bits) - 1)
    m = x.min(axis=axis, keepdims=True)
    M = x.max(axis=axis, keepdims=True)
    delta = (M - m) / levels
    scale = delta.astype(np.float16)
    zero = m.astype(np.float16)
    s64 = scale.astype(np.float64)
    z64 = zero.astype(np.float64)
    safe = np.where(s64 > 0, s64, 1.0)
    u = (x - z64) / safe
    c = np.clip(np.rint(u), 0.0, levels)
    c = np.where(s64 > 0, c, 0.0)
    xhat = c * s64 + z64
    return c.astype(np.uint8), scale, zero, xhat


def quantize_keys(K: np.ndarray, U, bits: int, G: int, g: int, axis: str = "token",
                  trace: bool = False):
    """The iteration of Algorithm 1's `Quant`, block update of Lemma 2.

    K is (n, d): n key vectors of one head.  For t = 1..T the g channels of
    block t are quantized (from their CURRENT values) and frozen at their
    dequantized values; if t < T the remaining channels receive
        k[t g:] += (B_t H_t) dvec,   dvec = deq(qtz(k_blk)) - k_blk.
    U = None (or r = 0, lambda = 0) is plain round-to-nearest.

    axis = "token"   : each key's d channels are cut into groups of G
                       consecutive channels (statistics per token, per group).
                       G | g: a block holds g/G whole groups.  g | G: a group
                       spans G/g blocks; its statistics are taken once, when
                       its first block is reached, from the current values of
                       all its G channels, and later blocks of that group reuse
                       them (codes clamped).
    axis = "channel" : the paper's own layout: statistics per channel over G
                       consecutive tokens (n must be a multiple of G).

    Returns dict(codes uint8 (n, d), scale fp16, zero fp16, xhat float64 (n, d));
    scale/zero are (n, d/G) for "token" and (n/G, d) for "channel".  With
    trace=True the dict also holds "states": the working copy after each
    iteration (after the update when t < T), for checking the invariants.
    """
    x = np.array(K, dtype=np.float64, copy=True)
    n, d = x.shape
    T = _check_block(d, g)
    levels = float((1 << bits) - 1)
    codes = np.zeros((n, d), dtype=np.uint8)
    if axis == "token":
        if d % G or not (g % G == 0 or G % g == 0):
            raise ValueError("need G | d and (G | g or g | G)")
        scale = np.zeros((n, d // G), dtype=np.float16)
        zero = np.zeros((n, d // G), dtype=np.float16)
    elif axis == "channel":
        if n % G:
            raise ValueError("token count must be a multiple of G")
        scale = np.zeros((n // G, d), dtype=np.float16)
        zero = np.zeros((n // G, d), dtype=np.float16)
    else:
        raise ValueError(axis)

    states = []
    for t in range(T):
        lo, hi = t * g, (t + 1) * g
        if axis == "token":
            # statistics of every group that starts inside this block
            first = lo // G if lo % G == 0 else None
            if first is not None:
                n_new = max(1, g // G)
                for gi in range(first, first + n_new):
                    seg = x[:, gi * G:(gi + 1) * G]
                    m = seg.min(axis=1)
                    M = seg.max(axis=1)
                    scale[:, gi] = ((M - m) / levels).astype(np.float16)
                    zero[:, gi] = m.astype(np.float16)
            gidx = np.arange(lo, hi) // G
            s64 = scale[:, gidx].astype(np.float64)
            z64 = zero[:, gidx].astype(np.float64)
        else:
            blk = x[:, lo:hi].reshape(n // G, G, g)
            m = blk.min(axis=1)
            M = blk.max(axis=1)
            scale[:, lo:hi] = ((M - m) / levels).astype(np.float16)
            zero[:, lo:hi] = m.astype(np.float16)
            s64 = np.repeat(scale[:, lo:hi].astype(np.float64), G, axis=0)
            z64 = np.repeat(zero[:, lo:hi].astype(np.float64), G, axis=0)
        xb = x[:, lo:hi]
        safe = np.where(s64 > 0, s64, 1.0)
        c = np.clip(np.rint((xb - z64) / safe), 0.0, levels)
        c = np.where(s64 > 0, c, 0.0)
        xq = c * s64 + z64
        dvec = xq - xb
        codes[:, lo:hi] = c.astype(np.uint8)
        x[:, lo:hi] = xq
        if U is not None and t < T - 1:
            x[:, hi:] += dvec @ np.asarray(U, dtype=np.float64)[hi:, lo:hi].T
        if trace:
            states.append(x.copy())
    out = {"codes": codes, "scale": scale, "zero": zero, "xhat": x}
    if trace:
        out["states"] = states
    return out


def dequantize_keys(codes: np.ndarray, scale: np.ndarray, zero: np.ndarray,
                    G: int, axis: str = "token") -> np.ndarray:
    """deq(c) = c * Delta + m  (Section 2), float64, from unpacked codes."""
    codes = np.asarray(codes)
    s64 = np.asarray(scale).astype(np.float64)
    z64 = np.asarray(zero).astype(np.float64)
    if axis == "token":
        s = np.repeat(s64, G, axis=-1)
        z = np.repeat(z64, G, axis=-1)
    else:
        s = np.repeat(s64, G, axis=-2)
        z = np.repeat(z64, G, axis=-2)
    return codes.astype(np.float64) * s + z


def key_scores(q: np.ndarray, codes: np.ndarray, scale: np.ndarray, zero: np.ndarray,
               G: int, out_scale: float = 1.0, axis: str = "token") -> np.ndarray:
    """Attention logits of decode-time queries against the QUANTIZED keys:
    out_scale * q . deq(code)^T, with deq as in Section 2.  This is what the
    decoding phase of Algorithm 1 feeds to the softmax for the tokens that have
    left the residual buffer (the full-precision tail is an ordinary q . k^T).

    q (n_q, d) float; codes (n, d) unpacked; scale/zero as for dequantize_keys.
    Returns (n_q, n) float64: the definition written out, dequantize then a
    library matrix product.
    """
    khat = dequantize_keys(codes, scale, zero, G, axis=axis)
    return float(out_scale) * (np.asarray(q, dtype=np.float64) @ khat.T)


def rope_rotate(x: np.ndarray, positions: np.ndarray, inv_freq: np.ndarray) -> np.ndarray:
    """Rotary position embedding of rows x (n, d) at integer positions (n,): channel pairs (c, c + d/2),
    c < d/2, are rotated by the angle positions * inv_freq[c]:
        x'_c       = x_c cos - x_{c+d/2} sin
        x'_{c+d/2} = x_{c+d/2} cos + x_c sin
    (the "rotate half" convention of the Llama models the paper evaluates).  float64."""
    x = np.asarray(x, dtype=np.float64)
    half = x.shape[-1] // 2
    ang = np.asarray(positions, dtype=np.float64)[:, None] * np.asarray(inv_freq, dtype=np.float64)[None, :]
    c, s_ = np.cos(ang), np.sin(ang)
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s_, b * c + a * s_], axis=-1)


def key_scores_rope(q: np.ndarray, codes: np.ndarray, scale: np.ndarray, zero: np.ndarray, G: int,
                    inv_freq: np.ndarray, pos0: int = 0, out_scale: float = 1.0,
                    axis: str = "token") -> np.ndarray:
    """Logits against keys that were quantized BEFORE the rotary embedding (the SQuat-pre variant of
    Section 4: the cache holds pre-RoPE keys and positions are applied on the fly after
    dequantization): out_scale * q . RoPE_{pos0 + t}(deq(code_t)).  q is taken as given (the caller
    has already rotated it to its own position).  `axis` as in dequantize_keys ("channel": the
    grouping Algorithm 1 prints, statistics per channel over G tokens).  Returns (n_q, n) float64."""
    khat = dequantize_keys(codes, scale, zero, G, axis=axis)
    rot = rope_rotate(khat, pos0 + np.arange(khat.shape[0]), inv_freq)
    return float(out_scale) * (np.asarray(q, dtype=np.float64) @ rot.T)


class CacheOracle:
    """Residual-buffer bookkeeping of Algorithm 1 for ONE head of ONE sequence,
    written out with Python lists (prefill: "r = l mod R", K_full = the last r
    keys; decoding: append, and when the buffer holds R keys quantize all of them
    and empty it), plus the value rule of the appendix "Details of Our Main
    Algorithm" (values per token, the most recent R in full precision, the oldest
    one quantized when token R + 1 arrives).  key_axis="token": keys use
    per-token groups of G channels (this build's contract), so a flush of R keys
    is R independent runs of `quantize_keys`; key_axis="channel": the grouping
    Algorithm 1 prints, a flush is R / 32 groups of 32 tokens quantized per
    channel (G then applies to the values only).
    """

    def __init__(self, U, bits: int, G: int, g: int, R: int, values: bool = False, key_axis: str = "token"):
        self.U, self.bits, self.G, self.g, self.R, self.values = U, bits, G, g, R, values
        self.key_axis = key_axis
        if key_axis == "channel" and R % 32:
            raise ValueError("per-channel keys are flushed in whole groups of 32 tokens")
        # codes: one entry per quantized key; scale / zero: one entry per key (token axis) or per group
        # of 32 keys (channel axis)
        self.k_codes, self.k_scale, self.k_zero = [], [], []
        self.k_full = []                                           # residual keys, oldest first
        self.v_codes, self.v_scale, self.v_zero = [], [], []
        self.v_full = []                                           # residual values, oldest first
        self.n_tokens = 0

    def _quant_keys(self, rows):
        rows = np.asarray(rows, dtype=np.float64)
        if self.key_axis == "channel":
            out = quantize_keys(rows, self.U, self.bits, 32, self.g, axis="channel")
            n_meta = len(rows) // 32
        else:
            out = quantize_keys(rows, self.U, self.bits, self.G, self.g)
            n_meta = len(rows)
        for i in range(len(rows)):
            self.k_codes.append(out["codes"][i])
        for i in range(n_meta):
            self.k_scale.append(out["scale"][i])
            self.k_zero.append(out["zero"][i])

    def _quant_value(self, row):
        out = quantize_keys(np.asarray(row, dtype=np.float64)[None], None, self.bits, self.G, len(row))
        self.v_codes.append(out["codes"][0])
        self.v_scale.append(out["scale"][0])
        self.v_zero.append(out["zero"][0])

    def prefill(self, K, V=None):
        K = np.asarray(K, dtype=np.float64)
        l = K.shape[0]
        r = l % self.R
        if l - r > 0:
            self._quant_keys(K[: l - r])
        self.k_full = [K[i] for i in range(l - r, l)]
        if self.values:
            V = np.asarray(V, dtype=np.float64)
            for i in range(l):
                self._push_value(V[i])
        self.n_tokens = l

    def _push_value(self, v):
        self.v_full.append(np.asarray(v, dtype=np.float64))
        if len(self.v_full) == self.R + 1:
            self._quant_value(self.v_full.pop(0))

    def append(self, k, v=None):
        self.k_full.append(np.asarray(k, dtype=np.float64))
        if len(self.k_full) == self.R:
            self._quant_keys(self.k_full)
            self.k_full = []
        if self.values:
            self._push_value(v)
        self.n_tokens += 1

    def scores(self, q, out_scale: float = 1.0):
        """Logits of q (n_q, d) against all cached keys: quantized ones first, then the residual ones."""
        q = np.asarray(q, dtype=np.float64)
        parts = []
        if self.k_codes:
            parts.append(key_scores(q, np.stack(self.k_codes), np.stack(self.k_scale), np.stack(self.k_zero),
                                    32 if self.key_axis == "channel" else self.G, out_scale, axis=self.key_axis))
        if self.k_full:
            parts.append(float(out_scale) * (q @ np.stack(self.k_full).T))
        return np.concatenate(parts, axis=1) if parts else np.zeros((q.shape[0], 0))

    def scores_rope(self, q, inv_freq, pos0: int = 0, out_scale: float = 1.0):
        """The same for a cache that holds keys as they are before the rotary embedding (SQuat-pre,
        Section 4): cached token t is rotated to position pos0 + t after dequantization (quantized
        keys) or as it is (residual keys), then meets q."""
        q = np.asarray(q, dtype=np.float64)
        parts = []
        nq = len(self.k_codes)
        if nq:
            parts.append(key_scores_rope(q, np.stack(self.k_codes), np.stack(self.k_scale), np.stack(self.k_zero),
                                         32 if self.key_axis == "channel" else self.G, inv_freq, pos0, out_scale,
                                         axis=self.key_axis))
        if self.k_full:
            rot = rope_rotate(np.stack(self.k_full), pos0 + nq + np.arange(len(self.k_full)), inv_freq)
            parts.append(float(out_scale) * (q @ rot.T))
        return np.concatenate(parts, axis=1) if parts else np.zeros((q.shape[0], 0))


# --------------------------------------------------------------------------- #
# Packed layout (ours to define; the paper does not fix one)
# --------------------------------------------------------------------------- #

def pack_codes(codes: np.ndarray, bits: int) -> np.ndarray:
    """Little-endian along channels: channel c of a key sits in 32-bit word
    c // (32/bits) at bit offset bits * (c mod 32/bits)."""
    codes = np.asarray(codes, dtype=np.uint32)
    per = 32 // bits
    d = codes.shape[-1]
    if d % per:
        raise ValueError("d must fill whole words")
    grp = codes.reshape(codes.shape[:-1] + (d // per, per))
    shifts = (np.arange(per, dtype=np.uint32) * np.uint32(bits))
    return np.bitwise_or.reduce(grp << shifts, axis=-1).astype(np.uint32)


def unpack_codes(words: np.ndarray, bits: int) -> np.ndarray:
    words = np.asarray(words, dtype=np.uint32)
    per = 32 // bits
    shifts = (np.arange(per, dtype=np.uint32) * np.uint32(bits))
    mask = np.uint32((1 << bits) - 1)
    out = (words[..., None] >> shifts) & mask
    return out.reshape(words.shape[:-1] + (words.shape[-1] * per,)).astype(np.uint8)


def pack_codes_tokens(codes: np.ndarray, bits: int) -> np.ndarray:
    """Packed layout of the per-channel mode (ours to define): tokens are cut
    into tiles of 32; within a tile every channel owns `bits` consecutive 32-bit
    words that hold its 32 codes little-endian ALONG TOKENS: token j of the
    tile sits in word j // (32/bits) at bit offset bits * (j mod 32/bits).

    codes (..., n, d) -> words (..., n/32, d, bits) uint32; n a multiple of 32.
    """
    codes = np.asarray(codes, dtype=np.uint32)
    n, d = codes.shape[-2:]
    if n % 32:
        raise ValueError("token count must be a multiple of 32")
    per = 32 // bits
    lead = codes.shape[:-2]
    # (..., tile, word, token-in-word, channel) -> (..., tile, channel, word, token-in-word)
    grp = codes.reshape(lead + (n // 32, bits, per, d))
    grp = np.ascontiguousarray(np.moveaxis(grp, -1, -3))
    shifts = (np.arange(per, dtype=np.uint32) * np.uint32(bits))
    return np.ascontiguousarray(np.bitwise_or.reduce(grp << shifts, axis=-1).astype(np.uint32))


def unpack_codes_tokens(words: np.ndarray, bits: int) -> np.ndarray:
    """Inverse of pack_codes_tokens: words (..., n/32, d, bits) -> codes (..., n, d) uint8."""
    words = np.asarray(words, dtype=np.uint32)
    per = 32 // bits
    tiles, d, nw = words.shape[-3:]
    if nw != bits:
        raise ValueError("last axis must hold `bits` words per channel")
    shifts = (np.arange(per, dtype=np.uint32) * np.uint32(bits))
    mask = np.uint32((1 << bits) - 1)
    out = (words[..., None] >> shifts) & mask                # (..., tile, d, word, token-in-word)
    out = np.moveaxis(out, -3, -1)                           # (..., tile, word, token-in-word, d)
    return out.reshape(words.shape[:-3] + (tiles * 32, d)).astype(np.uint8)


# --------------------------------------------------------------------------- #
# Teacher-forced replay: classify the disagreements of another implementation
# --------------------------------------------------------------------------- #

def _fp16_neighbours_mid(v: np.ndarray):
    """For float64 v: the fp16 value RNE picks, and |v - nearest fp16 rounding
    midpoint| (distance to the point where the choice would flip)."""
    h = v.astype(np.float16)
    h64 = h.astype(np.float64)
    up = np.nextafter(h, np.float16(np.inf)).astype(np.float64)
    dn = np.nextafter(h, np.float16(-np.inf)).astype(np.float64)
    other = np.where(v >= h64, up, dn)
    mid = 0.5 * (h64 + other)
    return h, np.abs(v - mid), other


def replay_classify(K: np.ndarray, U, bits: int, G: int, g: int,
                    codes_other: np.ndarray, scale_other: np.ndarray,
                    zero_other: np.ndarray, tol: float = 1e-5, axis: str = "token"):
    """Replay `quantize_keys` in float64 while FORCING the other
    implementation's codes and fp16 metadata for all earlier decisions, and
    classify every decision where float64 would have chosen differently.

    A differing code is `explained` when the float64 pre-rounding value
    (x - m_h)/Delta_h lies within `tol` of a rounding boundary (a half-integer,
    or the clamp edges); a differing fp16 scale/zero is explained when the other
    value is the adjacent fp16 number and the float64 value lies within
    tol * Delta of the fp16 rounding midpoint.  Anything else is `unexplained`.
    Forcing removes downstream cascades, so each root cause is counted once.

    `axis` as in quantize_keys; scale_other/zero_other are (n, d/G) for "token"
    and (n/G, d) for "channel".

    Returns dict with counts: n_codes, code_diff, code_unexplained,
    n_meta, meta_diff, meta_unexplained, and worst distances seen.
    """
    x = np.array(K, dtype=np.float64, copy=True)
    n, d = x.shape
    T = _check_block(d, g)
    levels = float((1 << bits) - 1)
    co = np.asarray(codes_other).astype(np.float64)
    so = np.asarray(scale_other).astype(np.float16)
    zo = np.asarray(zero_other).astype(np.float16)
    Ud = None if U is None else np.asarray(U, dtype=np.float64)
    if axis not in ("token", "channel"):
        raise ValueError(axis)
    if axis == "channel" and n % G:
        raise ValueError("token count must be a multiple of G")
    n_meta = 2 * n * (d // G) if axis == "token" else 2 * (n // G) * d
    out = dict(n_codes=n * d, code_diff=0, code_unexplained=0,
               n_meta=n_meta, meta_diff=0, meta_unexplained=0,
               worst_code_dist=0.0, worst_meta_dist=0.0)

    def check_meta(m, M, s_other, z_other):
        dl = (M - m) / levels
        for v, other in ((dl, s_other), (m, z_other)):
            mine, dist, neigh = _fp16_neighbours_mid(v)
            diff = mine != other
            if diff.any():
                o64 = other.astype(np.float64)
                adjacent = o64 == neigh
                ok = adjacent & (dist <= tol * np.maximum(dl, 1e-300))
                out["meta_diff"] += int(diff.sum())
                out["meta_unexplained"] += int((diff & ~ok).sum())
                rel = dist[diff] / np.maximum(dl[diff], 1e-300)
                out["worst_meta_dist"] = max(out["worst_meta_dist"], float(rel.max()))

    for t in range(T):
        lo, hi = t * g, (t + 1) * g
        if axis == "token":
            if lo % G == 0:
                n_new = max(1, g // G)
                first = lo // G
                for gi in range(first, first + n_new):
                    seg = x[:, gi * G:(gi + 1) * G]
                    check_meta(seg.min(axis=1), seg.max(axis=1), so[:, gi], zo[:, gi])
            gidx = np.arange(lo, hi) // G
            s64 = so[:, gidx].astype(np.float64)
            z64 = zo[:, gidx].astype(np.float64)
        else:
            blk = x[:, lo:hi].reshape(n // G, G, g)
            check_meta(blk.min(axis=1), blk.max(axis=1), so[:, lo:hi], zo[:, lo:hi])
            s64 = np.repeat(so[:, lo:hi].astype(np.float64), G, axis=0)
            z64 = np.repeat(zo[:, lo:hi].astype(np.float64), G, axis=0)
        xb = x[:, lo:hi]
        safe = np.where(s64 > 0, s64, 1.0)
        u = (xb - z64) / safe
        c = np.clip(np.rint(u), 0.0, levels)
        c = np.where(s64 > 0, c, 0.0)
        cg = co[:, lo:hi]
        diff = c != cg
        if diff.any():
            # distance of u to the boundary between the two candidate codes
            bound = 0.5 * (c + cg)
            dist = np.abs(u - bound)
            ok = (np.abs(c - cg) == 1) & (dist <= tol)
            out["code_diff"] += int(diff.sum())
            out["code_unexplained"] += int((diff & ~ok).sum())
            out["worst_code_dist"] = max(out["worst_code_dist"], float(dist[diff].max()))
        xq = cg * s64 + z64
        dvec = xq - xb
        x[:, lo:hi] = xq
        if Ud is not None and t < T - 1:
            x[:, hi:] += dvec @ Ud[hi:, lo:hi].T
    return out
