"""Pins for the float64 oracle: each test checks it against something other
than itself -- hand-worked numbers, closed forms, library routines used in a
different way, brute force on tiny sizes, or invariants the paper proves."""
import os

import numpy as np
import pytest
import scipy.optimize

from oracle import squat_oracle as O
from paper_2503_24358_amd import synth   # seeded input generators only (no method arithmetic)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            yield [p.strip() for p in line.split("|")]


# ----------------------------------------------------------------- quantizer
def test_rtn_hand_worked_cases():
    """Section 2 formulas, worked by hand (tests/golden/rtn_worked.txt)."""
    for bits, xs, dl, m, cs, dq in _rows("rtn_worked.txt"):
        x = np.array([float(v) for v in xs.split()])
        codes, scale, zero, xhat = O.rtn_group(x, int(bits))
        assert float(scale[0]) == float(dl)
        assert float(zero[0]) == float(m)
        assert codes.tolist() == [int(v) for v in cs.split()]
        assert xhat.tolist() == [float(v) for v in dq.split()]


def test_packed_size_matches_paper_kv_size():
    """Tables 1-2: the format's own share is the lower bound of the printed KV sizes."""
    for bits, group, frac, printed in _rows("kv_size.txt"):
        bits, group = int(bits), int(group)
        d = 128
        codes = np.zeros((1, d), dtype=np.uint8)
        words = O.pack_codes(codes, bits)
        nbytes = words.nbytes + 2 * 2 * (d // group)
        assert nbytes / (2 * d) == float(frac)
        assert float(frac) <= float(printed)


@pytest.mark.parametrize("bits", [2, 4])
def test_rtn_properties(bits):
    gen = np.random.default_rng(1)
    x = gen.standard_normal((200, 32)) * gen.uniform(0.01, 50, size=(200, 1))
    codes, scale, zero, xhat = O.rtn_group(x, bits, axis=1)
    L = (1 << bits) - 1
    assert codes.min() == 0 and codes.max() == L
    s = scale.astype(np.float64)
    # every element within half a step of its reconstruction, plus the slack the
    # fp16 rounding of zero/scale can add at the clamped ends
    slack = np.abs(zero.astype(np.float64)) * 2.0 ** -11 + L * s * 2.0 ** -11
    assert np.all(np.abs(xhat - x) <= 0.5 * s + slack + 1e-12)
    # min and max land on the extreme codes
    assert np.all(codes[np.arange(200), x.argmin(1)] == 0)
    assert np.all(codes[np.arange(200), x.argmax(1)] == L)


@pytest.mark.parametrize("bits,G,g", [(2, 32, 32), (4, 32, 64), (2, 128, 32), (4, 64, 128), (2, 32, 128)])
def test_r0_reduces_to_plain_rtn(bits, G, g):
    """Section 3.3: lambda = 0 (or r = 0) is a compression-based quantizer, i.e.
    independent per-group round-to-nearest of the ORIGINAL key."""
    gen = np.random.default_rng(2)
    K = gen.standard_normal((64, 128)) * 3
    d = 128
    for U in (None, np.zeros((d, d)), O.update_matrix_lowrank(gen.standard_normal((5, d)), 0.0, g)):
        out = O.quantize_keys(K, U, bits, G, g)
        c, s, z, xh = O.rtn_group(K.reshape(64, d // G, G), bits, axis=2)
        assert np.array_equal(out["codes"], c.reshape(64, d))
        assert np.array_equal(out["scale"], s.reshape(64, d // G))
        assert np.array_equal(out["zero"], z.reshape(64, d // G))
        assert np.array_equal(out["xhat"], xh.reshape(64, d))


def test_channel_axis_r0_is_per_channel_rtn():
    gen = np.random.default_rng(3)
    K = gen.standard_normal((96, 64))
    out = O.quantize_keys(K, None, 2, 32, 32, axis="channel")
    for blk in range(3):
        for ch in range(64):
            c, s, z, xh = O.rtn_group(K[blk * 32:(blk + 1) * 32, ch], 2)
            assert np.array_equal(out["codes"][blk * 32:(blk + 1) * 32, ch], c)
            assert out["scale"][blk, ch] == s[0] and out["zero"][blk, ch] == z[0]


def test_pack_unpack_roundtrip_and_layout():
    gen = np.random.default_rng(4)
    for bits in (2, 4):
        codes = gen.integers(0, 1 << bits, size=(7, 128)).astype(np.uint8)
        w = O.pack_codes(codes, bits)
        assert w.shape == (7, 128 * bits // 32) and w.dtype == np.uint32
        assert np.array_equal(O.unpack_codes(w, bits), codes)
    one = np.zeros((1, 128), dtype=np.uint8)
    one[0, 17] = 3
    w = O.pack_codes(one, 2)
    assert w[0, 1] == (3 << 2) and w.sum() == (3 << 2)
    one[0, 17] = 0
    one[0, 9] = 5
    w = O.pack_codes(one, 4)
    assert w[0, 1] == (5 << 4)


def test_dequantize_is_the_definition():
    gen = np.random.default_rng(5)
    K = gen.standard_normal((16, 128))
    Qh = gen.standard_normal((4, 128))
    U = O.update_matrix_lowrank(Qh, 0.05, 32)
    out = O.quantize_keys(K, U, 2, 32, 32)
    back = O.dequantize_keys(out["codes"], out["scale"], out["zero"], 32)
    assert np.array_equal(back, out["xhat"])
    # element by element, written out
    for i in (0, 7):
        for c in (0, 31, 32, 127):
            exp = float(out["codes"][i, c]) * float(out["scale"][i, c // 32]) + float(out["zero"][i, c // 32])
            assert back[i, c] == exp


# -------------------------------------------------------------- update matrix
@pytest.mark.parametrize("d,g,r,lam", [(16, 4, 3, 0.7), (24, 8, 5, 0.01), (12, 1, 2, 2.0), (128, 32, 16, 1e-3), (128, 64, 40, 5e-4)])
def test_three_routes_agree(d, g, r, lam):
    gen = np.random.default_rng(10 + d)
    Qh = gen.standard_normal((r, d)) * (30.0 if d == 128 else 1.0)
    U1 = O.update_matrix_lemma(Qh, lam, g)
    U2 = O.update_matrix_kkt(Qh, lam, g)
    U3 = O.update_matrix_lowrank(Qh, lam, g)
    sc = max(1.0, np.abs(U2).max())
    assert np.abs(U1 - U2).max() <= 1e-9 * sc
    assert np.abs(U3 - U2).max() <= 1e-9 * sc
    # strictly block lower triangular
    for t in range(d // g):
        assert not U1[t * g:(t + 1) * g, t * g:].any()


def test_update_matrix_is_the_constrained_minimiser_brute_force():
    """Lemma 2 on tiny d: a generic least-squares routine and a generic
    numerical optimiser both land on the same tail as B_t H_t d."""
    d, g, r, lam = 8, 2, 3, 1.3
    gen = np.random.default_rng(20)
    Qh = gen.standard_normal((r, d))
    U = O.update_matrix_lemma(Qh, lam, g)
    Mst = np.vstack([np.eye(d), np.sqrt(lam) * Qh])     # ||M delta||^2 = delta^T P delta
    for t in range(1, d // g):
        dvec = gen.standard_normal(g)
        b = np.zeros(t * g)
        b[-g:] = dvec
        tail_ls = np.linalg.lstsq(Mst[:, t * g:], -Mst[:, :t * g] @ b, rcond=None)[0]
        mine = U[t * g:, (t - 1) * g:t * g] @ dvec
        assert np.allclose(mine, tail_ls, atol=1e-11)

        def obj(z):
            dl = np.concatenate([b, z])
            return dl @ dl + lam * np.sum((Qh @ dl) ** 2)
        res = scipy.optimize.minimize(obj, np.zeros(d - t * g), method="BFGS", options={"gtol": 1e-10})
        assert np.allclose(mine, res.x, atol=1e-5)
        # no random perturbation does better
        f0 = obj(mine)
        for _ in range(50):
            assert obj(mine + 1e-3 * gen.standard_normal(d - t * g)) >= f0 - 1e-13


def test_g1_matches_one_coordinate_rule():
    """Prop. 1 is Lemma 2 at g = 1; the same tail also follows from the classic
    single-coordinate compensation on the trailing block of P (invert
    P[t-1:, t-1:], take its first column over its first entry)."""
    d, r, lam = 10, 3, 0.9
    gen = np.random.default_rng(21)
    Qh = gen.standard_normal((r, d))
    P = np.eye(d) + lam * Qh.T @ Qh
    P_inv = np.linalg.inv(P)
    U = O.update_matrix_lemma(Qh, lam, 1)
    for t in range(1, d):
        # Prop. 1 literally: B_t h_t with A_t the leading t x t block of P_inv
        A_t = P_inv[:t, :t]
        h_t = np.linalg.inv(A_t)[:, -1]
        B_t = P_inv[t:, :t]
        assert np.allclose(U[t:, t - 1], B_t @ h_t, atol=1e-11)
        # classic one-coordinate compensation on the trailing problem: pinning
        # coordinate 0 to e moves the others by e * Hinv[1:, 0] / Hinv[0, 0]
        Hinv = np.linalg.inv(P[t - 1:, t - 1:])
        assert np.allclose(U[t:, t - 1], Hinv[1:, 0] / Hinv[0, 0], atol=1e-11)


def test_lambda_zero_and_rank_zero_give_zero_matrix():
    gen = np.random.default_rng(22)
    Qh = gen.standard_normal((4, 32))
    assert not O.update_matrix_lemma(Qh, 0.0, 8).any()
    assert not O.update_matrix_lowrank(Qh, 0.0, 8).any()
    assert not O.update_matrix_lowrank(np.zeros((0, 32)), 1.0, 8).any()
    assert not O.update_matrix_lemma(np.zeros((3, 32)), 1.0, 8).any()


def test_hard_constraint_is_the_large_lambda_limit():
    d, g, r = 16, 4, 3
    gen = np.random.default_rng(23)
    Qh = gen.standard_normal((r, d))
    Uh = O.update_matrix_lowrank(Qh, np.inf, g)
    Ub = O.update_matrix_kkt(Qh, 1e9, g)
    assert np.abs(Uh - Ub).max() < 1e-5
    # each panel annihilates the subspace component of the frozen block's error
    for t in range(1, d // g):
        blk = slice((t - 1) * g, t * g)
        assert np.allclose(Qh[:, blk] + Qh[:, t * g:] @ Uh[t * g:, blk], 0, atol=1e-12)


# ------------------------------------------------------------- the iteration
def _setup(d=128, r=8, n=48, seed=30, qscale=20.0):
    gen = np.random.default_rng(seed)
    Qh = gen.standard_normal((r, d)) * qscale
    K = gen.standard_normal((n, d)) * 2
    K[:, gen.choice(d, 4, replace=False)] *= 10
    return Qh, K


@pytest.mark.parametrize("bits,G,g,lam", [(2, 32, 32, 1e-3), (4, 32, 64, 5e-4), (2, 64, 32, 1e-2), (2, 32, 32, np.inf)])
def test_each_step_is_lemma2_optimum_generic_solver(bits, G, g, lam):
    """Re-run the iteration with (a) the scalar quantizer applied to the current
    block and (b) the tail recomputed by a generic least-squares solve of
    Lemma 2's problem, and compare with quantize_keys driven by U."""
    d = 128
    Qh, K = _setup(d=d, n=6)
    U = O.update_matrix_lowrank(Qh, lam, g)
    out = O.quantize_keys(K, U, bits, G, g, trace=True)
    L = (1 << bits) - 1
    if np.isinf(lam):
        Mst = None
    else:
        Mst = np.vstack([np.eye(d), np.sqrt(lam) * Qh])
    for i in range(K.shape[0]):
        x = K[i].copy()
        meta = {}
        for t in range(d // g):
            lo, hi = t * g, (t + 1) * g
            if lo % G == 0:
                for gi in range(lo // G, lo // G + max(1, g // G)):
                    seg = x[gi * G:(gi + 1) * G]
                    meta[gi] = (np.float64(np.float16((seg.max() - seg.min()) / L)), np.float64(np.float16(seg.min())))
            xq = np.empty(g)
            for j in range(lo, hi):
                dl, m = meta[j // G]
                c = 0.0 if dl == 0 else min(max(np.rint((x[j] - m) / dl), 0), L)
                assert out["codes"][i, j] == c
                xq[j - lo] = c * dl + m
            dvec = xq - x[lo:hi]
            x[lo:hi] = xq
            if t < d // g - 1:
                if Mst is not None:
                    tail = np.linalg.lstsq(Mst[:, hi:], -Mst[:, lo:hi] @ dvec, rcond=None)[0]
                else:
                    # hard constraint: min ||tail|| s.t. Qh[:, hi:] tail = -Qh[:, blk] dvec
                    tail = np.linalg.lstsq(Qh[:, hi:], -Qh[:, lo:hi] @ dvec, rcond=None)[0]
                x[hi:] += tail
            assert np.allclose(x, out["states"][t][i], atol=1e-9)
        assert np.allclose(x, out["xhat"][i], atol=1e-9)


@pytest.mark.parametrize("g", [32, 64])
def test_soft_invariant_first_order_condition(g):
    """After the update of step t the accumulated change delta = state - k
    satisfies (P delta)[t g:] = 0 (stationarity of Lemma 2 accumulated)."""
    Qh, K = _setup()
    lam = 1e-3
    U = O.update_matrix_lemma(Qh, lam, g)
    out = O.quantize_keys(K, U, 2, 32, g, trace=True)
    P = np.eye(128) + lam * Qh.T @ Qh
    T = 128 // g
    for t in range(T - 1):
        delta = out["states"][t] - K
        resid = (delta @ P)[:, (t + 1) * g:]
        assert np.abs(resid).max() <= 1e-9 * np.abs(delta @ P).max()


def test_hard_invariant_error_orthogonal_until_last_block():
    """lambda = +inf: Qhat (state - k) = 0 after every step but the last, so the
    final error's projection is exactly the last block's own rounding error."""
    Qh, K = _setup(r=8)
    g = 32
    U = O.update_matrix_lowrank(Qh, np.inf, g)
    out = O.quantize_keys(K, U, 2, 32, g, trace=True)
    scale = np.abs(Qh).max() * np.abs(K).max()
    for t in range(3):
        assert np.abs((out["states"][t] - K) @ Qh.T).max() <= 1e-12 * scale
    e_last = out["xhat"][:, 96:] - out["states"][2][:, 96:]
    lhs = (out["xhat"] - K) @ Qh.T
    rhs = e_last @ Qh[:, 96:].T
    assert np.abs(lhs - rhs).max() <= 1e-12 * scale
    # and SQuat's projected error beats plain RTN's on average (Figure 2's claim)
    rtn = O.quantize_keys(K, None, 2, 32, g)
    assert np.mean(lhs ** 2) < np.mean(((rtn["xhat"] - K) @ Qh.T) ** 2)


def test_replay_classifier_accepts_itself_and_flags_a_planted_error():
    Qh, K = _setup(n=32)
    U = O.update_matrix_lowrank(Qh, 1e-3, 32)
    out = O.quantize_keys(K, U, 2, 32, 32)
    rep = O.replay_classify(K, U, 2, 32, 32, out["codes"], out["scale"], out["zero"])
    assert rep["code_diff"] == 0 and rep["meta_diff"] == 0
    bad = out["codes"].copy()
    bad[3, 100] = (bad[3, 100] + 1) % 4          # last block: nothing downstream
    rep = O.replay_classify(K, U, 2, 32, 32, bad, out["scale"], out["zero"])
    assert rep["code_diff"] == 1 and rep["code_unexplained"] == 1
    bad[3, 5] = (bad[3, 5] + 1) % 4              # first block: later codes no longer follow
    rep = O.replay_classify(K, U, 2, 32, 32, bad, out["scale"], out["zero"])
    assert rep["code_unexplained"] >= 2
    # a sign error in the propagation is caught as unexplained disagreements
    wrong = O.quantize_keys(K, -U, 2, 32, 32)
    rep = O.replay_classify(K, U, 2, 32, 32, wrong["codes"], wrong["scale"], wrong["zero"])
    assert rep["code_unexplained"] + rep["meta_unexplained"] > 0


def test_key_scores_are_the_definition():
    """q . deq(code)^T: explicit loops on a small case, one-hot queries read single dequantized
    channels, and all-equal codes give the closed form c * sum(q*scale) + sum(q*zero)."""
    gen = np.random.default_rng(7)
    n, d, G = 5, 128, 32
    codes = gen.integers(0, 4, size=(n, d)).astype(np.uint8)
    scale = gen.uniform(0.1, 2.0, size=(n, d // G)).astype(np.float16)
    zero = gen.standard_normal((n, d // G)).astype(np.float16)
    q = gen.standard_normal((3, d))
    got = O.key_scores(q, codes, scale, zero, G, out_scale=0.25)
    for i in range(3):
        for t in range(n):
            acc = 0.0
            for c in range(d):
                acc += q[i, c] * (float(codes[t, c]) * float(scale[t, c // G]) + float(zero[t, c // G]))
            assert abs(got[i, t] - 0.25 * acc) <= 1e-12 * max(1.0, abs(acc))
    eye = np.eye(d)[[0, 31, 32, 127]]
    back = O.dequantize_keys(codes, scale, zero, G)
    assert np.array_equal(O.key_scores(eye, codes, scale, zero, G), back[:, [0, 31, 32, 127]].T)
    const = np.full((n, d), 3, dtype=np.uint8)
    s64, z64 = scale.astype(np.float64), zero.astype(np.float64)
    qg = q.reshape(3, d // G, G).sum(axis=2)
    want = 3.0 * qg @ s64.T + qg @ z64.T
    assert np.allclose(O.key_scores(q, const, scale, zero, G), want, rtol=1e-12, atol=1e-12)
    # per-channel store: scale/zero indexed by (token group, channel)
    sc = gen.uniform(0.1, 2.0, size=(2, d)).astype(np.float16)
    zc = gen.standard_normal((2, d)).astype(np.float16)
    cc = gen.integers(0, 4, size=(64, d)).astype(np.uint8)
    got = O.key_scores(q, cc, sc, zc, 32, axis="channel")
    t, i = 40, 1
    acc = sum(q[i, c] * (float(cc[t, c]) * float(sc[1, c]) + float(zc[1, c])) for c in range(d))
    assert abs(got[i, t] - acc) <= 1e-12 * max(1.0, abs(acc))


def test_rope_logits_are_rotations_applied_after_dequantization():
    """rope_rotate is a position-dependent rotation of the channel pairs (c, c + 64): it preserves
    norms, composes additively in the position (so logits depend on relative positions only), equals
    explicit 2 x 2 rotations, and at angle zero key_scores_rope is key_scores."""
    gen = np.random.default_rng(11)
    n, d, G = 6, 128, 32
    inv_freq = 10000.0 ** (-np.arange(64) / 64.0)
    x = gen.standard_normal((n, d))
    pos = np.array([0, 1, 7, 100, 4095, 131071])
    y = O.rope_rotate(x, pos, inv_freq)
    assert np.allclose(np.linalg.norm(y, axis=1), np.linalg.norm(x, axis=1), rtol=1e-13)
    assert np.array_equal(y[0], x[0])                                   # position 0: identity
    for t in (2, 4):
        for c in (0, 5, 63):
            ang = pos[t] * inv_freq[c]
            R = np.array([[np.cos(ang), -np.sin(ang)], [np.sin(ang), np.cos(ang)]])
            assert np.allclose(R @ np.array([x[t, c], x[t, c + 64]]), [y[t, c], y[t, c + 64]], rtol=1e-12, atol=1e-12)
    # composition: rotating by p then by m equals rotating by p + m
    z = O.rope_rotate(O.rope_rotate(x, pos, inv_freq), np.full(n, 17), inv_freq)
    assert np.allclose(z, O.rope_rotate(x, pos + 17, inv_freq), rtol=1e-9, atol=1e-9)
    # relative positions: (R_m q) . (R_p k) = q . (R_{p-m} k)
    q = gen.standard_normal((2, d))
    m = 50
    lhs = O.rope_rotate(q, np.full(2, m), inv_freq) @ O.rope_rotate(x, pos + m, inv_freq).T
    assert np.allclose(lhs, q @ O.rope_rotate(x, pos, inv_freq).T, rtol=1e-9, atol=1e-9)
    codes = gen.integers(0, 4, size=(n, d)).astype(np.uint8)
    scale = gen.uniform(0.1, 2.0, size=(n, d // G)).astype(np.float16)
    zero = gen.standard_normal((n, d // G)).astype(np.float16)
    assert np.array_equal(O.key_scores_rope(q, codes, scale, zero, G, np.zeros(64), 9, 0.5),
                          O.key_scores(q, codes, scale, zero, G, 0.5))
    got = O.key_scores_rope(q, codes, scale, zero, G, inv_freq, pos0=3, out_scale=0.5)
    back = O.dequantize_keys(codes, scale, zero, G)
    for t in range(n):
        want = 0.5 * q @ O.rope_rotate(back[t:t + 1], np.array([3 + t]), inv_freq)[0]
        assert np.allclose(got[:, t], want, rtol=1e-12, atol=1e-12)
    # per-channel statistics (one scale / zero-point per channel and 32 tokens): element loops
    cc = gen.integers(0, 16, size=(64, d)).astype(np.uint8)
    sc = gen.uniform(0.1, 2.0, size=(2, d)).astype(np.float16)
    zc = gen.standard_normal((2, d)).astype(np.float16)
    assert np.array_equal(O.key_scores_rope(q, cc, sc, zc, 32, np.zeros(64), 9, 0.5, axis="channel"),
                          O.key_scores(q, cc, sc, zc, 32, 0.5, axis="channel"))
    got = O.key_scores_rope(q, cc, sc, zc, 32, inv_freq, pos0=11, out_scale=2.0, axis="channel")
    for t in (0, 31, 32, 63):
        key = [float(cc[t, c]) * float(sc[t // 32, c]) + float(zc[t // 32, c]) for c in range(d)]
        for i in range(2):
            acc = 0.0
            for c in range(64):
                ang = (11 + t) * inv_freq[c]
                acc += q[i, c] * (key[c] * np.cos(ang) - key[c + 64] * np.sin(ang))
                acc += q[i, c + 64] * (key[c + 64] * np.cos(ang) + key[c] * np.sin(ang))
            assert abs(got[i, t] - 2.0 * acc) <= 1e-11 * max(1.0, abs(acc))


def test_cache_rope_logits_are_the_plain_ones_of_rotated_keys():
    """CacheOracle.scores_rope: with zero frequencies it is `scores`; otherwise column t equals the plain
    logit of the cached key t (dequantized or buffered) rotated by hand to position pos0 + t, and shifting
    pos0 together with the query's position changes nothing (relative positions)."""
    gen = np.random.default_rng(12)
    d, G, R = 128, 32, 8
    inv_freq = 10000.0 ** (-np.arange(64) / 64.0)
    K = gen.standard_normal((21, d))
    q = gen.standard_normal((3, d))
    c = O.CacheOracle(None, 2, G, 128, R)
    c.prefill(K[:13])                                  # 8 quantized, 5 buffered
    for t in range(13, 21):
        c.append(K[t])                                 # ends with 16 quantized, 5 buffered
    assert len(c.k_codes) == 16 and len(c.k_full) == 5
    assert np.array_equal(c.scores_rope(q, np.zeros(64), 7, 0.25), c.scores(q, 0.25))
    got = c.scores_rope(q, inv_freq, pos0=5, out_scale=0.25)
    deq = O.dequantize_keys(np.stack(c.k_codes), np.stack(c.k_scale), np.stack(c.k_zero), G)
    cached = np.concatenate([deq, np.stack(c.k_full)])
    for t in range(21):
        ang = (5 + t) * inv_freq
        a, b = cached[t, :64], cached[t, 64:]
        rot = np.concatenate([a * np.cos(ang) - b * np.sin(ang), b * np.cos(ang) + a * np.sin(ang)])
        assert np.allclose(got[:, t], 0.25 * q @ rot, rtol=1e-12, atol=1e-12)
    qm = O.rope_rotate(q, np.full(3, 40), inv_freq)
    assert np.allclose(c.scores_rope(qm, inv_freq, pos0=40), c.scores_rope(q, inv_freq, pos0=0), rtol=1e-9, atol=1e-9)
    # keys grouped per channel: the same statement with the per-channel dequantization
    K = gen.standard_normal((75, d))
    c = O.CacheOracle(None, 4, G, 128, 32, key_axis="channel")
    c.prefill(K[:40])                                  # 32 quantized, 8 buffered
    for t in range(40, 75):
        c.append(K[t])                                 # ends with 64 quantized, 11 buffered
    assert len(c.k_codes) == 64 and len(c.k_scale) == 2 and len(c.k_full) == 11
    assert np.array_equal(c.scores_rope(q, np.zeros(64), 7, 0.25), c.scores(q, 0.25))
    got = c.scores_rope(q, inv_freq, pos0=5, out_scale=0.25)
    deq = O.dequantize_keys(np.stack(c.k_codes), np.stack(c.k_scale), np.stack(c.k_zero), 32, axis="channel")
    cached = np.concatenate([deq, np.stack(c.k_full)])
    for t in range(75):
        ang = (5 + t) * inv_freq
        a, b = cached[t, :64], cached[t, 64:]
        rot = np.concatenate([a * np.cos(ang) - b * np.sin(ang), b * np.cos(ang) + a * np.sin(ang)])
        assert np.allclose(got[:, t], 0.25 * q @ rot, rtol=1e-12, atol=1e-12)


def test_cache_bookkeeping_follows_algorithm_1():
    """Prefill split r = l mod R, flush every R decoded keys, values lag R tokens behind.  Per-token
    groups make every key independent, so whatever the order of the flushes the quantized store must
    equal one-shot quantization of the same prefix."""
    Qh, K = _setup(n=150)
    gen = np.random.default_rng(31)
    V = gen.standard_normal((150, 128))
    U = O.update_matrix_lowrank(Qh, 1e-3, 32)
    R = 32
    c = O.CacheOracle(U, 2, 32, 32, R, values=True)
    c.prefill(K[:70], V[:70])
    assert len(c.k_codes) == 64 and len(c.k_full) == 6            # 70 = 2 * 32 + 6
    assert len(c.v_codes) == 70 - R and len(c.v_full) == R
    for t in range(70, 150):
        c.append(K[t], V[t])
        n = t + 1
        assert len(c.k_full) == n % R and len(c.k_codes) == n - n % R
        assert len(c.v_codes) == n - R and len(c.v_full) == R
    ref = O.quantize_keys(K[:128], U, 2, 32, 32)
    assert np.array_equal(np.stack(c.k_codes), ref["codes"]) and np.array_equal(np.stack(c.k_scale), ref["scale"])
    assert np.array_equal(np.stack(c.k_full), K[128:150])
    vref = O.rtn_group(V[:118].reshape(118, 4, 32), 2, axis=2)
    assert np.array_equal(np.stack(c.v_codes), vref[0].reshape(118, 128))
    assert np.array_equal(np.stack(c.v_full), V[118:150])
    q = gen.standard_normal((3, 128))
    s = c.scores(q, 0.5)
    assert s.shape == (3, 150)
    assert np.allclose(s[:, 128:], 0.5 * q @ K[128:150].T, rtol=1e-13)
    assert np.allclose(s[:, :128], 0.5 * q @ ref["xhat"].T, rtol=1e-12, atol=1e-12)
    short = O.CacheOracle(U, 2, 32, 32, R, values=True)
    short.prefill(K[:5], V[:5])                                   # shorter than the buffer: nothing quantized
    assert not short.k_codes and len(short.k_full) == 5 and not short.v_codes and len(short.v_full) == 5
    # the grouping Algorithm 1 prints: every flush is one group of 32 tokens quantized per channel, and
    # groups are independent, so the store again equals one-shot quantization of the prefix
    pc = O.CacheOracle(U, 2, 64, 32, R, key_axis="channel")
    pc.prefill(K[:70])
    for t in range(70, 150):
        pc.append(K[t])
    refc = O.quantize_keys(K[:128], U, 2, 32, 32, axis="channel")
    assert np.array_equal(np.stack(pc.k_codes), refc["codes"]) and np.array_equal(np.stack(pc.k_scale), refc["scale"])
    assert np.array_equal(np.stack(pc.k_zero), refc["zero"]) and len(pc.k_scale) == 4
    assert np.array_equal(np.stack(pc.k_full), K[128:150])
    sp = pc.scores(q, 0.5)
    assert np.allclose(sp[:, :128], 0.5 * q @ refc["xhat"].T, rtol=1e-12, atol=1e-12)
    assert np.allclose(sp[:, 128:], 0.5 * q @ K[128:150].T, rtol=1e-13)
    assert not np.array_equal(refc["codes"], ref["codes"])        # the two groupings are different quantizers


# ------------------------------------------- per-channel mode (the paper's own layout)
@pytest.mark.parametrize("bits,g,lam", [(2, 32, 1e-3), (4, 64, 5e-4), (2, 32, np.inf)])
def test_channel_axis_each_step_generic_solver(bits, g, lam):
    """Algorithm 1's `Quant` with statistics per channel over G = 32 tokens: every
    channel of the block is quantized by the scalar quantizer applied to its 32
    current values, and every token's tail is recomputed by a generic
    least-squares solve of Lemma 2's problem."""
    d, G = 128, 32
    Qh, K = _setup(d=d, n=64)
    U = O.update_matrix_lowrank(Qh, lam, g)
    out = O.quantize_keys(K, U, bits, G, g, axis="channel", trace=True)
    Mst = None if np.isinf(lam) else np.vstack([np.eye(d), np.sqrt(lam) * Qh])
    for grp in range(2):
        x = K[grp * G:(grp + 1) * G].copy()
        for t in range(d // g):
            lo, hi = t * g, (t + 1) * g
            xq = np.empty((G, g))
            for j in range(lo, hi):
                c, s, z, xh = O.rtn_group(x[:, j], bits)
                assert np.array_equal(out["codes"][grp * G:(grp + 1) * G, j], c)
                assert out["scale"][grp, j] == s[0] and out["zero"][grp, j] == z[0]
                xq[:, j - lo] = xh
            dvec = xq - x[:, lo:hi]
            x[:, lo:hi] = xq
            if t < d // g - 1:
                for i in range(G):
                    if Mst is not None:
                        tail = np.linalg.lstsq(Mst[:, hi:], -Mst[:, lo:hi] @ dvec[i], rcond=None)[0]
                    else:
                        tail = np.linalg.lstsq(Qh[:, hi:], -Qh[:, lo:hi] @ dvec[i], rcond=None)[0]
                    x[i, hi:] += tail
            assert np.allclose(x, out["states"][t][grp * G:(grp + 1) * G], atol=1e-9)
        assert np.allclose(x, out["xhat"][grp * G:(grp + 1) * G], atol=1e-9)


def test_channel_axis_invariants():
    """The invariants do not depend on which scalar quantizer froze the block: soft
    first-order condition for finite lambda, exact orthogonality for lambda = +inf."""
    Qh, K = _setup(n=96)
    lam, g = 1e-3, 32
    P = np.eye(128) + lam * Qh.T @ Qh
    out = O.quantize_keys(K, O.update_matrix_lemma(Qh, lam, g), 2, 32, g, axis="channel", trace=True)
    for t in range(3):
        delta = out["states"][t] - K
        assert np.abs((delta @ P)[:, (t + 1) * g:]).max() <= 1e-9 * np.abs(delta @ P).max()
    out = O.quantize_keys(K, O.update_matrix_lowrank(Qh, np.inf, g), 2, 32, g, axis="channel", trace=True)
    scale = np.abs(Qh).max() * np.abs(K).max()
    for t in range(3):
        assert np.abs((out["states"][t] - K) @ Qh.T).max() <= 1e-12 * scale
    lhs = (out["xhat"] - K) @ Qh.T
    rtn = O.quantize_keys(K, None, 2, 32, g, axis="channel")
    assert np.mean(lhs ** 2) < np.mean(((rtn["xhat"] - K) @ Qh.T) ** 2)
    # read-back is the definition, element by element
    back = O.dequantize_keys(out["codes"], out["scale"], out["zero"], 32, axis="channel")
    assert np.array_equal(back, out["xhat"])
    for i, c in ((0, 0), (31, 5), (32, 5), (95, 127)):
        assert back[i, c] == float(out["codes"][i, c]) * float(out["scale"][i // 32, c]) + float(out["zero"][i // 32, c])


def test_token_axis_packing_layout_and_roundtrip():
    gen = np.random.default_rng(6)
    for bits in (2, 4):
        codes = gen.integers(0, 1 << bits, size=(3, 96, 128)).astype(np.uint8)
        w = O.pack_codes_tokens(codes, bits)
        assert w.shape == (3, 3, 128, bits) and w.dtype == np.uint32
        assert np.array_equal(O.unpack_codes_tokens(w, bits), codes)
    one = np.zeros((64, 128), dtype=np.uint8)
    one[32 + 17, 9] = 3                      # tile 1, token 17 of the tile, channel 9
    w = O.pack_codes_tokens(one, 2)
    assert w[1, 9, 1] == (3 << 2) and w.sum() == (3 << 2)
    one[32 + 17, 9] = 0
    one[9, 100] = 5                          # tile 0, token 9: 4-bit word 1, nibble 1
    w = O.pack_codes_tokens(one, 4)
    assert w[0, 100, 1] == (5 << 4) and w.sum() == (5 << 4)
    # same share of the 16-bit size as the per-token layout (Tables 1-2's KV size column)
    assert O.pack_codes_tokens(np.zeros((32, 128), np.uint8), 2).nbytes == O.pack_codes(np.zeros((32, 128), np.uint8), 2).nbytes


def test_replay_classifier_channel_axis():
    Qh, K = _setup(n=64)
    U = O.update_matrix_lowrank(Qh, 1e-3, 32)
    out = O.quantize_keys(K, U, 2, 32, 32, axis="channel")
    rep = O.replay_classify(K, U, 2, 32, 32, out["codes"], out["scale"], out["zero"], axis="channel")
    assert rep["code_diff"] == 0 and rep["meta_diff"] == 0 and rep["n_meta"] == 2 * 2 * 128
    bad = out["codes"].copy()
    bad[40, 100] = (bad[40, 100] + 1) % 4
    rep = O.replay_classify(K, U, 2, 32, 32, bad, out["scale"], out["zero"], axis="channel")
    assert rep["code_diff"] == 1 and rep["code_unexplained"] == 1
    # the per-token result is a different quantization: the channel-axis replay must reject it
    tok = O.quantize_keys(K, U, 2, 32, 32)
    rep = O.replay_classify(K, U, 2, 32, 32, tok["codes"], out["scale"], out["zero"], axis="channel")
    assert rep["code_unexplained"] > 0
    badz = out["zero"].copy()
    badz[1, 7] = np.nextafter(np.nextafter(badz[1, 7], np.float16(np.inf)), np.float16(np.inf))
    rep = O.replay_classify(K, U, 2, 32, 32, out["codes"], out["scale"], badz, axis="channel")
    assert rep["meta_unexplained"] >= 1


# ------------------------------------------------------------------ subspace
def test_subspace_matches_library_svd():
    gen = np.random.default_rng(40)
    Q = gen.standard_normal((4, 300, 64)) * np.linspace(3, 0.2, 64)
    A, ea = O.subspace(Q, 10)
    B, eb = O.subspace_svd(Q, 10)
    assert np.allclose(ea, eb, rtol=1e-10)
    assert np.allclose(A, B, atol=1e-7 * np.abs(B).max())


def test_subspace_planted_spectrum():
    """Q = A diag(s) B^T with orthonormal B: Qhat^T Qhat must equal
    B_r diag(s_r^2 * colnorm) B_r^T; with orthonormal A it is B_r diag(s_r^2) B_r^T."""
    gen = np.random.default_rng(41)
    n, d, r = 200, 32, 5
    A, _ = np.linalg.qr(gen.standard_normal((n, d)))
    B, _ = np.linalg.qr(gen.standard_normal((d, d)))
    s = np.linspace(10, 1, d)
    Q = (A * s) @ B.T
    Qh, eig = O.subspace(Q, r)
    assert np.allclose(eig, s[:r] ** 2, rtol=1e-10)
    assert np.allclose(Qh.T @ Qh, (B[:, :r] * s[:r] ** 2) @ B[:, :r].T, atol=1e-9)
    for i in range(r):
        assert np.isclose(abs(Qh[i] @ B[:, i]), s[i], rtol=1e-10)


def test_deviation_eckart_young():
    """Definition 1 summed over the rows equals the tail of the spectrum."""
    gen = np.random.default_rng(42)
    Q = gen.standard_normal((150, 24)) * np.linspace(4, 0.5, 24)
    r = 6
    Qh, _ = O.subspace(Q, r)
    dev = O.deviation_from_subspace(Q, Qh)
    s = np.linalg.svd(Q, compute_uv=False)
    assert np.isclose(np.sum(dev ** 2), np.sum(s[r:] ** 2), rtol=1e-10)


def test_gqa_pooling_is_sum_of_grams():
    gen = np.random.default_rng(43)
    Q = gen.standard_normal((4, 50, 16))
    assert np.allclose(O.gram(Q), sum(Q[h].T @ Q[h] for h in range(4)), atol=1e-10)
    assert np.allclose(O.gram(Q), O.gram([Q[0], Q[1], Q[2], Q[3]]), atol=1e-10)


def test_rank_deficient_queries_give_zero_rows():
    gen = np.random.default_rng(44)
    Q = gen.standard_normal((3, 16))
    Qh, eig = O.subspace(Q, 6)
    assert np.allclose(Qh[3:], 0, atol=1e-6) and np.all(eig[:3] > 0)


# ---------------------------------------------------------------------------
# Block power iteration on the Gram matrix and its refresh (Algorithm 1, remark on the SVD line)
# ---------------------------------------------------------------------------
def _planted_gram(seed, eigs):
    gen = synth.rng(seed)
    B, _ = np.linalg.qr(gen.standard_normal((128, 128)))
    return (B * np.asarray(eigs)) @ B.T, B


def test_gram_update_is_the_gram_of_all_queries_seen():
    gen = synth.rng(5200)
    old, new = gen.standard_normal((2, 300, 128)), gen.standard_normal((2, 17, 128))
    G = O.gram_update(O.gram(old), new)
    both = np.concatenate([old.reshape(-1, 128), new.reshape(-1, 128)])
    assert np.allclose(G, both.T @ both, rtol=1e-12, atol=1e-9)


def test_iteration_start_layout():
    X0 = O.iteration_start(None)
    assert X0.shape == (128, 32)
    assert all(X0[4 * j, j] == 1.0 and np.count_nonzero(X0[:, j]) == 1 for j in range(32))
    gen = synth.rng(5201)
    prev = gen.standard_normal((12, 128)) * 7
    prev[5] = 0.0                                                 # a zero row (r > rank) is dropped
    X0 = O.iteration_start(prev)
    assert np.allclose(X0[:, 0], prev[0] / np.linalg.norm(prev[0])) and np.allclose(X0[:, 5], prev[6] / np.linalg.norm(prev[6]))
    step = 128 // (32 - 11)
    assert all(X0[j * step, 11 + j] == 1.0 and np.count_nonzero(X0[:, 11 + j]) == 1 for j in range(21))


def test_subspace_iteration_fixed_point_and_residual_definition():
    eigs = np.concatenate([np.linspace(900, 300, 32), np.linspace(40, 1, 96)])
    G, B = _planted_gram(5202, eigs)
    Qh, th, resid = O.subspace_iteration(G, B[:, :32], 0, 16)     # exact invariant subspace: Ritz pairs are eigenpairs
    assert np.allclose(th, eigs[:16], rtol=1e-12) and resid.max() <= 1e-13
    for i in range(16):
        v = Qh[i] / np.sqrt(th[i])
        assert abs(abs(v @ B[:, i]) - 1.0) <= 1e-10 and v[np.argmax(np.abs(v))] > 0
    # a rotated basis of the same subspace gives the same result (Rayleigh-Ritz undoes the rotation)
    R, _ = np.linalg.qr(synth.rng(5203).standard_normal((32, 32)))
    Qh2, th2, _ = O.subspace_iteration(G, B[:, :32] @ R, 0, 16)
    assert np.allclose(th2, th, rtol=1e-10) and np.allclose(Qh2.T @ Qh2, Qh.T @ Qh, atol=1e-8 * th[0])
    # the residual is what it says, on a block that is NOT invariant
    X0 = O.iteration_start(None)
    Qh3, th3, resid3 = O.subspace_iteration(G, X0, 1, 8)
    for i in range(8):
        v = Qh3[i] / np.sqrt(th3[i])
        assert np.isclose(np.linalg.norm(G @ v - th3[i] * v) / th3[0], resid3[i], rtol=1e-9)
        assert np.isclose(v @ G @ v, th3[i], rtol=1e-12)          # Ritz value = Rayleigh quotient


def test_subspace_iteration_converges_to_the_library_decomposition_at_the_textbook_rate():
    # lambda_33 / lambda_16 = 0.1: the error of the 16 leading Ritz values shrinks like 0.1^(2 k)
    eigs = np.concatenate([np.linspace(1000, 500, 16), np.linspace(400, 100, 16), np.linspace(50, 1, 96)])
    G, B = _planted_gram(5204, eigs)
    X0 = O.iteration_start(None)
    errs = []
    prev = np.zeros(16)
    for k in range(0, 7):
        Qh, th, resid = O.subspace_iteration(G, X0, k, 16)
        assert np.all(th >= prev - 1e-9 * eigs[0])                # Ritz values grow monotonically towards the eigenvalues
        prev = th
        errs.append(np.abs(th - eigs[:16]).max() / eigs[0])
    assert errs[6] <= 1e-9 and errs[3] <= 1e-3
    assert all(errs[k + 1] <= 0.05 * errs[k] + 1e-13 for k in range(1, 5))
    Qh, th, resid = O.subspace_iteration(G, X0, 12, 16)
    w, V = np.linalg.eigh(G)
    Vr = V[:, ::-1][:, :16]
    assert np.linalg.norm(Qh.T @ Qh - (Vr * w[::-1][:16]) @ Vr.T) <= 1e-9 * w[-1] and resid.max() <= 1e-9
    # and equals `subspace` on actual queries once converged (well-separated planted directions)
    q = synth.queries(5205, 2, 600, planted_rank=12).astype(np.float64)
    ref, ev = O.subspace(q, 8)
    Qh, th, resid = O.subspace_iteration(O.gram(q), O.iteration_start(None), 40, 8)
    assert np.allclose(th, ev, rtol=1e-8) and np.linalg.norm(Qh.T @ Qh - ref.T @ ref) <= 1e-6 * ev[0]


def test_warm_started_refresh_is_worth_several_iterations():
    """The use the refresh is for: the Gram matrix grows by a few new queries and the previous Qhat starts the
    iteration.  Both starts contract at the same rate (lambda_33 / lambda_r per multiplication, squared in
    the Ritz values); the warm start begins more than an order of magnitude closer."""
    q_old = synth.queries(5206, 4, 2048, planted_rank=12).astype(np.float64)
    gen = synth.rng(5207)
    q_new = q_old[:, gen.integers(0, 2048, size=64)] + 0.3 * gen.standard_normal((4, 64, 128))
    r = 8
    prev, _ = O.subspace(q_old, r)
    G = O.gram_update(O.gram(q_old), q_new)
    exact, ev = O.subspace(np.concatenate([q_old, q_new], axis=1), r)
    err = lambda Qh: np.linalg.norm(Qh.T @ Qh - exact.T @ exact) / np.linalg.norm(exact.T @ exact)      # noqa: E731
    ks = (0, 1, 2, 3, 5, 8)
    warm = [err(O.subspace_iteration(G, O.iteration_start(prev), k, r)[0]) for k in ks]
    cold = [err(O.subspace_iteration(G, O.iteration_start(None), k, r)[0]) for k in ks]
    assert all(w <= c / 10 for w, c in zip(warm, cold))
    assert all(b < a for a, b in zip(warm, warm[1:])) and all(b < a for a, b in zip(cold, cold[1:]))
    assert warm[-1] <= 1e-5 and warm[3] <= 3e-3 and cold[3] >= 1e-2
