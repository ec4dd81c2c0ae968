"""GPU parity of squat_refresh_subspace (block power iteration on the running Gram matrix + Rayleigh-Ritz;
Algorithm 1's remark on its SVD line) against the oracle's `gram_update`, `iteration_start` and
`subspace_iteration` on the same Gram matrices, start blocks and iteration counts.

What is unique, and therefore compared: the running Gram matrix; the Ritz values; the matrix
Qhat^T Qhat = sum_i theta_i x_i x_i^T of the r leading Ritz pairs (signs and the basis inside a cluster of Ritz
values are free; the tolerance scales with the gap below the r-th Ritz value); the residual the call reports.
After enough iterations on a well-separated spectrum the result must also agree with the exact route."""
import numpy as np
import pytest
import torch

from oracle import squat_oracle as O
from paper_2503_24358_amd import squat, synth
from tests import util

pytestmark = pytest.mark.gpu


def _planted_grams(seed, heads, eigs):
    gen = synth.rng(seed)
    out = []
    for _ in range(heads):
        B, _ = np.linalg.qr(gen.standard_normal((128, 128)))
        G = (B * np.asarray(eigs)) @ B.T
        out.append(0.5 * (G + G.T))
    return np.stack(out)


def _compare(G, prev, k, r, qhat, eig, resid, tol=1e-5):
    """One head: GPU output against the oracle's iteration from the same start."""
    ref_q, ref_th, ref_res = O.subspace_iteration(G, O.iteration_start(prev), k, r)
    top = ref_th[0]
    assert np.all(np.abs(eig - ref_th) <= 2e-6 * top), np.abs(eig - ref_th).max() / top
    assert np.all(np.diff(eig) <= 0)
    # gap below the r-th Ritz value (in the full 32-wide block) decides how well the r-dimensional sum is defined
    _, th_all, _ = O.subspace_iteration(G, O.iteration_start(prev), k, 32)
    gap = (th_all[r - 1] - th_all[r]) / top if r < 32 else 1.0
    err = np.linalg.norm(qhat.T @ qhat - ref_q.T @ ref_q) / np.linalg.norm(ref_q.T @ ref_q)
    assert err <= tol / max(gap, 1e-3), (err, gap)
    assert abs(resid - ref_res.max()) <= 1e-5 + 1e-3 * ref_res.max(), (resid, ref_res.max())
    for i in range(r):
        if eig[i] > 1e-6 * top:
            v = qhat[i] / np.sqrt(eig[i])
            assert abs(np.linalg.norm(v) - 1.0) <= 1e-5
            assert v[np.argmax(np.abs(v))] > 0


@pytest.mark.parametrize("r,iterations,warm", [(16, 0, False), (16, 1, False), (16, 3, False), (8, 5, False), (32, 2, False),
                                               (16, 0, True), (16, 2, True), (8, 1, True), (32, 1, True), (1, 4, False)])
def test_iteration_matches_oracle_from_the_same_start(r, iterations, warm):
    eigs = np.concatenate([np.geomspace(5e4, 4e3, 16), np.geomspace(2.5e3, 6e2, 16), np.linspace(200, 1, 96)])
    H = 5
    G = _planted_grams(8100 + r, H, eigs)
    prev = None
    if warm:
        # a previous Qhat that is close to, but not, the present leading subspace
        gen = synth.rng(8200 + r)
        prev = np.stack([O.subspace_iteration(G[h] + 30.0 * _sym(gen.standard_normal((128, 128))), O.iteration_start(None), 30, r)[0]
                         for h in range(H)]).astype(np.float32)
    state = torch.from_numpy(G).cuda()
    before = state.clone()
    qhat_t, eig_t, res_t = squat.refresh_subspace(state, 1, r, iterations,
                                                  qhat_prev=None if prev is None else torch.from_numpy(prev).cuda())
    torch.cuda.synchronize()
    assert torch.equal(state, before)                      # no new queries: the state is left alone
    qhat, eig, res = (t.cpu().numpy().astype(np.float64) for t in (qhat_t, eig_t, res_t))
    for h in range(H):
        _compare(G[h], None if prev is None else prev[h].astype(np.float64), iterations, r, qhat[h], eig[h], res[h])


def _sym(a):
    return 0.5 * (a + a.T)


@pytest.mark.parametrize("dtype,hq,qpk", [(synth.BF16, 8, 4), (synth.F32, 2, 1), (synth.F16, 4, 2)])
def test_running_gram_state_and_exact_mode(dtype, hq, qpk):
    """accumulate = 0 builds the state from the prompt's queries, accumulate = 1 adds later ones: the state equals
    the Gram matrix of everything seen; iterations < 0 runs the exact solver on it (the same kernels as
    squat_build_subspace: identical output for identical queries)."""
    n_old, n_new, r = 1000, 77, 8
    q32 = synth.queries(8300, hq, n_old + n_new, planted_rank=12)
    raw, val = synth.store(q32, dtype)
    qt = util.to_device(raw, dtype)
    H = hq // qpk
    state = torch.full((H, 128, 128), 123.0, dtype=torch.float64, device="cuda")
    q1, e1, r1 = squat.refresh_subspace(state, qpk, r, -1, q_new=qt[:, :n_old], accumulate=False)
    qb, eb, _ = squat.build_subspace(qt[:, :n_old].contiguous(), qpk, r)
    torch.cuda.synchronize()
    assert torch.equal(q1, qb) and torch.equal(e1, eb) and not r1.any()
    s1 = state.cpu().numpy()
    for j in range(H):
        Gm = O.gram(val[j * qpk:(j + 1) * qpk, :n_old])
        assert np.linalg.norm(s1[j] - Gm) <= 2e-6 * np.linalg.norm(Gm) and np.array_equal(s1[j], s1[j].T)
    q2, e2, _ = squat.refresh_subspace(state, qpk, r, -1, q_new=qt[:, n_old:], accumulate=True)
    torch.cuda.synchronize()
    s2 = state.cpu().numpy()
    q2, e2 = q2.cpu().numpy().astype(np.float64), e2.cpu().numpy().astype(np.float64)
    for j in range(H):
        Gm = O.gram_update(O.gram(val[j * qpk:(j + 1) * qpk, :n_old]), val[j * qpk:(j + 1) * qpk, n_old:])
        assert np.linalg.norm(s2[j] - Gm) <= 2e-6 * np.linalg.norm(Gm)
        ref, ev = O.subspace(val[j * qpk:(j + 1) * qpk], r)
        assert np.allclose(e2[j], ev, rtol=1e-5)
        assert np.linalg.norm(q2[j].T @ q2[j] - ref.T @ ref) <= 1e-4 * np.linalg.norm(ref.T @ ref)


def test_warm_refresh_after_new_queries_converges_to_the_exact_route():
    """The decode-time use: the prompt's Qhat starts the iteration on the grown Gram matrix.  Each step matches
    the oracle's; with enough of them (well-separated planted directions) the result agrees with the exact
    solver's on the same state."""
    hq, qpk, n_old, n_new, r = 8, 4, 2048, 64, 8
    H = hq // qpk
    q32 = synth.queries(8400, hq, n_old + n_new, planted_rank=12)
    raw, val = synth.store(q32, synth.BF16)
    qt = util.to_device(raw, synth.BF16)
    state = torch.zeros((H, 128, 128), dtype=torch.float64, device="cuda")
    prev, _, _ = squat.refresh_subspace(state, qpk, r, -1, q_new=qt[:, :n_old], accumulate=False)
    squat.refresh_subspace(state, qpk, 0, 0, q_new=qt[:, n_old:], accumulate=True)        # r = 0: only the state moves
    exact, ev, _ = squat.refresh_subspace(state, qpk, r, -1)
    torch.cuda.synchronize()
    G = state.cpu().numpy()
    prev_h = prev.cpu().numpy().astype(np.float64)
    errs = []
    for k in (0, 2, 12, 40):
        qk, ek, rk = squat.refresh_subspace(state, qpk, r, k, qhat_prev=prev)
        torch.cuda.synchronize()
        qk, ek, rk = (t.cpu().numpy().astype(np.float64) for t in (qk, ek, rk))
        for h in range(H):
            _compare(G[h], prev_h[h], k, r, qk[h], ek[h], rk[h])
        ex = exact.cpu().numpy().astype(np.float64)
        errs.append(max(np.linalg.norm(qk[h].T @ qk[h] - ex[h].T @ ex[h]) / np.linalg.norm(ex[h].T @ ex[h]) for h in range(H)))
    assert errs[3] <= 1e-5 and errs[2] <= 1e-3 and errs[1] < errs[0], errs
    # in place: qhat_prev and qhat may be one buffer
    buf = prev.clone()
    squat.refresh_subspace(state, qpk, r, 2, qhat_prev=buf, qhat=buf)
    q2, _, _ = squat.refresh_subspace(state, qpk, r, 2, qhat_prev=prev)
    torch.cuda.synchronize()
    assert torch.equal(buf, q2)


def test_rank_deficient_state_falls_back_to_the_exact_solver():
    """20 queries span 20 directions: the 32-wide block cannot be orthonormalised, the head is flagged and the
    exact solver takes it (residual reported as 0); a healthy head in the same launch keeps the iteration."""
    gen = synth.rng(8500)
    q = np.zeros((2, 300, 128), dtype=np.float32)
    q[0, :20] = gen.standard_normal((20, 128))
    q[1] = synth.queries(8501, 1, 300, planted_rank=12)[0]
    qt = torch.from_numpy(q).cuda()
    state = torch.zeros((2, 128, 128), dtype=torch.float64, device="cuda")
    qhat, eig, res = squat.refresh_subspace(state, 1, 16, 6, q_new=qt, accumulate=False)
    torch.cuda.synchronize()
    qhat, eig, res = (t.cpu().numpy().astype(np.float64) for t in (qhat, eig, res))
    ref, ev = O.subspace(q[0].astype(np.float64), 16)
    assert res[0] == 0.0 and np.allclose(eig[0], ev, rtol=1e-5, atol=1e-5 * ev[0])
    assert np.linalg.norm(qhat[0].T @ qhat[0] - ref.T @ ref) <= 1e-4 * np.linalg.norm(ref.T @ ref)
    G1 = state[1].cpu().numpy()
    _compare(G1, None, 6, 16, qhat[1], eig[1], res[1])
    assert res[1] > 0.0


def test_refresh_is_deterministic():
    hq, qpk, r = 8, 4, 16
    raw, _ = synth.store(synth.queries(8600, hq, 512, planted_rank=12), synth.BF16)
    qt = util.to_device(raw, synth.BF16)
    H = hq // qpk
    state = torch.zeros((H, 128, 128), dtype=torch.float64, device="cuda")
    a = squat.refresh_subspace(state, qpk, r, 3, q_new=qt, accumulate=False)
    s_a = state.clone()
    b = squat.refresh_subspace(state, qpk, r, 3, q_new=qt, accumulate=False)
    torch.cuda.synchronize()
    assert torch.equal(state, s_a)
    for x, y in zip(a, b):
        assert torch.equal(x, y)
