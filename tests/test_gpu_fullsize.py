"""Parity at the benchmark's full size and launch configuration (the long-context workload of
bench.py: 32 layers x 8 KV heads stacked along the head axis, 32768 tokens per layer), checked on
sampled outputs that the float64 oracle can recompute one by one: whole heads for the Gram matrix,
subspace and update matrix, random (head, token) rows for codes, metadata and dequantized keys."""
import numpy as np
import pytest
import torch

from oracle import squat_oracle as O
from paper_2503_24358_amd import squat
from paper_2503_24358_amd.workload import LongContext

pytestmark = pytest.mark.gpu


def _bf16_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)


def _synthetic_stores(wl, seed):
    """Packed stores of the benchmark's shape filled by a seeded generator (a store is an INPUT of the logits
    calls: any words, scales and zero-points are a valid one): per-token layout and per-channel layout."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    H, n, d, bits = wl.heads, wl.n_tokens, wl.d, wl.bits
    def words(shape):
        return torch.randint(-2 ** 31, 2 ** 31 - 1, shape, dtype=torch.int32, device="cuda", generator=gen)
    def meta(shape):
        sc = (torch.rand(shape, device="cuda", generator=gen) * 1.5 + 0.05).half()
        ze = (torch.randn(shape, device="cuda", generator=gen) * 2.0).half()
        return sc, ze
    tok = (words((1, H, n, d * bits // 32)),) + meta((1, H, n, d // wl.group))
    chan = (words((1, H, n // 32, d, bits)),) + meta((1, H, n // 32, d))
    return tok, chan


@pytest.fixture(scope="module")
def run():
    wl = LongContext()
    H, n, d = wl.heads, wl.n_tokens, wl.d
    qhat, eig, gram = squat.build_subspace(wl.q, wl.q_per_kv, wl.r, want_gram=True)
    update = squat.prepare(qhat, wl.lam, wl.g)
    codes, scale, zero = squat.quantize_keys(wl.k, update, wl.bits, wl.group, wl.g)
    back = squat.dequantize_keys(codes, scale, zero, wl.bits, wl.group, torch.bfloat16)
    torch.cuda.synchronize()
    return dict(wl=wl, qhat=qhat, eig=eig, gram=gram, update=update, codes=codes, scale=scale, zero=zero, back=back)


def test_fullsize_subspace_and_update_on_sampled_heads(run):
    wl = run["wl"]
    for h in (0, 101, 255):
        q = _bf16_to_f64(run["wl"].q[h * wl.q_per_kv:(h + 1) * wl.q_per_kv])
        Gm = O.gram(q)
        gram = run["gram"][h].cpu().numpy().astype(np.float64)
        assert np.linalg.norm(gram - Gm) <= 5e-6 * np.linalg.norm(Gm)
        Qh, ev = O.subspace(q, wl.r)
        eig = run["eig"][h].cpu().numpy().astype(np.float64)
        assert np.allclose(eig, ev, rtol=2e-5)
        qhat = run["qhat"][h].cpu().numpy().astype(np.float64)
        # N(0,1) queries have a nearly flat spectrum (relative gaps ~1e-3): compare the projector-like
        # matrix with a bound scaled by the gap below the r-th eigenvalue, and check the eigen-equation
        full = np.linalg.eigvalsh(Gm)[::-1]
        gap = (full[wl.r - 1] - full[wl.r]) / full[0]
        err = np.linalg.norm(qhat.T @ qhat - Qh.T @ Qh) / np.linalg.norm(Qh.T @ Qh)
        assert err <= 2e-5 / gap, (err, gap)
        for i in range(wl.r):
            v = qhat[i] / np.sqrt(eig[i])
            assert abs(np.linalg.norm(v) - 1.0) <= 1e-5
            assert np.linalg.norm(Gm @ v - eig[i] * v) <= 2e-5 * eig[0]
        # update matrix from the GPU's own Qhat: fp64 result rounded to the fp16 grid
        U = run["update"][h].cpu().numpy().astype(np.float64)
        ref = O.update_matrix_lemma(qhat, wl.lam, wl.g)
        assert np.all(np.abs(U - ref) <= 2.0 ** -11 * np.abs(ref) + 2.0 ** -24)
        assert (U != ref.astype(np.float16).astype(np.float64)).mean() <= 1e-3


def test_fullsize_codes_and_dequantized_keys_on_sampled_rows(run):
    wl = run["wl"]
    gen = np.random.default_rng(9)
    heads = np.concatenate([[0, 255], gen.integers(0, wl.heads, size=22)])
    tot = dict(code_diff=0, code_unexplained=0, meta_diff=0, meta_unexplained=0, n_codes=0, worst_code_dist=0.0)
    free = 0
    for h in heads:
        toks = np.unique(np.concatenate([[0, 31, 32, wl.n_tokens - 1], gen.integers(0, wl.n_tokens, size=252)]))
        idx = torch.from_numpy(toks).cuda()
        k = _bf16_to_f64(run["wl"].k[0, h].index_select(0, idx))
        U = run["update"][h].cpu().numpy().astype(np.float64)
        codes = O.unpack_codes(run["codes"][0, h].index_select(0, idx).cpu().numpy().view(np.uint32), wl.bits)
        scale = run["scale"][0, h].index_select(0, idx).cpu().numpy()
        zero = run["zero"][0, h].index_select(0, idx).cpu().numpy()
        rep = O.replay_classify(k, U, wl.bits, wl.group, wl.g, codes, scale, zero)
        for key in tot:
            tot[key] = max(tot[key], rep[key]) if key.startswith("worst") else tot[key] + rep[key]
        ref = O.quantize_keys(k, U, wl.bits, wl.group, wl.g)
        free += int((ref["codes"] != codes).sum())
        # dequantize read-back: the definition applied to the GPU's own codes, rounded once to bf16
        want = O.dequantize_keys(codes, scale, zero, wl.group)
        got = _bf16_to_f64(run["back"][0, h].index_select(0, idx))
        m, e = np.frexp(want)
        want_bf16 = np.ldexp(np.rint(m * 256.0) / 256.0, e)
        assert (got != want_bf16).mean() <= 1e-4
    assert tot["code_unexplained"] == 0 and tot["meta_unexplained"] == 0, tot
    # root causes (decisions where float64 would have chosen differently given the same history) stay
    # within the 0.01 % budget; the free-running count also contains each root's downstream cascade
    # (a flipped code legitimately changes every later block of that key), bounded loosely
    assert tot["code_diff"] + tot["meta_diff"] <= 1e-4 * tot["n_codes"], tot
    assert free <= 1e-3 * tot["n_codes"], (tot, free)
    assert tot["worst_code_dist"] <= 1e-5


@pytest.mark.parametrize("bits,group", [(4, 32), (2, 128), (4, 128)])
def test_fullsize_other_long_context_variants_on_sampled_rows(run, bits, group):
    """The long-context configuration names 2- and 4-bit codes with statistics groups of 32 and 128 channels:
    the three variants next to the headline one, at the benchmark's size and launch configuration (86
    tiles per wavefront), sampled rows replayed by the oracle; dequantize read-back of the same rows."""
    wl = run["wl"]
    codes_t, scale_t, zero_t = squat.quantize_keys(wl.k, run["update"], bits, group, wl.g)
    back_t = squat.dequantize_keys(codes_t, scale_t, zero_t, bits, group, torch.bfloat16)
    torch.cuda.synchronize()
    plan = squat.quantize_keys_plan(wl.k.dtype, 1, wl.heads, wl.n_tokens, True, 0, bits, group, wl.g)
    assert plan.tiles_per_problem // (plan.workgroups_per_problem * plan.wavefronts_per_workgroup) >= 80
    assert torch.isfinite(scale_t).all() and torch.isfinite(zero_t).all() and (scale_t >= 0).all()
    gen = np.random.default_rng(100 * bits + group)
    heads = np.concatenate([[0, 255], gen.integers(0, wl.heads, size=10)])
    tot = dict(code_diff=0, code_unexplained=0, meta_diff=0, meta_unexplained=0, n_codes=0, worst_code_dist=0.0)
    free = 0
    for h in heads:
        toks = np.unique(np.concatenate([[0, 31, 32, wl.n_tokens - 1], gen.integers(0, wl.n_tokens, size=252)]))
        idx = torch.from_numpy(toks).cuda()
        k = _bf16_to_f64(wl.k[0, h].index_select(0, idx))
        U = run["update"][h].cpu().numpy().astype(np.float64)
        codes = O.unpack_codes(codes_t[0, h].index_select(0, idx).cpu().numpy().view(np.uint32), bits)
        scale = scale_t[0, h].index_select(0, idx).cpu().numpy()
        zero = zero_t[0, h].index_select(0, idx).cpu().numpy()
        rep = O.replay_classify(k, U, bits, group, wl.g, codes, scale, zero)
        for key in tot:
            tot[key] = max(tot[key], rep[key]) if key.startswith("worst") else tot[key] + rep[key]
        free += int((O.quantize_keys(k, U, bits, group, wl.g)["codes"] != codes).sum())
        want = O.dequantize_keys(codes, scale, zero, group)
        got = _bf16_to_f64(back_t[0, h].index_select(0, idx))
        m, e = np.frexp(want)
        assert (got != np.ldexp(np.rint(m * 256.0) / 256.0, e)).mean() <= 1e-4
    assert tot["code_unexplained"] == 0 and tot["meta_unexplained"] == 0, tot
    assert tot["code_diff"] + tot["meta_diff"] <= max(1, 1e-4 * tot["n_codes"]), tot
    assert free <= 1e-3 * tot["n_codes"], (tot, free)
    assert tot["worst_code_dist"] <= 1e-5
    c2, s2, z2 = squat.quantize_keys(wl.k, run["update"], bits, group, wl.g)
    torch.cuda.synchronize()
    assert torch.equal(c2, codes_t) and torch.equal(s2, scale_t) and torch.equal(z2, zero_t)


def test_fullsize_outputs_are_valid_everywhere(run):
    """Properties that hold at any size, over ALL outputs: no NaN/Inf metadata, scales non-negative,
    a bit-identical second run (deterministic), and the hot path leaves its input untouched."""
    wl = run["wl"]
    assert torch.isfinite(run["scale"]).all() and torch.isfinite(run["zero"]).all()
    assert (run["scale"] >= 0).all()
    assert torch.isfinite(run["update"]).all() and torch.isfinite(run["qhat"]).all()
    before = run["wl"].k[0, 7, :64].clone()
    c2, s2, z2 = squat.quantize_keys(wl.k, run["update"], wl.bits, wl.group, wl.g)
    torch.cuda.synchronize()
    assert torch.equal(c2, run["codes"]) and torch.equal(s2, run["scale"]) and torch.equal(z2, run["zero"])
    assert torch.equal(before, run["wl"].k[0, 7, :64])


def test_fullsize_per_channel_mode_on_sampled_token_groups(run):
    """The per-channel grouping at the benchmark's size and launch configuration: whole 32-token groups
    (the unit the oracle can recompute on its own) sampled from sampled heads."""
    wl = run["wl"]
    codes_t, scale_t, zero_t = squat.quantize_keys_per_channel(wl.k, run["update"], wl.bits, 32, wl.g)
    back_t = squat.dequantize_keys_per_channel(codes_t, scale_t, zero_t, wl.bits, 32, torch.bfloat16)
    torch.cuda.synchronize()
    assert torch.isfinite(scale_t).all() and torch.isfinite(zero_t).all() and (scale_t >= 0).all()
    gen = np.random.default_rng(19)
    heads = np.concatenate([[0, 255], gen.integers(0, wl.heads, size=14)])
    n_groups = wl.n_tokens // 32
    tot = dict(code_diff=0, code_unexplained=0, meta_diff=0, meta_unexplained=0, n_codes=0, worst_code_dist=0.0)
    for h in heads:
        groups = np.unique(np.concatenate([[0, n_groups - 1], gen.integers(0, n_groups, size=10)]))
        U = run["update"][h].cpu().numpy().astype(np.float64)
        for gi in groups:
            k = _bf16_to_f64(wl.k[0, h, gi * 32:(gi + 1) * 32])
            codes = O.unpack_codes_tokens(codes_t[0, h, gi:gi + 1].cpu().numpy().view(np.uint32), wl.bits)
            scale = scale_t[0, h, gi:gi + 1].cpu().numpy()
            zero = zero_t[0, h, gi:gi + 1].cpu().numpy()
            rep = O.replay_classify(k, U, wl.bits, 32, wl.g, codes, scale, zero, axis="channel")
            for key in tot:
                tot[key] = max(tot[key], rep[key]) if key.startswith("worst") else tot[key] + rep[key]
            want = O.dequantize_keys(codes, scale, zero, 32, axis="channel")
            got = _bf16_to_f64(back_t[0, h, gi * 32:(gi + 1) * 32])
            m, e = np.frexp(want)
            assert (got != np.ldexp(np.rint(m * 256.0) / 256.0, e)).mean() <= 1e-4
    assert tot["code_unexplained"] == 0 and tot["meta_unexplained"] == 0, tot
    assert tot["code_diff"] + tot["meta_diff"] <= max(1, 1e-4 * tot["n_codes"]), tot
    assert tot["worst_code_dist"] <= 1e-5
    c2, s2, z2 = squat.quantize_keys_per_channel(wl.k, run["update"], wl.bits, 32, wl.g)
    torch.cuda.synchronize()
    assert torch.equal(c2, codes_t) and torch.equal(s2, scale_t) and torch.equal(z2, zero_t)


def test_fullsize_logits_from_both_stores_on_sampled_tokens(run):
    """squat_key_scores and squat_key_scores_per_channel as bench.py launches them (one decode query per
    query head over all 32768 quantized tokens of every head): sampled (query head, token) logits against
    the oracle on the same seeded synthetic stores; every logit finite; second run bit-identical."""
    wl = run["wl"]
    n, d, qpk = wl.n_tokens, wl.d, wl.q_per_kv
    qdec = wl.q[:, n - 1, :].unsqueeze(0).contiguous()
    out_scale = d ** -0.5
    (tc, tsc, tze), (pc, ps, pz) = _synthetic_stores(wl, 2301)
    tok = squat.key_scores(qdec, tc, tsc, tze, wl.bits, wl.group, qpk, out_scale)
    chan = squat.key_scores_per_channel(qdec, pc, ps, pz, wl.bits, qpk, out_scale)
    torch.cuda.synchronize()
    assert tok.shape == chan.shape == (1, wl.heads * qpk, n)
    assert torch.isfinite(tok).all() and torch.isfinite(chan).all()
    gen = np.random.default_rng(23)
    for hq in np.concatenate([[0, wl.heads * qpk - 1], gen.integers(0, wl.heads * qpk, size=10)]):
        h = int(hq) // qpk
        q = _bf16_to_f64(qdec[0, hq])
        # per-token store: sampled tokens, including the first and last of the sequence
        ts = np.unique(np.concatenate([[0, 15, 16, n - 1], gen.integers(0, n, size=40)]))
        codes = O.unpack_codes(tc[0, h, ts].cpu().numpy().view(np.uint32), wl.bits)
        sc, ze = tsc[0, h, ts].cpu().numpy(), tze[0, h, ts].cpu().numpy()
        want = O.key_scores(q[None], codes, sc, ze, wl.group, out_scale)[0]
        bound = out_scale * (np.abs(q)[None] * np.abs(O.dequantize_keys(codes, sc, ze, wl.group))).sum(axis=1)
        got = tok[0, hq, ts].cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - want) <= 4e-5 * bound)
        # per-channel store: whole sampled token groups
        qmax = np.abs(_bf16_to_f64(qdec[0, h * qpk:(h + 1) * qpk])).max()
        for gi in np.unique(np.concatenate([[0, n // 32 - 1], gen.integers(0, n // 32, size=6)])):
            codes = O.unpack_codes_tokens(pc[0, h, gi:gi + 1].cpu().numpy().view(np.uint32), wl.bits)
            sc, ze = ps[0, h, gi:gi + 1].cpu().numpy(), pz[0, h, gi:gi + 1].cpu().numpy()
            want = O.key_scores(q[None], codes, sc, ze, 32, out_scale, axis="channel")[0]
            khat = np.abs(O.dequantize_keys(codes, sc, ze, 32, axis="channel"))
            bound = out_scale * (np.abs(q)[None] * khat).sum(axis=1)
            floor = out_scale * 128 * (2 ** wl.bits - 1) * 2.0 ** -24 * qmax * float(sc.astype(np.float64).max())
            got = chan[0, hq, gi * 32:(gi + 1) * 32].cpu().numpy().astype(np.float64)
            assert np.all(np.abs(got - want) <= 4e-5 * bound + floor)
    tok2 = squat.key_scores(qdec, tc, tsc, tze, wl.bits, wl.group, qpk, out_scale)
    chan2 = squat.key_scores_per_channel(qdec, pc, ps, pz, wl.bits, qpk, out_scale)
    torch.cuda.synchronize()
    assert torch.equal(tok, tok2) and torch.equal(chan, chan2)


def test_fullsize_pre_rope_logits_from_both_stores_on_sampled_tokens(run):
    """squat_key_scores_rope and squat_key_scores_rope_per_channel at the same launch shape: the stores read
    as pre-RoPE keys, token t rotated to position pos0 + t; sampled logits against the oracle on the same seeded
    synthetic stores (the key is dequantized and rotated in packed fp16: worst case 4 * 2^-11 * sum over rotary pairs
    of (|q_c| + |q_{c+64}|) * norm of the pair, see test_gpu_scores_rope.py; bound 2.0e-3 of that sum), every logit
    finite, second run bit-identical."""
    wl = run["wl"]
    n, d, qpk = wl.n_tokens, wl.d, wl.q_per_kv
    qdec = wl.q[:, n - 1, :].unsqueeze(0).contiguous()
    out_scale, pos0 = d ** -0.5, 98304
    inv32 = (10000.0 ** (-np.arange(64) / 64.0)).astype(np.float32)
    inv = torch.from_numpy(inv32).cuda()
    inv64 = inv32.astype(np.float64)
    (tc, tsc, tze), (pc, ps, pz) = _synthetic_stores(wl, 2901)
    tok = squat.key_scores_rope(qdec, tc, tsc, tze, wl.bits, wl.group, qpk, inv, pos0, out_scale)
    chan = squat.key_scores_rope_per_channel(qdec, pc, ps, pz, wl.bits, qpk, inv, pos0, out_scale)
    torch.cuda.synchronize()
    assert tok.shape == chan.shape == (1, wl.heads * qpk, n)
    assert torch.isfinite(tok).all() and torch.isfinite(chan).all()
    gen = np.random.default_rng(29)
    for hq in np.concatenate([[0, wl.heads * qpk - 1], gen.integers(0, wl.heads * qpk, size=10)]):
        h = int(hq) // qpk
        q = _bf16_to_f64(qdec[0, hq])
        ts = np.unique(np.concatenate([[0, 15, 16, n - 1], gen.integers(0, n, size=40)]))
        codes = O.unpack_codes(tc[0, h, ts].cpu().numpy().view(np.uint32), wl.bits)
        sc, ze = tsc[0, h, ts].cpu().numpy(), tze[0, h, ts].cpu().numpy()
        khat = O.dequantize_keys(codes, sc, ze, wl.group)
        rot = O.rope_rotate(khat, pos0 + ts, inv64)
        got = tok[0, hq, ts].cpu().numpy().astype(np.float64)
        qq = np.abs(q[:64]) + np.abs(q[64:])
        assert np.all(np.abs(got - out_scale * rot @ q) <= 2.0e-3 * out_scale * (np.sqrt(khat[:, :64] ** 2 + khat[:, 64:] ** 2) @ qq))
        assert np.median(np.abs(got - out_scale * rot @ q) / (out_scale * (np.abs(rot) @ np.abs(q)))) <= 1.5e-4
        for gi in np.unique(np.concatenate([[0, n // 32 - 1], gen.integers(0, n // 32, size=6)])):
            codes = O.unpack_codes_tokens(pc[0, h, gi:gi + 1].cpu().numpy().view(np.uint32), wl.bits)
            sc, ze = ps[0, h, gi:gi + 1].cpu().numpy(), pz[0, h, gi:gi + 1].cpu().numpy()
            want = O.key_scores_rope(q[None], codes, sc, ze, 32, inv64, pos0 + 32 * int(gi), out_scale, axis="channel")[0]
            khat = O.dequantize_keys(codes, sc, ze, 32, axis="channel")
            got = chan[0, hq, gi * 32:(gi + 1) * 32].cpu().numpy().astype(np.float64)
            assert np.all(np.abs(got - want) <= 2.0e-3 * out_scale * (np.sqrt(khat[:, :64] ** 2 + khat[:, 64:] ** 2) @ qq))
    tok2 = squat.key_scores_rope(qdec, tc, tsc, tze, wl.bits, wl.group, qpk, inv, pos0, out_scale)
    chan2 = squat.key_scores_rope_per_channel(qdec, pc, ps, pz, wl.bits, qpk, inv, pos0, out_scale)
    torch.cuda.synchronize()
    assert torch.equal(tok, tok2) and torch.equal(chan, chan2)
