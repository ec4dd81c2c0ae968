"""GPU parity of squat_key_scores_rope and squat_key_scores_rope_per_channel (logits against keys stored BEFORE the
rotary embedding: the key is dequantized, rotated to its position, and only then contracted with the query) against
the float64 oracle.

Accuracy of the kernels, and hence the bound of these tests: the queries enter as exact fp16 high/low pairs rotated in
fp32, the angles are good to ~1e-5 rad; the key is dequantized and rotated in packed fp16, where the dequantized value,
the cos/sin table entry, one product and the result are each rounded to fp16 (unit roundoff u = 2^-11).  For a rotary
pair (a, b) of norm rho = sqrt(a^2 + b^2) each rotated member is off by at most u (2 |a cos| + 3 |b sin| + |x'|) <=
4 u rho, so a logit is off by at most 4 u sum_{c < 64} (|q_c| + |q_{c+64}|) rho_c: the tests allow 2.0e-3 of that sum
(4 u = 1.95e-3).  The roundings do not line up: the observed worst case is several times smaller, and every test also
checks that the typical (median) error stays below 1.5e-4 of sum_c |q_c| |k_rot_c|."""
import numpy as np
import pytest
import torch

from oracle import squat_oracle as O
from paper_2503_24358_amd import squat, synth
from tests import util

pytestmark = pytest.mark.gpu

INV_FREQ = (10000.0 ** (-np.arange(64) / 64.0)).astype(np.float32)


def _store(seed, B, H, n, bits, G):
    gen = synth.rng(seed)
    x = synth.keys(seed + 1, H, n, batch=B)
    codes = np.empty((B, H, n, 128), dtype=np.uint8)
    scale = np.empty((B, H, n, 128 // G), dtype=np.float16)
    zero = np.empty_like(scale)
    for b in range(B):
        for h in range(H):
            out = O.quantize_keys(x[b, h].astype(np.float64), None, bits, G, 128)
            codes[b, h], scale[b, h], zero[b, h] = out["codes"], out["scale"], out["zero"]
    return gen, codes, scale, zero


def _dev(codes, scale, zero, bits):
    words = O.pack_codes(codes, bits)
    return (torch.from_numpy(words.view(np.int32)).cuda(), torch.from_numpy(scale).cuda(), torch.from_numpy(zero).cuda())


def _assert_logits(got, want, q, khat, rot, out_scale, where):
    """got / want: logits of one query head over the tokens of khat (dequantized, unrotated keys), rot the rotated keys."""
    rho = np.sqrt(khat[:, :64] ** 2 + khat[:, 64:] ** 2)
    qq = np.abs(q[:64]) + np.abs(q[64:])
    bound = abs(out_scale) * (rho @ qq)
    err = np.abs(got - want)
    assert np.all(err <= 2.0e-3 * bound + 1e-30), (where, float((err / (bound + 1e-30)).max()))
    typical = abs(out_scale) * (np.abs(rot) @ np.abs(q))
    if len(err) >= 64:
        assert np.median(err / (typical + 1e-30)) <= 1.5e-4, (where, float(np.median(err / (typical + 1e-30))))
    return float((err / (bound + 1e-30)).max())


def _check(qval, codes, scale, zero, G, qpk, inv_freq, pos0, out_scale, got):
    B, Hq = qval.shape[:2]
    got = got.cpu().numpy().astype(np.float64)
    worst = 0.0
    for b in range(B):
        for hq in range(Hq):
            h = hq // qpk
            want = O.key_scores_rope(qval[b, hq][None], codes[b, h], scale[b, h], zero[b, h], G, inv_freq, pos0, out_scale)[0]
            khat = O.dequantize_keys(codes[b, h], scale[b, h], zero[b, h], G)
            rot = O.rope_rotate(khat, pos0 + np.arange(khat.shape[0]), inv_freq)
            worst = max(worst, _assert_logits(got[b, hq], want, qval[b, hq], khat, rot, out_scale, (b, hq)))
    return worst


@pytest.mark.parametrize("bits,G", [(2, 32), (4, 32), (2, 64), (4, 128), (2, 128)])
@pytest.mark.parametrize("qdt", [synth.BF16, synth.F16, synth.F32])
def test_rope_scores_match_definition(bits, G, qdt):
    B, H, n, qpk = 2, 3, 1000, 4          # 62 full units and a ragged one of 8 tokens
    gen, codes, scale, zero = _store(5100 + bits + G, B, H, n, bits, G)
    q32 = (gen.standard_normal((B, H * qpk, 128)) * 3).astype(np.float32)
    qraw, qval = synth.store(q32, qdt)
    ct, st, zt = _dev(codes, scale, zero, bits)
    got = squat.key_scores_rope(util.to_device(qraw, qdt), ct, st, zt, bits, G, qpk, torch.from_numpy(INV_FREQ).cuda(),
                                pos0=0, out_scale=128 ** -0.5)
    torch.cuda.synchronize()
    assert got.shape == (B, H * qpk, n)
    _check(qval, codes, scale, zero, G, qpk, INV_FREQ, 0, 128 ** -0.5, got)


@pytest.mark.parametrize("pos0", [1, 4097, 131000, 2 ** 33 + 5])
def test_rope_scores_at_large_positions_and_long_ranges(pos0):
    """Angles of many thousands of radians (range reduction in fp64) and wavefront ranges of the maximum
    length (the query side's cos / sin recurrence runs 16 epochs of 64 tokens before it is re-seeded)."""
    B, H, n, qpk = 1, 2, 16 * 250, 2      # 250 units: one workgroup, 64 units per wavefront, the last one 58
    gen, codes, scale, zero = _store(5200, B, H, n, 2, 32)
    q32 = gen.standard_normal((B, H * qpk, 128)).astype(np.float32)
    qraw, qval = synth.store(q32, synth.BF16)
    ct, st, zt = _dev(codes, scale, zero, 2)
    got = squat.key_scores_rope(util.to_device(qraw, synth.BF16), ct, st, zt, 2, 32, qpk, torch.from_numpy(INV_FREQ).cuda(), pos0=pos0)
    torch.cuda.synchronize()
    _check(qval, codes, scale, zero, 32, qpk, INV_FREQ, pos0, 1.0, got)


def test_rope_scores_reduce_to_plain_scores_and_respect_relative_positions():
    B, H, n, qpk = 1, 2, 200, 4
    gen, codes, scale, zero = _store(5300, B, H, n, 2, 32)
    q32 = gen.standard_normal((B, H * qpk, 128)).astype(np.float32)
    qraw, qval = synth.store(q32, synth.F32)
    ct, st, zt = _dev(codes, scale, zero, 2)
    qt = util.to_device(qraw, synth.F32)
    zero_freq = torch.zeros(64, dtype=torch.float32, device="cuda")
    plain = squat.key_scores(qt, ct, st, zt, 2, 32, qpk).cpu().numpy().astype(np.float64)
    flat = squat.key_scores_rope(qt, ct, st, zt, 2, 32, qpk, zero_freq, pos0=77).cpu().numpy().astype(np.float64)
    _check(qval, codes, scale, zero, 32, qpk, np.zeros(64), 77, 1.0, torch.from_numpy(flat))
    assert np.abs(flat - plain).max() <= 6e-4 * np.abs(plain).max() + 1e-6
    # shifting the keys' positions by m and rotating the query by m leaves the logits unchanged
    m = 333
    inv = torch.from_numpy(INV_FREQ).cuda()
    base = squat.key_scores_rope(qt, ct, st, zt, 2, 32, qpk, inv, pos0=10).cpu().numpy().astype(np.float64)
    qrot = O.rope_rotate(qval.reshape(-1, 128), np.full(H * qpk, m), INV_FREQ).reshape(qval.shape).astype(np.float32)
    moved = squat.key_scores_rope(torch.from_numpy(qrot).cuda(), ct, st, zt, 2, 32, qpk, inv, pos0=10 + m)
    moved = moved.cpu().numpy().astype(np.float64)
    scale_ref = np.abs(base).max()
    assert np.abs(moved - base).max() <= 2e-3 * scale_ref


@pytest.mark.parametrize("bits,G", [(2, 32), (4, 32), (2, 64), (4, 128), (2, 128)])
@pytest.mark.parametrize("n", [333, 120])
def test_rope_scores_unaligned_rows_and_odd_ends(bits, G, n):
    """The two ways out of the kernel's loop over pairs of whole units.  n = 333: an odd number of tokens per
    (batch, head) puts the metadata rows of every second head off a 16-byte boundary, so every unit of the launch
    is fetched lane by lane (eight units per wavefront: the query-side operand changes inside that loop).
    n = 120: rows are aligned; the second wavefront is left with one pair, a single whole unit and a ragged unit."""
    B, H, qpk = 2, 3, 4
    gen, codes, scale, zero = _store(5250 + bits + G + n, B, H, n, bits, G)
    q32 = (gen.standard_normal((B, H * qpk, 128)) * 2).astype(np.float32)
    qraw, qval = synth.store(q32, synth.BF16)
    ct, st, zt = _dev(codes, scale, zero, bits)
    got = squat.key_scores_rope(util.to_device(qraw, synth.BF16), ct, st, zt, bits, G, qpk,
                                torch.from_numpy(INV_FREQ).cuda(), pos0=77, out_scale=0.5)
    torch.cuda.synchronize()
    _check(qval, codes, scale, zero, G, qpk, INV_FREQ, 77, 0.5, got)


def test_rope_scores_with_scales_beyond_the_packed_range():
    """The packed dequantization multiplies the fp16 scale by 2^9, which must stay an fp16 number: units in which
    some token has a scale above 127 take the fp32 dequantization instead (wave-uniform choice).  Stores with huge
    ranges in some tokens (scales up to ~3e3) next to ordinary ones, so that both forms run in one launch; the
    largest values whose rotated keys still fit fp16 (scale 2e4, zero-point -3e4) as well."""
    B, H, n, qpk = 1, 2, 16 * 37 + 5, 4
    gen, codes, scale, zero = _store(5350, B, H, n, 2, 32)
    big = gen.random((B, H, n)) < 0.07
    scale32 = scale.astype(np.float32)
    zero32 = zero.astype(np.float32)
    scale32[big] *= gen.uniform(100.0, 1500.0, size=(int(big.sum()), 1)).astype(np.float32)
    zero32[big] *= 300.0
    scale32[0, 0, 3] = [2.0e4, 127.0, 127.5, 128.0]
    zero32[0, 0, 3] = [-3.0e4, 0.0, 100.0, -100.0]
    scale, zero = scale32.astype(np.float16), zero32.astype(np.float16)
    assert np.isfinite(scale.astype(np.float64)).all() and np.isfinite(zero.astype(np.float64)).all()
    q32 = gen.standard_normal((B, H * qpk, 128)).astype(np.float32)
    qraw, qval = synth.store(q32, synth.BF16)
    ct, st, zt = _dev(codes, scale, zero, 2)
    for pos0 in (0, 50001):
        got = squat.key_scores_rope(util.to_device(qraw, synth.BF16), ct, st, zt, 2, 32, qpk,
                                    torch.from_numpy(INV_FREQ).cuda(), pos0=pos0, out_scale=0.25)
        torch.cuda.synchronize()
        assert torch.isfinite(got).all()
        _check(qval, codes, scale, zero, 32, qpk, INV_FREQ, pos0, 0.25, got)


def test_rope_scores_query_heads_strides_and_tiny_inputs():
    for qpk, n in ((1, 1), (3, 17), (8, 130)):
        B, H = 2, 2
        gen, codes, scale, zero = _store(5400 + n, B, H, n, 4, 64)
        q32 = gen.standard_normal((B, H * qpk, 128)).astype(np.float32)
        qraw, qval = synth.store(q32, synth.F16)
        ct, st, zt = _dev(codes, scale, zero, 4)
        big = torch.full((B, H * qpk, n + 24), -7.0, dtype=torch.float32, device="cuda")
        squat.key_scores_rope(util.to_device(qraw, synth.F16), ct, st, zt, 4, 64, qpk, torch.from_numpy(INV_FREQ).cuda(),
                              pos0=5, out_scale=0.3, out=big)
        torch.cuda.synchronize()
        _check(qval, codes, scale, zero, 64, qpk, INV_FREQ, 5, 0.3, big[..., :n])
        assert torch.all(big[..., n:] == -7.0)


# ---------------------------------------------------------------- per-channel store

def _store_pc(seed, B, H, n, bits):
    gen = synth.rng(seed)
    x = synth.keys(seed + 1, H, n, batch=B)
    codes = np.empty((B, H, n, 128), dtype=np.uint8)
    scale = np.empty((B, H, n // 32, 128), dtype=np.float16)
    zero = np.empty_like(scale)
    for b in range(B):
        for h in range(H):
            out = O.quantize_keys(x[b, h].astype(np.float64), None, bits, 32, 128, axis="channel")
            codes[b, h], scale[b, h], zero[b, h] = out["codes"], out["scale"], out["zero"]
    return gen, codes, scale, zero


def _dev_pc(codes, scale, zero, bits):
    words = O.pack_codes_tokens(codes, bits)
    return (torch.from_numpy(words.view(np.int32)).cuda(), torch.from_numpy(scale).cuda(), torch.from_numpy(zero).cuda())


def _check_pc(qval, codes, scale, zero, qpk, inv_freq, pos0, out_scale, got):
    B, Hq = qval.shape[:2]
    got = got.cpu().numpy().astype(np.float64)
    for b in range(B):
        for hq in range(Hq):
            h = hq // qpk
            want = O.key_scores_rope(qval[b, hq][None], codes[b, h], scale[b, h], zero[b, h], 32, inv_freq, pos0,
                                     out_scale, axis="channel")[0]
            khat = O.dequantize_keys(codes[b, h], scale[b, h], zero[b, h], 32, axis="channel")
            rot = O.rope_rotate(khat, pos0 + np.arange(khat.shape[0]), inv_freq)
            _assert_logits(got[b, hq], want, qval[b, hq], khat, rot, out_scale, (b, hq))


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("qdt", [synth.BF16, synth.F16, synth.F32])
def test_rope_scores_per_channel_match_definition(bits, qdt):
    B, H, n, qpk = 2, 3, 32 * 101, 4      # 101 token groups: two workgroups, 13 groups per wavefront, the last 10
    gen, codes, scale, zero = _store_pc(5500 + bits, B, H, n, bits)
    q32 = (gen.standard_normal((B, H * qpk, 128)) * 3).astype(np.float32)
    qraw, qval = synth.store(q32, qdt)
    ct, st, zt = _dev_pc(codes, scale, zero, bits)
    got = squat.key_scores_rope_per_channel(util.to_device(qraw, qdt), ct, st, zt, bits, qpk,
                                            torch.from_numpy(INV_FREQ).cuda(), pos0=0, out_scale=128 ** -0.5)
    torch.cuda.synchronize()
    assert got.shape == (B, H * qpk, n)
    _check_pc(qval, codes, scale, zero, qpk, INV_FREQ, 0, 128 ** -0.5, got)


@pytest.mark.parametrize("pos0,bits", [(1, 2), (131000, 4), (2 ** 33 + 5, 2)])
def test_rope_scores_per_channel_at_large_positions_and_long_ranges(pos0, bits):
    B, H, n, qpk = 1, 2, 32 * 90, 2       # 90 groups: up to 23 per wavefront (46 steps of the recurrence)
    gen, codes, scale, zero = _store_pc(5600 + bits, B, H, n, bits)
    q32 = gen.standard_normal((B, H * qpk, 128)).astype(np.float32)
    qraw, qval = synth.store(q32, synth.BF16)
    ct, st, zt = _dev_pc(codes, scale, zero, bits)
    got = squat.key_scores_rope_per_channel(util.to_device(qraw, synth.BF16), ct, st, zt, bits, qpk,
                                            torch.from_numpy(INV_FREQ).cuda(), pos0=pos0)
    torch.cuda.synchronize()
    _check_pc(qval, codes, scale, zero, qpk, INV_FREQ, pos0, 1.0, got)


def test_rope_scores_per_channel_reduce_to_plain_scores_heads_and_strides():
    for qpk, n in ((1, 32), (3, 64), (8, 160)):
        B, H = 2, 2
        gen, codes, scale, zero = _store_pc(5700 + n, B, H, n, 4)
        q32 = gen.standard_normal((B, H * qpk, 128)).astype(np.float32)
        qraw, qval = synth.store(q32, synth.F16)
        ct, st, zt = _dev_pc(codes, scale, zero, 4)
        qt = util.to_device(qraw, synth.F16)
        big = torch.full((B, H * qpk, n + 24), -7.0, dtype=torch.float32, device="cuda")
        squat.key_scores_rope_per_channel(qt, ct, st, zt, 4, qpk, torch.from_numpy(INV_FREQ).cuda(), pos0=5,
                                          out_scale=0.3, out=big)
        torch.cuda.synchronize()
        _check_pc(qval, codes, scale, zero, qpk, INV_FREQ, 5, 0.3, big[..., :n])
        assert torch.all(big[..., n:] == -7.0)
        # zero frequencies: the unrotated per-channel logits
        plain = squat.key_scores_per_channel(qt, ct, st, zt, 4, qpk).cpu().numpy().astype(np.float64)
        flat = squat.key_scores_rope_per_channel(qt, ct, st, zt, 4, qpk, torch.zeros(64, device="cuda"), pos0=77)
        assert np.abs(flat.cpu().numpy() - plain).max() <= 6e-4 * np.abs(plain).max() + 1e-6
    empty = squat.key_scores_rope_per_channel(qt, ct[:, :, :0], st[:, :, :0], zt[:, :, :0], 4, qpk,
                                              torch.from_numpy(INV_FREQ).cuda())
    assert empty.shape == (B, H * qpk, 0)
