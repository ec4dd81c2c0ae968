"""GPU parity of squat_key_scores_per_channel (attention logits straight from the per-channel packed
key store) against the float64 oracle: out_scale * q . deq(code)^T with the scale and zero-point of
(token group, channel).  Each q_c * Delta_c reaches the matrix cores as an fp16 high/low pair (relative
error < 2^-21, absolute floor 2^-25 of max|q| * max Delta of the token group; the test allows twice that), products with the codes
are exact, sums are fp32 over ~130 terms in two partly cancelling parts: the same 4e-5 * sum_c |q_c|
|deq_c| bound as for the per-token store, plus that floor (only visible when one channel's scale
dwarfs the others), 25 times inside the 1e-3 relative tolerance the build states for projections."""
import numpy as np
import pytest
import torch

from oracle import squat_oracle as O
from paper_2503_24358_amd import squat, synth
from tests import util

pytestmark = pytest.mark.gpu


def _store(seed, B, H, n, bits, heavy=False, key_gain=None):
    """A per-channel packed store produced by the oracle's quantizer (plain round-to-nearest is enough
    here: the scores call only reads the format)."""
    gen = synth.rng(seed)
    x = synth.keys(seed + 1, H, n, heavy_tail=heavy, batch=B)
    if key_gain is not None:
        x = x * np.asarray(key_gain, dtype=np.float32).reshape(1, H, 1, 1)
    codes = np.empty((B, H, n, 128), dtype=np.uint8)
    scale = np.empty((B, H, n // 32, 128), dtype=np.float16)
    zero = np.empty_like(scale)
    for b in range(B):
        for h in range(H):
            out = O.quantize_keys(x[b, h].astype(np.float64), None, bits, 32, 128, axis="channel")
            codes[b, h], scale[b, h], zero[b, h] = out["codes"], out["scale"], out["zero"]
    return gen, codes, scale, zero


def _dev(codes, scale, zero, bits):
    words = O.pack_codes_tokens(codes, bits)
    return (torch.from_numpy(words.view(np.int32)).cuda(), torch.from_numpy(scale).cuda(), torch.from_numpy(zero).cuda())


def _check(qval, codes, scale, zero, qpk, out_scale, got, bits=2):
    B, Hq = qval.shape[:2]
    got = got.cpu().numpy().astype(np.float64)
    worst = 0.0
    for b in range(B):
        for hq in range(Hq):
            h = hq // qpk
            want = O.key_scores(qval[b, hq][None], codes[b, h], scale[b, h], zero[b, h], 32, out_scale, axis="channel")[0]
            khat = np.abs(O.dequantize_keys(codes[b, h], scale[b, h], zero[b, h], 32, axis="channel"))
            bound = abs(out_scale) * (np.abs(qval[b, hq])[None] * khat).sum(axis=1)
            qmax = np.abs(qval[b, h * qpk:(h + 1) * qpk]).max()
            dmax = np.repeat(scale[b, h].astype(np.float64).max(axis=1), 32)          # per token group
            floor = abs(out_scale) * 128 * (2 ** bits - 1) * 2.0 ** -24 * qmax * dmax
            err = np.abs(got[b, hq] - want)
            assert np.all(err <= 4e-5 * bound + floor + 1e-30), (b, hq, float((err / (bound + 1e-30)).max()))
            worst = max(worst, float((err / (bound + 1e-30)).max()))
    return worst


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("qdt", [synth.BF16, synth.F16, synth.F32])
def test_scores_match_definition(bits, qdt):
    B, H, n, qpk = 2, 3, 992, 4           # 31 token groups: uneven shares for the four wavefronts
    gen, codes, scale, zero = _store(4100 + bits, B, H, n, bits)
    q32 = (gen.standard_normal((B, H * qpk, 128)) * 3).astype(np.float32)
    qraw, qval = synth.store(q32, qdt)
    ct, st, zt = _dev(codes, scale, zero, bits)
    got = squat.key_scores_per_channel(util.to_device(qraw, qdt), ct, st, zt, bits, qpk, out_scale=128 ** -0.5)
    torch.cuda.synchronize()
    assert got.shape == (B, H * qpk, n)
    _check(qval, codes, scale, zero, qpk, 128 ** -0.5, got, bits)


@pytest.mark.parametrize("qpk", [1, 2, 3, 8])
def test_scores_query_heads_per_kv_head(qpk):
    B, H, n = 1, 2, 160
    gen, codes, scale, zero = _store(4200 + qpk, B, H, n, 2, heavy=True)
    q32 = gen.standard_normal((B, H * qpk, 128)).astype(np.float32)
    qraw, qval = synth.store(q32, synth.BF16)
    ct, st, zt = _dev(codes, scale, zero, 2)
    got = squat.key_scores_per_channel(util.to_device(qraw, synth.BF16), ct, st, zt, 2, qpk)
    torch.cuda.synchronize()
    _check(qval, codes, scale, zero, qpk, 1.0, got)


def test_scores_long_sequence_several_workgroups():
    B, H, n, qpk = 1, 2, 32 * 150, 4      # 150 token groups: more than one workgroup per head
    gen, codes, scale, zero = _store(4250, B, H, n, 2)
    q32 = gen.standard_normal((B, H * qpk, 128)).astype(np.float32)
    qraw, qval = synth.store(q32, synth.BF16)
    ct, st, zt = _dev(codes, scale, zero, 2)
    got = squat.key_scores_per_channel(util.to_device(qraw, synth.BF16), ct, st, zt, 2, qpk, out_scale=0.5)
    torch.cuda.synchronize()
    _check(qval, codes, scale, zero, qpk, 0.5, got)


def test_scores_strided_output_single_group_and_empty_inputs():
    B, H, qpk = 2, 2, 4
    for bits, n in ((2, 32), (4, 32), (2, 96)):
        gen, codes, scale, zero = _store(4300 + n + bits, B, H, n, bits)
        q32 = gen.standard_normal((B, H * qpk, 128)).astype(np.float32)
        qraw, qval = synth.store(q32, synth.F16)
        ct, st, zt = _dev(codes, scale, zero, bits)
        big = torch.full((B, H * qpk, n + 40), -7.0, dtype=torch.float32, device="cuda")   # room for residual logits
        squat.key_scores_per_channel(util.to_device(qraw, synth.F16), ct, st, zt, bits, qpk, out=big)
        torch.cuda.synchronize()
        _check(qval, codes, scale, zero, qpk, 1.0, big[..., :n], bits)
        assert torch.all(big[..., n:] == -7.0)
    e = squat.key_scores_per_channel(torch.zeros((B, H * qpk, 128), dtype=torch.bfloat16, device="cuda"),
                                     ct[:, :, :0].contiguous(), st[:, :, :0].contiguous(), zt[:, :, :0].contiguous(), 2, qpk)
    assert e.shape == (B, H * qpk, 0)


def test_scores_special_queries_and_constant_channels():
    """One-hot queries read single dequantized channels; a constant channel (scale 0) contributes
    zero * q; a zero query gives exact zeros."""
    B, H, n, qpk = 1, 1, 64, 4
    gen, codes, scale, zero = _store(4400, B, H, n, 2)
    scale[0, 0, 1, 37] = 0
    codes[0, 0, 32:64, 37] = 0
    q = np.zeros((B, H * qpk, 128), dtype=np.float32)
    q[0, 0, 0] = 1.0
    q[0, 1, 37] = -2.0
    q[0, 2, 127] = 0.5
    qraw, qval = synth.store(q, synth.F32)
    ct, st, zt = _dev(codes, scale, zero, 2)
    got = squat.key_scores_per_channel(util.to_device(qraw, synth.F32), ct, st, zt, 2, qpk).cpu().numpy().astype(np.float64)
    back = O.dequantize_keys(codes[0, 0], scale[0, 0], zero[0, 0], 32, axis="channel")
    assert np.allclose(got[0, 0], back[:, 0], rtol=1e-6, atol=0)
    assert np.allclose(got[0, 1], -2.0 * back[:, 37], rtol=1e-6, atol=0)
    assert np.array_equal(got[0, 1, 32:64], (-2.0 * zero[0, 0, 1, 37].astype(np.float64)) * np.ones(32))
    assert np.allclose(got[0, 2], 0.5 * back[:, 127], rtol=1e-6, atol=0)
    assert not got[0, 3].any()


def test_scores_do_not_depend_on_the_magnitude_of_queries_or_keys():
    """Power-of-two normalisation inside the kernel: keys of size 1e-4 or 1e3, queries of size 1e-3 or
    1e3 meet the same relative bound."""
    B, H, n, qpk = 1, 4, 128, 2
    gen, codes, scale, zero = _store(4500, B, H, n, 2, key_gain=[1e-4, 1.0, 1e3, 3e-6])
    q32 = gen.standard_normal((B, H * qpk, 128)).astype(np.float32)
    q32[0, 0:2] *= 1e3
    q32[0, 2:4] *= 1e-3
    q32[0, 4:6] *= 7e-5
    qraw, qval = synth.store(q32, synth.F32)
    ct, st, zt = _dev(codes, scale, zero, 2)
    got = squat.key_scores_per_channel(util.to_device(qraw, synth.F32), ct, st, zt, 2, qpk)
    torch.cuda.synchronize()
    _check(qval, codes, scale, zero, qpk, 1.0, got)


def test_scores_on_the_quantize_kernels_own_output():
    """End to end on the GPU: per-channel quantize with an update matrix, then logits from the store,
    against the oracle applied to the GPU's own codes and metadata."""
    B, H, n, qpk = 2, 4, 640, 4
    x32 = synth.keys(4600, H, n, batch=B, heavy_tail=True)
    kraw, kval = synth.store(x32, synth.BF16)
    gen = synth.rng(4601)
    Qh = gen.standard_normal((H, 16, 128)) * 25
    U = np.stack([O.update_matrix_lowrank(Qh[h], 1e-3, 32) for h in range(H)]).astype(np.float32)
    ct, st, zt = squat.quantize_keys_per_channel(util.to_device(kraw, synth.BF16), torch.from_numpy(U).cuda(), 2, 32, 32)
    q32 = gen.standard_normal((B, H * qpk, 128)).astype(np.float32)
    qraw, qval = synth.store(q32, synth.BF16)
    got = squat.key_scores_per_channel(util.to_device(qraw, synth.BF16), ct, st, zt, 2, qpk, out_scale=0.1)
    torch.cuda.synchronize()
    codes = O.unpack_codes_tokens(util.codes_to_host(ct), 2)
    _check(qval, codes, util.half_to_host(st), util.half_to_host(zt), qpk, 0.1, got)
    exact = np.einsum("bqc,bqtc->bqt", qval, np.repeat(kval, qpk, axis=1)) * 0.1
    g = got.cpu().numpy().astype(np.float64)
    assert np.linalg.norm(g - exact) <= 0.8 * np.linalg.norm(exact)
