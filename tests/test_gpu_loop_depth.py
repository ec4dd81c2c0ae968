"""GPU parity at LOOP DEPTH: every instantiation of the two quantize kernels (bits x statistics group x
propagation block x key dtype; shared and per-batch update matrices; one and several workgroups per update
matrix) is taken through at least three tiles per wavefront, so that the persistent loop's back-edge, the
register prefetch of the next tile and the reuse of the LDS staging tile are exercised for all of them,
and compared with the float64 oracle (Algorithm 1 `Quant` + Lemma 2) code by code.

The launch shape comes from the library itself (`squat_quantize_keys_plan`, the same function the launcher
uses), and every test asserts the tiles per wavefront it achieved: a shape cannot silently fall back to one
tile per wavefront.

To keep the oracle's share small the launch is filled with COPIES of a few distinct problems (keys and
update matrices repeated along the head or batch axis): the oracle replays every key of the distinct
problems, and all copies must be bit-identical to them, which covers every workgroup of the launch.
"""
import numpy as np
import pytest
import torch

from oracle import squat_oracle as O
from paper_2503_24358_amd import squat, synth
from tests import util

pytestmark = pytest.mark.gpu

MISMATCH_BUDGET = 1e-4      # 0.01 % of codes
_TORCH_DT = {synth.BF16: torch.bfloat16, synth.F16: torch.float16, synth.F32: torch.float32}
_cache = {}


def _distinct_keys(seed, batch, heads, n, dtype):
    key = ("k", seed, batch, heads, n, dtype)
    if key not in _cache:
        raw, val = synth.store(synth.keys(seed, heads, n, batch=batch), dtype)
        _cache[key] = (util.to_device(raw, dtype), val)
    return _cache[key]


def _distinct_updates(seed, count, r, lam, g):
    key = ("u", seed, count, r, lam, g)
    if key not in _cache:
        gen = synth.rng(seed)
        Qh = gen.standard_normal((count, r, 128)) * 25.0
        U = np.stack([O.update_matrix_lowrank(Qh[i], lam, g) for i in range(count)]).astype(np.float32)
        # every other matrix on the fp16 grid, as squat_prepare may write it: the kernels then skip the
        # products with the low parts of the panels, so one launch runs both forms of the contraction
        U[1::2] = U[1::2].astype(np.float16).astype(np.float32)
        _cache[key] = U
    return _cache[key]


def _tiles_per_wavefront(plan):
    stride = plan.workgroups_per_problem * plan.wavefronts_per_workgroup
    return plan.tiles_per_problem // stride, -(-plan.tiles_per_problem // stride)


def _replay(kval, U, bits, G, g, codes, scale, zero, axis):
    """Oracle comparison of every (batch, head) problem of kval [B, H, n, 128]; U [H, ...] or [B, H, ...]."""
    tot = dict(code_diff=0, code_unexplained=0, meta_diff=0, meta_unexplained=0, n_codes=0)
    free = 0
    B, H = kval.shape[:2]
    for b in range(B):
        for h in range(H):
            Uh = None if U is None else (U[b, h] if U.ndim == 4 else U[h]).astype(np.float64)
            kw = {} if axis == "token" else {"axis": "channel"}
            ref = O.quantize_keys(kval[b, h], Uh, bits, G, g, **kw)
            free += int((ref["codes"] != codes[b, h]).sum())
            rep = O.replay_classify(kval[b, h], Uh, bits, G, g, codes[b, h], scale[b, h], zero[b, h], **kw)
            for k in tot:
                tot[k] += rep[k]
    assert tot["code_unexplained"] == 0 and tot["meta_unexplained"] == 0, tot
    assert tot["code_diff"] + tot["meta_diff"] <= max(2, MISMATCH_BUDGET * tot["n_codes"]), tot
    # free-running differences = the roots above plus their legitimate cascades: a flipped code changes the
    # later blocks of its key; with per-channel statistics a flipped scale or zero-point changes the later
    # blocks of all 32 tokens of its group
    if axis == "token":
        assert free <= max(64, 10 * MISMATCH_BUDGET * tot["n_codes"]), (free, tot)
    else:
        assert free <= max(2000, 30 * MISMATCH_BUDGET * tot["n_codes"]), (free, tot)
    return tot


def _run_token(kt, kval, U, bits, G, g, reps_axis, reps, min_tiles):
    """kt/kval: the distinct problems [B, H, n, 128]; the launch repeats them `reps` times along `reps_axis`
    (0 = batch, 1 = head); U: float32 [H, 128, 128] shared by the batch, [B, H, 128, 128] per batch entry, or
    None."""
    B, H, n, _ = kt.shape
    rep_shape = [1, 1, 1, 1]
    rep_shape[reps_axis] = reps
    k_all = kt.repeat(*rep_shape)
    Ut, usb = None, 0
    if U is not None:
        Ut = torch.from_numpy(U).cuda()
        if U.ndim == 4:
            Ut = Ut.repeat(reps if reps_axis == 0 else 1, reps if reps_axis == 1 else 1, 1, 1).contiguous()
            usb = Ut.stride(0)
        elif reps_axis == 1:
            Ut = Ut.repeat(reps, 1, 1).contiguous()
    plan = squat.quantize_keys_plan(k_all.dtype, k_all.shape[0], k_all.shape[1], n, U is not None, usb, bits, G, g)
    lo, hi = _tiles_per_wavefront(plan)
    assert lo >= min_tiles, (lo, hi, plan.problems, plan.workgroups_per_problem, plan.wavefronts_per_workgroup)
    codes_t, scale_t, zero_t = squat.quantize_keys(k_all, Ut, bits, G, g)
    torch.cuda.synchronize()
    # every copy equals the distinct problem it repeats, bit for bit
    for t in (codes_t, scale_t, zero_t):
        first = t[:B, :H]
        assert torch.equal(t, first.repeat(*rep_shape)), "copies of one problem differ inside a launch"
    codes = O.unpack_codes(util.codes_to_host(codes_t[:B, :H].contiguous()), bits)
    scale = util.half_to_host(scale_t[:B, :H].contiguous())
    zero = util.half_to_host(zero_t[:B, :H].contiguous())
    _replay(kval, U, bits, G, g, codes, scale, zero, "token")
    return plan, (lo, hi)


def _run_channel(kt, kval, U, bits, g, reps_axis, reps, min_tiles):
    B, H, n, _ = kt.shape
    rep_shape = [1, 1, 1, 1]
    rep_shape[reps_axis] = reps
    k_all = kt.repeat(*rep_shape)
    Ut, usb = None, 0
    if U is not None:
        Ut = torch.from_numpy(U).cuda()
        if U.ndim == 4:
            Ut = Ut.repeat(reps if reps_axis == 0 else 1, reps if reps_axis == 1 else 1, 1, 1).contiguous()
            usb = Ut.stride(0)
        elif reps_axis == 1:
            Ut = Ut.repeat(reps, 1, 1).contiguous()
    plan = squat.quantize_keys_plan(k_all.dtype, k_all.shape[0], k_all.shape[1], n, U is not None, usb, bits, 32, g,
                                    per_channel=True)
    lo, hi = _tiles_per_wavefront(plan)
    assert lo >= min_tiles, (lo, hi, plan.problems, plan.workgroups_per_problem, plan.wavefronts_per_workgroup)
    codes_t, scale_t, zero_t = squat.quantize_keys_per_channel(k_all, Ut, bits, 32, g)
    torch.cuda.synchronize()
    rep5 = rep_shape + [1]
    assert torch.equal(codes_t, codes_t[:B, :H].repeat(*rep5)), "copies of one problem differ inside a launch"
    assert torch.equal(scale_t, scale_t[:B, :H].repeat(*rep_shape))
    assert torch.equal(zero_t, zero_t[:B, :H].repeat(*rep_shape))
    codes = O.unpack_codes_tokens(util.codes_to_host(codes_t[:B, :H].contiguous()), bits)
    scale = util.half_to_host(scale_t[:B, :H].contiguous())
    zero = util.half_to_host(zero_t[:B, :H].contiguous())
    _replay(kval, U, bits, 32, g, codes, scale, zero, "channel")
    return plan, (lo, hi)


# One workgroup per update matrix (256 heads on 256 compute units): 38 tiles over the 12, 8 or 6 wavefronts
# of the workgroup.  All 54 instantiations of the per-token kernel: bits x G x g x dtype (g = 128 is the
# single-block instantiation that update = NULL also runs).
@pytest.mark.parametrize("dtype", [synth.BF16, synth.F16, synth.F32])
@pytest.mark.parametrize("g", [32, 64, 128])
@pytest.mark.parametrize("G", [32, 64, 128])
@pytest.mark.parametrize("bits", [2, 4])
def test_per_token_every_instantiation_at_loop_depth(bits, G, g, dtype):
    P, n = 8, 37 * 32 + 7                       # 37 full tiles and a ragged one
    kt, kval = _distinct_keys(7100, 1, P, n, dtype)
    U = _distinct_updates(7200 + g, P, 16, 1e-3, g)
    plan, (lo, hi) = _run_token(kt, kval, U, bits, G, g, reps_axis=1, reps=32, min_tiles=3)
    assert plan.problems == 256 and plan.workgroups_per_problem == 1 and plan.tiles_per_problem == 38


@pytest.mark.parametrize("bits,G", [(2, 32), (4, 128), (2, 64)])
def test_per_token_no_update_matrix_at_loop_depth(bits, G):
    P, n = 8, 37 * 32 + 7
    kt, kval = _distinct_keys(7100, 1, P, n, synth.BF16)
    _run_token(kt, kval, None, bits, G, 32, reps_axis=1, reps=32, min_tiles=3)


# Several workgroups per update matrix, the matrix shared by a batch: a wavefront's tiles then belong to
# different batch entries (the tile -> (batch entry, token) division is exercised inside the loop).
@pytest.mark.parametrize("bits,G,g,dtype", [(2, 32, 32, synth.BF16), (4, 128, 32, synth.BF16), (2, 128, 32, synth.BF16),
                                            (4, 32, 64, synth.F16), (2, 64, 32, synth.F32)])
def test_per_token_shared_update_many_workgroups_at_loop_depth(bits, G, g, dtype):
    Bd, H, n = 2, 4, 36 * 32 + 7
    kt, kval = _distinct_keys(7300, Bd, H, n, dtype)
    U = _distinct_updates(7400 + g, H, 16, 1e-3, g)
    plan, (lo, hi) = _run_token(kt, kval, U, bits, G, g, reps_axis=0, reps=32, min_tiles=3)
    assert plan.problems == H and plan.workgroups_per_problem == 64


# One update matrix per (batch entry, head): the per-batch stride of the update argument inside the loop.
@pytest.mark.parametrize("bits,G,g,dtype", [(2, 32, 32, synth.BF16), (4, 64, 64, synth.F16), (4, 32, 32, synth.F32)])
def test_per_token_per_batch_update_at_loop_depth(bits, G, g, dtype):
    Bd, H, n = 2, 8, 37 * 32 + 7
    kt, kval = _distinct_keys(7500, Bd, H, n, dtype)
    U = _distinct_updates(7600 + g, Bd * H, 16, 1e-3, g).reshape(Bd, H, 128, 128)
    plan, _ = _run_token(kt, kval, U, bits, G, g, reps_axis=0, reps=16, min_tiles=3)
    assert plan.problems == 256 and plan.workgroups_per_problem == 1


# ------------------------------------------------------------------ per-channel grouping
@pytest.mark.parametrize("dtype", [synth.BF16, synth.F16, synth.F32])
@pytest.mark.parametrize("g", [32, 64, 128])
@pytest.mark.parametrize("bits", [2, 4])
def test_per_channel_every_instantiation_at_loop_depth(bits, g, dtype):
    P, n = 8, 38 * 32
    kt, kval = _distinct_keys(7700, 1, P, n, dtype)
    U = _distinct_updates(7200 + g, P, 16, 1e-3, g)
    plan, _ = _run_channel(kt, kval, U, bits, g, reps_axis=1, reps=32, min_tiles=3)
    assert plan.problems == 256 and plan.workgroups_per_problem == 1 and plan.tiles_per_problem == 38


def test_per_channel_no_update_matrix_at_loop_depth():
    kt, kval = _distinct_keys(7700, 1, 8, 38 * 32, synth.BF16)
    _run_channel(kt, kval, None, 2, 32, reps_axis=1, reps=32, min_tiles=3)


@pytest.mark.parametrize("bits,g,dtype", [(2, 32, synth.BF16), (4, 64, synth.F16), (2, 32, synth.F32)])
def test_per_channel_shared_update_many_workgroups_at_loop_depth(bits, g, dtype):
    Bd, H, n = 2, 4, 37 * 32
    kt, kval = _distinct_keys(7800, Bd, H, n, dtype)
    U = _distinct_updates(7400 + g, H, 16, 1e-3, g)
    plan, _ = _run_channel(kt, kval, U, bits, g, reps_axis=0, reps=32, min_tiles=3)
    assert plan.problems == H and plan.workgroups_per_problem == 64


@pytest.mark.parametrize("bits,g,dtype", [(2, 32, synth.BF16), (4, 32, synth.F32)])
def test_per_channel_per_batch_update_at_loop_depth(bits, g, dtype):
    Bd, H, n = 2, 8, 38 * 32
    kt, kval = _distinct_keys(7900, Bd, H, n, dtype)
    U = _distinct_updates(7600 + g, Bd * H, 16, 1e-3, g).reshape(Bd, H, 128, 128)
    plan, _ = _run_channel(kt, kval, U, bits, g, reps_axis=0, reps=16, min_tiles=3)
    assert plan.problems == 256 and plan.workgroups_per_problem == 1
