"""squat_prepare_noalloc (the entry point for callers that cannot allocate: static scratch inside the
library) against squat_prepare, through the raw C ABI: same kernels, so the update matrices must agree bit
for bit (and squat_prepare itself is held to the oracle by test_gpu_parity.py); a spot check against the
float64 oracle (Lemma 2's panel in its rank-r form) guards against both being wrong together.  Calls are made
back to back on one stream, the later ones with smaller inputs, so stale scratch contents of an earlier call
would show."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import squat_oracle as O
from paper_2503_24358_amd import squat, synth

pytestmark = pytest.mark.gpu


def _both(Qh: np.ndarray, lam: float, g: int):
    """-> (update by squat_prepare, update by squat_prepare_noalloc), both via ctypes on the current stream."""
    L = squat.lib()
    H, r, d = Qh.shape
    qt = torch.from_numpy(Qh).cuda()
    want = torch.full((H, d, d), 7.0, dtype=torch.float32, device="cuda")
    got = torch.full((H, d, d), -7.0, dtype=torch.float32, device="cuda")
    nbytes = int(L.squat_prepare_workspace(H, d, r, g))
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    qp = ctypes.c_void_p(qt.data_ptr()) if r else None
    rc = L.squat_prepare(qp, H, d, r, ctypes.c_float(lam), g, ctypes.c_void_p(want.data_ptr()),
                         ctypes.c_void_p(ws.data_ptr()), ws.numel(), stream)
    assert rc == 0, squat.strerror(rc)
    rc = L.squat_prepare_noalloc(qp, H, d, r, ctypes.c_float(lam), g, ctypes.c_void_p(got.data_ptr()), stream)
    assert rc == 0, squat.strerror(rc)
    return want, got


def _qhat(seed, H, r):
    gen = synth.rng(seed)
    return (gen.standard_normal((H, r, 128)) * (np.linspace(60, 5, r)[None, :, None] if r else 1.0)).astype(np.float32)


def test_noalloc_matches_prepare_on_consecutive_calls_of_shrinking_size():
    calls = [(_qhat(9100, 24, 32), 1e-3, 32),         # Cholesky route: one flag per head in the scratch
             (_qhat(9101, 7, 16), 1e-3, 32),          # smaller, same route: flags 7..23 are stale
             (_qhat(9102, 5, 40), 5e-4, 64),          # r > 32: intermediate products in the scratch
             (_qhat(9103, 3, 34), 1e-3, 32),          # smaller again
             (_qhat(9104, 2, 16), float("inf"), 32),  # hard constraint: no scratch at all
             (_qhat(9105, 4, 8), 1e-3, 64)]
    pairs = [_both(*c) for c in calls]                # all enqueued before the first comparison
    torch.cuda.synchronize()
    for (Qh, lam, g), (want, got) in zip(calls, pairs):
        assert torch.equal(want, got), (Qh.shape, lam, g)
        U = got.cpu().numpy().astype(np.float64)
        for h in (0, Qh.shape[0] - 1):
            ref = O.update_matrix_lowrank(Qh[h].astype(np.float64), lam, g)
            assert np.linalg.norm(U[h] - ref) <= 3e-4 * max(np.linalg.norm(ref), 1e-30) + 1e-12


def test_noalloc_flagged_heads_take_the_fallback_route_through_the_static_flags():
    """A head whose Cholesky pivots span too much is flagged (in the scratch) and redone by the eigen route;
    the call before it left other flags behind."""
    H, r, g, lam = 4, 20, 32, 50.0
    gen = synth.rng(1450)
    Qh = gen.standard_normal((H, r, 128)).astype(np.float32)
    Qh[0] *= 3e4
    Qh[1] *= 3e4
    Qh[1, 8:] = 0.0
    Qh[2, 8:] = 0.0
    Qh[3] *= 1e-3
    first = _both(Qh, lam, g)
    second = _both(Qh[::-1].copy(), lam, g)           # the flagged head moves from slot 1 to slot 2
    third = _both(Qh[2:].copy(), lam, g)              # fewer heads, none flagged
    torch.cuda.synchronize()
    for want, got in (first, second, third):
        assert torch.equal(want, got)
    U = second[1].cpu().numpy().astype(np.float64)
    for h in range(H):
        ref = O.update_matrix_lowrank(Qh[::-1][h].astype(np.float64), lam, g)
        assert np.linalg.norm(U[h] - ref) <= 3e-4 * max(np.linalg.norm(ref), 1e-30) + 1e-12


def test_noalloc_rejects_problems_beyond_its_scratch_and_bad_arguments():
    L = squat.lib()
    fake = ctypes.c_void_p(0x1000)
    stream = torch.cuda.current_stream().cuda_stream
    call = lambda **kw: L.squat_prepare_noalloc(  # noqa: E731
        kw.get("q", fake), kw.get("h", 8), kw.get("d", 128), kw.get("r", 16), ctypes.c_float(kw.get("lam", 1e-3)),
        kw.get("g", 32), kw.get("u", fake), stream)
    # r = 64, g = 32: 3 panels x 64 x 160 x 8 bytes = 240 KiB per head; 18 heads exceed 4 MiB
    assert call(h=18, r=64) == -5
    assert call(h=(1 << 20) + 1, r=16) == -5          # more flags than the scratch holds
    assert call(d=64) == -2
    assert call(g=48) == -2
    assert call(lam=-1.0) == -7
    assert call(u=None) == -1
    assert call(q=None) == -1
    assert call(h=0) == 0
    # and the largest r > 32 problem that fits runs (17 heads) and matches
    want, got = _both(_qhat(9200, 17, 64), 1e-3, 32)
    torch.cuda.synchronize()
    assert torch.equal(want, got)
