"""The library under HIP graph capture: every call only enqueues kernels on the caller's stream (no allocation,
no synchronisation, no memset node), so a captured sequence of calls must replay to the same bits as the eager
calls, every time, with other work on the device between the replays."""
import pytest
import torch

from paper_2503_24358_amd import squat, synth
from tests import util

pytestmark = pytest.mark.gpu


def _inputs(seed, hq, qpk, n):
    q32 = synth.queries(seed, hq, n, planted_rank=12)
    qraw, _ = synth.store(q32, synth.BF16)
    k32 = synth.keys(seed + 1, hq // qpk, n)
    kraw, _ = synth.store(k32, synth.BF16)
    return util.to_device(qraw, synth.BF16), util.to_device(kraw, synth.BF16).unsqueeze(0)


def test_whole_path_and_logits_replay_from_a_graph():
    hq, qpk, n, r, d = 8, 4, 2080, 16, 128
    H = hq // qpk
    qt, kt = _inputs(4100, hq, qpk, n)
    dev = qt.device
    qhat = torch.empty((H, r, d), dtype=torch.float32, device=dev)
    eig = torch.empty((H, r), dtype=torch.float32, device=dev)
    ws = torch.empty(squat.build_subspace_workspace(n, H, qpk, d, r), dtype=torch.uint8, device=dev)
    upd = torch.empty((H, d, d), dtype=torch.float32, device=dev)
    wp = torch.empty(max(256, squat.prepare_workspace(H, d, r, 32)), dtype=torch.uint8, device=dev)
    codes = torch.empty((1, H, n, 8), dtype=torch.int32, device=dev)
    scale = torch.empty((1, H, n, 4), dtype=torch.float16, device=dev)
    zero = torch.empty_like(scale)
    back = torch.empty((1, H, n, d), dtype=torch.bfloat16, device=dev)
    qdec = qt[:, n - 1, :].unsqueeze(0).contiguous()
    logits = torch.empty((1, hq, n), dtype=torch.float32, device=dev)
    # the per-channel grouping and the pre-RoPE logits of both stores ride along (n is a multiple of 32)
    pcodes = torch.empty((1, H, n // 32, d, 2), dtype=torch.int32, device=dev)
    pscale = torch.empty((1, H, n // 32, d), dtype=torch.float16, device=dev)
    pzero = torch.empty_like(pscale)
    inv_freq = (10000.0 ** (-torch.arange(64, dtype=torch.float64, device=dev) / 64.0)).float()
    rope = torch.empty_like(logits)
    plogits = torch.empty_like(logits)
    prope = torch.empty_like(logits)
    outs = (qhat, eig, upd, codes, scale, zero, back, logits, pcodes, pscale, pzero, rope, plogits, prope)

    def path():
        squat.build_subspace(qt, qpk, r, qhat=qhat, eig=eig, ws=ws)
        squat.prepare(qhat, 1e-3, 32, update=upd, ws=wp)
        squat.quantize_keys(kt, upd, 2, 32, 32, codes=codes, scale=scale, zero=zero)
        squat.dequantize_keys(codes, scale, zero, 2, 32, out=back)
        squat.key_scores(qdec, codes, scale, zero, 2, 32, qpk, d ** -0.5, out=logits)
        squat.key_scores_rope(qdec, codes, scale, zero, 2, 32, qpk, inv_freq, 7, d ** -0.5, out=rope)
        squat.quantize_keys_per_channel(kt, upd, 2, 32, 32, codes=pcodes, scale=pscale, zero=pzero)
        squat.key_scores_per_channel(qdec, pcodes, pscale, pzero, 2, qpk, d ** -0.5, out=plogits)
        squat.key_scores_rope_per_channel(qdec, pcodes, pscale, pzero, 2, qpk, inv_freq, 7, d ** -0.5, out=prope)

    path()                                   # eager: also sets the kernels' attributes before any capture
    torch.cuda.synchronize()
    want = [t.clone() for t in outs]

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        path()
    for replay in range(3):
        for t in outs:                       # eager work between the replays: wipe every output
            t.view(torch.uint8).fill_(0xA5)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(outs, want):
            assert torch.equal(got.view(torch.uint8), ref.view(torch.uint8)), replay
