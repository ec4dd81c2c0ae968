"""Host-side checks that need no GPU: the C-ABI library loads, exports every
symbol the header declares, and rejects bad arguments before launching."""
import ctypes
import os
import re

import pytest

from paper_2503_24358_amd import squat

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "squat.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(squat_[a-z_]+)\s*\(", header))
    assert declared == set(squat.SYMBOLS)
    L = squat.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_version_and_strerror():
    assert squat.version() >= 100
    assert squat.strerror(0) == "ok"
    for code in range(-7, 0):
        assert squat.strerror(code) not in ("ok", "unknown status")
    assert squat.strerror(-99) == "unknown status"


def test_workspace_queries():
    assert squat.build_subspace_workspace(4096, 32, 1, 128, 16) >= 32 * 128 * 128 * 8
    assert squat.build_subspace_workspace(4096, 32, 1, 64, 16) == 0      # d != 128
    assert squat.prepare_workspace(8, 128, 16, 32) >= 8 * 3 * 16 * (32 + 128) * 8
    assert squat.prepare_workspace(8, 128, 16, 48) == 0


def test_argument_validation_happens_before_any_launch():
    L = squat.lib()
    fake = ctypes.c_void_p(0x1000)            # aligned, never dereferenced: every call below must fail first
    odd = ctypes.c_void_p(0x1004)
    q = lambda **kw: L.squat_quantize_keys(  # noqa: E731
        kw.get("k", fake), kw.get("dt", 2), kw.get("b", 1), kw.get("h", 1), kw.get("n", 32), kw.get("d", 128),
        kw.get("sb", 4096), kw.get("sh", 4096), kw.get("st", 128), kw.get("u", None), 0, kw.get("bits", 2),
        kw.get("G", 32), kw.get("g", 32), kw.get("codes", fake), fake, fake, None)
    assert q(d=64) == -2
    assert q(bits=3) == -2
    assert q(G=48) == -2
    assert q(g=16) == -2
    assert q(dt=7) == -3
    assert q(k=None) == -1
    assert q(codes=None) == -1
    assert q(st=120) == -2          # rows would overlap
    assert q(st=132) == -4          # not a multiple of 8 elements
    assert q(k=odd) == -4
    assert q(n=0) == 0              # empty input: nothing to do, nothing launched
    assert q(n=-1) == -2
    assert q(st=1 << 25) == -2      # bf16: a token stride of 2^26 bytes, same reason

    dq = lambda **kw: L.squat_dequantize_keys(  # noqa: E731
        kw.get("codes", fake), fake, fake, 1, 1, kw.get("n", 32), kw.get("d", 128), kw.get("bits", 2),
        kw.get("G", 32), kw.get("out", fake), kw.get("dt", 2), 4096, 4096, kw.get("st", 128), None)
    assert dq(d=256) == -2
    assert dq(bits=8) == -2
    assert dq(out=None) == -1
    assert dq(dt=5) == -3
    assert dq(st=130) == -4
    assert dq(n=0) == 0

    bs = lambda **kw: L.squat_build_subspace(  # noqa: E731
        kw.get("q", fake), kw.get("dt", 2), kw.get("n", 64), kw.get("h", 1), kw.get("qpk", 1), kw.get("d", 128),
        8192, kw.get("st", 128), kw.get("r", 8), kw.get("qhat", fake), None, None, kw.get("ws", fake),
        kw.get("wsb", 1 << 30), None)
    assert bs(d=96) == -2
    assert bs(r=129) == -2
    assert bs(r=-1) == -2
    assert bs(n=0) == -2
    assert bs(q=None) == -1
    assert bs(qhat=None) == -1
    assert bs(ws=None) == -5
    assert bs(wsb=16) == -5
    assert bs(dt=9) == -3
    assert bs(st=1 << 26) == -2     # bf16: a token stride of 2^27 bytes is beyond the kernel's 32-bit row offsets

    pr = lambda **kw: L.squat_prepare(  # noqa: E731
        kw.get("qhat", fake), 1, kw.get("d", 128), kw.get("r", 8), kw.get("lam", 1e-3), kw.get("g", 32),
        kw.get("u", fake), kw.get("ws", fake), kw.get("wsb", 1 << 30), None)
    assert pr(d=64) == -2
    assert pr(g=24) == -2
    assert pr(lam=-1.0) == -7
    assert pr(lam=float("nan")) == -7
    assert pr(u=None) == -1
    assert pr(qhat=None) == -1
    assert pr(ws=None) == -5
    assert pr(wsb=8) == -5


def test_per_channel_argument_validation_happens_before_any_launch():
    L = squat.lib()
    fake = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    q = lambda **kw: L.squat_quantize_keys_per_channel(  # noqa: E731
        kw.get("k", fake), kw.get("dt", 2), kw.get("b", 1), kw.get("h", 1), kw.get("n", 64), kw.get("d", 128),
        kw.get("sb", 8192), kw.get("sh", 8192), kw.get("st", 128), kw.get("u", None), 0, kw.get("bits", 2),
        kw.get("G", 32), kw.get("g", 32), kw.get("codes", fake), fake, fake, None)
    assert q(d=64) == -2
    assert q(bits=3) == -2
    assert q(G=64) == -2            # token groups are 32 tokens
    assert q(G=16) == -2
    assert q(g=16) == -2
    assert q(n=40) == -2            # not a multiple of the group
    assert q(dt=7) == -3
    assert q(k=None) == -1
    assert q(codes=None) == -1
    assert q(st=120) == -2
    assert q(st=132) == -4
    assert q(k=odd) == -4
    assert q(n=0) == 0
    assert q(n=-32) == -2

    dq = lambda **kw: L.squat_dequantize_keys_per_channel(  # noqa: E731
        kw.get("codes", fake), fake, fake, 1, 1, kw.get("n", 64), kw.get("d", 128), kw.get("bits", 2),
        kw.get("G", 32), kw.get("out", fake), kw.get("dt", 2), 8192, 8192, kw.get("st", 128), None)
    assert dq(d=256) == -2
    assert dq(bits=8) == -2
    assert dq(G=128) == -2
    assert dq(n=33) == -2
    assert dq(out=None) == -1
    assert dq(dt=5) == -3
    assert dq(st=130) == -4
    assert dq(codes=odd) == -4
    assert dq(n=0) == 0


def test_key_scores_argument_validation_happens_before_any_launch():
    L = squat.lib()
    fake = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    ks = lambda **kw: L.squat_key_scores(  # noqa: E731
        kw.get("codes", fake), fake, fake, 1, 2, kw.get("n", 64), kw.get("d", 128), kw.get("bits", 2),
        kw.get("G", 32), kw.get("q", fake), kw.get("dt", 2), kw.get("qpk", 4), 1024, kw.get("qsh", 128),
        kw.get("os", 1.0), kw.get("out", fake), 8 * 64, kw.get("ssh", 64), None)
    assert ks(d=64) == -2
    assert ks(bits=3) == -2
    assert ks(G=16) == -2
    assert ks(qpk=0) == -2
    assert ks(qpk=9) == -2
    assert ks(dt=4) == -3
    assert ks(os=float("nan")) == -7
    assert ks(q=None) == -1
    assert ks(out=None) == -1
    assert ks(qsh=64) == -2         # query rows would overlap
    assert ks(ssh=32) == -2         # score rows would overlap
    assert ks(codes=odd) == -4
    assert ks(n=0) == 0
    assert ks(n=-1) == -2
    kp = lambda **kw: L.squat_key_scores_per_channel(  # noqa: E731
        kw.get("codes", fake), kw.get("scale", fake), fake, 1, 2, kw.get("n", 64), kw.get("d", 128),
        kw.get("bits", 2), kw.get("G", 32), kw.get("q", fake), kw.get("dt", 2), kw.get("qpk", 4), 1024,
        kw.get("qsh", 128), kw.get("os", 1.0), kw.get("out", fake), 8 * 64, kw.get("ssh", 64), None)
    assert kp(d=64) == -2
    assert kp(bits=3) == -2
    assert kp(G=64) == -2           # token groups of 32 only
    assert kp(n=48) == -2           # whole token groups only
    assert kp(qpk=9) == -2
    assert kp(dt=4) == -3
    assert kp(os=float("nan")) == -7
    assert kp(q=None) == -1
    assert kp(ssh=32) == -2
    assert kp(codes=odd) == -4
    assert kp(scale=odd) == -4
    assert kp(n=0) == 0
    kr = lambda **kw: L.squat_key_scores_rope(  # noqa: E731
        kw.get("codes", fake), fake, fake, 1, 2, kw.get("n", 64), kw.get("d", 128), kw.get("bits", 2),
        kw.get("G", 32), kw.get("freq", fake), kw.get("pos0", 0), kw.get("q", fake), kw.get("dt", 2),
        kw.get("qpk", 4), 1024, kw.get("qsh", 128), kw.get("os", 1.0), kw.get("out", fake), 8 * 64,
        kw.get("ssh", 64), None)
    assert kr(d=64) == -2
    assert kr(bits=3) == -2
    assert kr(G=16) == -2
    assert kr(qpk=9) == -2
    assert kr(pos0=-1) == -2
    assert kr(dt=4) == -3
    assert kr(os=float("nan")) == -7
    assert kr(freq=None) == -1
    assert kr(q=None) == -1
    assert kr(ssh=32) == -2
    assert kr(codes=odd) == -4
    assert kr(n=0) == 0
    krp = lambda **kw: L.squat_key_scores_rope_per_channel(  # noqa: E731
        kw.get("codes", fake), kw.get("scale", fake), fake, 1, 2, kw.get("n", 64), kw.get("d", 128),
        kw.get("bits", 2), kw.get("G", 32), kw.get("freq", fake), kw.get("pos0", 0), kw.get("q", fake),
        kw.get("dt", 2), kw.get("qpk", 4), 1024, kw.get("qsh", 128), kw.get("os", 1.0), kw.get("out", fake), 8 * 64,
        kw.get("ssh", 64), None)
    assert krp(d=64) == -2
    assert krp(bits=3) == -2
    assert krp(G=64) == -2
    assert krp(n=48) == -2
    assert krp(qpk=9) == -2
    assert krp(pos0=1 << 40) == -2
    assert krp(dt=4) == -3
    assert krp(os=float("nan")) == -7
    assert krp(freq=None) == -1
    assert krp(ssh=32) == -2
    assert krp(codes=odd) == -4
    assert krp(scale=odd) == -4
    assert krp(n=0) == 0


def test_cache_configuration_and_creation_are_validated_on_the_host():
    L = squat.lib()
    ok = squat.CacheConfig(2, 8, 4, 128, 2, 32, 32, 32, 4096, 2, 1)
    need = L.squat_cache_arena_bytes(ctypes.byref(ok))
    per = 2 * 8 * 4096 * (32 + 8 + 8) + 2 * 8 * 32 * 256            # codes + scale + zero + residual, per tensor kind
    assert need >= 2 * per and need % 256 == 0
    keys_only = squat.CacheConfig(2, 8, 4, 128, 2, 32, 32, 32, 4096, 2, 0)
    assert per <= L.squat_cache_arena_bytes(ctypes.byref(keys_only)) < need
    for bad in (squat.CacheConfig(2, 8, 4, 64, 2, 32, 32, 32, 4096, 2, 0),      # d
                squat.CacheConfig(2, 8, 4, 128, 3, 32, 32, 32, 4096, 2, 0),     # bits
                squat.CacheConfig(2, 8, 4, 128, 2, 48, 32, 32, 4096, 2, 0),     # group
                squat.CacheConfig(2, 8, 0, 128, 2, 32, 32, 32, 4096, 2, 0),     # q_per_kv
                squat.CacheConfig(2, 8, 4, 128, 2, 32, 32, 32, 4100, 2, 0),     # capacity not a multiple of R
                squat.CacheConfig(2, 8, 4, 128, 2, 32, 32, 0, 4096, 2, 0),      # R
                squat.CacheConfig(2, 8, 4, 128, 2, 32, 32, 32, 4096, 5, 0),     # dtype
                squat.CacheConfig(2, 8, 4, 128, 2, 32, 32, 16, 4096, 2, 0, 1)): # per-channel keys: R not a multiple of 32
        assert L.squat_cache_arena_bytes(ctypes.byref(bad)) == 0
        h = ctypes.c_void_p()
        assert L.squat_cache_create(ctypes.byref(bad), ctypes.c_void_p(0x1000), 1 << 40, None, ctypes.byref(h)) == -2
    pc = squat.CacheConfig(2, 8, 4, 128, 2, 64, 32, 32, 4096, 2, 0, 1)          # per-channel keys: 4 scales per token
    assert L.squat_cache_arena_bytes(ctypes.byref(pc)) == L.squat_cache_arena_bytes(ctypes.byref(keys_only))
    h = ctypes.c_void_p()
    assert L.squat_cache_create(ctypes.byref(ok), None, need, None, ctypes.byref(h)) == -5
    assert L.squat_cache_create(ctypes.byref(ok), ctypes.c_void_p(0x1000), need - 1, None, ctypes.byref(h)) == -5
    assert L.squat_cache_create(ctypes.byref(ok), ctypes.c_void_p(0x1010), need, None, ctypes.byref(h)) == -4
    assert L.squat_cache_create(ctypes.byref(ok), ctypes.c_void_p(0x1000), need, None, None) == -1
    # a cache over a fake arena: bookkeeping calls that never touch the device
    assert L.squat_cache_create(ctypes.byref(ok), ctypes.c_void_p(0x100000), need, None, ctypes.byref(h)) == 0
    cnt = squat.CacheCounts()
    assert L.squat_cache_state(h, ctypes.byref(cnt)) == 0 and cnt.n_tokens == 0 and cnt.keys_residual == 0
    buf = squat.CacheBuffers()
    assert L.squat_cache_get_buffers(h, ctypes.byref(buf)) == 0 and buf.key_codes == 0x100000
    assert L.squat_cache_prefill(h, None, None, 64, 0, 0, 128, None) == -1            # NULL keys
    assert L.squat_cache_prefill(h, ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1000), 64, 0, 0, 100, None) == -4
    assert L.squat_cache_prefill(h, ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1000), -1, 0, 0, 128, None) == -2
    assert L.squat_cache_prefill(h, None, None, 0, 0, 0, 128, None) == 0               # nothing to do
    assert L.squat_cache_append(h, None, None, 0, 0, None) == -1
    fake = ctypes.c_void_p(0x1000)
    rope = lambda **kw: L.squat_cache_key_scores_rope(  # noqa: E731
        kw.get("c", h), kw.get("q", fake), kw.get("dt", 2), 4096, 128, kw.get("f", fake), kw.get("pos0", 0), 1.0,
        kw.get("s", fake), 1 << 20, 4096, None)
    assert rope(f=None) == -1 and rope(q=None) == -1 and rope(s=None) == -1 and rope(c=None) == -1
    assert rope(dt=6) == -3
    assert rope(pos0=-1) == -2 and rope(pos0=1 << 40) == -2
    assert rope() == 0                                                                 # empty cache: nothing launched
    hp = ctypes.c_void_p()
    assert L.squat_cache_create(ctypes.byref(pc), ctypes.c_void_p(0x100000), need, None, ctypes.byref(hp)) == 0
    assert rope(c=hp) == 0 and rope(c=hp, f=None) == -1                                # per-channel key store
    L.squat_cache_destroy(hp)
    assert L.squat_cache_reset(h) == 0
    L.squat_cache_destroy(h)
    assert L.squat_cache_state(None, ctypes.byref(cnt)) == -1


def test_quantize_plan_follows_the_documented_rule():
    """squat_quantize_keys_plan is a host-only query (without a GPU the library plans for 256 compute units):
    tiles of 32 tokens, problems = update matrices, persistent workgroups striding over a problem's tiles."""
    import torch
    bf16, f32 = torch.bfloat16, torch.float32
    # the benchmark's launch: 256 stacked heads, one workgroup each, 1024 tiles over 12 wavefronts
    p = squat.quantize_keys_plan(bf16, 1, 256, 32768, True, 0, 2, 32, 32)
    assert (p.problems, p.workgroups_per_problem, p.wavefronts_per_workgroup, p.tiles_per_problem) == (256, 1, 12, 1024)
    # one layer: 8 heads share the 256 compute units
    p = squat.quantize_keys_plan(bf16, 1, 8, 32768, True, 0, 2, 32, 32)
    assert (p.problems, p.workgroups_per_problem, p.tiles_per_problem) == (8, 32, 1024)
    # the decode flush: one tile per (sequence, head), the update matrix shared by the 64 sequences
    p = squat.quantize_keys_plan(bf16, 64, 256, 32, True, 0, 2, 32, 32)
    assert (p.problems, p.workgroups_per_problem, p.tiles_per_problem) == (256, 1, 64)
    # per-batch matrices: a problem per (sequence, head)
    p = squat.quantize_keys_plan(bf16, 4, 8, 100, True, 128 * 128 * 8, 2, 32, 32)
    assert (p.problems, p.tiles_per_problem) == (32, 4) and p.workgroups_per_problem == 4
    # a one-layer flush: 64 tiles per head spread over 32 workgroups each (two wavefronts busy per workgroup)
    p = squat.quantize_keys_plan(bf16, 64, 8, 32, True, 0, 2, 32, 32)
    assert (p.problems, p.workgroups_per_problem, p.tiles_per_problem) == (8, 32, 64)
    # never more workgroups than tiles
    p = squat.quantize_keys_plan(bf16, 1, 1, 100, True, 0, 2, 32, 32)
    assert (p.problems, p.workgroups_per_problem, p.tiles_per_problem) == (1, 4, 4)
    # fp32 keys run 6 wavefronts per workgroup, the two-tile-per-block and four-tile-statistics variants 8
    assert squat.quantize_keys_plan(f32, 1, 256, 1191, True, 0, 2, 32, 32).wavefronts_per_workgroup == 6
    assert squat.quantize_keys_plan(bf16, 1, 256, 1191, True, 0, 2, 32, 64).wavefronts_per_workgroup == 8
    assert squat.quantize_keys_plan(bf16, 1, 256, 1191, True, 0, 4, 128, 32).wavefronts_per_workgroup == 8
    # per-channel grouping: whole token groups only
    p = squat.quantize_keys_plan(bf16, 1, 256, 1216, True, 0, 2, 32, 32, per_channel=True)
    assert (p.problems, p.workgroups_per_problem, p.wavefronts_per_workgroup, p.tiles_per_problem) == (256, 1, 12, 38)
    L = squat.lib()
    out = squat.QuantizePlan()
    ref = ctypes.byref(out)
    assert L.squat_quantize_keys_plan(2, 1, 8, 1000, 1, 0, 2, 32, 32, 1, ref) == -2      # not a multiple of 32
    assert L.squat_quantize_keys_plan(2, 1, 8, 1024, 1, 0, 3, 32, 32, 0, ref) == -2
    assert L.squat_quantize_keys_plan(2, 1, 8, 1024, 1, 0, 2, 48, 32, 0, ref) == -2
    assert L.squat_quantize_keys_plan(2, 1, 8, 1024, 1, 0, 2, 64, 32, 1, ref) == -2      # per-channel groups are 32 tokens
    assert L.squat_quantize_keys_plan(9, 1, 8, 1024, 1, 0, 2, 32, 32, 0, ref) == -3
    assert L.squat_quantize_keys_plan(2, 1, 8, 1024, 1, 0, 2, 32, 32, 0, None) == -1


def test_refresh_subspace_argument_validation_happens_before_any_launch():
    L = squat.lib()
    fake = ctypes.c_void_p(0x1000)
    rf = lambda **kw: L.squat_refresh_subspace(  # noqa: E731
        kw.get("q", fake), kw.get("dt", 2), kw.get("n", 64), kw.get("h", 2), kw.get("qpk", 1), kw.get("d", 128),
        8192, kw.get("st", 128), kw.get("acc", 1), kw.get("state", fake), kw.get("r", 8), kw.get("it", 2),
        kw.get("prev", None), kw.get("rp", 0), kw.get("qhat", fake), None, None, kw.get("ws", fake),
        kw.get("wsb", 1 << 30), None)
    assert rf(d=64) == -2
    assert rf(r=33) == -2              # the iteration's block is 32 wide ...
    assert rf(r=33, it=-1, ws=None) == -5   # ... the exact mode takes any r (and fails later, on the missing workspace)
    assert rf(rp=33) == -2
    assert rf(n=-1) == -2
    assert rf(n=0, acc=0) == -2        # no queries and nothing to accumulate onto
    assert rf(state=None) == -1
    assert rf(qhat=None) == -1
    assert rf(q=None) == -1
    assert rf(dt=9) == -3
    assert rf(st=130) == -4
    assert rf(ws=None) == -5
    assert rf(wsb=16) == -5
    assert rf(h=0) == 0
    assert squat.lib().squat_refresh_subspace_workspace(64, 8, 4, 128, 16) >= 2 * 8 * 128 * 128 * 8
    assert squat.lib().squat_refresh_subspace_workspace(64, 8, 4, 96, 16) == 0
