"""The C ABI without a GPU: symbols, argument validation, error codes."""
import ctypes as C
import re
import os

import numpy as np
import pytest

from paper_2506_13472_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "rosaq.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(rosaq_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTED)
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), name


def _good(N=16, D=256, K=128, bits=4, mode=B.Q_NONE):
    rng = np.random.default_rng(0)
    W = (rng.standard_normal((N, D)) * 0.02).astype(np.float16)
    lam = np.arange(D, 0, -1.0)
    Q = None
    if mode == B.Q_FULL:
        Q = np.eye(D, dtype=np.float32)
    elif mode == B.Q_HEADWISE:
        Q = np.stack([np.eye(128, dtype=np.float32)] * (D // 128))
    return W, Q, lam, K, bits, mode


def _code(fn):
    with pytest.raises(B.RosaqError) as e:
        fn()
    assert B.rosaq_last_error() != ""
    return e.value.code


def test_pack_argument_errors():
    W, Q, lam, K, bits, mode = _good()
    assert _code(lambda: B.rosaq_pack_weights(None, Q, lam, K, bits, mode, host_only=True,
                                              out_features=16, in_features=256)) == -1
    assert _code(lambda: B.rosaq_pack_weights(W, Q, None, K, bits, mode, host_only=True)) == -1
    assert _code(lambda: B.rosaq_pack_weights(W, None, lam, K, bits, B.Q_FULL, host_only=True)) == -1
    assert _code(lambda: B.rosaq_pack_weights(W, Q, lam, K, 5, mode, host_only=True)) == -3
    assert _code(lambda: B.rosaq_pack_weights(W, Q, lam, K, bits, mode, group=64, host_only=True)) == -3
    assert _code(lambda: B.rosaq_pack_weights(W, Q, lam, K, bits, 7, host_only=True)) == -3
    assert _code(lambda: B.rosaq_pack_weights(W, Q, lam, K, bits, mode, select_rule=7, host_only=True)) == -3
    assert _code(lambda: B.rosaq_pack_weights(W, Q, lam, K, bits, mode, select_rule=3, select_arg=200,
                                              host_only=True)) == -2
    assert _code(lambda: B.rosaq_pack_weights(np.zeros((16, 384), np.float16), None, np.arange(384.0), 128, bits, mode,
                                              select_rule=1, host_only=True)) == -2   # 128 % 3 heads
    Wh, Qh, lamh, *_ = _good(mode=B.Q_HEADWISE)
    assert _code(lambda: B.rosaq_pack_weights(Wh, Qh, lamh, K, bits, B.Q_HEADWISE, head_dim=64,
                                              host_only=True)) == -3
    assert _code(lambda: B.rosaq_pack_weights(W[:, :200], Q, lam[:200], 72, bits, mode, host_only=True)) == -2
    assert _code(lambda: B.rosaq_pack_weights(W, Q, lam, 384, bits, mode, host_only=True)) == -2
    assert _code(lambda: B.rosaq_pack_weights(W, Q, lam, 64, bits, mode, host_only=True)) == -2
    assert _code(lambda: B.rosaq_pack_weights(W, Q, lam, K, bits, mode, ldw=100, host_only=True)) == -2
    out = C.c_void_p()
    assert B.lib().rosaq_pack_weights(None, None, C.byref(out)) == -1
    d = B.PackDesc()
    assert B.lib().rosaq_pack_weights(C.byref(d), None, None) == -1


def test_pack_rejects_nonfinite():
    W, Q, lam, K, bits, mode = _good()
    Wb = W.copy(); Wb[3, 7] = np.inf
    assert _code(lambda: B.rosaq_pack_weights(Wb, Q, lam, K, bits, mode, host_only=True)) == -7
    lb = lam.copy(); lb[5] = np.nan
    assert _code(lambda: B.rosaq_pack_weights(W, Q, lb, K, bits, mode, host_only=True)) == -7
    Wf, Qf, lamf, *_ = _good(mode=B.Q_FULL)
    Qb = Qf.copy(); Qb[0, 0] = np.nan
    assert _code(lambda: B.rosaq_pack_weights(Wf, Qb, lamf, K, bits, B.Q_FULL, host_only=True)) == -7
    Qo = Qf * np.float32(1e7)
    assert _code(lambda: B.rosaq_pack_weights(Wf, Qo, lamf, K, bits, B.Q_FULL, host_only=True)) == -7


def test_call_argument_errors_on_host_only_handle():
    W, Q, lam, K, bits, mode = _good()
    p = B.rosaq_pack_weights(W, Q, lam, K, bits, mode, host_only=True)
    assert (p.N, p.D, p.K, p.bits, p.group, p.q_mode) == (16, 256, 128, 4, 128, 0)
    assert p.device_bytes == 0
    ws_full = B.rosaq_workspace_bytes(p, 4)
    ws = B.rosaq_workspace_bytes_min(p, 4)      # the full size adds room for split launches
    assert ws >= 256 and ws % 256 == 0 and ws_full % 256 == 0 and ws_full >= ws + 16 * 16 * 16 * 4
    assert B.rosaq_workspace_bytes_batch([p, p], 4) >= ws_full
    assert B.rosaq_workspace_bytes(p, 0) == 0 and B.rosaq_workspace_bytes_min(p, 0) == 0
    assert B.rosaq_workspace_bytes(p, 65) == B.rosaq_workspace_bytes_min(p, 65)   # no splits above 64 rows
    X, Y, WS = 0x1000, 0x2000, 0x4000      # never dereferenced: every call fails validation first
    assert _code(lambda: B.rosaq_linear(p, 0, 4, 256, Y, 16, WS, ws)) == -1
    assert _code(lambda: B.rosaq_linear(p, X, 0, 256, Y, 16, WS, ws)) == -2
    assert _code(lambda: B.rosaq_linear(p, X, (1 << 20) + 1, 256, Y, 16, WS, 1 << 40)) == -2
    assert _code(lambda: B.rosaq_linear(p, X, 4, 128, Y, 16, WS, ws)) == -2
    assert _code(lambda: B.rosaq_linear(p, X, 4, 256, Y, 8, WS, ws)) == -2
    assert _code(lambda: B.rosaq_linear(p, X + 2, 4, 256, Y, 16, WS, ws)) == -5
    assert _code(lambda: B.rosaq_linear(p, X, 4, 260, Y, 16, WS, ws)) == -5
    assert _code(lambda: B.rosaq_linear(p, X, 4, 256, Y, 16, 0, ws)) == -6
    assert _code(lambda: B.rosaq_linear(p, X, 4, 256, Y, 16, WS, ws - 1)) == -6
    assert _code(lambda: B.rosaq_linear(p, X, 4, 256, Y, 16, WS + 16, ws)) == -5
    assert _code(lambda: B.rosaq_linear_headwise(p, X, 4, 256, Y, 16, WS, ws)) == -4
    assert _code(lambda: B.rosaq_linear(p, X, 4, 256, Y, 16, WS, ws)) == -10
    Wh, Qh, lamh, *_ = _good(mode=B.Q_HEADWISE)
    ph = B.rosaq_pack_weights(Wh, Qh, lamh, K, bits, B.Q_HEADWISE, host_only=True)
    assert _code(lambda: B.rosaq_linear(ph, X, 4, 256, Y, 16, WS, 1 << 30)) == -4
    assert _code(lambda: B.rosaq_linear_headwise(ph, X, 4, 256, Y, 16, WS, 1 << 30)) == -10
    assert B.lib().rosaq_linear(None, X, 4, 256, Y, 16, WS, ws, None) == -1
    assert B.lib().rosaq_packed_info(None, *([None] * 7)) == -1
    assert B.lib().rosaq_packed_export(None, *([None] * 5)) == -1
    B.lib().rosaq_free(None)
    p.free(); ph.free()


def test_mlp_block_argument_errors_on_host_only_handles():
    W, Q, lam, K, bits, mode = _good(mode=B.Q_FULL)                      # gate / up: 16 x 256, dense rotation
    g = B.rosaq_pack_weights(W, Q, lam, K, bits, B.Q_FULL, host_only=True)
    g3 = B.rosaq_pack_weights(W, Q, lam, K, 3, B.Q_FULL, host_only=True)
    Wd = np.zeros((48, 128), np.float16)                                   # a down layer would need D = 16
    d_wide = B.rosaq_pack_weights(Wd, None, np.arange(128.0), 0, bits, B.Q_NONE, host_only=True)
    W16 = np.zeros((256, 256), np.float16); W16[0, 0] = 1
    gq = B.rosaq_pack_weights(W16, Q, lam, K, bits, B.Q_FULL, host_only=True)       # 256 -> 256
    d_ok = B.rosaq_pack_weights(W16, None, lam, K, bits, B.Q_NONE, host_only=True)  # takes 256 channels
    d_rot = B.rosaq_pack_weights(W16, Q, lam, K, bits, B.Q_FULL, host_only=True)
    d_abs = B.rosaq_pack_weights(W16, Q, lam, K, bits, B.Q_FULL, host_only=True, rotation_absorbed=True)
    X, Y, WS = 0x1000, 0x2000, 0x4000      # never dereferenced: every call fails validation first
    try:
        n = B.rosaq_workspace_bytes_mlp(gq, gq, d_ok, 4)
        assert n % 256 == 0 and n > B.rosaq_workspace_bytes_min(gq, 4) + B.rosaq_workspace_bytes_min(d_ok, 4) - 1
        assert B.rosaq_workspace_bytes_mlp(gq, gq, d_abs, 4) == n          # absorbed rotation: no rotation at run time
        assert B.rosaq_workspace_bytes_mlp(gq, gq, d_rot, 4) == 0
        assert B.rosaq_workspace_bytes_mlp(g, g, d_wide, 4) == 0
        assert B.rosaq_workspace_bytes_mlp(gq, gq, d_ok, 0) == 0
        assert _code(lambda: B.rosaq_mlp_swiglu(g, g3, d_wide, X, 4, 256, Y, 48, WS, 1 << 30)) == -4   # gate / up differ
        assert _code(lambda: B.rosaq_mlp_swiglu(g, g, d_wide, X, 4, 256, Y, 48, WS, 1 << 30)) == -2    # width of down
        assert _code(lambda: B.rosaq_mlp_swiglu(gq, gq, d_rot, X, 4, 256, Y, 256, WS, 1 << 30)) == -4  # down rotates
        assert _code(lambda: B.rosaq_mlp_swiglu(gq, gq, d_ok, 0, 4, 256, Y, 256, WS, n)) == -1
        assert _code(lambda: B.rosaq_mlp_swiglu(gq, gq, d_ok, X, 4, 256, 0, 256, WS, n)) == -1
        assert _code(lambda: B.rosaq_mlp_swiglu(gq, gq, d_ok, X, 0, 256, Y, 256, WS, n)) == -2
        assert _code(lambda: B.rosaq_mlp_swiglu(gq, gq, d_ok, X, 4, 256, Y, 128, WS, n)) == -2          # ldy < N
        assert _code(lambda: B.rosaq_mlp_swiglu(gq, gq, d_ok, X, 4, 256, Y, 256, WS,
                                                B.rosaq_workspace_bytes_min(gq, 4))) == -6                # gate's share only
        assert _code(lambda: B.rosaq_mlp_swiglu(gq, gq, d_ok, X, 4, 256, Y, 256, WS + 16, n)) == -5
        assert _code(lambda: B.rosaq_mlp_swiglu(gq, gq, d_ok, X, 4, 256, Y, 256, WS, n)) == -10          # host-only handles
        assert B.lib().rosaq_mlp_swiglu(None, None, None, X, 4, 256, Y, 256, WS, n, None) == -1
    finally:
        for p in (g, g3, d_wide, gq, d_ok, d_rot, d_abs):
            p.free()


def test_tune_keys():
    for k in ("mt", "nt", "wpb"):
        B.rosaq_tune(k, 0)
    assert _code(lambda: B.rosaq_tune("mt", 3)) == -3          # 48-row tiles do not exist
    for v in (3, 6, 0):
        B.rosaq_tune("nt", v)                                  # 48- and 96-channel tiles do
    assert _code(lambda: B.rosaq_tune("nt", 5)) == -3
    assert _code(lambda: B.rosaq_tune("wpb", 3)) == -3
    assert _code(lambda: B.rosaq_tune("depth", 5)) == -3
    assert _code(lambda: B.rosaq_tune("stages", 0)) == -3
    assert _code(lambda: B.rosaq_tune("nope", 1)) == -3


def test_batch_argument_errors():
    W, Q, lam, K, bits, mode = _good()
    p = B.rosaq_pack_weights(W, Q, lam, K, bits, mode, host_only=True)
    p2 = B.rosaq_pack_weights(W[:8], Q, lam, K, bits, mode, host_only=True)
    lam3 = lam[::-1].copy()                       # other storage order -> other rotated input
    p3 = B.rosaq_pack_weights(W, Q, lam3, K, bits, mode, host_only=True)
    p4 = B.rosaq_pack_weights(W, Q, lam, K, 3, mode, host_only=True)
    X, Y, WS = 0x1000, 0x2000, 0x4000
    ws = B.rosaq_workspace_bytes(p, 4)
    ok = B.BatchArgs([p, p2], [Y, Y], [16, 8])
    assert _code(lambda: B.rosaq_linear_batch(ok, X, 4, 256, WS, ws)) == -10     # valid up to HOSTONLY
    assert _code(lambda: B.rosaq_linear_batch(B.BatchArgs([p, p3], [Y, Y], [16, 16]), X, 4, 256, WS, ws)) == -4
    assert _code(lambda: B.rosaq_linear_batch(B.BatchArgs([p, p4], [Y, Y], [16, 16]), X, 4, 256, WS, ws)) == -4
    assert _code(lambda: B.rosaq_linear_batch(B.BatchArgs([p] * 5, [Y] * 5, [16] * 5), X, 4, 256, WS, ws)) == -3
    assert _code(lambda: B.rosaq_linear_batch(B.BatchArgs([p, p2], [Y, 0], [16, 8]), X, 4, 256, WS, ws)) == -1
    assert _code(lambda: B.rosaq_linear_batch(B.BatchArgs([p, p2], [Y, Y], [16, 4]), X, 4, 256, WS, ws)) == -2
    assert B.lib().rosaq_linear_batch(None, 1, X, 4, 256, None, None, WS, ws, None) == -1
    ok.count = 0
    assert _code(lambda: B.rosaq_linear_batch(ok, X, 4, 256, WS, ws)) == -3
    for h in (p, p2, p3, p4):
        h.free()


def test_stream_probe_argument_errors():
    S, H, K = 0x10000, 0x20000, 0x30000
    ok = dict(src_ptr=S, src_bytes=256 * 8 * 1024, shared_ptr=H, shared_bytes=512 * 1024,
              shared_bytes_per_workgroup=8 * 1024, workgroups=256, threads=512, sink_ptr=K,
              sink_bytes=256 * 8 * 1024)
    def call(**kw):
        a = dict(ok); a.update(kw)
        return _code(lambda: B.rosaq_stream_probe(**a))
    assert call(src_ptr=0) == -1
    assert call(sink_ptr=0) == -1
    assert call(threads=100) == -3
    assert call(threads=2048) == -3
    assert call(workgroups=0) == -3
    assert call(src_bytes=1000) == -2
    assert call(src_bytes=0) == -2
    assert call(shared_bytes_per_workgroup=1024) == -2          # not 1 KiB per wave
    assert call(shared_bytes=512, shared_bytes_per_workgroup=8 * 1024) == -2
    assert call(shared_ptr=0) == -2
    assert call(sink_bytes=1024) == -6
    assert call(src_ptr=S + 4) == -5


def test_clone_of_host_only_handle():
    import ctypes as C
    W, Q, lam, K, bits, mode = _good(mode=B.Q_HEADWISE)
    p = B.rosaq_pack_weights(W, Q, lam, K, bits, mode, host_only=True)
    c = B.rosaq_packed_clone(p)
    a, b = B.rosaq_packed_export(p), B.rosaq_packed_export(c)
    p.free()                                        # the clone owns its own copies
    for k in a:
        assert np.array_equal(a[k].view(np.uint8), b[k].view(np.uint8)), k
    assert (c.N, c.D, c.K, c.bits, c.q_mode) == (16, 256, 128, 4, B.Q_HEADWISE)
    out = C.c_void_p()
    assert B.lib().rosaq_packed_clone(None, None, C.byref(out)) == -1
    assert B.lib().rosaq_packed_clone(c.handle, None, None) == -1
    c.free()


def test_pca_headwise_argument_errors():
    X = 0x10000
    assert _code(lambda: B.rosaq_pca_headwise(0, 64, 256, 256)) == -1
    assert _code(lambda: B.rosaq_pca_headwise(X, 0, 256, 256)) == -2
    assert _code(lambda: B.rosaq_pca_headwise(X, 64, 200, 256)) == -2
    assert _code(lambda: B.rosaq_pca_headwise(X, 64, 256, 128)) == -2
    assert _code(lambda: B.rosaq_pca_headwise(X + 1, 64, 256, 256)) == -5
    assert B.lib().rosaq_pca_headwise(X, 64, 256, 256, None, None, None) == -1
    assert _code(lambda: B.rosaq_pca_full(0, 64, 256, 256)) == -1
    assert _code(lambda: B.rosaq_pca_full(X, 0, 256, 256)) == -2
    assert _code(lambda: B.rosaq_pca_full(X, 64, 200, 256)) == -2
    assert _code(lambda: B.rosaq_pca_full(X, 64, 8320, 8320)) == -2
    assert _code(lambda: B.rosaq_pca_full(X, 64, 256, 128)) == -2
    assert _code(lambda: B.rosaq_pca_full(X + 1, 64, 256, 256)) == -5


def test_launch_shape_of_the_named_workloads():
    """The tile heuristic on the shapes the bench and the design notes quote (host logic only)."""
    shape = B.rosaq_launch_shape
    # LLaMA-7B attention at M = 64, INT4: q/k/v in one launch fill the 256 CUs exactly with 64x48 tiles
    # (3 * 256 channel tiles in chunks of 3), the o projection with 32x32 tiles
    assert shape(64, 3 * 4096, 4096, 4)[:3] == (4, 3, 8)
    assert shape(64, 4096, 4096, 4)[:3] == (2, 2, 8)
    # gate + up of a 7B MLP in one launch: 64x48 at M = 64, 32x96 (one round instead of three) at M = 32
    assert shape(64, 2 * 11008, 4096, 4)[:3] == (4, 3, 8)
    assert shape(32, 2 * 11008, 4096, 4)[:3] == (2, 6, 8)
    # 13B up projection at M = 64: 216 workgroups of 64x64 stay (the alternatives need a second round)
    assert shape(64, 13824, 5120, 4)[:3] == (4, 4, 8)
    # prefill-sized calls keep 64x64 tiles
    assert shape(4096, 4096, 4096, 4)[:3] == (4, 4, 8)
    assert shape(2048, 13824, 5120, 4)[:3] == (4, 4, 8)
    # single rows: one 16x16 tile and sixteen waves per workgroup
    assert shape(1, 4096, 4096, 4) == (1, 1, 16, 1, 1)
    # two tiles per workgroup in a launch of less than one round (13B down projection): sixteen waves too;
    # launches of several rounds keep eight
    assert shape(1, 5120, 13824, 4) == (1, 2, 16, 2, 1)
    assert shape(1, 13824, 5120, 4) == (1, 2, 8, 2, 1)
    # the contraction is split over workgroups only where whole 64-row tiles would leave the chip
    # under-filled over a long contraction: the 13B down projection runs as 80 tiles x 3 splits
    assert shape(64, 5120, 13824, 4) == (4, 4, 8, 1, 3)
    assert shape(64, 4096, 4096, 4)[4] == 1 and shape(64, 3 * 4096, 4096, 4)[4] == 1
    assert shape(64, 4096, 11008, 3)[4] == 1 and shape(256, 5120, 13824, 4)[4] == 1
    # all-fp16 layers (the dense rotation) never get the 48- or 96-channel tiles
    assert shape(64, 4096, 4096, 16)[1] in (1, 2, 4)
    # overrides go through
    B.rosaq_tune("mt", 2); B.rosaq_tune("nt", 6)
    try:
        assert shape(64, 4096, 4096, 3)[:2] == (2, 6)
    finally:
        B.rosaq_tune("mt", 0); B.rosaq_tune("nt", 0)
    B.rosaq_tune("splits", 5)
    try:
        assert shape(64, 4096, 4096, 4) == (4, 4, 8, 1, 5)
        assert shape(16, 4096, 4096, 4)[::4] == (1, 5)
        assert shape(65, 4096, 4096, 4)[4] == 1            # never above 64 rows
    finally:
        B.rosaq_tune("splits", 0)
    for bad in ((0, 4096, 4096, 4), (64, 4090, 4096, 4), (64, 4096, 4000, 4)):
        with pytest.raises(B.RosaqError) as e:
            shape(*bad)
        assert B.ERR_NAMES[e.value.code] == "SHAPE"
    with pytest.raises(B.RosaqError) as e:
        shape(64, 4096, 4096, 5)
    assert B.ERR_NAMES[e.value.code] == "ARG"


def test_bench_traffic_table_holds_the_shapes_the_heuristic_picks():
    """bench.py reports measured HBM traffic only for launch shapes it has a profile for: the two
    launches of its default workload must be among them, or the default line would say null."""
    import importlib.util, os
    spec = importlib.util.spec_from_file_location("bench", os.path.join(os.path.dirname(__file__), "..", "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    one = (1,) + tuple(B.rosaq_launch_shape(64, 4096, 4096, 4))
    qkv = (3,) + tuple(B.rosaq_launch_shape(64, 3 * 4096, 4096, 4))
    assert one in bench.MEASURED_TRAFFIC_KIB and qkv in bench.MEASURED_TRAFFIC_KIB


def test_block_map_covers_every_tile_exactly_once():
    """The workgroup -> (channel chunk, row group) map of the main GEMM: a bijection onto the launch's tiles
    plus padding workgroups, with every chunk on the XCD (workgroup % 8) equal to chunk % 8, for all small
    launch shapes and the ones of the named workloads."""
    shapes = [(c, m) for c in range(1, 70) for m in range(1, 14)]
    shapes += [(256, 1), (128, 2), (192, 1), (230, 2), (459, 1), (216, 64), (64, 64), (80, 16), (500, 64), (257, 9)]
    for chunks, mgroups in shapes:
        grid = B.rosaq_block_map(-1, chunks, mgroups)
        assert grid >= chunks * mgroups and grid % 8 == 0
        seen = set()
        for b in range(grid):
            t = B.rosaq_block_map(b, chunks, mgroups)
            if t is None:
                continue
            c, m = t
            assert 0 <= c < chunks and 0 <= m < mgroups
            assert c % 8 == b % 8                      # a chunk's workgroups share one XCD's L2
            assert t not in seen
            seen.add(t)
        assert len(seen) == chunks * mgroups, (chunks, mgroups)
        # padding stays bounded: chunk slots round up to whole XCD columns (and to blocks of 8 from 8 on),
        # row groups to blocks of 4
        cx = (chunks + 7) // 8
        assert grid <= 8 * (cx + (7 if cx >= 8 else 0)) * (mgroups + 3)
    with pytest.raises(B.RosaqError):
        B.rosaq_block_map(0, 0, 1)
