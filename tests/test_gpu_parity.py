"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import rosaq_oracle as O
from paper_2506_13472_amd import binding as B
from paper_2506_13472_amd import synth

pytestmark = pytest.mark.gpu

MAX_TOL = 2e-3      # max |y - y_ref| / (||x_row|| ||w_col||)
FRO_TOL = 1e-3      # ||y - y_ref||_F / ||y_ref||_F


def run_gpu(p, x16):
    from paper_2506_13472_amd import torch_glue as T
    x = torch.from_numpy(x16).cuda()
    y = T.linear(p, x)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def check_output(y, x16, Q, ref):
    y_ref = O.linear_ref(x16, Q, ref)
    scale = O.tolerance_scale(x16, ref)
    err = np.abs(y.astype(np.float64) - y_ref)
    max_rel = float(np.max(err / scale))
    fro = float(np.linalg.norm(err) / np.linalg.norm(y_ref))
    print(f"  max_rel={max_rel:.3e} fro={fro:.3e}", flush=True)
    assert np.all(np.isfinite(y))
    assert max_rel <= MAX_TOL, max_rel
    assert fro <= FRO_TOL, fro


def check_pack(p, ref):
    got = B.rosaq_packed_export(p)
    for k in ("salient_idx", "W_S", "codes", "scales", "zeros"):
        a, b = got[k], np.asarray(ref[k])
        if a.dtype == np.float16:
            a, b = a.view(np.uint16), b.astype(np.float16).view(np.uint16)
        assert np.array_equal(a, b), k


import functools


@functools.lru_cache(maxsize=4)
def make_case(seed, M, D, N, n_cal, mode, solver=None):
    """Inputs + rotation.  The oracle's Jacobi solver serves the 128-blocks and D <= 256;
    larger dense cases use its LAPACK route (checked against Jacobi in the CPU tests)."""
    if solver is None:
        solver = "jacobi" if (mode == O.MODE_HEADWISE or D <= 256) else "lapack"
    lay = synth.make_layer(seed, M, D, N, n_cal)
    if mode == O.MODE_NONE:
        Q, lam = None, np.abs(lay["X_cal"]).mean(axis=0)
    elif mode == O.MODE_FULL:
        Q, lam = O.pca_full(lay["X_cal"], solver)
        Q = Q.astype(np.float32)
    else:
        Q, lam = O.pca_headwise(lay["X_cal"], 128, solver)
        Q = Q.astype(np.float32)
    return lay, Q, lam


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("mode", [O.MODE_NONE, O.MODE_HEADWISE, O.MODE_FULL])
@pytest.mark.parametrize("M,D,N,K", [(4, 256, 48, 128), (64, 512, 200, 128), (37, 384, 130, 0),
                                     (16, 256, 64, 256), (100, 512, 96, 128)])
def test_small_shapes(bits, mode, M, D, N, K):
    print(f"case bits={bits} mode={mode} M={M} D={D} N={N} K={K}", flush=True)
    lay, Q, lam = make_case(100 + M, M, D, N, 300, mode)
    ref = O.pack(lay["W"], Q, lam, K, bits, mode)
    p = B.rosaq_pack_weights(lay["W"], Q, lam, K, bits, mode)
    check_pack(p, ref)
    y = run_gpu(p, lay["x"])
    check_output(y, lay["x"], Q, ref)
    p.free()


def test_config0_single_linear():
    """M=4, D=N=1024, full PCA rotation from 64 calibration rows, K=128, INT4 g128, seed 0."""
    print("case config0", flush=True)
    lay, Q, lam = make_case(0, 4, 1024, 1024, 64, O.MODE_FULL, solver="lapack")
    ref = O.pack(lay["W"], Q, lam, 128, 4, O.MODE_FULL)
    assert ref["salient_idx"].tolist() == list(range(128))
    p = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 4, B.Q_FULL)
    check_pack(p, ref)
    y = run_gpu(p, lay["x"])
    check_output(y, lay["x"], Q, ref)
    p.free()


@pytest.mark.parametrize("mt,nt,wpb", [(1, 1, 8), (1, 1, 16), (2, 2, 8), (4, 1, 8), (1, 4, 8), (4, 2, 8), (2, 4, 8), (2, 1, 16), (1, 2, 16),
                                       (4, 3, 8), (2, 3, 8), (2, 6, 8), (4, 6, 4)])
def test_tile_variants_agree_with_oracle_and_are_deterministic(mt, nt, wpb):
    print(f"case mt={mt} nt={nt} wpb={wpb}", flush=True)
    lay, Q, lam = make_case(7, 64, 1024, 256, 512, O.MODE_HEADWISE)
    ref = O.pack(lay["W"], Q, lam, 128, 4, O.MODE_HEADWISE)
    for k, v in (("mt", mt), ("nt", nt), ("wpb", wpb)):
        B.rosaq_tune(k, v)
    try:
        p = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 4, B.Q_HEADWISE)
        y0 = run_gpu(p, lay["x"])
        check_output(y0, lay["x"], Q, ref)
        for _ in range(5):
            assert np.array_equal(run_gpu(p, lay["x"]).view(np.uint16), y0.view(np.uint16))
        p.free()
    finally:
        for k in ("mt", "nt", "wpb"):
            B.rosaq_tune(k, 0)


@pytest.mark.parametrize("mode,bits", [(O.MODE_HEADWISE, 4), (O.MODE_FULL, 3), (O.MODE_NONE, 4)])
def test_batch_of_layers_sharing_the_rotation(mode, bits):
    """q/k/v-style batch: three layers with different widths share x and Q; one launch."""
    from paper_2506_13472_amd import torch_glue as T
    print(f"case batch mode={mode} bits={bits}", flush=True)
    M, D = 64, 512
    lay, Q, lam = make_case(21, M, D, 200, 300, mode)
    Ws = [lay["W"], synth.make_weight(31, 96, D), synth.make_weight(32, 330, D)]
    refs = [O.pack(W, Q, lam, 128, bits, mode) for W in Ws]
    ps = [B.rosaq_pack_weights(W, Q, lam, 128, bits, mode) for W in Ws]
    for p, ref in zip(ps, refs):
        check_pack(p, ref)
    x = torch.from_numpy(lay["x"]).cuda()
    ys = T.linear_batch(ps, x)
    torch.cuda.synchronize()
    for y, p, ref in zip(ys, ps, refs):
        yh = y.cpu().numpy()
        check_output(yh, lay["x"], Q, ref)
        # the batched launch and the single-layer call run the same arithmetic
        assert np.array_equal(run_gpu(p, lay["x"]).view(np.uint16), yh.view(np.uint16))
    for p in ps:
        p.free()


@pytest.mark.parametrize("mt,nt,wpb", [(1, 2, 8), (2, 4, 8), (4, 4, 8), (2, 3, 8), (4, 3, 8), (2, 6, 8), (4, 6, 4)])
@pytest.mark.parametrize("bits", [4, 3])
def test_chunks_that_span_the_layers_of_a_batch(mt, nt, wpb, bits):
    """Layers of 13, 6, 21 and 1 channel tiles in one launch: with every tile width some chunk
    ends in one layer and goes on in the next, and the last chunk runs past the end of the list."""
    from paper_2506_13472_amd import torch_glue as T
    print(f"case spanning chunks mt={mt} nt={nt} wpb={wpb} bits={bits}", flush=True)
    M, D = 50, 640
    lay, Q, lam = make_case(41, M, D, 200, 300, O.MODE_HEADWISE)
    Ws = [lay["W"], synth.make_weight(51, 96, D), synth.make_weight(52, 330, D), synth.make_weight(53, 9, D)]
    refs = [O.pack(W, Q, lam, 128, bits, O.MODE_HEADWISE) for W in Ws]
    ps = [B.rosaq_pack_weights(W, Q, lam, 128, bits, B.Q_HEADWISE) for W in Ws]
    x = torch.from_numpy(lay["x"]).cuda()
    singles = [run_gpu(p, lay["x"]) for p in ps]          # default tiles, one layer per launch
    for k, v in (("mt", mt), ("nt", nt), ("wpb", wpb)):
        B.rosaq_tune(k, v)
    try:
        ys = [torch.full((M, W.shape[0] + 3), 5.0, dtype=torch.float16, device="cuda") for W in Ws]
        T.linear_batch(ps, x, [y[:, :W.shape[0]] for y, W in zip(ys, Ws)])
        torch.cuda.synchronize()
    finally:
        for k in ("mt", "nt", "wpb"):
            B.rosaq_tune(k, 0)
    for y, W, ref, single in zip(ys, Ws, refs, singles):
        yh = y.cpu().numpy()
        assert np.all(yh[:, W.shape[0]:] == 5.0)          # nothing written past a layer's last channel
        check_output(yh[:, :W.shape[0]], lay["x"], Q, ref)
        if wpb == 8:                                       # same wave count, same summation order
            assert np.array_equal(yh[:, :W.shape[0]].view(np.uint16), single.view(np.uint16))
    for p in ps:
        p.free()


def test_strided_x_and_y():
    from paper_2506_13472_amd import torch_glue as T
    print("case strided", flush=True)
    lay, Q, lam = make_case(9, 20, 256, 64, 300, O.MODE_HEADWISE)
    ref = O.pack(lay["W"], Q, lam, 128, 4, O.MODE_HEADWISE)
    p = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 4, B.Q_HEADWISE)
    xb = torch.zeros((20, 256 + 64), dtype=torch.float16, device="cuda")
    xb[:, :256] = torch.from_numpy(lay["x"]).cuda()
    yb = torch.full((20, 64 + 8), 7.0, dtype=torch.float16, device="cuda")
    T.linear(p, xb[:, :256], yb[:, :64])
    torch.cuda.synchronize()
    yh = yb.cpu().numpy()
    assert np.all(yh[:, 64:] == 7.0)                  # nothing written outside y
    check_output(yh[:, :64], lay["x"], Q, ref)
    p.free()


def test_config1_attention_projection_full_size():
    """LLaMA-7B attention projection: D=N=4096, 32 heads, M=64, K=128, INT4, head-wise PCA from
    512 calibration rows; the launch configuration the bench times."""
    print("case config1", flush=True)
    lay, Q, lam = make_case(1, 64, 4096, 4096, 512, O.MODE_HEADWISE, solver="lapack")
    ref = O.pack(lay["W"], Q, lam, 128, 4, O.MODE_HEADWISE)
    p = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 4, B.Q_HEADWISE)
    check_pack(p, ref)
    y = run_gpu(p, lay["x"])
    check_output(y, lay["x"], Q, ref)
    p.free()


def test_stream_probe_runs_and_writes_nothing():
    print("case stream probe", flush=True)
    n = 256 * 8 * 4 * 1024
    src = torch.ones(n, dtype=torch.uint8, device="cuda")
    shared = torch.full((512 * 1024,), 2, dtype=torch.uint8, device="cuda")
    sink = torch.full((256 * 8 * 1024,), 9, dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    for per_wg in (0, 64 * 1024, 512 * 1024):
        B.rosaq_stream_probe(src.data_ptr(), n, shared.data_ptr(), shared.numel(), per_wg, 256, 512,
                             sink.data_ptr(), sink.numel(), st)
    torch.cuda.synchronize()
    assert bool((sink == 9).all())


def test_clone_runs_like_the_original_and_batches_with_it():
    from paper_2506_13472_amd import torch_glue as T
    print("case clone", flush=True)
    lay, Q, lam = make_case(9, 20, 256, 64, 300, O.MODE_HEADWISE)
    p = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 4, B.Q_HEADWISE)
    c = B.rosaq_packed_clone(p)
    y0 = run_gpu(p, lay["x"])
    p.free()
    y1 = run_gpu(c, lay["x"])
    assert np.array_equal(y0.view(np.uint16), y1.view(np.uint16))
    c2 = B.rosaq_packed_clone(c)
    ys = T.linear_batch([c, c2], torch.from_numpy(lay["x"]).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(ys[1].cpu().numpy().view(np.uint16), y0.view(np.uint16))
    c.free(); c2.free()


@pytest.mark.parametrize("rule,arg,K", [(B.SELECT_TOP_PER_HEAD, 0, 128), (B.SELECT_CONSECUTIVE, 200, 128),
                                        (B.SELECT_TOP_AND_BOTTOM, 0, 128), (B.SELECT_BOTTOM, 0, 128)])
def test_selection_rules_on_gpu(rule, arg, K):
    """Paper's per-head setting (32 salient channels per head at K = 128, 4 heads) and the
    ablation rules: other storage orders through the same kernels."""
    print(f"case select rule={rule} arg={arg} K={K}", flush=True)
    lay, Q, lam = make_case(33, 48, 512, 160, 400, O.MODE_HEADWISE)
    ref = O.pack(lay["W"], Q, lam, K, 4, O.MODE_HEADWISE, rule=rule, arg=arg)
    p = B.rosaq_pack_weights(lay["W"], Q, lam, K, 4, B.Q_HEADWISE, select_rule=rule, select_arg=arg)
    check_pack(p, ref)
    check_output(run_gpu(p, lay["x"]), lay["x"], Q, ref)
    p.free()


def test_rotation_absorbed_offline_per_head_salient():
    """The paper's own deployment of the attention output projection: 32 salient channels per
    head, rotation folded into the producer, so the layer receives rotated activations."""
    print("case absorbed", flush=True)
    lay, Q, lam = make_case(35, 64, 512, 192, 400, O.MODE_HEADWISE)
    ref = O.pack(lay["W"], Q, lam, 128, 4, O.MODE_HEADWISE, rule=O.RULE_TOP_PER_HEAD)
    p = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 4, B.Q_HEADWISE, select_rule=B.SELECT_TOP_PER_HEAD,
                             rotation_absorbed=True)
    assert p.q_mode == B.Q_NONE
    check_pack(p, ref)
    xhat16 = O.fp16_rne(O.rotate(lay["x"], O.round_rotation(Q, O.MODE_HEADWISE), O.MODE_HEADWISE))
    ref_rt = dict(ref); ref_rt["mode"] = O.MODE_NONE          # same stored layer, no run-time rotation
    check_output(run_gpu(p, xhat16), xhat16, None, ref_rt)
    p.free()


def test_device_rotation_packs_the_same_bits_as_the_host_path():
    """Dense rotations of D >= 1024 are multiplied into the weight on the GPU (fp64 FMA chain, one
    rounding to fp16); the host path and the oracle must give the same stored arrays."""
    print("case device rotation", flush=True)
    lay, Q, lam = make_case(0, 4, 1024, 300, 64, O.MODE_FULL)
    ref = O.pack(lay["W"], Q, lam, 128, 3, O.MODE_FULL)
    p_dev = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 3, B.Q_FULL)
    p_host = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 3, B.Q_FULL, host_only=True)
    check_pack(p_dev, ref)
    check_pack(p_host, ref)
    p_dev.free(); p_host.free()


def test_headwise_device_rotation_packs_the_same_bits_as_the_host_path():
    """Block-diagonal rotations of layers with at least 2^20 weights are multiplied in on the GPU too."""
    print("case device rotation head-wise", flush=True)
    lay, Q, lam = make_case(3, 4, 1024, 1030, 300, O.MODE_HEADWISE)
    ref = O.pack(lay["W"], Q, lam, 128, 4, O.MODE_HEADWISE)
    p_dev = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 4, B.Q_HEADWISE)
    p_host = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 4, B.Q_HEADWISE, host_only=True)
    check_pack(p_dev, ref)
    check_pack(p_host, ref)
    check_output(run_gpu(p_dev, lay["x"]), lay["x"], Q, ref)
    p_dev.free(); p_host.free()


@pytest.mark.parametrize("D,n_cal", [(256, 512), (1024, 700)])
def test_pca_headwise_on_gpu_against_oracle(D, n_cal):
    """Calibration on the GPU (one-sided Jacobi per head) against the oracle's PCA of the
    same fp16 activations: eigenvalues to 1e-10, eigenvectors to fp32 resolution, orthogonality,
    and the packed layer built from the GPU rotation equals the one built from the oracle's."""
    print(f"case gpu pca D={D}", flush=True)
    lay = synth.make_layer(55, 8, D, 64, n_cal)
    X16 = lay["X_cal"].astype(np.float16)
    Qo, lo = O.pca_headwise(X16, 128, "jacobi")
    xd = torch.from_numpy(X16).cuda()
    Qg, lg = B.rosaq_pca_headwise(xd.data_ptr(), n_cal, D, xd.stride(0))
    assert np.all(np.diff(lg.reshape(-1, 128), axis=1) <= 0) and np.all(lg >= 0)
    assert np.max(np.abs(lg - lo)) <= 1e-10 * lo.max()
    for h in range(D // 128):
        q = Qg[h].astype(np.float64)
        assert np.max(np.abs(q.T @ q - np.eye(128))) <= 2e-6
        big = np.argmax(np.abs(q), axis=0)
        assert np.all(q[big, np.arange(128)] > 0)                       # sign convention
        # well separated eigenvalues: same vectors up to sign (near-equal magnitudes may flip it)
        gap = np.minimum(np.abs(np.diff(lo[h * 128:(h + 1) * 128], prepend=np.inf)),
                         np.abs(np.diff(lo[h * 128:(h + 1) * 128], append=-np.inf)))
        ok = gap > 1e-5 * lo[h * 128]
        d = np.minimum(np.abs(q - Qo[h]).max(axis=0), np.abs(q + Qo[h]).max(axis=0))
        assert np.max(d[ok]) <= 2e-6, np.max(d[ok])
        # C_h = Q Lambda Q^T
        Ch = O.second_moment(X16[:, h * 128:(h + 1) * 128])
        assert np.linalg.norm(q @ np.diag(lg[h * 128:(h + 1) * 128]) @ q.T - Ch) <= 1e-5 * np.linalg.norm(Ch)
    # the GPU rotation drives the rest of the pipeline like any other Q, lambda
    ref = O.pack(lay["W"], Qg, lg, 128, 4, O.MODE_HEADWISE)
    p = B.rosaq_pack_weights(lay["W"], Qg, lg, 128, 4, B.Q_HEADWISE)
    check_pack(p, ref)
    check_output(run_gpu(p, lay["x"]), lay["x"], Qg, ref)
    p.free()


@pytest.mark.parametrize("mode,bits,M,D,N,K", [(O.MODE_HEADWISE, 4, 256, 512, 384, 128), (O.MODE_NONE, 3, 130, 384, 200, 128),
                                               (O.MODE_FULL, 4, 200, 1024, 256, 0), (O.MODE_HEADWISE, 3, 520, 256, 144, 128)])
def test_many_row_groups(mode, bits, M, D, N, K):
    """More than four row groups per channel chunk: the workgroups of an XCD are laid out in blocks of
    8 chunks x 4 row groups; ragged M and N."""
    print(f"case rows mode={mode} bits={bits} M={M} D={D} N={N} K={K}", flush=True)
    lay, Q, lam = make_case(300 + M, M, D, N, 300, mode)
    ref = O.pack(lay["W"], Q, lam, K, bits, mode)
    p = B.rosaq_pack_weights(lay["W"], Q, lam, K, bits, mode)
    for mt in (0, 1, 2):
        B.rosaq_tune("mt", mt)
        try:
            check_output(run_gpu(p, lay["x"]), lay["x"], Q, ref)
        finally:
            B.rosaq_tune("mt", 0)
    p.free()


def test_batch_with_many_row_groups():
    """Three layers in one launch at M = 300 (five row groups of 64): segment lookup and block order together."""
    from paper_2506_13472_amd import torch_glue as T
    print("case batch rows", flush=True)
    M, D = 300, 512
    lay, Q, lam = make_case(23, M, D, 200, 300, O.MODE_HEADWISE)
    Ws = [lay["W"], synth.make_weight(33, 96, D), synth.make_weight(34, 330, D)]
    refs = [O.pack(W, Q, lam, 128, 4, O.MODE_HEADWISE) for W in Ws]
    ps = [B.rosaq_pack_weights(W, Q, lam, 128, 4, B.Q_HEADWISE) for W in Ws]
    ys = T.linear_batch(ps, torch.from_numpy(lay["x"]).cuda())
    torch.cuda.synchronize()
    for y, p, ref in zip(ys, ps, refs):
        yh = y.cpu().numpy()
        check_output(yh, lay["x"], Q, ref)
        assert np.array_equal(run_gpu(p, lay["x"]).view(np.uint16), yh.view(np.uint16))
        p.free()


def test_prefill_sized_call():
    """M = 2048: 32 row groups per channel chunk."""
    M, D, N = 2048, 256, 2048
    print(f"case prefill M={M} D={D} N={N}", flush=True)
    lay, Q, lam = make_case(411, M, D, N, 300, O.MODE_HEADWISE)
    ref = O.pack(lay["W"], Q, lam, 128, 4, O.MODE_HEADWISE)
    p = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 4, B.Q_HEADWISE)
    check_output(run_gpu(p, lay["x"]), lay["x"], Q, ref)
    p.free()


def test_hipgraph_replays_match_eager_calls():
    """The run-time entry points allocate nothing and record only kernel launches, so they can be
    captured: every replay of the graph, with eager work in between, reproduces the eager bits."""
    from paper_2506_13472_amd import torch_glue as T
    print("case graph", flush=True)
    M, D = 64, 512
    lay, Q, lam = make_case(21, M, D, 200, 300, O.MODE_HEADWISE)
    Ws = [lay["W"], synth.make_weight(31, 96, D), synth.make_weight(32, 330, D)]
    ps = [B.rosaq_pack_weights(W, Q, lam, 128, 4, B.Q_HEADWISE) for W in Ws]
    lam_n = np.abs(lay["X_cal"]).mean(axis=0)
    pn = B.rosaq_pack_weights(Ws[1], None, lam_n, 128, 3, B.Q_NONE)
    x = torch.from_numpy(lay["x"]).cuda()
    ws = T.alloc_workspace(ps[0], M)
    ys = [torch.zeros((M, p.N), dtype=torch.float16, device="cuda") for p in ps]
    yn = torch.zeros((M, pn.N), dtype=torch.float16, device="cuda")
    eager = [y.cpu().numpy().copy() for y in T.linear_batch(ps, x)] + [T.linear(pn, x).cpu().numpy().copy()]
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        def calls():
            T.linear_batch(ps, x, ys, ws)
            T.linear(pn, x, yn, ws)
        calls()
        stream.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            calls()
        for rep in range(3):
            for y in ys + [yn]:
                y.zero_()
            T.linear(ps[0], x)                       # unrelated eager work between replays
            stream.synchronize()
            g.replay()
            stream.synchronize()
            for y, e in zip(ys + [yn], eager):
                assert np.array_equal(y.cpu().numpy().view(np.uint16), e.view(np.uint16)), rep
    for p in ps + [pn]:
        p.free()


def test_seeded_random_shapes_modes_and_tiles():
    """A seeded sweep over M, D, N, K, bits, rotation mode and forced tile shapes (ragged everything):
    stored arrays bit-exact, outputs within tolerance."""
    rng = np.random.default_rng(12345)
    tiles = [(0, 0, 0, 0), (1, 1, 8, 2), (1, 1, 16, 1), (1, 2, 8, 3), (1, 4, 8, 2), (2, 1, 8, 2), (2, 2, 8, 1),
             (2, 2, 8, 3), (2, 4, 8, 2), (4, 1, 8, 1), (4, 2, 8, 2), (4, 4, 8, 1), (4, 4, 4, 2), (2, 4, 4, 3),
             (4, 3, 8, 1), (2, 3, 8, 2), (2, 6, 8, 1), (2, 6, 8, 2), (4, 6, 4, 1), (1, 2, 16, 2), (2, 1, 16, 1)]
    for it in range(32):
        mode = int(rng.integers(0, 3))
        bits = int(rng.choice([3, 4]))
        D = int(rng.choice([128, 256, 384, 512, 768, 1024]))
        K = int(rng.choice([k for k in (0, 128, 256, D) if k <= D]))
        N = int(rng.integers(1, 700))
        M = int(rng.choice([1, 2, 7, 16, 17, 33, 64, 65, 100, 130, 257, 300]))
        mt, nt, wpb, depth = tiles[int(rng.integers(0, len(tiles)))]
        print(f"case {it}: mode={mode} bits={bits} M={M} D={D} N={N} K={K} tile=({mt},{nt},{wpb},{depth})", flush=True)
        lay = synth.make_layer(1000 + it, M, D, N, 200)
        if mode == O.MODE_NONE:
            Q, lam = None, np.abs(lay["X_cal"]).mean(axis=0)
        elif mode == O.MODE_FULL:
            Q, lam = synth.random_orthogonal_dense(it, D), synth.descending_spectrum(it + 1, D, 1)
        else:
            Q, lam = synth.random_orthogonal_blocks(it, D // 128), synth.descending_spectrum(it + 1, D, D // 128)
        ref = O.pack(lay["W"], Q, lam, K, bits, mode)
        p = B.rosaq_pack_weights(lay["W"], Q, lam, K, bits, mode)
        check_pack(p, ref)
        for k, v in (("mt", mt), ("nt", nt), ("wpb", wpb), ("depth", depth)):
            B.rosaq_tune(k, v)
        try:
            check_output(run_gpu(p, lay["x"]), lay["x"], Q, ref)
        finally:
            for k in ("mt", "nt", "wpb", "depth"):
                B.rosaq_tune(k, 0)
            p.free()



def test_seeded_random_batches_and_tiles():
    """A seeded sweep over batches of 2-4 layers of random widths, with forced tile shapes: every layer of
    the launch within tolerance of the oracle, nothing written outside a layer's output."""
    from paper_2506_13472_amd import torch_glue as T
    rng = np.random.default_rng(777)
    tiles = [(0, 0, 0, 0), (1, 1, 8, 2), (1, 2, 8, 2), (1, 4, 8, 2), (2, 2, 8, 1), (2, 4, 8, 2), (4, 2, 8, 2),
             (4, 4, 8, 1), (4, 3, 8, 1), (2, 3, 8, 2), (2, 6, 8, 1), (4, 6, 4, 1), (1, 1, 16, 1), (4, 4, 4, 2)]
    for it in range(20):
        mode = int(rng.integers(0, 3))
        bits = int(rng.choice([3, 4]))
        D = int(rng.choice([256, 384, 512, 768]))
        K = int(rng.choice([0, 128, 256]))
        Ns = [int(rng.integers(1, 400)) for _ in range(int(rng.integers(2, 5)))]
        M = int(rng.choice([1, 5, 16, 31, 64, 70, 129, 260]))
        mt, nt, wpb, depth = tiles[int(rng.integers(0, len(tiles)))]
        print(f"case {it}: mode={mode} bits={bits} M={M} D={D} Ns={Ns} K={K} tile=({mt},{nt},{wpb},{depth})", flush=True)
        x = synth.make_activations(3000 + it, M, D)
        if mode == O.MODE_NONE:
            Q, lam = None, synth.descending_spectrum(it + 1, D, 1)
        elif mode == O.MODE_FULL:
            Q, lam = synth.random_orthogonal_dense(it, D), synth.descending_spectrum(it + 1, D, 1)
        else:
            Q, lam = synth.random_orthogonal_blocks(it, D // 128), synth.descending_spectrum(it + 1, D, D // 128)
        Ws = [synth.make_weight(4000 + 10 * it + i, N, D) for i, N in enumerate(Ns)]
        refs = [O.pack(W, Q, lam, K, bits, mode) for W in Ws]
        ps = [B.rosaq_pack_weights(W, Q, lam, K, bits, mode) for W in Ws]
        ys = [torch.full((M, N + 5), -3.0, dtype=torch.float16, device="cuda") for N in Ns]
        for k, v in (("mt", mt), ("nt", nt), ("wpb", wpb), ("depth", depth)):
            B.rosaq_tune(k, v)
        try:
            T.linear_batch(ps, torch.from_numpy(x).cuda(), [y[:, :N] for y, N in zip(ys, Ns)])
            torch.cuda.synchronize()
        finally:
            for k in ("mt", "nt", "wpb", "depth"):
                B.rosaq_tune(k, 0)
        for y, N, ref in zip(ys, Ns, refs):
            yh = y.cpu().numpy()
            assert np.all(yh[:, N:] == -3.0)
            check_output(yh[:, :N], x, Q, ref)
        for p in ps:
            p.free()


@pytest.mark.parametrize("rot_mt", [2, 4])
def test_dense_rotation_with_48_channel_tiles(rot_mt):
    """The all-fp16 rotation launch with 48-channel tiles on a width they do not divide (40 channel
    tiles): the last chunk runs past the end and the rotated activations still come out right."""
    print(f"case dense rotation rot_mt={rot_mt} rot_nt=3", flush=True)
    lay, Q, lam = make_case(61, 50, 640, 200, 300, O.MODE_FULL)
    ref = O.pack(lay["W"], Q, lam, 128, 4, O.MODE_FULL)
    p = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 4, B.Q_FULL)
    y_default = run_gpu(p, lay["x"])
    B.rosaq_tune("rot_mt", rot_mt); B.rosaq_tune("rot_nt", 3); B.rosaq_tune("rot_splits", 1)
    try:
        y = run_gpu(p, lay["x"])
    finally:
        B.rosaq_tune("rot_mt", 0); B.rosaq_tune("rot_nt", 0); B.rosaq_tune("rot_splits", 0)
    check_output(y, lay["x"], Q, ref)
    check_output(y_default, lay["x"], Q, ref)
    p.free()


@pytest.mark.parametrize("M,D,slabs", [(64, 1024, 8), (17, 1024, 3), (50, 640, 16), (33, 640, 7), (64, 2048, 2),
                                       (48, 384, 12), (64, 2048, 4)])
def test_dense_rotation_as_slabs_of_the_contraction(M, D, slabs):
    """The alternative rotation of calls of 17 to 64 rows through slabs of the contraction and a
    summing launch (ragged slabs, a slab of one k-step, 16 and 32 k-steps per slab): against the
    oracle, against the single-launch rotation, and twice for bit-identical results."""
    print(f"case slab rotation M={M} D={D} slabs={slabs}", flush=True)
    lay, Q, lam = make_case(67, M, D, 136, 300, O.MODE_FULL)
    ref = O.pack(lay["W"], Q, lam, 128, 4, O.MODE_FULL)
    p = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 4, B.Q_FULL)
    B.rosaq_tune("rot_splits", 1)
    try:
        y_single = run_gpu(p, lay["x"])
        B.rosaq_tune("rot_splits", slabs)
        y = run_gpu(p, lay["x"])
        y_again = run_gpu(p, lay["x"])
    finally:
        B.rosaq_tune("rot_splits", 0)
    check_output(y, lay["x"], Q, ref)
    assert np.array_equal(y.view(np.uint16), y_again.view(np.uint16))
    # the two routes add the same fp32 products in different orders
    assert np.linalg.norm(y.astype(np.float64) - y_single) <= 1e-3 * np.linalg.norm(y_single.astype(np.float64))
    p.free()


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("mode,N,D,K,rule", [(O.MODE_HEADWISE, 200, 512, 128, O.RULE_TOP), (O.MODE_FULL, 130, 384, 0, O.RULE_TOP),
                                             (O.MODE_NONE, 48, 256, 256, O.RULE_TOP), (O.MODE_HEADWISE, 96, 512, 256, O.RULE_TOP_AND_BOTTOM),
                                             (O.MODE_FULL, 260, 512, 128, O.RULE_BOTTOM)])
def test_device_pack_equals_host_pack_and_oracle(bits, mode, N, D, K, rule):
    """The offline step on the GPU (rotation, quantiser, images) against the oracle's canonical arrays,
    and the fragment images it leaves in device memory against the ones the host builder makes from
    those arrays: bit for bit, padding rows included."""
    print(f"case device pack bits={bits} mode={mode} N={N} D={D} K={K} rule={rule}", flush=True)
    lay, Q, lam = make_case(200 + N, 8, D, N, 300, mode)
    ref = O.pack(lay["W"], Q, lam, K, bits, mode, rule=rule)
    p = B.rosaq_pack_weights(lay["W"], Q, lam, K, bits, mode, select_rule=rule)
    h = B.rosaq_pack_weights(lay["W"], Q, lam, K, bits, mode, select_rule=rule, host_only=True)
    try:
        check_pack(p, ref)
        check_pack(h, ref)
        for which in (0, 1):
            dev_img = B.rosaq_packed_image(p, which + 2)
            host_img = B.rosaq_packed_image(h, which)
            assert dev_img.shape == host_img.shape and np.array_equal(dev_img, host_img), which
    finally:
        p.free()
        h.free()


def test_device_pack_strided_weights_and_overflow():
    """ldw > D goes through a pitched upload; a rotation that overflows fp16 is reported."""
    lay, Q, lam = make_case(77, 8, 256, 40, 300, O.MODE_FULL)
    Wp = np.zeros((40, 320), np.float16)
    Wp[:, :256] = lay["W"]
    ref = O.pack(lay["W"], Q, lam, 128, 4, O.MODE_FULL)
    p = B.rosaq_pack_weights(Wp, Q, lam, 128, 4, B.Q_FULL, ldw=320, in_features=256)
    try:
        check_pack(p, ref)
    finally:
        p.free()
    with pytest.raises(B.RosaqError) as e:
        B.rosaq_pack_weights(lay["W"], Q * np.float32(1e7), lam, 128, 4, B.Q_FULL)
    assert B.ERR_NAMES[e.value.code] == "NONFINITE"


@pytest.mark.parametrize("D,n_cal,solver", [(256, 512, "jacobi"), (256, 100, "jacobi"), (1024, 700, "lapack")])
def test_pca_full_on_gpu_against_oracle(D, n_cal, solver):
    """Layer-wise PCA on the GPU (one-sided Jacobi on the calibration activations) against the oracle's
    PCA of the second moment of the same fp16 activations: eigenvalues to 1e-10 of the largest one,
    eigenvectors of well separated eigenvalues to fp32 resolution, orthogonality, reconstruction --
    with more rows than channels and with fewer (a null space of any orthonormal completion)."""
    print(f"case gpu pca full D={D} n_cal={n_cal}", flush=True)
    lay = synth.make_layer(56, 8, D, 64, n_cal)
    X16 = lay["X_cal"].astype(np.float16)
    Qo, lo = O.pca_full(X16, solver)
    xd = torch.from_numpy(X16).cuda()
    Qg, lg = B.rosaq_pca_full(xd.data_ptr(), n_cal, D, xd.stride(0))
    assert np.all(np.diff(lg) <= 0) and np.all(lg >= 0)
    assert np.max(np.abs(lg - lo)) <= 1e-10 * lo.max()
    q = Qg.astype(np.float64)
    assert np.max(np.abs(q.T @ q - np.eye(D))) <= 4e-6
    big = np.argmax(np.abs(q), axis=0)
    assert np.all(q[big, np.arange(D)] > 0)                          # sign convention
    gap = np.minimum(np.abs(np.diff(lo, prepend=np.inf)), np.abs(np.diff(lo, append=-np.inf)))
    ok = gap > 1e-5 * lo[0]
    assert ok.sum() >= min(n_cal, D) // 4
    d = np.minimum(np.abs(q - Qo).max(axis=0), np.abs(q + Qo).max(axis=0))
    assert np.max(d[ok]) <= 5e-6, np.max(d[ok])
    C = O.second_moment(X16)
    assert np.linalg.norm(q @ np.diag(lg) @ q.T - C) <= 1e-5 * np.linalg.norm(C)
    # the rotated calibration set has a diagonal second moment (Eq. 4)
    R = O.second_moment(X16.astype(np.float64) @ q)
    assert np.linalg.norm(R - np.diag(np.diag(R))) <= 1e-5 * np.linalg.norm(C)
    # the GPU rotation drives the rest of the pipeline like any other Q, lambda
    ref = O.pack(lay["W"], Qg, lg, 128, 4, O.MODE_FULL)
    p = B.rosaq_pack_weights(lay["W"], Qg, lg, 128, 4, B.Q_FULL)
    check_pack(p, ref)
    check_output(run_gpu(p, lay["x"]), lay["x"], Qg, ref)
    p.free()
