"""GPU parity of the fused gate / up launch with the silu * up epilogue against the oracle."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import rosaq_oracle as O
from paper_2506_13472_amd import binding as B
from paper_2506_13472_amd import torch_glue as T
from test_gpu_parity import MAX_TOL, make_case

pytestmark = pytest.mark.gpu


def check_swiglu(y, x16, Q, pg, pu):
    """out = silu(g) u.  With |dg| <= tol scale_g and |du| <= tol scale_u (the linear layer's bound) and
    |silu'| <= 1.1:  |d out| <= 1.1 |u| |dg| + |silu(g)| |du| + the final fp16 rounding 2^-11 |out|."""
    g, u = O.linear_ref(x16, Q, pg), O.linear_ref(x16, Q, pu)
    ref = O.silu(g) * u
    bound = (1.1 * np.abs(u) * MAX_TOL * O.tolerance_scale(x16, pg) +
             np.abs(O.silu(g)) * MAX_TOL * O.tolerance_scale(x16, pu) + 2.0 ** -10 * np.abs(ref) + 1e-7)
    err = np.abs(y.astype(np.float64) - ref)
    fro = float(np.linalg.norm(err) / np.linalg.norm(ref))
    print(f"  swiglu max err/bound={float(np.max(err / bound)):.3e} fro={fro:.3e}", flush=True)
    assert np.all(np.isfinite(y))
    assert np.all(err <= bound)
    assert fro <= 2e-3


def run(pg, pu, x16):
    x = torch.from_numpy(x16).cuda()
    M = x.shape[0]
    y = torch.full((M, pg.N), 3.0, dtype=torch.float16, device="cuda")
    ws = T.alloc_workspace(pg, M)
    B.rosaq_linear_swiglu(pg, pu, x.data_ptr(), M, x.stride(0), y.data_ptr(), y.stride(0),
                          ws.data_ptr(), ws.numel(), T.current_stream_ptr())
    torch.cuda.synchronize()
    return y.cpu().numpy()


@pytest.mark.parametrize("mode,bits,M,D,N", [(O.MODE_FULL, 4, 64, 512, 200), (O.MODE_HEADWISE, 3, 37, 512, 96),
                                             (O.MODE_NONE, 4, 5, 256, 130), (O.MODE_FULL, 4, 150, 384, 72)])
def test_swiglu_small_shapes(mode, bits, M, D, N):
    print(f"case swiglu mode={mode} bits={bits} M={M} D={D} N={N}", flush=True)
    lay, Q, lam = make_case(300 + M, M, D, N, 300, mode)
    Wu = (lay["W"][::-1] * np.float16(1.5)).astype(np.float16)
    refs = [O.pack(W, Q, lam, 128, bits, mode) for W in (lay["W"], Wu)]
    ps = [B.rosaq_pack_weights(W, Q, lam, 128, bits, mode) for W in (lay["W"], Wu)]
    try:
        check_swiglu(run(ps[0], ps[1], lay["x"]), lay["x"], Q, refs[0], refs[1])
        for nt in (2, 4, 6, 3, 1):                       # odd tile counts fall back to an even one
            B.rosaq_tune("nt", nt)
            B.rosaq_tune("mt", 2 if nt in (3, 6) else 0)
            check_swiglu(run(ps[0], ps[1], lay["x"]), lay["x"], Q, refs[0], refs[1])
    finally:
        B.rosaq_tune("nt", 0)
        B.rosaq_tune("mt", 0)
        for p in ps:
            p.free()


def test_swiglu_rejects_layers_that_differ():
    lay, Q, lam = make_case(301, 8, 256, 64, 300, O.MODE_FULL)
    a = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 4, B.Q_FULL)
    b = B.rosaq_pack_weights(lay["W"][:48].copy(), Q, lam, 128, 4, B.Q_FULL)
    c = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 3, B.Q_FULL)
    try:
        for other in (b, c):
            with pytest.raises(B.RosaqError) as e:
                run(a, other, lay["x"])
            assert B.ERR_NAMES[e.value.code] == "MODE"
    finally:
        for p in (a, b, c):
            p.free()


def test_swiglu_7b_mlp_full_size():
    """4096 -> 11008, INT4, dense 4096 x 4096 rotation, M = 64: the launch of the decode step."""
    from paper_2506_13472_amd import synth
    print("case swiglu 7B gate/up", flush=True)
    D, N, M = 4096, 11008, 64
    Q = synth.random_orthogonal_dense(90, D)
    lam = synth.descending_spectrum(91, D, 1)
    x = synth.make_activations(92, M, D)
    Ws = [synth.make_weight(93 + j, N, D) for j in range(2)]
    refs = [O.pack(W, Q, lam, 128, 4, O.MODE_FULL) for W in Ws]
    ps = [B.rosaq_pack_weights(W, Q, lam, 128, 4, B.Q_FULL) for W in Ws]
    try:
        check_swiglu(run(ps[0], ps[1], x), x, Q, refs[0], refs[1])
    finally:
        for p in ps:
            p.free()


def run_two_calls(pg, pu, pd, x16):
    """silu(gate) * up into a row-major buffer, then the down projection as a call of its own."""
    x = torch.from_numpy(x16).cuda()
    M = x.shape[0]
    h = torch.empty((M, pg.N), dtype=torch.float16, device="cuda")
    ws = T.alloc_workspace(pg, M)
    B.rosaq_linear_swiglu(pg, pu, x.data_ptr(), M, x.stride(0), h.data_ptr(), h.stride(0),
                          ws.data_ptr(), ws.numel(), T.current_stream_ptr())
    y = T.linear(pd, h)
    torch.cuda.synchronize()
    return h.cpu().numpy(), y.cpu().numpy()


def run_mlp(pg, pu, pd, x16, ws_bytes=None):
    x = torch.from_numpy(x16).cuda()
    M = x.shape[0]
    y = torch.full((M, pd.N), 3.0, dtype=torch.float16, device="cuda")
    n = B.rosaq_workspace_bytes_mlp(pg, pu, pd, M) if ws_bytes is None else ws_bytes
    ws = torch.full((n,), 0xA5, dtype=torch.uint8, device="cuda")     # tickets start out dirty
    B.rosaq_mlp_swiglu(pg, pu, pd, x.data_ptr(), M, x.stride(0), y.data_ptr(), y.stride(0),
                       ws.data_ptr(), ws.numel(), T.current_stream_ptr())
    torch.cuda.synchronize()
    return y.cpu().numpy()


@pytest.mark.parametrize("mode,bits,M,D,F,N,Kd", [(O.MODE_FULL, 4, 64, 512, 384, 200, 128),
                                                  (O.MODE_HEADWISE, 3, 37, 256, 256, 96, 128),
                                                  (O.MODE_NONE, 4, 5, 256, 640, 130, 0),
                                                  (O.MODE_FULL, 4, 150, 384, 1024, 72, 256)])
def test_mlp_block_equals_the_two_calls_and_the_oracle(mode, bits, M, D, F, N, Kd):
    """rosaq_mlp_swiglu writes the gated product straight into the down projection's input fragments:
    bit for bit the result of rosaq_linear_swiglu followed by rosaq_linear, and within the linear
    layer's tolerance of the oracle's down projection of the fp16 intermediate the GPU produced."""
    print(f"case mlp block mode={mode} bits={bits} M={M} D={D} F={F} N={N}", flush=True)
    lay, Q, lam = make_case(320 + M, M, D, F, 300, mode)
    Wu = (lay["W"][::-1] * np.float16(1.5)).astype(np.float16)
    down = synth_down(321 + M, N, F)
    lam_d = np.abs(np.random.default_rng(5).standard_normal(F)) + 0.1      # salient channels scattered
    ref_d = O.pack(down, None, lam_d, Kd, bits, O.MODE_NONE)
    pg, pu = (B.rosaq_pack_weights(W, Q, lam, 128, bits, mode) for W in (lay["W"], Wu))
    pd = B.rosaq_pack_weights(down, None, lam_d, Kd, bits, B.Q_NONE)
    try:
        h, y2 = run_two_calls(pg, pu, pd, lay["x"])
        y = run_mlp(pg, pu, pd, lay["x"])
        assert np.array_equal(y.view(np.uint16), y2.view(np.uint16))
        # the down launch cut over three workgroups per tile (the gated launch never is): another
        # summation order, held to the oracle only
        B.rosaq_tune("splits", 3)
        try:
            y_split = run_mlp(pg, pu, pd, lay["x"])
        finally:
            B.rosaq_tune("splits", 0)
        from test_gpu_parity import check_output
        check_output(y, h, None, ref_d)
        check_output(y_split, h, None, ref_d)
    finally:
        for p in (pg, pu, pd):
            p.free()


def synth_down(seed, N, F):
    from paper_2506_13472_amd import synth
    return synth.make_weight(seed, N, F)


def test_mlp_block_rejects_what_it_cannot_chain():
    lay, Q, lam = make_case(340, 8, 256, 256, 300, O.MODE_FULL)
    g = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 4, B.Q_FULL)
    d_rot = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 4, B.Q_FULL)            # rotates at run time
    d_narrow = B.rosaq_pack_weights(lay["W"][:, :128].copy(), None, lam[:128], 0, 4, B.Q_NONE)
    try:
        for down, code in ((d_rot, "MODE"), (d_narrow, "SHAPE")):
            with pytest.raises(B.RosaqError) as e:
                run_mlp(g, g, down, lay["x"], ws_bytes=1 << 24)
            assert B.ERR_NAMES[e.value.code] == code
            assert B.rosaq_workspace_bytes_mlp(g, g, down, 8) == 0
    finally:
        for p in (g, d_rot, d_narrow):
            p.free()


def test_mlp_block_7b_full_size():
    """The FFN of a 7B-shaped decode layer at M = 64: 4096 -> 11008 (dense rotation) -> 4096 (no rotation)."""
    from paper_2506_13472_amd import synth
    print("case mlp block 7B", flush=True)
    D, F, M = 4096, 11008, 64
    Q = synth.random_orthogonal_dense(90, D)
    lam = synth.descending_spectrum(91, D, 1)
    x = synth.make_activations(92, M, D)
    Wg, Wu = (synth.make_weight(93 + j, F, D) for j in range(2))
    Wd = synth.make_weight(96, D, F)
    lam_d = np.abs(np.random.default_rng(6).standard_normal(F)) + 0.1
    pg, pu = (B.rosaq_pack_weights(W, Q, lam, 128, 4, B.Q_FULL) for W in (Wg, Wu))
    pd = B.rosaq_pack_weights(Wd, None, lam_d, 128, 4, B.Q_NONE)
    try:
        h, y2 = run_two_calls(pg, pu, pd, x)
        y = run_mlp(pg, pu, pd, x)
        assert np.all(np.isfinite(y))
        assert np.array_equal(y.view(np.uint16), y2.view(np.uint16))
    finally:
        for p in (pg, pu, pd):
            p.free()
