"""GPU parity of launches whose contraction is split over several workgroups per output tile
(fp32 partial tiles + tickets in the caller's workspace), against the CPU oracle."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import rosaq_oracle as O
from paper_2506_13472_amd import binding as B
from paper_2506_13472_amd import torch_glue as T
from test_gpu_parity import check_output, check_pack, make_case

pytestmark = pytest.mark.gpu


def _tune(**kw):
    for k, v in kw.items():
        B.rosaq_tune(k, v)


def _reset():
    _tune(mt=0, nt=0, wpb=0, depth=0, splits=0, rot_splits=0)


@pytest.mark.parametrize("splits", [2, 3, 5, 16])
@pytest.mark.parametrize("M,nt", [(64, 4), (33, 2), (20, 6), (7, 4), (1, 2)])
def test_split_launch_matches_oracle(splits, M, nt):
    """Head-wise layer, D = 1024 (4 fp16 k-steps + 7 groups: splits that get no unit at all included),
    N not a multiple of the chunk width, every split count and several tile widths."""
    print(f"case split={splits} M={M} nt={nt}", flush=True)
    lay, Q, lam = make_case(31, 64, 1024, 232, 512, O.MODE_HEADWISE)
    x = lay["x"][:M]
    ref = O.pack(lay["W"], Q, lam, 128, 4, O.MODE_HEADWISE)
    p = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 4, B.Q_HEADWISE)
    try:
        _tune(nt=nt, splits=splits)
        assert B.rosaq_launch_shape(M, 240, 1024, 4)[4] == splits
        xd = torch.from_numpy(x).cuda()
        ws = T.alloc_workspace(p, M)
        y0 = T.linear(p, xd, ws=ws)
        torch.cuda.synchronize()
        y0 = y0.cpu().numpy()
        check_output(y0, x, Q, ref)
        # the same workspace again (tickets must be back at zero) and bit-identical results
        for _ in range(3):
            y1 = T.linear(p, xd, ws=ws)
            torch.cuda.synchronize()
            assert np.array_equal(y1.cpu().numpy().view(np.uint16), y0.view(np.uint16))
    finally:
        _reset()
        p.free()


@pytest.mark.parametrize("mode,bits", [(O.MODE_NONE, 3), (O.MODE_FULL, 4)])
def test_split_launch_other_modes_and_dense_rotation_split(mode, bits):
    """INT3 without rotation, and a dense rotation that runs as two slabs of its contraction."""
    print(f"case split mode={mode} bits={bits}", flush=True)
    lay, Q, lam = make_case(32, 48, 512, 160, 300, mode)
    ref = O.pack(lay["W"], Q, lam, 128, bits, mode)
    p = B.rosaq_pack_weights(lay["W"], Q, lam, 128, bits, mode)
    check_pack(p, ref)
    try:
        for M in (48, 17, 3):
            _tune(splits=3, rot_splits=2)
            x = lay["x"][:M]
            y = T.linear(p, torch.from_numpy(x).cuda())
            torch.cuda.synchronize()
            check_output(y.cpu().numpy(), x, Q, ref)
    finally:
        _reset()
        p.free()


def test_split_batch_and_workspace_sizes():
    """Three layers in one split launch; a workspace with no room for partial tiles runs unsplit
    and gives the result of an unsplit launch."""
    print("case split batch", flush=True)
    M, D = 64, 512
    lay, Q, lam = make_case(33, M, D, 96, 512, O.MODE_HEADWISE)
    Ws = [synth_w for synth_w in (lay["W"], lay["W"][::-1].copy(), lay["W"][:80].copy())]
    refs = [O.pack(W, Q, lam, 128, 4, O.MODE_HEADWISE) for W in Ws]
    ps = [B.rosaq_pack_weights(W, Q, lam, 128, 4, B.Q_HEADWISE) for W in Ws]
    x = torch.from_numpy(lay["x"]).cuda()
    try:
        _tune(splits=4)
        full = B.rosaq_workspace_bytes_batch(ps, M)
        small = B.rosaq_workspace_bytes_min(ps[0], M)
        assert full > small
        ws = torch.empty(full, dtype=torch.uint8, device="cuda")
        ys = T.linear_batch(ps, x, ws=ws)
        torch.cuda.synchronize()
        for y, ref in zip(ys, refs):
            check_output(y.cpu().numpy(), lay["x"], Q, ref)
        ws_small = torch.empty(small, dtype=torch.uint8, device="cuda")
        ys_small = T.linear_batch(ps, x, ws=ws_small)
        _tune(splits=1)
        ys_unsplit = T.linear_batch(ps, x, ws=ws)
        torch.cuda.synchronize()
        for a, b in zip(ys_small, ys_unsplit):
            assert np.array_equal(a.cpu().numpy().view(np.uint16), b.cpu().numpy().view(np.uint16))
    finally:
        _reset()
        for p in ps:
            p.free()


def test_split_inside_a_captured_graph_replays():
    """The tickets return to zero at the end of every launch, so a captured call can be replayed."""
    print("case split graph", flush=True)
    lay, Q, lam = make_case(34, 64, 512, 128, 512, O.MODE_HEADWISE)
    ref = O.pack(lay["W"], Q, lam, 128, 4, O.MODE_HEADWISE)
    p = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 4, B.Q_HEADWISE)
    try:
        _tune(splits=4)
        x = torch.from_numpy(lay["x"]).cuda()
        y = torch.zeros((64, 128), dtype=torch.float16, device="cuda")
        ws = T.alloc_workspace(p, 64)
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            T.linear(p, x, y, ws)
            stream.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                T.linear(p, x, y, ws)
            for _ in range(4):
                y.zero_()
                g.replay()
                stream.synchronize()
                check_output(y.cpu().numpy(), lay["x"], Q, ref)
    finally:
        _reset()
        p.free()
