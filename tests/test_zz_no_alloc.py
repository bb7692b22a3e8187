"""The entry point that allocates nothing (library-owned static scratch) against rosaq_linear_headwise."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import rosaq_oracle as O
from paper_2506_13472_amd import binding as B
from paper_2506_13472_amd import torch_glue as T
from test_gpu_parity import check_output, make_case

pytestmark = pytest.mark.gpu


def _both(p, x16, splits):
    """(static entry point, workspace entry point) outputs for the same call."""
    M = x16.shape[0]
    x = torch.from_numpy(x16).cuda()
    y_ws = torch.full((M, p.N), 7.0, dtype=torch.float16, device="cuda")
    y_st = torch.full((M, p.N), -7.0, dtype=torch.float16, device="cuda")
    B.rosaq_tune("splits", splits)
    try:
        # the same number of bytes the static call will use, so both take the same launch shape
        nbytes = min(B.rosaq_workspace_bytes(p, M), 8 << 20)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        sp = T.current_stream_ptr()
        B.rosaq_linear_headwise(p, x.data_ptr(), M, x.stride(0), y_ws.data_ptr(), y_ws.stride(0),
                                ws.data_ptr(), ws.numel(), sp)
        B.rosaq_linear_headwise_static(p, x.data_ptr(), M, x.stride(0), y_st.data_ptr(), y_st.stride(0), sp)
        torch.cuda.synchronize()
    finally:
        B.rosaq_tune("splits", 0)
    return y_st.cpu().numpy(), y_ws.cpu().numpy()


@pytest.mark.parametrize("splits", [0, 3])
def test_static_scratch_entry_point_matches_workspace_entry_point(splits):
    print(f"case no-alloc splits={splits}", flush=True)
    lay, Q, lam = make_case(41, 64, 1024, 232, 512, O.MODE_HEADWISE)
    ref = O.pack(lay["W"], Q, lam, 128, 4, O.MODE_HEADWISE)
    p = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 4, B.Q_HEADWISE)
    try:
        # two calls in a row on the shared array, the second with a smaller input
        for M in (64, 5):
            x = lay["x"][:M]
            y_st, y_ws = _both(p, x, splits)
            assert np.array_equal(y_st.view(np.uint16), y_ws.view(np.uint16)), M
            check_output(y_st, x, Q, ref)
    finally:
        p.free()


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    print("case no-alloc limits", flush=True)
    lay, Q, lam = make_case(41, 64, 1024, 232, 512, O.MODE_HEADWISE)
    p = B.rosaq_pack_weights(lay["W"], Q, lam, 128, 4, B.Q_HEADWISE)
    pn = B.rosaq_pack_weights(lay["W"], None, lam, 128, 4, B.Q_NONE)
    try:
        x = torch.zeros((8192, 1024), dtype=torch.float16, device="cuda")
        y = torch.zeros((8192, 232), dtype=torch.float16, device="cuda")
        assert B.rosaq_workspace_bytes_min(p, 4096) > (8 << 20)
        with pytest.raises(B.RosaqError) as e:
            B.rosaq_linear_headwise_static(p, x.data_ptr(), 4096, 1024, y.data_ptr(), 232)
        assert B.ERR_NAMES[e.value.code] == "WORKSPACE"
        with pytest.raises(B.RosaqError) as e:
            B.rosaq_linear_headwise_static(pn, x.data_ptr(), 64, 1024, y.data_ptr(), 232)
        assert B.ERR_NAMES[e.value.code] == "MODE"
        with pytest.raises(B.RosaqError) as e:
            B.rosaq_linear_headwise_static(p, 0, 64, 1024, y.data_ptr(), 232)
        assert B.ERR_NAMES[e.value.code] == "NULL"
    finally:
        p.free()
        pn.free()
