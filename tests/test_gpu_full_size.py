"""GPU parity at the full sizes of the MLP workloads (INT3 7B MLP, INT4 13B MLP sweep).

The dense rotations are seeded random orthogonal matrices (a PCA of an 11008^2 or 13824^2
second moment takes minutes; Q and the eigenvalues are inputs of the library, and parity does
not depend on where they come from).  Down projections keep the full contraction length and a
512-row sample of the output channels, which the oracle evaluates exactly.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import rosaq_oracle as O
from paper_2506_13472_amd import binding as B
from paper_2506_13472_amd import synth
from test_gpu_parity import check_output, check_pack, run_gpu

pytestmark = pytest.mark.gpu


def _case(seed, D, N, bits):
    W = synth.make_weight(seed, N, D)
    Q = synth.random_orthogonal_dense(seed + 1, D)
    lam = synth.descending_spectrum(seed + 2, D, 1)
    ref = O.pack(W, Q, lam, 128, bits, O.MODE_FULL)
    p = B.rosaq_pack_weights(W, Q, lam, 128, bits, B.Q_FULL)
    check_pack(p, ref)
    return Q, ref, p


def test_7b_mlp_gate_int3_full_rotation():
    print("case 7B gate/up 4096->11008 INT3", flush=True)
    Q, ref, p = _case(40, 4096, 11008, 3)
    x = synth.make_activations(41, 64, 4096)
    check_output(run_gpu(p, x), x, Q, ref)
    p.free()


def test_7b_mlp_down_int3_full_rotation_sampled_rows():
    print("case 7B down 11008->(512 of 4096) INT3", flush=True)
    Q, ref, p = _case(50, 11008, 512, 3)
    x = synth.make_activations(51, 64, 11008)
    check_output(run_gpu(p, x), x, Q, ref)
    p.free()


def test_13b_mlp_up_int4_m_sweep():
    print("case 13B up 5120->13824 INT4, M in 1,16,64,256", flush=True)
    Q, ref, p = _case(60, 5120, 13824, 4)
    for M in (1, 16, 64, 256):
        print(f"  M={M}", flush=True)
        x = synth.make_activations(61 + M, M, 5120)
        check_output(run_gpu(p, x), x, Q, ref)
    p.free()


def test_13b_mlp_down_int4_sampled_rows():
    print("case 13B down 13824->(512 of 5120) INT4", flush=True)
    Q, ref, p = _case(70, 13824, 512, 4)
    for M in (1, 64, 256):
        x = synth.make_activations(71 + M, M, 13824)
        check_output(run_gpu(p, x), x, Q, ref)
    p.free()


def test_7b_decode_layer_mlp_int4_gate_up_batch_and_unrotated_down():
    """The MLP calls of the 7B decode workload: gate and up (4096 -> 11008, INT4) share one dense
    rotation and go through one batched launch; down (11008 -> 4096, INT4) is not rotated, its
    salient channels chosen by activation magnitude."""
    from paper_2506_13472_amd import torch_glue as T
    print("case 7B decode MLP INT4: gate/up batch + down", flush=True)
    D, F, M = 4096, 11008, 64
    Q = synth.random_orthogonal_dense(81, D)
    lam = synth.descending_spectrum(82, D, 1)
    Ws = [synth.make_weight(83, F, D), synth.make_weight(84, F, D)]
    refs = [O.pack(W, Q, lam, 128, 4, O.MODE_FULL) for W in Ws]
    ps = [B.rosaq_pack_weights(W, Q, lam, 128, 4, B.Q_FULL) for W in Ws]
    x = synth.make_activations(85, M, D)
    ys = T.linear_batch(ps, torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    for y, p, ref in zip(ys, ps, refs):
        check_pack(p, ref)
        check_output(y.cpu().numpy(), x, Q, ref)
        p.free()
    Wd = synth.make_weight(86, 1024, F)               # 1024 of the 4096 output channels
    xd = synth.make_activations(87, M, F)
    lam_d = np.abs(synth.make_activations(88, 512, F).astype(np.float64)).mean(axis=0)
    ref = O.pack(Wd, None, lam_d, 128, 4, O.MODE_NONE)
    p = B.rosaq_pack_weights(Wd, None, lam_d, 128, 4, B.Q_NONE)
    check_pack(p, ref)
    check_output(run_gpu(p, xd), xd, None, ref)
    p.free()


def test_7b_attention_qkv_batch_full_size():
    """The launch configuration the bench times: q, k, v (4096 -> 4096 each, INT4, K = 128) share one
    head-wise rotation and go through one rosaq_linear_batch call at M = 64."""
    from paper_2506_13472_amd import torch_glue as T
    from test_gpu_parity import make_case
    print("case 7B q/k/v batch full size", flush=True)
    lay, Q, lam = make_case(1, 64, 4096, 4096, 512, O.MODE_HEADWISE, solver="lapack")
    Ws = [lay["W"], synth.make_weight(91, 4096, 4096), synth.make_weight(92, 4096, 4096)]
    ps = [B.rosaq_pack_weights(W, Q, lam, 128, 4, B.Q_HEADWISE) for W in Ws]
    ys = T.linear_batch(ps, torch.from_numpy(lay["x"]).cuda())
    torch.cuda.synchronize()
    for W, y, p in zip(Ws, ys, ps):
        ref = O.pack(W, Q, lam, 128, 4, O.MODE_HEADWISE)
        check_pack(p, ref)
        check_output(y.cpu().numpy(), lay["x"], Q, ref)
        p.free()
