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
