"""Host packer of the library against the oracle: bit-exact canonical arrays (no GPU)."""
import numpy as np
import pytest

from oracle import rosaq_oracle as O
from paper_2506_13472_amd import binding as B
from paper_2506_13472_amd import synth


def _compare(p, ref):
    got = B.rosaq_packed_export(p)
    for k in ("salient_idx", "W_S", "codes", "scales", "zeros"):
        a, b = got[k], ref[k]
        if a.dtype == np.float16:
            a, b = a.view(np.uint16), np.asarray(b, np.float16).view(np.uint16)
        assert a.shape == b.shape, k
        assert np.array_equal(a, b), f"{k}: {np.sum(a != b)} of {a.size} differ"


def rounding_margin(What):
    """Smallest distance of an fp64 rotated weight to an fp16 rounding midpoint, in
    units of the fp64 summation error of its dot product (D * 2^-53 * |value| scale).
    Two independent fp64 summations round to the same fp16 when this is large."""
    a = np.abs(What).ravel()
    a = a[a > 2.0 ** -14]
    e = np.floor(np.log2(a))
    ulp = 2.0 ** (e - 10)
    frac = a / ulp - np.floor(a / ulp)
    dist = np.abs(frac - 0.5) * ulp
    err = What.shape[1] * 2.0 ** -53 * np.maximum(a, 1e-30) * 4
    return float(np.min(dist / err))


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("N,D,K", [(40, 256, 128), (16, 128, 0), (24, 384, 384), (17, 512, 256)])
def test_mode_none_is_unconditionally_bit_exact(bits, N, D, K):
    lay = synth.make_layer(10 + bits, 4, D, N, 64)
    lam = np.abs(lay["X_cal"]).mean(axis=0)          # 'Mixed' baseline key: activation magnitude
    ref = O.pack(lay["W"], None, lam, K, bits, O.MODE_NONE)
    p = B.rosaq_pack_weights(lay["W"], None, lam, K, bits, B.Q_NONE, host_only=True)
    _compare(p, ref)


@pytest.mark.parametrize("bits", [4, 3])
def test_full_rotation_bit_exact(bits):
    lay = synth.make_layer(0, 4, 256, 48, 64)        # rank-deficient calibration (64 rows < D)
    Q, lam = O.pca_full(lay["X_cal"], "jacobi")
    Q32 = Q.astype(np.float32)
    ref = O.pack(lay["W"], Q32, lam, 128, bits, O.MODE_FULL)
    assert rounding_margin(ref["What"]) > 1e3
    p = B.rosaq_pack_weights(lay["W"], Q32, lam, 128, bits, B.Q_FULL, host_only=True)
    _compare(p, ref)


@pytest.mark.parametrize("bits", [4, 3])
def test_headwise_rotation_bit_exact(bits):
    lay = synth.make_layer(1, 4, 512, 40, 512)
    Qb, lam = O.pca_headwise(lay["X_cal"], 128, "jacobi")
    Qb32 = Qb.astype(np.float32)
    ref = O.pack(lay["W"], Qb32, lam, 128, bits, O.MODE_HEADWISE)
    assert rounding_margin(ref["What"]) > 1e3
    p = B.rosaq_pack_weights(lay["W"], Qb32, lam, 128, bits, B.Q_HEADWISE, host_only=True)
    _compare(p, ref)
    # global top-K over all heads: a prefix of each head
    sal = B.rosaq_packed_export(p)["salient_idx"]
    for h in range(4):
        loc = sal[(sal >= 128 * h) & (sal < 128 * (h + 1))] - 128 * h
        assert loc.tolist() == list(range(len(loc)))


def test_strided_weight_and_unsorted_eigenvalues():
    rng = np.random.default_rng(3)
    N, D = 20, 256
    big = (rng.standard_normal((N, D + 40)) * 0.03).astype(np.float16)
    lam = rng.random(D)
    lam[10] = lam[200] = lam.max()                   # a tie at the top
    ref = O.pack(big[:, :D], None, lam, 64 + 64, 4, O.MODE_NONE)
    p = B.rosaq_pack_weights(big, None, lam, 128, 4, B.Q_NONE, host_only=True, ldw=D + 40,
                             out_features=N, in_features=D)
    _compare(p, ref)


def test_degenerate_groups_match():
    W = np.zeros((16, 256), np.float16)
    W[1, 128:] = 0.25                                 # constant group
    W[2, 128:] = np.linspace(-2, -1, 128)             # all negative
    W[3, 130] = 6e-5                                  # tiny range, fp16 subnormal scale territory
    lam = np.arange(256, 0, -1.0)
    for bits in (3, 4):
        ref = O.pack(W, None, lam, 128, bits, O.MODE_NONE)
        p = B.rosaq_pack_weights(W, None, lam, 128, bits, B.Q_NONE, host_only=True)
        _compare(p, ref)


def test_f16_conversion_of_rotated_weights_covers_subnormals_and_ties():
    # Q = c * I scales W by a constant: exercises the library's fp64 -> fp16 rounding on every
    # fp16 input value, including results that land on ties and in the subnormal range
    D = 128
    allh = np.arange(0, 0x7c00, dtype=np.uint16).view(np.float16)         # all finite positives
    n = (allh.size + D - 1) // D
    W = np.zeros(n * D, np.float16); W[:allh.size] = allh
    W = W.reshape(n, D); W[1::2] *= np.float16(-1)
    lam = np.arange(D, 0, -1.0)
    for c in (np.float32(1.0) / 3, np.float32(2.0 ** -11) * 3, np.float32(0.75), np.float32(2.0 ** -12)):
        Q = (np.eye(D) * c).astype(np.float32)
        ref = O.pack(W, Q, lam, D, 4, O.MODE_FULL)
        p = B.rosaq_pack_weights(W, Q, lam, D, 4, B.Q_FULL, host_only=True)
        _compare(p, ref)


@pytest.mark.parametrize("rule,arg,K", [(B.SELECT_TOP_PER_HEAD, 0, 128), (B.SELECT_BOTTOM, 0, 128),
                                        (B.SELECT_CONSECUTIVE, 77, 128), (B.SELECT_TOP_AND_BOTTOM, 0, 128),
                                        (B.SELECT_TOP_PER_HEAD, 0, 256)])
def test_selection_rules_bit_exact(rule, arg, K):
    lay = synth.make_layer(5, 4, 512, 40, 512)
    Qb, lam = O.pca_headwise(lay["X_cal"], 128, "jacobi")
    Qb32 = Qb.astype(np.float32)
    ref = O.pack(lay["W"], Qb32, lam, K, 4, O.MODE_HEADWISE, rule=rule, arg=arg)
    p = B.rosaq_pack_weights(lay["W"], Qb32, lam, K, 4, B.Q_HEADWISE, host_only=True,
                             select_rule=rule, select_arg=arg)
    _compare(p, ref)
    if rule == B.SELECT_TOP_PER_HEAD:
        sal = B.rosaq_packed_export(p)["salient_idx"]
        assert [int(np.sum((sal >= 128 * h) & (sal < 128 * (h + 1)))) for h in range(4)] == [K // 4] * 4


def test_rotation_absorbed_packs_the_same_arrays():
    lay = synth.make_layer(6, 4, 256, 24, 300)
    Qb, lam = O.pca_headwise(lay["X_cal"], 128, "jacobi")
    Qb32 = Qb.astype(np.float32)
    ref = O.pack(lay["W"], Qb32, lam, 128, 4, O.MODE_HEADWISE)
    p = B.rosaq_pack_weights(lay["W"], Qb32, lam, 128, 4, B.Q_HEADWISE, host_only=True,
                             rotation_absorbed=True)
    _compare(p, ref)
    assert p.q_mode == B.Q_NONE


def _decode_image(wS_words, wq_words, N, D, K, bits):
    """The documented fragment layout read back with plain loops, written from the layout's description
    and not from the packer: returns W_S bits [N x K], codes [N x (D-K)], scale bits and zero bits [N x G]."""
    G = (D - K) // 128
    tiles = 8 * ((N + 127) // 128)
    ks_s = K // 32
    W_S = np.zeros((N, K), np.uint16)
    halves = wS_words.view(np.uint16).reshape(tiles, max(ks_s, 1), 64, 8) if ks_s else None
    for n in range(N):
        t, r = divmod(n, 16)
        for ks in range(ks_s):
            for j in range(4):                       # lane = 16 j + r holds channels 32 ks + 8 j .. + 7
                W_S[n, 32 * ks + 8 * j: 32 * ks + 8 * j + 8] = halves[t, ks, 16 * j + r]
    code_dwords = 256 if bits == 4 else 192
    rec = wq_words.reshape(tiles, max(G, 1), code_dwords + 16) if G else None
    codes = np.zeros((N, D - K), np.uint8)
    scales = np.zeros((N, G), np.uint16)
    zeros = np.zeros((N, G), np.uint16)
    for n in range(N):
        t, r = divmod(n, 16)
        for g in range(G):
            sz = int(rec[t, g, code_dwords + r])
            scales[n, g], zeros[n, g] = sz & 0xFFFF, sz >> 16
            for j in range(4):
                lane = 16 * j + r
                if bits == 4:
                    w = [int(v) for v in rec[t, g, 4 * lane: 4 * lane + 4]]
                    for ks in range(4):
                        for e in range(8):           # element e of k-step ks: nibble (e >> 1) + 4 (e & 1)
                            codes[n, 128 * g + 32 * ks + 8 * j + e] = (w[ks] >> (4 * ((e >> 1) + 4 * (e & 1)))) & 15
                else:
                    w = [int(v) for v in rec[t, g, 3 * lane: 3 * lane + 3]]
                    for ks in range(4):
                        for e in range(8):           # pair P = 4 ks + e / 2; odd elements in the high half
                            P, half = 4 * ks + (e >> 1), 16 * (e & 1)
                            if P < 15:
                                c = (w[P // 5] >> (half + 3 * (P % 5))) & 7
                            else:                    # the sixteenth pair: bit b of the code in dword b, bit 15 / 31
                                c = sum(((w[b] >> (half + 15)) & 1) << b for b in range(3))
                            codes[n, 128 * g + 32 * ks + 8 * j + e] = c
    return W_S, codes, scales, zeros


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("N,D,K", [(40, 384, 128), (130, 256, 0), (17, 256, 256)])
def test_device_image_follows_the_documented_fragment_layout(bits, N, D, K):
    """rosaq_packed_image (what the kernels read) decoded by an independent reader of the layout gives back
    the canonical arrays; rows beyond N are padding (zero weights, scale 2^-14)."""
    lay = synth.make_layer(900 + bits + N, 4, D, N, 64)
    lam = np.abs(lay["X_cal"]).mean(axis=0)
    p = B.rosaq_pack_weights(lay["W"], None, lam, K, bits, B.Q_NONE, host_only=True)
    got = B.rosaq_packed_export(p)
    wS = B.rosaq_packed_image(p, 0)
    wq = B.rosaq_packed_image(p, 1)
    tiles = 8 * ((N + 127) // 128)
    G = (D - K) // 128
    assert wS.size == tiles * (K // 32) * 64 * 4
    assert wq.size == tiles * G * ((256 if bits == 4 else 192) + 16)
    W_S, codes, scales, zeros = _decode_image(wS, wq, N, D, K, bits)
    assert np.array_equal(W_S, got["W_S"].view(np.uint16).reshape(N, K))
    assert np.array_equal(codes, got["codes"].reshape(N, D - K))
    assert np.array_equal(scales, got["scales"].view(np.uint16).reshape(N, G))
    assert np.array_equal(zeros, got["zeros"].view(np.uint16).reshape(N, G))
    if G:
        rec = wq.reshape(tiles, G, -1)
        pad_rows = [(n // 16, n % 16) for n in range(N, tiles * 16)]
        cd = 256 if bits == 4 else 192
        assert all(int(rec[t, g, cd + r]) == 0x0400 for t, r in pad_rows for g in range(G))
    p.free()
