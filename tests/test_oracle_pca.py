"""Pins for the oracle's PCA (Sec. 3.1 Eq. 4, Sec. 3.1.1 Eq. 6) and selection (Sec. 3.2)."""
import numpy as np
import pytest

from oracle import rosaq_oracle as O
from paper_2506_13472_amd import synth


def _cal(seed, n_cal, D):
    return synth.make_layer(seed, 4, D, 8, n_cal)["X_cal"]


@pytest.mark.parametrize("D,n_cal", [(8, 32), (64, 256), (128, 512), (96, 40)])
def test_jacobi_invariants(D, n_cal):
    X = _cal(1, n_cal, D)
    C = O.second_moment(X)
    Q, lam = O.pca_full(X, "jacobi")
    assert np.max(np.abs(Q.T @ Q - np.eye(D))) <= 1e-10
    assert np.all(np.diff(lam) <= 0) and np.all(lam >= 0)
    assert abs(lam.sum() - np.trace(C)) <= 1e-10 * np.trace(C)
    assert np.linalg.norm(Q @ np.diag(lam) @ Q.T - C) <= 1e-10 * np.linalg.norm(C)
    # (X Q)^T (X Q) / N_cal is diagonal = Lambda: rotated channels are uncorrelated
    Xh = X @ Q
    G = Xh.T @ Xh / n_cal
    assert np.linalg.norm(G - np.diag(lam)) <= 1e-10 * np.linalg.norm(C)


@pytest.mark.parametrize("D,n_cal", [(16, 64), (128, 512), (200, 64)])
def test_jacobi_matches_lapack(D, n_cal):
    X = _cal(2, n_cal, D)
    C = O.second_moment(X)
    Qj, lj = O.pca_full(X, "jacobi")
    w = np.linalg.eigvalsh(C)[::-1]
    assert np.max(np.abs(lj - np.maximum(w, 0))) <= 1e-10 * w[0]
    Ql, ll = O.pca_full(X, "lapack")
    r = min(D, n_cal)
    # separated eigenvalues: same eigenvectors (after the sign convention)
    gaps = np.minimum(np.abs(np.diff(ll[:r])).min(), ll[r - 1] if r < D else np.inf)
    if gaps > 1e-6 * ll[0]:
        assert np.max(np.abs(Qj[:, :r] - Ql[:, :r])) <= 1e-6
    # null space (rank-deficient C): same subspace, any basis
    if r < D:
        Pj = Qj[:, r:] @ Qj[:, r:].T
        Pl = Ql[:, r:] @ Ql[:, r:].T
        assert np.max(np.abs(Pj - Pl)) <= 1e-8


def test_closed_form_orthogonal_columns():
    # X with mutually orthogonal columns of norm sigma_c * sqrt(N): C = diag(sigma^2),
    # so lambda = sigma^2 sorted and Q is a signed permutation.
    rng = np.random.default_rng(3)
    n = 32
    Hm, _ = np.linalg.qr(rng.standard_normal((n, n)))
    D = 12
    sig = np.array([3.0, 0.5, 7.0, 1.0, 2.0, 9.0, 0.25, 4.0, 6.0, 5.0, 8.0, 0.75])
    X = Hm[:, :D] * sig * np.sqrt(n)
    Q, lam = O.pca_full(X, "jacobi")
    assert np.allclose(lam, np.sort(sig ** 2)[::-1], rtol=1e-12)
    order = np.argsort(-sig)
    P = np.zeros((D, D))
    P[order, np.arange(D)] = 1.0
    assert np.max(np.abs(np.abs(Q) - P)) <= 1e-10
    # with Q a permutation the salient rule is the magnitude rule of the 'Mixed' baseline
    sal, _ = O.select_salient(lam, 4)
    assert sorted(order[sal].tolist()) == sorted(np.argsort(-sig)[:4].tolist())


def test_jacobi_degenerate_inputs():
    lam, V = O.jacobi_eigh(np.zeros((5, 5)))
    assert np.all(lam == 0) and np.allclose(V, np.eye(5))
    lam, V = O.jacobi_eigh(np.array([[2.0, 1.0], [1.0, 2.0]]))  # equal diagonal: 45 degrees
    assert np.allclose(sorted(lam), [1.0, 3.0])
    lam, V = O.jacobi_eigh(np.diag([3.0, 1.0, 2.0]))
    assert np.allclose(lam, [3.0, 1.0, 2.0]) and np.allclose(V, np.eye(3))


def test_headwise_is_blockdiag_of_per_head_pca():
    D, hd = 256, 64
    X = _cal(4, 300, D)
    Qb, lam = O.pca_headwise(X, hd, "jacobi")
    assert Qb.shape == (4, hd, hd)
    for h in range(4):
        Qh, lh = O.pca_full(X[:, h * hd:(h + 1) * hd], "jacobi")
        assert np.array_equal(Qh, Qb[h]) and np.array_equal(lh, lam[h * hd:(h + 1) * hd])
    Qd = O.expand_blockdiag(Qb)
    assert np.max(np.abs(Qd.T @ Qd - np.eye(D))) <= 1e-10
    A = np.random.default_rng(0).standard_normal((5, D))
    assert np.allclose(O.rotate(A, Qb, O.MODE_HEADWISE), O.rotate(A, Qd, O.MODE_FULL), atol=1e-12)


def test_select_bruteforce_and_ties():
    rng = np.random.default_rng(5)
    for D, K in [(8, 3), (16, 16), (16, 0), (40, 8)]:
        lam = rng.random(D)
        sal, perm = O.select_salient(lam, K)
        # brute force: a channel is salient iff fewer than K channels beat it
        beat = [(np.sum(lam > lam[c]) + np.sum((lam == lam[c]) & (np.arange(D) < c))) for c in range(D)]
        want = [c for c in range(D) if beat[c] < K]
        assert sal.tolist() == want
        assert sorted(perm.tolist()) == list(range(D))
        assert perm[:K].tolist() == want and np.all(np.diff(perm[K:]) > 0)
    lam = np.array([1.0, 5.0, 5.0, 5.0, 0.0, 5.0])
    sal, perm = O.select_salient(lam, 2)
    assert sal.tolist() == [1, 2]                      # ties -> lower index
    assert perm.tolist() == [1, 2, 0, 3, 4, 5]


def test_select_full_mode_is_prefix_and_headwise_is_prefix_per_head():
    X = _cal(6, 128, 128)
    _, lam = O.pca_full(X, "jacobi")
    sal, _ = O.select_salient(lam, 32)
    assert sal.tolist() == list(range(32))
    D, hd = 256, 64
    Xh = _cal(7, 300, D)
    _, lamh = O.pca_headwise(Xh, hd, "jacobi")
    sal, _ = O.select_salient(lamh, 64)
    for h in range(D // hd):
        loc = sal[(sal >= h * hd) & (sal < (h + 1) * hd)] - h * hd
        assert loc.tolist() == list(range(len(loc)))   # a prefix of the head's sorted channels


def test_top_rotated_channel_dominates():
    # qualitative claim of the paper's activation-statistics appendix: in the
    # rotated space the first channel carries more mean magnitude than any
    # original channel does.
    lay = synth.make_layer(0, 64, 128, 8, 512)
    Q, lam = O.pca_full(lay["X_cal"], "jacobi")
    rot = np.abs(lay["X_cal"] @ Q).mean(axis=0)
    orig = np.abs(lay["X_cal"]).mean(axis=0)
    assert np.argmax(rot) == 0 and rot[0] >= orig.max()


def test_selection_rules_by_definition():
    rng = np.random.default_rng(11)
    D, K, hd = 256, 64, 128
    lam = rng.random(D)
    lam[5] = lam[200] = lam.max()                       # ties
    lam[7] = lam[130] = lam.min()
    rank_desc = sorted(range(D), key=lambda c: (-lam[c], c))
    rank_asc = sorted(range(D), key=lambda c: (lam[c], c))
    sal, perm = O.select_salient(lam, K, O.RULE_BOTTOM)
    assert sal.tolist() == sorted(rank_asc[:K])
    sal, _ = O.select_salient(lam, K, O.RULE_CONSECUTIVE, arg=37)
    assert sal.tolist() == list(range(37, 37 + K))
    sal, _ = O.select_salient(lam, K, O.RULE_TOP_AND_BOTTOM)
    top = rank_desc[:K // 2]
    bottom = [c for c in rank_asc if c not in top][:K // 2]
    assert sal.tolist() == sorted(top + bottom) and len(set(sal.tolist())) == K
    sal, perm = O.select_salient(lam, K, O.RULE_TOP_PER_HEAD, head_dim=hd)
    for h in range(D // hd):
        want = sorted(sorted(range(h * hd, (h + 1) * hd), key=lambda c: (-lam[c], c))[:K // 2])
        assert sal[(sal >= h * hd) & (sal < (h + 1) * hd)].tolist() == want
    assert sorted(perm.tolist()) == list(range(D)) and perm[:K].tolist() == sal.tolist()
    # all-equal spectrum: halves of TOP_AND_BOTTOM stay disjoint
    sal, _ = O.select_salient(np.ones(16), 8, O.RULE_TOP_AND_BOTTOM)
    assert sal.tolist() == list(range(8))
    # sorted-within-head spectrum (what head-wise PCA gives): per-head rule = prefix of each head
    lam2 = np.concatenate([np.sort(rng.random(hd))[::-1] for _ in range(2)])
    sal, _ = O.select_salient(lam2, 64, O.RULE_TOP_PER_HEAD, head_dim=hd)
    assert sal.tolist() == list(range(32)) + list(range(128, 160))


def test_top_and_bottom_is_the_union_of_top_and_bottom():
    # salient-channel ablation appendix: the combined scheme takes both the channels Top selects
    # and the channels Bottom selects.  With K' per side that is the rule called with K = 2 K'
    # (K always counts the fp16 block), checked here against the two rules run on their own.
    rng = np.random.default_rng(5)
    lam = rng.random(384)
    for k_side in (32, 64, 128):
        top, _ = O.select_salient(lam, k_side, O.RULE_TOP)
        bottom, _ = O.select_salient(lam, k_side, O.RULE_BOTTOM)
        both, perm = O.select_salient(lam, 2 * k_side, O.RULE_TOP_AND_BOTTOM)
        assert both.tolist() == sorted(set(top.tolist()) | set(bottom.tolist()))
        assert len(both) == 2 * k_side and perm[:2 * k_side].tolist() == both.tolist()


def test_top_rule_beats_the_ablation_rules_on_output_error():
    # synthetic analogue of the paper's salient-channel ablation: keeping the top-eigenvalue
    # channels in fp16 gives a smaller output error than bottom / a consecutive block elsewhere
    lay = synth.make_layer(3, 32, 384, 48, 512)
    Q, lam = O.pca_full(lay["X_cal"], "jacobi")
    Q32 = Q.astype(np.float32)
    err = {}
    for name, rule, arg, K in (("top", O.RULE_TOP, 0, 128), ("bottom", O.RULE_BOTTOM, 0, 128),
                               ("block", O.RULE_CONSECUTIVE, 150, 128),
                               ("both_as_in_the_paper", O.RULE_TOP_AND_BOTTOM, 0, 256),
                               ("both_same_budget", O.RULE_TOP_AND_BOTTOM, 0, 128)):
        p = O.pack(lay["W"], Q32, lam, K, 3, O.MODE_FULL, rule=rule, arg=arg)
        err[name] = O.quality_report(lay["x"], lay["W"], Q32, p)
    assert err["top"] < err["bottom"] and err["top"] < err["block"]
    # the paper's table: Top & Bottom (both sets, 2 K channels in fp16) lands next to Top, far from
    # Bottom; the extra K bottom channels carry almost no energy, so they buy next to nothing
    assert err["both_as_in_the_paper"] < err["bottom"]
    assert abs(err["both_as_in_the_paper"] - err["top"]) < 0.25 * err["top"]
    # with the fp16 budget held at K (K/2 + K/2) the bottom half is wasted: worse than Top
    assert err["top"] < err["both_same_budget"] < err["bottom"]


def test_headwise_pca_beats_global_pca_when_calibration_rows_are_scarce():
    # synthetic analogue of the head-wise ablation appendix (one PCA per head, Eq. 6, against one
    # PCA over the concatenated heads, Eq. 8): with D / 2 calibration rows the per-head rotation
    # gives the smaller output error on held-out activations, for every seed
    from oracle import ablation_table as A
    for seed in (0, 1, 2):
        r = A.headwise_ablation(seed, n_cal=256)
        assert r["head-wise PCA, K/H per head"] < r["global PCA"]
        assert r["head-wise PCA, top-K over all heads"] < r["global PCA"]
        assert r["global PCA"] < 0.5 * r["no rotation (top-K by magnitude)"]


def test_ablation_table_selection_rows_order_like_the_paper():
    from oracle import ablation_table as A
    r = A.selection_ablation(0, D=384, N=48, n_cal=512, M=64, starts=3)
    assert r["Top"] < 0.6 * r["Random"] and r["Top"] < 0.6 * r["Bottom"]
    assert abs(r["Top & Bottom"] - r["Top"]) < 0.25 * r["Top"]
    assert r["Bottom"] <= r["none (all low-bit)"] * 1.05
