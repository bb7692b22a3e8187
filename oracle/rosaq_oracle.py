"""CPU oracle for the ROSAQ rotated mixed-precision linear layer.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of what
the HIP library must compute.  It shares no code with the library, is never
imported by the product path, and exists so that tests, the smoke check and the
bench's CPU-baseline leg have something independent to compare against.

Notation.  The paper writes the rotation as R and a weight as W in R^{d x d'}
(inputs on rows).  Here the rotation is called Q and weights use the PyTorch
layout W[out, in] = W[N, D]; the rotated weight is What = W Q, which is the
transpose of the paper's R^T W, and the layer is y = (x Q) What^T.

Steps (paper passages they follow):
  pca_full / pca_headwise   Sec. 3.1 Eq. 4 (X^T X = R Lambda R^T, columns sorted
                            by eigenvalue) and Sec. 3.1.1 Eq. 5-6 (one PCA per head)
  rotate_weights            Eq. 1-2 (X W = (X R)(R^T W)), transposed layout
  select_salient            Sec. 3.2 (channels with the K largest eigenvalues); the per-head
                            setting of the weight-splitting appendix and the ablation rules of App. B
  quantize_groups           Eq. 2, Sec. 3.3, Sec. 4.1 (per-group, 128 channels,
                            INT3/INT4); the formula itself is not in the paper,
                            the reading used is asymmetric min-max round-to-nearest
  pack                      Eq. 3 split [R_S^T W_S ; Q(R_N^T W_N)]
  linear_ref                Eq. 3 evaluated in fp64 on the stored representation
                            (Eq. 6 when the rotation is block diagonal)
  swiglu_ref                silu(gate) * up on two such layers (the FFN around W_G, W_U of the
                            weight-splitting appendix)

Pins (tests/test_oracle_*.py): orthogonality, trace and reconstruction of the
eigen-decomposition, agreement with LAPACK, a closed form with orthogonal
calibration columns, the rotation identity of Eq. 1 without quantisation,
K = D reducing to a plain fp16-weight GEMM, Q = I reducing to textbook group
quantisation, brute-force nearest-code search, exact round trip of
representable weights, the calibration-set error identity
||Xhat (What - What_stored)^T||_F^2 = N_cal * sum_j lambda_j ||col_j diff||^2,
and a triple-loop matmul on tiny inputs.
"""
from __future__ import annotations

import numpy as np

MODE_NONE = 0
MODE_FULL = 1
MODE_HEADWISE = 2

MIN_SCALE = 2.0 ** -14  # smallest normal fp16; floor for the group scale


# --------------------------------------------------------------------------
# small helpers
# --------------------------------------------------------------------------
def fp16_rne(a) -> np.ndarray:
    """Round fp64 values to fp16 (round-half-to-even, one rounding)."""
    return np.asarray(a, dtype=np.float64).astype(np.float16)


def as_f64(a) -> np.ndarray:
    return np.asarray(a).astype(np.float64)


# --------------------------------------------------------------------------
# Sec. 3.1, Eq. 4: PCA of the calibration second-moment matrix
# --------------------------------------------------------------------------
def second_moment(X) -> np.ndarray:
    """C = X^T X / N_cal, uncentred (Eq. 4 has no mean subtraction; dividing by
    the row count changes neither the eigenvectors nor their order)."""
    X = as_f64(X)
    return X.T @ X / X.shape[0]


def _round_robin_pairs(n: int):
    """Yield n-1 (n even) rounds of n/2 disjoint index pairs covering all pairs."""
    m = n + (n & 1)
    idx = list(range(m))
    for _ in range(m - 1):
        p = np.array(idx[: m // 2])
        q = np.array(idx[m // 2:][::-1])
        keep = (p < n) & (q < n)
        lo = np.minimum(p[keep], q[keep])
        hi = np.maximum(p[keep], q[keep])
        yield lo, hi
        idx = [idx[0]] + [idx[-1]] + idx[1:-1]


def jacobi_eigh(C, tol: float = 1e-13, max_sweeps: int = 100):
    """Cyclic Jacobi eigensolver for a real symmetric matrix.

    Each sweep visits every off-diagonal pair (p, q) once; a plane rotation
    zeroes C[p, q].  The pairs of one round are disjoint (round-robin order), so
    a round is applied as one orthogonal similarity.  Stops when the
    off-diagonal Frobenius norm is <= tol * ||C||_F.
    Returns (eigenvalues, eigenvectors as columns), unsorted.
    """
    A = as_f64(C).copy()
    n = A.shape[0]
    assert A.shape == (n, n)
    A = 0.5 * (A + A.T)
    V = np.eye(n)
    normA = np.linalg.norm(A)
    if n == 1 or normA == 0.0:
        return np.diag(A).copy(), V
    rounds = list(_round_robin_pairs(n))
    tiny = np.finfo(np.float64).eps * normA / n
    for _ in range(max_sweeps):
        off = np.linalg.norm(A - np.diag(np.diag(A)))
        if off <= tol * normA:
            break
        for p, q in rounds:
            apq = A[p, q]
            app = A[p, p]
            aqq = A[q, q]
            # entries already at round-off level are set to zero without a rotation
            small = np.abs(apq) <= tiny
            A[p[small], q[small]] = 0.0
            A[q[small], p[small]] = 0.0
            act = ~small
            # rotation angle: tan(2 theta) = 2 a_pq / (a_qq - a_pp); t = tan(theta), smaller root
            tau = np.where(act, (aqq - app) / (2.0 * np.where(act, apq, 1.0)), 0.0)
            t = np.where(act, np.sign(tau) / (np.abs(tau) + np.hypot(1.0, tau)), 0.0)
            t = np.where(act & (tau == 0.0), 1.0, t)
            c = 1.0 / np.sqrt(1.0 + t * t)
            s = t * c
            # A <- J^T A J with J = I except J[p,p]=c, J[p,q]=s, J[q,p]=-s, J[q,q]=c
            Ap = A[:, p].copy()
            Aq = A[:, q].copy()
            A[:, p] = c * Ap - s * Aq
            A[:, q] = s * Ap + c * Aq
            Ap = A[p, :].copy()
            Aq = A[q, :].copy()
            A[p, :] = c[:, None] * Ap - s[:, None] * Aq
            A[q, :] = s[:, None] * Ap + c[:, None] * Aq
            Vp = V[:, p].copy()
            Vq = V[:, q].copy()
            V[:, p] = c * Vp - s * Vq
            V[:, q] = s * Vp + c * Vq
    return np.diag(A).copy(), V


def sort_eigpairs(lam, V):
    """Eigenvalues descending (ties keep the lower original index first), negative
    round-off clamped to zero, eigenvector sign fixed so that the entry of
    largest magnitude is positive (reproducibility only)."""
    lam = as_f64(lam)
    order = np.argsort(-lam, kind="stable")
    lam = np.maximum(lam[order], 0.0)
    V = as_f64(V)[:, order].copy()
    big = np.argmax(np.abs(V), axis=0)
    sign = np.sign(V[big, np.arange(V.shape[1])])
    sign[sign == 0] = 1.0
    return lam, V * sign


def eig_sym(C, solver: str = "jacobi"):
    """Sorted eigen-decomposition with either the Jacobi solver above or LAPACK
    (numpy.linalg.eigh).  LAPACK is used only for sizes where Jacobi in numpy
    would take hours; the tests check the two agree at the small sizes."""
    if solver == "jacobi":
        lam, V = jacobi_eigh(C)
    elif solver == "lapack":
        lam, V = np.linalg.eigh(as_f64(C))
    else:
        raise ValueError(solver)
    return sort_eigpairs(lam, V)


def pca_full(X_cal, solver: str = "jacobi"):
    """Layer-wise PCA (Sec. 3.1, Eq. 4).  Returns Q [D, D] (eigenvectors as
    columns, xhat = x Q) and the eigenvalues [D], descending."""
    lam, V = eig_sym(second_moment(X_cal), solver)
    return V, lam


def pca_headwise(X_cal, head_dim: int = 128, solver: str = "jacobi"):
    """Head-wise PCA (Sec. 3.1.1, Eq. 6): one PCA per head on that head's
    columns of the calibration set.  Returns Q blocks [H, hd, hd] and the
    eigenvalues [D] (descending inside each head, head after head)."""
    X = as_f64(X_cal)
    D = X.shape[1]
    assert D % head_dim == 0
    H = D // head_dim
    Qb = np.empty((H, head_dim, head_dim))
    lam = np.empty(D)
    for h in range(H):
        sl = slice(h * head_dim, (h + 1) * head_dim)
        lh, Vh = eig_sym(second_moment(X[:, sl]), solver)
        Qb[h] = Vh
        lam[sl] = lh
    return Qb, lam


def expand_blockdiag(Qb) -> np.ndarray:
    """Dense [D, D] matrix with the blocks Qb[h] on its diagonal."""
    Qb = as_f64(Qb)
    H, hd, _ = Qb.shape
    Q = np.zeros((H * hd, H * hd))
    for h in range(H):
        Q[h * hd:(h + 1) * hd, h * hd:(h + 1) * hd] = Qb[h]
    return Q


# --------------------------------------------------------------------------
# Eq. 1-2: rotate inputs and weights
# --------------------------------------------------------------------------
def rotate(A, Q, mode: int) -> np.ndarray:
    """A Q in fp64 for a row-major A[., D].  mode NONE: Q is ignored (R = I, the
    'Mixed' baseline of Sec. 4.1); FULL: Q [D, D]; HEADWISE: Q [H, hd, hd]."""
    A = as_f64(A)
    if mode == MODE_NONE:
        return A.copy()
    if mode == MODE_FULL:
        return A @ as_f64(Q)
    if mode == MODE_HEADWISE:
        Qb = as_f64(Q)
        H, hd, _ = Qb.shape
        out = np.empty_like(A)
        for h in range(H):
            sl = slice(h * hd, (h + 1) * hd)
            out[:, sl] = A[:, sl] @ Qb[h]
        return out
    raise ValueError(mode)


def rotate_weights(W16, Q, mode: int):
    """What = W Q in fp64 (Eq. 1 in the [out, in] layout), then a single rounding
    to fp16: the quantiser's input is that fp16 matrix.  Returns (What fp64,
    What16 fp16)."""
    What = rotate(W16, Q, mode)
    return What, fp16_rne(What)


# --------------------------------------------------------------------------
# Sec. 3.2: salient channel identification
# --------------------------------------------------------------------------
RULE_TOP = 0            # Sec. 3.2: the K largest eigenvalues (the method)
RULE_TOP_PER_HEAD = 1   # weight-splitting appendix: the same number of salient channels in every head
RULE_BOTTOM = 2         # ablation of App. B: the K smallest eigenvalues
RULE_CONSECUTIVE = 3    # ablation of App. B: K consecutive channels from a given start ("Random")
RULE_TOP_AND_BOTTOM = 4 # ablation of App. B: the channels of Top and of Bottom together (K counts both halves)


def select_salient(lam, K: int, rule: int = RULE_TOP, arg: int = 0, head_dim: int = 128):
    """Salient rotated channels, reported ascending, and the storage permutation
    perm = [salient ; every other channel ascending].  Ties go to the lower channel.

    TOP            the K largest eigenvalues (Sec. 3.2)
    TOP_PER_HEAD   K / H largest inside every block of head_dim channels (the paper keeps
                   32 per head for the attention output projection)
    BOTTOM         the K smallest eigenvalues
    CONSECUTIVE    channels arg .. arg + K - 1 (the caller draws the random start)
    TOP_AND_BOTTOM the union of what TOP and BOTTOM pick with K/2 each: the K/2 largest, then
                   the K/2 smallest among the remaining channels.  K is the size of the fp16
                   block, as for every rule, so the appendix's combined scheme for its K' (both
                   the K' channels of Top and the K' channels of Bottom) is this rule with
                   K = 2 K'.  "Among the remaining" only matters when eigenvalues tie across
                   the two halves or K > D/2; it keeps the two halves disjoint.
    """
    lam = as_f64(lam)
    D = lam.shape[0]
    assert 0 <= K <= D
    desc = np.argsort(-lam, kind="stable")          # largest first, ties: lower index first
    asc = np.argsort(lam, kind="stable")            # smallest first, ties: lower index first
    if rule == RULE_TOP:
        chosen = desc[:K]
    elif rule == RULE_TOP_PER_HEAD:
        H = D // head_dim
        assert D % head_dim == 0 and K % H == 0
        per = K // H
        chosen = np.concatenate([h * head_dim + np.argsort(-lam[h * head_dim:(h + 1) * head_dim],
                                                           kind="stable")[:per] for h in range(H)]) \
            if K else np.zeros(0, np.int64)
    elif rule == RULE_BOTTOM:
        chosen = asc[:K]
    elif rule == RULE_CONSECUTIVE:
        assert 0 <= arg <= D - K
        chosen = np.arange(arg, arg + K)
    elif rule == RULE_TOP_AND_BOTTOM:
        assert K % 2 == 0
        top = desc[:K // 2]
        taken = np.zeros(D, dtype=bool)
        taken[top] = True
        bottom = [c for c in asc if not taken[c]][:K // 2]
        chosen = np.concatenate([top, np.array(bottom, dtype=np.int64)])
    else:
        raise ValueError(rule)
    sal = np.sort(chosen).astype(np.int32)
    mask = np.ones(D, dtype=bool)
    mask[sal] = False
    rest = np.nonzero(mask)[0].astype(np.int32)
    return sal, np.concatenate([sal, rest]).astype(np.int32)


# --------------------------------------------------------------------------
# Sec. 3.3 / Eq. 2: per-group low-bit quantiser
# --------------------------------------------------------------------------
def quantize_groups(w16, bits: int, group: int = 128):
    """Asymmetric min-max round-to-nearest quantiser on fp16 values.

    w16 [N, C] with C % group == 0; groups are runs of `group` consecutive
    columns.  Per (row, group):
        qmax = 2^bits - 1
        s = fp16(max((max w - min w) / qmax, 2^-14))        (fp64 arithmetic)
        z = clamp(rint(-min w / s), 0, qmax)                 (an integer)
        q = clamp(rint(w / s) + z, 0, qmax)
    rint is round-half-to-even.  Returns codes uint8 [N, C], scales fp16 [N, C/g],
    zeros fp16 [N, C/g] (integer valued).
    """
    w = as_f64(w16)
    N, C = w.shape
    assert C % group == 0
    G = C // group
    qmax = float(2 ** bits - 1)
    wg = w.reshape(N, G, group)
    mx = wg.max(axis=2)
    mn = wg.min(axis=2)
    s16 = fp16_rne(np.maximum((mx - mn) / qmax, MIN_SCALE))
    s = as_f64(s16)
    z = np.clip(np.rint(-mn / s), 0.0, qmax)
    q = np.clip(np.rint(wg / s[:, :, None]) + z[:, :, None], 0.0, qmax)
    return (q.reshape(N, C).astype(np.uint8), s16, z.astype(np.float16))


def dequantize_groups(codes, scales, zeros, group: int = 128) -> np.ndarray:
    """(q - z) * s in fp64."""
    q = as_f64(codes)
    N, C = q.shape
    G = C // group
    s = as_f64(scales)[:, :, None]
    z = as_f64(zeros)[:, :, None]
    return ((q.reshape(N, G, group) - z) * s).reshape(N, C)


# --------------------------------------------------------------------------
# Eq. 3: the stored mixed-precision layer
# --------------------------------------------------------------------------
def pack(W16, Q, lam, K: int, bits: int, mode: int, group: int = 128, rule: int = RULE_TOP,
         arg: int = 0) -> dict:
    """Offline steps for one linear: rotate (Eq. 1), pick salient channels
    (Sec. 3.2), keep them in fp16 and quantise the rest group by group in
    storage order (Eq. 3, Sec. 3.3)."""
    W16 = np.asarray(W16, dtype=np.float16)
    N, D = W16.shape
    assert (D - K) % group == 0
    What, What16 = rotate_weights(W16, Q, mode)
    sal, perm = select_salient(lam, K, rule, arg)
    W_S = What16[:, sal].copy()
    W_N = What16[:, perm[K:]]
    if D > K:
        codes, scales, zeros = quantize_groups(W_N, bits, group)
    else:
        codes = np.zeros((N, 0), np.uint8)
        scales = np.zeros((N, 0), np.float16)
        zeros = np.zeros((N, 0), np.float16)
    return dict(N=N, D=D, K=K, bits=bits, group=group, mode=mode,
                salient_idx=sal, perm=perm, W_S=W_S, codes=codes,
                scales=scales, zeros=zeros, What=What, What16=What16)


def stored_weights(p: dict) -> np.ndarray:
    """The dequantised stored layer in storage order: [W_S | (q - z) s], fp64."""
    lo = dequantize_groups(p["codes"], p["scales"], p["zeros"], p["group"]) \
        if p["D"] > p["K"] else np.zeros((p["N"], 0))
    return np.concatenate([as_f64(p["W_S"]), lo], axis=1)


def round_rotation(Q, mode: int):
    """The run-time rotation is the fp16 rounding of Q."""
    if mode == MODE_NONE or Q is None:
        return None
    return as_f64(fp16_rne(Q))


def linear_ref(x16, Q, p: dict, q_round: bool = True) -> np.ndarray:
    """Eq. 3 in fp64 on the stored representation:
        xhat = x fp16(Q)                    (no intermediate rounding of xhat)
        y = xhat[:, salient] W_S^T + xhat[:, rest] ((q - z) s)^T
    q_round=False uses Q unrounded (for identities that need exact orthogonality)."""
    mode = p["mode"]
    Qr = round_rotation(Q, mode) if q_round else Q
    xhat = rotate(x16, Qr, mode)
    return xhat[:, p["perm"]] @ stored_weights(p).T


def silu(t) -> np.ndarray:
    """t / (1 + exp(-t)) in fp64, written so that large |t| neither overflows nor loses digits."""
    t = as_f64(t)
    e = np.exp(-np.abs(t))                       # in (0, 1]
    return np.where(t >= 0, t / (1.0 + e), t * e / (1.0 + e))


def swiglu_ref(x16, Q, p_gate: dict, p_up: dict) -> np.ndarray:
    """The gated pair of the FFN on two stored layers that share input and rotation (the up and
    gate projections are split alike, weight-splitting appendix): silu(y_gate) * y_up with both
    outputs the fp64 evaluation of Eq. 3, nothing rounded in between."""
    return silu(linear_ref(x16, Q, p_gate)) * linear_ref(x16, Q, p_up)


def tolerance_scale(x16, p: dict) -> np.ndarray:
    """||x_row||_2 * ||w_col||_2 per output element: the denominator of the
    max-error acceptance bound (w_col = the dequantised stored row of a channel)."""
    xn = np.linalg.norm(as_f64(x16), axis=1)
    wn = np.linalg.norm(stored_weights(p), axis=1)
    return xn[:, None] * wn[None, :]


def quality_report(x16, W16, Q, p: dict) -> float:
    """Relative Frobenius distance between the stored layer's output and the
    unquantised x W^T (model error, not a parity gate)."""
    exact = as_f64(x16) @ as_f64(W16).T
    return float(np.linalg.norm(linear_ref(x16, Q, p) - exact) / np.linalg.norm(exact))
