"""Pins for the fp64 oracle: each oracle function is checked against something
the paper or the mathematics fixes, never against the oracle itself.

  Philox words      published known-answer vectors (tests/golden)
  Gaussian          moments + Kolmogorov-Smirnov against the normal CDF
  Gram + eigen      closed-form spectrum X = Q diag(sigma) R; PAC bias
                    = tail energy (Section 4.2); rank-<=k exactness
  thin QR           hand-rolled Gram-Schmidt written here
  complement        Lemma 4 by Monte Carlo; Q1^T Q2 = 0
  basis             P^T P = I
  reconstruction    r = d-k  =>  X~ = X ; Theorem 1 by Monte Carlo; a wrong
                    scale converges to the biased mean the algebra predicts
  variance          proof of Theorem 2 (equality) by brute force to 1 %
  compress / dW     loops over the definition on tiny inputs; textbook
                    special cases
"""
import os

import numpy as np
import pytest
from scipy import stats

import synth_inputs as si
from oracle import prac_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ Philox
def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for row in rows:
        v = [int(t, 16) for t in row]
        out = orc.philox4x32_10(*v[0:4], *v[4:6])
        assert [int(x) for x in out] == v[6:10]


def test_philox_stream_mapping():
    # word idx depends on (seed, draw, stream, idx) only: block b, lane idx%4
    seed, draw, stream = 0x0123456789ABCDEF, 7, 1
    w = orc.philox_words(seed, draw, stream, 4099)
    assert w.dtype == np.uint32 and w.shape == (4099,)
    for idx in (0, 1, 5, 4098):
        blk = idx // 4
        ref = orc.philox4x32_10(blk & 0xFFFFFFFF, blk >> 32, stream, draw,
                                seed & 0xFFFFFFFF, seed >> 32)
        assert int(ref[idx % 4]) == int(w[idx])
    # a prefix regenerates identically; other streams / draws / seeds differ
    assert np.array_equal(orc.philox_words(seed, draw, stream, 100), w[:100])
    for other in ((seed + 1, draw, stream), (seed, draw + 1, stream), (seed, draw, 0)):
        assert not np.array_equal(orc.philox_words(*other, 100), w[:100])
    # seed_hi reaches the key: seeds differing only in the high word differ
    assert not np.array_equal(orc.philox_words(seed ^ (1 << 40), draw, stream, 8), w[:8])


def test_uniform_open_interval_and_exact():
    w = np.array([0, 1, 511, 512, 0xFFFFFFFF], dtype=np.uint32)
    u = orc.words_to_uniform(w)
    assert np.array_equal(u, (np.array([0, 0, 0, 1, 2**23 - 1]) + 0.5) / 2**23)
    assert u.min() > 0.0 and u.max() < 1.0
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)  # exact in fp32


def test_gaussian_moments_and_ks():
    z = orc.philox_normal(seed=11, draw=3, stream=1, n=2_000_000)
    n = z.size
    assert abs(z.mean()) < 4.0 / np.sqrt(n)
    assert abs(z.var() - 1.0) < 4.0 * np.sqrt(2.0 / n)
    assert abs((z ** 4).mean() - 3.0) < 4.0 * np.sqrt(96.0 / n)
    assert abs((z ** 3).mean()) < 4.0 * np.sqrt(15.0 / n)
    assert stats.kstest(z[:200_000], "norm").pvalue > 1e-3
    # consecutive values (cos / sin twins, neighbouring blocks) are uncorrelated
    assert abs(np.mean(z[0::2] * z[1::2])) < 4.0 / np.sqrt(n / 2)
    assert abs(np.mean(z[1:-1:2] * z[2::2])) < 4.0 / np.sqrt(n / 2)


def test_gaussian_matrix_layout():
    S = orc.gaussian_matrix(seed=5, draw=2, rows=7, cols=3)
    flat = orc.philox_normal(5, 2, orc.STREAM_S, 21)
    assert S.shape == (7, 3) and S[4, 2] == flat[4 * 3 + 2]


# ------------------------------------------------------- Gram + eigenspace
def _exact_case(N=96, d=24, alpha=0.8, seed=3):
    X, info = si.activation(N, d, alpha, seed, exact_spectrum=True)
    return X, info["R"], info["sigma"]


def test_gram_eigen_closed_form_spectrum():
    X, R, sig = _exact_case()
    k = 5
    Q1, lam = orc.principal_subspace(orc.gram(X), k)
    assert np.allclose(lam, sig ** 2, rtol=1e-10, atol=1e-14)
    # top-k right singular vectors are the first k rows of R (X = Z diag(sigma) R)
    proj_true = R[:k].T @ R[:k]
    assert np.abs(Q1 @ Q1.T - proj_true).max() < 1e-10
    # PAC bias equals the tail energy (Section 4.2)
    assert np.isclose(np.linalg.norm(X - X @ Q1 @ Q1.T) ** 2, np.sum(sig[k:] ** 2), rtol=1e-10)
    # third opinion from a library SVD, called here and not in the oracle
    Vt = np.linalg.svd(X, full_matrices=False)[2]
    assert np.abs(Q1 @ Q1.T - Vt[:k].T @ Vt[:k]).max() < 1e-10


def test_gram_is_xtx_by_loops_and_row_stride():
    rng = np.random.default_rng(0)
    X = rng.standard_normal((9, 4))
    G = orc.gram(X)
    for a in range(4):
        for b in range(4):
            assert np.isclose(G[a, b], sum(X[n, a] * X[n, b] for n in range(9)), rtol=1e-13)
    Gs = orc.gram(X, row_stride=4)   # rows 0, 4, 8
    assert np.allclose(Gs, sum(np.outer(X[n], X[n]) for n in (0, 4, 8)), rtol=1e-13)


def test_rank_k_input_is_captured_exactly():
    rng = np.random.default_rng(1)
    k, d, N = 3, 10, 40
    X = rng.standard_normal((N, k)) @ rng.standard_normal((k, d))
    Q1, lam = orc.principal_subspace(orc.gram(X), k)
    assert np.linalg.norm(X - X @ Q1 @ Q1.T) < 1e-12 * np.linalg.norm(X)
    assert np.all(np.abs(lam[k:]) < 1e-10 * lam[0])


# ------------------------------------------------------------------ thin QR
def _gram_schmidt(A):
    """Classical definition of the thin QR: orthogonalise column by column
    against the previous ones (done twice for accuracy), normalise with a
    positive norm -> R has a positive diagonal by construction."""
    A = A.copy()
    n = A.shape[1]
    Q = np.zeros_like(A)
    for j in range(n):
        v = A[:, j].copy()
        for _ in range(2):
            for i in range(j):
                v -= (Q[:, i] @ v) * Q[:, i]
        Q[:, j] = v / np.sqrt(v @ v)
    return Q


def test_thin_qr_positive_matches_gram_schmidt():
    A = np.random.default_rng(2).standard_normal((15, 6))
    Q, R = orc.thin_qr_positive(A)
    assert np.all(np.diag(R) > 0) and np.allclose(np.tril(R, -1), 0)
    assert np.allclose(Q @ R, A, atol=1e-13)
    assert np.allclose(Q, _gram_schmidt(A), atol=1e-12)


# -------------------------------------------------------- complement basis
def _fixed_q1(d, k, seed):
    return si.orthonormal_basis(d, k, seed)


def test_complement_is_orthonormal_and_orthogonal_to_q1():
    d, k, r = 20, 4, 6
    Q1 = _fixed_q1(d, k, 4)
    S = orc.gaussian_matrix(9, 0, d, r)
    Q2 = orc.complement_basis(Q1, S)
    assert np.abs(Q1.T @ Q2).max() < 1e-14
    assert np.abs(Q2.T @ Q2 - np.eye(r)).max() < 1e-14
    # Q2 is the Gram-Schmidt basis of the projected columns, in order
    So = S - Q1 @ (Q1.T @ S)
    assert np.allclose(Q2, _gram_schmidt(So), atol=1e-12)
    # and spans nothing outside span{S_o}
    assert np.linalg.matrix_rank(np.concatenate([So, Q2], axis=1), tol=1e-10) == r


def test_lemma4_expected_projector_monte_carlo():
    # E[Q2 Q2^T] = r/(d-k) (I - Q1 Q1^T)
    d, k, r, draws = 10, 3, 2, 20000
    Q1 = _fixed_q1(d, k, 5)
    acc = np.zeros((d, d))
    for t in range(draws):
        Q2 = orc.complement_basis(Q1, orc.gaussian_matrix(21, t, d, r))
        acc += Q2 @ Q2.T
    target = r / (d - k) * (np.eye(d) - Q1 @ Q1.T)
    # entries of Q2Q2^T are bounded by 1 -> std error <= 1/sqrt(draws)
    assert np.abs(acc / draws - target).max() < 4.0 * 0.5 / np.sqrt(draws)


def test_basis_orthonormal_all_rank_splits():
    X, _ = si.activation(64, 16, 0.8, seed=6)
    for k, r in ((4, 4), (0, 5), (6, 10), (16, 0), (1, 1)):
        P, s = orc.fit_basis(X, k, r, seed=1, draw=0)
        assert P.shape == (16, k + r)
        assert np.abs(P.T @ P - np.eye(k + r)).max() < 1e-13
        assert s == ((16 - k) / r if r else 0.0)


# ------------------------------------------------- reconstruction and scale
def test_full_complement_reconstructs_exactly():
    # r = d - k  =>  s = 1, P square orthogonal, X~ = X
    X, _ = si.activation(32, 12, 0.8, seed=7)
    for k in (0, 5):
        P, s = orc.fit_basis(X, k, 12 - k, seed=3, draw=1)
        assert s == 1.0
        Xh = orc.reconstruct(orc.compress(X, P), P, k, s)
        assert np.abs(Xh - X).max() < 1e-12 * np.abs(X).max()


def _mc_reconstruction(X, k, r, draws, scale=None, seed=17):
    d = X.shape[1]
    Q1, _ = orc.principal_subspace(orc.gram(X), k) if k else (np.zeros((d, 0)), None)
    s = orc.scaling_factor(d, k, r) if scale is None else scale
    mean = np.zeros_like(X)
    err2 = np.zeros(draws)
    for t in range(draws):
        Q2 = orc.complement_basis(Q1, orc.gaussian_matrix(seed, t, d, r))
        P = np.concatenate([Q1, Q2], axis=1)
        Xh = orc.reconstruct(orc.compress(X, P), P, k, s)
        mean += Xh
        err2[t] = np.sum((Xh - X) ** 2)
    return Q1, mean / draws, err2


def test_theorem1_unbiased_and_variance_identity_tiny():
    # N=6, d=12, k=3, r=4: E[X~] = X and
    # E||X~ - X||^2 = ((d-k)/r - 1) ||X (I - Q1 Q1^T)||^2  (equality in the proof)
    X, _ = si.activation(6, 12, 0.8, seed=8)
    k, r, draws = 3, 4, 100_000
    Q1, mean, err2 = _mc_reconstruction(X, k, r, draws)
    tail = np.sum((X - X @ Q1 @ Q1.T) ** 2)
    closed = ((12 - k) / r - 1.0) * tail
    assert abs(err2.mean() / closed - 1.0) < 0.01
    # unbiased: the mean is within 4 standard errors, the error budget taken
    # from the closed-form variance
    se = np.sqrt(closed / draws)
    assert np.linalg.norm(mean - X) < 4.0 * se


def test_wrong_scale_is_biased_as_predicted():
    # scale = f*s gives E[X~] = X Q1 Q1^T + f X (I - Q1 Q1^T) != X
    X, _ = si.activation(6, 12, 0.8, seed=9)
    k, r, draws, f = 3, 4, 20_000, 0.5
    s = orc.scaling_factor(12, k, r)
    Q1, mean, _ = _mc_reconstruction(X, k, r, draws, scale=f * s)
    tailX = X - X @ Q1 @ Q1.T
    predicted = X @ Q1 @ Q1.T + f * tailX
    se = np.sqrt(f * f * (s - 1.0) * np.sum(tailX ** 2) / draws)
    assert np.linalg.norm(mean - predicted) < 4.0 * se
    assert np.linalg.norm(mean - X) > 20.0 * se


@pytest.mark.parametrize("alpha", [0.5, 0.8, 1.5])
def test_variance_identity_rank_sweep_spectra_shrunk(alpha):
    # the rank-sweep spectra shrunk to d = 32; RAC (k=0) and a hybrid split
    X, _ = si.activation(8, 32, alpha, seed=10, exact_spectrum=False)
    for k, r in ((0, 8), (4, 4)):
        Q1, _, err2 = _mc_reconstruction(X, k, r, 40_000, seed=23)
        tail = np.sum((X - X @ Q1 @ Q1.T) ** 2) if k else np.sum(X ** 2)
        closed = ((32 - k) / r - 1.0) * tail
        assert abs(err2.mean() / closed - 1.0) < 0.015


# ------------------------------------------------------ compress / dW / fwd
def test_compress_definition_and_special_cases():
    rng = np.random.default_rng(12)
    X = rng.standard_normal((5, 7))
    P = si.orthonormal_basis(7, 3, 13)
    C = orc.compress(X, P)
    for n in range(5):
        for j in range(3):
            assert np.isclose(C[n, j], sum(X[n, a] * P[a, j] for a in range(7)), rtol=1e-13)
    # identity columns pick out the first c channels
    assert np.array_equal(orc.compress(X, np.eye(7)[:, :4]), X[:, :4])
    # with the exact principal basis the first block carries the top-k energy
    Xe, R, sig = _exact_case()
    Pk, _ = orc.fit_basis(Xe, 5, 3, seed=1, draw=0)
    assert np.isclose(np.sum(orc.compress(Xe, Pk)[:, :5] ** 2), np.sum(sig[:5] ** 2), rtol=1e-10)


def test_weight_grad_definition_by_loops():
    rng = np.random.default_rng(14)
    N, d, m, k, r = 6, 8, 3, 2, 3
    X = rng.standard_normal((N, d))
    dY = rng.standard_normal((N, m))
    P, s = orc.fit_basis(X, k, r, seed=2, draw=0)
    C = orc.compress(X, P)
    dW = orc.weight_grad(C, dY, P, k, s)
    for a in range(d):
        for b in range(m):
            acc = 0.0
            for n in range(N):
                xt = sum(C[n, j] * P[a, j] * (1.0 if j < k else s) for j in range(k + r))
                acc += xt * dY[n, b]
            assert np.isclose(dW[a, b], acc, rtol=1e-12, atol=1e-14)
    # the reassociated form P_s (C^T dY) is the same matrix
    Ps = P * np.concatenate([np.ones(k), np.full(r, s)])[None, :]
    assert np.allclose(Ps @ (C.T @ dY), dW, rtol=1e-12, atol=1e-14)
    # linear in dY
    dY2 = rng.standard_normal((N, m))
    assert np.allclose(orc.weight_grad(C, dY + 2 * dY2, P, k, s),
                       dW + 2 * orc.weight_grad(C, dY2, P, k, s), rtol=1e-12)


def test_weight_grad_exact_when_complement_is_full():
    # r = d - k  =>  dW = X^T dY, the textbook linear-layer gradient (Lemma 1)
    rng = np.random.default_rng(15)
    X = rng.standard_normal((20, 9))
    dY = rng.standard_normal((20, 4))
    P, s = orc.fit_basis(X, 3, 6, seed=4, draw=2)
    dW = orc.weight_grad(orc.compress(X, P), dY, P, 3, s)
    assert np.allclose(dW, X.T @ dY, rtol=1e-11, atol=1e-12)
    # and dY = X A gives dW = G A
    A = rng.standard_normal((9, 4))
    assert np.allclose(orc.weight_grad(orc.compress(X, P), X @ A, P, 3, s),
                       orc.gram(X) @ A, rtol=1e-11, atol=1e-12)


def test_forward_definition():
    rng = np.random.default_rng(16)
    X, W = rng.standard_normal((4, 5)), rng.standard_normal((5, 3))
    Y = orc.forward(X, W)
    assert np.isclose(Y[2, 1], sum(X[2, a] * W[a, 1] for a in range(5)), rtol=1e-13)
