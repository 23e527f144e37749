"""fp64 CPU oracle for the PRAC per-layer path.  TEST INFRASTRUCTURE ONLY.

This module is the slow, plain reference that the HIP library is checked
against.  Only tests, the smoke check and the bench's cpu_baseline leg may
import it; the product path never does.  It shares no code, tables or
helpers with the HIP sources, and every function takes and returns plain
numpy float64 / integer arrays.

Notation follows the paper with the repo's names in brackets:
  X  (N x d)   saved input activation of a linear layer, d = paper's n
  Q1 [U_k]     d x k   top-k right singular vectors of X, k = paper's r_1
  Q2 [Q_r]     d x r   orthonormal basis of (I - Q1 Q1^T) S, r = paper's r_2
  s            (d - k) / r, the paper's scaling factor (its symbol is k)
  P            [Q1 | Q2], kept UNSCALED; s is applied at reconstruction
  C            X P  (N x (k+r)), the compressed activation

Every function below is pinned by tests/test_oracle_*.py against something
other than itself (published Philox known answers, closed-form spectra,
Gram-Schmidt, Lemma 4 / Theorem 1 / the variance identity by Monte Carlo,
the r = d - k exactness case, textbook GEMM).  No function here is
"parity unpinned".
"""
from __future__ import annotations

import numpy as np

_U32 = np.uint64(0xFFFFFFFF)

# --------------------------------------------------------------------------
# Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): the counter-based
# generator behind "S_ij ~ i.i.d. N(0,1)" (Section 4.3, Eq. S_o; Alg. 1).
# The paper fixes only the distribution; the stream layout is this build's.
# --------------------------------------------------------------------------
_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = np.uint64(0x9E3779B9)
_PHILOX_W1 = np.uint64(0xBB67AE85)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Ten Philox-4x32 rounds on arrays of 32-bit counters.

    All arguments are integer arrays (or scalars) holding values < 2**32;
    returns four uint64 arrays with values < 2**32.
    """
    c0 = np.asarray(c0, dtype=np.uint64) & _U32
    c1 = np.asarray(c1, dtype=np.uint64) & _U32
    c2 = np.asarray(c2, dtype=np.uint64) & _U32
    c3 = np.asarray(c3, dtype=np.uint64) & _U32
    k0 = np.asarray(k0, dtype=np.uint64) & _U32
    k1 = np.asarray(k1, dtype=np.uint64) & _U32
    for rnd in range(10):
        if rnd > 0:  # the key is bumped between rounds (nine bumps in all)
            k0 = (k0 + _PHILOX_W0) & _U32
            k1 = (k1 + _PHILOX_W1) & _U32
        p0 = _PHILOX_M0 * c0  # full 64-bit products of 32-bit operands
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _U32
        hi1, lo1 = p1 >> np.uint64(32), p1 & _U32
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return c0, c1, c2, c3


def philox_words(seed: int, draw: int, stream: int, n: int) -> np.ndarray:
    """First n 32-bit words of the stream (seed, draw, stream).

    Block b (counter = (b_lo, b_hi, stream, draw), key = (seed_lo, seed_hi))
    yields words 4b .. 4b+3, so element idx depends on (seed, draw, stream,
    idx) only.
    """
    if not (0 <= draw < 2**32 and 0 <= stream < 2**32 and 0 <= seed < 2**64):
        raise ValueError("seed < 2^64, draw < 2^32, stream < 2^32 required")
    nblk = (n + 3) // 4
    blk = np.arange(nblk, dtype=np.uint64)
    x = philox4x32_10(blk & _U32, blk >> np.uint64(32),
                      np.uint64(stream), np.uint64(draw),
                      np.uint64(seed & 0xFFFFFFFF), np.uint64(seed >> 32))
    return np.stack(x, axis=1).reshape(-1)[:n].astype(np.uint32)


def words_to_uniform(words: np.ndarray) -> np.ndarray:
    """u = ((w >> 9) + 1/2) * 2^-23: an odd multiple of 2^-24 in (0, 1),
    exactly representable in fp32 and fp64."""
    return ((words.astype(np.uint64) >> np.uint64(9)).astype(np.float64) + 0.5) * 2.0 ** -23


def philox_normal(seed: int, draw: int, stream: int, n: int) -> np.ndarray:
    """n standard normals by Box-Muller on consecutive word pairs:
    z_{2j} = sqrt(-2 ln u_{2j}) cos(2 pi u_{2j+1}), z_{2j+1} the sine twin."""
    n4 = 4 * ((n + 3) // 4)
    u = words_to_uniform(philox_words(seed, draw, stream, n4))
    rad = np.sqrt(-2.0 * np.log(u[0::2]))
    ang = 2.0 * np.pi * u[1::2]
    z = np.empty(n4, dtype=np.float64)
    z[0::2] = rad * np.cos(ang)
    z[1::2] = rad * np.sin(ang)
    return z[:n]


STREAM_V0 = 0  # start block of the subspace iteration (GPU side only)
STREAM_S = 1   # the Gaussian matrix S of Eq. (S_o)


def gaussian_matrix(seed: int, draw: int, rows: int, cols: int,
                    stream: int = STREAM_S) -> np.ndarray:
    """S (rows x cols), S_ij ~ N(0,1); element (i, j) is stream index
    i*cols + j."""
    return philox_normal(seed, draw, stream, rows * cols).reshape(rows, cols)


# --------------------------------------------------------------------------
# Principal subspace (Section 4.2 PAC; Alg. 1, principal-subspace update)
# --------------------------------------------------------------------------
def gram(X: np.ndarray, row_stride: int = 1) -> np.ndarray:
    """G = Xs^T Xs over rows 0, stride, 2*stride, ... of X.  The right
    singular vectors of X are the eigenvectors of X^T X."""
    Xs = np.asarray(X, dtype=np.float64)[::row_stride]
    return Xs.T @ Xs


def principal_subspace(G: np.ndarray, k: int):
    """Top-k eigenvectors of the symmetric PSD matrix G, by a full symmetric
    eigendecomposition.  Returns (Q1 (d x k), all eigenvalues descending)."""
    lam, V = np.linalg.eigh(np.asarray(G, dtype=np.float64))
    order = np.argsort(lam)[::-1]
    lam = lam[order]
    return V[:, order[:k]].copy(), lam


# --------------------------------------------------------------------------
# Random complement basis (Section 4.3, Eq. (S_o); Lemma 4)
# --------------------------------------------------------------------------
def thin_qr_positive(A: np.ndarray):
    """Thin QR with diag(R) > 0 (the unique factorisation that Lemma 1 and
    Lemma 4 rely on)."""
    Q, R = np.linalg.qr(A, mode="reduced")
    sgn = np.where(np.diag(R) < 0.0, -1.0, 1.0)
    return Q * sgn[None, :], R * sgn[:, None]


def complement_basis(Q1: np.ndarray, S: np.ndarray) -> np.ndarray:
    """Q2 = Q-factor of S_o = (I - Q1 Q1^T) S.  The projection is applied
    twice so that Q1^T Q2 vanishes to rounding."""
    So = np.asarray(S, dtype=np.float64).copy()
    if Q1.shape[1] > 0:
        for _ in range(2):
            So = So - Q1 @ (Q1.T @ So)
    Q2, _ = thin_qr_positive(So)
    return Q2


def scaling_factor(d: int, k: int, r: int) -> float:
    """The paper's scaling factor (n - r_1) / r_2 (Theorem 1; Alg. 1 line 1)."""
    return (d - k) / r


def fit_basis(X: np.ndarray, k: int, r: int, seed: int, draw: int,
              row_stride: int = 1):
    """P = [Q1 | Q2] (d x (k+r), unscaled) and s = (d-k)/r, as in the two
    refresh branches of Alg. 1 taken together."""
    d = X.shape[1]
    if k > 0:
        Q1, _ = principal_subspace(gram(X, row_stride), k)
    else:
        Q1 = np.zeros((d, 0))
    if r > 0:
        Q2 = complement_basis(Q1, gaussian_matrix(seed, draw, d, r))
        s = scaling_factor(d, k, r)
    else:
        Q2 = np.zeros((d, 0))
        s = 0.0
    return np.concatenate([Q1, Q2], axis=1), s


# --------------------------------------------------------------------------
# Compress / reconstruct / weight gradient (Alg. 1 compression step; Alg. 2
# backward; Lemma 1)
# --------------------------------------------------------------------------
def compress(X: np.ndarray, P: np.ndarray) -> np.ndarray:
    """C = X P = [X Q1 | X Q2]; the scale is NOT folded in here."""
    return np.asarray(X, dtype=np.float64) @ np.asarray(P, dtype=np.float64)


def reconstruct(C: np.ndarray, P: np.ndarray, k: int, scale: float) -> np.ndarray:
    """X~ = C_1 Q1^T + scale * C_2 Q2^T (Alg. 2 backward, with the
    transposes the listing omits)."""
    C = np.asarray(C, dtype=np.float64)
    P = np.asarray(P, dtype=np.float64)
    return C[:, :k] @ P[:, :k].T + scale * (C[:, k:] @ P[:, k:].T)


def weight_grad(C: np.ndarray, dY: np.ndarray, P: np.ndarray, k: int,
                scale: float) -> np.ndarray:
    """dW = X~^T dY in the paper's order: reconstruct first, then the
    ordinary linear-layer weight gradient (Lemma 1)."""
    return reconstruct(C, P, k, scale).T @ np.asarray(dY, dtype=np.float64)


def forward(X: np.ndarray, W: np.ndarray) -> np.ndarray:
    """Y = X W with W stored d x m (Lemma 1's layout)."""
    return np.asarray(X, dtype=np.float64) @ np.asarray(W, dtype=np.float64)
