"""Seeded synthetic inputs shared by the oracle-side and the HIP-side tests.

Holds none of the method's arithmetic: only the recipes that stand in for
LLaMA activations (a power-law singular spectrum with a few outlier
channels, standing in for the paper's qualitative picture of a few dominant
singular values followed by a long, slowly decaying tail) and for the
upstream gradient dY, plus exact bf16 <-> fp64 conversions.

Small cases are drawn with numpy's PCG64 in fp64 so that tests are
reproducible bit for bit on any machine.  Full-size cases (tens of millions
of elements) can be drawn on a torch device with torch's seeded generator;
the recipe is the same, the random stream is not.
"""
from __future__ import annotations

import numpy as np
import torch


# ----------------------------------------------------------------- dtype I/O
def round_to(x: np.ndarray, dtype: str) -> torch.Tensor:
    """Round an fp64 numpy array to 'f32' or 'bf16' (round-to-nearest-even)
    and return a CPU torch tensor of that dtype."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float64))
    if dtype == "f32":
        return t.to(torch.float32)
    if dtype == "bf16":
        return t.to(torch.float32).to(torch.bfloat16)
    raise ValueError(dtype)


def as_f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of any torch tensor (bf16 / fp32 / fp64, any device) to
    a numpy fp64 array."""
    return t.detach().to("cpu").to(torch.float64).numpy()


# ------------------------------------------------------------------- recipes
def haar_orthogonal(d: int, rng: np.random.Generator) -> np.ndarray:
    """Haar-distributed d x d orthogonal matrix: Q factor of a Gaussian
    matrix with the sign convention diag(R) > 0."""
    Q, R = np.linalg.qr(rng.standard_normal((d, d)))
    return Q * np.where(np.diag(R) < 0.0, -1.0, 1.0)[None, :]


def power_law_sigma(d: int, alpha: float) -> np.ndarray:
    return np.arange(1, d + 1, dtype=np.float64) ** (-alpha)


def outlier_channels(d: int, n_out: int, rng: np.random.Generator) -> np.ndarray:
    """The first n_out entries of a seeded permutation of the d channels."""
    return rng.permutation(d)[:n_out]


def activation(N: int, d: int, alpha: float, seed: int, n_out: int = 0,
               out_scale: float = 1.0, exact_spectrum: bool = False,
               sigma: np.ndarray | None = None, batch: int = 0):
    """X = Z diag(sigma) R (fp64) with Z ~ N(0,1) (N x d), sigma_i = i^-alpha,
    R Haar; then n_out channels (columns) multiplied by out_scale.  `batch` > 0
    draws another Z for the same R and channels: the next batch of one layer.

    exact_spectrum=True replaces Z by an N x d matrix with orthonormal
    columns, so that (without outliers) the singular values of X are exactly
    sigma and its top-k right singular vectors are the first k rows of R.
    Returns (X, info) with info = dict(R=, sigma=, channels=).
    """
    rng = np.random.default_rng(seed)
    sig = power_law_sigma(d, alpha) if sigma is None else np.asarray(sigma, dtype=np.float64)
    Z = rng.standard_normal((N, d))
    if batch:
        Z = np.random.default_rng([seed, batch]).standard_normal((N, d))
    if exact_spectrum:
        if N < d:
            raise ValueError("exact_spectrum needs N >= d")
        Z, _ = np.linalg.qr(Z)
    R = haar_orthogonal(d, rng)
    X = (Z * sig[None, :]) @ R
    ch = outlier_channels(d, n_out, rng) if n_out else np.zeros(0, dtype=np.int64)
    if n_out:
        X[:, ch] *= out_scale
    return X, dict(R=R, sigma=sig, channels=ch)


def grad_output(N: int, m: int, std: float, seed: int) -> np.ndarray:
    """dY ~ N(0, std^2) i.i.d. (fp64)."""
    return np.random.default_rng(seed).standard_normal((N, m)) * std


def orthonormal_basis(d: int, c: int, seed: int) -> np.ndarray:
    """Any d x c matrix with orthonormal columns (a stand-in basis for tests
    of compress / weight-grad that do not need a fitted one)."""
    Q, _ = np.linalg.qr(np.random.default_rng(seed).standard_normal((d, c)))
    return Q


# ------------------------------------------------- full-size, on a torch device
def activation_torch(N: int, d: int, alpha: float, seed: int, n_out: int,
                     out_scale: float, dtype: torch.dtype, device,
                     ld: int | None = None, chunk: int = 4096, batch: int = 0,
                     gap_after: int = 0, gap_shrink: float = 1.0) -> torch.Tensor:
    """Same recipe as activation(), drawn with torch's generator on `device`
    in fp32 and rounded to `dtype`.  `seed` fixes the layer (R, sigma, outlier
    channels); `batch` picks the token draw Z, so that different batches of one
    layer share their spectrum and principal subspace, as successive training
    batches do.  Returns an (N, d) view into an (N, ld) buffer when ld > d
    (padded leading dimension).  gap_after = k > 0 multiplies sigma_{k+1..d} by gap_shrink, which opens an
    eigenvalue gap after the k-th direction (for tests that compare projectors)."""
    # the layer's mixing matrix diag(sigma) R is built on the host (numpy QR), like activation()
    rng = np.random.default_rng(seed)
    sig = power_law_sigma(d, alpha)
    if gap_after > 0:
        sig[gap_after:] *= gap_shrink
    M64 = sig[:, None] * haar_orthogonal(d, rng)
    if n_out:
        M64[:, outlier_channels(d, n_out, rng)] *= out_scale
    M = torch.from_numpy(M64.astype(np.float32)).to(device)
    gz = torch.Generator(device=device)
    gz.manual_seed(seed * 1000003 + 17 * batch + 1)
    ld = d if ld is None else ld
    buf = torch.zeros((N, ld), device=device, dtype=dtype)
    for r0 in range(0, N, chunk):
        r1 = min(N, r0 + chunk)
        Z = torch.randn((r1 - r0, d), generator=gz, device=device, dtype=torch.float32)
        buf[r0:r1, :d] = (Z @ M).to(dtype)
    return buf[:, :d]


def grad_output_torch(N: int, m: int, std: float, seed: int, dtype: torch.dtype,
                      device, ld: int | None = None) -> torch.Tensor:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    ld = m if ld is None else ld
    buf = torch.zeros((N, ld), device=device, dtype=dtype)
    buf[:, :m] = (torch.randn((N, m), generator=g, device=device, dtype=torch.float32) * std).to(dtype)
    return buf[:, :m]
