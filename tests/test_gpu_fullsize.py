"""Parity at the configurations' full sizes (bf16), in the launch configuration bench.py
times (packed basis and packed C handed in, bf16 dW).  At the LLaMA-1B / LLaMA-130M / rank-sweep
shapes EVERY output element is compared with the fp64 oracle; only the LLaMA-7B shapes, where the
oracle's own product would take minutes, are compared on sampled columns.  Inputs are drawn on the
device by the seeded recipes of synth_inputs; the C handed to the weight gradient is a torch
product (an input recipe, not the library under test).

Two criteria per output:
  * relative Frobenius error <= 1e-2 over the whole output (the stated bf16 tolerance) and over
    every 128-row (column) tile of it, so that one wrong tile cannot hide in the total;
  * an element-wise bound that follows from the arithmetic.  With u = 2^-8 (the unit roundoff of bf16: 8 significant bits):
      C  = X P         P is rounded to bf16, C once more:  |err| <= u sum|x||p| + u|C| <= 2u |x_n| |p_j|
      X~ = C Ps^T      Ps rounded, X~ rounded:             |err| <= 2u |c_n| |ps_i|
      Y  = X W         only Y is rounded (fp32 sums):      |err| <= u |Y| (1 + 2^-6) + 2^-14 |x_n| |w_j|
      dW = Ps (C^T dY) T = C^T dY and Ps rounded, dW rounded: |err| <= 3u |ps_i| |t_j|, checked against 4u
    (|.| of a vector: its 2-norm; Cauchy-Schwarz bounds the sums).  fp32 accumulation adds terms of
    the order of 1e-6 of the same products, far inside the slack of each bound.
"""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import prac_oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
N = 32768
U = 2.0 ** -8


@pytest.fixture(scope="module")
def ctx():
    from paper_2602_23111_amd.prac import Prac

    p = Prac(0)
    yield p
    p.close()


def rel_fro(got, ref):
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))


def sample_rows(n, count, seed):
    idx = np.random.default_rng(seed).choice(n - 8, size=count - 8, replace=False)
    return np.sort(np.concatenate([idx, np.arange(n - 8, n)]))      # always include the last rows


class Parity:
    """Accumulates the comparison of one output matrix, handed over in row chunks."""

    def __init__(self, what, tile_rows=128):
        self.what, self.tile_rows = what, tile_rows
        self.err2 = self.ref2 = 0.0
        self.worst_tile = 0.0
        self.worst_elem = 0.0     # max over elements of |err| / bound

    def add(self, got, ref, bound):
        err = np.abs(got - ref)
        self.err2 += float(np.sum(err * err))
        self.ref2 += float(np.sum(ref * ref))
        self.worst_elem = max(self.worst_elem, float(np.max(err / bound)))
        t = self.tile_rows
        for r0 in range(0, got.shape[0], t):
            e = np.linalg.norm(err[r0:r0 + t])
            self.worst_tile = max(self.worst_tile, float(e / max(np.linalg.norm(ref[r0:r0 + t]), 1e-300)))

    def check(self):
        total = np.sqrt(self.err2 / self.ref2)
        assert total < 1e-2, f"{self.what}: relative Frobenius error {total:.3e}"
        assert self.worst_tile < 1e-2, f"{self.what}: worst row tile {self.worst_tile:.3e}"
        assert self.worst_elem <= 1.0, f"{self.what}: element error at {self.worst_elem:.3f} of its bound"


def check_compress_all_rows(X, Cm, P64, chunk=8192):
    par = Parity("C")
    pn = np.linalg.norm(P64, axis=0)[None, :]
    for r0 in range(0, X.shape[0], chunk):
        X64 = si.as_f64(X[r0:r0 + chunk])
        ref = orc.compress(X64, P64)
        par.add(si.as_f64(Cm[r0:r0 + chunk]), ref, 2 * U * np.linalg.norm(X64, axis=1)[:, None] * pn + 1e-300)
    par.check()


def scaled_row_norms(P64, k, s):
    w = np.concatenate([np.ones(k), np.full(P64.shape[1] - k, s)])
    return np.linalg.norm(P64 * w[None, :], axis=1)


def check_weight_grad_columns(dW, C64, dY64, P64, k, s, cols=None):
    """dW (d x m, device) against the oracle (paper order: reconstruct, then X~^T dY) on the given
    columns (all of them when cols is None); tiles are 128 columns wide."""
    ref = orc.weight_grad(C64, dY64, P64, k, s)
    got = si.as_f64(dW if cols is None else dW[:, cols])
    T = C64.T @ dY64                                  # only for the bound: |t_j|
    bound = 4 * U * scaled_row_norms(P64, k, s)[:, None] * np.linalg.norm(T, axis=0)[None, :] + 1e-300
    par = Parity("dW", tile_rows=128)
    par.add(got.T, ref.T, bound.T)                    # row tiles of the transpose = column tiles of dW
    if cols is not None:
        par.worst_tile = 0.0                          # sampled columns are not tiles
    par.check()


# ------------------------------------------------------------------------ compress
COMPRESS_SHAPES = [
    # d, ldx, k, r, alpha, outliers, factor
    (2048, 2048, 128, 128, 0.8, 8, 30.0),    # LLaMA-1B attention / up / gate input (headline)
    (5461, 5464, 128, 128, 0.8, 8, 30.0),    # LLaMA-1B down input (padded leading dimension)
    (768, 768, 64, 64, 1.0, 4, 20.0),        # LLaMA-130M attention / up / gate input
    (2048, 2048, 64, 64, 1.0, 4, 20.0),      # LLaMA-130M down input; rank sweep (64, 64)
    (2048, 2048, 0, 256, 0.5, 0, 1.0),       # rank sweep: random-only basis
    (2048, 2048, 256, 256, 1.5, 0, 1.0),     # rank sweep (256, 256)
    (2048, 2048, 512, 512, 0.8, 0, 1.0),     # rank sweep (512, 512)
]


@pytest.mark.parametrize("d,ldx,k,r,alpha,n_out,factor", COMPRESS_SHAPES)
def test_compress_full_size_every_row(ctx, d, ldx, k, r, alpha, n_out, factor):
    from paper_2602_23111_amd.prac import C_PACKED
    c = k + r
    X = si.activation_torch(N, d, alpha, 3000, n_out, factor, torch.bfloat16, DEV, ld=ldx)
    P32 = si.round_to(si.orthonormal_basis(d, c, seed=1), "f32")
    Pd = P32.to(DEV)
    flat = ctx.compress(X, Pd, P_lp=ctx.pack_basis(Pd), layout=C_PACKED)      # as bench.py launches it
    Cm = ctx.unpack_compressed(flat, N, c)
    torch.cuda.synchronize()
    assert torch.equal(Cm, ctx.compress(X, Pd, P_lp=ctx.pack_basis(Pd)))       # row-major launch agrees
    check_compress_all_rows(X, Cm, si.as_f64(P32))


# ------------------------------------------------------------------ weight gradient
WGRAD_SHAPES = [
    # d, m, lddy, k, r
    (2048, 2048, 2048, 128, 128),     # LLaMA-1B attention projections (headline)
    (2048, 5461, 5464, 128, 128),     # LLaMA-1B up / gate
    (5461, 2048, 2048, 128, 128),     # LLaMA-1B down
    (768, 768, 768, 64, 64),          # LLaMA-130M attention projections
    (768, 2048, 2048, 64, 64),        # LLaMA-130M up / gate
    (2048, 768, 768, 64, 64),         # LLaMA-130M down
    (2048, 2048, 2048, 0, 256),       # rank sweep
    (2048, 2048, 2048, 64, 64),
    (2048, 2048, 2048, 256, 256),
    (2048, 2048, 2048, 512, 512),
]


@pytest.mark.parametrize("d,m,lddy,k,r", WGRAD_SHAPES)
def test_weight_grad_full_size_every_element(ctx, d, m, lddy, k, r):
    from paper_2602_23111_amd.prac import C_PACKED
    from test_gpu_parity import pack_c_reference
    c = k + r
    s = orc.scaling_factor(d, k, r)
    X = si.activation_torch(N, d, 0.8, 3001, 8, 30.0, torch.bfloat16, DEV)
    P32 = si.round_to(si.orthonormal_basis(d, c, seed=3), "f32")
    Pd = P32.to(DEV)
    Cin = torch.empty((N, c), dtype=torch.bfloat16, device=DEV)
    for r0 in range(0, N, 4096):
        Cin[r0:r0 + 4096] = (X[r0:r0 + 4096].float() @ Pd).to(torch.bfloat16)
    del X
    dY = si.grad_output_torch(N, m, 1e-3, 3101, torch.bfloat16, DEV, ld=lddy)
    Cpk = pack_c_reference(Cin.cpu()).to(DEV)
    dW = ctx.weight_grad(Cpk, dY, Pd, k, r, s, P_lp=ctx.pack_basis(Pd), out_dtype=torch.bfloat16, layout=C_PACKED)
    dW_rm = ctx.weight_grad(Cin, dY, Pd, k, r, s, P_lp=ctx.pack_basis(Pd), out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert torch.equal(dW, dW_rm)
    check_weight_grad_columns(dW, si.as_f64(Cin), si.as_f64(dY), si.as_f64(P32), k, s)


def test_weight_grad_shared_full_size_every_element(ctx):
    # query / key / value gradients from the one compressed activation they share (Section 5.1)
    from paper_2602_23111_amd.prac import C_PACKED
    from test_gpu_parity import pack_c_reference
    d, m, k, r = 2048, 2048, 128, 128
    c = k + r
    s = orc.scaling_factor(d, k, r)
    X = si.activation_torch(N, d, 0.8, 3001, 8, 30.0, torch.bfloat16, DEV)
    P32 = si.round_to(si.orthonormal_basis(d, c, seed=3), "f32")
    Pd = P32.to(DEV)
    Cin = torch.empty((N, c), dtype=torch.bfloat16, device=DEV)
    for r0 in range(0, N, 4096):
        Cin[r0:r0 + 4096] = (X[r0:r0 + 4096].float() @ Pd).to(torch.bfloat16)
    del X
    dYs = [si.grad_output_torch(N, m, 1e-3, 3110 + h, torch.bfloat16, DEV) for h in range(3)]
    Cpk = pack_c_reference(Cin.cpu()).to(DEV)
    lp = ctx.pack_basis(Pd)
    outs = ctx.weight_grad_shared(Cpk, dYs, Pd, k, r, s, P_lp=lp, out_dtype=torch.bfloat16, layout=C_PACKED)
    torch.cuda.synchronize()
    C64, P64 = si.as_f64(Cin), si.as_f64(P32)
    for dYh, dWh in zip(dYs, outs):
        check_weight_grad_columns(dWh, C64, si.as_f64(dYh), P64, k, s)


# ------------------------------------------------------------------------- Gram, fit
def test_gram_full_size_every_element(ctx):
    # the streaming Gram path at the headline size against the oracle's X^T X, element by element: fp32 sums
    # of N bf16 products, |err| <= a few 1e-6 of |x_i| |x_j| (column norms), checked against 2e-5 of it
    d = 2048
    X = si.activation_torch(N, d, 0.8, 3000, 8, 30.0, torch.bfloat16, DEV)
    G = ctx.gram(X)
    torch.cuda.synchronize()
    X64 = si.as_f64(X)
    ref = orc.gram(X64)
    got = si.as_f64(G)
    cn = np.linalg.norm(X64, axis=0)
    assert rel_fro(got, ref) < 2e-5
    assert np.max(np.abs(got - ref) / (cn[:, None] * cn[None, :])) < 2e-5
    assert np.array_equal(got, got.T)


def test_fit_basis_full_size_projector_with_gap(ctx):
    # the cold fit at the headline size on an activation whose spectrum drops after the k-th direction:
    # projector of Q1 against the oracle's exact top-k eigenvectors of X^T X
    d, k, r = 2048, 128, 128
    X = si.activation_torch(N, d, 0.8, 3000, 8, 30.0, torch.bfloat16, DEV, gap_after=k, gap_shrink=0.8)
    P, _, _ = ctx.fit_basis(X, k, r, seed=1234, draw=0)
    ctx.sync_status()
    Q1, lam = orc.principal_subspace(orc.gram(si.as_f64(X)), k)
    assert lam[k - 1] / lam[k] >= 1.05
    U = si.as_f64(P)[:, :k]
    assert np.abs(U @ U.T - Q1 @ Q1.T).max() < 1e-3
    P64 = si.as_f64(P)
    assert np.abs(P64.T @ P64 - np.eye(k + r)).max() < 1e-5


def test_fit_basis_full_size_invariants(ctx):
    d, k, r = 2048, 128, 128
    X = si.activation_torch(N, d, 0.8, 3000, 8, 30.0, torch.bfloat16, DEV)
    P, lp, scale = ctx.fit_basis(X, k, r, seed=1234, draw=0)
    ctx.sync_status()
    P64 = si.as_f64(P)
    assert np.abs(P64.T @ P64 - np.eye(k + r)).max() < 1e-5
    assert scale == pytest.approx((d - k) / r)
    # energy captured by Q1 against the exact top-k eigenvalue sum of X^T X (oracle)
    X64 = si.as_f64(X)
    _, lam = orc.principal_subspace(orc.gram(X64), k)
    captured = float(np.sum((X64 @ P64[:, :k]) ** 2))
    assert captured >= (1 - 1e-3) * lam[:k].sum()
    assert captured <= (1 + 1e-6) * lam[:k].sum()


@pytest.mark.parametrize("k,r", [(128, 128), (512, 512)])      # headline ranks; the rank sweep's widest basis
def test_fit_basis_warm_start_as_benchmarked(ctx, k, r):
    # the refits inside bench.py's timed region: next batch of the same layer, two Gram-free tracking
    # steps from the previous Q1 (no oversampling).  These spectra have no gap at k, so what is checked
    # is what is unique: orthonormality and the energy inside / outside Q1.
    d = 2048
    X0 = si.activation_torch(N, d, 0.8, 3000, 8, 30.0, torch.bfloat16, DEV, batch=0)
    X1 = si.activation_torch(N, d, 0.8, 3000, 8, 30.0, torch.bfloat16, DEV, batch=1)
    P, _, _ = ctx.fit_basis(X0, k, r, seed=1234, draw=0)
    P, _, scale = ctx.fit_basis(X1, k, r, seed=1234, draw=1, P=P, warm_start=True, iters=2, oversample=-1)
    ctx.sync_status()
    P64 = si.as_f64(P)
    assert np.abs(P64.T @ P64 - np.eye(k + r)).max() < 1e-5
    X64 = si.as_f64(X1)
    _, lam = orc.principal_subspace(orc.gram(X64), k)
    captured = float(np.sum((X64 @ P64[:, :k]) ** 2))
    assert (1 - 1e-3) * lam[:k].sum() <= captured <= (1 + 1e-6) * lam[:k].sum()
    # what the estimator's variance is proportional to: the energy left outside Q1 (Theorem 2) is within
    # 1 % of the smallest possible (the exact top-k subspace)
    total = float(np.sum(X64 ** 2))
    assert total - captured <= 1.01 * (total - lam[:k].sum())


# ---------------------------------------------------------------- fused forward
@pytest.mark.parametrize("w_layout,m", [(0, 2048), (1, 2048), (1, 6144)])   # 6144: query, key and value in one launch
def test_fused_forward_full_size_every_row(ctx, w_layout, m):
    from paper_2602_23111_amd.prac import C_PACKED
    d, k, r = 2048, 128, 128
    c = k + r
    X = si.activation_torch(N, d, 0.8, 3000, 8, 30.0, torch.bfloat16, DEV)
    g = torch.Generator(device=DEV)
    g.manual_seed(7)
    W = (torch.randn((d, m) if w_layout == 0 else (m, d), generator=g, device=DEV) * 0.02).to(torch.bfloat16)
    P32 = si.round_to(si.orthonormal_basis(d, c, seed=1), "f32")
    Pd = P32.to(DEV)
    lp = ctx.pack_basis(Pd)
    Y, flat = ctx.compress_fused_fwd(X, W, Pd, w_layout=w_layout, P_lp=lp, layout=C_PACKED)
    torch.cuda.synchronize()
    Cm = ctx.unpack_compressed(flat, N, c)
    check_compress_all_rows(X, Cm, si.as_f64(P32))
    W64 = si.as_f64(W if w_layout == 0 else W.t())
    wn = np.linalg.norm(W64, axis=0)[None, :]
    par = Parity("Y")
    for r0 in range(0, N, 8192):
        X64 = si.as_f64(X[r0:r0 + 8192])
        ref = orc.forward(X64, W64)
        bound = U * (1 + 2.0 ** -6) * np.abs(ref) + 2.0 ** -14 * np.linalg.norm(X64, axis=1)[:, None] * wn
        par.add(si.as_f64(Y[r0:r0 + 8192]), ref, bound + 1e-300)
    par.check()


# --------------------------------------------------------------- reconstruction
def test_reconstruct_full_size_every_row(ctx):
    from paper_2602_23111_amd.prac import C_PACKED
    d, k, r = 2048, 128, 128
    c = k + r
    s = orc.scaling_factor(d, k, r)
    X = si.activation_torch(N, d, 0.8, 3000, 8, 30.0, torch.bfloat16, DEV)
    P32 = si.round_to(si.orthonormal_basis(d, c, seed=1), "f32")
    Pd = P32.to(DEV)
    flat = ctx.compress(X, Pd, P_lp=ctx.pack_basis(Pd), layout=C_PACKED)
    Cm = ctx.unpack_compressed(flat, N, c)
    Xh = ctx.reconstruct(flat, Pd, k, r, s, N=N, layout=C_PACKED)
    torch.cuda.synchronize()
    assert torch.equal(Xh, ctx.reconstruct(Cm, Pd, k, r, s))
    P64 = si.as_f64(P32)
    pn = scaled_row_norms(P64, k, s)[None, :]
    par = Parity("X~")
    for r0 in range(0, N, 8192):
        C64 = si.as_f64(Cm[r0:r0 + 8192])
        ref = orc.reconstruct(C64, P64, k, s)
        par.add(si.as_f64(Xh[r0:r0 + 8192]), ref, 2 * U * np.linalg.norm(C64, axis=1)[:, None] * pn + 1e-300)
    par.check()


# ---- LLaMA-7B-shaped layer (N = 16384; up / gate 4096 -> 11008, down 11008 -> 4096; k = r = 256; spectrum
# i^-0.8 with 16 outlier channels x50; the basis refitted every step from every fourth token)
N7, K7, R7 = 16384, 256, 256


@pytest.mark.parametrize("d,m", [(4096, 11008), (11008, 4096)])
def test_llama7b_layer_compress_and_weight_grad(ctx, d, m):
    from paper_2602_23111_amd.prac import C_PACKED
    c = K7 + R7
    s = orc.scaling_factor(d, K7, R7)
    X = si.activation_torch(N7, d, 0.8, 5000, 16, 50.0, torch.bfloat16, DEV)
    P32 = si.round_to(si.orthonormal_basis(d, c, seed=11), "f32")
    Pd = P32.to(DEV)
    lp = ctx.pack_basis(Pd)
    flat = ctx.compress(X, Pd, P_lp=lp, layout=C_PACKED)
    Cm = ctx.unpack_compressed(flat, N7, c)
    torch.cuda.synchronize()
    check_compress_all_rows(X, Cm, si.as_f64(P32), chunk=4096)       # every row of C
    del X
    # the weight gradient from the library's own packed C, against the oracle's on the same (rounded) C,
    # on sampled columns: the oracle's reconstruct-then-multiply takes minutes for all of them here
    dY = si.grad_output_torch(N7, m, 1e-3, 5100, torch.bfloat16, DEV)
    dW = ctx.weight_grad(flat, dY, Pd, K7, R7, s, P_lp=lp, out_dtype=torch.bfloat16, layout=C_PACKED)
    torch.cuda.synchronize()
    cols = np.sort(np.concatenate([np.random.default_rng(13).choice(m - 2, size=46, replace=False), [m - 2, m - 1]]))
    cols_t = torch.from_numpy(cols).to(DEV)
    check_weight_grad_columns(dW, si.as_f64(Cm), si.as_f64(dY[:, cols_t]), si.as_f64(P32), K7, s, cols=cols_t)
    # every 128-column tile of dW carries the energy its share of T predicts (no tile left unwritten or
    # written twice): ||dW[:, tile]||_F against ||Ps T[:, tile]||_F from an fp32 product on the device
    T = (Cm.float().t() @ dY.float())
    w = torch.cat([torch.ones(K7, device=DEV), torch.full((R7,), s, device=DEV)])
    ref = Pd @ (w[:, None] * T)
    for c0 in range(0, m, 128):
        a, b = float(dW[:, c0:c0 + 128].float().norm()), float(ref[:, c0:c0 + 128].norm())
        assert abs(a - b) <= 1e-2 * b, (c0, a, b)


@pytest.mark.parametrize("iters", [1, 2])      # bench.py's LLaMA-7B workloads run one tracking step per refit
def test_llama7b_per_step_refit_from_token_subsample(ctx, iters):
    # cold fit on batch 0, then the per-step refit as that workload runs it: tracking steps from
    # the previous Q1 on every fourth token of the next batch
    stride, D7 = 4, 4096
    X0 = si.activation_torch(N7, D7, 0.8, 5000, 16, 50.0, torch.bfloat16, DEV, batch=0)
    X1 = si.activation_torch(N7, D7, 0.8, 5000, 16, 50.0, torch.bfloat16, DEV, batch=1)
    P, _, _ = ctx.fit_basis(X0, K7, R7, seed=77, draw=0, row_stride=stride)
    P, _, scale = ctx.fit_basis(X1, K7, R7, seed=77, draw=1, P=P, warm_start=True, iters=iters, oversample=-1,
                                row_stride=stride)
    ctx.sync_status()
    assert scale == pytest.approx((D7 - K7) / R7)
    P64 = si.as_f64(P)
    assert np.abs(P64.T @ P64 - np.eye(K7 + R7)).max() < 1e-5
    Xs = si.as_f64(X1[::stride])
    _, lam = orc.principal_subspace(orc.gram(Xs), K7)
    captured = float(np.sum((Xs @ P64[:, :K7]) ** 2))
    assert (1 - 1e-3) * lam[:K7].sum() <= captured <= (1 + 1e-6) * lam[:K7].sum()
    total = float(np.sum(Xs ** 2))
    assert total - captured <= 1.02 * (total - lam[:K7].sum())
