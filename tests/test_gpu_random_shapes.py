"""GPU parity on randomly drawn shapes, through the C ABI binding against the fp64 oracle: compress, weight
gradient (row-major and packed C), reconstruction and the fused forward in the first test, the Gram matrix and the
basis fit with its options and refresh branches in the second; the gradients of several layers from one shared C
under every launch form, bf16 gradients with accumulation, the packed layouts and the entry point that allocates
nothing in the third; bf16 and fp32.

The draws mix what the fixed cases of test_gpu_parity.py hold apart: token counts of 1 to a few thousand, feature
counts below one k-tile (8, 64, 72, 200) up to 1100, output widths from 8 to 1000, any rank split (k = 0, r = 0,
k + r up to 600), leading dimensions that are exact, padded by a whole 16-byte chunk or unaligned (the generic
kernels), a basis packed beforehand or packed inside the call.  Padding is NaN, so any use of it shows.
Tolerances as in test_gpu_parity.py: relative Frobenius error 1e-2 for bf16 data, 1e-5 for fp32 data.
"""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import prac_oracle as orc

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
CASES_PER_SEED = 60


@pytest.fixture(scope="module")
def ctx():
    from paper_2602_23111_amd.prac import Prac

    p = Prac(0)
    yield p
    p.close()


def rel(a, b):
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def pad(t, ld):
    buf = torch.full((t.shape[0], ld), float("nan"), dtype=t.dtype, device=DEV)
    buf[:, :t.shape[1]] = t.to(DEV)
    return buf[:, :t.shape[1]]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_shapes_match_oracle(ctx, seed):
    from paper_2602_23111_amd.prac import C_PACKED

    rng = np.random.default_rng(seed)
    bad = []
    for it in range(CASES_PER_SEED):
        dt = "bf16" if rng.random() < 0.8 else "f32"
        tol = 1e-2 if dt == "bf16" else 1e-5
        N = int(rng.choice([1, 7, 100, 129, 500, 1023, 2048, 3001, 4097]))
        d = int(rng.choice([8, 64, 72, 200, 256, 264, 333, 512, 520, 768, 1100]))
        m = int(rng.choice([8, 40, 96, 128, 136, 200, 203, 512, 640, 1000]))
        c = int(rng.integers(1, min(d, 600) + 1))
        k = int(rng.integers(0, c + 1))
        r = c - k
        s = float(d - k) / r if r else 0.0
        ldx = d + int(rng.choice([0, 0, 8, 3]))
        lddy = m + int(rng.choice([0, 0, 8, 5]))
        with_lp = rng.random() < 0.7
        tag = f"seed {seed} case {it}: {dt} N={N} d={d} m={m} k={k} r={r} ldx={ldx} lddy={lddy} lp={with_lp}"
        print(tag, flush=True)  # names the case should a kernel fault

        X64, _ = si.activation(N, d, 0.8, seed=it + 17)
        Xt = si.round_to(X64, dt)
        dYt = si.round_to(si.grad_output(N, m, 1e-2, seed=it), dt)
        P32 = si.round_to(si.orthonormal_basis(d, c, it), "f32")
        P64 = si.as_f64(P32)
        Xd, dYd, Pd = pad(Xt, ldx), pad(dYt, lddy), P32.to(DEV)
        lp = ctx.pack_basis(Pd) if with_lp else None

        def check(what, got, ref):
            e = rel(got, ref) if np.linalg.norm(ref) > 0 else float(np.abs(got).max())
            if not e < tol:
                bad.append(f"{what}: {tag}: {e:.3g}")

        Cm = ctx.compress(Xd, Pd, P_lp=lp)
        ctx.sync_status()
        check("compress", si.as_f64(Cm), orc.compress(si.as_f64(Xt), P64))

        dW = ctx.weight_grad(Cm, dYd, Pd, k, r, s, P_lp=lp)
        ctx.sync_status()
        ref_dw = orc.weight_grad(si.as_f64(Cm), si.as_f64(dYt), P64, k, s)
        check("weight_grad", si.as_f64(dW), ref_dw)

        if dt == "bf16" and ldx % 8 == 0 and lp is not None:
            Cp = ctx.compress(Xd, Pd, P_lp=lp, layout=C_PACKED)
            dW2 = ctx.weight_grad(Cp, dYd, Pd, k, r, s, P_lp=lp, layout=C_PACKED)
            ctx.sync_status()
            check("weight_grad, packed C", si.as_f64(dW2), ref_dw)

        Xh = ctx.reconstruct(Cm, Pd, k, r, s)
        ctx.sync_status()
        check("reconstruct", si.as_f64(Xh), orc.reconstruct(si.as_f64(Cm), P64, k, s))

        if it % 3 == 0:
            Wt = si.round_to(np.random.default_rng(it).standard_normal((d, m)) * 0.05, dt)
            Y, C2 = ctx.compress_fused_fwd(Xd, Wt.to(DEV), Pd, w_layout=0, P_lp=lp)
            ctx.sync_status()
            check("fused forward Y", si.as_f64(Y), orc.forward(si.as_f64(Xt), si.as_f64(Wt)))
            check("fused forward C", si.as_f64(C2), orc.compress(si.as_f64(Xt), P64))
    assert not bad, "\n".join(bad)


@pytest.mark.parametrize("seed", [0, 1])
def test_random_fit_shapes_match_oracle(ctx, seed):
    """Gram matrix and basis fit on random shapes and options: token counts from 1 (batches of fewer rows than k:
    the rank of the data is below k) to 4100, d from 8 to 768, any k and r, row subsampling, iteration counts, block
    widths, the refresh branches and the warm (tracking) refit.  Checked is what is unique: the Gram matrix; P
    orthonormal; the energy Q1 captures of the sampled rows against the sum of the oracle's top-k eigenvalues; Q2
    column by column against the oracle's complement of the Q1 the library returned; the branch that is not
    refreshed left bit-exact; the packed copy equal to pack_basis of the master."""
    from paper_2602_23111_amd.prac import PRAC_REFRESH_PRINCIPAL, PRAC_REFRESH_RANDOM

    rng = np.random.default_rng(seed)
    bad = []
    for it in range(40):
        dt = "bf16" if rng.random() < 0.6 else "f32"
        N = int(rng.choice([1, 50, 300, 1000, 2500, 4100]))
        d = int(rng.choice([8, 64, 100, 136, 256, 300, 520, 768]))
        k = int(rng.integers(0, min(d - 1, 300) + 1))
        r = int(rng.integers(0 if k > 0 else 1, min(d - k, 200) + 1))
        stride = int(rng.choice([1, 1, 2, 4]))
        iters = int(rng.choice([0, 2, 5]))
        over = int(rng.choice([0, 0, -1, 3]))
        ldx = d + int(rng.choice([0, 0, 8, 3]))
        mode = int(rng.choice([0, 0, 1, 2, 3]))   # 0 cold, 1 random block only, 2 principal block again, 3 warm refit
        tag = (f"seed {seed} case {it}: {dt} N={N} d={d} k={k} r={r} stride={stride} iters={iters} over={over} "
               f"ldx={ldx} mode={mode}")
        print(tag, flush=True)
        Xt = si.round_to(si.activation(N, d, 0.8, seed=it + 100 * seed)[0], dt)
        Xd = pad(Xt, ldx)
        Xs = si.as_f64(Xt)[::stride]

        G = ctx.gram(Xd, row_stride=stride)
        ctx.sync_status()
        if not rel(si.as_f64(G), orc.gram(si.as_f64(Xt), stride)) < 2e-5:
            bad.append(f"gram: {tag}")
        c = k + r
        if mode == 1:
            P0 = si.round_to(si.orthonormal_basis(d, max(k, 1), it), "f32")[:, :k]
            P = torch.zeros((d, c), dtype=torch.float32, device=DEV)
            P[:, :k] = P0.to(DEV)
            ctx.fit_basis(None, k, r, seed=5, draw=it, refresh=PRAC_REFRESH_RANDOM, P=P, d=d, pack=False)
            ctx.sync_status()
            got = si.as_f64(P)
            if not np.array_equal(got[:, :k], si.as_f64(P0)):
                bad.append(f"Q1 touched: {tag}")
            if r > 0:
                Q2 = orc.complement_basis(si.as_f64(P0), orc.gaussian_matrix(5, it, d, r))
                if not np.abs(got[:, k:] - Q2).max() < 1e-4:
                    bad.append(f"Q2: {tag}")
            continue
        warm = mode == 3
        P, lp, scale = ctx.fit_basis(Xd, k, r, seed=5, draw=it, row_stride=stride, iters=iters,
                                     oversample=0 if warm else over)
        ctx.sync_status()
        if warm:
            P, lp, scale = ctx.fit_basis(Xd, k, r, seed=5, draw=it + 1, row_stride=stride, iters=max(iters, 1),
                                         oversample=-1, warm_start=True, P=P.clone())
            ctx.sync_status()
        if mode == 2 and k > 0:
            Pk = P.clone()
            ctx.fit_basis(Xd, k, r, seed=5, draw=it, row_stride=stride, iters=iters, oversample=over,
                          refresh=PRAC_REFRESH_PRINCIPAL, P=Pk, pack=False)
            ctx.sync_status()
            if not torch.equal(Pk[:, k:], P[:, k:]):
                bad.append(f"Q2 touched: {tag}")
        P64 = si.as_f64(P)
        e = np.abs(P64.T @ P64 - np.eye(c)).max()
        if not e < 1e-4:
            bad.append(f"orthonormality {e:.3g}: {tag}")
        if k > 0:
            _, lam = orc.principal_subspace(orc.gram(Xs), k)
            captured, top = float(np.sum((Xs @ P64[:, :k]) ** 2)), lam[:k].sum()
            # the default block (k columns of oversampling, 8 iterations) captures all but 1e-3; narrower blocks and
            # fewer iterations are held to 5e-2 here (their own tests state what they reach)
            slack = 1e-3 if (iters == 0 and not warm and over >= 0) else 5e-2
            if not (1 - slack) * top <= captured <= (1 + 1e-5) * top + 1e-9:
                bad.append(f"energy {captured / max(top, 1e-300):.5f}: {tag}")
        if r > 0:
            Q2 = orc.complement_basis(P64[:, :k], orc.gaussian_matrix(5, it + (1 if warm else 0), d, r))
            if not np.abs(P64[:, k:] - Q2).max() < 1e-4:
                bad.append(f"Q2 against the oracle: {tag}")
        if abs(scale - ((d - k) / r if r else 0.0)) > 1e-6 * max(1.0, scale):
            bad.append(f"scale {scale}: {tag}")
        if lp is not None and not torch.equal(lp, ctx.pack_basis(P)):
            bad.append(f"packed copy: {tag}")
    assert not bad, "\n".join(bad)


@pytest.mark.parametrize("seed", [0, 1])
def test_random_shared_gradients_and_packed_paths(ctx, seed):
    """bf16 data: one to four gradients from one shared C (row-major or packed) in fp32 or bf16 with beta 0 or 0.5,
    under the built-in launch form, the one-launch form, both forms of the tail and forced token-split counts; the
    entry point with static scratch against the ordinary one bit for bit; the reconstruction from packed C; the fused
    forward with m x d weights writing packed C."""
    from paper_2602_23111_amd import prac as pr

    rng = np.random.default_rng(seed)
    bad = []
    for it in range(30):
        N = int(rng.choice([1, 100, 129, 1023, 2048, 4097, 8200]))
        d = int(rng.choice([8, 72, 200, 256, 333, 520, 768, 1100, 2048]))
        c = int(rng.integers(1, min(d, 600) + 1))
        k = int(rng.integers(0, c + 1))
        r = c - k
        s = float(d - k) / r if r else 0.0
        n_out = int(rng.integers(1, 5))
        ms = [int(rng.choice([8, 40, 96, 128, 136, 200, 203, 512, 640, 1000])) for _ in range(n_out)]
        pady = [int(rng.choice([0, 0, 8, 5])) for _ in range(n_out)]
        out_bf16 = rng.random() < 0.5
        beta = float(rng.choice([0.0, 0.0, 0.5]))
        packed = rng.random() < 0.5
        tune = int(rng.choice([0, 0, 1, 2, 3, 4]))  # built-in, one launch, tail as two launches, tail as one, forced splits
        splits = int(rng.choice([1, 2, 4, 8, 16]))
        ldx = d + int(rng.choice([0, 8]))
        ldw = d + int(rng.choice([0, 8, 3]))
        tag = (f"seed {seed} case {it}: N={N} d={d} k={k} r={r} m={ms} pad={pady} bf16 dW={out_bf16} beta={beta} "
               f"packed={packed} tune={tune}/{splits} ldx={ldx} ldw={ldw}")
        print(tag, flush=True)
        Xt = si.round_to(si.activation(N, d, 0.8, seed=it + 31)[0], "bf16")
        dYts = [si.round_to(si.grad_output(N, m, 1e-2, seed=it + 7 * h), "bf16") for h, m in enumerate(ms)]
        P32 = si.round_to(si.orthonormal_basis(d, c, it), "f32")
        P64 = si.as_f64(P32)
        Xd, Pd = pad(Xt, ldx), P32.to(DEV)
        dYd = [pad(t, m + p) for t, m, p in zip(dYts, ms, pady)]
        lp = ctx.pack_basis(Pd)
        layout = pr.C_PACKED if packed else pr.C_ROWMAJOR
        try:
            ctx.set_tuning(pr.TUNE_WGRAD_ONE_LAUNCH, 1 if tune == 1 else 0)
            ctx.set_tuning(pr.TUNE_WGRAD_TAIL, 1 if tune == 2 else (2 if tune == 3 else 0))
            ctx.set_tuning(pr.TUNE_CTDY_SPLITS, splits if tune == 4 else 0)
            Cm = ctx.compress(Xd, Pd, P_lp=lp)
            Cp = ctx.compress(Xd, Pd, P_lp=lp, layout=pr.C_PACKED)
            ctx.sync_status()
            C64 = si.as_f64(Cm)
            if not torch.equal(ctx.unpack_compressed(Cp, N, c), Cm):
                bad.append(f"packed C is not the row-major C: {tag}")
            old = [si.round_to(np.random.default_rng(it + h).standard_normal((d, m)) * 1e-2, "bf16" if out_bf16 else "f32")
                   for h, m in enumerate(ms)]
            got = ctx.weight_grad_shared(Cp if packed else Cm, dYd, Pd, k, r, s, P_lp=lp,
                                         outs=[o.to(DEV).clone() for o in old], beta=beta, layout=layout)
            ctx.sync_status()
            for h in range(n_out):
                ref = orc.weight_grad(C64, si.as_f64(dYts[h]), P64, k, s) + beta * si.as_f64(old[h])
                if not rel(si.as_f64(got[h]), ref) < 1e-2:
                    bad.append(f"gradient {h}: {tag}")
            o1 = torch.zeros((d, ms[0]), dtype=torch.bfloat16 if out_bf16 else torch.float32, device=DEV)
            o2 = torch.zeros_like(o1)
            try:
                ctx.weight_grad(Cp if packed else Cm, dYd[0], Pd, k, r, s, P_lp=lp, out=o1, layout=layout, static=True)
                ctx.weight_grad(Cp if packed else Cm, dYd[0], Pd, k, r, s, P_lp=lp, out=o2, layout=layout)
                ctx.sync_status()
                if not torch.equal(o1, o2):
                    bad.append(f"static scratch differs from the ordinary call: {tag}")
            except pr.PracError as ex:
                if "TOOBIG" not in str(ex):
                    raise
        finally:
            ctx.set_tuning(pr.TUNE_WGRAD_ONE_LAUNCH, 0)
            ctx.set_tuning(pr.TUNE_WGRAD_TAIL, 0)
            ctx.set_tuning(pr.TUNE_CTDY_SPLITS, 0)
        Xh = ctx.reconstruct(Cp, Pd, k, r, s, N=N, layout=pr.C_PACKED)
        ctx.sync_status()
        if not rel(si.as_f64(Xh), orc.reconstruct(C64, P64, k, s)) < 1e-2:
            bad.append(f"reconstruction from packed C: {tag}")
        Wt = si.round_to(np.random.default_rng(it).standard_normal((ms[0], d)) * 0.05, "bf16")
        Y, C2 = ctx.compress_fused_fwd(Xd, pad(Wt, ldw), Pd, w_layout=1, P_lp=lp, layout=pr.C_PACKED)
        ctx.sync_status()
        if not rel(si.as_f64(Y), orc.forward(si.as_f64(Xt), si.as_f64(Wt).T)) < 1e-2:
            bad.append(f"fused forward Y: {tag}")
        # the fused launch walks the k-tiles in another order than compress: last-bit differences only
        if not torch.equal(C2, Cp) and not rel(si.as_f64(C2.float()), si.as_f64(Cp.float())) < 1e-3:
            bad.append(f"fused forward C: {tag}")
    assert not bad, "\n".join(bad)
