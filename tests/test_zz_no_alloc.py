"""The entry point that allocates nothing (prac_weight_grad_static) against prac_weight_grad: same
kernels, scratch in the library's static block instead of the ctx block.  Two calls in a row, the
second with a smaller input (the block still holds the first call's contents), each compared bit
for bit with prac_weight_grad and, to the bf16 tolerance, with the fp64 oracle."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import prac_oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def rel_fro(got, ref):
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))


def _case(ctx, N, d, m, k, r, seed, layout_packed, odt):
    from paper_2602_23111_amd.prac import C_PACKED, C_ROWMAJOR
    from test_gpu_parity import pack_c_reference
    c = k + r
    s = orc.scaling_factor(d, k, r)
    Xt = si.round_to(si.activation(N, d, 0.8, seed=seed, n_out=2, out_scale=20.0)[0], "bf16")
    dYt = si.round_to(si.grad_output(N, m, 1e-2, seed=seed + 1), "bf16")
    P32 = si.round_to(si.orthonormal_basis(d, c, seed=seed + 2), "f32")
    Ct = si.round_to(orc.compress(si.as_f64(Xt), si.as_f64(P32)), "bf16")
    Pd, dYd = P32.to(DEV), dYt.to(DEV)
    lp = ctx.pack_basis(Pd)
    Cd = pack_c_reference(Ct).to(DEV) if layout_packed else Ct.to(DEV)
    layout = C_PACKED if layout_packed else C_ROWMAJOR
    want = ctx.weight_grad(Cd, dYd, Pd, k, r, s, P_lp=lp, out_dtype=odt, layout=layout)
    got = torch.full((d, m), float("nan"), dtype=odt, device=DEV)
    ctx.weight_grad(Cd, dYd, Pd, k, r, s, P_lp=lp, out=got, layout=layout, static=True)
    ctx.sync_status()
    assert torch.equal(got, want)
    ref = orc.weight_grad(si.as_f64(Ct), si.as_f64(dYt), si.as_f64(P32), k, s)
    assert rel_fro(si.as_f64(got), ref) < 1e-2
    return got


@pytest.mark.parametrize("one_launch", [0, 1])   # the three-launch default and the one-launch variant (its counters
def test_static_weight_grad_two_calls_second_smaller(one_launch):   # live in the static block too)
    from paper_2602_23111_amd.prac import TUNE_WGRAD_ONE_LAUNCH, Prac
    ctx = Prac(0)
    try:
        ctx.set_tuning(TUNE_WGRAD_ONE_LAUNCH, one_launch)
        _case(ctx, 4096, 512, 640, 32, 32, seed=11, layout_packed=True, odt=torch.bfloat16)
        _case(ctx, 1000, 328, 200, 24, 16, seed=21, layout_packed=False, odt=torch.float32)   # smaller, row-major C
        _case(ctx, 4096, 512, 640, 32, 32, seed=11, layout_packed=True, odt=torch.bfloat16)   # and the first again
    finally:
        ctx.close()


def test_static_weight_grad_rejects_what_does_not_fit():
    from paper_2602_23111_amd.prac import C_ROWMAJOR, STATIC_SCRATCH_BYTES, Prac, PracError, call_shape
    ctx = Prac(0)
    try:
        N, d, m, k, r = 512, 2048, 16384, 512, 512
        sh = call_shape("weight_grad", N, d, k, r, m=[m], c_layout=C_ROWMAJOR, have_p_lp=False)
        assert ctx.workspace_bytes(sh) > STATIC_SCRATCH_BYTES
        Cd = torch.zeros((N, k + r), dtype=torch.bfloat16, device=DEV)
        dYd = torch.zeros((N, m), dtype=torch.bfloat16, device=DEV)
        Pd = torch.zeros((d, k + r), dtype=torch.float32, device=DEV)
        out = torch.full((d, m), 7.0, dtype=torch.bfloat16, device=DEV)
        with pytest.raises(PracError) as e:
            ctx.weight_grad(Cd, dYd, Pd, k, r, 3.0, out=out, static=True)
        assert e.value.status == -7
        ctx.sync_status()
        assert bool((out == 7.0).all())            # nothing was enqueued
    finally:
        ctx.close()
