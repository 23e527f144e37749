"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol that include/prac.h declares, and rejects bad arguments before it
looks at the context or touches the device."""
import ctypes as C
import os
import re

import pytest

from paper_2602_23111_amd import prac

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DUMMY = C.c_void_p(0x1000)  # never dereferenced: argument checks come first


@pytest.fixture(scope="module")
def lib():
    return prac.load_library()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "prac.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = sorted(set(re.findall(r"\b(prac_[a-z_0-9]+)\s*\(", header)))
    assert declared == sorted(prac.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_strerror_and_lp_bytes(lib):
    assert lib.prac_strerror(0) == b"ok"
    assert lib.prac_strerror(-1) == b"invalid argument"
    assert lib.prac_strerror(-99) == b"unknown status"
    # P^T as c x round_up(d,64) plus P as d x round_up(c,64), bf16, first part 256-byte aligned
    d, c = 100, 24
    first = (c * 128 * 2 + 255) // 256 * 256
    second = (first + d * 64 * 2 + 255) // 256 * 256
    third = (second + (256 // 16) * 8 * 64 * 8 * 2 + 255) // 256 * 256   # P fragments, d padded to 256
    assert lib.prac_basis_lp_bytes(d, c) == third + (128 // 32) * 2 * 64 * 8 * 2
    assert lib.prac_basis_lp_bytes(0, 4) == 0


def _compress(lib, ctx=None, X=DUMMY, dt=1, N=8, d=16, ldx=16, P=DUMMY, lp=None, ldp=4, c=4, Cp=DUMMY, ldc=4,
              layout=0):
    return lib.prac_compress(ctx, X, dt, N, d, ldx, P, lp, ldp, c, Cp, ldc, layout)


def test_compress_argument_checks(lib):
    assert _compress(lib) == -6                    # valid arguments, null ctx
    assert _compress(lib, X=None) == -1
    assert _compress(lib, P=None) == -1
    assert _compress(lib, Cp=None) == -1
    assert _compress(lib, dt=7) == -1
    assert _compress(lib, N=0) == -1
    assert _compress(lib, N=1 << 31) == -1         # token counts are below 2^31
    assert _compress(lib, N=(1 << 31) - 1) == -6
    assert _compress(lib, ldx=15) == -1            # ldx < d
    assert _compress(lib, c=17, ldp=17, ldc=17) == -1  # c > d
    assert _compress(lib, ldp=3) == -1
    assert _compress(lib, ldc=3) == -1
    assert _compress(lib, ldc=0, layout=1) == -6   # packed layout ignores ldc
    assert _compress(lib, layout=2) == -1
    assert _compress(lib, lp=C.c_void_p(0x1008)) == -1  # packed copy must be 16-byte aligned


def _wgrad(lib, ctx=None, Cm=DUMMY, dY=DUMMY, dt=1, N=8, m=6, ldc=4, lddy=6, P=DUMMY, lp=None, d=16, ldp=4,
           k=2, r=2, scale=7.0, dW=DUMMY, odt=0, lddw=6, beta=0.0, layout=0):
    return lib.prac_weight_grad(ctx, Cm, dY, dt, N, m, ldc, layout, lddy, P, lp, d, ldp, k, r, scale, dW, odt,
                                lddw, beta)


def test_weight_grad_argument_checks(lib):
    assert _wgrad(lib) == -6
    assert _wgrad(lib, dY=None) == -1
    assert _wgrad(lib, k=-1) == -1
    assert _wgrad(lib, N=1 << 31) == -1
    assert _wgrad(lib, k=0, r=0) == -1
    assert _wgrad(lib, k=10, r=7, ldc=17, ldp=17) == -1   # k + r > d
    assert _wgrad(lib, ldc=3) == -1
    assert _wgrad(lib, ldc=0, layout=1) == -6
    assert _wgrad(lib, lddy=5) == -1
    assert _wgrad(lib, lddw=5) == -1
    assert _wgrad(lib, odt=3) == -1


def _fit(lib, ctx=None, X=DUMMY, dt=1, N=8, d=16, ldx=16, k=2, r=2, seed=1, draw=0, refresh=3, opts=None,
         P=DUMMY, ldp=4, lp=None):
    scale = C.c_float(-1.0)
    rc = lib.prac_fit_basis(ctx, X, dt, N, d, ldx, k, r, seed, draw, refresh, opts, P, ldp, lp, C.byref(scale))
    return rc, scale.value


def test_static_weight_grad_argument_checks(lib):
    # same checks as prac_weight_grad, before the ctx is looked at
    f = lib.prac_weight_grad_static
    args = lambda **kw: _wgrad_args(**kw)
    assert f(*_wgrad_args()) == -6
    assert f(*_wgrad_args(dY=None)) == -1
    assert f(*_wgrad_args(k=10, r=7, ldc=17, ldp=17)) == -1
    assert f(*_wgrad_args(lddw=5)) == -1
    assert lib.prac_strerror(-7) == b"request needs more scratch than the static block holds"


def _wgrad_args(ctx=None, Cm=DUMMY, dY=DUMMY, dt=1, N=8, m=6, ldc=4, lddy=6, P=DUMMY, lp=None, d=16, ldp=4,
                k=2, r=2, scale=7.0, dW=DUMMY, odt=0, lddw=6, beta=0.0, layout=0):
    return (ctx, Cm, dY, dt, N, m, ldc, layout, lddy, P, lp, d, ldp, k, r, scale, dW, odt, lddw, beta)


def test_fit_basis_argument_checks(lib):
    assert _fit(lib)[0] == -6
    assert _fit(lib, P=None)[0] == -1
    assert _fit(lib, k=9, r=8, ldp=17)[0] == -1          # k + r > d
    assert _fit(lib, k=0, r=0)[0] == -1
    assert _fit(lib, ldp=3)[0] == -1
    assert _fit(lib, X=None)[0] == -1                    # Q1 refresh needs X
    assert _fit(lib, X=None, refresh=2)[0] == -6         # ... but a Q2-only refresh does not
    assert _fit(lib, X=None, k=0, r=4)[0] == -6          # nor does a purely random basis
    assert _fit(lib, draw=1 << 32)[0] == -1
    assert _fit(lib, refresh=4)[0] == -1
    bad = prac.FitOpts(-1, 0, 0, 0)
    assert _fit(lib, opts=C.byref(bad))[0] == -1


def test_other_entry_points_reject_bad_arguments(lib):
    assert lib.prac_gram(None, DUMMY, 1, 8, 16, 16, 1, DUMMY, 16) == -6
    assert lib.prac_gram(None, DUMMY, 1, 8, 16, 16, 0, DUMMY, 16) == -1   # row_stride < 1
    assert lib.prac_gram(None, DUMMY, 1, 8, 16, 16, 1, DUMMY, 15) == -1   # ldg < d
    assert lib.prac_philox_words(None, 1, 0, 0, DUMMY, 16) == -6
    assert lib.prac_philox_words(None, 1, 0, 0, None, 16) == -1
    assert lib.prac_philox_normal(None, 1, 1 << 32, 0, DUMMY, 16) == -1
    assert lib.prac_pack_basis(None, DUMMY, 16, 4, 4, DUMMY) == -6
    assert lib.prac_pack_basis(None, DUMMY, 16, 3, 4, DUMMY) == -1
    f = lib.prac_compress_fused_fwd
    assert f(None, DUMMY, 1, 8, 16, 16, DUMMY, 6, 6, 0, DUMMY, None, 4, 4, DUMMY, 6, DUMMY, 4, 0) == -6
    assert f(None, DUMMY, 1, 8, 16, 16, DUMMY, 6, 6, 2, DUMMY, None, 4, 4, DUMMY, 6, DUMMY, 4, 0) == -1  # layout
    assert f(None, DUMMY, 1, 8, 16, 16, DUMMY, 6, 6, 1, DUMMY, None, 4, 4, DUMMY, 6, DUMMY, 4, 0) == -1  # ldw < d
    assert f(None, DUMMY, 1, 8, 16, 16, DUMMY, 6, 6, 0, DUMMY, None, 4, 4, DUMMY, 5, DUMMY, 4, 0) == -1  # ldy < m
    assert lib.prac_unpack_compressed(None, DUMMY, 8, 4, DUMMY, 4) == -6
    assert lib.prac_unpack_compressed(None, DUMMY, 8, 4, DUMMY, 3) == -1
    assert lib.prac_set_tuning(None, 1, 8) == -6 and lib.prac_set_tuning(None, 3, 8) == -1 and lib.prac_set_tuning(None, 2, 2000) == -1
    assert lib.prac_set_tuning(None, 4, 3) == -1 and lib.prac_set_tuning(None, 4, 2) == -6 and lib.prac_set_tuning(None, 5, 0) == -1
    assert lib.prac_profile_select(None, 10) == -1 and lib.prac_profile_select(None, 9) == -6
    n64 = C.c_int64(0)
    assert lib.prac_profile_read_each(None, None, 4, C.byref(n64)) == -1       # cap > 0 needs a buffer
    assert lib.prac_profile_read_each(None, None, 0, C.byref(n64)) == -6
    # packed C: 8 * ceil(N/128) x ceil(c/32) blocks of 64 lanes x 8 bf16
    assert lib.prac_compressed_bytes(100, 40, 1, 1, 0) == 8 * 2 * 64 * 8 * 2
    assert lib.prac_compressed_bytes(100, 40, 1, 0, 48) == 100 * 48 * 2
    assert lib.prac_compressed_bytes(100, 40, 0, 1, 0) == 0      # packed is bf16 only
    wgs = lib.prac_weight_grad_shared
    ptrs, i64s = (C.c_void_p * 2)(DUMMY, DUMMY), (C.c_int64 * 2)(6, 6)
    args = lambda n_out, lds: (None, DUMMY, 1, 8, 4, 0, n_out, ptrs, i64s, lds, DUMMY, None, 16, 4, 2, 2, 7.0, ptrs, 1,
                               i64s, 0.0)
    assert wgs(*args(2, i64s)) == -6
    assert wgs(*args(0, i64s)) == -1 and wgs(*args(5, i64s)) == -1          # 1 .. PRAC_MAX_SHARED outputs
    assert wgs(*args(2, (C.c_int64 * 2)(6, 5))) == -1                       # lddy[1] < m[1]
    rec = lib.prac_reconstruct
    assert rec(None, DUMMY, 1, 8, 4, 0, DUMMY, 16, 4, 2, 2, 7.0, DUMMY, 16) == -6
    assert rec(None, DUMMY, 1, 8, 3, 0, DUMMY, 16, 4, 2, 2, 7.0, DUMMY, 16) == -1    # ldc < k + r
    assert rec(None, DUMMY, 1, 8, 4, 0, DUMMY, 16, 4, 2, 2, 7.0, DUMMY, 15) == -1    # ldxh < d
    assert rec(None, DUMMY, 1, 8, 4, 0, DUMMY, 3, 4, 2, 2, 7.0, DUMMY, 16) == -1     # k + r > d
    assert rec(None, DUMMY, 1, 8, 0, 1, DUMMY, 16, 4, 2, 2, 7.0, DUMMY, 16) == -6    # packed C ignores ldc
    assert lib.prac_destroy(None) == -6 and lib.prac_sync_status(None) == -6


def test_create_fails_cleanly_without_a_device(lib):
    import torch

    if torch.cuda.is_available():
        pytest.skip("a GPU is visible")
    h = C.c_void_p()
    assert lib.prac_create(C.byref(h), 0, None) == -3 and not h.value


def test_ws_kernels_isa_keeps_hands_off_ring_and_accumulators():
    """The inline-assembly matrix blocks hide in-flight loads and MFMAs from the compiler; the compiled
    code must not move those registers where it cannot know better (see lint_isa.py)."""
    import shutil

    if not (shutil.which("hipcc") or os.path.exists("/opt/rocm/bin/hipcc")):
        pytest.skip("hipcc not available")
    from paper_2602_23111_amd import lint_isa

    assert lint_isa.lint_text(lint_isa.compile_isa()) == []
    # the check itself: an accumulator copy between matrix blocks must be reported
    planted = """_Zfake_ws_kernelv: ; @fake
\t;;#ASMSTART
v_mfma_f32_32x32x16_bf16 a[0:15], v[2:5], v[6:9], a[0:15]
global_load_dwordx4 v[10:13], v20, s[2:3]
\t;;#ASMEND
\tv_accvgpr_read_b32 v30, a3
\tv_mov_b32_e32 v11, v40
\t;;#ASMSTART
s_waitcnt vmcnt(0)
\t;;#ASMEND
.Lfunc_end0:
"""
    assert len(lint_isa.lint_text(planted)) == 2
    # after a block that drains the matrix pipeline the accumulators may be read, the ring still not
    drained = planted.replace("\tv_accvgpr_read_b32 v30, a3\n", "\t;;#ASMSTART\ns_nop 15\ns_nop 15\ns_nop 15\ns_nop 15\n"
                                                                "\t;;#ASMEND\n\tv_accvgpr_read_b32 v30, a3\n")
    found = lint_isa.lint_text(drained)
    assert len(found) == 1 and "ring register" in found[0]
    # a streaming kernel whose metadata reports spilled vector registers is reported too
    meta = "\n  - .name:           _Zfake_ws_kernelv\n    .vgpr_count:     256\n    .vgpr_spill_count: 12\n    .wavefront_size: 64\n"
    clean = planted.replace("\tv_accvgpr_read_b32 v30, a3\n\tv_mov_b32_e32 v11, v40\n", "")
    assert lint_isa.lint_text(clean) == []
    found = lint_isa.lint_text(clean + meta)
    assert len(found) == 1 and "spilled" in found[0]


# ---- scratch sizing (prac_workspace_bytes / prac_reserve_workspace) ----------------------------
def test_workspace_bytes_matches_the_documented_scratch_of_each_call(lib):
    BAD = (1 << 64) - 1
    ws = lambda sh: int(lib.prac_workspace_bytes(None, C.byref(sh)))
    up = lambda b: (b + 255) // 256 * 256
    N, d, m, k, r = 32768, 2048, 2048, 128, 128
    c = k + r
    lp = int(lib.prac_basis_lp_bytes(d, c))
    # compress with a packed basis handed in needs nothing; without one, room for the packed copy
    assert ws(prac.call_shape("compress", N, d, k, r)) == 0
    assert ws(prac.call_shape("compress", N, d, k, r, have_p_lp=False)) == up(lp)
    # fused forward: W in fragment order, d padded to 256 rows, m to 256 columns
    assert ws(prac.call_shape("fused_fwd", N, d, k, r, m=[m])) == 2048 * 2048 * 2
    # weight gradient at the headline shape: 16 token ranges of fp32 partial sums + T in fragment order (bf16)
    assert ws(prac.call_shape("weight_grad", N, d, k, r, m=[m])) == 16 * c * m * 4 + c * m * 2
    # three outputs sharing C: 5 token ranges (256 CUs / 48 tiles)
    assert ws(prac.call_shape("weight_grad", N, d, k, r, m=[m, m, m])) == 3 * (5 * c * m * 4 + c * m * 2)
    # row-major C has to be packed first
    extra = int(lib.prac_compressed_bytes(N, c, 1, 1, 0))
    assert ws(prac.call_shape("weight_grad", N, d, k, r, m=[m], c_layout=0)) == 16 * c * m * 4 + c * m * 2 + extra
    # strided kernels (fp32 data): T, and nothing else for an fp32 dW
    assert ws(prac.call_shape("weight_grad", 2048, 512, 32, 32, m=[1376], dt=0, odt=0, c_layout=0)) == up(64 * 1376 * 4)
    # reconstruction: Ps^T in fragment order (k-blocks over 256, column blocks over d)
    assert ws(prac.call_shape("reconstruct", N, d, k, r)) == 16 * 64 * 1024
    # the tracking refit is cheaper than the Gram-based fit, and a random-only refresh cheaper still
    cold = ws(prac.call_shape("fit_basis", N, d, k, r))
    track = ws(prac.call_shape("fit_basis", N, d, k, r, warm_start=True, oversample=-1, iters=2))
    rnd = ws(prac.call_shape("fit_basis", N, d, k, r, refresh=2))
    assert cold > d * d * 4 and 0 < rnd < track < cold
    assert ws(prac.call_shape("gram", N, d, 0, 0)) > 0
    # shapes the entry points would reject
    assert ws(prac.call_shape("compress", N, d, 0, 0)) == BAD
    assert ws(prac.call_shape("weight_grad", N, d, k, r, m=[])) == BAD
    assert ws(prac.call_shape("weight_grad", N, 100, 64, 64, m=[m])) == BAD      # k + r > d
    bad_op = prac.call_shape("compress", N, d, k, r)
    bad_op.op = 99
    assert ws(bad_op) == BAD
    assert int(lib.prac_workspace_bytes(None, None)) == BAD
    assert lib.prac_reserve_workspace(None, 1 << 20) == -6
    assert lib.prac_reserve_workspace(None, BAD) == -1


def test_fit_plan_holds_every_split_product():
    """The split-sum block of the fit's scratch plan is at least as large as every split product the fit
    issues, for every rank split and refresh branch (a random-only refresh with k > 2 r once was not)."""
    lib = prac.load_library()
    for d in (384, 768, 2048, 4096):
        for k, r in ((0, 64), (64, 0), (16, 16), (96, 16), (256, 32), (32, 256), (128, 128), (512, 64), (1024, 8)):
            if k + r > d:
                continue
            for refresh in (1, 2, 3):
                for opts in (dict(), dict(warm_start=True, oversample=-1, iters=2), dict(oversample=8)):
                    # 32768 rows, and batches of fewer rows than k (part of Q1 is then drawn like Q2)
                    for N in (32768, 300, 1):
                        sh = prac.call_shape("fit_basis", N, d, k, r, refresh=refresh, **opts)
                        assert lib.prac_debug_fit_slab_margin(C.byref(sh)) >= 0, (N, d, k, r, refresh, opts)
