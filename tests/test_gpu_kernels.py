"""Kernel-level parity: each HIP kernel, called through the C ABI's test entry
points, against the matching step of the CPU oracle on the same seeded inputs.
Sizes span several tiles and a ragged tail."""
import math

import numpy as np
import pytest

from oracle import oracle as orc
from gpu_util import (BF16_KERNEL_TOL, F32_KERNEL_TOL, dt_code, empty_dev, quantise, rel_err, stream_ptr, to_dev,
                      to_np, torch_mod)

pytestmark = pytest.mark.gpu


def _tol(dtype):
    return F32_KERNEL_TOL if dtype == "f32" else BF16_KERNEL_TOL


class _TestLib:
    """The test build of the library (single-kernel entry points) with the binding's helpers bound to it."""

    def __init__(self):
        from paper_2201_12465_amd import binding
        self._b = binding
        self.FL_ERR_UNSUPPORTED = binding.FL_ERR_UNSUPPORTED

    def lib(self):
        return self._b.test_lib()

    def check(self, status):
        self._b.check(status, self._b.test_lib())


def _lib():
    return _TestLib()


GEMM_SHAPES = [(32, 192, 64), (200, 136, 72), (257, 264, 328), (1024, 768, 256), (130, 8, 8)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode", ["nt", "nn", "tn"])
@pytest.mark.parametrize("shape", GEMM_SHAPES)
def test_gemm_plain(dtype, mode, shape):
    b = _lib()
    M, N, K = shape
    if mode == "tn" and M % 8:
        M += 8 - M % 8          # the k-major A operand is contiguous along M
    rng = np.random.default_rng(hash((mode, shape)) % 2**32)
    A = quantise(rng.standard_normal((M, K)), dtype)     # logical A(m,k)
    Bm = quantise(rng.standard_normal((N, K)), dtype)    # logical B(n,k)
    ref = A.astype(np.float64) @ Bm.astype(np.float64).T
    a_kc, b_kc = {"nt": (1, 1), "nn": (1, 0), "tn": (0, 0)}[mode]
    dA = to_dev(A if a_kc else A.T.copy(), dtype)
    dB = to_dev(Bm if b_kc else Bm.T.copy(), dtype)
    for splits in ([1] if mode != "tn" else [1, 0, 3]):
        dC = empty_dev((M, N), dtype)
        s = splits if splits else b.lib().fl_test_gemm_splits(dt_code(dtype), M, N, K)
        part = empty_dev((max(s, 1) * M * N,), "f32")
        if splits == 3:      # k-ranges are whole k-tiles (32 fp32 / 64 bf16 values); none may be empty
            kt = 32 if dtype == "f32" else 64
            kps = -(-(-(-K // 3)) // kt) * kt
            if 2 * kps >= K:
                continue
        b.check(b.lib().fl_test_gemm(dt_code(dtype), a_kc, b_kc, dA.data_ptr(), dB.data_ptr(), dC.data_ptr(), M, N, K,
                                     None, None, 0, None, 0, None, splits, part.data_ptr(), stream_ptr()))
        torch_mod().cuda.synchronize()
        assert rel_err(to_np(dC), ref) <= _tol(dtype), (mode, shape, splits)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode", ["nt", "nn", "tn"])
@pytest.mark.parametrize("tmw", [1, 2])
@pytest.mark.parametrize("shape", [(200, 136, 72), (328, 264, 192)])
def test_gemm_tile_heights(dtype, mode, tmw, shape):
    """The register-staged kernel with 64x128 (tmw=1) and 128x128 (tmw=2) tiles, ragged M, N and K."""
    b = _lib()
    M, N, K = shape
    rng = np.random.default_rng(hash((mode, shape, tmw)) % 2**32)
    A = quantise(rng.standard_normal((M, K)), dtype)
    Bm = quantise(rng.standard_normal((N, K)), dtype)
    ref = A.astype(np.float64) @ Bm.astype(np.float64).T
    a_kc, b_kc = {"nt": (1, 1), "nn": (1, 0), "tn": (0, 0)}[mode]
    dA = to_dev(A if a_kc else A.T.copy(), dtype)
    dB = to_dev(Bm if b_kc else Bm.T.copy(), dtype)
    dC = empty_dev((M, N), dtype)
    b.lib().fl_test_gemm_force_variant(-2)
    b.lib().fl_test_gemm_force_tile_height(tmw)
    try:
        b.check(b.lib().fl_test_gemm(dt_code(dtype), a_kc, b_kc, dA.data_ptr(), dB.data_ptr(), dC.data_ptr(), M, N, K,
                                     None, None, 0, None, 0, None, 1, None, stream_ptr()))
        torch_mod().cuda.synchronize()
    finally:
        b.lib().fl_test_gemm_force_variant(-1)
        b.lib().fl_test_gemm_force_tile_height(0)
    assert rel_err(to_np(dC), ref) <= _tol(dtype), (dtype, mode, tmw, shape)


@pytest.mark.parametrize("variant", [-2, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11])
@pytest.mark.parametrize("mode", ["nt", "nn", "tn"])
@pytest.mark.parametrize("shape", [(304, 264, 192), (520, 392, 128), (8, 8, 64), (1000, 776, 640)])
def test_gemm_bf16_pipelined_variants(variant, mode, shape):
    """Every tile/stage variant of the pipelined bf16 kernel (-2 = the plain kernel), ragged M and N."""
    b = _lib()
    M, N, K = shape
    rng = np.random.default_rng(hash((mode, shape)) % 2**32)
    A = quantise(rng.standard_normal((M, K)), "bf16")
    Bm = quantise(rng.standard_normal((N, K)), "bf16")
    ref = A.astype(np.float64) @ Bm.astype(np.float64).T
    a_kc, b_kc = {"nt": (1, 1), "nn": (1, 0), "tn": (0, 0)}[mode]
    dA = to_dev(A if a_kc else A.T.copy(), "bf16")
    dB = to_dev(Bm if b_kc else Bm.T.copy(), "bf16")
    b.lib().fl_test_gemm_force_variant(variant)
    try:
        for splits in (1, 2):
            if splits == 2 and K < 128:
                continue
            dC = empty_dev((M, N), "bf16")
            part = empty_dev((splits * M * N,), "f32")
            b.check(b.lib().fl_test_gemm(1, a_kc, b_kc, dA.data_ptr(), dB.data_ptr(), dC.data_ptr(), M, N, K, None,
                                         None, 0, None, 0, None, splits, part.data_ptr(), stream_ptr()))
            torch_mod().cuda.synchronize()
            assert rel_err(to_np(dC), ref) <= BF16_KERNEL_TOL, (variant, mode, shape, splits)
    finally:
        b.lib().fl_test_gemm_force_variant(-1)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("act", [0, 1, 2])
def test_gemm_forward_epilogue(dtype, act):
    """v = x W^T + b; preact; act; + residual  (the forward linear layers)."""
    b = _lib()
    M, N, K = 200, 264, 136
    rng = np.random.default_rng(5 + act)
    x = quantise(rng.standard_normal((M, K)), dtype)
    W = quantise(rng.standard_normal((N, K)) * 0.2, dtype)
    bias = quantise(rng.standard_normal(N), dtype)
    res = quantise(rng.standard_normal((M, N)), dtype)
    u = orc.linear_fwd(x, W, bias)
    g = u if act == 0 else orc.act_fwd(u, "relu" if act == 1 else "gelu")
    ref = g + res
    dC, dU = empty_dev((M, N), dtype), empty_dev((M, N), dtype)
    tx, tW, tb, tr = (to_dev(a, dtype) for a in (x, W, bias, res))   # keep the device copies alive
    b.check(b.lib().fl_test_gemm(dt_code(dtype), 1, 1, tx.data_ptr(), tW.data_ptr(), dC.data_ptr(), M, N, K,
                                 tb.data_ptr(), tr.data_ptr(), act, dU.data_ptr(), 0, None, 1, None, stream_ptr()))
    torch_mod().cuda.synchronize()
    assert rel_err(to_np(dC), ref) <= _tol(dtype)
    assert rel_err(to_np(dU), u) <= _tol(dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("dact", [1, 2])
def test_gemm_backward_epilogue(dtype, dact):
    """dx = (dy W + skip) * act'(aux)  (the input-gradient GEMMs)."""
    b = _lib()
    M, N, K = 136, 200, 264      # dy [M,K] (k = out features), W [K,N] k-major, dx [M,N]
    rng = np.random.default_rng(9 + dact)
    dy = quantise(rng.standard_normal((M, K)), dtype)
    W = quantise(rng.standard_normal((K, N)) * 0.2, dtype)
    skip = quantise(rng.standard_normal((M, N)), dtype)
    u = quantise(rng.standard_normal((M, N)), dtype)
    aux = u if dact == 2 else quantise(np.maximum(u, 0), dtype)
    lin = dy.astype(np.float64) @ W.astype(np.float64) + skip
    ref = orc.act_bwd(lin, u, "relu" if dact == 1 else "gelu")
    dC = empty_dev((M, N), dtype)
    tdy, tW, ts, ta = (to_dev(a, dtype) for a in (dy, W, skip, aux))
    b.check(b.lib().fl_test_gemm(dt_code(dtype), 1, 0, tdy.data_ptr(), tW.data_ptr(), dC.data_ptr(), M, N, K, None,
                                 ts.data_ptr(), 0, None, dact, ta.data_ptr(), 1, None, stream_ptr()))
    torch_mod().cuda.synchronize()
    assert rel_err(to_np(dC), ref) <= _tol(dtype)


@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11])
def test_gemm_epilogues_on_every_pipelined_variant(variant):
    """Bias, pre-activation copy, GELU and residual (forward form), and skip + GELU' (backward form), through
    the staged epilogue of every tile shape of the pipelined kernel; ragged M and N, several tiles.  Then the
    launches that select the other epilogue kinds of the specialised instances."""
    b = _lib()
    M, N, K = 520, 392, 128
    rng = np.random.default_rng(40 + variant)
    x = quantise(rng.standard_normal((M, K)), "bf16")
    W = quantise(rng.standard_normal((N, K)) * 0.2, "bf16")
    bias = quantise(rng.standard_normal(N), "bf16")
    res = quantise(rng.standard_normal((M, N)), "bf16")
    u_saved = quantise(rng.standard_normal((M, N)), "bf16")
    u = orc.linear_fwd(x, W, bias)
    ref_fwd = orc.act_fwd(u, "gelu") + res
    ref_bwd = orc.act_bwd(x.astype(np.float64) @ W.astype(np.float64).T + res, u_saved, "gelu")
    tx, tW, tb, tr, tu = (to_dev(a, "bf16") for a in (x, W, bias, res, u_saved))
    b.lib().fl_test_gemm_force_variant(variant)
    try:
        dC, dU = empty_dev((M, N), "bf16"), empty_dev((M, N), "bf16")
        b.check(b.lib().fl_test_gemm(1, 1, 1, tx.data_ptr(), tW.data_ptr(), dC.data_ptr(), M, N, K, tb.data_ptr(),
                                     tr.data_ptr(), 2, dU.data_ptr(), 0, None, 1, None, stream_ptr()))
        torch_mod().cuda.synchronize()
        assert rel_err(to_np(dC), ref_fwd) <= BF16_KERNEL_TOL, variant
        assert rel_err(to_np(dU), u) <= BF16_KERNEL_TOL, variant
        dC = empty_dev((M, N), "bf16")
        b.check(b.lib().fl_test_gemm(1, 1, 1, tx.data_ptr(), tW.data_ptr(), dC.data_ptr(), M, N, K, None,
                                     tr.data_ptr(), 0, None, 2, tu.data_ptr(), 1, None, stream_ptr()))
        torch_mod().cuda.synchronize()
        assert rel_err(to_np(dC), ref_bwd) <= BF16_KERNEL_TOL, variant
        # the other epilogue kinds of an instance: ReLU forward with and without the pre-activation copy, ReLU'
        # backward, bias + residual only, bias only
        ref_relu = orc.act_fwd(u, "relu") + res
        for with_preact in (True, False):
            dC, dU = empty_dev((M, N), "bf16"), empty_dev((M, N), "bf16")
            b.check(b.lib().fl_test_gemm(1, 1, 1, tx.data_ptr(), tW.data_ptr(), dC.data_ptr(), M, N, K, tb.data_ptr(),
                                         tr.data_ptr(), 1, dU.data_ptr() if with_preact else None, 0, None, 1, None,
                                         stream_ptr()))
            torch_mod().cuda.synchronize()
            assert rel_err(to_np(dC), ref_relu) <= BF16_KERNEL_TOL, (variant, with_preact)
            if with_preact:
                assert rel_err(to_np(dU), u) <= BF16_KERNEL_TOL, variant
        ref_relu_bwd = orc.act_bwd(x.astype(np.float64) @ W.astype(np.float64).T + res, u_saved, "relu")
        dC = empty_dev((M, N), "bf16")
        b.check(b.lib().fl_test_gemm(1, 1, 1, tx.data_ptr(), tW.data_ptr(), dC.data_ptr(), M, N, K, None,
                                     tr.data_ptr(), 0, None, 1, tu.data_ptr(), 1, None, stream_ptr()))
        torch_mod().cuda.synchronize()
        assert rel_err(to_np(dC), ref_relu_bwd) <= BF16_KERNEL_TOL, variant
        for with_res in (True, False):
            dC = empty_dev((M, N), "bf16")
            b.check(b.lib().fl_test_gemm(1, 1, 1, tx.data_ptr(), tW.data_ptr(), dC.data_ptr(), M, N, K, tb.data_ptr(),
                                         tr.data_ptr() if with_res else None, 0, None, 0, None, 1, None, stream_ptr()))
            torch_mod().cuda.synchronize()
            assert rel_err(to_np(dC), u + (res if with_res else 0.0)) <= BF16_KERNEL_TOL, (variant, with_res)
    finally:
        b.lib().fl_test_gemm_force_variant(-1)


def test_gelu_in_the_gemm_epilogues_matches_the_exact_erf_form():
    """The epilogues' GELU and GELU' (a branch-free rational erf) against the oracle's exact erf form on
    |u| <= 6, through the fp32 GEMM so that nothing but the activation arithmetic rounds: absolute error
    below 2e-6 where the layer tolerance for a whole fp32 layer is 1e-4 of the largest value."""
    b = _lib()
    M, N, K = 4096, 8, 8
    u = np.linspace(-6.0, 6.0, M).astype(np.float32)
    A = np.zeros((M, K), np.float32)
    Bm = np.zeros((N, K), np.float32)
    Bm[:, 0] = 1.0
    A[:, 0] = u                                                     # A B^T = u, the same in all 8 columns
    dA, dB = to_dev(A, "f32"), to_dev(Bm, "f32")
    dC = empty_dev((M, N), "f32")
    b.check(b.lib().fl_test_gemm(0, 1, 1, dA.data_ptr(), dB.data_ptr(), dC.data_ptr(), M, N, K, None, None, 2, None, 0,
                                 None, 1, None, stream_ptr()))
    torch_mod().cuda.synchronize()
    ref = orc.gelu_fwd(u.astype(np.float64))[:, None].repeat(N, 1)
    assert np.max(np.abs(to_np(dC) - ref)) <= 2e-6
    A[:, 0] = 1.0                                                   # A B^T = 1, times gelu'(aux)
    aux = np.random.default_rng(0).uniform(-6.0, 6.0, (M, N)).astype(np.float32)
    dA, daux = to_dev(A, "f32"), to_dev(aux, "f32")
    b.check(b.lib().fl_test_gemm(0, 1, 1, dA.data_ptr(), dB.data_ptr(), dC.data_ptr(), M, N, K, None, None, 0, None, 2,
                                 daux.data_ptr(), 1, None, stream_ptr()))
    torch_mod().cuda.synchronize()
    ref = orc.gelu_bwd(np.ones((M, N)), aux.astype(np.float64))
    assert np.max(np.abs(to_np(dC) - ref)) <= 2e-6


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_mfma_probe_runs_and_reports_its_work(dtype):
    """The MFMA-only loop behind the benchmark's measured matrix-core ceiling: it runs, writes every output
    and reports the operations it launched."""
    import ctypes
    b = _lib()
    wgs, iters = 64, 10
    out = torch_mod().full((wgs * 256,), float("nan"), dtype=torch_mod().float32, device="cuda")
    flops = ctypes.c_double(0.0)
    b.check(b.lib().fl_test_mfma_probe(dt_code(dtype), wgs, iters, out.data_ptr(), ctypes.byref(flops), stream_ptr()))
    torch_mod().cuda.synchronize()
    assert bool(torch_mod().isfinite(out).all())
    assert flops.value == wgs * 4 * iters * 8 * 2.0 * 32 * 32 * (16 if dtype == "bf16" else 2)
    assert b.lib().fl_test_mfma_probe(dt_code(dtype), 0, iters, out.data_ptr(), None, stream_ptr()) != 0


def test_gemm_rejects_bad_shapes():
    b = _lib()
    d = empty_dev((64 * 64,), "f32")
    p = d.data_ptr()
    # N not a multiple of 8; misaligned pointer
    assert b.lib().fl_test_gemm(0, 1, 1, p, p, p, 16, 12, 16, None, None, 0, None, 0, None, 1, None, 0) == b.FL_ERR_UNSUPPORTED
    assert b.lib().fl_test_gemm(0, 1, 1, p + 4, p, p, 16, 16, 16, None, None, 0, None, 0, None, 1, None, 0) == b.FL_ERR_UNSUPPORTED
    assert b"launch_gemm" in b.lib().fl_last_error()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(32, 64), (203, 768), (1024, 256), (7, 1032), (5, 4096), (300, 2048), (70, 4096)])
def test_layernorm_forward_backward(dtype, shape):
    b = _lib()
    M, D = shape
    rng = np.random.default_rng(M * 31 + D)
    x = quantise(rng.standard_normal((M, D)) * 2 + 0.5, dtype)
    gam = quantise(1 + 0.1 * rng.standard_normal(D), dtype)
    bet = quantise(0.1 * rng.standard_normal(D), dtype)
    dy = quantise(rng.standard_normal((M, D)), dtype)
    add = quantise(rng.standard_normal((M, D)), dtype)
    eps = 1e-5
    y, xhat, rstd = orc.layernorm_fwd(x, gam, bet, eps)
    dx, dg, db = orc.layernorm_bwd(dy, xhat, rstd, gam)
    dX, dG, dB = to_dev(x, dtype), to_dev(gam, dtype), to_dev(bet, dtype)
    dYo, mean, rs = empty_dev((M, D), dtype), empty_dev((M,), "f32"), empty_dev((M,), "f32")
    b.check(b.lib().fl_test_layernorm_fwd(dt_code(dtype), dX.data_ptr(), dG.data_ptr(), dB.data_ptr(), eps, M, D,
                                          dYo.data_ptr(), mean.data_ptr(), rs.data_ptr(), stream_ptr()))
    torch_mod().cuda.synchronize()
    assert rel_err(to_np(dYo), y) <= _tol(dtype)
    assert rel_err(to_np(mean), x.astype(np.float64).mean(-1)) <= 1e-5
    assert rel_err(to_np(rs), rstd[:, 0]) <= 1e-5
    ws = empty_dev((b.lib().fl_test_layernorm_bwd_ws_floats(M, D),), "f32")
    tdy, tadd = to_dev(dy, dtype), to_dev(add, dtype)
    for with_add in (False, True):
        odx, odg, odb, ods = (empty_dev((M, D), dtype), empty_dev((D,), dtype), empty_dev((D,), dtype),
                              empty_dev((D,), dtype))
        b.check(b.lib().fl_test_layernorm_bwd(dt_code(dtype), tdy.data_ptr(), dX.data_ptr(),
                                              mean.data_ptr(), rs.data_ptr(), dG.data_ptr(),
                                              tadd.data_ptr() if with_add else None, M, D,
                                              odx.data_ptr(), odg.data_ptr(), odb.data_ptr(), ods.data_ptr(),
                                              ws.data_ptr(), stream_ptr()))
        torch_mod().cuda.synchronize()
        want = dx + (add if with_add else 0)
        assert rel_err(to_np(odx), want) <= _tol(dtype)
        assert rel_err(to_np(odg), dg) <= _tol(dtype)
        assert rel_err(to_np(odb), db) <= _tol(dtype)
        assert rel_err(to_np(ods), want.sum(0)) <= _tol(dtype) * 4   # column sums of values near zero mean


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(32, 192), (1000, 264), (4096, 3072), (1, 8)])
def test_colsum(dtype, shape):
    b = _lib()
    M, N = shape
    rng = np.random.default_rng(M + N)
    a = quantise(rng.standard_normal((M, N)), dtype)
    ws = empty_dev((b.lib().fl_test_colsum_ws_floats(M, N),), "f32")
    out = empty_dev((N,), dtype)
    ta = to_dev(a, dtype)
    b.check(b.lib().fl_test_colsum(dt_code(dtype), ta.data_ptr(), M, N, ws.data_ptr(), out.data_ptr(),
                                   stream_ptr()))
    torch_mod().cuda.synchronize()
    assert rel_err(to_np(out), a.astype(np.float64).sum(0)) <= _tol(dtype)


@pytest.mark.parametrize("shapes", [[(8, 8)], [(64, 64), (72, 200)], [(2304, 768), (768, 768), (3072, 768), (768, 3072)],
                                    [(136, 8), (8, 1000), (200, 328)]])
def test_transposed_weight_copies_are_exact(shapes):
    """Data movement only: every element must arrive unchanged, also in ragged edge tiles and with
    several matrices in one launch."""
    import ctypes
    b = _lib()
    rng = np.random.default_rng(len(shapes) * 1000 + shapes[0][0])
    src_np = [quantise(rng.standard_normal(sh), "bf16") for sh in shapes]
    src = [to_dev(a, "bf16") for a in src_np]
    dst = [empty_dev((sh[1], sh[0]), "bf16") for sh in shapes]
    n = len(shapes)
    arr_p = ctypes.c_void_p * n
    arr_i = ctypes.c_int32 * n
    b.check(b.lib().fl_test_transpose_bf16(n, arr_p(*[t.data_ptr() for t in src]), arr_p(*[t.data_ptr() for t in dst]),
                                           arr_i(*[sh[0] for sh in shapes]), arr_i(*[sh[1] for sh in shapes]),
                                           stream_ptr()))
    torch_mod().cuda.synchronize()
    for a, d in zip(src_np, dst):
        assert np.array_equal(to_np(d), a.T)


def test_transpose_rejects_sizes_that_are_not_multiples_of_eight():
    import ctypes
    b = _lib()
    t = empty_dev((16, 12), "bf16")
    o = empty_dev((12, 16), "bf16")
    rc = b.lib().fl_test_transpose_bf16(1, (ctypes.c_void_p * 1)(t.data_ptr()), (ctypes.c_void_p * 1)(o.data_ptr()),
                                        (ctypes.c_int32 * 1)(16), (ctypes.c_int32 * 1)(12), stream_ptr())
    assert rc != 0


ATTN_CASES = [  # B, T, H, dh, lengths
    (2, 16, 4, 16, None),
    (2, 200, 2, 32, [200, 65]),
    (1, 129, 1, 96, [100]),
    (1, 64, 2, 128, None),
    (3, 37, 2, 64, [1, 20, 37]),
    (2, 128, 3, 64, [64, 128]),
    (2, 197, 2, 64, None),
    (1, 300, 2, 192, [171]),
    (2, 70, 1, 256, [70, 33]),
    (2, 75, 2, 48, [75, 9]),      # head sizes between the multiples of 32: padded kernel instances
    (1, 45, 1, 112, None),
    # head sizes 129..192 (bf16 forward: two key groups of wavefronts per query block, merged at the end):
    (2, 30, 1, 192, [30, 7]),     # less than one 32-key block: the second group sees no key at all
    (2, 64, 2, 192, [64, 33]),    # exactly one tile; one key for the second group
    (1, 130, 1, 160, [97]),       # padded instance, an odd number of tiles
    (2, 257, 1, 192, [257, 128]), # a last tile of one key; a length on a tile boundary
]


@pytest.mark.parametrize("causal,p_drop", [(False, 0.0), (True, 0.0), (False, 0.2), (True, 0.35)])
@pytest.mark.parametrize("dtype", ["f32", "f32-general", "bf16", "bf16-general"])
@pytest.mark.parametrize("case", ATTN_CASES)
def test_attention_forward_backward(dtype, case, causal, p_drop):
    """Both types run the MFMA kernels where the head size allows; "-general" forces the general ones.
    With p_drop > 0 the oracle regenerates the identical keep mask from the same seed."""
    b = _lib()
    general = dtype.endswith("-general")
    dtype = dtype.split("-")[0]
    b.lib().fl_test_attention_force_general(1 if general else 0)
    try:
        _attention_case(b, dtype, case, causal, p_drop)
    finally:
        b.lib().fl_test_attention_force_general(0)


@pytest.mark.parametrize("causal,p_drop", [(False, 0.0), (True, 0.0), (False, 0.2), (True, 0.35)])
def test_attention_forward_large_head_with_a_sequence_of_one_key(causal, p_drop):
    """Forward only (output and log-sum-exp against the oracle): with one key and dropout the reference gradient
    is exactly 0 and the kernels return the rounding noise of the stored output, see
    test_one_kernel_attention_backward_agrees_with_the_two_kernel_path."""
    _attention_case(_lib(), "bf16", (2, 30, 1, 192, [30, 1]), causal, p_drop, check_backward=False)


ATTN_ONE_KERNEL_BWD_CASES = [  # head size 64 and T <= 224: the one-kernel backward (2, 4, 6 or 8 wavefronts)
    (2, 1, 2, 64, None),
    (2, 32, 1, 64, [32, 5]),
    (1, 64, 3, 64, [33]),
    (2, 65, 2, 64, [65, 64]),
    (2, 100, 2, 64, [31, 100]),
    (1, 130, 2, 64, [97]),
    (2, 192, 1, 64, [192, 40]),
    (2, 224, 2, 64, [224, 129]),
    (1, 225, 1, 64, [200]),       # one row too long: falls back to the two-kernel path
]


@pytest.mark.parametrize("causal,p_drop", [(False, 0.0), (True, 0.0), (False, 0.2), (True, 0.35)])
@pytest.mark.parametrize("unfused", [False, True])
@pytest.mark.parametrize("case", ATTN_ONE_KERNEL_BWD_CASES + [c for c in ATTN_CASES if c[3] == 64])
def test_attention_backward_in_one_kernel_and_in_two(case, unfused, causal, p_drop):
    """Head size 64 with T <= 224 runs dQ, dK and dV in one kernel; `unfused` puts the same problem on the
    dQ + dK/dV kernels.  Both are checked against the oracle."""
    b = _lib()
    b.lib().fl_test_attention_force_unfused_bwd(1 if unfused else 0)
    try:
        _attention_case(b, "bf16", case, causal, p_drop)
    finally:
        b.lib().fl_test_attention_force_unfused_bwd(0)


@pytest.mark.parametrize("causal,p_drop", [(False, 0.0), (True, 0.3)])
@pytest.mark.parametrize("case", [(2, 192, 1, 64, [192, 1]), (3, 128, 2, 64, [128, 64, 100]), (2, 197, 3, 64, None)])
def test_one_kernel_attention_backward_agrees_with_the_two_kernel_path(case, causal, p_drop):
    """Same inputs (the forward's own O and log-sum-exp), same mask: the two paths differ in the order
    of their fp32 sums only.  Includes a sequence of length 1 under dropout, where the reference
    gradient is exactly 0 and both paths return the rounding noise of the stored O (delta = dO . O), which
    is why that case is compared between the paths and not with the oracle."""
    b = _lib()
    got = {}
    for unfused in (False, True):
        b.lib().fl_test_attention_force_unfused_bwd(1 if unfused else 0)
        try:
            got[unfused] = _attention_case(b, "bf16", case, causal, p_drop, check_backward=False)
        finally:
            b.lib().fl_test_attention_force_unfused_bwd(0)
    assert rel_err(got[False], got[True]) <= 4e-3      # one bf16 rounding step of the largest element


def _attention_case(b, dtype, case, causal=False, p_drop=0.0, check_backward=True):
    B, T, H, dh, lengths = case
    seed = (0x9E3779B9 << 32) | (B * 7919 + T)
    keep = None
    p_drop = float(np.float32(p_drop))       # the ABI takes a C float: the oracle gets the same value
    if p_drop > 0:
        from oracle import dropout as odr
        keep = odr.keep_mask_attention(B, H, T, p_drop, seed)
    D = H * dh
    rng = np.random.default_rng(B * 1000 + T)
    qkv = quantise(rng.standard_normal((B, T, 3 * D)), dtype)
    dO = quantise(rng.standard_normal((B, T, D)), dtype)
    Q, K, V = (orc.split_heads(qkv[..., i * D:(i + 1) * D].astype(np.float64), H) for i in range(3))
    Oh, P = orc.attention_fwd(Q, K, V, lengths, causal, keep)
    O = orc.merge_heads(Oh)
    S = (Q @ K.transpose(0, 1, 3, 2)) / math.sqrt(dh)
    if lengths is not None:
        S = np.where(orc.key_mask(lengths, B, T)[:, None, None, :], -np.inf, S)
    if causal:
        S = np.where(np.triu(np.ones((T, T), bool), 1)[None, None], -np.inf, S)
    lse_ref = np.log(np.exp(S - S.max(-1, keepdims=True)).sum(-1)) + S.max(-1)
    dQ, dK, dV = orc.attention_bwd(orc.split_heads(dO.astype(np.float64), H), Q, K, V, P, keep)
    dqkv_ref = np.concatenate([orc.merge_heads(dQ), orc.merge_heads(dK), orc.merge_heads(dV)], -1)
    torch = torch_mod()
    dl = torch.tensor(lengths, dtype=torch.int32, device="cuda") if lengths is not None else None
    dqkv_in = to_dev(qkv, dtype)
    o, lse = empty_dev((B, T, D), dtype), empty_dev((B, H, T), "f32")
    b.check(b.lib().fl_test_attention_fwd(dt_code(dtype), dqkv_in.data_ptr(), dl.data_ptr() if dl is not None else None,
                                          int(causal), p_drop, seed, B, T, H, dh, o.data_ptr(), lse.data_ptr(),
                                          stream_ptr()))
    torch.cuda.synchronize()
    assert rel_err(to_np(o), O) <= _tol(dtype)
    assert rel_err(to_np(lse), lse_ref) <= 1e-5
    # backward consumes the GPU's own o and lse, as in the layer
    dqkv, delta = empty_dev((B, T, 3 * D), dtype), empty_dev((B, H, T), "f32")
    tdo = to_dev(dO, dtype)
    b.check(b.lib().fl_test_attention_bwd(dt_code(dtype), dqkv_in.data_ptr(), o.data_ptr(), tdo.data_ptr(),
                                          lse.data_ptr(), dl.data_ptr() if dl is not None else None, int(causal),
                                          p_drop, seed, B, T, H, dh, dqkv.data_ptr(), delta.data_ptr(),
                                          stream_ptr()))
    torch.cuda.synchronize()
    got = to_np(dqkv)
    if not check_backward:
        return got
    # delta_i = sum_j P_ij dP_ij is taken as dO_i . O_i from the stored (rounded) O; dropout scales the
    # probabilities, and with them that rounding noise, by 1/(1-p)
    gtol = _tol(dtype) * 2 / (1.0 - p_drop)
    for i, name in enumerate("qkv"):
        assert rel_err(got[..., i * D:(i + 1) * D], dqkv_ref[..., i * D:(i + 1) * D]) <= gtol, name
    if lengths is not None:      # masked keys: exactly zero gradient rows
        for bi, n in enumerate(lengths):
            assert np.all(got[bi, n:, D:] == 0.0)
    return got


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,N,site,p", [(37, 64, 2, 0.1), (300, 776, 3, 0.5), (1, 8, 4, 0.9), (513, 3072, 3, 0.25)])
def test_dropout_mask_is_bit_identical_to_the_oracle(dtype, M, N, site, p):
    """The device generator (Philox4x32-10) and the keep decision are integer work: applied to ones, the
    kernel must reproduce the oracle's mask exactly (0 or the scale 1/(1-p) rounded to the storage type)."""
    from oracle import dropout as odr
    b = _lib()
    seed = (0xC0FFEE << 32) | 0xDEADBEEF
    ones = to_dev(np.ones((M, N), np.float32), dtype)
    out = empty_dev((M, N), dtype)
    b.check(b.lib().fl_test_dropout_mul(dt_code(dtype), ones.data_ptr(), out.data_ptr(), M, N, site, p, seed,
                                        stream_ptr()))
    torch_mod().cuda.synchronize()
    got = to_np(out)
    p = float(np.float32(p))                 # the ABI takes a C float
    want = odr.keep_mask_rows(M, N, site, p, seed)
    assert np.array_equal(got != 0, want != 0)
    scale = quantise(np.array([np.float32(1.0 / (1.0 - p))]), dtype)[0]
    assert np.all(got[got != 0] == scale)
