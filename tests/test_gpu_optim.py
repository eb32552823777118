"""Parity of the fused optimizer step, zero-grad and gradient accumulation with the CPU oracle."""
import numpy as np
import pytest

from oracle import optim as oo
from oracle import oracle as orc
from gpu_util import BF16_TOL, F32_TOL, empty_dev, quantise, rel_err, stream_ptr, to_dev, to_np, torch_mod
from workloads import CONFIGS, PARAM_NAMES, make_inputs

pytestmark = pytest.mark.gpu

SIZES = [8, 776, 4096 * 3 + 8, 768 * 768]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("kind,hyper", [
    ("sgd", dict(lr=0.05)),
    ("sgd", dict(lr=0.05, momentum=0.9, weight_decay=0.01)),
    ("adam", dict(lr=1e-2, beta1=0.9, beta2=0.98, eps=1e-6)),
    ("adam", dict(lr=1e-2, beta1=0.8, beta2=0.9, eps=1e-8, weight_decay=0.1)),
])
def test_optimizer_steps_match_oracle(dtype, kind, hyper):
    from paper_2201_12465_amd import binding as b
    torch = torch_mod()
    rng = np.random.default_rng(3)
    ps = [quantise(rng.standard_normal(n), dtype) for n in SIZES]
    dp = [to_dev(p, dtype) for p in ps]
    dm = [torch.zeros(n, dtype=torch.float32, device="cuda") for n in SIZES]
    dv = [torch.zeros(n, dtype=torch.float32, device="cuda") for n in SIZES]
    ref_p = [p.astype(np.float64) for p in ps]
    ref_m = [np.zeros(n) for n in SIZES]
    ref_v = [np.zeros(n) for n in SIZES]
    # the parameter is rounded to the storage type after every step on the GPU; the oracle is fed the
    # GPU's rounded parameter each step so that one step's arithmetic is compared, not the drift
    tol = 1e-6 if dtype == "f32" else 2.0 ** -8
    for step in range(1, 4):
        gs = [quantise(rng.standard_normal(n), dtype) for n in SIZES]
        dg = [to_dev(g, dtype) for g in gs]
        b.opt_step(kind, dtype, dp, dg, dm, dv if kind == "adam" else None, SIZES, stream_ptr(), step=step, **hyper)
        torch.cuda.synchronize()
        for i in range(len(SIZES)):
            if kind == "sgd":
                kw = {k: v for k, v in hyper.items()}
                ref_p[i], ref_m[i] = oo.sgd_step(ref_p[i], gs[i], ref_m[i], **kw)
            else:
                ref_p[i], ref_m[i], ref_v[i] = oo.adam_step(ref_p[i], gs[i], ref_m[i], ref_v[i], step=step, **hyper)
            got = to_np(dp[i])
            assert rel_err(got, ref_p[i]) <= tol, (kind, dtype, step, i)
            if kind == "adam" or hyper.get("momentum"):
                assert rel_err(to_np(dm[i]), ref_m[i]) <= 1e-5
            if kind == "adam":
                assert rel_err(to_np(dv[i]), ref_v[i]) <= 1e-5
            ref_p[i] = got          # continue from the stored (rounded) parameter


def test_master_copies_keep_small_adam_steps_that_bf16_storage_loses():
    """100 Adam steps of lr = 1e-4 on bf16 weights ~ N(0, 0.02) (spacing 6e-5 near 0.02): with fp32 master
    copies the parameters follow the fp64 oracle; without them most of every update is rounded away."""
    from paper_2201_12465_amd import binding as b
    torch = torch_mod()
    rng = np.random.default_rng(11)
    n, steps, hyper = 4096, 100, dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8)
    p0 = quantise(0.02 * rng.standard_normal(n), "bf16")
    grads = [quantise(rng.standard_normal(n) + 0.5, "bf16") for _ in range(steps)]   # a consistent drift plus noise
    ref_p, ref_m, ref_v = p0.astype(np.float64), np.zeros(n), np.zeros(n)
    for t, g in enumerate(grads, 1):
        ref_p, ref_m, ref_v = oo.adam_step(ref_p, g, ref_m, ref_v, step=t, **hyper)
    moved = float(np.max(np.abs(ref_p - p0)))
    out = {}
    for with_master in (True, False):
        dp = to_dev(p0, "bf16")
        master = torch.from_numpy(p0.astype(np.float32)).cuda() if with_master else None
        dm, dv = torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
        for t, g in enumerate(grads, 1):
            b.opt_step("adam", "bf16", [dp], [to_dev(g, "bf16")], [dm], [dv], [n], stream_ptr(), step=t,
                       master=[master] if with_master else None, **hyper)
        torch.cuda.synchronize()
        out[with_master] = float(np.max(np.abs(to_np(dp) - ref_p))) / moved
        if with_master:   # what is left is the one rounding of the result to bf16: half a spacing of the value
            half_ulp = 2.0 ** (np.floor(np.log2(np.abs(ref_p))) - 8)
            assert np.all(np.abs(to_np(dp) - ref_p) <= 1.02 * half_ulp)
        if with_master:
            assert float(np.max(np.abs(master.cpu().numpy().astype(np.float64) - ref_p))) / moved <= 1e-4
            assert torch.equal(dp, master.to(torch.bfloat16))      # the bf16 parameter is the rounded master copy
    assert out[True] <= 0.05        # that rounding (at most 4.9e-4 / 2 here) against a movement of ~1e-2
    assert out[False] >= 5 * out[True], out


def test_zero_grad_and_argument_checks():
    from paper_2201_12465_amd import binding as b
    torch = torch_mod()
    g = [torch.full((n,), 3.0, dtype=torch.bfloat16, device="cuda") for n in SIZES]
    b.zero_grad("bf16", g, SIZES, stream_ptr())
    torch.cuda.synchronize()
    assert all(float(t.float().abs().max()) == 0.0 for t in g)
    p = torch.zeros(12, device="cuda")
    with pytest.raises(b.FlError) as e:                      # numel not a multiple of 8
        b.opt_step("sgd", "f32", [p], [p], None, None, [12], stream_ptr(), lr=0.1)
    assert e.value.status == b.FL_ERR_UNSUPPORTED
    with pytest.raises(b.FlError) as e:                      # Adam without state
        b.opt_step("adam", "f32", [p], [p], None, None, [8], stream_ptr(), lr=0.1)
    assert e.value.status == b.FL_ERR_UNSUPPORTED
    with pytest.raises(b.FlError) as e:                      # Adam step counter starts at 1
        b.opt_step("adam", "f32", [p], [p], [p], [p], [8], stream_ptr(), lr=0.1, step=0)
    assert e.value.status == b.FL_ERR_INVALID_ARG


@pytest.mark.parametrize("name", ["cfg2_small_f32", "cfg3_bert_base_bf16"])
def test_gradient_accumulation_over_two_micro_batches(name):
    """backward(accumulate) adds to the stored gradients: two micro-batches against the oracle's sum."""
    from paper_2201_12465_amd import binding as b
    torch = torch_mod()
    cfg = CONFIGS[name].with_(B=4, act="gelu")      # GELU: no ReLU-kink bookkeeping needed here
    dt = cfg.dtype
    inps = [make_inputs(cfg, seed=s, nontrivial=True) for s in (0, 1)]
    params = inps[0]["params"]
    layer = b.Layer(cfg.B, cfg.T, cfg.D, cfg.H, cfg.F, cfg.act, cfg.norm, dt, cfg.eps)
    p = {k: to_dev(v, dt) for k, v in params.items()}
    g = {k: empty_dev(v.shape, dt) for k, v in params.items()}
    sizes = [int(np.prod(params[k].shape)) for k in PARAM_NAMES]
    b.zero_grad(dt, [g[k] for k in PARAM_NAMES], sizes, stream_ptr())
    ref = {k: np.zeros(params[k].shape) for k in PARAM_NAMES}
    for inp in inps:
        X, dY = to_dev(inp["X"], dt), to_dev(inp["dY"], dt)
        Y, dX = empty_dev(X.shape, dt), empty_dev(X.shape, dt)
        L = torch.tensor(inp["lengths"], dtype=torch.int32, device="cuda") if inp["lengths"] is not None else None
        layer.forward(p, X, L, cfg.B, cfg.T, Y, stream_ptr())
        layer.backward(p, dY, dX, g, stream_ptr(), accumulate=True)
        torch.cuda.synchronize()
        _, _, rg = orc.layer_forward_backward(params, inp["X"], inp["dY"], inp["lengths"], heads=cfg.H, act=cfg.act,
                                              norm=cfg.norm, eps=cfg.eps)
        for k in PARAM_NAMES:
            ref[k] = oo.accumulate(ref[k], rg[k])
    tol = F32_TOL if dt == "f32" else BF16_TOL
    errs = {k: rel_err(to_np(g[k]), ref[k]) for k in PARAM_NAMES}
    assert all(v <= tol for v in errs.values()), errs
    layer.destroy()
