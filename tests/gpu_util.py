"""Helpers for the GPU parity tests: torch is used only to own device memory."""
import numpy as np

F32_TOL = 1e-4    # spec tolerance of the fp32 path (error relative to the tensor's infinity norm)
BF16_TOL = 2e-2   # spec tolerance of the bf16-storage / fp32-accumulate path
# Kernel-level bounds derived from the arithmetic: one bf16 rounding of the output is at most
# 2^-9 of each element, plus fp32 accumulation error; fp32 kernels accumulate in fp32.
F32_KERNEL_TOL = 2e-5
BF16_KERNEL_TOL = 6e-3


def torch_mod():
    import torch
    return torch


def to_dev(a, dtype):
    """numpy array -> contiguous device tensor of the storage type ("f32" | "bf16")."""
    torch = torch_mod()
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16).contiguous() if dtype == "bf16" else t.contiguous()


def empty_dev(shape, dtype):
    torch = torch_mod()
    td = {"f32": torch.float32, "bf16": torch.bfloat16, "i32": torch.int32}[dtype]
    # NaN-filled so that an element the kernel forgets to write is caught
    t = torch.empty(shape, dtype=td, device="cuda")
    if dtype != "i32":
        t.fill_(float("nan"))
    return t


def to_np(t):
    torch = torch_mod()
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def rel_err(got, ref):
    """max |got - ref| / max |ref| (error relative to the reference tensor's infinity norm)."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), "non-finite values in the GPU result"
    den = np.max(np.abs(ref))
    if den == 0.0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - ref)) / den)


def rel_err_l2(got, ref):
    """||got - ref||_2 / ||ref||_2, reported beside rel_err."""
    got, ref = np.asarray(got, np.float64).ravel(), np.asarray(ref, np.float64).ravel()
    den = float(np.linalg.norm(ref))
    num = float(np.linalg.norm(got - ref))
    return num if den == 0.0 else num / den


def log_errors(test, errs, l2=None, extra=None):
    """Appends one JSON line with a parity test's measured errors to the file named by FL_PARITY_LOG
    (if set): the figures quoted in the design notes come from there."""
    import json
    import os
    path = os.environ.get("FL_PARITY_LOG")
    if not path:
        return
    rec = {"test": test, "max_inf": max(errs.values()), "inf": errs}
    if l2 is not None:
        rec["max_l2"] = max(l2.values())
        rec["l2"] = l2
    if extra:
        rec.update(extra)
    with open(path, "a") as f:
        f.write(json.dumps(rec) + "\n")


def stream_ptr():
    torch = torch_mod()
    return torch.cuda.current_stream().cuda_stream


def dt_code(dtype):
    return 0 if dtype == "f32" else 1


def quantise(a, dtype):
    from workloads import round_to_bf16
    a = np.asarray(a, np.float32)
    return round_to_bf16(a) if dtype == "bf16" else a
