"""Shared helpers of the GPU parity tests: upload of seeded inputs, the error metric, tolerances."""
import numpy as np

# tolerances of the benchmark definition: max|gpu - oracle| / max|oracle| per output tensor
TOL = {"f32": 1e-4, "bf16": 2e-2}


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.max(np.abs(ref))
    return float(np.max(np.abs(got - ref)) / (den if den > 0 else 1.0))


def rel_l2(got, ref):
    """||got - ref||_2 / ||ref||_2 over the whole tensor (reported beside the max-norm error, never the bar)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = float(np.sqrt(np.sum(np.abs(ref) ** 2)))
    return float(np.sqrt(np.sum(np.abs(got - ref) ** 2)) / (den if den > 0 else 1.0))


def check_outputs(pairs, where=""):
    """pairs: {name: (got, ref, tol)}.  The bar is the max-norm relative error of each tensor; a failure message
    lists every tensor's max-norm and L2 relative errors."""
    rep, bad = {}, []
    for name, (got, ref, tol) in pairs.items():
        e, l2 = rel_err(got, ref), rel_l2(got, ref)
        rep[name] = f"max {e:.2e} / l2 {l2:.2e} (tol {tol:g})"
        if not e <= tol:
            bad.append(name)
    assert not bad, f"{where}: over tolerance: {bad}; all outputs: {rep}"
    return rep


def dev(a, io=None):
    """numpy float32 (already rounded to the I/O dtype by workloads) -> cuda tensor of that dtype."""
    import torch
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    if io == "bf16":
        t = t.to(torch.bfloat16)
    return t


def host(t):
    import torch
    if t is None:
        return None
    if t.dtype == torch.bfloat16:
        t = t.float()
    return t.detach().cpu().numpy()


def sel_inputs_dev(p, io):
    """Device tensors of a workloads.make_selective dict: I/O tensors in `io`, parameters in fp32."""
    return dict(
        u=dev(p["u"], io), delta=dev(p["delta"], io), A=dev(p["A"]), Bm=dev(p["Bm"], io), Cm=dev(p["Cm"], io),
        Dskip=dev(p["Dskip"]), delta_bias=dev(p["delta_bias"]), z=dev(p["z"], io), x0=dev(p["x0"]),
    )
