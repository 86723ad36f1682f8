"""Helpers of the GPU parity tests: device buffers through torch, calls through the C ABI binding."""
import numpy as np


def device_inputs(B, alpha, X):
    import torch

    dev = torch.device("cuda:0")
    return (torch.from_numpy(B).to(dev), torch.from_numpy(alpha).to(dev), torch.from_numpy(X).to(dev))


def gpu_pack(biq, B_dev, mu=8):
    import torch

    q, m, n = B_dev.shape
    K = torch.empty(biq.biq_packed_bytes(m, n, q), dtype=torch.uint8, device=B_dev.device)
    K.fill_(0xA5)  # poison: padding must be written by the kernel
    biq.biq_pack(B_dev, K, m, n, q, mu)
    return K


def gpu_gemm(biq, K, alpha_dev, X_dev, m, n, q, mu, plan=None):
    import torch

    batch = X_dev.shape[0]
    Y = torch.full((batch, m), float("nan"), dtype=torch.float32, device=X_dev.device)
    if plan is None:
        ws_bytes = biq.biq_workspace_bytes(m, n, q, batch, mu)
    else:
        ws_bytes = biq.biq_plan_workspace_bytes(biq.biq_plan_check(m, n, q, batch, mu, plan), m, batch)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=X_dev.device) if ws_bytes else None
    if plan is None:
        biq.biq_gemm(K, alpha_dev, X_dev, Y, m, n, q, batch, mu, workspace=ws)
    else:
        biq.biq_gemm_ex(K, alpha_dev, X_dev, Y, m, n, q, batch, mu, plan, workspace=ws)
    torch.cuda.synchronize()
    return Y


def assert_within_tolerance(Y_gpu, Y_ref, alpha, X, what=""):
    """The stated bar: per input vector a, max|dy| <= 1e-4 * max_r(sum_i |alpha_i[r]|) * ||x_a||_1
    and relative L2 error <= 1e-5, per vector and over all of Y.  Y_ref is fp64."""
    Y_gpu = np.asarray(Y_gpu, dtype=np.float64)
    Y_ref = np.asarray(Y_ref, dtype=np.float64)
    assert Y_gpu.shape == Y_ref.shape, (Y_gpu.shape, Y_ref.shape)
    assert np.all(np.isfinite(Y_gpu)), "%s: non-finite output" % what
    amax = np.abs(alpha.astype(np.float64)).sum(axis=0).max()
    l1 = np.abs(X.astype(np.float64)).sum(axis=1)
    err = np.abs(Y_gpu - Y_ref).max(axis=1)
    bound = 1e-4 * amax * l1
    assert np.all(err <= bound), "%s: max abs error %s exceeds %s" % (what, err.max(), bound.min())
    num = np.sqrt(((Y_gpu - Y_ref) ** 2).sum(axis=1))
    den = np.sqrt((Y_ref ** 2).sum(axis=1))
    rel = num / np.maximum(den, 1e-300)
    assert np.all(rel <= 1e-5), "%s: per-vector relative L2 error %s" % (what, rel.max())
    tot = np.sqrt(((Y_gpu - Y_ref) ** 2).sum()) / max(np.sqrt((Y_ref ** 2).sum()), 1e-300)
    assert tot <= 1e-5, "%s: relative L2 error %s" % (what, tot)
    return float(err.max()), float(tot)
