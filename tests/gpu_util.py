"""Helpers for the GPU parity tests: upload seeded host data, run the HIP library through the
C ABI, and compare with the CPU oracle under the stated tolerances."""
import numpy as np

from paper_2502_20493_amd import binding as ukst

TOL = {"f32": 1e-5, "bf16": 1e-2}  # |y_gpu - y_oracle| <= TOL * sum|x*w| per output


def to_device(data, dtype):
    import torch
    if dtype == "bf16":
        x = torch.from_numpy(data["x_bits"].view(np.int16)).view(torch.bfloat16).cuda()
        w = torch.from_numpy(data["w_bits"].view(np.int16)).view(torch.bfloat16).cuda()
    else:
        x = torch.from_numpy(data["x"]).cuda()
        w = torch.from_numpy(data["w"]).cuda()
    return x.contiguous(), w.contiguous()


def run_gpu(data, dtype, P, path=ukst.UKST_PATH_AUTO, guard=0, sentinel=-777.0, workspace=False):
    """Returns y as a numpy fp32 array.  With guard > 0 the output lives in the middle of a larger
    buffer filled with a sentinel, and the bands before/after are checked to be untouched.
    workspace=False: ukst_conv_transpose2d_path; None: ukst_conv_transpose2d_ws with a workspace
    of ukst_workspace_bytes allocated for the call."""
    import torch
    x, w = to_device(data, dtype)
    B, Cin, H, W = x.shape
    Cout, _, n, _ = w.shape
    OH, OW = ukst.ukst_output_shape(H, W, n, P)
    numel = B * Cout * OH * OW
    buf = torch.full((numel + 2 * guard,), sentinel, dtype=torch.float32, device="cuda")
    y = buf[guard:guard + numel].view(B, Cout, OH, OW)
    ukst.ukst_conv_transpose2d(x, w, P, y=y, path=path, workspace=workspace)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    if guard:
        assert (host[:guard] == sentinel).all(), "wrote before the output tensor"
        assert (host[guard + numel:] == sentinel).all(), "wrote past the output tensor"
    return host[guard:guard + numel].reshape(B, Cout, OH, OW)


def check_against_oracle(y_gpu, y_ref, S, tol, planes=None, exact=False):
    """Element-by-element check.  planes: list of b*Cout+co ids the oracle computed."""
    B, Cout = y_gpu.shape[:2]
    g = y_gpu.reshape(B * Cout, -1)
    r = y_ref.reshape(B * Cout, -1)
    s = S.reshape(B * Cout, -1)
    if planes is not None:
        g, r, s = g[planes], r[planes], s[planes]
    g = g.astype(np.float64)
    assert np.isfinite(g).all()
    if exact:
        assert np.array_equal(g, r), f"max abs diff {np.abs(g - r).max()}"
        return 0.0
    err = np.abs(g - r)
    assert (err <= tol * s).all(), (
        f"worst err/S = {np.max(err / np.maximum(s, 1e-300)):.3e} (tol {tol}), "
        f"max err {err.max():.3e}")
    zero = s == 0
    assert (g[zero] == 0).all(), "outputs whose window meets no input must be exactly 0"
    return float(np.max(err / np.maximum(s, 1e-30)))


def _dev(a32, bits, dtype):
    import torch
    if dtype == "bf16":
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda().contiguous()
    return torch.from_numpy(a32).cuda().contiguous()


def _guarded(shape, guard, sentinel):
    import torch
    numel = int(np.prod(shape))
    buf = torch.full((numel + 2 * guard,), sentinel, dtype=torch.float32, device="cuda")
    return buf, buf[guard:guard + numel].view(*shape)


def _read_guarded(buf, shape, guard, sentinel):
    host = buf.cpu().numpy()
    numel = int(np.prod(shape))
    if guard:
        assert (host[:guard] == sentinel).all(), "wrote before the output tensor"
        assert (host[guard + numel:] == sentinel).all(), "wrote past the output tensor"
    return host[guard:guard + numel].reshape(shape)


def run_gpu_grad_input(data, dyd, dtype, H, W, P, guard=0, sentinel=-777.0):
    """dx as a numpy fp32 array, computed by the HIP library; guard bands as in run_gpu."""
    import torch
    dy = _dev(dyd["dy"], dyd.get("dy_bits"), dtype)
    w = _dev(data["w"], data.get("w_bits"), dtype)
    shape = (dy.shape[0], w.shape[1], H, W)
    buf, dx = _guarded(shape, guard, sentinel)
    ukst.ukst_conv_transpose2d_grad_input(dy, w, H, W, P, dx=dx)
    torch.cuda.synchronize()
    return _read_guarded(buf, shape, guard, sentinel)


def run_gpu_grad_weight(data, dyd, dtype, n, P, guard=0, sentinel=-777.0):
    """dw as a numpy fp32 array, computed by the HIP library; guard bands as in run_gpu."""
    import torch
    x = _dev(data["x"], data.get("x_bits"), dtype)
    dy = _dev(dyd["dy"], dyd.get("dy_bits"), dtype)
    shape = (dy.shape[1], x.shape[1], n, n)
    buf, dw = _guarded(shape, guard, sentinel)
    ukst.ukst_conv_transpose2d_grad_weight(x, dy, n, P, dw=dw)
    torch.cuda.synchronize()
    return _read_guarded(buf, shape, guard, sentinel)


def check_elements(g, r, s, tol, exact=False):
    """Element-by-element check of any gradient tensor against the oracle (same shapes)."""
    g = np.asarray(g, dtype=np.float64)
    assert g.shape == r.shape and np.isfinite(g).all()
    if exact:
        assert np.array_equal(g, r), f"max abs diff {np.abs(g - r).max()}"
        return 0.0
    err = np.abs(g - r)
    assert (err <= tol * s).all(), (
        f"worst err/S = {np.max(err / np.maximum(s, 1e-300)):.3e} (tol {tol}), max err {err.max():.3e}")
    assert (g[s == 0] == 0).all(), "elements that meet no product must be exactly 0"
    return float(np.max(err / np.maximum(s, 1e-30)))
