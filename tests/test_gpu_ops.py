"""Per-kernel parity: each HIP operator against the oracle's matching sub-function."""
import numpy as np
import pytest
import torch

import synth
from gpu_common import RTOL, assert_close_scaled
from oracle import spd_oracle as O

pytestmark = pytest.mark.gpu


def P():
    import paper_2405_18400_amd as pkg
    return pkg


def mat(rows, cols, dtype, seed, std=0.02):
    rng = np.random.default_rng(seed)
    w = (rng.standard_normal((rows, cols), dtype=np.float32) * std).astype(np.float32)
    if dtype == "bf16":
        bits = synth.bf16_bits(w).reshape(rows, cols)
        return bits, synth.bf16_widen(bits)
    if dtype == "fp16":      # key/value cache only: numpy's own binary16 rounding (to nearest even)
        h = w.astype(np.float16)
        return h, h.astype(np.float32)
    return w, w


def dev(a, dtype):
    if dtype == "fp16":
        return torch.from_numpy(a).cuda()
    return P().binding.to_device(a, dtype)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("rows,cols", [(4096, 4096), (4096, 11008), (6, 40), (258, 520), (2, 2048 + 8), (1024, 256)])
@pytest.mark.parametrize("norm,resid", [(False, False), (True, False), (False, True)])
def test_gemv(dtype, rows, cols, norm, resid):
    Wst, W = mat(rows, cols, dtype, 1)
    gst, g = mat(1, cols, dtype, 2, std=1.0)
    rng = np.random.default_rng(3)
    x = rng.standard_normal(cols, dtype=np.float32)
    r = rng.standard_normal(rows, dtype=np.float32)
    xin = O.rmsnorm(x, g[0], 1e-5).astype(np.float32) if norm else x
    want = W.astype(np.float64) @ xin.astype(np.float64) + (r if resid else 0)
    y = torch.from_numpy(r.copy()).cuda() if resid else torch.zeros(rows, device="cuda")
    P().spd_op_gemv(dtype, dev(Wst, dtype), torch.from_numpy(x).cuda(), y,
                    gain=dev(gst.reshape(-1), dtype) if norm else None, eps=1e-5, residual=y if resid else None)
    torch.cuda.synchronize()
    assert_close_scaled(y.cpu().numpy(), want, 2e-5, "gemv")   # fp32 accumulation of exact products


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("rows,cols", [(11008, 4096), (7, 24), (1025, 264)])
def test_swiglu(dtype, rows, cols):
    Gst, G = mat(rows, cols, dtype, 4, std=0.05)
    Ust, U = mat(rows, cols, dtype, 5, std=0.05)
    gst, g = mat(1, cols, dtype, 6, std=1.0)
    x = np.random.default_rng(7).standard_normal(cols, dtype=np.float32)
    xn = O.rmsnorm(x.astype(np.float64), g[0].astype(np.float64), 1e-5)
    want = O.silu(G.astype(np.float64) @ xn) * (U.astype(np.float64) @ xn)
    u = torch.zeros(rows, device="cuda")
    P().spd_op_swiglu(dtype, dev(Gst, dtype), dev(Ust, dtype), torch.from_numpy(x).cuda(), u, gain=dev(gst.reshape(-1), dtype), eps=1e-5)
    torch.cuda.synchronize()
    assert_close_scaled(u.cpu().numpy(), want, 2e-5, "swiglu")


@pytest.mark.parametrize("dtype,dh", [("bf16", 128), ("fp32", 64), ("bf16", 64), ("fp32", 128), ("fp16", 128), ("fp16", 64), ("fp16", 32)])
@pytest.mark.parametrize("heads,kv", [(4, 4), (8, 1), (8, 2)])
@pytest.mark.parametrize("n_ctx,cap", [(1, 8), (7, 300), (128, 128), (129, 300), (256, 256), (257, 600), (1044, 1100)])
def test_attention(dtype, dh, heads, kv, n_ctx, cap):
    rng = np.random.default_rng(n_ctx + heads)
    Kst, K = mat(kv * cap, dh, dtype, 11, std=1.0)
    Vst, V = mat(kv * cap, dh, dtype, 12, std=1.0)
    q = rng.standard_normal((heads, dh), dtype=np.float32)
    Kt = torch.from_numpy(K.reshape(kv, cap, dh)[:, :n_ctx].astype(np.float64)).repeat_interleave(heads // kv, 0)
    Vt = torch.from_numpy(V.reshape(kv, cap, dh)[:, :n_ctx].astype(np.float64)).repeat_interleave(heads // kv, 0)
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q.astype(np.float64))[:, None, :], Kt, Vt)[:, 0, :].numpy()
    out = torch.zeros(heads, dh, device="cuda")
    P().spd_op_attention(dtype, torch.from_numpy(q).cuda(), dev(Kst, dtype).view(kv, cap, dh), dev(Vst, dtype).view(kv, cap, dh), out, n_ctx)
    torch.cuda.synchronize()
    assert_close_scaled(out.cpu().numpy(), want, 1e-5, "attention")
    # a second call reuses zeroed counters and gives the same bits
    out2 = torch.zeros(heads, dh, device="cuda")
    P().spd_op_attention(dtype, torch.from_numpy(q).cuda(), dev(Kst, dtype).view(kv, cap, dh), dev(Vst, dtype).view(kv, cap, dh), out2, n_ctx)
    assert torch.equal(out, out2)
