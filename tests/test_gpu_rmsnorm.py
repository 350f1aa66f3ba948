"""GPU parity of the RMSNorm + JVP kernel (through the C ABI) against the fp64 oracle, element by element."""
import numpy as np
import pytest
import torch

from oracle.rmsnorm_jvp_ref import rmsnorm_jvp_ref
from paper_2510_08431_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make(seed, shape, dtype, x_std=1.0):
    g = torch.Generator().manual_seed(seed)
    x = (x_std * torch.randn(*shape, generator=g)).to(dtype)
    tx = (0.5 * torch.randn(*shape, generator=g)).to(dtype)
    w = 1.0 + 0.2 * torch.randn(shape[-1], generator=g)
    return x, tx, w


def bound(x, tx, w, eps, dtype):
    """Element-wise error bound.  bf16: the layer rounds the normalised value to bf16, the product with the gain
    is rounded again on storing: twice the unit round-off 2^-8 of the value.  Both dtypes: fp32 evaluation of the two row sums, r and
    the difference tx r - x r^3 mean(x tx), whose terms may cancel: a few fp32 ulps of the terms."""
    x64, tx64, w64 = x.double().numpy(), tx.double().numpy(), w.double().numpy()
    y, ty = rmsnorm_jvp_ref(x64, tx64, w64, eps)
    r = 1.0 / np.sqrt((x64 ** 2).mean(-1, keepdims=True) + eps)
    # (the row sum of x tx cancels too: its fp32 error scales with mean |x tx|, not with |mean x tx|)
    terms = (np.abs(tx64) * r + np.abs(x64) * r ** 3 * np.abs(x64 * tx64).mean(-1, keepdims=True)) * np.abs(w64)
    rel = 2.0 ** -7 * 1.01 if dtype == torch.bfloat16 else 0.0
    return y, ty, rel * np.abs(y) + 2e-6 * np.abs(y) + 1e-30, rel * np.abs(ty) + 3e-6 * terms + 1e-30


def check(x, tx, w, eps, label, inplace=False):
    dx, dtx, dw = x.to(DEV), tx.to(DEV), w.to(DEV)
    if inplace:
        y, ty = binding.attn_jvp_rmsnorm_fwd(dx, dtx, dw, eps, out=(dx, dtx))
    else:
        y, ty = binding.attn_jvp_rmsnorm_fwd(dx, dtx, dw, eps)
    torch.cuda.synchronize()
    y_ref, ty_ref, by, bty = bound(x, tx, w, eps, x.dtype)
    ey = np.abs(y.cpu().double().numpy() - y_ref)
    ety = np.abs(ty.cpu().double().numpy() - ty_ref)
    print(f"[{label}] worst err/bound y={np.max(ey / by):.3f} ty={np.max(ety / bty):.3f}", flush=True)
    assert np.isfinite(ey).all() and np.isfinite(ety).all()
    assert (ey <= by).all(), f"{label}: y off by up to {np.max(ey / by):.2f} x the bound"
    assert (ety <= bty).all(), f"{label}: ty off by up to {np.max(ety / bty):.2f} x the bound"


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("rows", [1, 63, 64, 65, 1000])
def test_rmsnorm_jvp_shapes(dtype, d, rows):
    x, tx, w = make(17 * d + rows, (rows, d), dtype)
    check(x, tx, w, 1e-6, f"rmsnorm {dtype} rows={rows} d={d}")


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_rmsnorm_jvp_qk_norm_of_the_video_workload(dtype):
    """The QK-normalisation in front of the video self-attention workload: every (batch, head, token) row of q."""
    x, tx, w = make(5, (1, 12, 32760, 128), dtype)
    check(x, tx, w, 1e-6, f"rmsnorm {dtype} [1,12,32760,128]")


def test_rmsnorm_jvp_in_place_magnitudes_and_zero_rows():
    x, tx, w = make(9, (300, 128), torch.bfloat16, x_std=300.0)
    check(x, tx, w, 1e-5, "rmsnorm in place, |x| ~ 300", inplace=True)
    x, tx, w = make(10, (300, 128), torch.bfloat16, x_std=1e-3)
    check(x, tx, w, 1e-6, "rmsnorm |x| ~ 1e-3 (eps matters)")
    x, tx, w = make(11, (130, 128), torch.float32)
    x[::7] = 0.0
    check(x, tx, w, 1e-6, "rmsnorm zero rows")       # y = 0, ty = tx w / sqrt(eps)
    x, tx, w = make(12, (64, 128), torch.float32)
    check(x, x.clone(), w, 0.0, "rmsnorm tx = x, eps = 0 (ty ~ 0 by scale invariance)")


def test_rmsnorm_jvp_runs_on_the_given_stream_and_rejects_bad_arguments():
    x, tx, w = make(13, (256, 128), torch.bfloat16)
    dx, dtx, dw = x.to(DEV), tx.to(DEV), w.to(DEV)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        y, ty = binding.attn_jvp_rmsnorm_fwd(dx, dtx, dw, 1e-6)
    s.synchronize()
    y2, ty2 = binding.attn_jvp_rmsnorm_fwd(dx, dtx, dw, 1e-6)
    torch.cuda.synchronize()
    assert torch.equal(y, y2) and torch.equal(ty, ty2)
    with pytest.raises(binding.AttnJvpError):
        binding.attn_jvp_rmsnorm_fwd(dx[:, :96].contiguous(), dtx[:, :96].contiguous(), dw[:96].contiguous(), 1e-6)
    with pytest.raises(ValueError):
        binding.attn_jvp_rmsnorm_fwd(dx, dtx, dw.to(torch.bfloat16), 1e-6)
