"""Parity of the fp32 matrix-core kernel (fp32 inputs, d in {32, 64, 96, 128}; through the C-ABI) against the fp64
CPU oracle, element by element.

Tolerance: max |x - x_ref| / RMS(x_ref) <= 1e-5 for O and tO and |lse - lse_ref| <= 1e-5 up to 256 keys, the size
of the fp32 configuration the tolerance is stated for.  Beyond that it grows like sqrt(Lkv): l, r and the
accumulators are fp32 running sums of Lkv terms, whose rounding error grows like 2^-24 sqrt(Lkv); measured RMS
errors are 4e-7 (256 keys), 7e-7 (1000), 1.4e-6 (4096), the same in the fp32 vector kernel, with maxima over
10^5 elements 10 to 16 times the RMS.  tol(Lkv) = 1e-5 for Lkv <= 256, else 1.5e-5 sqrt(Lkv / 256).
"""
import numpy as np
import pytest
import torch

from oracle.attn_jvp_ref import attn_jvp_ref
from paper_2510_08431_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 1e-5


def tol_for(Lkv):
    return TOL if Lkv <= 256 else 1.5e-5 * (Lkv / 256) ** 0.5


def rel_err(x, ref):
    return float(np.abs(x - ref).max() / max(np.sqrt((ref ** 2).mean()), 1e-300))


def random_inputs(seed, B, H, Lq, Lkv, d, tangent_std=1.0, qk_gain=1.0):
    g = torch.Generator().manual_seed(seed)
    mk = lambda L, s: s * torch.randn(B, H, L, d, generator=g)
    return {"q": mk(Lq, qk_gain), "k": mk(Lkv, qk_gain), "v": mk(Lkv, 1.0),
            "tq": mk(Lq, tangent_std), "tk": mk(Lkv, tangent_std), "tv": mk(Lkv, tangent_std)}


def run(t, scale, kernel=binding.KERNEL_MFMA, names=("q", "k", "v", "tq", "tk", "tv"), **kw):
    args = [t[n].to(DEV) if n in names else None for n in ("q", "k", "v", "tq", "tk", "tv")]
    o, to, lse = binding.attn_jvp_fwd_ex(*args, scale, kernel=kernel, **kw)
    torch.cuda.synchronize()
    return o, to, lse


def to_np(res):
    return tuple(None if x is None else x.cpu().double().numpy() for x in res)


def compare(got, ref, label, Lkv, rows=None, extra_tol=0.0):
    tol = tol_for(Lkv) + extra_tol
    o, to, lse = got
    if rows is not None:
        o, to, lse = o[:, :, rows], to[:, :, rows], lse[:, :, rows]
    e_o, e_to, e_lse = rel_err(o, ref[0]), rel_err(to, ref[1]), float(np.abs(lse - ref[2]).max())
    print(f"[{label}] err O={e_o:.3e} tO={e_to:.3e} lse={e_lse:.3e}", flush=True)
    assert np.isfinite(o).all() and np.isfinite(to).all() and np.isfinite(lse).all(), label
    assert e_o <= tol, f"{label}: O error {e_o}"
    assert e_to <= tol, f"{label}: tO error {e_to}"
    assert e_lse <= tol, f"{label}: lse error {e_lse}"


def sc(d):
    """1/sqrt(d) as the float32 the C-ABI takes: the oracle must see the same number."""
    return float(np.float32(d ** -0.5))


def oracle(t, scale, **kw):
    return attn_jvp_ref(t["q"], t["k"], t["v"], t["tq"], t["tk"], t["tv"], scale, **kw)


@pytest.mark.parametrize("d", [32, 64, 96, 128])
@pytest.mark.parametrize("Lq,Lkv", [(1, 1), (70, 45), (64, 32), (130, 257), (129, 31), (300, 1000)])
def test_shapes(d, Lq, Lkv):
    """Several query tiles with a ragged last one, several key blocks with a ragged tail, single rows."""
    t = random_inputs(900 + d + Lq, 2, 2, Lq, Lkv, d)
    compare(to_np(run(t, sc(d))), oracle(t, sc(d)), f"mfma-f32 d={d} Lq={Lq} Lkv={Lkv}", Lkv)


def test_every_key_length_up_to_four_blocks():
    """Every position of the ragged key tail inside a block, first and later blocks."""
    d, Lq = 64, 40
    base = random_inputs(31, 1, 1, Lq, 130, d)
    for Lkv in range(1, 131):
        t = {n: (x if n in ("q", "tq") else x[:, :, :Lkv].contiguous()) for n, x in base.items()}
        got, ref = to_np(run(t, 0.125)), oracle(t, 0.125)
        for g, r, name in zip(got, ref, ("o", "to", "lse")):
            err = np.abs(g - r).max() / max(np.sqrt((r ** 2).mean()), 1e-30) if name != "lse" else np.abs(g - r).max()
            if name == "to" and Lkv == 1:       # one key: tO = tV_0 exactly, no scale to divide by if it is tiny
                err = np.abs(g - r).max() / max(np.sqrt((r ** 2).mean()), 1e-3)
            assert np.isfinite(g).all() and err <= TOL, f"Lkv={Lkv} {name}: {err}"
    print("[mfma-f32 key lengths 1..130] ok", flush=True)


def test_query_lengths_around_tile_edges():
    d, Lkv = 128, 100
    for Lq in (31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257):
        t = random_inputs(40 + Lq, 1, 2, Lq, Lkv, d)
        compare(to_np(run(t, sc(d))), oracle(t, sc(d)), f"mfma-f32 Lq={Lq}", Lkv)


@pytest.mark.parametrize("gain", [3.0, 6.0])
def test_peaked_softmax_takes_the_rescale_path(gain):
    """Scores with a standard deviation of 9 and 36 nats: single keys dominate rows (the cancelling terms of tO), and
    at 36 nats a block's maximum often exceeds the row reference by more than its 32 nats of slack, so that the
    accumulators are rescaled again and again.
    An fp32 score of size |S| carries an absolute error of a few 2^-24 |S| (its 128-term fp32 dot product), which the
    exponential turns into a relative error of the weights; with one key dominating a row nothing averages it out.
    Measured on these inputs: 6 to 20 times 2^-24 max|S| for O, tO and lse (3 to 6 times in the fp32 vector kernel,
    whose dot products are summed in four shorter chains).  Allowed here: 40 times."""
    d = 128
    t = random_inputs(77, 1, 2, 200, 1500, d, qk_gain=gain)
    s_max = float((t["q"].double() @ t["k"].double().transpose(-1, -2)).abs().max()) * sc(d)
    compare(to_np(run(t, sc(d))), oracle(t, sc(d)), f"mfma-f32 peaked gain={gain} max|S|={s_max:.0f}", 1500,
            extra_tol=40 * 2.0 ** -24 * s_max)


@pytest.mark.parametrize("step", [0.05, 0.25])
def test_increasing_scores(step):
    """Keys ordered so that every query's scores grow along the sequence, by 2 * step nats per key.  The kernel's
    row reference trails the row maximum by up to 32 nats: at 0.1 nat per key the weights climb to e^32 before the
    first move of the reference near the end; at 0.5 nat per key the reference moves, and the accumulators are
    rescaled, every other block (the extra tolerance as in the peaked case)."""
    d, Lq, Lkv = 64, 64, 320
    g = torch.Generator().manual_seed(5)
    u = torch.randn(d, generator=g)
    u /= u.norm()
    t = random_inputs(6, 1, 1, Lq, Lkv, d)
    t["q"] = 0.3 * t["q"] + 2.0 * u                                   # every query points along u
    t["k"] = 0.3 * t["k"] + torch.arange(Lkv).view(1, 1, Lkv, 1) * step * u   # keys grow along u
    s_max = float((t["q"].double() @ t["k"].double().transpose(-1, -2)).abs().max())
    compare(to_np(run(t, 1.0)), oracle(t, 1.0), f"mfma-f32 increasing scores max|S|={s_max:.0f}", Lkv,
            extra_tol=40 * 2.0 ** -24 * s_max)


@pytest.mark.parametrize("scale", [0.0, float(np.float32(-0.2))])
def test_non_positive_scale(scale):
    t = random_inputs(61, 1, 2, 150, 77, 64)
    compare(to_np(run(t, scale)), oracle(t, scale), f"mfma-f32 scale={scale}", 77)


def test_auto_takes_this_kernel_for_fp32_inputs():
    t = random_inputs(8, 1, 2, 256, 256, 64)
    auto, mfma, vec = (to_np(run(t, 0.125, kernel=k)) for k in (binding.KERNEL_AUTO, binding.KERNEL_MFMA, binding.KERNEL_FP32))
    for a, b in zip(auto, mfma):
        np.testing.assert_array_equal(a, b)
    assert any((a != b).any() for a, b in zip(auto, vec)), "AUTO gave the vector kernel's bits"
    # d = 256 is not built for the matrix cores: AUTO falls back to the vector kernel, an explicit request fails
    t = random_inputs(9, 1, 1, 40, 50, 256)
    compare(to_np(run(t, 1 / 16, kernel=binding.KERNEL_AUTO)), oracle(t, 1 / 16), "auto fp32 d=256", 50)
    with pytest.raises(binding.AttnJvpError):
        run(t, 1 / 16, kernel=binding.KERNEL_MFMA)


@pytest.mark.parametrize("d", [64, 128])
def test_null_kv_tangents_equal_explicit_zeros(d):
    """tk = tv = NULL skips two of the six products; the skipped products add exact zeros, so the bits agree."""
    t = random_inputs(70 + d, 1, 2, 200, 333, d)
    t["tk"].zero_(); t["tv"].zero_()
    zeros = to_np(run(t, sc(d)))
    null = to_np(run(t, sc(d), names=("q", "k", "v", "tq")))
    for a, b, name in zip(null, zeros, ("o", "to", "lse")):
        np.testing.assert_array_equal(a, b, err_msg=f"{name} differs between NULL and zero key/value tangents")
    compare(null, oracle(t, sc(d)), f"mfma-f32 tk=tv=NULL d={d}", 333)


@pytest.mark.parametrize("d", [32, 128])
def test_no_tangents_gives_the_same_o_and_lse(d):
    t = random_inputs(80 + d, 1, 2, 130, 500, d)
    full = run(t, sc(d))
    o, to, lse = run(t, sc(d), names=("q", "k", "v"))
    assert to is None
    assert torch.equal(o, full[0]) and torch.equal(lse, full[2])


@pytest.mark.parametrize("case", ["all", "null-kv", "no-tangents"])
def test_blhd_layout_gives_the_same_bits(case):
    d = 96
    names = {"all": ("q", "k", "v", "tq", "tk", "tv"), "null-kv": ("q", "k", "v", "tq"), "no-tangents": ("q", "k", "v")}[case]
    t = random_inputs(90, 2, 3, 150, 210, d)
    ref = run(t, 0.1, names=names)
    tt = {n: x.transpose(1, 2).contiguous() for n, x in t.items()}        # [B, L, H, d]
    got = run(tt, 0.1, names=names, layout=binding.LAYOUT_BLHD)
    assert torch.equal(got[0].transpose(1, 2), ref[0]) and torch.equal(got[2], ref[2])
    if case != "no-tangents":
        assert torch.equal(got[1].transpose(1, 2), ref[1])


def test_many_heads_side_stream_and_preallocated_outputs():
    t = random_inputs(12, 3, 24, 140, 96, 64)          # 72 heads x 2 tiles: not a multiple of 8 workgroups... and
    t2 = random_inputs(13, 2, 8, 256, 64, 64)          # 16 heads x 2 tiles = 32: the XCD-contiguous tile order
    side = torch.cuda.Stream()
    for tt in (t, t2):
        dev = {n: x.to(DEV) for n, x in tt.items()}
        out = tuple(torch.full_like(dev["q"], float("nan")) for _ in range(2)) + (
            torch.full(dev["q"].shape[:3], float("nan"), device=DEV),)
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            res = binding.attn_jvp_fwd_ex(dev["q"], dev["k"], dev["v"], dev["tq"], dev["tk"], dev["tv"], 0.125,
                                          out=out, stream=side, kernel=binding.KERNEL_MFMA)
        side.synchronize()
        assert all(a.data_ptr() == b.data_ptr() for a, b in zip(res, out))
        compare(to_np(res), oracle(tt, 0.125), f"mfma-f32 heads={tt['q'].shape[0] * tt['q'].shape[1]} side stream", 96)


def test_image_dit_shape_in_fp32_sampled_rows():
    """One launch at the image-DiT configuration's size (B2 H16 L4096 d128) with fp32 inputs; the oracle on a seeded
    sample of query rows of four heads, tile edges included."""
    B, H, L, d = 2, 16, 4096, 128
    t = random_inputs(2024, B, H, L, L, d, tangent_std=0.5)
    got = to_np(run(t, sc(d)))
    g = np.random.default_rng(3)
    rows = np.unique(np.concatenate([[0, 127, 128, L - 129, L - 128, L - 1], g.integers(0, L, 58)]))
    for b, h in ((0, 0), (0, 7), (1, 3), (1, 15)):
        sl = {n: x[b:b + 1, h:h + 1] for n, x in t.items()}
        ref = oracle(sl, sc(d), rows=rows)
        compare(tuple(x[b:b + 1, h:h + 1] for x in got), ref, f"mfma-f32 image-DiT shape b{b} h{h}", L, rows=rows)


def test_video_length_key_sequence():
    """Lkv = 32760 (the video workloads' length: 1023 full key blocks and a ragged one of 24), two heads, two query
    tiles, every row compared."""
    B, H, Lq, Lkv, d = 1, 2, 200, 32760, 128
    t = random_inputs(3276, B, H, Lq, Lkv, d, tangent_std=0.5)
    compare(to_np(run(t, sc(d))), oracle(t, sc(d)), "mfma-f32 Lkv=32760", Lkv)
