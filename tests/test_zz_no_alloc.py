"""attn_jvp_fwd_static (the entry point that allocates nothing: its scratch is a static device array of the library)
against attn_jvp_fwd_ex with a caller-lent workspace, through the C ABI.

The two run the same kernels on the same inputs, so the outputs must agree bit for bit (which is inside the
parity tolerances by any measure); the first result is also checked against the fp64 oracle.  Two calls in a row,
the second on a smaller input: the array keeps the first call's contents, and the second call must not be
disturbed by them.  The file name makes pytest collect it last; it passes alone in a fresh process as well.
"""
import ctypes

import numpy as np
import pytest
import torch

from oracle.attn_jvp_ref import attn_jvp_ref
from paper_2510_08431_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(seed, B, H, Lq, Lkv, d, qk_gain=1.0):
    g = torch.Generator().manual_seed(seed)
    mk = lambda L, s: (s * torch.randn(B, H, L, d, generator=g)).to(torch.bfloat16)
    return {"q": mk(Lq, qk_gain), "k": mk(Lkv, qk_gain), "v": mk(Lkv, 1.0),
            "tq": mk(Lq, 0.5), "tk": mk(Lkv, 0.5), "tv": mk(Lkv, 0.5)}


def _call_c(entry, dev, out, dims, scale, opts):
    """Straight through ctypes: pointers, sizes and the options struct, nothing else."""
    vp = ctypes.c_void_p
    args = [vp(dev[n].data_ptr()) for n in ("q", "k", "v", "tq", "tk", "tv")] + [vp(x.data_ptr()) for x in out]
    rc = entry(*args, *dims, ctypes.c_float(scale), ctypes.byref(opts))
    assert rc == 0, binding.attn_jvp_strerror(rc)


def _run_both(t, flags=0):
    lib = binding.load_library()
    B, H, Lq, d = t["q"].shape
    Lkv = t["k"].shape[2]
    scale = d ** -0.5
    dev = {n: x.to(DEV) for n, x in t.items()}
    mk_out = lambda: (torch.full((B, H, Lq, d), float("nan"), device=DEV), torch.full((B, H, Lq, d), float("nan"), device=DEV),
                      torch.full((B, H, Lq), float("nan"), device=DEV))
    out_static, out_ws = mk_out(), mk_out()
    need = binding.attn_jvp_workspace_bytes(B, H, Lq, Lkv, d)
    assert 0 < need <= binding.attn_jvp_static_scratch_bytes()
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    stream = torch.cuda.current_stream(DEV).cuda_stream
    torch.cuda.synchronize()

    opts = binding.AttnJvpOpts()
    opts.stream = stream
    opts.flags = flags
    before = torch.cuda.memory_allocated(DEV)
    _call_c(lib.attn_jvp_fwd_static, dev, out_static, (B, H, Lq, Lkv, d), scale, opts)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated(DEV) == before          # torch's allocator was not involved

    opts_ws = binding.AttnJvpOpts()
    opts_ws.stream = stream
    opts_ws.flags = flags
    opts_ws.workspace = ws.data_ptr()
    opts_ws.workspace_bytes = need
    _call_c(lib.attn_jvp_fwd_ex, dev, out_ws, (B, H, Lq, Lkv, d), scale, opts_ws)
    torch.cuda.synchronize()
    for a, b, name in zip(out_static, out_ws, ("o", "to", "lse")):
        assert torch.isfinite(a).all(), name
        assert torch.equal(a, b), f"{name}: static scratch and lent workspace disagree"
    return out_static


def test_static_scratch_entry_point_twice_second_call_smaller():
    # first call: 2 heads x 4100 keys (ragged tail) on the fp16 value path, which uses the scratch for the fp16
    # copies of V and tV, the per-head statistics, the tile flags and the tickets; head 1 has peaked scores, so
    # all three launches of that path do work and the flags matter
    t1 = _inputs(901, 1, 2, 300, 4100, 128)
    t1["q"][:, 1] *= 8 ** 0.5
    t1["k"][:, 1] *= 8 ** 0.5
    print("[static scratch] call 1: B1 H2 Lq300 Lkv4100 d128", flush=True)
    o, to, lse = _run_both(t1)
    ref = attn_jvp_ref(t1["q"], t1["k"], t1["v"], t1["tq"], t1["tk"], t1["tv"], 128 ** -0.5)
    rel = lambda x, r: float(np.abs(x.cpu().double().numpy() - r).max() / np.sqrt((r ** 2).mean()))
    e_o, e_to, e_lse = rel(o, ref[0]), rel(to, ref[1]), float(np.abs(lse.cpu().double().numpy() - ref[2]).max())
    print(f"[static scratch] call 1 against the oracle: O {e_o:.3e} tO {e_to:.3e} lse {e_lse:.3e}", flush=True)
    assert e_o <= 1e-2 and e_to <= 2e-2 and e_lse <= 1e-3
    # second call, smaller in every dimension: the array still holds call 1's copies, flags and statistics
    t2 = _inputs(902, 1, 1, 130, 2100, 128)
    print("[static scratch] call 2: B1 H1 Lq130 Lkv2100 d128", flush=True)
    o2, to2, lse2 = _run_both(t2)
    ref2 = attn_jvp_ref(t2["q"], t2["k"], t2["v"], t2["tq"], t2["tk"], t2["tv"], 128 ** -0.5)
    e_o, e_to, e_lse = rel(o2, ref2[0]), rel(to2, ref2[1]), float(np.abs(lse2.cpu().double().numpy() - ref2[2]).max())
    print(f"[static scratch] call 2 against the oracle: O {e_o:.3e} tO {e_to:.3e} lse {e_lse:.3e}", flush=True)
    assert e_o <= 1e-2 and e_to <= 2e-2 and e_lse <= 1e-3
    # third: a padded head dimension (d = 64: the scratch also holds the zero-padded copies of the six inputs)
    t3 = _inputs(903, 1, 2, 200, 2300, 64)
    print("[static scratch] call 3: B1 H2 Lq200 Lkv2300 d64", flush=True)
    _run_both(t3)


def test_static_scratch_rejects_what_does_not_fit():
    lib = binding.load_library()
    B, H, L, d = 1, 13, 32760, 128          # one head more than fits
    assert binding.attn_jvp_workspace_bytes(B, H, L, L, d) > binding.attn_jvp_static_scratch_bytes()
    x = torch.zeros(16, device=DEV)         # never dereferenced: the size check comes first
    vp = ctypes.c_void_p
    rc = lib.attn_jvp_fwd_static(*[vp(x.data_ptr())] * 9, B, H, L, L, d, ctypes.c_float(0.1), None)
    assert rc == 6 and "static" in binding.attn_jvp_strerror(rc)


def test_static_entry_point_captured_in_a_hip_graph():
    """What the entry point is for: a caller under HIP graph capture cannot allocate.  The call is captured (kernel
    launches only: no allocation, no memset node, no attribute or symbol look-up, all of which the warm-up call
    before the capture has done) and replayed several times on changing inputs, with eager work and synchronisations
    between the replays; every replay must equal an eager call with a lent workspace bit for bit."""
    lib = binding.load_library()
    B, H, Lq, Lkv, d = 1, 2, 300, 2100, 128            # fp16 value path (2100 keys), ragged tiles and key blocks
    scale = d ** -0.5
    sets = [_inputs(31, B, H, Lq, Lkv, d), _inputs(32, B, H, Lq, Lkv, d, qk_gain=2.0)]
    dev = {n: x.to(DEV) for n, x in sets[0].items()}   # the graph's fixed input buffers
    out = (torch.empty(B, H, Lq, d, device=DEV), torch.empty(B, H, Lq, d, device=DEV), torch.empty(B, H, Lq, device=DEV))
    side = torch.cuda.Stream(DEV)
    opts = binding.AttnJvpOpts()
    opts.stream = side.cuda_stream
    with torch.cuda.stream(side):
        _call_c(lib.attn_jvp_fwd_static, dev, out, (B, H, Lq, Lkv, d), scale, opts)      # warm-up, eager
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        _call_c(lib.attn_jvp_fwd_static, dev, out, (B, H, Lq, Lkv, d), scale, opts)
    torch.cuda.synchronize()
    ws = torch.empty(binding.attn_jvp_workspace_bytes(B, H, Lq, Lkv, d), dtype=torch.uint8, device=DEV)
    for rep in range(4):
        t = sets[rep % 2]
        for n in dev:
            dev[n].copy_(t[n])                         # eager work between the replays
        for x in out:
            x.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [x.clone() for x in out]
        eager = binding.attn_jvp_fwd_ex(dev["q"], dev["k"], dev["v"], dev["tq"], dev["tk"], dev["tv"], scale, workspace=ws)
        torch.cuda.synchronize()
        for a, b, name in zip(got, eager, ("o", "to", "lse")):
            assert torch.equal(a, b), f"replay {rep}: {name} differs from the eager call"
