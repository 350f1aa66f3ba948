"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and turns invalid arguments into error codes before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "attn_jvp.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2510_08431_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return binding.load_library()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(attn_jvp_\w+)\s*\(", text)))


def test_header_symbols_exported(lib):
    names = declared_functions()
    assert {"attn_jvp_fwd", "attn_jvp_fwd_ex", "attn_jvp_fwd_static", "attn_jvp_static_scratch_bytes", "attn_jvp_rmsnorm_fwd",
            "attn_jvp_mfma_rate_probe", "attn_jvp_strerror", "attn_jvp_version", "attn_jvp_workspace_bytes"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in the header but not exported"


def test_opts_struct_layout_matches_header(tmp_path):
    """The ctypes mirror of attn_jvp_opts has the size and field offsets a C compiler gives the header's struct."""
    import subprocess
    from paper_2510_08431_amd.binding import AttnJvpOpts
    fields = [n for n, _ in AttnJvpOpts._fields_]
    src = tmp_path / "layout.c"
    prints = "\n".join(f'    printf("{n} %zu\\n", offsetof(attn_jvp_opts, {n}));' for n in fields)
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "attn_jvp.h"\nint main(void) {\n'
                   '    printf("sizeof %zu\\n", sizeof(attn_jvp_opts));\n' + prints + "\n    return 0;\n}\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)],
                   check=True)
    got = dict(line.split() for line in subprocess.run([str(exe)], check=True, capture_output=True,
                                                       text=True).stdout.splitlines())
    assert int(got.pop("sizeof")) == ctypes.sizeof(AttnJvpOpts)
    assert set(got) == set(fields)
    for n in fields:
        assert int(got[n]) == getattr(AttnJvpOpts, n).offset, n


def test_workspace_bytes(lib):
    lib.attn_jvp_workspace_bytes.restype = ctypes.c_size_t
    n = lib.attn_jvp_workspace_bytes(1, 12, 32760, 32760, 128)
    # two fp16 copies (whole 32-key blocks: 32768 keys) + 12 x 32 B of statistics (rounded up to 256) + one int per 128-row query tile + 512 B of
    # lock-step tickets + 32 B of partial statistics per head and 1024-row block of the longer sequence
    assert n == 2 * 12 * 32768 * 128 * 2 + 512 + 12 * 256 * 4 + 512 + 12 * 32 * 32
    for d, width in ((32, 64), (96, 128)):                             # padded to the next width the MFMA kernel is built for
        pad = (2 * 2 * 256 * width * 2) + 4 * (2 * 256 * width * 2)   # zero-padded q, tq and k, v, tk, tv
        f16 = 2 * 2 * 256 * width * 2 + 256 + 256 + 512 + 256         # fp16 copies + statistics + 4 tile flags + tickets + partials
        assert lib.attn_jvp_workspace_bytes(1, 2, 256, 256, d) == pad + f16
    assert lib.attn_jvp_workspace_bytes(1, 2, 256, 256, 64) == 2 * 2 * 256 * 64 * 2 + 256 + 256 + 512 + 256   # built natively: no padded copies
    assert lib.attn_jvp_workspace_bytes(1, 2, 256, 256, 48) == 0      # the MFMA kernel has no use for d = 48
    assert lib.attn_jvp_workspace_bytes(0, 2, 256, 256, 128) == 0


def test_version_and_strerror(lib):
    assert lib.attn_jvp_version() >= 100
    msgs = [lib.attn_jvp_strerror(c).decode() for c in range(0, 8)]
    assert msgs[0] == "ok" and len(set(msgs)) == 8 and all(msgs)


def _call(lib, ptrs=None, dims=(1, 1, 8, 8, 128), scale=0.1, opts=None, static=False):
    p = [0x1000 * (i + 1) for i in range(9)] if ptrs is None else ptrs
    args = [ctypes.c_void_p(x) for x in p] + list(dims) + [ctypes.c_float(scale)]
    if static:
        return lib.attn_jvp_fwd_static(*args, ctypes.byref(opts) if opts is not None else None)
    if opts is None:
        return lib.attn_jvp_fwd(*args)
    return lib.attn_jvp_fwd_ex(*args, ctypes.byref(opts))


def test_static_entry_point_rejects_on_the_host(lib):
    """attn_jvp_fwd_static: the limit of its scratch array, a caller workspace and the common argument checks are
    all refused before anything touches a device (fake addresses, no GPU needed)."""
    from paper_2510_08431_amd.binding import AttnJvpOpts
    limit = lib.attn_jvp_static_scratch_bytes()
    assert limit == 200 << 20
    lib.attn_jvp_workspace_bytes.restype = ctypes.c_size_t
    assert lib.attn_jvp_workspace_bytes(1, 12, 32760, 32760, 128) <= limit      # the headline shape fits
    assert lib.attn_jvp_workspace_bytes(1, 40, 75600, 75600, 128) > limit
    assert _call(lib, dims=(1, 40, 75600, 75600, 128), static=True) == 6         # TOO_LARGE
    assert _call(lib, dims=(1, 13, 32760, 32760, 128), static=True) == 6
    o = AttnJvpOpts(); o.workspace = 0x10000; o.workspace_bytes = 1 << 20        # brings its own scratch: refused
    assert _call(lib, opts=o, static=True) == 3
    good = [0x1000 * (i + 1) for i in range(9)]
    p = list(good); p[0] = 0
    assert _call(lib, p, static=True) == 1
    p = list(good); p[2] += 8
    assert _call(lib, p, static=True) == 4
    assert _call(lib, dims=(1, 1, 0, 8, 128), static=True) == 2
    assert _call(lib, dims=(1, 1, 8, 8, 48), static=True) == 3


def test_set_up_failure_launches_nothing(lib):
    """With no usable device every precondition check passes and the first set-up call (the device query, made
    before any enqueue) fails: the call must come back with LAUNCH_FAILED, not crash, having launched nothing.
    Only meaningful where no GPU is visible; skipped on a GPU machine (there the pointers would be dereferenced)."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible: fake pointers would reach a kernel")
    from paper_2510_08431_amd.binding import AttnJvpOpts
    assert _call(lib) == 5
    o = AttnJvpOpts(); o.workspace = 0x10000; o.workspace_bytes = 1 << 30
    assert _call(lib, dims=(1, 1, 256, 4096, 128), opts=o) == 5                  # fp16 value path: eight kernels, none enqueued
    assert _call(lib, dims=(1, 1, 256, 4096, 128), static=True) == 5


def test_argument_validation_returns_codes_without_launching(lib):
    """Fake (never dereferenced) addresses: every call here must be rejected on the host."""
    from paper_2510_08431_amd.binding import AttnJvpOpts
    good = [0x1000 * (i + 1) for i in range(9)]
    for i in range(9):
        p = list(good); p[i] = 0
        assert _call(lib, p) == 1                         # NULL_PTR
    p = list(good); p[3] = 0; p[4] = 0                    # tq and tk absent but tv given
    assert _call(lib, p) == 1
    p = list(good); p[3] = p[4] = p[5] = p[7] = 0         # no tangents and no `to`: legal, the next check decides
    assert _call(lib, p, dims=(1, 1, 8, 8, 48)) == 3
    p = list(good); p[4] = 0; p[5] = 0                    # tk = tv = NULL is legal: the next check decides
    assert _call(lib, p, dims=(1, 1, 8, 8, 48)) == 3      # ... here the unsupported head dim
    for i in range(5):
        for bad in (0, -3):
            dims = [1, 1, 8, 8, 128]; dims[i] = bad
            assert _call(lib, dims=dims) == 2             # BAD_SHAPE
    assert _call(lib, scale=float("nan")) == 2
    assert _call(lib, scale=float("inf")) == 2
    assert _call(lib, dims=(1, 1, 8, 8, 48)) == 3         # UNSUPPORTED head dim
    for i in range(9):
        p = list(good); p[i] += 8
        assert _call(lib, p) == 4                         # MISALIGNED
    o = AttnJvpOpts(); o.in_dtype = 7
    assert _call(lib, opts=o) == 3
    o = AttnJvpOpts(); o.out_dtype = 5
    assert _call(lib, opts=o) == 3
    o = AttnJvpOpts(); o.kernel = 9
    assert _call(lib, opts=o) == 3
    o = AttnJvpOpts(); o.reserved = 1
    assert _call(lib, opts=o) == 3
    o = AttnJvpOpts(); o.layout = 2                        # unknown layout
    assert _call(lib, opts=o) == 3
    o = AttnJvpOpts(); o.flags = 32                        # unknown flag bit
    assert _call(lib, opts=o) == 3
    o = AttnJvpOpts(); o.workspace = 0x10010; o.workspace_bytes = 1 << 20   # workspace not 256-byte aligned
    assert _call(lib, opts=o) == 4
    o = AttnJvpOpts(); o.kernel = 2; o.in_dtype = 1        # MFMA kernels with fp32 inputs: d in {32, 64, 96, 128} only
    assert _call(lib, dims=(1, 1, 8, 8, 256), opts=o) == 3
    o = AttnJvpOpts(); o.kernel = 2                        # MFMA kernel with d = 96 and no workspace for the padded copies
    assert _call(lib, dims=(1, 1, 8, 8, 96), opts=o) == 3
    for bad_scale in (0.0, -0.125):                        # MFMA kernel needs scale > 0 (AUTO then takes the fp32 kernel)
        o = AttnJvpOpts(); o.kernel = 2
        assert _call(lib, scale=bad_scale, opts=o) == 3


def test_rmsnorm_argument_validation_returns_codes_without_launching(lib):
    """Fake (never dereferenced) addresses: every call here must be rejected on the host."""
    vp = ctypes.c_void_p
    def call(ptrs=None, rows=8, d=128, eps=1e-6, dtype=0):
        p = [0x1000 * (i + 1) for i in range(5)] if ptrs is None else ptrs
        return lib.attn_jvp_rmsnorm_fwd(*[vp(a) for a in p], rows, d, eps, dtype, None)
    good = [0x1000 * (i + 1) for i in range(5)]
    for i in range(5):
        p = list(good); p[i] = 0
        assert call(p) == 1
        p = list(good); p[i] += 4
        assert call(p) == 4
    assert call(rows=0) == 2 and call(d=0) == 2 and call(eps=-1.0) == 2 and call(eps=float("nan")) == 2
    assert call(d=96) == 3 and call(dtype=5) == 3


def test_rate_probe_argument_validation_returns_codes_without_launching(lib):
    """The measurement aid checks its arguments on the host like the other entry points (no GPU needed)."""
    import ctypes
    fn = lib.attn_jvp_mfma_rate_probe
    ok = 0x10000
    assert fn(None, ok, 0, 10, None, None, None) == 1
    assert fn(ok, None, 0, 10, None, None, None) == 1
    assert fn(ok, ok, 0, 0, None, None, None) == 2
    assert fn(ok, ok, 1, 2_000_001, None, None, None) == 2
    assert fn(ok + 4, ok, 0, 10, None, None, None) == 4
    assert fn(ok, ok + 8, 0, 10, None, None, None) == 4


def test_binding_rejects_cpu_tensors_and_bad_shapes():
    import torch
    from paper_2510_08431_amd import binding
    q = torch.zeros(1, 1, 4, 128, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        binding.attn_jvp_fwd(q, q, q, q, q, q, 0.1)       # CPU tensors: no CPU path exists
    with pytest.raises(ValueError):
        binding._check_inputs(q, q, q, q, q, q[:, :, :2])
    with pytest.raises(ValueError):
        binding._check_inputs(q, q, q.float(), q, q, q)


def test_workload_shapes_match_configs():
    from paper_2510_08431_amd.workloads import CONFIGS, make_head, sample_rows
    assert CONFIGS[3].Lq == 21 * 30 * 52 == 32760 and CONFIGS[5].Lq == 21 * 45 * 80 == 75600
    assert abs(CONFIGS[3].flops - 1.978e13) / 1.978e13 < 1e-3
    h = make_head(CONFIGS[1], 0, 1)
    assert h["q"].shape == (256, 64) and h["q"].dtype.is_floating_point
    h2 = make_head(CONFIGS[1], 0, 1)
    assert all((h[k] == h2[k]).all() for k in h)          # seeded: reproducible
    rows = sample_rows(CONFIGS[3], 64)
    assert rows.min() == 0 and rows.max() == 32759 and len(set(rows.tolist())) == len(rows)


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; any other --gpus value ends with a message and a non-zero status before anything
    touches a GPU (so this runs anywhere)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_product_path_does_not_reach_the_oracle():
    """Nothing under the package, and nothing in bench.py outside its CPU-baseline leg, imports the test oracle."""
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg = os.path.join(root, "paper_2510_08431_amd")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            assert not re.search(r"^\s*(from|import)\s+oracle\b", open(os.path.join(pkg, name)).read(), re.M), name
    bench = open(os.path.join(root, "bench.py")).read()
    imports = [m.start() for m in re.finditer(r"^\s*(from|import)\s+oracle\b", bench, re.M)]
    assert len(imports) == 2           # the attention oracle and the RMSNorm oracle, each inside `if not args.no_cpu_baseline`
    for pos in imports:
        assert "no_cpu_baseline" in bench[max(0, pos - 600):pos]
