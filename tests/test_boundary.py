"""Host-side checks of the C-ABI boundary that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments with status codes before any launch."""
import ctypes as C
import os
import re

import pytest

import paper_2501_10714_amd as moe
from paper_2501_10714_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(moe.lib_path()):
        from paper_2501_10714_amd import build
        build.build()
    return moe.load()


def header_functions():
    text = open(os.path.join(ROOT, "include", "moe_mi355x.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = header_functions()
    assert set(names) == set(binding.ENTRY_POINTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_capacity_matches_formula(lib):
    assert moe.moe_capacity(256, 4, 1, 1.25) == 80
    assert moe.moe_capacity(8192, 16, 2, 1.2) == 1229
    assert moe.moe_capacity(32768, 64, 6, 1.5) == 4608
    assert moe.moe_capacity(65536, 32, 1, 1.0) == 2048
    assert moe.moe_capacity(0, 4, 1, 1.0) == -1 and moe.moe_capacity(8, 4, 1, -1.0) == -1


def test_capacity_equals_the_oracle_over_a_sweep(lib):
    """moe_capacity (the product) against the oracle's T = ceil(k f N / E), on values where the product k f N / E is
    a whole number, just above one, or not representable."""
    from oracle import moe_oracle as O
    for n in (1, 7, 256, 1000, 8192, 32768, 65536, 99999):
        for e in (1, 3, 4, 16, 32, 64, 130, 256):
            for k in (1, 2, 6, 8):
                for f in (0.25, 0.3, 1.0, 1.1, 1.2, 1.25, 1.5, 2.0, 7.3):
                    assert moe.moe_capacity(n, e, k, f) == O.capacity(n, e, k, f), (n, e, k, f)


def test_config_validation(lib):
    ok = moe.MoeConfig.make(64, 64, 4, 128, 2, 0, moe.DT_F32, moe.ACT_RELU)
    ws, sv = moe.moe_workspace_bytes(ok)
    assert ws > 0 and sv > 0
    bad = [dict(N=0), dict(k=5), dict(dtype=7), dict(act=9), dict(M=66), dict(E=300, k=2), dict(k=9, E=16)]
    for kw in bad:
        a = dict(N=64, M=64, E=4, H=128, k=2, capacity=0, dtype=moe.DT_F32, act=moe.ACT_RELU)
        a.update(kw)
        with pytest.raises(moe.MoeError):
            moe.moe_workspace_bytes(moe.MoeConfig.make(**a))
        assert moe.moe_last_error() != ""


def test_null_pointers_are_rejected_before_any_launch(lib):
    cfg = moe.MoeConfig.make(64, 64, 4, 128, 2, 0, moe.DT_F32, moe.ACT_RELU)
    null = C.c_void_p(0)
    st = lib.moe_dispatch(C.byref(cfg), null, null, null, null)
    assert st == 1 and "NULL" in moe.moe_last_error()
    st = lib.moe_route(C.byref(cfg), *([null] * 13), C.c_size_t(0), null)
    assert st == 1
    st = lib.moe_layer_fwd(None, *([null] * 8), C.c_size_t(0), null, C.c_size_t(0), null)
    assert st == 1 and "cfg" in moe.moe_last_error()
    # workspace too small: status 3 (fake non-NULL pointers are never dereferenced on the host)
    fake = C.c_void_p(4096)
    st = lib.moe_route(C.byref(cfg), *([fake] * 13), C.c_size_t(16), null)
    assert st == 3 and "workspace" in moe.moe_last_error()
    glu = moe.MoeConfig.make(64, 64, 4, 128, 2, 0, moe.DT_F32, moe.ACT_SWIGLU)
    st = lib.moe_expert_ffn_fwd(C.byref(glu), fake, fake, fake, null, fake, fake, fake, fake, fake, null, C.c_size_t(0), null)
    assert st == 1 and "w3" in moe.moe_last_error()


def test_saved_layout_is_disjoint_and_ordered(lib):
    cfg = moe.MoeConfig.make(100, 64, 4, 128, 2, 0, moe.DT_BF16, moe.ACT_SWIGLU)
    _, total = moe.moe_workspace_bytes(cfg)
    end = 0
    for name in moe.SAVED:
        off, n = moe.moe_saved_offset(cfg, name)
        assert off >= end and off % 256 == 0
        end = off + n
    assert end <= total


def test_misaligned_pointers_and_the_new_calls_are_validated_on_the_host(lib):
    cfg = moe.MoeConfig.make(64, 64, 4, 128, 2, 0, moe.DT_F32, moe.ACT_RELU)
    null, fake, odd = C.c_void_p(0), C.c_void_p(4096), C.c_void_p(4100)
    st = lib.moe_dispatch(C.byref(cfg), odd, fake, fake, null)
    assert st == 1 and "16-byte aligned" in moe.moe_last_error()
    # the layer after the gate: dtopk_w is required, the chunk count is checked
    st = lib.moe_layer_bwd_routed(C.byref(cfg), fake, fake, null, fake, fake, C.c_size_t(1 << 30), fake, fake, null, fake,
                                  null, fake, C.c_size_t(1 << 30), C.c_int32(1), null)
    assert st == 1 and "dtopk_w" in moe.moe_last_error()
    st = lib.moe_layer_fwd_routed(C.byref(cfg), fake, fake, null, fake, fake, fake, C.c_size_t(1 << 30), fake,
                                  C.c_size_t(1 << 30), C.c_int32(99), null, null)
    assert st == 1 and "chunks" in moe.moe_last_error()
    # expert choice: one slot per expert and a positive number of tokens per expert
    with pytest.raises(moe.MoeError, match="expert choice"):
        moe.moe_workspace_bytes(moe.MoeConfig.make(64, 64, 4, 128, 2, 8, moe.DT_F32, moe.ACT_RELU, 3))
    with pytest.raises(moe.MoeError, match="expert choice"):
        moe.moe_workspace_bytes(moe.MoeConfig.make(64, 64, 4, 128, 4, 0, moe.DT_F32, moe.ACT_RELU, 3))
    ws, _ = moe.moe_workspace_bytes(moe.MoeConfig.make(64, 64, 4, 128, 4, 16, moe.DT_F32, moe.ACT_RELU, 3))
    assert ws > 0
    # X-MoE: projection width
    for d_proj in (0, 6, 260):
        with pytest.raises(moe.MoeError, match="d_proj"):
            moe.moe_route_xmoe_workspace_bytes(cfg, d_proj)
    assert moe.moe_route_xmoe_workspace_bytes(cfg, 32) > 0


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one-GPU" in r.stderr and r.stdout.strip() == ""


def test_the_product_path_never_reaches_the_oracle():
    """Nothing under the package imports oracle/ or tests/, and bench.py does so only inside its cpu_baseline leg."""
    import ast
    pkg = os.path.join(ROOT, "paper_2501_10714_amd")
    for fn in sorted(os.listdir(pkg)):
        if fn.endswith(".py"):
            text = open(os.path.join(pkg, fn)).read()
            assert "oracle" not in text and "moe_harness" not in text, fn
    tree = ast.parse(open(os.path.join(ROOT, "bench.py")).read())
    for node in ast.walk(tree):
        if isinstance(node, ast.FunctionDef):
            uses = [n for n in ast.walk(node) if isinstance(n, (ast.Import, ast.ImportFrom))
                    and "oracle" in (getattr(n, "module", None) or " ".join(a.name for a in n.names))]
            assert not uses or node.name == "cpu_baseline", node.name
    top = [n for n in tree.body if isinstance(n, (ast.Import, ast.ImportFrom))]
    assert all("oracle" not in (getattr(n, "module", None) or " ".join(a.name for a in n.names)) for n in top)
    assert "moe_harness" not in open(os.path.join(ROOT, "bench.py")).read()


def test_bench_traffic_constant_is_the_profile_total():
    """roofline.traffic of bench.py is a constant taken from the rocprofv3 byte-counter summary under profiles/: the two
    must say the same (read + written GB per step of the six expert-GEMM launches at the Mixtral shape)."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    text = open(os.path.join(ROOT, "profiles", "gg_mfma_kernel_mixtral_hbm_traffic.md")).read()
    m = re.search(r"Per step \(six launches\): ([0-9.]+) GB read \+ ([0-9.]+) GB written = ([0-9.]+) GB", text)
    assert m, "summary line not found in the profile"
    read_gb, written_gb, total_gb = map(float, m.groups())
    t = bench.MEASURED_GEMM_TRAFFIC["mixtral"]
    assert abs(t["read"] / 1e9 - read_gb) < 0.05 and abs(t["written"] / 1e9 - written_gb) < 0.05
    assert abs((t["read"] + t["written"]) / 1e9 - total_gb) < 0.1
