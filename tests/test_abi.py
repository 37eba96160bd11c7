"""CPU-only checks of the C-ABI boundary: the library loads, exports every symbol the
header declares, and rejects bad arguments on the host before any GPU work."""
import ctypes
import os
import re

import pytest

from paper_2505_13644_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(ROOT, "tests", "golden")


def declared_symbols():
    inc = os.path.join(ROOT, "include")
    text = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ctm_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported_and_bound():
    names = declared_symbols()
    assert {"ctm_create_mlp", "ctm_laplacian", "ctm_weighted_laplacian", "ctm_biharmonic_rand"} <= set(names)
    handle = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(handle, n), f"{n} declared in ctm.h but not exported"
        assert n in B.SIGNATURES, f"{n} has no Python binding"
    assert set(B.SIGNATURES) == set(names)


def test_rows_per_point_matches_paper_vector_counts():
    # Sec. 3.1: collapsed Taylor mode carries 1 + (K-1) R + 1 vectors, standard 1 + K R.
    with open(os.path.join(GOLDEN, "vector_counts.txt")) as fh:
        rows = [tuple(map(int, l.split())) for l in fh if l.strip() and not l.startswith("#")]
    assert rows
    for K, R, standard, collapsed in rows:
        assert standard == 1 + K * R
        assert B.ctm_rows_per_point(K, R) == collapsed
    assert B.ctm_rows_per_point(3, 4) == -1
    assert B.ctm_rows_per_point(2, 0) == -1
    # the ratio the paper quotes for the exact Laplacian at D = 50
    assert round(B.ctm_rows_per_point(2, 50) / (1 + 2 * 50), 2) == 0.51


@pytest.mark.parametrize("dtype", [B.CTM_F32, B.CTM_F64])
@pytest.mark.parametrize("K,R", [(2, 50), (2, 16), (2, 10), (4, 32), (2, 5), (2, 1), (4, 1), (2, 254), (2, 255),
                                 (2, 1000), (4, 84), (4, 85), (4, 300)])
def test_tile_plan_invariants(dtype, K, R):
    P, MB, Rp, passes = B.ctm_tile_plan(dtype, K, R)
    rho = B.ctm_rows_per_point(K, Rp)
    assert P >= 1 and P * rho <= 16 * MB <= 256          # whole points fit the tile
    assert passes >= 1 and Rp * passes >= R > Rp * (passes - 1) - passes  # every direction is covered once
    assert (passes - 1) * Rp < R
    if passes == 1:
        assert Rp == R


def test_tile_plan_for_benchmark_configs_wastes_no_rows():
    assert B.ctm_tile_plan(B.CTM_F32, 2, 50)[:2] == (4, 13)      # 4 points x 52 rows = 13 x 16
    P, MB, _, _ = B.ctm_tile_plan(B.CTM_F32, 2, 16)
    assert P * 18 == 16 * MB
    P, MB, _, _ = B.ctm_tile_plan(B.CTM_F32, 2, 10)
    assert P * 12 == 16 * MB


def test_invalid_arguments_are_rejected_on_the_host():
    L = B.lib()
    out = ctypes.c_void_p(None)
    dims = (ctypes.c_int * 3)(5, 16, 1)
    fake = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    assert L.ctm_create_mlp(2, dims, fake, None, B.CTM_F32, B.CTM_ACT_TANH, None, None) == -1
    assert L.ctm_create_mlp(2, None, fake, None, B.CTM_F32, B.CTM_ACT_TANH, None, ctypes.byref(out)) == -1
    assert L.ctm_create_mlp(2, dims, fake, None, 7, B.CTM_ACT_TANH, None, ctypes.byref(out)) == -3
    assert L.ctm_create_mlp(2, dims, fake, None, B.CTM_F32, 9, None, ctypes.byref(out)) == -3
    assert L.ctm_create_mlp(2, dims, fake, None, 4, B.CTM_ACT_SIN, None, ctypes.byref(out)) == -3
    assert L.ctm_create_mlp(1, dims, fake, None, B.CTM_F32, B.CTM_ACT_TANH, None, ctypes.byref(out)) == -2
    bad = (ctypes.c_int * 3)(5, 0, 1)
    assert L.ctm_create_mlp(2, bad, fake, None, B.CTM_F32, B.CTM_ACT_TANH, None, ctypes.byref(out)) == -2
    wide = (ctypes.c_int * 3)(5, 16, 1025)  # more outputs than the last-layer kernel takes
    assert L.ctm_create_mlp(2, wide, fake, None, B.CTM_F32, B.CTM_ACT_TANH, None, ctypes.byref(out)) == -4
    assert "outputs" in B.ctm_last_error()
    holes = (ctypes.c_void_p * 2)(0x1000, None)
    assert L.ctm_create_mlp(2, dims, holes, None, B.CTM_F32, B.CTM_ACT_TANH, None, ctypes.byref(out)) == -1
    odd = (ctypes.c_void_p * 2)(0x1002, 0x2000)
    assert L.ctm_create_mlp(2, dims, odd, None, B.CTM_F32, B.CTM_ACT_TANH, None, ctypes.byref(out)) == -6
    assert out.value is None
    # operator calls without a handle
    assert L.ctm_laplacian(None, None, 4, None, 5, 0, 1.0, None, None, None, 0, None) == -1
    assert "handle" in B.ctm_last_error()
    assert L.ctm_weighted_laplacian(None, None, 4, None, 5, None, None, None, 0, None) == -1
    assert L.ctm_biharmonic_rand(None, None, 4, None, 5, 0, None, None, None, 0, None) == -1
    assert L.ctm_workspace_bytes(None, 2, 4, 5) == 0
    assert L.ctm_destroy_mlp(None) == 0
    # every other entry point that takes a handle: NULL is an error reported on the host, never a crash
    assert L.ctm_weighted_laplacian_rand(None, None, 4, None, 5, 0, None, 0, 0, None, None, None, 0, None) == -1
    assert L.ctm_biharmonic_exact(None, None, 4, None, None, None, 0, None) == -1
    assert L.ctm_taylor_standard(None, 2, None, 4, None, 5, 0, 1.0, None, None, None, 0, None) == -1
    assert L.ctm_taylor_standard(None, 3, None, 4, None, 5, 0, 1.0, None, None, None, 0, None) == -4
    assert L.ctm_laplacian_fwd(None, None, 4, None, 5, 0, 1.0, None, None, None, 0, None) == -1
    assert L.ctm_laplacian_bwd(None, 4, 5, 1.0, None, 0, None, None, None, None, None, 0, None) == -1
    assert L.ctm_biharmonic_rand_fwd(None, None, 4, None, 5, 0, None, None, None, 0, None) == -1
    assert L.ctm_biharmonic_rand_bwd(None, 4, 5, None, 0, None, None, None, None, None, 0, None) == -1
    assert L.ctm_update_mlp(None, None, None, None) == -1
    assert L.ctm_biharmonic_exact_fwd(None, None, 4, None, None, None, 0, None) == -1
    assert L.ctm_biharmonic_exact_bwd(None, 4, None, 0, None, None, None, None, None, 0, None) == -1
    assert L.ctm_biharmonic_exact_tape_bytes(None, 4) == 0 and L.ctm_biharmonic_exact_backward_workspace_bytes(None, 4) == 0
    for fn in (L.ctm_tape_bytes, L.ctm_backward_workspace_bytes, L.ctm_biharmonic_tape_bytes, L.ctm_biharmonic_backward_workspace_bytes):
        assert fn(None, 4, 5) == 0
    assert L.ctm_biharmonic_exact_workspace_bytes(None, 4) == 0
    assert L.ctm_workspace_bytes_standard(None, 2, 4, 5) == 0
    assert L.ctm_weighted_laplacian_rand_workspace_bytes(None, 4, 5, 3, 0, 0) == 0
    with pytest.raises(B.CtmError):
        B.ctm_tile_plan(B.CTM_F32, 3, 5)
    with pytest.raises(B.CtmError):
        B.ctm_tile_plan(5, 2, 5)


def test_product_package_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2505_13644_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b|oracle[/.](operators|nested_dual)", text, flags=re.M), \
                    f"{f} reaches into the oracle package"


def test_plain_c_driver_of_the_abi_compiles_and_passes(tmp_path):
    # include/ctm.h is a C header: a C11 program that calls every entry point with arguments the host must refuse (the
    # same program runs under ASan / UBSan through tests/sanitize_host.py)
    import shutil
    import subprocess
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        pytest.skip("no C compiler")
    exe = str(tmp_path / "abi_host_driver")
    lib_dir = os.path.dirname(B.LIB_PATH)
    subprocess.run([cc, "-std=c11", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "abi_host_driver.c"), "-o", exe, "-L", lib_dir, "-lctm",
                    f"-Wl,-rpath,{lib_dir}", "-L/opt/rocm/lib", "-Wl,-rpath,/opt/rocm/lib"], check=True)
    import torch
    env = dict(os.environ)
    if not torch.cuda.is_available():
        env["CTM_DRIVER_NO_GPU"] = "1"
    r = subprocess.run([exe], env=env, capture_output=True, text=True)
    assert r.returncode == 0 and "abi host driver: ok" in r.stdout, r.stdout + r.stderr
