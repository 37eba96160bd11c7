"""Host-sanitizer pass over the C ABI (CPU only, no GPU needed):

    python tests/sanitize_host.py

compiles the HOST code of libctm.so with AddressSanitizer and UndefinedBehaviorSanitizer (device code is compiled as
usual), compiles tests/abi_host_driver.c with the same sanitizers and runs it: every host-side refusal, the tile plan,
the exact-fraction interpolation coefficients and the handle-creation failure path of a machine without a GPU.
Not collected by pytest (it rebuilds the whole library, about two minutes); tests/test_abi.py runs the same driver
against the ordinary library on every CPU run.
"""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
from paper_2505_13644_amd import build as B  # noqa: E402

SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def main():
    out = os.path.join(ROOT, "_build", "san")
    os.makedirs(out, exist_ok=True)
    objs = []
    for src in B.SOURCES:
        obj = os.path.join(out, src.replace(".hip", ".o"))
        srcs = [os.path.join(B.CSRC, f) for f in os.listdir(B.CSRC)] + [os.path.join(ROOT, "include", "ctm.h")]
        if not os.path.exists(obj) or os.path.getmtime(obj) < max(os.path.getmtime(f) for f in srcs):
            B._run([B.HIPCC, *B.FLAGS, *SAN, "-c", os.path.join(B.CSRC, src), "-o", obj])
            print("compiled", src, flush=True)
        objs.append(obj)
    lib = os.path.join(out, "libctm.so")
    B._run([B.HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-shared-libsan", *objs, "-o", lib])
    clang = os.path.join(os.path.dirname(os.path.realpath(B.HIPCC)), "..", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/llvm/bin/clang"
    exe = os.path.join(out, "abi_host_driver")
    B._run([clang, "-std=c11", "-g", "-fsanitize=address", "-fsanitize=undefined", "-shared-libsan", "-fno-omit-frame-pointer",
            "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "abi_host_driver.c"), "-o", exe,
            "-L", out, "-lctm", f"-Wl,-rpath,{out}", "-L/opt/rocm/lib", "-Wl,-rpath,/opt/rocm/lib"])
    res = subprocess.run([clang, "-print-resource-dir"], capture_output=True, text=True).stdout.strip()
    rt = next((d for d, _, files in os.walk(os.path.realpath(res)) if "libclang_rt.asan-x86_64.so" in files), res)
    env = dict(os.environ, CTM_DRIVER_NO_GPU="1", ASAN_OPTIONS="detect_leaks=1:halt_on_error=1", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1",
               LD_LIBRARY_PATH=rt + os.pathsep + os.environ.get("LD_LIBRARY_PATH", ""))
    r = subprocess.run([exe], env=env, capture_output=True, text=True)
    sys.stdout.write(r.stdout)
    sys.stderr.write(r.stderr[-4000:])
    print("sanitizer run exit status", r.returncode)
    return r.returncode


if __name__ == "__main__":
    sys.exit(main())
