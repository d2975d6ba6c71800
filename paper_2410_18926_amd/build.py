"""Build the HIP library: hipcc for gfx950 -> paper_2410_18926_amd/liblorann.so (in-tree)."""
from __future__ import annotations

import pathlib
import shutil
import subprocess

HERE = pathlib.Path(__file__).resolve().parent
SRC = HERE / "csrc" / "lorann.hip"
LIB = HERE / "liblorann.so"

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    # packed fp32 instructions are kept off: some of their forms have produced wrong results on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # matrix-core results go to ordinary vector registers: the epilogues read every result register once, and
    # from the accumulation registers each read costs an extra move
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-Wall", "-Wno-unused-function",
]


SAN_LIB = HERE / "liblorann_san.so"


def build_sanitized() -> pathlib.Path:
    """The same library with AddressSanitizer and UndefinedBehaviorSanitizer in its HOST code (argument checks, index
    loading, workspace planning; device code is compiled as usual).  Load it with LORANN_LIB=<path> and clang's
    sanitizer runtime first in the process (sanitizer_runtime())."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    flags = [f for f in FLAGS if f != "-O3"] + ["-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                                                 "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer"]
    res = subprocess.run([hipcc, *flags, "-o", str(SAN_LIB), str(SRC)], capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l))
    return SAN_LIB


def sanitizer_runtime() -> str:
    clang = pathlib.Path(shutil.which("hipcc") or "/opt/rocm/bin/hipcc").resolve().parent.parent / "llvm" / "bin" / "clang"
    if not clang.exists():
        clang = pathlib.Path("/opt/rocm/llvm/bin/clang")
    return subprocess.run([str(clang), "--print-file-name=libclang_rt.asan-x86_64.so"], check=True, capture_output=True, text=True).stdout.strip()


def sources():
    return [SRC] + sorted((HERE / "csrc").glob("*.hpp")) + [HERE.parent / "include" / "lorann.h"]


def build(force: bool = True, verbose: bool = False) -> pathlib.Path:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not force and LIB.exists() and all(LIB.stat().st_mtime >= s.stat().st_mtime for s in sources()):
        return LIB
    cmd = [hipcc, *FLAGS, "-o", str(LIB), str(SRC)]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "packed-fp32-ops"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed:\n{err}")
    if verbose and err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
