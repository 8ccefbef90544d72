"""Build libkvm.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libkvm.so")
SOURCES = ["kvm_api.hip", "fold.hip", "fold_fused.hip", "score_mfma.hip", "attn_rows.hip", "attn_mfma.hip", "peaks.hip", "prep.hip", "backward.hip", "backward_mfma.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17",
         # packed fp32 VALU forms are kept out of the generated code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


STAMP = LIB + ".srchash"


def source_hash() -> str:
    """Digest of everything the library is built from: sources, headers, flags."""
    import hashlib
    h = hashlib.sha256(" ".join(FLAGS + SOURCES).encode())
    files = sorted(os.listdir(CSRC))
    paths = [os.path.join(CSRC, f) for f in files if f.endswith((".hip", ".h"))]
    paths.append(os.path.join(os.path.dirname(HERE), "include", "kvm.h"))
    for p in paths:
        with open(p, "rb") as f:
            h.update(p[len(os.path.dirname(HERE)):].encode())
            h.update(f.read())
    return h.hexdigest()


def is_stale() -> bool:
    """True when libkvm.so is missing or was built from other sources than the tree holds now
    (compared by content, so that copying the tree to another machine changes nothing)."""
    if not os.path.exists(LIB) or not os.path.exists(STAMP):
        return True
    with open(STAMP) as f:
        return f.read().strip() != source_hash()


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = [_hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", *objs, "-o", LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    with open(STAMP, "w") as f:
        f.write(source_hash() + "\n")
    if verbose:
        print(f"built {LIB}", file=sys.stderr)
    return LIB


def build_host_checked(out_dir: str):
    """Host side only (`--cuda-host-only`: no kernel is compiled), with AddressSanitizer and UBSan,
    as a library of its own in `out_dir`: for tests of the host logic on a machine without a GPU.
    The device images the host objects refer to are replaced by zero-filled placeholders, so this
    build can check arguments, sizes and plans but can launch nothing.  Returns (library path,
    path of the sanitizer runtime to preload into the process that loads it)."""
    os.makedirs(out_dir, exist_ok=True)
    san = ["-fsanitize=address,undefined", "-fno-omit-frame-pointer"]
    flags = ["-O1", "-g", "--cuda-host-only", "--offload-arch=gfx950", "-fPIC", "-std=c++17", *san]

    def one(src):
        obj = os.path.join(out_dir, src.replace(".hip", ".o"))
        r = subprocess.run([_hipcc(), *flags, "-c", os.path.join(CSRC, src), "-o", obj], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc (host only) failed for {src}:\n{r.stdout}\n{r.stderr}")
        return obj

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(one, SOURCES))
    undefined = subprocess.run(["nm", "-u", *objs], capture_output=True, text=True, check=True).stdout
    images = sorted({t for t in undefined.split() if t.startswith("__hip_fatbin_")})
    stub = os.path.join(out_dir, "device_image_placeholders.cpp")
    with open(stub, "w") as f:
        for name in images:
            f.write(f'extern "C" {{ __attribute__((aligned(4096))) char {name}[4096] = {{0}}; }}\n')
    stub_o = stub.replace(".cpp", ".o")
    subprocess.run(["g++", "-fPIC", "-c", stub, "-o", stub_o], check=True)
    lib = os.path.join(out_dir, "libkvm_hostcheck.so")
    r = subprocess.run([_hipcc(), "-shared", "-fPIC", "--cuda-host-only", *san, "-shared-libsan", *objs, stub_o, "-o", lib],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link (host only) failed:\n{r.stdout}\n{r.stderr}")
    clang = os.path.join(os.path.dirname(os.path.realpath(_hipcc())), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/llvm/bin/clang"
    runtime = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True,
                             check=True).stdout.strip()
    return lib, runtime


if __name__ == "__main__":
    build()
