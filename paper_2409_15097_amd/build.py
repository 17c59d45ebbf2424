"""Builds libbbm.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree next to this file."""
import os
import shutil
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libbbm.so")
SOURCES = ["bbm_error.hip", "bbm_preprocess.hip", "bbm_index.hip", "bbm_colindex.hip", "bbm_attn.hip", "bbm_attn_bwd.hip", "bbm_reorder.hip", "bbm_probe.hip"]

# packed-fp32 VALU ops are switched off for device code (the host pass warns that it ignores the feature)
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
               "-mllvm", "-amdgpu-mfma-vgpr-form", "-fno-honor-nans"]


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: libbbm cannot be built")


def build_library(verbose: bool = False, extra_flags=()) -> str:
    """Compiles every translation unit and links libbbm.so.  Always rebuilds."""
    hipcc = hipcc_path()
    obj_dir = os.path.join(PKG_DIR, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    procs = []
    for src in SOURCES:
        obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
        cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c",
               os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    objs = []
    for src, obj, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out)
        objs.append(obj)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}")
    return LIB_PATH


def build_host_sanitized(out_dir: str) -> str:
    """Host-side check build: every translation unit's HOST code (argument validation, workspace arithmetic, launch
    set-up) compiled with AddressSanitizer and UndefinedBehaviorSanitizer, no device code at all (the device images
    the host objects refer to are replaced by empty stubs, so nothing in this library can be launched).  Returns the
    path of the shared library; load it with the sanitizer runtime preloaded (sanitizer_runtime())."""
    hipcc = hipcc_path()
    os.makedirs(out_dir, exist_ok=True)
    procs, objs = [], []
    for src in SOURCES:
        obj = os.path.join(out_dir, src.replace(".hip", ".o"))
        cmd = [hipcc, "--offload-arch=gfx950", "--cuda-host-only", "-fno-gpu-sanitize", "-fsanitize=address,undefined",
               "-fno-omit-frame-pointer", "-O1", "-g", "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
               "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError(f"hipcc (host only, sanitized) failed on {src}:\n{out}")
    undefined = subprocess.run(["nm", "-u", *objs], stdout=subprocess.PIPE, text=True, check=True).stdout
    images = sorted({w for line in undefined.splitlines() for w in line.split() if w.startswith("__hip_fatbin_")})
    stub_c = os.path.join(out_dir, "device_image_stubs.c")
    with open(stub_c, "w") as f:
        f.writelines(f"const char {name}[64] __attribute__((aligned(4096))) = {{0}};\n" for name in images)
    stub_o = stub_c[:-2] + ".o"
    subprocess.run(["gcc", "-fPIC", "-c", stub_c, "-o", stub_o], check=True)
    lib = os.path.join(out_dir, "libbbm_hostsan.so")
    r = subprocess.run([hipcc, "-shared", "-fPIC", "-fno-gpu-sanitize", "-fsanitize=address,undefined", *objs, stub_o, "-o", lib],
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}")
    return lib


def sanitizer_runtime() -> str:
    """Path of the AddressSanitizer runtime that matches hipcc's clang (to be preloaded into an uninstrumented python)."""
    clang = os.path.join(os.path.dirname(os.path.realpath(hipcc_path())), "..", "lib", "llvm", "bin", "clang++")
    if not os.path.exists(clang):
        clang = "/opt/rocm/lib/llvm/bin/clang++"
    out = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], stdout=subprocess.PIPE, text=True, check=True).stdout.strip()
    if not os.path.isabs(out) or not os.path.exists(out):
        raise RuntimeError(f"sanitizer runtime not found ({out})")
    return out


if __name__ == "__main__":
    print(build_library(verbose=True))
