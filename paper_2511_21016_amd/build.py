"""Build libgka.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgka.so")
SOURCES = ["gka_api.hip", "gka_state_pass.hip", "gka_chunk_solve.hip", "gka_fused.hip", "gka_decode.hip",
           "gka_backward.hip", "gka_readout.hip", "gka_sketch.hip", "gka_small_dim.hip"]
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-FP32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def build_library(verbose=True, extra_flags=()):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    os.makedirs(os.path.join(CSRC, "_build"), exist_ok=True)
    for src in SOURCES:
        obj = os.path.join(CSRC, "_build", src.replace(".hip", ".o"))
        cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if out.strip() and verbose:
            print(out)
        if pr.returncode != 0:
            failed = True
            print(f"hipcc failed on {src}", file=sys.stderr)
    if failed:
        raise RuntimeError("libgka build failed")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


HOST_SANITIZED_LIB = os.path.join(CSRC, "_build", "libgka_hostsan.so")


def sanitizer_runtime():
    """Path of the AddressSanitizer runtime of hipcc's clang (to be preloaded into the process that loads the
    sanitized library)."""
    clang = os.path.join(os.path.dirname(os.path.realpath(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"))),
                         "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/llvm/bin/clang"
    return subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], check=True, stdout=subprocess.PIPE,
                          text=True).stdout.strip()


def build_host_sanitized(verbose=False):
    """A second library whose HOST code (argument validation, launch plans, workspace carving: gka_api.hip) is
    compiled with AddressSanitizer and UndefinedBehaviorSanitizer; device code and the other objects are the
    regular ones. Only the CPU tests of the boundary load it; GPU sanitizers are not involved."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = [os.path.join(CSRC, "_build", src.replace(".hip", ".o")) for src in SOURCES]
    if not all(os.path.exists(o) for o in objs):
        build_library(verbose=verbose)
    san_obj = os.path.join(CSRC, "_build", "gka_api.hostsan.o")
    host_flags = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                  "-Xarch_host", "-fno-sanitize=vptr", "-Xarch_host", "-fno-sanitize-recover=all",
                  "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    cmd = [hipcc, *HIPCC_FLAGS, *host_flags, "-c", os.path.join(CSRC, "gka_api.hip"), "-o", san_obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    pr = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if pr.returncode != 0:
        raise RuntimeError("sanitized build of gka_api.hip failed:\n" + pr.stdout)
    objs[SOURCES.index("gka_api.hip")] = san_obj
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
           "-fno-sanitize=vptr", "-shared-libsan", "-o", HOST_SANITIZED_LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return HOST_SANITIZED_LIB


if __name__ == "__main__":
    build_library()
