"""Builds libheisd_verify.so (hand-written HIP for gfx950) next to this file with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libheisd_verify.so")
SOURCES = [os.path.join(HERE, "csrc", "heisd_api.hip")]
HEADERS = [os.path.join(HERE, "csrc", n) for n in sorted(os.listdir(os.path.join(HERE, "csrc"))) if n.endswith(".h")]
HEADERS.append(os.path.join(os.path.dirname(HERE), "include", "heisd_verify.h"))

# packed-fp32 instructions are switched off on purpose: the compiler must not fuse pairs of
# fp32 operations into v_pk_* forms for these kernels.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(force: bool = True) -> str:
    """Compile the library.  With force=False an up-to-date library is kept."""
    if not force and os.path.exists(LIB):
        newest = max(os.path.getmtime(p) for p in SOURCES + HEADERS)
        if os.path.getmtime(LIB) >= newest:
            return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + SOURCES + ["-o", tmp]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build())
